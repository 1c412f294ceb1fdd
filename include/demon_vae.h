/*
 * demon_vae.h -- C ABI of the windowed VAE decode, and of its mirror the windowed encode, for AMD MI355X (gfx950).
 *
 * The operation is the windowed decode of paper section 3.6: a temporal audio
 * latent (25 Hz) is cut into windows, every window is extended by a halo of
 * latent frames on both sides, the extended windows go through the 1-D
 * convolutional audio decoder as one batch, the halos are trimmed and the
 * frame-aligned interiors (prod(strides) samples per latent frame, 1920 at
 * 48 kHz) are written side by side into the waveform.  With a halo at least as
 * large as the decoder's receptive field the result equals the full decode.
 *
 * The decoder is the synthetic stack of the benchmark description (the paper
 * does not list the layers of the trained model):
 *   for each upsample block l:  Snake -> ConvTranspose1d(kernel 2 s_l, stride s_l, padding s_l/2)
 *                               then n_res residual units  h += Conv1d_k1(Snake(Conv1d_k,dil(Snake(h))))
 *   head:                       Snake -> Conv1d(head_kernel) -> tanh
 *   snake(x) = x + sin(alpha_c x)^2 / (beta_c + 1e-9), per channel c.
 *
 * All entry points return a status and never throw or abort.  A handle may be
 * used by one host thread at a time, and its decode calls must go to one
 * stream (or be ordered by the caller): they share the handle's workspace.
 * Decode calls are asynchronous on the given HIP stream and allocate nothing.
 * With two or more windows the bf16 path runs half of the windows on a second,
 * internal stream that it forks from and joins back into the given stream
 * within the call, so the call is ordered on the given stream like any other
 * work and can be captured into a graph.
 * A window grid (clips, frames, range, window, halo) seen for the first time has its table written by a small
 * kernel on the same stream; the 16 most recent grids are kept.  A call recorded into a HIP graph pins its grid's
 * entry for the life of the handle (the graph holds the table's address), so at most 16 different grids can be
 * recorded per handle; a further one returns DEMON_ERR_WORKSPACE.
 *
 * Options (demon_vae_config fields wide_operands, flags, small_tile_wgs; on the benchmark stacks the results stay
 * within the same tolerances).  A field left at 0 takes the default, which the environment can change for a whole
 * process (read once when the library is loaded):
 *   DEMON_VAE_WIDE_OPERANDS=bf16x2  default of wide_operands becomes 2
 *   DEMON_VAE_NO_FUSED=1            as if DEMON_VAE_FLAG_NO_FUSED were set in every config
 *   DEMON_VAE_ONE_STREAM=1          as if DEMON_VAE_FLAG_ONE_STREAM were set in every config
 *   DEMON_VAE_SMALL_TILE_WGS=n      default of small_tile_wgs becomes n (0 = never)
 */
#ifndef DEMON_VAE_H
#define DEMON_VAE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; only the entry points declared here are exported. */
#if defined(__GNUC__)
#define DEMON_API __attribute__((visibility("default")))
#else
#define DEMON_API
#endif

typedef struct demon_vae demon_vae; /* opaque; owned by the library */

typedef enum {
    DEMON_OK = 0,
    DEMON_ERR_INVALID_ARG = 1, /* null pointer, bad range, bad layer description, wrong weight count */
    DEMON_ERR_UNSUPPORTED = 2, /* a layer shape the kernels do not cover (see demon_vae_create) */
    DEMON_ERR_WORKSPACE = 3,   /* the call needs more frames, clips or windows than create() sized for */
    DEMON_ERR_HIP = 4          /* a HIP runtime call or a kernel launch failed */
} demon_status;

typedef enum {
    DEMON_F32 = 0, /* fp32 storage and arithmetic (reference-precision path)            */
    DEMON_BF16 = 1 /* bf16 weights and latent, 16-bit MFMA operands (bf16; on levels of 512 channels
                      and more IEEE half or, with wide_operands = 2, hi + lo bf16 pairs), fp32
                      accumulation and epilogues, residual stream stored as IEEE half.  Conversions to
                      half saturate at +-65504 instead of overflowing to infinity                      */
} demon_dtype;

/* demon_vae_config.flags */
#define DEMON_VAE_FLAG_NO_FUSED   1   /* every residual unit as two kernels (no fused units)          */
#define DEMON_VAE_FLAG_ONE_STREAM 2   /* no internal second stream: all launches on the given stream  */
#define DEMON_VAE_FLAG_NO_WIDE_TILE 4 /* dilated convs never use the 128 x 256 tile (bit-identical results) */
#define DEMON_VAE_FLAG_NO_HEAD_FUSION 8 /* the head always runs as its own kernel (bit-identical results) */

/* Layer stack and workspace limits.  Arrays are read during the call only. */
typedef struct {
    int latent_channels;  /* C0 */
    int n_blocks;         /* number of upsample blocks, 1..16 */
    const int* strides;   /* [n_blocks], each even and >= 2 */
    const int* widths;    /* [n_blocks], output channels of each block */
    int n_res;            /* residual units per block, 0..8 */
    const int* dilations; /* [n_res] */
    int res_kernel;       /* odd; 7 in the benchmark stacks */
    int head_kernel;      /* odd */
    int out_channels;     /* 1..8; 2 = stereo */
    demon_dtype dtype;
    int max_frames;       /* longest latent (frames per clip) a decode call may pass */
    int max_clips;        /* most clips a decode call may pass */
    long long max_extended_frames; /* most latent frames, summed over all extended windows (window + halos)
                                      of one call, the workspace must hold; 0 = 3 * max_frames * max_clips */
    /* Options of the bf16 path; 0 = default in each. */
    int wide_operands;    /* levels of 512 channels and more: 1 = IEEE half operands on the f16 MFMA (the default),
                             2 = hi + lo bf16 pairs on the bf16 MFMA (two MFMAs per k-step in the transposed and 1x1
                             convolutions) for stacks whose wide-level activations may leave the half range */
    int flags;            /* DEMON_VAE_FLAG_* */
    int small_tile_wgs;   /* launches of at most this many 128 x 128 tiles use 64 x 64 tiles instead (bit-identical
                             results, more workgroups for a single playback window); default 192, negative = never */
} demon_vae_config;

/* One window of the grid: interior latent frames [begin, end) of clip `clip`, decoded from the
 * extended region [lo, hi) = [max(0, begin - halo), min(n_frames, end + halo)). */
typedef struct {
    int clip;
    int begin, end;
    int lo, hi;
} demon_window;

/*
 * Number of fp32 values demon_vae_create expects: per block up.alpha[C_in], up.beta[C_in],
 * up.weight[C_in, C, 2s], up.bias[C]; per residual unit a1.alpha[C], a1.beta[C],
 * c1.weight[C, C, res_kernel], c1.bias[C], a2.alpha[C], a2.beta[C], c2.weight[C, C, 1], c2.bias[C];
 * then head.alpha[C], head.beta[C], head.weight[out_channels, C, head_kernel], head.bias[out_channels]
 * -- in that order, each tensor C-contiguous.  Host only.  Returns 0 for an invalid description.
 */
DEMON_API size_t demon_vae_weight_count(const demon_vae_config* cfg);

/*
 * Receptive field of the layer stack in latent frames (host only, no GPU needed): output frame f
 * depends on latent frames [f - *halo_left, f + *halo_right].  Derived by propagating index
 * intervals backwards through the stack: a k-tap convolution of dilation d widens an interval by
 * d (k-1)/2 on both sides; a transposed convolution (kernel k, stride s, padding p) maps output
 * samples [a, b] to inputs [ceil((a + p - k + 1)/s), floor((b + p)/s)].  This is the analytic
 * counterpart of the measured convergence distance of section 3.6.
 */
DEMON_API demon_status demon_vae_rf_from_config(const demon_vae_config* cfg, int* halo_left, int* halo_right);

/*
 * Output samples [*lo, *hi] that latent frames [frame_a, frame_b] can influence, ignoring clip
 * edges (the forward cone; host only).
 */
DEMON_API demon_status demon_vae_forward_support(const demon_vae_config* cfg, int frame_a, int frame_b,
                                       long long* lo, long long* hi);

/*
 * The window grid of section 3.6 for frames [frame_begin, frame_end) of each of n_clips clips of
 * n_frames frames: windows start at frame_begin and step by `window`, the last one may be short;
 * each is extended by `halo` frames, clamped to the clip.  Host only.  Writes at most `capacity`
 * entries to `out` (may be NULL to count) and the total number to *n_windows.
 * INVALID_ARG: n_clips < 1, n_frames < 1, frame_begin < 0, frame_end > n_frames,
 * frame_begin >= frame_end, window < 1, halo < 0, n_windows NULL.
 */
DEMON_API demon_status demon_vae_plan_windows(int n_clips, int n_frames, int frame_begin, int frame_end,
                                    int window, int halo, demon_window* out, int capacity,
                                    int* n_windows);

/*
 * Builds a decoder on the current HIP device.  `host_weights` (host memory, fp32, canonical order,
 * demon_vae_weight_count(cfg) values) is copied and repacked during the call and may be freed
 * afterwards; for DEMON_BF16 the values are rounded to bf16 (nearest even) here.  Allocates device
 * weights and a workspace for max_extended_frames frames of extended windows.  *out receives the handle.
 * INVALID_ARG: null pointers, bad layer description (odd stride, even kernel, non-positive sizes),
 * n_floats != demon_vae_weight_count.  UNSUPPORTED: head_kernel > 15; DEMON_BF16 only: latent_channels
 * not a multiple of 16, a width not a multiple of 32, or a dilated kernel spanning more than 64 samples.  HIP: no device / allocation
 * failure.
 */
DEMON_API demon_status demon_vae_create(const demon_vae_config* cfg, const float* host_weights, size_t n_floats,
                              demon_vae** out);

/* Frees device memory and the handle.  NULL is ignored.  The caller must have synchronised the
 * streams it used with this handle. */
DEMON_API void demon_vae_destroy(demon_vae* vae);

/* Receptive field of this decoder (same as demon_vae_rf_from_config). Host only. */
DEMON_API demon_status demon_vae_receptive_field(const demon_vae* vae, int* halo_left, int* halo_right);

/*
 * Full decode (section 3.6, the un-windowed baseline): every clip is one window covering
 * [0, n_frames) with no halo.
 *   d_latent : device, [n_clips, latent_channels, n_frames], frames fastest; fp32 for DEMON_F32,
 *              bf16 (16-bit) for DEMON_BF16.  Read only.
 *   d_out    : device, fp32, [n_clips, out_channels, n_frames * S] planar, S = prod(strides).
 *   stream   : hipStream_t (NULL = default stream).
 */
DEMON_API demon_status demon_vae_decode(demon_vae* vae, const void* d_latent, int n_clips, int n_frames,
                              float* d_out, void* stream);

/*
 * Windowed decode of latent frames [frame_begin, frame_end) of every clip: gather the extended
 * windows, run them through the decoder as one batch, trim the halos, write the interiors.
 * Writes only d_out[:, :, frame_begin*S : frame_end*S); the rest of d_out is left untouched, so a
 * partial re-decode splices into an existing waveform.  `halo` in latent frames; -1 = the analytic
 * receptive field; a smaller halo is legal but inexact near window joins.
 * frame_end - frame_begin <= window decodes a single playback window.
 * Layouts as for demon_vae_decode (d_latent and d_out are whole-clip buffers).
 * INVALID_ARG: null pointers, n_clips < 1, n_frames < 1, frame_begin < 0, frame_end > n_frames,
 * frame_begin >= frame_end, window < 1, halo < -1.  WORKSPACE: n_frames > max_frames,
 * n_clips > max_clips, more than 4096 windows, extended windows that exceed the workspace, or (under
 * stream capture) a new grid when all cached grids are held by graphs.  UNSUPPORTED (bf16 path): one
 * extended window whose widest activation plane exceeds 4 026 531 840 bytes (32-bit offsets within a
 * window; about 300 s of audio in ONE window of the x1920 stack -- decode it in several windows).
 */
DEMON_API demon_status demon_vae_decode_windowed(demon_vae* vae, const void* d_latent, int n_clips, int n_frames,
                                       int frame_begin, int frame_end, int window, int halo,
                                       float* d_out, void* stream);

/*
 * The same windowed decode with the 16-bit render fused into the stitch (section 3.6 states its
 * exactness criterion on the 16-bit PCM render).  Each sample is quantised in fp32 as
 * q = rint(32767 * clamp(y, -1, 1)), ties to even, and written channel-interleaved:
 *   d_pcm : device, int16, [n_clips, n_frames * S, out_channels]; only samples
 *           [frame_begin*S, frame_end*S) of every clip are written.
 * All other arguments, limits and errors as for demon_vae_decode_windowed.
 */
DEMON_API demon_status demon_vae_decode_windowed_pcm16(demon_vae* vae, const void* d_latent, int n_clips, int n_frames,
                                             int frame_begin, int frame_end, int window, int halo,
                                             int16_t* d_pcm, void* stream);

/*
 * Latent similarity filter (section 3.5): per clip, mse = mean over all elements of
 * (curr - prev)^2, accumulated in double precision in a fixed order and rounded to fp32;
 * unchanged = (mse < threshold).  The paper's threshold is 1e-3.  A caller that finds
 * unchanged != 0 skips the decode of that clip and keeps the previous waveform.
 *   d_curr, d_prev : device, [n_clips, elems_per_clip] (any channel/frame order, the same in both);
 *                    fp32 for DEMON_F32, bf16 for DEMON_BF16.  Read only.
 *   d_mse          : device, fp32 [n_clips], or NULL.
 *   d_unchanged    : device, int [n_clips] (1 = below threshold), or NULL.  Not both NULL.
 * No handle and no workspace are needed.  INVALID_ARG: null pointers, n_clips outside [1, 65535],
 * elems_per_clip < 1, unknown dtype, threshold negative or NaN.
 */
DEMON_API demon_status demon_vae_latent_similarity(const void* d_curr, const void* d_prev, int n_clips, long long elems_per_clip,
                                         demon_dtype dtype, float threshold, float* d_mse, int* d_unchanged, void* stream);

/*
 * Windowed decode behind the similarity gate (section 3.5: a clip whose latent is nearly unchanged
 * skips the decode and keeps its previous audio).  d_skip: device, int [n_clips], read when the call
 * executes on the stream, e.g. the d_unchanged output of demon_vae_latent_similarity issued to the same
 * stream before: no host round trip.  Clips with a non-zero flag are not decoded and their part of
 * d_out is left as it is; the other clips are decoded exactly as by demon_vae_decode_windowed.
 * All other arguments, limits and errors as there; INVALID_ARG also for a NULL d_skip.
 */
DEMON_API demon_status demon_vae_decode_windowed_gated(demon_vae* vae, const void* d_latent, int n_clips, int n_frames,
                                             int frame_begin, int frame_end, int window, int halo,
                                             const int* d_skip, float* d_out, void* stream);

/*
 * ---- The windowed encode (the mirror path; section 3.7 names separate encode and decode engines, Table III times
 * the encode and notes its sampling step on the output moments).  The paper prints no encoder layers; the encoder
 * here is the mirror of the decoder the config describes:
 *   stem:                        Conv1d(head_kernel) from the out_channels-channel waveform to widths[n_blocks-1]
 *   for l = n_blocks .. 1:       n_res residual units of width widths[l-1] (as in the decoder), then
 *                                Snake -> Conv1d(kernel 2 s_l, stride s_l, padding s_l/2) to widths[l-2],
 *                                and for l = 1 to 2 x latent_channels: the moments (mean | log-variance)
 *   sampling step:               z = mean + exp(logvar / 2) * eps, eps ~ N(0, 1) supplied by the caller
 * S = prod(strides) samples make one latent frame, exactly.  Windowed: the samples of every window of latent frames
 * are extended by `halo` frames' worth of samples on both sides (clamped to the clip), the extended windows are
 * encoded as one batch, each as if it were a whole clip, and the halo frames are trimmed; with a halo of at least the
 * encoder's receptive field the result equals the full encode.
 */

/*
 * Number of fp32 values demon_vae_create_encoder expects: stem.weight[C, out_channels, head_kernel], stem.bias[C]
 * (C = widths[n_blocks-1]); then for l = n_blocks .. 1, C = widths[l-1]: per residual unit the eight tensors of a
 * decoder unit; then down.alpha[C], down.beta[C], down.weight[C_out, C, 2 s_l], down.bias[C_out] with
 * C_out = widths[l-2], and 2 latent_channels for l = 1.  Host only.  Returns 0 for an invalid description.
 */
DEMON_API size_t demon_vae_encoder_weight_count(const demon_vae_config* cfg);

/*
 * Receptive field of the encoder (host only): the moments of latent frame f depend on the waveform samples
 * [f S - *samples_left, f S + S - 1 + *samples_right], i.e. on *halo_left / *halo_right further frames' worth of
 * samples (the sample counts rounded up to whole frames).  Interval propagation backwards from the moments: a strided
 * conv reads inputs n s - s/2 .. n s + 3s/2 - 1 for output n, a k-tap conv of dilation d widens by d (k-1)/2.
 * samples_left / samples_right may be NULL.
 */
DEMON_API demon_status demon_vae_encoder_rf_from_config(const demon_vae_config* cfg, int* halo_left, int* halo_right,
                                                        long long* samples_left, long long* samples_right);

/*
 * Builds the encoder on the current HIP device; arguments, limits and errors as for demon_vae_create
 * (max_frames, max_clips, max_extended_frames size its workspace in latent frames), with the weight order of
 * demon_vae_encoder_weight_count.  UNSUPPORTED also for wide_operands = 2 and a stem width that is not a multiple
 * of 8.  The handle is freed with demon_vae_destroy; demon_vae_receptive_field returns the encoder's halo; the decode
 * entry points reject it (INVALID_ARG), as the encode entry points reject a decoder.
 */
DEMON_API demon_status demon_vae_create_encoder(const demon_vae_config* cfg, const float* host_weights, size_t n_floats,
                                                demon_vae** out);

/*
 * Windowed encode of latent frames [frame_begin, frame_end) of every clip.
 *   d_wave    : device, fp32, [n_clips, out_channels, n_frames * S] planar (the decoder's output layout).  Read only.
 *   d_eps     : device, fp32, [n_clips, latent_channels, n_frames], the N(0, 1) draw of the sampling step; NULL: z = mean.
 *   d_moments : device, fp32, [n_clips, 2 latent_channels, n_frames] (channels 0 .. C0-1 mean, C0 .. 2 C0-1 log-variance), or NULL.
 *   d_latent  : device, [n_clips, latent_channels, n_frames], frames fastest; fp32 for DEMON_F32, bf16 for DEMON_BF16
 *               (the layout demon_vae_decode reads), or NULL.  Not both outputs NULL.
 * Only frames [frame_begin, frame_end) of the outputs are written.  `halo` in latent frames; -1 = the encoder's
 * receptive field.  Asynchronous on `stream`, allocates nothing; window grids are cached as for the decode.
 * Errors as for demon_vae_decode_windowed.
 */
DEMON_API demon_status demon_vae_encode_windowed(demon_vae* enc, const float* d_wave, int n_clips, int n_frames,
                                                 int frame_begin, int frame_end, int window, int halo,
                                                 const float* d_eps, float* d_moments, void* d_latent, void* stream);

/* Full encode: every clip is one window covering [0, n_frames) with no halo. */
DEMON_API demon_status demon_vae_encode(demon_vae* enc, const float* d_wave, int n_clips, int n_frames, const float* d_eps,
                                        float* d_moments, void* d_latent, void* stream);

/*
 * For callers that cannot allocate device memory or may not let a library hold a workspace of its own choosing --
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc: demon_vae_decode_windowed with
 * everything the call needs besides its inputs and outputs (window table, activation buffers, window waveforms) in
 * a static device array of DEMON_VAE_STATIC_SCRATCH_BYTES that is part of the library's image.  Each GPU the library
 * runs on holds its own copy until the process ends.  The call allocates nothing, copies nothing from the host (a
 * kernel writes the window table) and runs on the given stream only; it can be captured without a preceding call.
 * Same arguments, layouts, results (bit for bit) and INVALID_ARG cases as demon_vae_decode_windowed; max_frames,
 * max_clips and max_extended_frames of the handle do not apply.  WORKSPACE: more than 4096 windows, or extended
 * windows whose buffers exceed the array (the message states the bytes needed; for the x1920 benchmark stack about
 * 1.2 MB per extended latent frame, i.e. about 100 frames: one 3 s playback window with its halos).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU -- from different streams,
 * threads or handles -- race.  The array keeps the previous call's contents; nothing in it needs clearing (whatever
 * a call reads of it and has not written itself only reaches results that are dropped).
 */
#define DEMON_VAE_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
DEMON_API demon_status demon_vae_decode_windowed_static(demon_vae* vae, const void* d_latent, int n_clips, int n_frames,
                                              int frame_begin, int frame_end, int window, int halo,
                                              float* d_out, void* stream);

/*
 * Equal-power crossfade of a chunk boundary of the playback stream (Fig. 1 and section 3.1: each decoded
 * chunk is crossfaded into the output stream; section 4.8.2 names a 50 ms equal-power fade, 2400 samples at 48 kHz):
 *   d_out[c][i] = cos(t_i) * d_prev_tail[c][i] + sin(t_i) * d_next_head[c][i],  t_i = (pi/2)(i + 1/2)/n_samples
 * for planes c < n_planes, samples i < n_samples; plane c of a buffer starts c * stride floats after
 * its pointer, so the segments may lie inside larger planar waveforms.  All device, fp32.  d_out may
 * alias either input exactly (same pointer and stride).  INVALID_ARG: null pointers, n_planes outside
 * [1, 65535], n_samples < 1, a negative stride, or output planes that overlap.
 */
DEMON_API demon_status demon_vae_crossfade(const float* d_prev_tail, long long prev_stride, const float* d_next_head, long long next_stride,
                                 float* d_out, long long out_stride, int n_planes, int n_samples, void* stream);

/*
 * Test aid: after the next decode calls, copy the activation produced by layer `layer` (0-based
 * index into the sequence up_0, res_0_0 .. res_0_{n_res-1}, up_1, ...; -1 disables) of all
 * extended windows to d_dst as fp32, row-major [extended samples at that level, channels].
 * At most `capacity` floats are written.  d_dst is device memory owned by the caller.
 */
DEMON_API demon_status demon_vae_debug_tap(demon_vae* vae, int layer, float* d_dst, size_t capacity);

/*
 * Benchmark instrumentation.  level 0 = off (default); 1 = HIP events on the decode stream at the
 * boundaries gather | convolutions | head | stitch; 2 = an event after every kernel launch.  The
 * events are created here, not in the decode calls.
 */
DEMON_API demon_status demon_vae_set_timing(demon_vae* vae, int level);

/*
 * Elapsed milliseconds between consecutive events, averaged over the decode calls made since the last
 * demon_vae_set_timing / demon_vae_get_timing (at most the last 32; all of them must have had the same
 * layer count); the caller must have synchronised the stream.  Level 1 yields 4 values (gather, all convolutions, head, stitch); level 2
 * yields one value per launch in launch order (gather, then per block the transposed conv and per
 * residual unit the dilated and the 1x1 conv, then head, stitch).  Writes at most `capacity` values
 * to `ms` (host memory) and the number available to *n.
 */
DEMON_API demon_status demon_vae_get_timing(demon_vae* vae, float* ms, int capacity, int* n);

/*
 * Test aids (host only, no GPU): the packed weight layouts the kernels read and the host's fp32 -> half conversion,
 * exported so that the CPU tests can check them against the layouts the kernel comments state.
 *   pack_bf16     : `w` in the PyTorch layout (conv [cout, cin, k]; transposed conv [cin, cout, 2 stride], stride > 0)
 *                   -> blocks [row tile][channel chunk][tap] of the tile variant (0: 128 x 64, 1: 64 x 64, 2: 32 x 16,
 *                   3: 256 x 32), as bf16 or (as_half) the same values as IEEE half; permute_rows: row order of the
 *                   generic kernel's accumulator tiles.  dst holds cout * cin * k (times stride) 16-bit values.
 *   pack_w1_fused : 1x1 weights [c][c] of a fused unit (c = 64, 128), rows and K axis permuted.
 */
DEMON_API void demon_vae_test_pack_bf16(const float* w, int cin, int cout, int ntaps, int stride, int variant,
                                        int as_half, int permute_rows, uint16_t* dst);
DEMON_API void demon_vae_test_pack_w1_fused(const float* w, int c, uint16_t* dst);
DEMON_API uint16_t demon_vae_test_f32_to_f16(float v);

/* Message of the last error returned on this thread (empty string if none). Never NULL. */
DEMON_API const char* demon_vae_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DEMON_VAE_H */
