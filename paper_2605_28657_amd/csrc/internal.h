// Internal declarations shared by the host code and the kernel launchers of libdemon_vae.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/demon_vae.h"

namespace demon {

// ---- error reporting -------------------------------------------------------------------------
demon_status fail(demon_status st, const char* fmt, ...);   // records the thread-local message
void clear_error();

// ---- layer stack (host) ----------------------------------------------------------------------
struct Stack {
    int c0 = 0;
    std::vector<int> strides, widths, dilations;
    int res_kernel = 7, head_kernel = 7, out_channels = 2;
    int total_stride() const { int s = 1; for (int v : strides) s *= v; return s; }
};

// Validates the description and copies it. Returns DEMON_OK or INVALID_ARG (message recorded).
demon_status stack_from_config(const demon_vae_config* cfg, Stack* out);
size_t stack_weight_count(const Stack& st);
void stack_receptive_field(const Stack& st, int* left, int* right);
void stack_forward_support(const Stack& st, long long a, long long b, long long* lo, long long* hi);
size_t stack_encoder_weight_count(const Stack& st);
// halo of the windowed encode in latent frames and (optional) the cone in samples before / after a frame
void stack_encoder_receptive_field(const Stack& st, int* left, int* right, long long* samples_left, long long* samples_right);

// ---- windows ---------------------------------------------------------------------------------
// One extended window ("slot") as the kernels see it.  Frames are latent frames; at a level with
// R samples per frame the slot owns workspace rows [row0*R, (row0+len)*R).
struct Slot {
    int row0;     // first workspace frame of the slot (prefix sum of len)
    int len;      // extended length hi - lo
    int clip;
    int lo;       // first latent frame of the extended region
    int crop;     // begin - lo: frames trimmed on the left
    int n_int;    // end - begin: interior frames
    int begin;    // interior start (absolute frame)
    int pad;
};

// ---- kernels (launchers; all asynchronous on `stream`) -----------------------------------------
// Activations live in "row-major time x channels" layout: element (row, c) at row*C + c.

// MFMA operand formats of the bf16 path.  Weights are bf16 values in every format (exact in half as well).
enum OperandFmt { OP_BF16 = 0,     // one bf16 plane
                  OP_BF16X2 = 1,   // hi + lo bf16 planes, two MFMAs per k-step
                  OP_F16 = 2 };    // one IEEE half plane, f16 MFMA

struct ConvArgs {
    const void* x;        // input activation [rows_in, cin] (fp32 path: fp32; bf16 path: activated bf16 operand)
    void* y;              // output activation [rows_out, cout] (fp32 path: fp32; bf16 path: half); bf16 dilated conv: unused
    void* ya = nullptr;   // bf16 path: activated bf16 copy of the output for the next layer (Snake out_alpha/out_inv_beta)
    const void* res;      // residual (same layout as y) or nullptr; bf16 path: must equal y (in place)
    const void* w;        // packed weights (layout private to each kernel family)
    const float* bias;    // [cout]
    const float* in_alpha;   const float* in_inv_beta;    // Snake on the input, or nullptr
    const float* out_alpha;  const float* out_inv_beta;   // Snake on the output, or nullptr
    const Slot* slots;    // device
    int n_slots;
    int max_len;          // longest slot (frames)
    int max_int;          // longest interior (frames)
    int margin;           // rows of the OUTPUT level beyond each window's interior that later layers still
                          // read (the shrinking cone of the receptive field); rows further out are not computed
    int r_in;             // samples per frame of the input level
    int cin, cout;
    int ntaps;            // conv: kernel size; convT: 2
    int dil;              // conv: dilation; convT: unused
    int stride;           // 0 = Conv1d; s > 0 = ConvTranspose1d(kernel 2s, stride s, padding s/2)
    int down = 0;         // s > 0 = strided Conv1d(kernel 2s, stride s, padding s/2) (the encoder); ntaps = 2s, stride = 0
    // bf16 path only: format of the MFMA operand read (x) and of the one emitted (ya), see kernels_bf16.hip
    int in_fmt = OP_BF16, out_fmt = OP_BF16;
    long long in_lo_off = 0, out_lo_off = 0;     // OP_BF16X2: element offset of the lo plane
    long long small_tile_wgs = 192;              // bf16 path: a launch of at most this many 128 x 128 tiles uses 64 x 64 tiles (0: never)
    bool wide_tile_ok = true;                    // bf16 path: dilated convs with many columns may use the 128 x 256 tile
};

hipError_t launch_conv_f32(const ConvArgs& a, hipStream_t stream);   // in_alpha must be nullptr (see launch_snake_f32)
hipError_t launch_snake_f32(const float* x, float* y, const float* alpha, const float* inv_beta, int C,
                            size_t n, hipStream_t stream);
// bf16 MFMA implicit GEMM.  `variant` is the tile configuration chosen when the weights were packed.
hipError_t launch_conv_bf16(const ConvArgs& a, int variant, hipStream_t stream);

// Packed weight sizes / packing (host).  w_src is the PyTorch layout: conv [cout, cin, k]; convT [cin, cout, 2s].
size_t packed_f32_count(int cin, int cout, int ntaps, int stride);
void pack_f32(const float* w_src, int cin, int cout, int ntaps, int stride, float* dst);
int  choose_variant_bf16(int cin, int m);   // -1 if unsupported
size_t packed_bf16_count(int cin, int cout, int ntaps, int stride, int variant);
// `as_half`: the 16-bit weights are IEEE half (for a layer whose activation operand is OP_F16), else bf16.
// `permute_rows`: row order of launch_conv_bf16's accumulator tiles (not for the layouts the fused units read).
// `down` = s > 0: a strided Conv1d [cout, cin, 2s] in its merged-row form (see kernels_bf16.hip); ntaps, stride unused.
void pack_bf16(const float* w_src, int cin, int cout, int ntaps, int stride, int variant, bool as_half, bool permute_rows,
               uint16_t* dst, int down = 0);
uint16_t f32_to_bf16_rne(float v);
uint16_t f32_to_f16_rne(float v);

// Fused residual unit (bf16 path, C = 64 or 128): y = x + W1 snake2(W7 (*) snake1(x) + b7) + b1, x != y.
struct FusedArgs {
    const void* x; void* y;  // residual stream in its HBM storage type (half)
    uint16_t* ya = nullptr;  // optional: bf16(snake(y; a3, ib3)) for an unfused consumer
    const float* a3 = nullptr; const float* ib3 = nullptr;
    const uint16_t* w7;      // packed as pack_bf16 does for an MT = C, KC = 64 tile
    const uint16_t* w1;      // packed by pack_w1_fused
    const float* b7; const float* b1;
    const float* a1; const float* ib1; const float* a2; const float* ib2;
    const Slot* slots; int n_slots, max_len, max_int, margin;
    int r, c, ntaps, dil;
    // optional: the decoder's head in the same kernel (64 channels, the unit feeds nothing else; y is then not written).
    // hw: half-precision MFMA fragments (pack_head_mfma), hb bias, ha / hib the head's Snake, hy planar window waveforms
    // [oc][total_rows] (rows counted like the unit's), hk the head's kernel size (odd, <= 7)
    const uint16_t* hw = nullptr; const float* hb = nullptr; const float* ha = nullptr; const float* hib = nullptr;
    float* hy = nullptr; long long total_rows = 0; int oc = 0, hk = 0;
};
hipError_t launch_res_unit_fused(const FusedArgs& a, hipStream_t stream);
void pack_w1_fused(const float* w, int C, uint16_t* dst);

// fused residual unit for 256 channels (kernels_bf16_wide.hip): reads the pre-activated bf16 operand, updates the
// half residual stream in place
struct WideArgs {
    const uint16_t* xa; void* y;
    uint16_t* ya = nullptr;  // optional: bf16(snake(y; a3, ib3)) for the consumer; must not be the buffer of xa
    const float* a3 = nullptr; const float* ib3 = nullptr;
    const uint16_t* w7;      // packed as pack_bf16 does for variant 3 (MT = 256, KC = 32)
    const uint16_t* w1;      // packed by pack_w1_wide
    const float* b7; const float* b1; const float* a2; const float* ib2;
    const Slot* slots; int n_slots, max_len, max_int, margin;
    int r, c, ntaps, dil;
};
hipError_t launch_res_unit_wide(const WideArgs& a, hipStream_t stream);
void pack_w1_wide(const float* w /*[256][256]*/, uint16_t* dst);

struct IoArgs {
    const Slot* slots; int n_slots; int max_len;
};
// latent [n_clips, c0, n_frames] (fp32 or bf16) -> level-0 activation [frames, c0] fp32; with `xa` (bf16 path) the
// activated operand snake(x; alpha, inv_beta) instead, in operand format xa_fmt (lo plane at xa + xa_lo_off)
hipError_t launch_gather(const void* latent, float* x0, int c0, int n_frames, bool bf16,
                         const Slot* slots, int n_slots, int max_len, hipStream_t stream,
                         uint16_t* xa = nullptr, int xa_fmt = OP_BF16, long long xa_lo_off = 0,
                         const float* alpha = nullptr, const float* inv_beta = nullptr);
// encoder stem: Conv1d(k, ch -> C) + bias from the planar fp32 waveform [n_clips, ch, n_frames * S] into the residual
// stream y (half or fp32) of the rows each window needs (interior widened by `margin`); with ya (half path only) also
// the activated operand snake(y; alpha, inv_beta) in format ya_fmt.  w: fp32 [k][ch][C].
hipError_t launch_stem(const float* wave, void* y, bool y_half, uint16_t* ya, int ya_fmt, const float* w, const float* bias,
                       const float* alpha, const float* inv_beta, int ch, int C, int k, int S, int n_frames, int margin,
                       const Slot* slots, int n_slots, int max_len, int max_int, hipStream_t stream);
// encoder: moments of the windows' interior frames -> moments_out fp32 [n_clips, 2 C0, n_frames] and the sampled latent
// [n_clips, C0, n_frames] (bf16 for the half path, fp32 otherwise); eps fp32 [n_clips, C0, n_frames] or nullptr (z = mean)
hipError_t launch_sample(const void* m, bool m_half, const float* eps, float* moments_out, void* latent_out, bool latent_bf16,
                         int C0, int n_frames, const Slot* slots, int n_slots, int max_int, hipStream_t stream);
// head: Snake -> Conv1d(k, cin -> oc) -> tanh; output planar fp32 [oc, total_rows]
// `fast` selects the hardware-sine Snake (alpha given in revolutions) used by the bf16 path.
// `x_half`: the input is the bf16 path's half-precision residual stream, else fp32.
hipError_t launch_head(const void* x, bool x_half, float* y, const float* w /*[k][cin][oc]*/, const float* bias,
                       const float* alpha, const float* inv_beta, int cin, int oc, int k, int r,
                       long long total_rows, bool fast, const Slot* slots, int n_slots, int max_int,
                       hipStream_t stream);
// MFMA head of the bf16 path (cin 32 or 64, oc <= 32); weights packed by pack_head_mfma
size_t head_mfma_frag_count(int cin, int k);          // 16-byte x 64-lane fragments
void pack_head_mfma(const float* w /*[oc][cin][k]*/, int cin, int oc, int k, uint16_t* dst);
hipError_t launch_head_mfma(const void* x, float* y, const uint16_t* wfrag, const float* bias, const float* alpha,
                            const float* inv_beta, int cin, int oc, int k, int r, long long total_rows,
                            const Slot* slots, int n_slots, int max_len, int max_int, hipStream_t stream);
// crop + stitch: planar slot waveform -> d_out [n_clips, oc, n_frames*S]
hipError_t launch_stitch(const float* y, float* out, int oc, int S, int n_frames, long long total_rows,
                         const Slot* slots, int n_slots, int max_int, hipStream_t stream);
// crop + stitch + 16-bit render: planar slot waveform -> d_pcm [n_clips, n_frames*S, oc] interleaved int16
hipError_t launch_stitch_pcm16(const float* y, int16_t* pcm, int oc, int S, int n_frames, long long total_rows,
                               const Slot* slots, int n_slots, int max_int, hipStream_t stream);
// window table written on the device (no host copy); per_clip windows and clip_frames extended frames per clip.
// Windows from index `split` on form the second group: their rows count from `split_row0` (n_clips * per_clip, 0: one group).
hipError_t launch_plan_slots(Slot* dst, int n_clips, int per_clip, int clip_frames, int n_frames, int frame_begin,
                             int frame_end, int window, int halo, int split, int split_row0, hipStream_t stream);
// decode gate: dst = src with the windows of clips whose skip flag is set emptied
hipError_t launch_gate_slots(const Slot* src, Slot* dst, int n, const int* skip, hipStream_t stream);
// latent similarity filter: per clip mse = mean((a-b)^2) over n elements and the gate mse < threshold
hipError_t launch_latent_mse(const void* a, const void* b, int n_clips, long long n, bool bf16, float threshold,
                             float* mse, int* unchanged, hipStream_t stream);
// equal-power crossfade of n_planes planar segments of n samples
hipError_t launch_crossfade(const float* tail, long long tail_stride, const float* head, long long head_stride,
                            float* out, long long out_stride, int n_planes, int n, hipStream_t stream);
// debug tap: activation -> fp32 copy; src_type 0 fp32, 1 bf16, 2 half
hipError_t launch_to_f32(const void* x, float* dst, size_t n, int src_type, hipStream_t stream);

}  // namespace demon
