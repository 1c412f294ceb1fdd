// C ABI of libdemon_vae: decoder construction (weight repacking, workspace), window plans and the
// launch sequence of the windowed decode (paper section 3.6: extend, decode, trim).
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <memory>
#include <mutex>
#include <new>

#include "internal.h"

using namespace demon;

namespace {

constexpr int kMaxSlots = 4096;
constexpr int kPlanCache = 16;
constexpr int kTimingRing = 32;        // decode calls whose events are kept for demon_vae_get_timing
// bf16 path: blocks at least this wide carry their MFMA operands with more mantissa bits than bf16.  There the
// branch gain (weight std x sqrt(fan-in)) is about one, so operand rounding passes into the output at full
// strength.  Default: IEEE half operands on the f16 MFMA for every convolution of such a block (same rate as bf16;
// the operands have the range of the half residual stream they are computed from).  The alternative (config field
// wide_operands) carries hi + lo bf16 pairs instead, for the inputs of the block's transposed conv and of its 1x1
// convs (two MFMAs per k-step there; the dilated convs then take plain bf16).
constexpr int kSplitWidth = 512;
constexpr long long kHeadFusionFrames = 256;   // calls with at most this many extended frames run the head inside the last unit
// Defaults of the config fields wide_operands / flags / small_tile_wgs where they are left at 0, from the environment
// (read once when the library is loaded; for A/B timing of a whole program without touching its configs).
const int g_env_wide_fmt = [] {
    const char* e = getenv("DEMON_VAE_WIDE_OPERANDS");
    return (e && strcmp(e, "bf16x2") == 0) ? (int)OP_BF16X2 : (int)OP_F16;
}();
const bool g_env_no_fused = getenv("DEMON_VAE_NO_FUSED") != nullptr;
const bool g_env_one_stream = getenv("DEMON_VAE_ONE_STREAM") != nullptr;
const long long g_env_small_tile_wgs = [] {
    const char* e = getenv("DEMON_VAE_SMALL_TILE_WGS");
    return e ? atoll(e) : 192ll;
}();

struct ConvLayer {
    int cin = 0, cout = 0, ntaps = 0, dil = 1, stride = 0, variant = -1;
    int down = 0;                      // s > 0: strided Conv1d(kernel 2s, stride s, padding s/2) of the encoder (ntaps = 2s)
    int in_fmt = OP_BF16;              // bf16 path: format of the activation operand (the weights are packed to match)
    bool generic = true;               // bf16 path: runs on launch_conv_bf16 (row order of its accumulator tiles)
    int margin = 0;                    // output rows beyond the interior that later layers read
    const void* w = nullptr;
    const float* bias = nullptr;
    const float* in_alpha = nullptr;   const float* in_inv_beta = nullptr;
    const float* out_alpha = nullptr;  const float* out_inv_beta = nullptr;
};

// fused: one kernel per unit that reads the half residual stream itself (64, 128 channels);
// wide: one kernel per unit that reads the pre-activated operand (256 channels); else two kernels
struct ResUnit { ConvLayer dilated, pointwise; bool fused = false, wide = false; const uint16_t* w1_fused = nullptr; };
// up: the block's resampling layer -- the decoder's transposed conv (before the units) or the encoder's strided conv (after them)
struct Block { ConvLayer up; std::vector<ResUnit> res; };
// The layer sequence in processing order: a resampling convolution (conv) or a residual unit (unit), and the layer that
// takes this step's output as an activated MFMA operand (bf16 path; nullptr: the next layer reads the residual stream).
struct Step { const ConvLayer* conv = nullptr; const ResUnit* unit = nullptr; const ConvLayer* consumer = nullptr; };

struct Plan {
    bool valid = false;
    int n_clips = 0, n_frames = 0, frame_begin = 0, frame_end = 0, window = 0, halo = 0;
    int n_slots = 0, max_len = 0, max_int = 0;
    long long total_frames = 0;
    // The windows form one or two groups of consecutive table entries.  A group owns the workspace region that starts
    // at frame0 x (largest per-frame activation size), and the rows of its windows count from the region's start: two
    // groups can then be at different layers at the same time without touching each other's bytes (the bytes a window
    // occupies depend on the layer's rate x width).
    int n_groups = 1;
    int g_first[2] = {0, 0}, g_count[2] = {0, 0};
    long long g_frame0[2] = {0, 0}, g_frames[2] = {0, 0};
    Slot* d_slots = nullptr;
    unsigned long long last_use = 0;
    // A call on this grid was recorded into a HIP graph: the graph holds the address of this entry's table (and the
    // grid's launch shapes), so the entry is never evicted while the handle lives.
    bool pinned = false;
    // The kernel that writes this entry's table has only been recorded into a graph so far, not executed: the next call
    // on this grid launches it again (eagerly, or into the graph being recorded, which must not depend on another graph
    // having been replayed first).
    bool table_pending = false;
};

// The device memory a decode call works in besides its inputs and outputs: the handle's own (allocated at create) or,
// for demon_vae_decode_windowed_static, pieces of the static scratch array below.
struct Workspace {
    void* buf[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    float* head_out = nullptr;
    Slot* slot_gated = nullptr;
    size_t act_elems = 0;              // elements one activation buffer holds (= offset of the lo plane of a split operand)
};

// Scratch of demon_vae_decode_windowed_static, the entry point for callers that cannot allocate: window table, activation
// buffers and window waveforms of one call.  Every GPU the library runs on holds its own copy until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: kernels get the address looked up there.
constexpr size_t kStaticScratchBytes = DEMON_VAE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};      // per device: address of its copy of `scratch`
std::mutex g_scratch_mutex;

// Address of the current device's copy of the static scratch array (looked up once per device).
hipError_t static_scratch(int device, unsigned char** out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

struct demon_vae {
    Stack st;
    demon_dtype dtype = DEMON_F32;
    int max_frames = 0, max_clips = 0;
    long long cap_frames = 0;
    long long per_frame = 0;           // largest rate x width of a layer: elements of one latent frame at its widest
    int rf_left = 0, rf_right = 0;
    int device = 0;
    bool has_split_operands = false;   // bf16 path: some layer carries its operand as hi + lo planes
    long long small_tile_wgs = 192;    // bf16 path: launches of at most this many 128 x 128 tiles use 64 x 64 tiles
    bool wide_tile_ok = true;          // bf16 path: dilated convs with many columns may use the 128 x 256 tile
    bool head_fusable = false;         // bf16 path: the last layer is a fused 64-channel unit that can run the head in its kernel

    void* d_params = nullptr;          // one allocation: all packed weights, biases, Snake parameters
    std::vector<Block> blocks;         // in processing order (encoder: from the audio rate down)
    std::vector<Step> steps;
    const ConvLayer* first_consumer = nullptr;     // bf16 path: the layer whose operand the gather (stem) writes
    bool encoder = false;              // the mirror path: waveform -> moments / latent
    const float* stem_w = nullptr;  const float* stem_bias = nullptr;      // encoder stem, fp32 [k][channels][C]
    int stem_cout = 0, stem_margin = 0;
    const float* head_w = nullptr;  const float* head_bias = nullptr;
    const uint16_t* head_wfrag = nullptr;   // bf16 path: half-precision MFMA fragments of the head weights (or nullptr)
    const float* head_alpha = nullptr;  const float* head_inv_beta = nullptr;
    int head_cin = 0;

    // fp32 path: residual stream ping/pong + Snake scratch, all fp32.
    // bf16 path: buf[0], buf[1] residual stream ping/pong (half), buf[2] bf16 activated branch tensor,
    // buf[3], buf[4] bf16 activated operand of the next layer (each bf16 buffer: hi plane + lo plane).
    // head_out: planar window waveforms [out_channels, cap_frames*S]; slot_gated: per-call copy of a window table with
    // the skipped clips emptied (gated decode)
    Workspace ws;
    unsigned char* scratch = nullptr;              // this device's copy of the static scratch array
    Slot* d_slot_arena = nullptr;
    hipStream_t stream2 = nullptr;                 // second lane of the bf16 layer sequence (default priority, non-blocking)
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    Plan plans[kPlanCache];
    unsigned long long use_counter = 0;

    int timing = 0;                    // 0 off, 1 group boundaries, 2 every launch
    std::vector<hipEvent_t> events;    // kTimingRing sets of marks_per_call events
    int marks_per_call = 0;
    int n_marks = 0;                   // marks recorded by the current/last call
    int timed_calls = 0;               // calls recorded since the last set_timing / get_timing

    int tap_layer = -1;
    float* tap_dst = nullptr;
    size_t tap_cap = 0;
};

namespace {

// Host-side staging of the parameter arena: offsets are assigned while packing, pointers afterwards.
struct Arena {
    std::vector<unsigned char> bytes;
    size_t reserve(size_t n) {
        const size_t off = (bytes.size() + 255) & ~(size_t)255;
        bytes.resize(off + n);
        return off;
    }
};

struct SnakeOff { size_t alpha, inv_beta; };

SnakeOff pack_snake(Arena& ar, const float* alpha, const float* beta, int c, bool fast)
{
    SnakeOff o;
    o.alpha = ar.reserve(sizeof(float) * c);
    o.inv_beta = ar.reserve(sizeof(float) * c);
    float* a = reinterpret_cast<float*>(ar.bytes.data() + o.alpha);
    float* b = reinterpret_cast<float*>(ar.bytes.data() + o.inv_beta);
    for (int i = 0; i < c; ++i) {
        // the fast Snake feeds the hardware sine, which takes revolutions
        a[i] = fast ? (float)((double)alpha[i] / (2.0 * M_PI)) : alpha[i];
        b[i] = (float)(1.0 / ((double)beta[i] + 1e-9));
    }
    return o;
}

size_t pack_floats(Arena& ar, const float* src, size_t n)
{
    const size_t off = ar.reserve(sizeof(float) * n);
    memcpy(ar.bytes.data() + off, src, sizeof(float) * n);
    return off;
}

size_t pack_conv(Arena& ar, const float* w, ConvLayer& L, bool bf16)
{
    if (bf16) {
        const size_t n = packed_bf16_count(L.cin, L.cout, L.ntaps, L.stride, L.variant);
        const size_t off = ar.reserve(n * 2);
        pack_bf16(w, L.cin, L.cout, L.ntaps, L.stride, L.variant, L.in_fmt == OP_F16, L.generic, reinterpret_cast<uint16_t*>(ar.bytes.data() + off), L.down);
        return off;
    }
    const size_t n = packed_f32_count(L.cin, L.cout, L.ntaps, L.stride);
    const size_t off = ar.reserve(n * 4);
    pack_f32(w, L.cin, L.cout, L.ntaps, L.stride, reinterpret_cast<float*>(ar.bytes.data() + off));
    return off;
}

demon_status hip_fail(hipError_t e, const char* what)
{
    return fail(DEMON_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// The window grid of one clip, walked on the host: windows, extended frames, longest window and interior.
struct GridCount { long long per_clip = 0, clip_frames = 0; int max_len = 0, max_int = 0; };

GridCount count_grid(int n_frames, int fb, int fe, int window, int halo)
{
    GridCount g;
    for (long long b = fb; b < fe; b += window) {
        const long long e = std::min<long long>(b + window, fe);
        const int len = (int)(std::min<long long>(n_frames, e + halo) - std::max<long long>(0, b - halo));
        g.clip_frames += len;
        g.max_len = std::max(g.max_len, len);
        g.max_int = std::max(g.max_int, (int)(e - b));
        ++g.per_clip;
    }
    return g;
}

#define HIP_TRY(expr, what) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_fail(e_, what); } while (0)

// bf16 path: a window's activation plane is addressed with 32-bit byte offsets through a buffer descriptor
demon_status check_plane(const demon_vae* v, int max_len)
{
    if (v->dtype != DEMON_BF16) return DEMON_OK;
    const long long bytes = (long long)max_len * v->per_frame * 2;
    if (bytes > 0xf0000000ll)
        return fail(DEMON_ERR_UNSUPPORTED, "a window of %d frames has an activation plane of %lld bytes; the kernels address one window "
                    "with 32-bit offsets (limit %lld bytes): decode it in several windows", max_len, bytes, 0xf0000000ll);
    return DEMON_OK;
}

// Looks the window grid up in the plan cache; on a miss the table of the least recently used entry that no graph holds is
// rewritten by a small kernel on the decode stream, so the call stays asynchronous (kernels of earlier calls that still
// read the replaced table precede that kernel on the stream) and can itself be recorded into a graph.
demon_status get_plan(demon_vae* v, int n_clips, int n_frames, int fb, int fe, int window, int halo, bool two_groups,
                      hipStream_t stream, Plan** out)
{
    ++v->use_counter;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing(stream, &cap), "hipStreamIsCapturing");
    const bool capturing = cap != hipStreamCaptureStatusNone;
    Plan* victim = nullptr;
    for (Plan& p : v->plans) {
        if (p.valid && p.n_clips == n_clips && p.n_frames == n_frames && p.frame_begin == fb && p.frame_end == fe &&
            p.window == window && p.halo == halo && (p.n_groups == 2) == (two_groups && p.n_slots >= 2)) {
            p.last_use = v->use_counter;
            if (capturing) p.pinned = true;
            if (p.table_pending) {
                const int split = p.n_groups == 2 ? p.g_first[1] : p.n_slots;
                HIP_TRY(launch_plan_slots(p.d_slots, p.n_clips, p.n_slots / p.n_clips, (int)(p.total_frames / p.n_clips), p.n_frames,
                                          p.frame_begin, p.frame_end, p.window, p.halo, split, (int)p.g_frame0[1], stream), "window table");
                if (!capturing) p.table_pending = false;
            }
            *out = &p;
            return DEMON_OK;
        }
        if (p.pinned) continue;
        if (!victim || (victim->valid && (!p.valid || p.last_use < victim->last_use))) victim = &p;
    }
    if (!victim)
        return fail(DEMON_ERR_WORKSPACE, "all %d cached window grids are held by recorded graphs; a further grid needs another handle", kPlanCache);
    const GridCount gc = count_grid(n_frames, fb, fe, window, halo);
    const long long n_slots = gc.per_clip * n_clips;
    if (n_slots > kMaxSlots)
        return fail(DEMON_ERR_WORKSPACE, "%lld windows exceed the limit of %d", n_slots, kMaxSlots);
    const long long total = gc.clip_frames * n_clips;
    if (total > v->cap_frames)
        return fail(DEMON_ERR_WORKSPACE, "extended windows need %lld frames, the workspace holds %lld", total, v->cap_frames);
    const demon_status prc = check_plane(v, gc.max_len);
    if (prc != DEMON_OK) return prc;
    // two groups of about equal size (in frames) for the bf16 path, whose layer sequence can run on two streams: the
    // second group starts at the window whose first row is nearest to half of the rows
    int n_groups = 1, split = (int)n_slots;
    long long frame0_b = 0;
    if (two_groups && n_slots >= 2) {
        long long best = -1, row = 0, i = 0;
        for (int c = 0; c < n_clips; ++c)
            for (long long b = fb; b < fe; b += window, ++i) {
                const long long e = std::min<long long>(b + window, fe);
                const long long d = row > total - row ? row - (total - row) : (total - row) - row;
                if (i >= 1 && (best < 0 || d < best)) { best = d; split = (int)i; frame0_b = row; }
                row += std::min<long long>(n_frames, e + halo) - std::max<long long>(0, b - halo);
            }
        n_groups = 2;
    }
    const int idx = (int)(victim - v->plans);
    Slot* d = v->d_slot_arena + (size_t)idx * kMaxSlots;
    victim->valid = false;
    HIP_TRY(launch_plan_slots(d, n_clips, (int)gc.per_clip, (int)gc.clip_frames, n_frames, fb, fe, window, halo, split, (int)frame0_b, stream),
            "window table");
    victim->valid = true;
    victim->pinned = capturing;
    victim->table_pending = capturing;
    victim->n_clips = n_clips; victim->n_frames = n_frames; victim->frame_begin = fb; victim->frame_end = fe;
    victim->window = window; victim->halo = halo;
    victim->n_slots = (int)n_slots; victim->max_len = gc.max_len; victim->max_int = gc.max_int;
    victim->total_frames = total; victim->d_slots = d; victim->last_use = v->use_counter;
    victim->n_groups = n_groups;
    victim->g_first[0] = 0; victim->g_count[0] = split; victim->g_frame0[0] = 0; victim->g_frames[0] = n_groups == 2 ? frame0_b : total;
    victim->g_first[1] = split; victim->g_count[1] = (int)n_slots - split; victim->g_frame0[1] = frame0_b; victim->g_frames[1] = total - frame0_b;
    *out = victim;
    return DEMON_OK;
}


// two window groups on two streams unless a mode wants one ordered launch sequence (per-launch timing, debug tap)
bool wants_two_groups(const demon_vae* v)
{
    return v->dtype == DEMON_BF16 && v->stream2 && v->timing < 2 && !(v->tap_layer >= 0 && v->tap_dst);
}

// What one call reads and writes besides the handle's own memory.
struct Io {
    // decode: latent in, waveform (fp32 planar or interleaved int16) out, optional per-clip skip flags
    const void* d_latent = nullptr; const int* d_skip = nullptr; float* d_out = nullptr; int16_t* d_pcm = nullptr;
    // encode: waveform in, moments and / or sampled latent out, optional noise of the sampling step
    const float* d_wave = nullptr; const float* d_eps = nullptr; float* d_moments = nullptr; void* d_zout = nullptr;
    int n_frames = 0;
};

// The launch sequence of one call over the windows of `plan`, in the memory of `ws`: the decoder's
// gather | layers | head | stitch, or the encoder's stem | layers | sampling step.
demon_status run_pass(demon_vae* v, const Workspace& ws, const Plan* plan, const Io& io, hipStream_t stream)
{
    const bool bf = v->dtype == DEMON_BF16;
    const bool enc = v->encoder;
    const bool dual = wants_two_groups(v);
    // the head inside the last unit's kernel, unless the debug tap wants that unit's output in memory
    // (bit-identical either way).  Only for calls of a few windows, where a launch less is what counts: for a whole clip
    // the fused launch takes as long as the two it replaces.
    const bool head_in_unit = v->head_fusable && !(v->tap_layer >= 0 && v->tap_dst) && plan->total_frames <= kHeadFusionFrames;
    const int n_frames = io.n_frames;
    const Slot* slots = plan->d_slots;
    const int ns = plan->n_slots, ml = plan->max_len;
    if (io.d_skip) {
        // gated decode: every kernel reads a copy of the table in which the skipped clips' windows are empty
        HIP_TRY(launch_gate_slots(plan->d_slots, ws.slot_gated, ns, io.d_skip, stream), "decode gate");
        slots = ws.slot_gated;
    }

    // the convolution launches address a group of windows (gs, gn) on a stream gst: all windows on the caller's
    // stream, or two halves on two streams (see the bf16 path below)
    const Slot* gs = slots;
    int gn = ns, g = 0;
    hipStream_t gst = stream;
    bool marks_on = true;
    auto select_group = [&](int which, hipStream_t on) {
        g = which; gs = slots + plan->g_first[which]; gn = plan->g_count[which]; gst = on;
    };
    // element offset of the current group's region in every activation buffer
    auto goff = [&]() -> size_t { return (size_t)plan->g_frame0[g] * (size_t)v->per_frame; };

    v->n_marks = 0;
    const int ring_base = (v->timed_calls % kTimingRing) * v->marks_per_call;
    auto mark = [&](int level) -> hipError_t {
        if (!marks_on || v->timing < level || v->n_marks >= v->marks_per_call) return hipSuccess;
        return hipEventRecord(v->events[ring_base + v->n_marks++], stream);
    };
    // level 1 marks: start, after gather (stem), after the last convolution, after head (sampling step), after stitch.
    // level 2 adds a mark after every convolution launch.
    HIP_TRY(mark(1), "event");

    const int S = v->st.total_stride();
    void* cur = ws.buf[0];
    void* other = ws.buf[1];
    int r = enc ? S : 1, layer_id = 0;
    const size_t n_steps = v->steps.size();
    const long long lo_off = (long long)ws.act_elems;        // lo plane of a split bf16 tensor
    auto tap = [&](const void* x, int c) -> hipError_t {
        const int id = layer_id++;
        if (id != v->tap_layer || !v->tap_dst) return hipSuccess;
        // the groups' regions are apart in the workspace; the tap lays them end to end
        const size_t first = (size_t)plan->g_frame0[g] * r * c, want = (size_t)plan->g_frames[g] * r * c;
        if (first >= v->tap_cap) return hipSuccess;
        return launch_to_f32(x, v->tap_dst + first, std::min(want, v->tap_cap - first), bf ? 2 : 0, gst);
    };
    auto conv_args = [&](const ConvLayer& L, const void* x, void* y, const void* res) {
        ConvArgs a;
        a.x = x; a.y = y; a.res = res; a.w = L.w; a.bias = L.bias;
        a.in_alpha = L.in_alpha; a.in_inv_beta = L.in_inv_beta;
        a.out_alpha = L.out_alpha; a.out_inv_beta = L.out_inv_beta;
        a.slots = gs; a.n_slots = gn; a.max_len = ml; a.max_int = plan->max_int; a.margin = L.margin; a.r_in = r;
        a.cin = L.cin; a.cout = L.cout; a.ntaps = L.ntaps; a.dil = L.dil; a.stride = L.stride; a.down = L.down;
        a.in_fmt = L.in_fmt;
        a.in_lo_off = a.out_lo_off = lo_off;
        a.small_tile_wgs = v->small_tile_wgs;
        a.wide_tile_ok = v->wide_tile_ok;
        return a;
    };
    // samples per frame after a resampling layer
    auto resampled = [](int rate, const ConvLayer& L) { return L.down > 0 ? rate / L.down : rate * L.stride; };

    if (!bf) {
        // ---- fp32 path: Snake on a layer's input runs as its own kernel into buf[2]
        if (enc)
            HIP_TRY(launch_stem(io.d_wave, cur, false, nullptr, 0, v->stem_w, v->stem_bias, nullptr, nullptr, v->st.out_channels,
                                v->stem_cout, v->st.head_kernel, S, n_frames, v->stem_margin, slots, ns, ml, plan->max_int, stream), "stem");
        else
            HIP_TRY(launch_gather(io.d_latent, (float*)cur, v->st.c0, n_frames, false, slots, ns, ml, stream), "gather");
        HIP_TRY(mark(1), "event");
        auto run_conv = [&](const ConvLayer& L, const void* x, void* y, const void* res) -> hipError_t {
            ConvArgs a = conv_args(L, x, y, res);
            if (L.in_alpha) {
                hipError_t e = launch_snake_f32((const float*)x, (float*)ws.buf[2], L.in_alpha, L.in_inv_beta, L.cin,
                                                (size_t)plan->total_frames * r * L.cin, stream);
                if (e != hipSuccess) return e;
                a.x = ws.buf[2];
                a.in_alpha = a.in_inv_beta = nullptr;
            }
            return launch_conv_f32(a, stream);
        };
        for (size_t si = 0; si < n_steps; ++si) {
            const Step& T = v->steps[si];
            const bool last = si + 1 == n_steps;
            if (T.conv) {
                HIP_TRY(run_conv(*T.conv, cur, other, nullptr), "resampling convolution");
                HIP_TRY(mark(last ? 1 : 2), "event");
                std::swap(cur, other);
                r = resampled(r, *T.conv);
                HIP_TRY(tap(cur, T.conv->cout), "debug tap");
            } else {
                const ResUnit& U = *T.unit;
                HIP_TRY(run_conv(U.dilated, cur, other, nullptr), "dilated convolution");
                HIP_TRY(mark(2), "event");
                HIP_TRY(run_conv(U.pointwise, other, cur, cur), "pointwise convolution");   // in place on the residual stream
                HIP_TRY(mark(last ? 1 : 2), "event");
                HIP_TRY(tap(cur, U.pointwise.cout), "debug tap");
            }
        }
    } else {
        // ---- bf16 path.  h (half) ping-pongs between buf[0] and buf[1]; the activated bf16 operand `a` of the
        // next layer that wants one ping-pongs between buf[3] and buf[4]; buf[2] holds the activated branch tensor
        // between the dilated and the 1x1 conv of a two-kernel unit.  Each producer writes `a` with its consumer's Snake.
        uint16_t* acur = (uint16_t*)ws.buf[3];
        uint16_t* aoth = (uint16_t*)ws.buf[4];
        uint16_t* mid = (uint16_t*)ws.buf[2];
        for (int gi = 0; gi < plan->n_groups; ++gi) {
            select_group(gi, stream);
            if (enc) {
                const ConvLayer* C = v->first_consumer;
                HIP_TRY(launch_stem(io.d_wave, (uint16_t*)ws.buf[0] + goff(), true, C ? (uint16_t*)ws.buf[3] + goff() : nullptr,
                                    C ? C->in_fmt : 0, v->stem_w, v->stem_bias, C ? C->in_alpha : nullptr, C ? C->in_inv_beta : nullptr,
                                    v->st.out_channels, v->stem_cout, v->st.head_kernel, S, n_frames, v->stem_margin, gs, gn, ml,
                                    plan->max_int, stream), "stem");
            } else {
                const ConvLayer& U0 = *v->first_consumer;
                HIP_TRY(launch_gather(io.d_latent, nullptr, v->st.c0, n_frames, true, gs, gn, ml, stream, (uint16_t*)ws.buf[3] + goff(),
                                      U0.in_fmt, lo_off, U0.in_alpha, U0.in_inv_beta), "gather");
            }
        }
        HIP_TRY(mark(1), "event");
        auto layers = [&]() -> demon_status {
        cur = (uint16_t*)ws.buf[0] + goff(); other = (uint16_t*)ws.buf[1] + goff();      // half: 2 bytes
        acur = (uint16_t*)ws.buf[3] + goff(); aoth = (uint16_t*)ws.buf[4] + goff(); mid = (uint16_t*)ws.buf[2] + goff();
        r = enc ? S : 1; layer_id = 0;
        for (size_t si = 0; si < n_steps; ++si) {
            const Step& T = v->steps[si];
            const bool last = si + 1 == n_steps;
            // the layer that consumes this step's output through an activated operand; nullptr when that layer reads the
            // residual stream itself (narrow fused unit, head, sampling step)
            const ConvLayer* C = T.consumer;
            if (T.conv) {
                ConvArgs a = conv_args(*T.conv, acur, other, nullptr);
                if (C) { a.ya = aoth; a.out_alpha = C->in_alpha; a.out_inv_beta = C->in_inv_beta; a.out_fmt = C->in_fmt; }
                HIP_TRY(launch_conv_bf16(a, T.conv->variant, gst), "resampling convolution");
                if (C) std::swap(acur, aoth);
                HIP_TRY(mark(last ? 1 : 2), "event");
                std::swap(cur, other);
                r = resampled(r, *T.conv);
                HIP_TRY(tap(cur, T.conv->cout), "debug tap");
                continue;
            }
            const ResUnit& U = *T.unit;
            if (U.fused) {
                FusedArgs f;
                f.x = cur; f.y = other;
                if (C) { f.ya = acur; f.a3 = C->in_alpha; f.ib3 = C->in_inv_beta; }
                f.w7 = (const uint16_t*)U.dilated.w; f.w1 = U.w1_fused;
                f.b7 = U.dilated.bias; f.b1 = U.pointwise.bias;
                f.a1 = U.dilated.in_alpha; f.ib1 = U.dilated.in_inv_beta;
                f.a2 = U.dilated.out_alpha; f.ib2 = U.dilated.out_inv_beta;
                f.slots = gs; f.n_slots = gn; f.max_len = ml; f.max_int = plan->max_int; f.margin = U.pointwise.margin;
                f.r = r; f.c = U.dilated.cin; f.ntaps = U.dilated.ntaps; f.dil = U.dilated.dil;
                if (C && C->in_fmt != OP_BF16) return fail(DEMON_ERR_UNSUPPORTED, "a fused unit cannot feed a layer with wide operands");
                if (last && head_in_unit) {
                    f.hw = v->head_wfrag; f.hb = v->head_bias; f.ha = v->head_alpha; f.hib = v->head_inv_beta;
                    f.hy = ws.head_out + plan->g_frame0[g] * r; f.total_rows = plan->total_frames * r;
                    f.oc = v->st.out_channels; f.hk = v->st.head_kernel;
                }
                HIP_TRY(launch_res_unit_fused(f, gst), "fused residual unit");
                std::swap(cur, other);
                HIP_TRY(mark(2), "event");
            } else if (U.wide) {
                WideArgs f;
                f.xa = acur; f.y = cur;
                if (C) { f.ya = aoth; f.a3 = C->in_alpha; f.ib3 = C->in_inv_beta; }
                f.w7 = (const uint16_t*)U.dilated.w; f.w1 = U.w1_fused;
                f.b7 = U.dilated.bias; f.b1 = U.pointwise.bias;
                f.a2 = U.dilated.out_alpha; f.ib2 = U.dilated.out_inv_beta;
                f.slots = gs; f.n_slots = gn; f.max_len = ml; f.max_int = plan->max_int; f.margin = U.pointwise.margin;
                f.r = r; f.c = U.dilated.cin; f.ntaps = U.dilated.ntaps; f.dil = U.dilated.dil;
                if (C && C->in_fmt != OP_BF16) return fail(DEMON_ERR_UNSUPPORTED, "a fused unit cannot feed a layer with wide operands");
                HIP_TRY(launch_res_unit_wide(f, gst), "fused residual unit (256 channels)");
                if (C) std::swap(acur, aoth);
                HIP_TRY(mark(2), "event");
            } else {
                ConvArgs d = conv_args(U.dilated, acur, nullptr, nullptr);
                d.ya = mid; d.out_fmt = U.pointwise.in_fmt;   // Snake between the convolutions: the layer's own out_alpha
                HIP_TRY(launch_conv_bf16(d, U.dilated.variant, gst), "dilated convolution");
                HIP_TRY(mark(2), "event");
                ConvArgs q = conv_args(U.pointwise, mid, cur, cur);   // in place on the residual stream
                if (C) { q.ya = acur; q.out_alpha = C->in_alpha; q.out_inv_beta = C->in_inv_beta; q.out_fmt = C->in_fmt; }
                HIP_TRY(launch_conv_bf16(q, U.pointwise.variant, gst), "pointwise convolution");
            }
            HIP_TRY(mark(last ? 1 : 2), "event");
            HIP_TRY(tap(cur, U.pointwise.cout), "debug tap");
        }
        return DEMON_OK;
        };
        // Windows are independent through the whole stack, so the layer sequence can run as two sequences over half of
        // the windows each, on two streams: the ramp and tail of one sequence's launches (a last round of workgroups
        // that fills a fraction of the CUs, prologues, epilogues) overlap with the other's.  Not with per-launch
        // timing or the debug tap, which want one ordered sequence.
        const bool two = dual && plan->n_groups == 2;
        if (two) {
            marks_on = false;
            HIP_TRY(hipEventRecord(v->ev_fork, stream), "event");
            HIP_TRY(hipStreamWaitEvent(v->stream2, v->ev_fork, 0), "hipStreamWaitEvent");
        }
        demon_status lrc = DEMON_OK;
        for (int gi = 0; gi < plan->n_groups && lrc == DEMON_OK; ++gi) {
            select_group(gi, two && gi == 1 ? v->stream2 : stream);
            lrc = layers();
        }
        if (two) {
            // also after a failed launch: the second stream joins the caller's again (an open capture stays well-formed)
            const hipError_t e1 = hipEventRecord(v->ev_join, v->stream2);
            const hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(stream, v->ev_join, 0) : e1;
            if (lrc != DEMON_OK) return lrc;
            HIP_TRY(e2, "joining the second stream");
            marks_on = true;
            HIP_TRY(mark(1), "event");                       // after the last convolution
        }
        if (lrc != DEMON_OK) return lrc;
    }
    const size_t hbytes = bf ? 2 : sizeof(float);                           // half or fp32 residual stream
    const char* final_base = (const char*)cur - goff() * hbytes;           // the buffer the last layer wrote, without the group offset
    if (enc) {
        // sampling step on the moments, trim and scatter into the caller's [clip, channel, frame] arrays
        for (int gi = 0; gi < plan->n_groups; ++gi) {
            select_group(gi, stream);
            HIP_TRY(launch_sample(final_base + goff() * hbytes, bf, io.d_eps, io.d_moments, io.d_zout, bf, v->st.c0, n_frames, gs, gn,
                                  plan->max_int, stream), "sampling step");
        }
        HIP_TRY(mark(1), "event");
        if (v->timing > 0) ++v->timed_calls;
        return DEMON_OK;
    }
    // head and stitch, group by group on the caller's stream; the window waveforms are planar [channel][all rows]
    const long long total_rows = plan->total_frames * r;
    for (int gi = 0; gi < plan->n_groups && !head_in_unit; ++gi) {
        select_group(gi, stream);
        const void* x = final_base + goff() * hbytes;
        float* y = ws.head_out + plan->g_frame0[gi] * r;
        if (v->head_wfrag) {
            HIP_TRY(launch_head_mfma(x, y, v->head_wfrag, v->head_bias, v->head_alpha, v->head_inv_beta, v->head_cin,
                                     v->st.out_channels, v->st.head_kernel, r, total_rows, gs, gn, ml, plan->max_int, stream), "head");
        } else {
            HIP_TRY(launch_head(x, bf, y, v->head_w, v->head_bias, v->head_alpha, v->head_inv_beta, v->head_cin,
                                v->st.out_channels, v->st.head_kernel, r, total_rows, bf, gs, gn, plan->max_int, stream), "head");
        }
    }
    HIP_TRY(mark(1), "event");
    for (int gi = 0; gi < plan->n_groups; ++gi) {
        select_group(gi, stream);
        const float* y = ws.head_out + plan->g_frame0[gi] * r;
        if (io.d_pcm)
            HIP_TRY(launch_stitch_pcm16(y, io.d_pcm, v->st.out_channels, r, n_frames, total_rows, gs, gn, plan->max_int, stream), "stitch");
        else
            HIP_TRY(launch_stitch(y, io.d_out, v->st.out_channels, r, n_frames, total_rows, gs, gn, plan->max_int, stream), "stitch");
    }
    HIP_TRY(mark(1), "event");
    if (v->timing > 0) ++v->timed_calls;
    return DEMON_OK;
}

// Builds a decoder (encoder = false) or its mirror, the encoder (true), on the current device.
demon_status create_impl(const demon_vae_config* cfg, const float* host_weights, size_t n_floats, bool encoder, demon_vae** out)
{
    clear_error();
    if (!out) return fail(DEMON_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!host_weights) return fail(DEMON_ERR_INVALID_ARG, "host_weights is NULL");
    Stack st;
    demon_status rc = stack_from_config(cfg, &st);
    if (rc != DEMON_OK) return rc;
    if (cfg->dtype != DEMON_F32 && cfg->dtype != DEMON_BF16) return fail(DEMON_ERR_INVALID_ARG, "unknown dtype %d", (int)cfg->dtype);
    if (cfg->max_frames < 1 || cfg->max_clips < 1) return fail(DEMON_ERR_INVALID_ARG, "max_frames and max_clips must be >= 1");
    const size_t need = encoder ? stack_encoder_weight_count(st) : stack_weight_count(st);
    if (n_floats != need) return fail(DEMON_ERR_INVALID_ARG, "got %zu weights, the layer stack needs %zu", n_floats, need);
    const bool bf = cfg->dtype == DEMON_BF16;
    if (cfg->wide_operands < 0 || cfg->wide_operands > 2) return fail(DEMON_ERR_INVALID_ARG, "wide_operands must be 0, 1 or 2");
    if (cfg->flags & ~(DEMON_VAE_FLAG_NO_FUSED | DEMON_VAE_FLAG_ONE_STREAM | DEMON_VAE_FLAG_NO_WIDE_TILE | DEMON_VAE_FLAG_NO_HEAD_FUSION)) return fail(DEMON_ERR_INVALID_ARG, "unknown flag bits 0x%x", (unsigned)cfg->flags);
    // 0 in a field = the default, which the environment may have changed (see the header)
    const int g_wide_fmt = cfg->wide_operands == 1 ? (int)OP_F16 : cfg->wide_operands == 2 ? (int)OP_BF16X2 : g_env_wide_fmt;
    const bool g_allow_fused = !((cfg->flags & DEMON_VAE_FLAG_NO_FUSED) || g_env_no_fused);
    const bool g_dual_stream = !((cfg->flags & DEMON_VAE_FLAG_ONE_STREAM) || g_env_one_stream);
    if (bf) {
        if (st.c0 % 16) return fail(DEMON_ERR_UNSUPPORTED, "bf16 path: latent_channels %d is not a multiple of 16", st.c0);
        for (int c : st.widths)
            if (c % 32) return fail(DEMON_ERR_UNSUPPORTED, "bf16 path: width %d is not a multiple of 32", c);
        for (int d : st.dilations)
            if ((st.res_kernel - 1) * d > 64)
                return fail(DEMON_ERR_UNSUPPORTED, "bf16 path: kernel %d with dilation %d spans more than 64 samples", st.res_kernel, d);
        if (encoder && g_wide_fmt == OP_BF16X2)
            return fail(DEMON_ERR_UNSUPPORTED, "the encoder's strided convolutions take one operand plane: wide_operands = 2 is for decoders");
    }
    if (st.head_kernel > 15) return fail(DEMON_ERR_UNSUPPORTED, "head_kernel %d exceeds 15", st.head_kernel);
    if (encoder && st.widths.back() % 8) return fail(DEMON_ERR_UNSUPPORTED, "encoder: the stem's width %d is not a multiple of 8", st.widths.back());

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(DEMON_ERR_HIP, "no HIP device available");

    std::unique_ptr<demon_vae> v(new (std::nothrow) demon_vae);
    if (!v) return fail(DEMON_ERR_HIP, "out of host memory");

    v->st = st; v->dtype = cfg->dtype; v->max_frames = cfg->max_frames; v->max_clips = cfg->max_clips;
    v->encoder = encoder;
    if (cfg->max_extended_frames < 0) return fail(DEMON_ERR_INVALID_ARG, "max_extended_frames must be >= 0");
    v->cap_frames = cfg->max_extended_frames > 0 ? cfg->max_extended_frames : 3ll * cfg->max_frames * cfg->max_clips;
    if (encoder) stack_encoder_receptive_field(st, &v->rf_left, &v->rf_right, nullptr, nullptr);
    else stack_receptive_field(st, &v->rf_left, &v->rf_right);
    v->wide_tile_ok = !(cfg->flags & DEMON_VAE_FLAG_NO_WIDE_TILE);
    v->small_tile_wgs = cfg->small_tile_wgs > 0 ? cfg->small_tile_wgs : cfg->small_tile_wgs < 0 ? 0 : g_env_small_tile_wgs;
    if (hipGetDevice(&v->device) != hipSuccess) return fail(DEMON_ERR_HIP, "hipGetDevice failed");
    {
        // the static scratch array of demon_vae_decode_windowed_static: its address on this device
        const hipError_t se = static_scratch(v->device, &v->scratch);
        if (se != hipSuccess) return hip_fail(se, "hipGetSymbolAddress(static scratch)");
    }

    // ---- pack parameters (offsets first, device pointers after the upload)
    Arena ar;
    struct Pending { ConvLayer* L; size_t w, bias; SnakeOff in, outp; bool has_in, has_out; };
    std::vector<Pending> pend;
    struct FusedFix { ResUnit* U; size_t off; };
    std::vector<FusedFix> fused_fix;
    const int nb = (int)st.strides.size(), nres = (int)st.dilations.size();
    v->blocks.resize(nb);
    for (int b = 0; b < nb; ++b) v->blocks[b].res.resize(nres);

    const float* w = host_weights;
    // one residual unit of width c whose output goes, as an operand, to a layer of format `next_fmt`
    auto pack_unit = [&](ResUnit& U, int c, int j, int next_fmt) -> demon_status {
        ConvLayer& D = U.dilated;
        D.cin = c; D.cout = c; D.ntaps = st.res_kernel; D.dil = st.dilations[j];
        ConvLayer& P = U.pointwise;
        P.cin = c; P.cout = c; P.ntaps = 1; P.dil = 1;
        const bool wide_ops = bf && c >= kSplitWidth;
        P.in_fmt = wide_ops ? g_wide_fmt : (int)OP_BF16;
        if (P.in_fmt == OP_BF16X2) v->has_split_operands = true;
        D.in_fmt = (wide_ops && g_wide_fmt == OP_F16) ? (int)OP_F16 : (int)OP_BF16;
        if (bf) {
            D.variant = choose_variant_bf16(c, c);
            P.variant = choose_variant_bf16(c, c);
            if (D.variant < 0 || P.variant < 0) return fail(DEMON_ERR_UNSUPPORTED, "bf16 path: no kernel for %d channels", c);
        }
        // a fused unit writes plain bf16 operands: a unit stays on the two-kernel path when the layer after it wants
        // its input in a wider format
        const bool feeds_split = next_fmt != OP_BF16;
        U.fused = bf && (c == 64 || c == 128) && (st.res_kernel - 1) * st.dilations[j] <= 64 && !wide_ops && g_allow_fused && !feeds_split;
        if (U.fused) { D.variant = (c == 64) ? 1 : 0; D.generic = false; }     // weight blocks of C x 64
        U.wide = bf && c == 256 && (st.res_kernel - 1) * st.dilations[j] <= 64 && !wide_ops && g_allow_fused && !feeds_split;
        if (U.wide) { D.variant = 3; D.generic = false; }                      // weight blocks of 256 x 32
        Pending pd{&D, 0, 0, {}, {}, true, true};
        pd.in = pack_snake(ar, w, w + c, c, bf);     w += 2 * c;
        pd.w = pack_conv(ar, w, D, bf);              w += (size_t)c * c * st.res_kernel;
        pd.bias = pack_floats(ar, w, c);             w += c;
        pd.outp = pack_snake(ar, w, w + c, c, bf);   w += 2 * c;      // Snake between the two convolutions
        Pending pp{&P, 0, 0, {}, {}, false, false};
        if (U.fused || U.wide) {
            const size_t off = ar.reserve((size_t)c * c * 2);
            if (U.wide) pack_w1_wide(w, reinterpret_cast<uint16_t*>(ar.bytes.data() + off));
            else pack_w1_fused(w, c, reinterpret_cast<uint16_t*>(ar.bytes.data() + off));
            fused_fix.push_back({&U, off});
        }
        pp.w = pack_conv(ar, w, P, bf);              w += (size_t)c * c;
        pp.bias = pack_floats(ar, w, c);             w += c;
        pend.push_back(pd);
        pend.push_back(pp);
        return DEMON_OK;
    };
    auto wide_fmt_of = [&](int width) { return (bf && width >= kSplitWidth) ? g_wide_fmt : (int)OP_BF16; };

    long long per_frame = st.c0, rate = 1;
    size_t stem_w_off = 0, stem_b_off = 0;
    SnakeOff hs{};  size_t hw = 0, hwf = 0, hb = 0;  bool head_mfma = false;
    const int oc = st.out_channels, hk = st.head_kernel;
    if (!encoder) {
        int cin = st.c0;
        for (int l = 0; l < nb; ++l) {
            const int s = st.strides[l], c = st.widths[l];
            Block& B = v->blocks[l];
            {
                ConvLayer& L = B.up;
                L.cin = cin; L.cout = c; L.ntaps = 2; L.stride = s;
                L.in_fmt = wide_fmt_of(c);
                if (L.in_fmt == OP_BF16X2) v->has_split_operands = true;
                if (bf) {
                    L.variant = choose_variant_bf16(cin, s * c);
                    if (L.variant < 0) return fail(DEMON_ERR_UNSUPPORTED, "bf16 path: no kernel for a %d -> %d stride-%d upsampling", cin, c, s);
                }
                Pending p{&L, 0, 0, {}, {}, true, false};
                p.in = pack_snake(ar, w, w + cin, cin, bf);  w += 2 * cin;
                p.w = pack_conv(ar, w, L, bf);               w += (size_t)cin * c * 2 * s;
                p.bias = pack_floats(ar, w, c);              w += c;
                pend.push_back(p);
            }
            for (int j = 0; j < nres; ++j) {
                // the last unit of a block feeds the next block's transposed conv
                const int next_fmt = (j + 1 == nres && l + 1 < nb) ? wide_fmt_of(st.widths[l + 1]) : (int)OP_BF16;
                rc = pack_unit(B.res[j], c, j, next_fmt);
                if (rc != DEMON_OK) return rc;
            }
            cin = c;
            rate *= s;
            per_frame = std::max(per_frame, rate * c);
        }
        // Rows each layer must produce beyond a window's interior (the receptive-field cone, walked from the
        // head back to the first block): a k-tap conv of dilation d reads d(k-1)/2 rows further out than it
        // writes; a transposed conv writing margin m reads inputs up to (m + p)/s + 1 rows out.
        {
            int m = (st.head_kernel - 1) / 2;
            for (int l = nb - 1; l >= 0; --l) {
                Block& B = v->blocks[l];
                for (int j = nres - 1; j >= 0; --j) {
                    B.res[j].pointwise.margin = m;
                    B.res[j].dilated.margin = m;
                    m += st.dilations[j] * ((st.res_kernel - 1) / 2);
                }
                B.up.margin = m;
                m = (m + st.strides[l] / 2) / st.strides[l] + 1;
            }
        }
        // head: weights as [tap][cin][out_channel] fp32
        hs = pack_snake(ar, w, w + cin, cin, bf);  w += 2 * cin;
        hw = ar.reserve(sizeof(float) * (size_t)hk * cin * oc);
        {
            float* dst = reinterpret_cast<float*>(ar.bytes.data() + hw);
            for (int o = 0; o < oc; ++o)
                for (int i = 0; i < cin; ++i)
                    for (int t = 0; t < hk; ++t) {
                        float val = w[((size_t)o * cin + i) * hk + t];
                        if (bf) { const uint32_t u = (uint32_t)f32_to_bf16_rne(val) << 16; memcpy(&val, &u, 4); }
                        dst[((size_t)t * cin + i) * oc + o] = val;
                    }
        }
        w += (size_t)oc * cin * hk;
        head_mfma = bf && (cin == 64 || cin == 32) && head_mfma_frag_count(cin, hk) <= 40;
        if (head_mfma) {
            // from the bf16-rounded weights, like every other weight of this path
            std::vector<float> wr((size_t)oc * cin * hk);
            for (size_t i = 0; i < wr.size(); ++i) { const uint32_t u = (uint32_t)f32_to_bf16_rne((w - (size_t)oc * cin * hk)[i]) << 16; memcpy(&wr[i], &u, 4); }
            hwf = ar.reserve(head_mfma_frag_count(cin, hk) * 64 * 16);
            pack_head_mfma(wr.data(), cin, oc, hk, reinterpret_cast<uint16_t*>(ar.bytes.data() + hwf));
        }
        hb = pack_floats(ar, w, oc);
        w += oc;
        v->head_cin = cin;
    } else {
        // ---- encoder: stem from the waveform, then per block (from the audio rate down) the units and the strided conv
        for (int s : st.strides) rate *= s;
        const int cs = st.widths[nb - 1];
        v->stem_cout = cs;
        stem_w_off = ar.reserve(sizeof(float) * (size_t)hk * oc * cs);
        {
            // [C][channels][k] -> [k][channels][C]
            float* dst = reinterpret_cast<float*>(ar.bytes.data() + stem_w_off);
            for (int o = 0; o < cs; ++o)
                for (int i = 0; i < oc; ++i)
                    for (int t = 0; t < hk; ++t) {
                        float val = w[((size_t)o * oc + i) * hk + t];
                        if (bf) { const uint32_t u = (uint32_t)f32_to_bf16_rne(val) << 16; memcpy(&val, &u, 4); }
                        dst[((size_t)t * oc + i) * cs + o] = val;
                    }
        }
        w += (size_t)cs * oc * hk;
        stem_b_off = pack_floats(ar, w, cs);  w += cs;
        per_frame = rate * cs;
        for (int b = 0; b < nb; ++b) {
            const int l = nb - 1 - b;
            const int s = st.strides[l], c = st.widths[l];
            const int cn = l > 0 ? st.widths[l - 1] : 2 * st.c0;
            Block& B = v->blocks[b];
            per_frame = std::max(per_frame, rate * c);
            ConvLayer& L = B.up;               // the strided conv after the units
            L.cin = c; L.cout = cn; L.ntaps = 2 * s; L.stride = 0; L.down = s;
            L.in_fmt = (bf && c >= kSplitWidth) ? (int)OP_F16 : (int)OP_BF16;
            for (int j = 0; j < nres; ++j) {
                // the last unit of a block feeds the block's strided conv
                rc = pack_unit(B.res[j], c, j, j + 1 == nres ? L.in_fmt : (int)OP_BF16);
                if (rc != DEMON_OK) return rc;
            }
            if (bf) {
                L.variant = choose_variant_bf16(c * (s / 2), cn);
                if (L.variant == 1) L.variant = cn % 32 == 0 ? 2 : -1;      // the 256-column tile has no strided form
                if (L.variant < 0) return fail(DEMON_ERR_UNSUPPORTED, "bf16 path: no kernel for a %d -> %d stride-%d downsampling", c, cn, s);
            }
            Pending p{&L, 0, 0, {}, {}, true, false};
            p.in = pack_snake(ar, w, w + c, c, bf);  w += 2 * c;
            p.w = pack_conv(ar, w, L, bf);           w += (size_t)cn * c * 2 * s;
            p.bias = pack_floats(ar, w, cn);         w += cn;
            pend.push_back(p);
            rate /= s;
            per_frame = std::max(per_frame, rate * cn);
        }
        // Rows each layer must produce beyond a window's interior, walked from the moments back to the stem: a strided
        // conv writing margin m reads inputs up to m s + s/2 rows out, a k-tap conv of dilation d d(k-1)/2 rows further.
        {
            int m = 0;
            for (int b = nb - 1; b >= 0; --b) {
                Block& B = v->blocks[b];
                const int s = st.strides[nb - 1 - b];
                B.up.margin = m;
                m = m * s + s / 2;
                for (int j = nres - 1; j >= 0; --j) {
                    B.res[j].pointwise.margin = m;
                    B.res[j].dilated.margin = m;
                    m += st.dilations[j] * ((st.res_kernel - 1) / 2);
                }
            }
            v->stem_margin = m;
        }
        rate = 1;                              // no window waveforms to hold
    }

    // ---- device memory
    const size_t act_elems = (size_t)v->cap_frames * (size_t)per_frame;
    v->ws.act_elems = act_elems;
    v->per_frame = per_frame;
    const size_t head_bytes = encoder ? 256 : (size_t)v->cap_frames * (size_t)rate * oc * sizeof(float);
    auto cleanup = [&]() {
        if (v->d_params) (void)hipFree(v->d_params);
        for (void* b : v->ws.buf) if (b) (void)hipFree(b);
        if (v->ws.head_out) (void)hipFree(v->ws.head_out);
        if (v->d_slot_arena) (void)hipFree(v->d_slot_arena);
        if (v->ws.slot_gated) (void)hipFree(v->ws.slot_gated);
        if (v->ev_fork) (void)hipEventDestroy(v->ev_fork);
        if (v->ev_join) (void)hipEventDestroy(v->ev_join);
        if (v->stream2) (void)hipStreamDestroy(v->stream2);
    };
    hipError_t e = hipMalloc(&v->d_params, ar.bytes.size());
    // fp32 path: 4 bytes per element; bf16 path: half residual stream (2 bytes), bf16 operand buffers with hi and lo planes (4)
    for (int i = 0; e == hipSuccess && i < (bf ? 5 : 3); ++i) e = hipMalloc(&v->ws.buf[i], act_elems * ((bf && i < 2) ? 2 : 4));
    if (e == hipSuccess) e = hipMalloc((void**)&v->ws.head_out, head_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&v->d_slot_arena, sizeof(Slot) * kMaxSlots * kPlanCache);
    if (e == hipSuccess) e = hipMalloc((void**)&v->ws.slot_gated, sizeof(Slot) * kMaxSlots);
    if (e == hipSuccess && bf && g_dual_stream) {
        e = hipStreamCreateWithFlags(&v->stream2, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&v->ev_fork, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&v->ev_join, hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipMemcpy(v->d_params, ar.bytes.data(), ar.bytes.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { cleanup(); return hip_fail(e, "allocating device memory"); }

    const unsigned char* base = static_cast<const unsigned char*>(v->d_params);
    auto fptr = [&](size_t off) { return reinterpret_cast<const float*>(base + off); };
    for (const Pending& p : pend) {
        p.L->w = base + p.w;
        p.L->bias = fptr(p.bias);
        if (p.has_in) { p.L->in_alpha = fptr(p.in.alpha); p.L->in_inv_beta = fptr(p.in.inv_beta); }
        if (p.has_out) { p.L->out_alpha = fptr(p.outp.alpha); p.L->out_inv_beta = fptr(p.outp.inv_beta); }
    }
    for (const FusedFix& f : fused_fix) f.U->w1_fused = reinterpret_cast<const uint16_t*>(base + f.off);
    if (encoder) {
        v->stem_w = fptr(stem_w_off); v->stem_bias = fptr(stem_b_off);
    } else {
        v->head_alpha = fptr(hs.alpha); v->head_inv_beta = fptr(hs.inv_beta);
        v->head_w = fptr(hw); v->head_bias = fptr(hb);
        if (head_mfma) v->head_wfrag = reinterpret_cast<const uint16_t*>(base + hwf);
    }

    // ---- the layer sequence in processing order, each step with the layer that takes its output as an MFMA operand
    // (bf16 path): the next step's resampling conv or the dilated conv of its unit, unless that unit reads the residual
    // stream itself (narrow fused unit) or nothing follows (head, sampling step)
    for (int b = 0; b < nb; ++b) {
        Block& B = v->blocks[b];
        if (!encoder) { Step t; t.conv = &B.up; v->steps.push_back(t); }
        for (int j = 0; j < nres; ++j) { Step t; t.unit = &B.res[j]; v->steps.push_back(t); }
        if (encoder) { Step t; t.conv = &B.up; v->steps.push_back(t); }
    }
    auto operand_layer = [](const Step& t) -> const ConvLayer* {
        if (t.conv) return t.conv;
        return t.unit->fused ? nullptr : &t.unit->dilated;
    };
    for (size_t i = 0; i + 1 < v->steps.size(); ++i) v->steps[i].consumer = operand_layer(v->steps[i + 1]);
    v->first_consumer = operand_layer(v->steps[0]);
    // the head can run inside the last residual unit's kernel when that unit is the fused 64-channel form
    if (!encoder && head_mfma && !(cfg->flags & DEMON_VAE_FLAG_NO_HEAD_FUSION) && !v->steps.empty()) {
        const Step& last = v->steps.back();
        v->head_fusable = last.unit && last.unit->fused && last.unit->dilated.cin == 64 && oc <= 8 && hk <= 7 &&
                          last.unit->pointwise.margin == (hk - 1) / 2;
    }

    *out = v.release();
    return DEMON_OK;
}

}  // namespace

extern "C" {

demon_status demon_vae_create(const demon_vae_config* cfg, const float* host_weights, size_t n_floats, demon_vae** out)
{
    return create_impl(cfg, host_weights, n_floats, false, out);
}

demon_status demon_vae_create_encoder(const demon_vae_config* cfg, const float* host_weights, size_t n_floats, demon_vae** out)
{
    return create_impl(cfg, host_weights, n_floats, true, out);
}

void demon_vae_destroy(demon_vae* v)
{
    if (!v) return;
    (void)hipFree(v->d_params);
    for (void* b : v->ws.buf) if (b) (void)hipFree(b);
    (void)hipFree(v->ws.head_out);
    (void)hipFree(v->d_slot_arena);
    (void)hipFree(v->ws.slot_gated);
    for (hipEvent_t e : v->events) (void)hipEventDestroy(e);
    if (v->ev_fork) (void)hipEventDestroy(v->ev_fork);
    if (v->ev_join) (void)hipEventDestroy(v->ev_join);
    if (v->stream2) (void)hipStreamDestroy(v->stream2);
    delete v;
}

demon_status demon_vae_receptive_field(const demon_vae* v, int* halo_left, int* halo_right)
{
    if (!v || !halo_left || !halo_right) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    *halo_left = v->rf_left; *halo_right = v->rf_right;
    return DEMON_OK;
}

static demon_status decode_checked(demon_vae* v, const void* d_latent, int n_clips, int n_frames,
                                   int frame_begin, int frame_end, int window, int halo, const int* d_skip,
                                   float* d_out, int16_t* d_pcm, void* stream)
{
    clear_error();
    if (!v || !d_latent || (!d_out && !d_pcm)) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    if (v->encoder) return fail(DEMON_ERR_INVALID_ARG, "this handle is an encoder (demon_vae_create_encoder): use demon_vae_encode_windowed");
    if (n_clips < 1) return fail(DEMON_ERR_INVALID_ARG, "n_clips must be >= 1");
    if (n_frames < 1) return fail(DEMON_ERR_INVALID_ARG, "n_frames must be >= 1");
    if (frame_begin < 0) return fail(DEMON_ERR_INVALID_ARG, "frame_begin must be >= 0");
    if (frame_end > n_frames) return fail(DEMON_ERR_INVALID_ARG, "frame_end %d exceeds n_frames %d", frame_end, n_frames);
    if (frame_begin >= frame_end) return fail(DEMON_ERR_INVALID_ARG, "empty frame range [%d, %d)", frame_begin, frame_end);
    if (window < 1) return fail(DEMON_ERR_INVALID_ARG, "window must be >= 1");
    if (halo < -1) return fail(DEMON_ERR_INVALID_ARG, "halo must be >= -1");
    if (n_frames > v->max_frames) return fail(DEMON_ERR_WORKSPACE, "n_frames %d exceeds max_frames %d", n_frames, v->max_frames);
    if (n_clips > v->max_clips) return fail(DEMON_ERR_WORKSPACE, "n_clips %d exceeds max_clips %d", n_clips, v->max_clips);
    if (halo == -1) halo = std::max(v->rf_left, v->rf_right);
    Plan* plan = nullptr;
    const demon_status rc = get_plan(v, n_clips, n_frames, frame_begin, frame_end, window, halo, wants_two_groups(v), (hipStream_t)stream, &plan);
    if (rc != DEMON_OK) return rc;
    Io io;
    io.d_latent = d_latent; io.d_skip = d_skip; io.d_out = d_out; io.d_pcm = d_pcm; io.n_frames = n_frames;
    return run_pass(v, v->ws, plan, io, (hipStream_t)stream);
}

demon_status demon_vae_decode_windowed(demon_vae* v, const void* d_latent, int n_clips, int n_frames,
                                       int frame_begin, int frame_end, int window, int halo,
                                       float* d_out, void* stream)
{
    if (!d_out) { clear_error(); return fail(DEMON_ERR_INVALID_ARG, "NULL argument"); }
    return decode_checked(v, d_latent, n_clips, n_frames, frame_begin, frame_end, window, halo, nullptr, d_out, nullptr, stream);
}

demon_status demon_vae_decode_windowed_gated(demon_vae* v, const void* d_latent, int n_clips, int n_frames,
                                             int frame_begin, int frame_end, int window, int halo,
                                             const int* d_skip, float* d_out, void* stream)
{
    if (!d_out || !d_skip) { clear_error(); return fail(DEMON_ERR_INVALID_ARG, "NULL argument"); }
    return decode_checked(v, d_latent, n_clips, n_frames, frame_begin, frame_end, window, halo, d_skip, d_out, nullptr, stream);
}

demon_status demon_vae_decode_windowed_pcm16(demon_vae* v, const void* d_latent, int n_clips, int n_frames,
                                             int frame_begin, int frame_end, int window, int halo,
                                             int16_t* d_pcm, void* stream)
{
    if (!d_pcm) { clear_error(); return fail(DEMON_ERR_INVALID_ARG, "NULL argument"); }
    return decode_checked(v, d_latent, n_clips, n_frames, frame_begin, frame_end, window, halo, nullptr, nullptr, d_pcm, stream);
}

demon_status demon_vae_decode_windowed_static(demon_vae* v, const void* d_latent, int n_clips, int n_frames,
                                              int frame_begin, int frame_end, int window, int halo,
                                              float* d_out, void* stream_)
{
    clear_error();
    hipStream_t stream = (hipStream_t)stream_;
    if (!v || !d_latent || !d_out) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    if (v->encoder) return fail(DEMON_ERR_INVALID_ARG, "this handle is an encoder (demon_vae_create_encoder): use demon_vae_encode_windowed");
    if (n_clips < 1) return fail(DEMON_ERR_INVALID_ARG, "n_clips must be >= 1");
    if (n_frames < 1) return fail(DEMON_ERR_INVALID_ARG, "n_frames must be >= 1");
    if (frame_begin < 0) return fail(DEMON_ERR_INVALID_ARG, "frame_begin must be >= 0");
    if (frame_end > n_frames) return fail(DEMON_ERR_INVALID_ARG, "frame_end %d exceeds n_frames %d", frame_end, n_frames);
    if (frame_begin >= frame_end) return fail(DEMON_ERR_INVALID_ARG, "empty frame range [%d, %d)", frame_begin, frame_end);
    if (window < 1) return fail(DEMON_ERR_INVALID_ARG, "window must be >= 1");
    if (halo < -1) return fail(DEMON_ERR_INVALID_ARG, "halo must be >= -1");
    if (halo == -1) halo = std::max(v->rf_left, v->rf_right);
    if (!v->scratch) return fail(DEMON_ERR_HIP, "the static scratch array was not found on this device");

    // the window grid, counted on the host without building it (the table itself is written by a kernel)
    const GridCount gc = count_grid(n_frames, frame_begin, frame_end, window, halo);
    const long long per_clip = gc.per_clip, clip_frames = gc.clip_frames;
    const int max_len = gc.max_len, max_int = gc.max_int;
    if (per_clip * n_clips > kMaxSlots)
        return fail(DEMON_ERR_WORKSPACE, "%lld windows exceed the limit of %d", per_clip * n_clips, kMaxSlots);
    const long long total = clip_frames * n_clips;
    const demon_status prc = check_plane(v, max_len);
    if (prc != DEMON_OK) return prc;

    // carve the call's memory out of the static array: window table, activation buffers, window waveforms
    const bool bf = v->dtype == DEMON_BF16;
    const size_t act_elems = (size_t)total * (size_t)v->per_frame;
    const size_t planes = (bf && v->has_split_operands) ? 2 : 1;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off = (at + bytes + 255) & ~(size_t)255; return at; };
    const size_t at_slots = take(sizeof(Slot) * (size_t)(per_clip * n_clips));
    size_t at_buf[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < (bf ? 5 : 3); ++i) at_buf[i] = take(act_elems * (bf ? (i < 2 ? 2 : 2 * planes) : 4));
    const size_t at_head = take((size_t)total * (size_t)v->st.total_stride() * v->st.out_channels * sizeof(float));
    if (off > kStaticScratchBytes)
        return fail(DEMON_ERR_WORKSPACE, "the call needs %zu bytes of scratch for %lld extended frames, the static array holds %zu",
                    off, total, kStaticScratchBytes);
    Workspace ws;
    for (int i = 0; i < (bf ? 5 : 3); ++i) ws.buf[i] = v->scratch + at_buf[i];
    ws.head_out = reinterpret_cast<float*>(v->scratch + at_head);
    ws.act_elems = act_elems;

    Plan plan;
    plan.valid = true;
    plan.n_clips = n_clips; plan.n_frames = n_frames; plan.frame_begin = frame_begin; plan.frame_end = frame_end;
    plan.window = window; plan.halo = halo;
    plan.n_slots = (int)(per_clip * n_clips); plan.max_len = max_len; plan.max_int = max_int;
    plan.total_frames = total;
    plan.n_groups = 1;
    plan.g_first[0] = 0; plan.g_count[0] = plan.n_slots; plan.g_frame0[0] = 0; plan.g_frames[0] = total;
    plan.d_slots = reinterpret_cast<Slot*>(v->scratch + at_slots);
    HIP_TRY(launch_plan_slots(plan.d_slots, n_clips, (int)per_clip, (int)clip_frames, n_frames, frame_begin, frame_end, window, halo,
                              plan.n_slots, 0, stream),
            "window table");
    Io io;
    io.d_latent = d_latent; io.d_out = d_out; io.n_frames = n_frames;
    return run_pass(v, ws, &plan, io, stream);
}

demon_status demon_vae_encode_windowed(demon_vae* v, const float* d_wave, int n_clips, int n_frames,
                                       int frame_begin, int frame_end, int window, int halo,
                                       const float* d_eps, float* d_moments, void* d_latent, void* stream)
{
    clear_error();
    if (!v || !d_wave || (!d_moments && !d_latent)) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    if (!v->encoder) return fail(DEMON_ERR_INVALID_ARG, "this handle is a decoder (demon_vae_create): use demon_vae_decode_windowed");
    if (n_clips < 1) return fail(DEMON_ERR_INVALID_ARG, "n_clips must be >= 1");
    if (n_frames < 1) return fail(DEMON_ERR_INVALID_ARG, "n_frames must be >= 1");
    if (frame_begin < 0) return fail(DEMON_ERR_INVALID_ARG, "frame_begin must be >= 0");
    if (frame_end > n_frames) return fail(DEMON_ERR_INVALID_ARG, "frame_end %d exceeds n_frames %d", frame_end, n_frames);
    if (frame_begin >= frame_end) return fail(DEMON_ERR_INVALID_ARG, "empty frame range [%d, %d)", frame_begin, frame_end);
    if (window < 1) return fail(DEMON_ERR_INVALID_ARG, "window must be >= 1");
    if (halo < -1) return fail(DEMON_ERR_INVALID_ARG, "halo must be >= -1");
    if (n_frames > v->max_frames) return fail(DEMON_ERR_WORKSPACE, "n_frames %d exceeds max_frames %d", n_frames, v->max_frames);
    if (n_clips > v->max_clips) return fail(DEMON_ERR_WORKSPACE, "n_clips %d exceeds max_clips %d", n_clips, v->max_clips);
    if ((long long)n_frames * v->st.total_stride() > 0x7fffffffll) return fail(DEMON_ERR_UNSUPPORTED, "clips longer than 2^31 samples");
    if (halo == -1) halo = std::max(v->rf_left, v->rf_right);
    Plan* plan = nullptr;
    const demon_status rc = get_plan(v, n_clips, n_frames, frame_begin, frame_end, window, halo, wants_two_groups(v), (hipStream_t)stream, &plan);
    if (rc != DEMON_OK) return rc;
    Io io;
    io.d_wave = d_wave; io.d_eps = d_eps; io.d_moments = d_moments; io.d_zout = d_latent; io.n_frames = n_frames;
    return run_pass(v, v->ws, plan, io, (hipStream_t)stream);
}

demon_status demon_vae_encode(demon_vae* v, const float* d_wave, int n_clips, int n_frames, const float* d_eps,
                              float* d_moments, void* d_latent, void* stream)
{
    // one window per clip covering [0, n_frames), no halo: the same kernels as the windowed encode
    return demon_vae_encode_windowed(v, d_wave, n_clips, n_frames, 0, n_frames, n_frames > 0 ? n_frames : 1, 0, d_eps, d_moments, d_latent, stream);
}

demon_status demon_vae_decode(demon_vae* v, const void* d_latent, int n_clips, int n_frames, float* d_out, void* stream)
{
    // one window per clip covering [0, n_frames), no halo: the same kernels as the windowed decode
    return demon_vae_decode_windowed(v, d_latent, n_clips, n_frames, 0, n_frames, n_frames > 0 ? n_frames : 1, 0, d_out, stream);
}

demon_status demon_vae_latent_similarity(const void* d_curr, const void* d_prev, int n_clips, long long elems_per_clip,
                                         demon_dtype dtype, float threshold, float* d_mse, int* d_unchanged, void* stream)
{
    clear_error();
    if (!d_curr || !d_prev || (!d_mse && !d_unchanged)) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    if (n_clips < 1 || n_clips > 65535) return fail(DEMON_ERR_INVALID_ARG, "n_clips must be in [1, 65535]");
    if (elems_per_clip < 1) return fail(DEMON_ERR_INVALID_ARG, "elems_per_clip must be >= 1");
    if (dtype != DEMON_F32 && dtype != DEMON_BF16) return fail(DEMON_ERR_INVALID_ARG, "unknown dtype");
    if (!(threshold >= 0.0f)) return fail(DEMON_ERR_INVALID_ARG, "threshold must be >= 0");
    HIP_TRY(launch_latent_mse(d_curr, d_prev, n_clips, elems_per_clip, dtype == DEMON_BF16, threshold, d_mse, d_unchanged,
                              (hipStream_t)stream), "latent similarity");
    return DEMON_OK;
}

demon_status demon_vae_crossfade(const float* d_prev_tail, long long prev_stride, const float* d_next_head, long long next_stride,
                                 float* d_out, long long out_stride, int n_planes, int n_samples, void* stream)
{
    clear_error();
    if (!d_prev_tail || !d_next_head || !d_out) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    if (n_planes < 1 || n_planes > 65535) return fail(DEMON_ERR_INVALID_ARG, "n_planes must be in [1, 65535]");
    if (n_samples < 1) return fail(DEMON_ERR_INVALID_ARG, "n_samples must be >= 1");
    if (prev_stride < 0 || next_stride < 0 || out_stride < 0) return fail(DEMON_ERR_INVALID_ARG, "negative plane stride");
    if (n_planes > 1 && out_stride < n_samples) return fail(DEMON_ERR_INVALID_ARG, "output planes overlap");
    HIP_TRY(launch_crossfade(d_prev_tail, prev_stride, d_next_head, next_stride, d_out, out_stride, n_planes, n_samples,
                             (hipStream_t)stream), "crossfade");
    return DEMON_OK;
}

demon_status demon_vae_set_timing(demon_vae* v, int level)
{
    if (!v) return fail(DEMON_ERR_INVALID_ARG, "NULL handle");
    if (level < 0 || level > 2) return fail(DEMON_ERR_INVALID_ARG, "timing level must be 0, 1 or 2");
    size_t launches = 3;                                    // gather, head, stitch
    for (const Block& B : v->blocks) launches += 1 + 2 * B.res.size();
    v->marks_per_call = (int)launches + 1;
    while (level > 0 && v->events.size() < (size_t)v->marks_per_call * kTimingRing) {
        hipEvent_t e;
        hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess) return hip_fail(rc, "hipEventCreate");
        v->events.push_back(e);
    }
    v->timing = level;
    v->n_marks = 0;
    v->timed_calls = 0;
    return DEMON_OK;
}

demon_status demon_vae_get_timing(demon_vae* v, float* ms, int capacity, int* n)
{
    if (!v || !n) return fail(DEMON_ERR_INVALID_ARG, "NULL argument");
    const int avail = v->n_marks > 0 ? v->n_marks - 1 : 0;
    *n = avail;
    const int calls = v->timed_calls < kTimingRing ? v->timed_calls : kTimingRing;
    if (!ms || calls == 0) return DEMON_OK;
    for (int i = 0; i < avail && i < capacity; ++i) {
        double sum = 0;
        for (int c = 0; c < calls; ++c) {
            float t = 0;
            const int base = c * v->marks_per_call;
            hipError_t rc = hipEventElapsedTime(&t, v->events[base + i], v->events[base + i + 1]);
            if (rc != hipSuccess) return hip_fail(rc, "hipEventElapsedTime");
            sum += t;
        }
        ms[i] = (float)(sum / calls);
    }
    v->timed_calls = 0;
    return DEMON_OK;
}

void demon_vae_test_pack_bf16(const float* w, int cin, int cout, int ntaps, int stride, int variant, int as_half,
                              int permute_rows, uint16_t* dst)
{
    pack_bf16(w, cin, cout, ntaps, stride, variant, as_half != 0, permute_rows != 0, dst);
}

void demon_vae_test_pack_w1_fused(const float* w, int c, uint16_t* dst) { pack_w1_fused(w, c, dst); }

uint16_t demon_vae_test_f32_to_f16(float v) { return f32_to_f16_rne(v); }

demon_status demon_vae_debug_tap(demon_vae* v, int layer, float* d_dst, size_t capacity)
{
    if (!v) return fail(DEMON_ERR_INVALID_ARG, "NULL handle");
    if (layer >= 0 && !d_dst) return fail(DEMON_ERR_INVALID_ARG, "d_dst is NULL");
    v->tap_layer = layer; v->tap_dst = d_dst; v->tap_cap = capacity;
    return DEMON_OK;
}

}  // extern "C"
