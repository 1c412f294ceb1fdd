// Fused residual unit for 256 channels:
//     h += W1 * snake2(W7 (*) a + b7) + b1,      a = bf16(snake1(h)) written by the producer of h
// in one kernel: the activated branch tensor between the two convolutions never goes to HBM, and the 1x1
// convolution (a short reduction with a long epilogue, bound by HBM when it runs on its own) costs one more
// K loop instead of a launch.
//
// Workgroup = 4 waves, tile = all 256 channels x 128 time columns, every wave all 256 rows of its 32 columns
// (8 accumulator tiles of 32 x 32).  The dilated convolution runs as in kernels_bf16.hip on the pre-activated
// bf16 operand, with K stages of 32 channels so that two workgroups fit the LDS of a CU.  As in the narrow fused
// unit, a lane of an accumulator tile holds column j and rows 8g + 4h + {0..3}, which after bias + Snake are the
// B fragments of the 1x1 convolution once its K axis is permuted to that order (fused_k_to_channel); its weights,
// 128 KB, do not fit the LDS and are streamed through the weight buffers in 8 blocks of 32 k-slots.
// In the 1x1 convolution the roles are swapped: the fragments are the row operand (rows = time), the weights the
// column operand, so its accumulator tile is [time][output channel slot]; the weight rows are packed so that slot j
// of tile mo is channel 8 j + mo.  A lane then owns 8 consecutive channels (16 bytes of half) of a time row and 32
// lanes the whole row: residual loads and stores are contiguous straight from the accumulators.
// The residual stream is updated in place (only this tile reads or writes its elements); the emitted operand of
// the next layer goes to a second buffer because neighbouring tiles still read this tile's input rows.
#include <algorithm>

#include "device_common.h"

namespace demon {

namespace {

constexpr int W_CH = 256, W_KC = 32, W_LDK = W_KC + 8, W_NT = 128, W_TM = W_CH / 32, W_MAXSPAN = 64;
constexpr int W_XR_MAX = W_NT + W_MAXSPAN;
constexpr int W_SEGS = W_KC / 8, W_RPP = 256 / W_SEGS;
constexpr int W_A_CH = W_CH * W_SEGS, W_A_ITERS = W_A_CH / 256;
constexpr int W_X_ITERS = (W_XR_MAX + W_RPP - 1) / W_RPP;
constexpr int W_NCHUNKS = W_CH / W_KC;

struct WideParams {
    const uint16_t* xa;          // activated input, bf16 [rows][256]
    hres_t* y;                   // residual stream, in place
    uint16_t* ya;                // optional bf16(snake_next(y)) (EMIT); not the buffer of xa
    const uint16_t* w7;          // [chunk][tap] blocks of 256 x 32 bf16
    const uint16_t* w1;          // [chunk] blocks of 256 x 32 bf16, K axis permuted
    const float* b7; const float* b1;
    const float* a2; const float* ib2;    // Snake between the two convolutions (alpha in revolutions, 1/(beta+eps))
    const float* a3; const float* ib3;    // Snake of the consumer (EMIT)
    const Slot* slots;
    int r, ntaps, tap0, tap_step, margin;
};

template <bool EMIT>
__global__ __launch_bounds__(256) void res_unit_wide_kernel(WideParams p)
{
    fp16_saturate_on();
    constexpr int CH = W_CH, KC = W_KC, LDK = W_LDK, NT = W_NT, TM = W_TM;
    constexpr int A_ITERS = W_A_ITERS, X_ITERS = W_X_ITERS, SEGS = W_SEGS, RPP = W_RPP;
    constexpr int AS_BYTES = 2 * CH * LDK * 2, XS_BYTES = W_XR_MAX * LDK * 2;
    constexpr int SMEM_BYTES = AS_BYTES + XS_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
    __shared__ __attribute__((aligned(16))) float prm[4 * CH];     // b7 | a2 | ib2 | b1
    uint16_t* As = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Xs = reinterpret_cast<uint16_t*>(smem + AS_BYTES);

    const Slot s = p.slots[blockIdx.y];
    const int nrows = s.len * p.r;
    const int out_lo = max(0, s.crop * p.r - p.margin);
    const int out_hi = min(nrows, (s.crop + s.n_int) * p.r + p.margin);
    // Workgroups are dealt to the 8 XCDs round-robin by linear id, and each XCD has its own L2: XCD x takes a contiguous
    // eighth of a window's tiles, in order, so that neighbouring tiles (which share their halo rows) run on the same
    // XCD at about the same time.  The eighths rotate with the window index (the last one may be short).
    const int tiles8 = (int)(gridDim.x >> 3);
    const int tile = (int)((blockIdx.x + blockIdx.y) & 7u) * tiles8 + (int)(blockIdx.x >> 3);
    const int n0 = out_lo + tile * NT;
    if (n0 >= out_hi) return;
    const long long rowbase = (long long)s.row0 * p.r;

    const int last_off = p.tap0 + (p.ntaps - 1) * p.tap_step;
    const int minoff = min(p.tap0, last_off);
    const int XR = NT + max(p.tap0, last_off) - minoff;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wn = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS;

    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.xa + rowbase * CH, (unsigned)nrows * CH * 2u);
    const __amdgpu_buffer_rsrc_t rs_y = make_rsrc(p.y + rowbase * CH, (unsigned)out_hi * CH * (unsigned)sizeof(hres_t));
    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(p.ya + rowbase * CH, EMIT ? (unsigned)out_hi * CH * 2u : 0u);
    const int nstages = W_NCHUNKS * p.ntaps;
    const __amdgpu_buffer_rsrc_t rs_w7 = make_rsrc(p.w7, (unsigned)nstages * (W_A_CH * 16u));
    const __amdgpu_buffer_rsrc_t rs_w1 = make_rsrc(p.w1, (unsigned)W_NCHUNKS * (W_A_CH * 16u));

    // Staging pattern.  An LDS row is 80 bytes (20 banks), so the 8 lanes that one cycle of a 16-byte LDS write serves
    // must not hold two neighbouring rows (rows r and r + 1 overlap in 4 banks): lanes 0..3 of each group of 8 take the
    // four pieces of row r, lanes 4..7 those of row r + 4, which starts 16 banks further.  A pass of 256 threads covers
    // 64 rows; srow is the thread's row within a pass.
    const int srow = 8 * (tid >> 5) + ((tid >> 3) & 3) + 4 * ((tid >> 2) & 1);
    const unsigned a_voff = (unsigned)(srow * SEGS + seg) * 16u;
    const unsigned x_voff = ((unsigned)((n0 + minoff + srow) * CH) + seg * 8u) * 2u;     // may wrap "negative": out of range
    constexpr unsigned x_row_step = RPP * CH * 2u;

    u32x4 ra[A_ITERS], rb[A_ITERS];     // rb: second set, only for the blocks of the 1x1 weights (requested two ahead)
    u32x4 rx[X_ITERS];
    auto load_set = [&](u32x4 (&r)[A_ITERS], __amdgpu_buffer_rsrc_t rs, int block) __attribute__((always_inline)) {
        const unsigned base = (unsigned)block * (W_A_CH * 16u);
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) r[it] = __builtin_amdgcn_raw_buffer_load_b128(rs, a_voff, base + it * 4096u, 0);
    };
    auto store_set = [&](const u32x4 (&r)[A_ITERS], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
            *reinterpret_cast<u32x4*>(&As[buf * CH * LDK + (srow + it * RPP) * LDK + seg * 8]) = r[it];
    };
    auto load_a = [&](__amdgpu_buffer_rsrc_t rs, int block) __attribute__((always_inline)) { load_set(ra, rs, block); };
    auto store_a = [&](int buf) __attribute__((always_inline)) { store_set(ra, buf); };
    auto load_x = [&](int chunk) __attribute__((always_inline)) {
        const unsigned coff = x_voff + (unsigned)(chunk * KC) * 2u;
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                        // uniform
            rx[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, coff + it * x_row_step, 0, 0);
        }
    };
    auto store_x = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                        // uniform
            const int xr = srow + it * RPP;
            if (xr >= W_XR_MAX) continue;
            *reinterpret_cast<u32x4*>(&Xs[xr * LDK + seg * 8]) = rx[it];
        }
    };

    // every request of the prologue is issued before the first result is waited for, in the order of use
    load_a(rs_w7, 0);
    load_x(0);
    constexpr int PRM_ITERS = 4 * CH / 256;
    float pv[PRM_ITERS];
#pragma unroll
    for (int it = 0; it < PRM_ITERS; ++it) {
        const float* src = it == 0 ? p.b7 : it == 1 ? p.a2 : it == 2 ? p.ib2 : p.b1;      // 256 threads, 256 channels
        pv[it] = src[tid];
    }
    store_a(0);
    store_x();
#pragma unroll
    for (int it = 0; it < PRM_ITERS; ++it) prm[it * CH + tid] = pv[it];
    __syncthreads();

    // accumulators start at the bias: lane (j, h) holds rows (channels) mi*32 + 8g + 4h + {0..3} of column j
    f32x16 acc[TM];
    auto init_acc = [&](int which) __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b4 = *reinterpret_cast<const float4*>(&prm[which * CH + mi * 32 + 8 * g + 4 * h]);
                acc[mi][4 * g + 0] = b4.x; acc[mi][4 * g + 1] = b4.y; acc[mi][4 * g + 2] = b4.z; acc[mi][4 * g + 3] = b4.w;
            }
    };
    init_acc(0);

    // ---- dilated conv: K loop over (chunk, tap) stages, fixed order; the last stage is peeled, its shadow hides the
    // fetch of the first block of the 1x1 weights
    int chunk = 0, tap = 0;
    auto mma_stage = [&](int stage) __attribute__((always_inline)) {
        __builtin_amdgcn_s_setprio(1);
        const int off = p.tap0 + tap * p.tap_step - minoff;
        const uint16_t* abase = &As[(stage & 1) * CH * LDK + j * LDK + h * 8];
        const uint16_t* xbase = &Xs[(wn * 32 + j + off) * LDK + h * 8];
        // The stage's 16 MFMAs in the order (k-step, row tile), each weight fragment requested three MFMAs before it is used
        // (four fragment registers in rotation).  Left to itself the compiler reads the first k-step's fragments one at a time
        // into one register set, and each of those MFMAs waits out the full LDS latency of its read.
        static_assert(KC == 32 && TM == 8, "two k-steps of eight row tiles");
        auto afrag = [&](int i) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8*>(abase + (i & 7) * 32 * LDK + (i >> 3) * 16);
        };
        const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(xbase);
        const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(xbase + 16);
        bf16x8 a[4];
        a[0] = afrag(0); a[1] = afrag(1); a[2] = afrag(2);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i + 3 < 16) a[(i + 3) & 3] = afrag(i + 3);
            acc[i & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], (i >> 3) ? b1 : b0, acc[i & 7], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);            // b0, b1, three fragments, the fourth
#pragma unroll
        for (int i = 0; i < 12; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        __builtin_amdgcn_s_setprio(0);
    };
    // Weight blocks are requested two stages ahead, alternating between the two register sets (the second set is otherwise
    // only used by the 1x1 convolution): with one workgroup per CU (a single playback window) nothing else hides the
    // latency of a block's load, and one stage of MFMAs is shorter than it.  The request is unconditional (past the last
    // block it is out of the descriptor's range and reads nothing): behind a branch the compiler could not count it, and the
    // wait for the older block would wait for it as well.
    auto iter = [&](int stage, u32x4 (&rload)[A_ITERS], const u32x4 (&rstore)[A_ITERS]) __attribute__((always_inline)) {
        int ntap = tap + 1, nchunk = chunk;
        if (ntap == p.ntaps) { ntap = 0; ++nchunk; }
        const bool new_chunk = nchunk != chunk;
        load_set(rload, rs_w7, stage + 2);
        if (new_chunk) load_x(nchunk);
        mma_stage(stage);
        if (new_chunk) {
            __syncthreads();
            store_x();
        }
        store_set(rstore, (stage + 1) & 1);
        __syncthreads();
        tap = ntap; chunk = nchunk;
    };
    load_set(rb, rs_w7, 1);
    for (int stage = 0; stage + 1 < nstages; stage += 2) {
        iter(stage, ra, rb);
        if (stage + 2 < nstages) iter(stage + 1, rb, ra);
    }
    load_a(rs_w1, 0);
    mma_stage(nstages - 1);

    // ---- Snake on the accumulators; repack them as the B fragments of the 1x1 conv (k step kk = 2 mi + g/2)
    u32x4 mid[CH / 16];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = mi * 32 + 8 * g + 4 * h;
            const float4 a4 = *reinterpret_cast<const float4*>(&prm[CH + c]);
            const float4 i4 = *reinterpret_cast<const float4*>(&prm[2 * CH + c]);
            u32x4& f = mid[2 * mi + g / 2];
            f[2 * (g & 1) + 0] = pack_bf16x2(snake_fast(acc[mi][4 * g + 0], a4.x, i4.x), snake_fast(acc[mi][4 * g + 1], a4.y, i4.y));
            f[2 * (g & 1) + 1] = pack_bf16x2(snake_fast(acc[mi][4 * g + 2], a4.z, i4.z), snake_fast(acc[mi][4 * g + 3], a4.w, i4.w));
        }

    // ---- 1x1 conv: K = 256 channels straight from registers, weights streamed through the two weight buffers; block
    // c + 2 is requested before block c is used (odd blocks travel in ra, even ones in rb).  The residual values of
    // the epilogue are requested in the second half of the loop, where the fragments already used have freed registers.
    __syncthreads();                                   // all waves are done with the last stage's operands
    store_a(0);
    load_set(ra, rs_w1, 1);
    load_set(rb, rs_w1, 2);
    // accumulator tile mo of the 1x1 conv: [time row 8g + 4h + q][channel slot j] = channel 8 j + mo; starts at its bias
#pragma unroll
    for (int mo = 0; mo < TM; ++mo) {
        const float b1v = prm[3 * CH + j * TM + mo];
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[mo][q] = b1v;
    }
    __syncthreads();
    u32x4 resv[16];                                    // 8 halves: the lane's channels of time row gq
    auto row_offset = [&](int gq) -> unsigned {
        return (unsigned)((n0 + wn * 32 + 8 * (gq >> 2) + 4 * h + (gq & 3)) * CH + j * TM) * 2u;
    };
#pragma unroll
    for (int c = 0; c < W_NCHUNKS; ++c) {
        const uint16_t* abase = &As[(c & 1) * CH * LDK + j * LDK + h * 8];
#pragma unroll
        for (int mo = 0; mo < TM; ++mo) {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(abase + mo * 32 * LDK);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(abase + mo * 32 * LDK + 16);
            acc[mo] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mid[2 * c]), a0, acc[mo], 0, 0, 0);
            acc[mo] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mid[2 * c + 1]), a1, acc[mo], 0, 0, 0);
        }
        if (c + 1 < W_NCHUNKS) {
            if ((c + 1) & 1) store_set(ra, (c + 1) & 1); else store_set(rb, (c + 1) & 1);
            __syncthreads();
            if (c + 3 < W_NCHUNKS) { if ((c + 3) & 1) load_set(ra, rs_w1, c + 3); else load_set(rb, rs_w1, c + 3); }
        }
        if (c >= W_NCHUNKS / 2) {                      // chunks 4..7 request four time rows each
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int gq = (c - W_NCHUNKS / 2) * 4 + q;
                resv[gq] = __builtin_amdgcn_raw_buffer_load_b128(rs_y, row_offset(gq), 0, 0);
            }
        }
    }
    static_assert(W_NCHUNKS / 2 * 4 == 16, "four time rows per chunk of the second half");

    // ---- residual add, half store in place, optional Snake + bf16 operand for the next layer, straight from the
    // accumulators.  Rows past out_hi are outside the descriptors and dropped.
    float a3v[TM], i3v[TM];
#pragma unroll
    for (int mo = 0; mo < TM; ++mo) {
        a3v[mo] = EMIT ? p.a3[j * TM + mo] : 0.f;
        i3v[mo] = EMIT ? p.ib3[j * TM + mo] : 0.f;
    }
#pragma unroll
    for (int gq = 0; gq < 16; ++gq) {
        const unsigned off = row_offset(gq);
        const f16x8 r = __builtin_bit_cast(f16x8, resv[gq]);
        f16x8 o;
#pragma unroll
        for (int mo = 0; mo < TM; ++mo) o[mo] = (_Float16)(acc[mo][gq] + (float)r[mo]);     // round to nearest even
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), rs_y, off, 0, 0);
        if (EMIT) {
            // the next layer's operand is Snake of the STORED value
            u32x4 sh;
#pragma unroll
            for (int mo = 0; mo < TM; mo += 2)
                sh[mo / 2] = pack_bf16x2(snake_fast((float)o[mo], a3v[mo], i3v[mo]), snake_fast((float)o[mo + 1], a3v[mo + 1], i3v[mo + 1]));
            __builtin_amdgcn_raw_buffer_store_b128(sh, rs_a, off, 0, 0);
        }
    }
}

}  // namespace

// W1 [256][256] -> 8 blocks of 256 row slots x 32 k-slots, the K axis in the accumulator row order of the narrow fused
// unit, the rows in the order of the swapped-role accumulator tiles
void pack_w1_wide(const float* w, uint16_t* dst)
{
    for (int c = 0; c < W_NCHUNKS; ++c)
        for (int slot = 0; slot < W_CH; ++slot) {
            const int o = (slot % 32) * W_TM + slot / 32;          // row slot (mo, j) holds output channel 8 j + mo
            for (int e = 0; e < W_KC; ++e) {
                const int kp = c * W_KC + e, kk = kp / 16, h = (kp / 8) % 2, q = kp % 8;
                const int ch = 32 * (kk / 2) + 8 * (2 * (kk % 2) + q / 4) + 4 * h + q % 4;
                dst[((size_t)c * W_CH + slot) * W_KC + e] = f32_to_bf16_rne(w[(size_t)o * W_CH + ch]);
            }
        }
}

hipError_t launch_res_unit_wide(const WideArgs& a, hipStream_t stream)
{
    WideParams p;
    p.xa = a.xa; p.y = (hres_t*)a.y; p.ya = a.ya; p.w7 = a.w7; p.w1 = a.w1; p.b7 = a.b7; p.b1 = a.b1;
    p.a2 = a.a2; p.ib2 = a.ib2; p.a3 = a.a3; p.ib3 = a.ib3;
    p.slots = a.slots; p.r = a.r; p.ntaps = a.ntaps;
    p.tap0 = -((a.ntaps - 1) / 2) * a.dil; p.tap_step = a.dil; p.margin = a.margin;
    if (a.c != W_CH || a.ntaps < 1 || (a.ntaps - 1) * a.dil > W_MAXSPAN || a.margin < 0 || !a.xa || !a.y || a.xa == a.ya) return hipErrorInvalidValue;
    if (a.ya && (!a.a3 || !a.ib3)) return hipErrorInvalidValue;
    // one window's activation plane must fit a 32-bit byte offset (buffer descriptors)
    if ((long long)a.max_len * a.r * a.c * 2 > 0xf0000000ll) return hipErrorInvalidValue;
    const long long out_rows = std::min((long long)a.max_int * a.r + 2ll * a.margin, (long long)a.max_len * a.r);
    dim3 grid((unsigned)((out_rows + W_NT - 1) / W_NT + 7) / 8 * 8, (unsigned)a.n_slots);       // whole groups of 8 tiles; the surplus exits at once
    if (a.ya) hipLaunchKernelGGL((res_unit_wide_kernel<true>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((res_unit_wide_kernel<false>), grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace demon
