// Fused residual unit for the narrow, high-rate levels (C = 64 or 128 channels):
//     h_out = h + W1 * snake2(W7 (*) snake1(h) + b7) + b1
// in one kernel, so that the activated branch tensor never goes to HBM.
//
// The dilated conv runs as in kernels_bf16.hip (implicit GEMM, rows = output channels, columns = time,
// one weight block in LDS, the next waiting in registers), except that the kernel reads the half-precision residual stream itself and
// applies Snake while staging (cheaper in HBM traffic than a separate bf16 operand at these rates),
// and that every wave owns ALL C rows of its 32*TN columns.  A lane of a 32x32 MFMA accumulator tile
// holds column j and rows 8g + 4h + {0..3}; the B operand of the next MFMA wants, for the same column
// j, eight K values per lane.  So after bias + Snake the accumulators ARE the B fragments of the 1x1
// conv, provided its K axis is permuted to the accumulator's row order: k-slot (kk, h, e) <-> channel
// 32 (kk/2) + 8 (2 (kk%2) + e/4) + 4 h + e%4.  The 1x1 weights are packed in that order at create.
// In the 1x1 conv the roles are swapped: these fragments are the row operand (rows = time) and the weights the
// column operand, so its accumulator tile is [time][output channel] and a lane holds one output-channel slot j of
// each of the C/32 channel tiles.  The weight rows are packed so that slot j of tile mo is channel j C/32 + mo:
// a lane then owns C/32 consecutive channels of a time row, 32 lanes a whole row, and residual loads and
// stores are contiguous without a transposition through LDS.
// The result is written to a second buffer (neighbouring tiles still read this tile's input rows).
// With EMIT the kernel also writes bf16(snake_next(h_out)), the operand of the next (unfused) layer.
#include <algorithm>
#include <type_traits>

#include "device_common.h"

namespace demon {

constexpr int FUSED_MAXSPAN = 64;

struct FusedParams {
    const hres_t* x; hres_t* y;
    uint16_t* ya;                // optional activated bf16 copy of y (EMIT)
    const uint16_t* w7;          // [chunk][tap] blocks of C x 64 bf16
    const uint16_t* w1;          // [C][C] bf16, K axis permuted (see above)
    const float* b7; const float* b1;
    const float* a1; const float* ib1;    // Snake on the input (alpha in revolutions, 1/(beta+eps))
    const float* a2; const float* ib2;    // Snake between the two convolutions
    const float* a3; const float* ib3;    // Snake of the consumer (EMIT)
    const Slot* slots;
    int r, ntaps, tap0, tap_step, nchunks, margin;
    // HEAD: the decoder's head (Snake -> Conv1d(hk) -> tanh) on this unit's output, in the same kernel
    const uint16_t* hw;          // half-precision MFMA fragments of the head weights (pack_head_mfma)
    const float* hb; const float* ha; const float* hib;
    float* hy;                   // planar window waveforms [oc][total_rows]
    long long total_rows;
    int oc, hk;
};

// channel that k-slot kp (0..C-1) of the permuted 1x1 weight matrix multiplies
static inline int fused_k_to_channel(int kp)
{
    const int kk = kp / 16, h = (kp / 8) % 2, e = kp % 8;
    return 32 * (kk / 2) + 8 * (2 * (kk % 2) + e / 4) + 4 * h + e % 4;
}

void pack_w1_fused(const float* w /*[C][C]*/, int C, uint16_t* dst)
{
    const int tm = C / 32;
    for (int slot = 0; slot < C; ++slot) {
        const int o = (slot % 32) * tm + slot / 32;        // row slot (mo, j) holds output channel j * tm + mo
        for (int kp = 0; kp < C; ++kp) dst[(size_t)slot * C + kp] = f32_to_bf16_rne(w[(size_t)o * C + fused_k_to_channel(kp)]);
    }
}

// HEAD (64 channels, no EMIT): the unit is the decoder's last layer before the head.  Its output rows do not go to memory:
// Snake with the head's parameters, rounded to half, they fill an LDS tile (the activation tile's space, free after the K
// loop), the head's weight fragments take the weight buffer, and every wave runs the head's k x 4 k-steps on its 64
// columns exactly as head_mfma_kernel does (same operands, same order: the same bits).  A tile's head outputs need the
// unit's outputs (k-1)/2 columns to both sides, so tiles advance by NT - (k-1) columns and the first and last (k-1)/2
// columns of a tile only serve as context.  Saves the unit's 128-byte-per-row store, the head's read of it and a launch.
constexpr int FUSED_HEAD_MAXK = 7;      // k x 64 weight pieces of 16 bytes travel in two registers per thread

template <int CH, int TN, bool EMIT, bool HEAD = false>
__global__ __launch_bounds__(256, (CH == 128 && TN == 2) ? 2 : 3) void res_unit_fused_kernel(FusedParams p)
{
    static_assert(!HEAD || (CH == 64 && !EMIT), "the head follows a 64-channel unit that feeds nothing else");
    fp16_saturate_on();
    constexpr int KC = 64;
    constexpr int LDK = KC + 8;
    constexpr int NT = 4 * 32 * TN;               // four waves side by side in time
    constexpr int WTN = 32 * TN;
    constexpr int XR_MAX = NT + FUSED_MAXSPAN;
    constexpr int TM = CH / 32;
    constexpr int SEGS = KC / 8;
    constexpr int RPP = 256 / SEGS;
    constexpr int A_CH = CH * SEGS;
    constexpr int A_ITERS = A_CH / 256;
    constexpr int X_ITERS = (XR_MAX + RPP - 1) / RPP;
    constexpr int LD1 = CH + 8;                   // padded row of the 1x1 weight tile
    constexpr int W1_CH = CH * CH / 8;            // 16-byte chunks of the 1x1 weights
    static_assert(A_CH % 256 == 0 && W1_CH % 256 == 0, "staging loops assume whole passes");
    // 64 channels: LDS and registers are budgeted for three workgroups per CU (they hide each other's barriers and latencies
    // markedly better than two).  128 channels: two workgroups per CU with twice the columns per wave (TN = 2, 128
    // accumulator registers): 0.75 instead of 1.25 fragment reads per MFMA, half the weight staging and a quarter less
    // halo per column; per launch the same time as three workgroups of 128 columns, per step 1 % less (less LDS traffic
    // under the power limit).  Its residual values are requested after the 1x1 conv (no registers before).
    // Common to both: one weight buffer (the next block waits in registers and is stored between two
    // barriers), an activation tile without row padding (16-byte pieces XOR-swizzled by the row instead), the 1x1
    // weights and the residual values requested after the K loop.
    constexpr int LDX = KC;                       // unpadded row of the activation tile; piece sg of row r sits at sg ^ (r & 7)
    constexpr int AS_BYTES = CH * LDK * 2, XS_BYTES = XR_MAX * LDX * 2;
    constexpr int SMEM_BYTES = AS_BYTES + XS_BYTES;
    static_assert(CH * LD1 * 2 <= SMEM_BYTES, "the 1x1 weights reuse the buffers of the dilated conv");
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
    // per-channel vectors used after the K loop (bias of both convolutions, Snake between them): read from global
    // memory where they are used, each load would be waited for in turn
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
    const int hhalf = HEAD ? (p.hk - 1) / 2 : 0;
    // HEAD: the unit's columns start (k-1)/2 before the interior also at a clip edge (rows before the window are zero)
    const int n0 = HEAD ? s.crop * p.r - hhalf + tile * (NT - 2 * hhalf) : out_lo + tile * NT;
    const int h_lo = s.crop * p.r, h_hi = (s.crop + s.n_int) * p.r;     // HEAD: the interior rows the head produces
    if (HEAD ? (n0 + hhalf >= h_hi) : (n0 >= out_hi)) return;
    const long long rowbase = (long long)s.row0 * p.r;

    const int last_off = p.tap0 + (p.ntaps - 1) * p.tap_step;
    const int minoff = min(p.tap0, last_off);
    const int XR = NT + max(p.tap0, last_off) - minoff;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wn = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS, xr0 = tid / SEGS;

    // descriptors: one window of the input, the computed part of the window for the outputs
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.x + rowbase * CH, (unsigned)nrows * CH * (unsigned)sizeof(hres_t));
    const __amdgpu_buffer_rsrc_t rs_y = make_rsrc(p.y + rowbase * CH, (unsigned)out_hi * CH * (unsigned)sizeof(hres_t));
    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(p.ya + rowbase * CH, EMIT ? (unsigned)out_hi * CH * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(p.w7, (unsigned)(p.nchunks * p.ntaps) * (A_CH * 16u));

    const int nstages = p.nchunks * p.ntaps;
    const unsigned a_voff = tid * 16u;
    const unsigned x_voff = ((unsigned)((n0 + minoff + xr0) * CH) + seg * 8u) * (unsigned)sizeof(hres_t);   // may wrap "negative": out of range
    constexpr unsigned x_row_step = RPP * CH * (unsigned)sizeof(hres_t);

    u32x4 ra[A_ITERS];
    u32x4 rx[X_ITERS];           // 8 channels of one row (half)
    float al[8], ib[8];

    auto load_a = [&](int stage) __attribute__((always_inline)) {
        const unsigned base = (unsigned)stage * (A_CH * 16u);
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) ra[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, a_voff, base + it * 4096u, 0);
    };
    auto store_a = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) {
            const int q = tid + it * 256;
            *reinterpret_cast<u32x4*>(&As[(q / SEGS) * LDK + (q % SEGS) * 8]) = ra[it];
        }
    };
    auto load_x = [&](int chunk) __attribute__((always_inline)) {
        const unsigned coff = x_voff + (unsigned)(chunk * KC) * (unsigned)sizeof(hres_t);
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                        // uniform
            rx[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, coff + it * x_row_step, 0, 0);
        }
        const int cbase = chunk * KC + seg * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { al[e] = p.a1[cbase + e]; ib[e] = p.ib1[cbase + e]; }
    };
    auto store_x = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                        // uniform
            const int xr = xr0 + it * RPP;
            if (xr >= XR_MAX) continue;
            u32x4 v;
            const f16x8 hv = __builtin_bit_cast(f16x8, rx[it]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float e0 = (float)hv[2 * q], e1 = (float)hv[2 * q + 1];
                e0 = snake_fast(e0, al[2 * q], ib[2 * q]);
                e1 = snake_fast(e1, al[2 * q + 1], ib[2 * q + 1]);
                v[q] = pack_bf16x2(e0, e1);
            }
            *reinterpret_cast<u32x4*>(&Xs[xr * LDX + ((seg ^ (xr & 7)) * 8)]) = v;
        }
    };

    u32x4 rw1[W1_CH / 256];      // the 1x1 weights on their way to LDS
    auto load_w1 = [&]() __attribute__((always_inline)) {
        const u32x4* src = reinterpret_cast<const u32x4*>(p.w1);
#pragma unroll
        for (int it = 0; it < W1_CH / 256; ++it) rw1[it] = src[tid + it * 256];
    };

    // every request of the prologue is issued before the first result is waited for, in the order of use
    load_a(0);
    load_x(0);
    constexpr int PRM_ITERS = 4 * CH / 256;
    float pv[PRM_ITERS];
#pragma unroll
    for (int it = 0; it < PRM_ITERS; ++it) {
        const int i = tid + it * 256, which = i / CH, c = i % CH;
        const float* src = which == 0 ? p.b7 : which == 1 ? p.a2 : which == 2 ? p.ib2 : p.b1;
        pv[it] = src[c];
    }
    // The residual values this lane adds in the epilogue are requested in one go after the K loop, in the shadow of the
    // Snake and the 1x1 convolution: loaded where they are used, each would be waited for in turn, a chain of memory
    // latencies per tile (and held through the K loop they cost the registers of the third workgroup).
    // epilogue geometry: lane (j, h) owns channels j TM .. j TM + TM - 1 of time rows 8g + 4h + q of every 32-column tile
    using res_t = std::conditional_t<TM == 2, uint32_t, u32x2>;         // TM halves
    res_t resv[TN][16];
    auto res_offset = [&](int ni, int gq) -> unsigned {
        const int col = n0 + wn * WTN + ni * 32 + 8 * (gq >> 2) + 4 * h + (gq & 3);
        return (unsigned)(col * CH + j * TM) * 2u;
    };
    auto load_res = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int gq = 0; gq < 16; ++gq) {
                if constexpr (TM == 2) resv[ni][gq] = __builtin_amdgcn_raw_buffer_load_b32(rs_x, res_offset(ni, gq), 0, 0);
                else resv[ni][gq] = __builtin_amdgcn_raw_buffer_load_b64(rs_x, res_offset(ni, gq), 0, 0);
            }
    };
    store_a();
    store_x();
#pragma unroll
    for (int it = 0; it < PRM_ITERS; ++it) prm[tid + it * 256] = pv[it];
    __syncthreads();

    // accumulators start at the bias: lane (j, h) holds rows (channels) mi*32 + 8g + 4h + {0..3}
    f32x16 acc[TM][TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 b4 = *reinterpret_cast<const float4*>(&prm[mi * 32 + 8 * g + 4 * h]);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
                acc[mi][ni][4 * g + 0] = b4.x; acc[mi][ni][4 * g + 1] = b4.y;
                acc[mi][ni][4 * g + 2] = b4.z; acc[mi][ni][4 * g + 3] = b4.w;
            }
        }

    // ---- dilated conv: K loop over (chunk, tap) stages, fixed order
    int chunk = 0, tap = 0;
    for (int stage = 0; stage < nstages; ++stage) {
        int ntap = tap + 1, nchunk = chunk;
        if (ntap == p.ntaps) { ntap = 0; ++nchunk; }
        const bool more = stage + 1 < nstages;
        const bool new_chunk = more && nchunk != chunk;
        if (more) load_a(stage + 1);
        if (new_chunk) load_x(nchunk);

        const int off = p.tap0 + tap * p.tap_step - minoff;
        const uint16_t* abase = &As[j * LDK + h * 8];
        const int xrow = wn * WTN + j + off;                  // + ni * 32: the same row & 7
        const uint16_t* xbase = &Xs[xrow * LDX];
        const int r7 = xrow & 7;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const bf16x8*>(abase + mi * 32 * LDK + ks * 16);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(xbase + ni * 32 * LDX + (((2 * ks + h) ^ r7) * 8));
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }
        if constexpr (CH == 128) {
            // order of the stage's fragment reads and MFMAs: one k-step's reads plus two ahead, then one read per MFMA, so
            // that a fragment is requested a few MFMAs before it is used instead of right before the MFMAs of its own k-step
            // (the 64-channel form has no registers left for the fragments in flight)
            constexpr int R = (KC / 16) * (TM + TN), M = (KC / 16) * TM * TN;
            constexpr int LEAD = (TM + TN + 2) < R ? (TM + TN + 2) : R;
            constexpr int PAIRS = (R - LEAD) < M ? (R - LEAD) : M;
            __builtin_amdgcn_sched_group_barrier(0x100, LEAD, 0);
#pragma unroll
            for (int i = 0; i < PAIRS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, M - PAIRS, 0);
        }
        if (more) {
            __syncthreads();                                  // every wave is done with the weight buffer (and the X tile)
            if (new_chunk) store_x();
            store_a();
            __syncthreads();
        }
        tap = ntap; chunk = nchunk;
    }
    constexpr bool RES_LAST = CH == 128 && TN == 2;     // no registers for the residual values until the 1x1 conv is done
    load_w1();
    if (!RES_LAST) load_res();

    // ---- bias + Snake on the accumulators; repack them as the B fragments of the 1x1 conv
    u32x4 mid[CH / 16][TN];      // bf16x8 fragments, built from packed pairs
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = mi * 32 + 8 * g + 4 * h;
            const float4 a4 = *reinterpret_cast<const float4*>(&prm[CH + c]);
            const float4 i4 = *reinterpret_cast<const float4*>(&prm[2 * CH + c]);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
                const float v0 = snake_fast(acc[mi][ni][4 * g + 0], a4.x, i4.x);
                const float v1 = snake_fast(acc[mi][ni][4 * g + 1], a4.y, i4.y);
                const float v2 = snake_fast(acc[mi][ni][4 * g + 2], a4.z, i4.z);
                const float v3 = snake_fast(acc[mi][ni][4 * g + 3], a4.w, i4.w);
                u32x4& f = mid[2 * mi + g / 2][ni];
                f[2 * (g & 1) + 0] = pack_bf16x2(v0, v1);
                f[2 * (g & 1) + 1] = pack_bf16x2(v2, v3);
            }
        }
    }

    // ---- stage the 1x1 weights over the (now free) buffers of the dilated conv
    __syncthreads();                                   // all waves are done with the last stage's operands
#pragma unroll
    for (int it = 0; it < W1_CH / 256; ++it) {
        const int q = tid + it * 256;
        *reinterpret_cast<u32x4*>(&As[(q / (CH / 8)) * LD1 + (q % (CH / 8)) * 8]) = rw1[it];
    }
    __syncthreads();

    // ---- 1x1 conv: K = C channels straight from registers, as the row operand (rows = time); the accumulator tile
    // [time][channel slot] starts at the bias of the lane's channel j TM + mo
#pragma unroll
    for (int mo = 0; mo < TM; ++mo) {
        const float b1v = prm[3 * CH + j * TM + mo];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[mo][ni][q] = b1v;
    }
#pragma unroll
    for (int kk = 0; kk < CH / 16; ++kk) {
        bf16x8 af[TM];
#pragma unroll
        for (int mo = 0; mo < TM; ++mo) af[mo] = *reinterpret_cast<const bf16x8*>(&As[(mo * 32 + j) * LD1 + kk * 16 + h * 8]);
#pragma unroll
        for (int mo = 0; mo < TM; ++mo)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
                acc[mo][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mid[kk][ni]), af[mo], acc[mo][ni], 0, 0, 0);
    }

    if (RES_LAST) load_res();

    // ---- residual add and half store to the other buffer, straight from the accumulators: register 4g + q of tile
    // (mo, ni) is time row 8g + 4h + q, channel j TM + mo.  Rows past out_hi are outside the descriptors and dropped.
    float a3v[TM], i3v[TM];
#pragma unroll
    for (int mo = 0; mo < TM; ++mo) {
        a3v[mo] = EMIT ? p.a3[j * TM + mo] : 0.f;
        i3v[mo] = EMIT ? p.ib3[j * TM + mo] : 0.f;
    }
    // HEAD: the tile of head operands takes the activation tile's space (nothing reads that after the K loop; every wave
    // has passed the barriers that staged the 1x1 weights), rows shifted by (k-1)/2 so that a tap is a row offset >= 0
    constexpr int LDH = CH + 8;
    _Float16* Hs = reinterpret_cast<_Float16*>(smem + AS_BYTES);
    static_assert(!HEAD || (NT + FUSED_HEAD_MAXK - 1) * LDH * 2 <= XS_BYTES, "the head's operand tile fits the activation tile's space");
    float hav[TM], hiv[TM];
    u32x4 rhw[2];                 // the head's weight fragments on their way to LDS (at most 2 x 256 pieces of 16 bytes)
    const int n_hw = HEAD ? p.hk * (CH / 16) * 2 * 8 : 0;
    if constexpr (HEAD) {
#pragma unroll
        for (int mo = 0; mo < TM; ++mo) { hav[mo] = p.ha[j * TM + mo]; hiv[mo] = p.hib[j * TM + mo]; }
        const u32x4* src = reinterpret_cast<const u32x4*>(p.hw);          // [fragment][lane = h * 32 + channel][8 halves]
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int q = tid + it * 256;
            rhw[it] = q < n_hw ? src[(q / 8) * 32 + q % 8] : u32x4{0, 0, 0, 0};
        }
        // rows of the operand tile past the unit's columns (context of columns that are not produced): defined, unused
        for (int q = tid; q < 2 * hhalf * (CH / 2); q += 256) {
            const int rr = q / (CH / 2), cc = q % (CH / 2);
            const int row = rr < hhalf ? rr : NT + rr;
            *reinterpret_cast<uint32_t*>(&Hs[row * LDH + 2 * cc]) = 0u;
        }
    }
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int gq = 0; gq < 16; ++gq) {
            const unsigned off = res_offset(ni, gq);
            float v[TM];
            typedef _Float16 halfs_t __attribute__((ext_vector_type(TM)));
            const halfs_t r = __builtin_bit_cast(halfs_t, resv[ni][gq]);
            static_assert(sizeof(halfs_t) == sizeof(res_t), "TM halves");
            halfs_t o;
#pragma unroll
            for (int mo = 0; mo < TM; ++mo) {
                v[mo] = acc[mo][ni][gq] + (float)r[mo];
                o[mo] = (_Float16)v[mo];                         // round to nearest even
            }
            if constexpr (HEAD) {
                // the head's operand: Snake of the (half) value the unit would have stored, in fp32, rounded once to half;
                // rows outside the window are the head conv's zero padding
                const int col = wn * WTN + ni * 32 + 8 * (gq >> 2) + 4 * h + (gq & 3);
                const int n = n0 + col;
                f16x2 av = {(_Float16)0.f, (_Float16)0.f};
                if (n >= 0 && n < nrows) {
                    av[0] = (_Float16)keep_f32(snake_fast((float)o[0], hav[0], hiv[0]));
                    av[1] = (_Float16)keep_f32(snake_fast((float)o[1], hav[1], hiv[1]));
                }
                *reinterpret_cast<f16x2*>(&Hs[(col + hhalf) * LDH + j * TM]) = av;
                continue;
            }
            if constexpr (TM == 2) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, o), rs_y, off, 0, 2);
            else __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, o), rs_y, off, 0, 2);
            if (EMIT) {
                // the next layer's operand is Snake of the STORED value
                uint32_t sh[TM / 2];
#pragma unroll
                for (int mo = 0; mo < TM; mo += 2) {
                    const float e0 = snake_fast((float)o[mo], a3v[mo], i3v[mo]);
                    const float e1 = snake_fast((float)o[mo + 1], a3v[mo + 1], i3v[mo + 1]);
                    sh[mo / 2] = pack_bf16x2(e0, e1);
                }
                if constexpr (TM == 2) __builtin_amdgcn_raw_buffer_store_b32(sh[0], rs_a, off, 0, 2);
                else { const u32x2 s2 = {sh[0], sh[1]}; __builtin_amdgcn_raw_buffer_store_b64(s2, rs_a, off, 0, 2); }
            }
        }
    if constexpr (HEAD) {
        // ---- the head on this tile: weights -> LDS (over the 1x1 weights), then per wave 2 column tiles x k taps x 4 k-steps
        uint16_t* Ws = reinterpret_cast<uint16_t*>(smem);          // [fragment][h][channel < 8][8 halves]
        __syncthreads();                                   // the operand tile is complete; nobody reads the 1x1 weights any more
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int q = tid + it * 256;
            if (q < n_hw) reinterpret_cast<u32x4*>(Ws)[q] = rhw[it];
        }
        __syncthreads();
        typedef _Float16 f16x8v __attribute__((ext_vector_type(8)));
        constexpr int KS = CH / 16;
        float hbv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) hbv[q] = (4 * h + q < p.oc) ? p.hb[4 * h + q] : 0.f;
        f32x16 hacc[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int q = 0; q < 16; ++q) hacc[mi][q] = q < 4 ? hbv[q] : 0.f;
        for (int t = 0; t < p.hk; ++t) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                f16x8v bw = {0, 0, 0, 0, 0, 0, 0, 0};
                if (j < 8) bw = *reinterpret_cast<const f16x8v*>(&Ws[(((t * KS + ks) * 2 + h) * 8 + j) * 8]);
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    const f16x8v av = *reinterpret_cast<const f16x8v*>(&Hs[(wn * WTN + mi * 32 + j + t) * LDH + ks * 16 + h * 8]);
                    // weights as the row operand: the accumulator tile is [output channel][time]
                    hacc[mi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bw, av, hacc[mi], 0, 0, 0);
                }
            }
        }
        // lane (j, h) holds time column j and output channels 4 h + {0..3} in its first four registers
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const int col = wn * WTN + mi * 32 + j;
            const int n = n0 + col;
            if (col < hhalf || col >= NT - hhalf || n < h_lo || n >= h_hi) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = 4 * h + q;
                if (c < p.oc) p.hy[(size_t)c * p.total_rows + rowbase + n] = tanhf(hacc[mi][q]);
            }
        }
    }
}

hipError_t launch_res_unit_fused(const FusedArgs& a, hipStream_t stream)
{
    FusedParams p;
    p.x = (const hres_t*)a.x; p.y = (hres_t*)a.y; p.ya = a.ya; p.w7 = a.w7; p.w1 = a.w1; p.b7 = a.b7; p.b1 = a.b1;
    p.a1 = a.a1; p.ib1 = a.ib1; p.a2 = a.a2; p.ib2 = a.ib2; p.a3 = a.a3; p.ib3 = a.ib3;
    p.slots = a.slots; p.r = a.r; p.ntaps = a.ntaps;
    p.tap0 = -((a.ntaps - 1) / 2) * a.dil; p.tap_step = a.dil;
    p.nchunks = a.c / 64; p.margin = a.margin;
    if ((a.c != 64 && a.c != 128) || (a.ntaps - 1) * a.dil > FUSED_MAXSPAN || a.margin < 0 || a.x == a.y) return hipErrorInvalidValue;
    if (a.ya && (!a.a3 || !a.ib3)) return hipErrorInvalidValue;
    // one window's activation plane must fit a 32-bit byte offset (buffer descriptors)
    if ((long long)a.max_len * a.r * a.c * (long long)sizeof(hres_t) > 0xf0000000ll) return hipErrorInvalidValue;
    const long long out_rows = std::min((long long)a.max_int * a.r + 2ll * a.margin, (long long)a.max_len * a.r);
    const bool emit = a.ya != nullptr;
    if (a.hw) {
        // the unit before the head, with the head in the same kernel: tiles advance by NT - (k - 1) interior columns
        if (a.c != 64 || a.ya || !a.hy || !a.hb || !a.ha || !a.hib || a.hk < 1 || (a.hk & 1) == 0 || a.hk > FUSED_HEAD_MAXK ||
            a.oc < 1 || a.oc > 8 || a.margin < (a.hk - 1) / 2) return hipErrorInvalidValue;
        p.hw = a.hw; p.hb = a.hb; p.ha = a.ha; p.hib = a.hib; p.hy = a.hy; p.total_rows = a.total_rows; p.oc = a.oc; p.hk = a.hk;
        constexpr int NT = 4 * 32 * 2;
        const long long interior = (long long)a.max_int * a.r;
        const long long per_tile = NT - (a.hk - 1);
        dim3 grid((unsigned)((interior + per_tile - 1) / per_tile + 7) / 8 * 8, (unsigned)a.n_slots);
        hipLaunchKernelGGL((res_unit_fused_kernel<64, 2, false, true>), grid, dim3(256), 0, stream, p);
        return hipGetLastError();
    }
    p.hw = nullptr; p.hb = p.ha = p.hib = nullptr; p.hy = nullptr; p.total_rows = 0; p.oc = p.hk = 0;
    if (a.c == 64) {
        constexpr int NT = 4 * 32 * 2;
        dim3 grid((unsigned)((out_rows + NT - 1) / NT + 7) / 8 * 8, (unsigned)a.n_slots);       // whole groups of 8 tiles; the surplus exits at once
        if (emit) hipLaunchKernelGGL((res_unit_fused_kernel<64, 2, true>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((res_unit_fused_kernel<64, 2, false>), grid, dim3(256), 0, stream, p);
    } else {
        constexpr int NT = 4 * 32 * 2;
        dim3 grid((unsigned)((out_rows + NT - 1) / NT + 7) / 8 * 8, (unsigned)a.n_slots);       // whole groups of 8 tiles; the surplus exits at once
        if (emit) hipLaunchKernelGGL((res_unit_fused_kernel<128, 2, true>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((res_unit_fused_kernel<128, 2, false>), grid, dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace demon
