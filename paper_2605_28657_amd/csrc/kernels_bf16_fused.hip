// Fused residual unit for the narrow, high-rate levels (C = 64 or 128 channels):
//     h_out = h + W1 * snake2(W7 (*) snake1(h) + b7) + b1
// in one kernel, so that the activated branch tensor never goes to HBM.
//
// The dilated conv runs as in kernels_bf16.hip (implicit GEMM, rows = output channels, columns = time,
// activation tile staged once per channel chunk with Snake applied, weight blocks double-buffered),
// with every wave owning ALL C rows of its 32*TN columns.  A lane of a 32x32 MFMA accumulator tile
// holds column j and rows 8g + 4h + {0..3}; the B operand of the next MFMA wants, for the same column
// j, eight K values per lane.  So after bias + Snake the accumulators ARE the B fragments of the 1x1
// conv, provided its K axis is permuted to the accumulator's row order: k-slot (kk, h, e) <-> channel
// 32 (kk/2) + 8 (2 (kk%2) + e/4) + 4 h + e%4.  The 1x1 weights are packed in that order at create.
// The result is written to a second buffer (neighbouring tiles still read this tile's input rows).
#include <stdlib.h>

#include <algorithm>

#include "device_common.h"

namespace demon {

constexpr int FUSED_MAXSPAN = 64;
// DEMON_VAE_C64_STREAMING=1 selects the non-persistent kernel for 64-channel units (A/B timing).
static const bool g_c64_streaming = getenv("DEMON_VAE_C64_STREAMING") != nullptr;

struct FusedParams {
    const float* x; float* y;
    const uint16_t* w7;          // [chunk][tap] blocks of C x 64 bf16
    const uint16_t* w1;          // [C][C] bf16, K axis permuted (see above)
    const float* b7; const float* b1;
    const float* a1; const float* ib1;    // Snake on the input (alpha in revolutions, 1/(beta+eps))
    const float* a2; const float* ib2;    // Snake between the two convolutions
    const Slot* slots;
    int r, ntaps, tap0, tap_step, nchunks, margin;
};

// channel that k-slot kp (0..C-1) of the permuted 1x1 weight matrix multiplies
static inline int fused_k_to_channel(int kp)
{
    const int kk = kp / 16, h = (kp / 8) % 2, e = kp % 8;
    return 32 * (kk / 2) + 8 * (2 * (kk % 2) + e / 4) + 4 * h + e % 4;
}

void pack_w1_fused(const float* w /*[C][C]*/, int C, uint16_t* dst)
{
    for (int o = 0; o < C; ++o)
        for (int kp = 0; kp < C; ++kp) dst[(size_t)o * C + kp] = f32_to_bf16_rne(w[(size_t)o * C + fused_k_to_channel(kp)]);
}

template <int CH, int TN>
__global__ __launch_bounds__(256) void res_unit_fused_kernel(FusedParams p)
{
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
    static_assert(CH * LD1 <= 2 * CH * LDK, "the 1x1 weights reuse the dilated-conv weight buffers");

    __shared__ __attribute__((aligned(16))) uint16_t As[2 * CH * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Xs[XR_MAX * LDK];

    const Slot s = p.slots[blockIdx.y];
    const int nrows = s.len * p.r;
    const int out_lo = max(0, s.crop * p.r - p.margin);
    const int out_hi = min(nrows, (s.crop + s.n_int) * p.r + p.margin);
    const int n0 = out_lo + blockIdx.x * NT;
    if (n0 >= out_hi) return;
    const long long rowbase = (long long)s.row0 * p.r;

    const int last_off = p.tap0 + (p.ntaps - 1) * p.tap_step;
    const int minoff = min(p.tap0, last_off);
    const int XR = NT + max(p.tap0, last_off) - minoff;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wn = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS, xr0 = tid / SEGS;

    const int nstages = p.nchunks * p.ntaps;
    const u32x4* wblk = reinterpret_cast<const u32x4*>(p.w7);

    u32x4 ra[A_ITERS];
    u32x4 rx[X_ITERS][2];
    float al[8], ib[8];

    auto load_a = [&](int stage) __attribute__((always_inline)) {
        const u32x4* src = wblk + (size_t)stage * A_CH;
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) ra[it] = src[tid + it * 256];
    };
    auto store_a = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) {
            const int q = tid + it * 256;
            *reinterpret_cast<u32x4*>(&As[buf * CH * LDK + (q / SEGS) * LDK + (q % SEGS) * 8]) = ra[it];
        }
    };
    auto load_x = [&](int chunk) __attribute__((always_inline)) {
        const int cbase = chunk * KC + seg * 8;
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            const int srow = n0 + minoff + xr;
            const bool ok = xr < XR && srow >= 0 && srow < nrows;
            const size_t e0 = (size_t)(rowbase + srow) * CH + cbase;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = reinterpret_cast<const u32x4*>(p.x + e0)[q];
                rx[it][q] = v;
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { al[e] = p.a1[cbase + e]; ib[e] = p.ib1[cbase + e]; }
    };
    auto store_x = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            if (xr >= XR_MAX) continue;
            u32x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float e0 = __uint_as_float(rx[it][q >> 1][(2 * q) & 3]), e1 = __uint_as_float(rx[it][q >> 1][(2 * q + 1) & 3]);
                e0 = snake_fast(e0, al[2 * q], ib[2 * q]);
                e1 = snake_fast(e1, al[2 * q + 1], ib[2 * q + 1]);
                v[q] = (uint32_t)f32_to_bf16_bits(e0) | ((uint32_t)f32_to_bf16_bits(e1) << 16);
            }
            *reinterpret_cast<u32x4*>(&Xs[xr * LDK + seg * 8]) = v;
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    load_a(0);
    load_x(0);
    store_a(0);
    store_x();
    __syncthreads();

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
        const uint16_t* abase = &As[(stage & 1) * CH * LDK + j * LDK + h * 8];
        const uint16_t* xbase = &Xs[(wn * WTN + j + off) * LDK + h * 8];
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const bf16x8*>(abase + mi * 32 * LDK + ks * 16);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(xbase + ni * 32 * LDK + ks * 16);
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }
        if (more) {
            if (new_chunk) {
                __syncthreads();
                store_x();
            }
            store_a((stage + 1) & 1);
            __syncthreads();
        }
        tap = ntap; chunk = nchunk;
    }

    // ---- stage the 1x1 weights into the (now free) weight buffers
    __syncthreads();
    {
        const u32x4* src = reinterpret_cast<const u32x4*>(p.w1);
#pragma unroll
        for (int it = 0; it < W1_CH / 256; ++it) {
            const int q = tid + it * 256;
            *reinterpret_cast<u32x4*>(&As[(q / (CH / 8)) * LD1 + (q % (CH / 8)) * 8]) = src[q];
        }
    }

    // ---- bias + Snake on the accumulators; repack them as the B fragments of the 1x1 conv
    bf16x8 mid[CH / 16][TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = mi * 32 + 8 * g + 4 * h;
            const float4 b4 = *reinterpret_cast<const float4*>(p.b7 + c);
            const float4 a4 = *reinterpret_cast<const float4*>(p.a2 + c);
            const float4 i4 = *reinterpret_cast<const float4*>(p.ib2 + c);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
                const float v0 = snake_fast(acc[mi][ni][4 * g + 0] + b4.x, a4.x, i4.x);
                const float v1 = snake_fast(acc[mi][ni][4 * g + 1] + b4.y, a4.y, i4.y);
                const float v2 = snake_fast(acc[mi][ni][4 * g + 2] + b4.z, a4.z, i4.z);
                const float v3 = snake_fast(acc[mi][ni][4 * g + 3] + b4.w, a4.w, i4.w);
                bf16x8& f = mid[2 * mi + g / 2][ni];
                f[4 * (g & 1) + 0] = (__bf16)v0; f[4 * (g & 1) + 1] = (__bf16)v1;
                f[4 * (g & 1) + 2] = (__bf16)v2; f[4 * (g & 1) + 3] = (__bf16)v3;
            }
        }
    }
    __syncthreads();

    // ---- 1x1 conv, K = C channels straight from registers, computed TRANSPOSED: the activated tile is
    // the A operand (rows = time) and the weights the B operand (columns = output channel), so a lane
    // ends up with one output channel and 16 time rows, and every global access of the epilogue is a
    // run of 32 consecutive channels (128 contiguous bytes) of one row.
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < CH / 16; ++kk) {
        bf16x8 wf[TM];
#pragma unroll
        for (int mo = 0; mo < TM; ++mo) wf[mo] = *reinterpret_cast<const bf16x8*>(&As[(mo * 32 + j) * LD1 + kk * 16 + h * 8]);
#pragma unroll
        for (int mo = 0; mo < TM; ++mo)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
                acc[mo][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mid[kk][ni], wf[mo], acc[mo][ni], 0, 0, 0);
    }

    // ---- bias + residual, fp32 store to the other buffer: lane (j, h) holds channel mo*32 + j, rows 8g + 4h + r
#pragma unroll
    for (int mo = 0; mo < TM; ++mo) {
        const int c = mo * 32 + j;
        const float b = p.b1[c];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int col = n0 + wn * WTN + ni * 32 + 8 * g + 4 * h + r;
                    if (col >= out_hi) continue;
                    const size_t idx = (size_t)(rowbase + col) * CH + c;
                    p.y[idx] = acc[mo][ni][4 * g + r] + b + p.x[idx];
                }
    }
}

// ------------------------------------------------------------------------------------------------
// C = 64: persistent variant.  All weights of the unit (57 KB + 8 KB) stay in LDS for the lifetime of
// the workgroup, which walks over many time tiles: the K loop of a tile has no barrier at all, the
// fp32 rows of the next tile are fetched while the current tile is in the MFMA loop, and Snake + the
// bf16 conversion of those rows go into the second activation buffer afterwards (one barrier per tile).
template <int TN>
__global__ __launch_bounds__(256) void res_unit_c64_persistent_kernel(FusedParams p, int tiles_per_slot, int total_tiles)
{
    constexpr int CH = 64;
    constexpr int LDK = CH + 8;                   // activation tile row (bf16)
    constexpr int NT = 4 * 32 * TN;
    constexpr int WTN = 32 * TN;
    constexpr int XR_MAX = NT + FUSED_MAXSPAN;
    constexpr int TM = CH / 32;
    constexpr int SEGS = CH / 8;
    constexpr int RPP = 256 / SEGS;
    constexpr int X_ITERS = (XR_MAX + RPP - 1) / RPP;
    constexpr int MAXTAPS = 7;
    constexpr int LDW = MAXTAPS * CH + 8;         // dilated-conv weight row: [tap][channel] + pad
    constexpr int LD1 = CH + 8;

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* W7s = smem;                          // [CH][LDW]
    uint16_t* W1s = W7s + CH * LDW;                // [CH][LD1]
    uint16_t* Xs = W1s + CH * LD1;                 // [2][XR_MAX][LDK]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wn = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS, xr0 = tid / SEGS;

    const int last_off = p.tap0 + (p.ntaps - 1) * p.tap_step;
    const int minoff = min(p.tap0, last_off);
    const int XR = NT + max(p.tap0, last_off) - minoff;

    // tile -> (slot, first column); returns false for the empty tiles of short windows
    auto tile_info = [&](int tile, long long& rowbase, int& nrows, int& n0, int& out_hi) __attribute__((always_inline)) -> bool {
        const Slot s = p.slots[tile / tiles_per_slot];
        nrows = s.len * p.r;
        const int out_lo = max(0, s.crop * p.r - p.margin);
        out_hi = min(nrows, (s.crop + s.n_int) * p.r + p.margin);
        n0 = out_lo + (tile % tiles_per_slot) * NT;
        rowbase = (long long)s.row0 * p.r;
        return n0 < out_hi;
    };
    auto next_valid = [&](int tile) __attribute__((always_inline)) -> int {
        long long rb; int nr, n0, oh;
        while (tile < total_tiles && !tile_info(tile, rb, nr, n0, oh)) tile += gridDim.x;
        return tile;
    };

    u32x4 rx[X_ITERS][2];
    float al[8], ib[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { al[e] = p.a1[seg * 8 + e]; ib[e] = p.ib1[seg * 8 + e]; }

    auto load_x = [&](long long rowbase, int nrows, int n0) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            const int srow = n0 + minoff + xr;
            const bool ok = xr < XR && srow >= 0 && srow < nrows;
            const size_t e0 = (size_t)(rowbase + srow) * CH + seg * 8;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = reinterpret_cast<const u32x4*>(p.x + e0)[q];
                rx[it][q] = v;
            }
        }
    };
    auto store_x = [&](int buf) __attribute__((always_inline)) {
        uint16_t* dst = Xs + buf * XR_MAX * LDK;
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            if (xr >= XR_MAX) continue;
            u32x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float e0 = __uint_as_float(rx[it][q >> 1][(2 * q) & 3]), e1 = __uint_as_float(rx[it][q >> 1][(2 * q + 1) & 3]);
                e0 = snake_fast(e0, al[2 * q], ib[2 * q]);
                e1 = snake_fast(e1, al[2 * q + 1], ib[2 * q + 1]);
                v[q] = (uint32_t)f32_to_bf16_bits(e0) | ((uint32_t)f32_to_bf16_bits(e1) << 16);
            }
            *reinterpret_cast<u32x4*>(&dst[xr * LDK + seg * 8]) = v;
        }
    };

    int cur = next_valid(blockIdx.x);
    if (cur >= total_tiles) return;
    long long rowbase; int nrows, n0, out_hi;
    tile_info(cur, rowbase, nrows, n0, out_hi);
    load_x(rowbase, nrows, n0);

    // weights -> LDS, once per workgroup
    {
        const u32x4* src = reinterpret_cast<const u32x4*>(p.w7);       // [tap] blocks of CH x CH
        for (int q = tid; q < p.ntaps * CH * SEGS; q += 256) {
            const int t = q / (CH * SEGS), rem = q % (CH * SEGS);
            *reinterpret_cast<u32x4*>(&W7s[(rem / SEGS) * LDW + t * CH + (rem % SEGS) * 8]) = src[q];
        }
        const u32x4* src1 = reinterpret_cast<const u32x4*>(p.w1);
        for (int q = tid; q < CH * SEGS; q += 256)
            *reinterpret_cast<u32x4*>(&W1s[(q / SEGS) * LD1 + (q % SEGS) * 8]) = src1[q];
    }
    store_x(0);
    __syncthreads();

    // per-lane epilogue constants: channels mi*32 + 8g + 4h + {0..3}
    float4 b7v[TM][4], a2v[TM][4], i2v[TM][4];
    float b1s[TM];
#pragma unroll
    for (int mo = 0; mo < TM; ++mo) b1s[mo] = p.b1[mo * 32 + j];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = mi * 32 + 8 * g + 4 * h;
            b7v[mi][g] = *reinterpret_cast<const float4*>(p.b7 + c);
            a2v[mi][g] = *reinterpret_cast<const float4*>(p.a2 + c);
            i2v[mi][g] = *reinterpret_cast<const float4*>(p.ib2 + c);
        }

    int buf = 0;
    while (cur < total_tiles) {
        const int nxt = next_valid(cur + gridDim.x);
        long long rowbase_n = 0; int nrows_n = 0, n0_n = 0, out_hi_n = 0;
        if (nxt < total_tiles) {
            tile_info(nxt, rowbase_n, nrows_n, n0_n, out_hi_n);
            load_x(rowbase_n, nrows_n, n0_n);
        }
        // residual values of this tile (fp32), fetched early, in the layout of the transposed 1x1 conv:
        // lane (j, h) owns channel mo*32 + j and rows 8g + 4h + r
        float res[TM][TN][16];
#pragma unroll
        for (int mo = 0; mo < TM; ++mo)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int col = n0 + wn * WTN + ni * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                    res[mo][ni][q] = (col < out_hi) ? p.x[(size_t)(rowbase + col) * CH + mo * 32 + j] : 0.f;
                }

        f32x16 acc[TM][TN];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

        const uint16_t* xt = Xs + buf * XR_MAX * LDK;
        for (int t = 0; t < p.ntaps; ++t) {
            const int off = p.tap0 + t * p.tap_step - minoff;
            const uint16_t* abase = &W7s[j * LDW + t * CH + h * 8];
            const uint16_t* xbase = &xt[(wn * WTN + j + off) * LDK + h * 8];
#pragma unroll
            for (int ks = 0; ks < CH / 16; ++ks) {
                bf16x8 af[TM], bfr[TN];
#pragma unroll
                for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const bf16x8*>(abase + mi * 32 * LDW + ks * 16);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(xbase + ni * 32 * LDK + ks * 16);
#pragma unroll
                for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                    for (int ni = 0; ni < TN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
            }
        }

        bf16x8 mid[CH / 16][TN];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    const float v0 = snake_fast(acc[mi][ni][4 * g + 0] + b7v[mi][g].x, a2v[mi][g].x, i2v[mi][g].x);
                    const float v1 = snake_fast(acc[mi][ni][4 * g + 1] + b7v[mi][g].y, a2v[mi][g].y, i2v[mi][g].y);
                    const float v2 = snake_fast(acc[mi][ni][4 * g + 2] + b7v[mi][g].z, a2v[mi][g].z, i2v[mi][g].z);
                    const float v3 = snake_fast(acc[mi][ni][4 * g + 3] + b7v[mi][g].w, a2v[mi][g].w, i2v[mi][g].w);
                    bf16x8& f = mid[2 * mi + g / 2][ni];
                    f[4 * (g & 1) + 0] = (__bf16)v0; f[4 * (g & 1) + 1] = (__bf16)v1;
                    f[4 * (g & 1) + 2] = (__bf16)v2; f[4 * (g & 1) + 3] = (__bf16)v3;
                }

#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < CH / 16; ++kk) {
            bf16x8 wf[TM];
#pragma unroll
            for (int mo = 0; mo < TM; ++mo) wf[mo] = *reinterpret_cast<const bf16x8*>(&W1s[(mo * 32 + j) * LD1 + kk * 16 + h * 8]);
#pragma unroll
            for (int mo = 0; mo < TM; ++mo)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    acc[mo][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mid[kk][ni], wf[mo], acc[mo][ni], 0, 0, 0);   // transposed
        }

#pragma unroll
        for (int mo = 0; mo < TM; ++mo)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int col = n0 + wn * WTN + ni * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                    if (col >= out_hi) continue;
                    p.y[(size_t)(rowbase + col) * CH + mo * 32 + j] = acc[mo][ni][q] + b1s[mo] + res[mo][ni][q];
                }

        if (nxt < total_tiles) store_x(buf ^ 1);
        __syncthreads();
        cur = nxt; buf ^= 1;
        rowbase = rowbase_n; nrows = nrows_n; n0 = n0_n; out_hi = out_hi_n;
    }
}

static size_t c64_persistent_lds_bytes(int TN)
{
    const int NT = 4 * 32 * TN;
    return sizeof(uint16_t) * ((size_t)64 * (7 * 64 + 8) + 64 * 72 + 2 * (size_t)(NT + FUSED_MAXSPAN) * 72);
}

hipError_t launch_res_unit_fused(const FusedArgs& a, hipStream_t stream)
{
    FusedParams p;
    p.x = a.x; p.y = a.y; p.w7 = a.w7; p.w1 = a.w1; p.b7 = a.b7; p.b1 = a.b1;
    p.a1 = a.a1; p.ib1 = a.ib1; p.a2 = a.a2; p.ib2 = a.ib2;
    p.slots = a.slots; p.r = a.r; p.ntaps = a.ntaps;
    p.tap0 = -((a.ntaps - 1) / 2) * a.dil; p.tap_step = a.dil;
    p.nchunks = a.c / 64; p.margin = a.margin;
    if ((a.c != 64 && a.c != 128) || (a.ntaps - 1) * a.dil > FUSED_MAXSPAN || a.margin < 0 || a.x == a.y) return hipErrorInvalidValue;
    if ((long long)a.max_len * a.r > 0x3fffffffll) return hipErrorInvalidValue;
    const long long out_rows = std::min((long long)a.max_int * a.r + 2ll * a.margin, (long long)a.max_len * a.r);
    if (a.c == 64 && a.ntaps <= 7 && !g_c64_streaming) {
        constexpr int TN = 2, NT = 4 * 32 * TN;
        const size_t lds = c64_persistent_lds_bytes(TN);
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&res_unit_c64_persistent_kernel<TN>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        const int tiles_per_slot = (int)((out_rows + NT - 1) / NT);
        const long long total = (long long)tiles_per_slot * a.n_slots;
        if (total > 0x7fffffffll) return hipErrorInvalidValue;
        int ncu = 256;
        (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, 0);
        const int grid = (int)std::min<long long>(total, ncu);
        hipLaunchKernelGGL((res_unit_c64_persistent_kernel<TN>), dim3((unsigned)grid), dim3(256), lds, stream, p, tiles_per_slot, (int)total);
    } else if (a.c == 64) {
        constexpr int NT = 4 * 32 * 2;
        dim3 grid((unsigned)((out_rows + NT - 1) / NT), (unsigned)a.n_slots);
        hipLaunchKernelGGL((res_unit_fused_kernel<64, 2>), grid, dim3(256), 0, stream, p);
    } else {
        constexpr int NT = 4 * 32 * 1;
        dim3 grid((unsigned)((out_rows + NT - 1) / NT), (unsigned)a.n_slots);
        hipLaunchKernelGGL((res_unit_fused_kernel<128, 1>), grid, dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace demon
