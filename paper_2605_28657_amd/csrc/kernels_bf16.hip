// bf16 MFMA implicit-GEMM convolution kernels for gfx950 (CDNA4).
//
// Every convolution of the decoder is one GEMM  D[mu, n] = sum_{t, i} A[mu, (t, i)] * X[n + off_t, i]:
//   Conv1d(k, dilation d):            mu = output channel, off_t = (t - (k-1)/2) d
//   ConvTranspose1d(2s, s, p = s/2):  polyphase form, mu = phi*cout + o, column n = input position m in [0, L],
//                                     taps j in {0,1} with off_j = -j and weight W[i, o, phi + j s];
//                                     column m, row mu lands on output sample m s - p + phi, channel o,
//                                     i.e. on the contiguous run ((m s - p) cout + mu) of the time-major output.
//   strided Conv1d(2s, s, p = s/2):   (the encoder's downsampling) the s/2 input rows n s/2 .. n s/2 + s/2 - 1 of the
//                                     time-major input are ONE row of (s/2) cin channels; output n then reads the four
//                                     merged rows 2n - 1 .. 2n + 2: mu = output channel, taps u in {0..3} with
//                                     off_u = u - 1 on columns that advance two merged rows per output, and weight
//                                     W[o, i, u s/2 + rho] for merged channel rho cin + i.
//
// Data flow.  The residual stream h is IEEE half in HBM (rounding it to bf16 after every layer alone would
// use up the error budget of the bf16 path; all arithmetic on it is fp32).  MFMA operands are bf16 and are produced exactly once, by
// the kernel that computes the value: every epilogue that writes h also writes a = bf16(snake(h)) with
// the Snake parameters of the layer that will consume it, so the GEMM kernels stage their activation
// operand with plain 16-byte copies (no transcendental work in the K loop, none repeated per row tile
// or per halo).  Activations are time-major [rows, channels]: the 8 consecutive K values an MFMA lane
// needs are 16 contiguous bytes, and a tap is a row offset into the same LDS tile.
//
// Operand formats.  Where rounding an activation operand to bf16 costs too much accuracy (the wide, low-rate
// levels, whose branch gain is about one) it is carried with more mantissa bits: as IEEE half (11 bits) on the
// f16 MFMA, which runs at the bf16 rate -- the weights, bf16 values, are exact in half, and the operand has the
// range of the half residual stream it is computed from -- or as hi + lo, hi = bf16(v), lo = bf16(v - hi), in
// two planes with two bf16 MFMAs per k-step against the same weight fragment (16 bits, at twice the MFMA work).
//
// All global accesses go through buffer descriptors that cover exactly one window (rows of other
// windows, rows before the window and rows past the part of the cone being computed are out of range:
// loads return zero = the convolution's zero padding at a clip edge, stores are dropped), so the
// kernel has no per-row branches and all offsets are 32-bit.
//
// Orientation of the accumulators.  The activation fragments are the row operand of the MFMA (rows = time) and the
// weight fragments the column operand, so a 32 x 32 accumulator tile is [time][GEMM row slot]: lane (j, h) holds slot j
// of each of the wave's TM row tiles, for the time rows 8g + 4h + {0..3}.  The weights are packed so that slot j of
// tile mi is GEMM row j TM + mi of the wave's block: a lane owns TM consecutive output channels of a time row and 32
// lanes a contiguous run of 32 TM channels, so residual loads and all stores go straight from the accumulators in
// whole runs (no transposition through LDS).
//
// Accumulation is fp32 in a fixed order (chunk-major, then tap, then channel), independent of where the
// tile sits in the window, so a windowed decode reproduces the full decode bit for bit.
#include <stdlib.h>

#include <algorithm>
#include <type_traits>

#include "device_common.h"

namespace demon {

constexpr int MAXSPAN = 64;    // largest (max tap offset - min tap offset) the LDS tile is sized for

enum { MODE_ACT = 0,   // bias + Snake, bf16 out only                     (dilated conv of a residual unit)
       MODE_RES = 1,   // bias + residual add in fp32, half out in place  (1x1 conv of a residual unit)
       MODE_UP  = 2,   // bias, polyphase scatter, half out               (ConvTranspose1d)
       MODE_DOWN = 3 };// bias, half out; columns step two input rows     (strided Conv1d on merged rows)
// MODE_RES, MODE_UP and MODE_DOWN may in addition emit the activated operand of the next layer: EMIT = 0 none, else the
// operand format + 1 (1 bf16, 2 bf16 hi + lo, 3 half).  IN is the operand format of the input.

struct MfmaParams {
    const uint16_t* xa;      // activated input, 16-bit [rows][cin] in the kernel's IN format; lo plane at xa + in_lo_off
    const uint16_t* w;       // packed weight blocks
    const float* bias;
    hres_t* y;               // residual-stream output; MODE_RES: also the residual source (in place); unused in MODE_ACT
    uint16_t* ya;            // activated output in the kernel's EMIT format; lo plane at ya + out_lo_off
    const float* out_alpha; const float* out_inv_beta;   // Snake applied before writing ya
    const Slot* slots;
    int r_in, cin, cout, ntaps, tap0, tap_step, stride, nchunks, margin;
    int mtiles_x;            // > 0: blockIdx.x enumerates (column tile, row tile), see the kernel; 0: blockIdx.z = row tile
    int xcd_group;           // with mtiles_x: 1 = all row tiles of a column tile on one XCD, 0 = row tiles dealt over the XCDs
    unsigned w_bytes;
    int pack_ratio;          // the weights are packed in blocks of pack_ratio * MT rows (1, or 2 for the small-grid tile)
    long long in_lo_off, out_lo_off;     // element offsets of the lo planes
};

struct Variant { int MT, NT, KC; };
// variant 3 only names a weight layout: blocks of 256 x 32 for the fused 256-channel unit (kernels_bf16_wide.hip)
static const Variant kVariants[4] = {{128, 128, 64}, {64, 256, 64}, {32, 128, 16}, {256, 128, 32}};

int choose_variant_bf16(int cin, int m)
{
    if (cin % 64 == 0 && m % 128 == 0) return 0;
    if (cin % 64 == 0 && m % 64 == 0) return 1;
    if (cin % 16 == 0 && m % 32 == 0) return 2;
    return -1;
}

uint16_t f32_to_bf16_rne(float v)
{
    uint32_t u;
    __builtin_memcpy(&u, &v, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

uint16_t f32_to_f16_rne(float v)
{
    uint32_t u;
    __builtin_memcpy(&u, &v, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);                       // NaN
    if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);                      // rounds to >= 2^16: infinity
    if (a < 0x33000001u) return sign;                                             // <= 2^-25: rounds to zero
    if (a < 0x38800000u) {                                                        // subnormal half: units of 2^-24
        const int shift = 126 - (int)(a >> 23);                                   // 14 .. 24
        const uint32_t m = (a & 0x7fffffu) | 0x800000u;
        const uint32_t q = m >> shift, rem = m & ((1u << shift) - 1u), halfway = 1u << (shift - 1);
        return (uint16_t)(sign | (q + ((rem > halfway || (rem == halfway && (q & 1u))) ? 1u : 0u)));
    }
    const uint32_t r = a + 0xfffu + ((a >> 13) & 1u);                             // normal: round the 13 dropped bits
    return (uint16_t)(sign | ((r - 0x38000000u) >> 13));
}

// Packed layout: [M/MT][chunk][tap] blocks of MT x KC bf16 (row-major), the order the kernel walks them.
size_t packed_bf16_count(int cin, int cout, int ntaps, int stride, int variant)
{
    (void)variant;
    const size_t M = stride > 0 ? (size_t)stride * cout : (size_t)cout;
    return M * (size_t)ntaps * cin;
}

// GEMM row held by row slot r of a packed block: within each block of 64 slots (the rows of one wave), slot
// mi * 32 + j is row 2 j + mi (see "orientation of the accumulators"); identity for the tiles with 32 rows per wave
// and for the layouts read by the fused units.
static inline int slot_to_row(int r, bool permute)
{
    if (!permute) return r;
    const int blk = r / 64, sl = r % 64;
    return blk * 64 + (sl % 32) * 2 + sl / 32;
}

void pack_bf16(const float* w, int cin, int cout, int ntaps, int stride, int variant, bool as_half, bool permute_rows,
               uint16_t* dst, int down)
{
    const Variant v = kVariants[variant];
    const bool perm = permute_rows && v.MT % 64 == 0;
    const int M = stride > 0 ? stride * cout : cout;
    // strided conv (down = s): merged channel rho cin + i of merged tap u is W[o, i, u s/2 + rho]
    const int merge = down > 0 ? down / 2 : 1;
    const int kcin = cin * merge, ktaps = down > 0 ? 4 : ntaps;
    const int nch = kcin / v.KC;
    size_t pos = 0;
    for (int mt = 0; mt < M / v.MT; ++mt)
        for (int c = 0; c < nch; ++c)
            for (int t = 0; t < ktaps; ++t)
                for (int i = 0; i < v.MT; ++i)
                    for (int e = 0; e < v.KC; ++e) {
                        const int mu = mt * v.MT + slot_to_row(i, perm), ci = c * v.KC + e;
                        float val;
                        if (down > 0) {
                            const int rho = ci / cin, ii = ci - rho * cin;
                            val = w[((size_t)mu * cin + ii) * (2 * down) + t * merge + rho];
                        } else if (stride == 0) {
                            val = w[((size_t)mu * cin + ci) * ntaps + t];
                        } else {
                            const int phi = mu / cout, o = mu - phi * cout;
                            val = w[((size_t)ci * cout + o) * (2 * stride) + phi + t * stride];
                        }
                        // bf16 values in either case: the half form of the rounded value (exact unless tiny)
                        const uint16_t b = f32_to_bf16_rne(val);
                        if (as_half) {
                            const uint32_t bits = (uint32_t)b << 16;
                            float bv;
                            __builtin_memcpy(&bv, &bits, 4);
                            dst[pos++] = f32_to_f16_rne(bv);
                        } else {
                            dst[pos++] = b;
                        }
                    }
}

template <int MT, int NT, int KC, int WM, int WN, int MODE, int IN, int EMIT>
__global__ __launch_bounds__(64 * WM * WN) void conv_mfma_kernel(MfmaParams p)
{
    fp16_saturate_on();
    constexpr int NTH = 64 * WM * WN;           // threads per workgroup
    constexpr int LDK = KC + 8;                 // padded LDS row (bf16 elements): 16-byte multiple, bank-spread
    // rows of the activation tile: the dilated conv reaches MAXSPAN rows past its NT columns, the 1x1 conv
    // none and the transposed conv one; a smaller tile lets more workgroups share a CU
    constexpr int XS = (MODE == MODE_DOWN) ? 2 : 1;        // input rows per GEMM column
    constexpr int XR_MAX = XS * NT + (MODE == MODE_ACT ? MAXSPAN : 8);
    constexpr int WTM = MT / WM, WTN = NT / WN; // tile of one wave
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int SEGS = KC / 8;                // 16-byte segments per row
    constexpr int RPP = NTH / SEGS;             // rows staged per pass
    constexpr int A_CH = MT * SEGS;             // 16-byte chunks of an A block
    constexpr int A_ITERS = (A_CH + NTH - 1) / NTH;
    constexpr int X_ITERS = (XR_MAX + RPP - 1) / RPP;
    constexpr bool SPLIT_IN = IN == OP_BF16X2;
    constexpr int NP = SPLIT_IN ? 2 : 1;        // operand planes (hi, lo)
    static_assert(WM * WN == 2 || WM * WN == 4 || WM * WN == 8, "two, four or eight waves per workgroup");
    static_assert(TM == 1 || TM == 2 || TM == 4, "a lane owns one channel, or one or two pairs of consecutive channels");
    // A wave's 32-row slot tiles come in pairs (the packed order: slot j of tile 2b + k of a wave is GEMM row 64 b + 2 j + k
    // of the wave's rows): a lane owns the channel pairs mu0 + 64 b + {0, 1}.
    constexpr int PW = TM >= 2 ? 2 : 1;         // channels per pair
    constexpr int PR = TM / PW;                 // pairs per lane
    static_assert(MODE != MODE_ACT || EMIT > 0, "the dilated conv only has the activated output");
    static_assert(MODE != MODE_DOWN || IN != OP_BF16X2, "the strided conv takes one operand plane");

    // Three workgroups per CU hide each other's barriers and load latencies markedly better than two (-10 to -28 % per
    // launch), and the 128 x 128 tile gets there with one weight buffer in LDS instead of two (46 KB with the dilated
    // conv's activation tile; the next blocks wait in registers and are stored between two barriers) and with the
    // residual values requested after the K loop instead of before it.
    constexpr int NBUF = (MT == 128) ? 1 : 2;
    constexpr bool LATE_RES = MT == 128;
    constexpr bool PF2 = MT == 64 && NT == 64;     // the small-grid tile: weight blocks requested several stages ahead
    constexpr int PFD = PF2 ? 4 : 1;               // weight blocks in flight: the block of stage t travels in register set t % PFD
    constexpr int AS_BYTES = NBUF * MT * LDK * 2, XS_BYTES = NP * XR_MAX * LDK * 2;
    constexpr int SMEM_BYTES = AS_BYTES + XS_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
    uint16_t (*As)[MT * LDK] = reinterpret_cast<uint16_t (*)[MT * LDK]>(smem);
    uint16_t (*Xs)[XR_MAX * LDK] = reinterpret_cast<uint16_t (*)[XR_MAX * LDK]>(smem + AS_BYTES);

    const Slot s = p.slots[blockIdx.y];
    const int nrows = s.len * p.r_in;                       // valid input rows of this window
    // output rows that later layers read: the interior widened by `margin`, clamped to the window
    const int r_out = (MODE == MODE_UP) ? p.r_in * p.stride : (MODE == MODE_DOWN) ? p.r_in / 2 : p.r_in;
    const int nrows_o = s.len * r_out;
    const int out_lo = max(0, s.crop * r_out - p.margin);
    const int out_hi = min(nrows_o, (s.crop + s.n_int) * r_out + p.margin);
    if (out_hi <= out_lo) return;                           // an empty window (a gated clip)
    // GEMM columns: output rows (conv) or input positions m whose s outputs m s - p .. m s - p + s - 1 touch them
    const int col_lo = (MODE == MODE_UP) ? (out_lo + p.stride / 2) / p.stride : out_lo;
    const int ncols = (MODE == MODE_UP) ? (out_hi - 1 + p.stride / 2) / p.stride + 1 : out_hi;
    // Workgroups are dealt to the 8 XCDs round-robin by linear id, and each XCD has its own L2.  All row tiles
    // of a column tile read the same activation rows, so they get ids that are equal mod 8 and adjacent in
    // dispatch order: id = 8 * ((column tile / 8) * mtiles + row tile) + column tile % 8.
    // (With xcd_group = 0 the id is column tile * mtiles + row tile: XCD x then only ever touches the row tiles
    // = x mod 8, one eighth of a weight matrix too large for one L2, and reads every activation row once.)
    int mtile = (int)blockIdx.z, ntile = (int)blockIdx.x;
    if (p.mtiles_x > 0 && p.xcd_group) {
        const unsigned q = blockIdx.x >> 3;
        mtile = (int)(q % (unsigned)p.mtiles_x);
        // ... rotated by the window index, so that windows with fewer than 8 column tiles still use all XCDs
        ntile = (int)(q / (unsigned)p.mtiles_x) * 8 + (int)((blockIdx.x - blockIdx.y) & 7u);
    } else if (p.mtiles_x > 0) {
        mtile = (int)(blockIdx.x % (unsigned)p.mtiles_x);
        ntile = (int)(blockIdx.x / (unsigned)p.mtiles_x);
    }
    const int n0 = col_lo + ntile * NT;
    if (n0 >= ncols) return;
    const int m0 = mtile * MT;
    const long long rowbase = (long long)s.row0 * p.r_in;
    const long long rowbase_o = (long long)s.row0 * r_out;

    const int last_off = p.tap0 + (p.ntaps - 1) * p.tap_step;
    const int minoff = min(p.tap0, last_off);
    const int XR = XS * (NT - 1) + 1 + max(p.tap0, last_off) - minoff;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS, xr0 = tid / SEGS;

    // ---- descriptors (uniform)
    const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(p.w, p.w_bytes);
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.xa + rowbase * p.cin, (unsigned)nrows * p.cin * 2u);
    const __amdgpu_buffer_rsrc_t rs_xl = make_rsrc(p.xa + p.in_lo_off + rowbase * p.cin, SPLIT_IN ? (unsigned)nrows * p.cin * 2u : 0u);

    const int nstages = p.nchunks * p.ntaps;
    // a row tile's blocks are nstages apart in the packed order; with blocks packed for a tile of pack_ratio * MT rows
    // this tile is a contiguous slice of every such block
    const unsigned w_blk = (unsigned)p.pack_ratio * (A_CH * 16u);
    const unsigned w_tile0 = (unsigned)(mtile / p.pack_ratio) * nstages * w_blk + (unsigned)(mtile % p.pack_ratio) * (A_CH * 16u);
    const unsigned a_voff = tid * 16u;
    const unsigned x_voff = ((unsigned)((XS * n0 + minoff + xr0) * p.cin) + seg * 8u) * 2u;    // may wrap "negative": out of range
    const unsigned x_row_step = (unsigned)(RPP * p.cin) * 2u;

    u32x4 rs[PFD][A_ITERS];
    u32x4 (&ra)[A_ITERS] = rs[0];
    u32x4 rx[X_ITERS][NP];

    auto load_a_to = [&](u32x4 (&r)[A_ITERS], int stage) __attribute__((always_inline)) {
        const unsigned base = w_tile0 + (unsigned)stage * w_blk;
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
            if (A_CH % NTH == 0 || tid + it * NTH < A_CH)
                r[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, a_voff, base + it * (NTH * 16u), 0);
    };
    auto store_a_from = [&](const u32x4 (&r)[A_ITERS], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) {
            const int q = tid + it * NTH;
            if (A_CH % NTH == 0 || q < A_CH)
                *reinterpret_cast<u32x4*>(&As[buf][(q / SEGS) * LDK + (q % SEGS) * 8]) = r[it];
        }
    };
    auto load_a = [&](int stage) __attribute__((always_inline)) { load_a_to(ra, stage); };
    auto store_a = [&](int buf) __attribute__((always_inline)) { store_a_from(ra, buf); };
    auto load_x = [&](int chunk) __attribute__((always_inline)) {
        const unsigned coff = x_voff + (unsigned)(chunk * KC) * 2u;
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                        // uniform
            const unsigned off = coff + it * x_row_step;
            rx[it][0] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, off, 0, 0);
            if (SPLIT_IN) rx[it][NP - 1] = __builtin_amdgcn_raw_buffer_load_b128(rs_xl, off, 0, 0);
        }
    };
    auto store_x = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                        // uniform
            const int xr = xr0 + it * RPP;
            if (xr >= XR_MAX) continue;
            *reinterpret_cast<u32x4*>(&Xs[0][xr * LDK + seg * 8]) = rx[it][0];
            if (SPLIT_IN) *reinterpret_cast<u32x4*>(&Xs[NP - 1][xr * LDK + seg * 8]) = rx[it][NP - 1];
        }
    };

    // this lane's GEMM rows: accumulator tile mi holds row mu0 + 64 (mi / 2) + mi % 2; the accumulators start at their bias
    const int mu0 = m0 + wm * WTM + j * PW;
    auto chan = [&](int mi) -> int {            // output channel of accumulator tile mi
        const int mu = mu0 + (mi >> 1) * 64 + (mi & 1);
        return (MODE == MODE_UP) ? mu % p.cout : mu;
    };
    f32x16 acc[TM][TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
        const float bv = p.bias[chan(mi)];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[mi][ni][q] = bv;
    }

    // Element index (in the window) of this lane's channels at time row gq = 4g + q of time tile ni.  Conv: (col, mu0);
    // transposed conv: column m, row mu = phi*cout + o lands on sample m s - p + phi, i.e. on the run starting at
    // (m s - p) cout + mu.  A negative row wraps to a huge offset = out of range.
    // (one per-lane product; the offsets of the 16 x TN time rows are uniform multiples of the row length)
    const int s_up = p.stride, p_up = p.stride / 2;
    const int lane_col = n0 + wn * WTN + 4 * h;
    const unsigned e_lane = (MODE == MODE_UP) ? (unsigned)((lane_col * s_up - p_up) * p.cout + mu0) : (unsigned)(lane_col * p.cout + mu0);
    const unsigned col_elems = (MODE == MODE_UP) ? (unsigned)(s_up * p.cout) : (unsigned)p.cout;
    auto elem = [&](int ni, int gq) -> unsigned {
        return e_lane + (unsigned)(ni * 32 + 8 * (gq >> 2) + (gq & 3)) * col_elems;
    };
    const unsigned out_rows = (unsigned)out_hi;
    const __amdgpu_buffer_rsrc_t rs_y = make_rsrc(MODE == MODE_ACT ? nullptr : p.y + rowbase_o * p.cout,
                                                  MODE == MODE_ACT ? 0u : out_rows * p.cout * (unsigned)sizeof(hres_t));
    // The residual values this lane will add are requested in one go, before the K loop or (LATE_RES) right after it:
    // issued in the epilogue where they are used, each of the loads would be waited for in turn (they cannot move
    // above the in-place stores), a chain of memory latencies per tile.
    using pack_t = std::conditional_t<PW == 2, uint32_t, uint16_t>;     // PW 16-bit values
    pack_t resv[MODE == MODE_RES ? PR : 1][MODE == MODE_RES ? TN : 1][16];
    auto load_res = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int pr = 0; pr < PR; ++pr)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int gq = 0; gq < 16; ++gq) {
                    const unsigned off = (elem(ni, gq) + 64u * pr) * 2u;
                    if constexpr (PW == 2) resv[pr][ni][gq] = __builtin_amdgcn_raw_buffer_load_b32(rs_y, off, 0, 0);
                    else resv[pr][ni][gq] = __builtin_amdgcn_raw_buffer_load_b16(rs_y, off, 0, 0);
                }
    };
    if (MODE == MODE_RES && !LATE_RES) load_res();

    load_a(0);
    load_x(0);
    store_a(0);
#pragma unroll
    for (int t = 1; t < PFD; ++t) load_a_to(rs[t], t);             // past the last stage: out of range, nothing is read
    store_x();
    __syncthreads();

    int chunk = 0, tap = 0;
    auto mma = [&](int stage) __attribute__((always_inline)) {
        __builtin_amdgcn_s_setprio(1);
        const int off = p.tap0 + tap * p.tap_step - minoff;
        const uint16_t* abase = &As[NBUF == 2 ? (stage & 1) : 0][(wm * WTM + j) * LDK + h * 8];
        const int xoff = ((wn * WTN + j) * XS + off) * LDK + h * 8;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            u32x4 af[TM], bfr[NP][TN];
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const u32x4*>(abase + mi * 32 * LDK + ks * 16);
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    bfr[pl][ni] = *reinterpret_cast<const u32x4*>(&Xs[pl][xoff + ni * 32 * XS * LDK + ks * 16]);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                    for (int pl = 0; pl < NP; ++pl) {
                        // activations are the row operand: the accumulator tile is [time][row slot]
                        if (IN == OP_F16)
                            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, bfr[pl][ni]), __builtin_bit_cast(f16x8, af[mi]), acc[mi][ni], 0, 0, 0);
                        else
                            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfr[pl][ni]), __builtin_bit_cast(bf16x8, af[mi]), acc[mi][ni], 0, 0, 0);
                    }
        }
        // Order of the stage's fragment reads and MFMAs: one k-step's reads plus two ahead, then one read per MFMA, so that a
        // fragment is requested a few MFMAs before it is used instead of right before the MFMAs of its own k-step.
        constexpr int R = (KC / 16) * (TM + NP * TN), M = (KC / 16) * TM * TN * NP;
        constexpr int LEAD = (TM + NP * TN + 2) < R ? (TM + NP * TN + 2) : R;
        constexpr int PAIRS = (R - LEAD) < M ? (R - LEAD) : M;
        __builtin_amdgcn_sched_group_barrier(0x100, LEAD, 0);
#pragma unroll
        for (int i = 0; i < PAIRS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, M - PAIRS, 0);
        __builtin_amdgcn_s_setprio(0);
    };
    // The weight block of stage s + PFD is requested before stage s is computed, into the register set whose block
    // (stage s) went to LDS a stage ago.  U = s % PFD is a compile-time constant (the loop is unrolled by PFD), so the sets
    // stay in registers.  One block in flight is enough where three workgroups share the CU and cover each other's loads
    // (two blocks: the same step time, 16 more registers); launches with few workgroups (the small-grid tile: one wave per
    // SIMD, nothing else to hide a load behind) keep four in flight (-3.5 % on a 3 s playback window).  The request is
    // unconditional -- past the last stage its offset is outside the descriptor and nothing is read -- because behind a
    // branch the compiler cannot count it, and every wait for an older block would then wait for all loads.
    auto body = [&](int stage, auto U) __attribute__((always_inline)) {
        constexpr int u = decltype(U)::value;
        int ntap = tap + 1, nchunk = chunk;
        if (ntap == p.ntaps) { ntap = 0; ++nchunk; }
        const bool more = stage + 1 < nstages;
        const bool new_chunk = more && nchunk != chunk;
        load_a_to(rs[u], stage + PFD);
        if (new_chunk) load_x(nchunk);
        mma(stage);
        if (more) {
            if (new_chunk || NBUF == 1) {
                __syncthreads();              // every wave is done with the old X tile (and the single weight buffer)
                if (new_chunk) store_x();
            }
            store_a_from(rs[(u + 1) % PFD], NBUF == 2 ? ((stage + 1) & 1) : 0);
            __syncthreads();
        }
        tap = ntap; chunk = nchunk;
    };
    for (int stage = 0; stage < nstages; stage += PFD) {
        body(stage, std::integral_constant<int, 0>{});
        if constexpr (PFD == 4) {
            if (stage + 1 < nstages) body(stage + 1, std::integral_constant<int, 1 % PFD>{});
            if (stage + 2 < nstages) body(stage + 2, std::integral_constant<int, 2 % PFD>{});
            if (stage + 3 < nstages) body(stage + 3, std::integral_constant<int, 3 % PFD>{});
        }
    }
    static_assert(PFD == 1 || PFD == 4, "the stage loop is unrolled by hand");

    if (MODE == MODE_RES && LATE_RES) load_res();

    // ---- epilogue, straight from the accumulators: register gq of tile (mi, ni) is time row 8g + 4h + q of time tile
    // ni and GEMM row mu0 + mi.  Rows past out_hi (and, for the transposed conv, before row 0) are out of range of the
    // descriptors and dropped.
    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(p.ya + rowbase_o * p.cout, EMIT > 0 ? out_rows * p.cout * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rs_al = make_rsrc(p.ya + p.out_lo_off + rowbase_o * p.cout, EMIT == 2 ? out_rows * p.cout * 2u : 0u);
    float oa[TM], ob[TM];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
        oa[mi] = EMIT > 0 ? p.out_alpha[chan(mi)] : 0.f;
        ob[mi] = EMIT > 0 ? p.out_inv_beta[chan(mi)] : 0.f;
    }
#pragma unroll
    for (int pr = 0; pr < PR; ++pr)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int gq = 0; gq < 16; ++gq) {
            const unsigned e = elem(ni, gq) + 64u * pr;
            float v[PW];
#pragma unroll
            for (int k = 0; k < PW; ++k) v[k] = acc[PW * pr + k][ni][gq];
            if (MODE == MODE_RES) {
#pragma unroll
                for (int k = 0; k < PW; ++k)
                    v[k] += (float)__builtin_bit_cast(_Float16, (uint16_t)(resv[pr][ni][gq] >> (16 * k)));
            }
            if (MODE != MODE_ACT) {
                // half store of h; the next layer's operand is Snake of the STORED value
                if constexpr (PW == 2) {
                    const uint32_t hb = pack_f16x2(v[0], v[1]);           // round to nearest even
                    __builtin_amdgcn_raw_buffer_store_b32(hb, rs_y, e * 2u, 0, 0);
                    const f16x2 hv = __builtin_bit_cast(f16x2, hb);
                    v[0] = (float)hv[0]; v[1] = (float)hv[1];
                } else {
                    const _Float16 hv = (_Float16)v[0];
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(uint16_t, hv), rs_y, e * 2u, 0, 0);
                    v[0] = (float)hv;
                }
            }
            if (EMIT > 0) {
                float a[PW];
#pragma unroll
                for (int k = 0; k < PW; ++k) {
                    a[k] = snake_fast(v[k], oa[PW * pr + k], ob[PW * pr + k]);
                    if (EMIT == 3) a[k] = keep_f32(a[k]);                 // fp32 Snake, then one rounding
                }
                if constexpr (PW == 2) {
                    const uint32_t ab = EMIT == 3 ? pack_f16x2(a[0], a[1]) : pack_bf16x2(a[0], a[1]);
                    __builtin_amdgcn_raw_buffer_store_b32(ab, rs_a, e * 2u, 0, 0);
                    if (EMIT == 2)                                         // lo plane: what the hi plane's rounding left over
                        __builtin_amdgcn_raw_buffer_store_b32(pack_bf16x2(a[0] - __uint_as_float(ab << 16), a[1] - __uint_as_float(ab & 0xffff0000u)),
                                                              rs_al, e * 2u, 0, 0);
                } else {
                    const uint16_t ab = EMIT == 3 ? __builtin_bit_cast(uint16_t, (_Float16)a[0]) : f32_to_bf16_bits(a[0]);
                    __builtin_amdgcn_raw_buffer_store_b16(ab, rs_a, e * 2u, 0, 0);
                    if (EMIT == 2)
                        __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_bits(a[0] - bf16_bits_to_f32(ab)), rs_al, e * 2u, 0, 0);
                }
            }
        }
}

template <int MT, int NT, int KC, int WM, int WN>
static hipError_t launch_variant(const MfmaParams& p, int mode, int in_fmt, int emit, dim3 grid, hipStream_t stream)
{
    // input format x emitted format: the pairs the layer sequence can ask for.  A layer with hi + lo input never emits
    // half and one with half input never emits hi + lo (a stack uses one of the two for its wide levels); a transposed
    // conv with plain bf16 input emits either when no residual unit sits between it and a wide block.
#define DEMON_LAUNCH(MODE_, IN_, EM_) \
    hipLaunchKernelGGL((conv_mfma_kernel<MT, NT, KC, WM, WN, MODE_, IN_, EM_>), grid, dim3(64 * WM * WN), 0, stream, p)
#define DEMON_CASE(MODE_, IN_, EM_) if (in_fmt == IN_ && emit == EM_) { DEMON_LAUNCH(MODE_, IN_, EM_); return hipGetLastError(); }
    if (mode == MODE_ACT) {
        DEMON_CASE(MODE_ACT, OP_BF16, 1) DEMON_CASE(MODE_ACT, OP_BF16, 2) DEMON_CASE(MODE_ACT, OP_F16, 3)
    } else if constexpr (MT == 128 && NT == 256) {
        if (mode != MODE_UP) return hipErrorInvalidValue;         // the 128 x 256 tile runs dilated and transposed convs
        DEMON_CASE(MODE_UP, OP_BF16, 0) DEMON_CASE(MODE_UP, OP_BF16, 1) DEMON_CASE(MODE_UP, OP_BF16, 2) DEMON_CASE(MODE_UP, OP_BF16, 3)
        DEMON_CASE(MODE_UP, OP_F16, 1) DEMON_CASE(MODE_UP, OP_F16, 3)
    } else if (mode == MODE_RES) {
        DEMON_CASE(MODE_RES, OP_BF16, 0) DEMON_CASE(MODE_RES, OP_BF16, 1) DEMON_CASE(MODE_RES, OP_BF16, 2) DEMON_CASE(MODE_RES, OP_BF16, 3)
        DEMON_CASE(MODE_RES, OP_BF16X2, 0) DEMON_CASE(MODE_RES, OP_BF16X2, 1) DEMON_CASE(MODE_RES, OP_BF16X2, 2)
        DEMON_CASE(MODE_RES, OP_F16, 0) DEMON_CASE(MODE_RES, OP_F16, 1) DEMON_CASE(MODE_RES, OP_F16, 3)
    } else if (mode == MODE_DOWN) {
        if constexpr (NT <= 128) {       // its activation tile holds two input rows per column
            DEMON_CASE(MODE_DOWN, OP_BF16, 0) DEMON_CASE(MODE_DOWN, OP_BF16, 1) DEMON_CASE(MODE_DOWN, OP_BF16, 3)
            DEMON_CASE(MODE_DOWN, OP_F16, 0) DEMON_CASE(MODE_DOWN, OP_F16, 1) DEMON_CASE(MODE_DOWN, OP_F16, 3)
        }
    } else {
        DEMON_CASE(MODE_UP, OP_BF16, 0) DEMON_CASE(MODE_UP, OP_BF16, 1) DEMON_CASE(MODE_UP, OP_BF16, 2) DEMON_CASE(MODE_UP, OP_BF16, 3)
        DEMON_CASE(MODE_UP, OP_BF16X2, 1) DEMON_CASE(MODE_UP, OP_BF16X2, 2)
        DEMON_CASE(MODE_UP, OP_F16, 1) DEMON_CASE(MODE_UP, OP_F16, 3)
    }
#undef DEMON_CASE
#undef DEMON_LAUNCH
    return hipErrorInvalidValue;
}

// Launches of the 128 x 128 tile that would leave most CUs without a workgroup (one playback window at the wide, low-rate
// levels) use a 64 x 64 tile on the same packed weights instead: four times the workgroups, and the same K order, so
// the results are bit-identical to the large tile's.  ConvArgs::small_tile_wgs is the threshold (0: never).
hipError_t launch_conv_bf16(const ConvArgs& a, int variant, hipStream_t stream)
{
    if (variant < 0 || variant > 2) return hipErrorInvalidValue;
    Variant v = kVariants[variant];
    const int M = a.stride > 0 ? a.stride * a.cout : a.cout;
    // strided conv: the kernel sees merged input rows of (s/2) cin channels, four taps, two rows per column
    const int merge = a.down > 0 ? a.down / 2 : 1;
    if (a.down > 0 && (a.down % 2 != 0 || a.stride != 0 || a.ntaps != 2 * a.down || a.r_in % a.down != 0 || a.res)) return hipErrorInvalidValue;
    const int cin = a.cin * merge, r_in = a.r_in / merge, ntaps = a.down > 0 ? 4 : a.ntaps;
    MfmaParams p;
    p.xa = (const uint16_t*)a.x; p.w = (const uint16_t*)a.w; p.bias = a.bias;
    p.y = (hres_t*)a.y; p.ya = (uint16_t*)a.ya;
    p.out_alpha = a.out_alpha; p.out_inv_beta = a.out_inv_beta;
    p.slots = a.slots;
    p.r_in = r_in; p.cin = cin; p.cout = a.cout; p.ntaps = ntaps; p.stride = a.stride;
    p.nchunks = cin / v.KC; p.margin = a.margin;
    p.in_lo_off = a.in_lo_off; p.out_lo_off = a.out_lo_off;
    const size_t wb = (size_t)M * ntaps * cin * 2;
    if (wb > 0xffffffffull) return hipErrorInvalidValue;
    p.w_bytes = (unsigned)wb;
    int mode;
    if (a.down > 0) { p.tap0 = -1; p.tap_step = 1; mode = MODE_DOWN; }
    else if (a.stride > 0) { p.tap0 = 0; p.tap_step = -1; mode = MODE_UP; }
    else { p.tap0 = -((a.ntaps - 1) / 2) * a.dil; p.tap_step = a.dil; mode = a.res ? MODE_RES : MODE_ACT; }
    if (a.in_fmt < OP_BF16 || a.in_fmt > OP_F16 || a.out_fmt < OP_BF16 || a.out_fmt > OP_F16) return hipErrorInvalidValue;
    const int emit = a.ya ? a.out_fmt + 1 : 0;
    const int span = (ntaps - 1) * ((a.stride > 0 || a.down > 0) ? 1 : a.dil);
    // shape checks: everything the kernel's indexing assumes
    if (span > (mode == MODE_ACT ? MAXSPAN : 8) || M % v.MT != 0 || cin % v.KC != 0 || a.cout % 4 != 0 || a.margin < 0) return hipErrorInvalidValue;
    if (mode == MODE_ACT && emit == 0) return hipErrorInvalidValue;
    if (emit > 0 && (!a.out_alpha || !a.out_inv_beta)) return hipErrorInvalidValue;
    if (mode != MODE_ACT && !a.y) return hipErrorInvalidValue;
    if (mode == MODE_RES && a.res != a.y) return hipErrorInvalidValue;            // the residual add is in place
    // one window's activation plane must fit a 32-bit byte offset (buffer descriptors)
    const long long r_out = a.down > 0 ? (long long)a.r_in / a.down : (long long)a.r_in * (a.stride > 0 ? a.stride : 1);
    const long long max_in_bytes = (long long)a.max_len * a.r_in * a.cin * 2;
    const long long max_out_bytes = (long long)a.max_len * r_out * a.cout * (long long)sizeof(hres_t);
    if (max_in_bytes > 0xf0000000ll || max_out_bytes > 0xf0000000ll) return hipErrorInvalidValue;
    // most columns any window needs: interior plus margins, never more than the longest window
    long long out_rows = std::min((long long)a.max_int * r_out + 2ll * a.margin, (long long)a.max_len * r_out);
    const long long ncols = a.stride > 0 ? out_rows / a.stride + 2 : out_rows;
    // Grid order (L2 miss traffic; X = activation bytes, W = weight bytes, 8 XCDs with 4 MB of L2 each).
    //  * W fits one L2: the row tiles of a column tile go to the same XCD, adjacent in dispatch order; they share
    //    its activation rows in that L2 and the weights stay resident: about X + 8 W.
    //  * W larger, more than 8 row tiles: ids run over row tiles first, so XCD x owns the row tiles = x mod 8 (an
    //    eighth of W, resident) and reads all activations: about 8 X + W.
    //  * else column tiles fastest (blockIdx.x): workgroups in flight share one row tile of the weights: mtiles X + W.
    p.pack_ratio = 1;
    bool small_tile = false;
    if (variant == 0 && ((ncols + v.NT - 1) / v.NT) * (M / v.MT) * a.n_slots <= a.small_tile_wgs) {
        small_tile = true;
        v.MT = 64; v.NT = 64; p.pack_ratio = 2;
    }
    // Dilated convs with enough columns run a 128 x 256 tile on the same packed weights (four waves side by side, every
    // wave all 128 rows of its 64 columns: 0.75 instead of 1 fragment read per MFMA, half the weight staging per column, two
    // workgroups per CU): -7 % on the 512-channel dilated convs.  Only when the launch still has 768 such workgroups (three per CU):
    // with fewer the larger tile's last round costs more than the tile saves (+5 % on the 1024-channel level of a 60 s clip).
    // Same K order, so the results are bit-identical to the 128 x 128 tile's.
    // Transposed convs too where the weight matrix is small (at most four row tiles: -8 ... -12 % at 128 and 256 input
    // channels; with more row tiles the square tile is as fast or faster).
    const bool wide_n = a.wide_tile_ok && variant == 0 && !small_tile && a.in_fmt != OP_BF16X2 &&
                        (mode == MODE_ACT || (mode == MODE_UP && M / v.MT <= 4)) &&
                        ((ncols + 255) / 256) * (M / v.MT) * a.n_slots >= 768;
    if (wide_n) v.NT = 256;
    const long long ntiles = (ncols + v.NT - 1) / v.NT;
    const int mtiles = M / v.MT;
    const long long ntiles8 = (ntiles + 7) / 8 * 8;           // whole groups of 8 column tiles; the surplus exits at once
    const bool w_fits_l2 = wb <= (4u << 20);
    const bool m_fastest = mtiles > 1 && ntiles8 * mtiles < 0x7fffffffll && (w_fits_l2 || mtiles > 8);
    p.mtiles_x = m_fastest ? mtiles : 0;
    p.xcd_group = w_fits_l2 ? 1 : 0;
    dim3 grid(m_fastest ? (unsigned)(ntiles8 * mtiles) : (unsigned)ntiles, (unsigned)a.n_slots, m_fastest ? 1u : (unsigned)mtiles);
    switch (variant) {
        case 0: if (wide_n) return launch_variant<128, 256, 64, 1, 4>(p, mode, a.in_fmt, emit, grid, stream);
                return small_tile ? launch_variant<64, 64, 64, 1, 2>(p, mode, a.in_fmt, emit, grid, stream)
                                  : launch_variant<128, 128, 64, 2, 2>(p, mode, a.in_fmt, emit, grid, stream);
        case 1: return launch_variant<64, 256, 64, 1, 4>(p, mode, a.in_fmt, emit, grid, stream);
        default: return launch_variant<32, 128, 16, 1, 4>(p, mode, a.in_fmt, emit, grid, stream);
    }
}

}  // namespace demon
