// bf16 MFMA implicit-GEMM convolution kernels for gfx950 (CDNA4).
//
// Every convolution of the decoder is one GEMM  D[mu, n] = sum_{t, i} A[mu, (t, i)] * X[n + off_t, i]:
//   Conv1d(k, dilation d):            mu = output channel, off_t = (t - (k-1)/2) d
//   ConvTranspose1d(2s, s, p = s/2):  polyphase form, mu = phi*cout + o, column n = input position m in [0, L],
//                                     taps j in {0,1} with off_j = -j and weight W[i, o, phi + j s];
//                                     column m, row mu lands on output sample m s - p + phi, channel o,
//                                     i.e. on the contiguous run ((m s - p) cout + mu) of the time-major output.
// Activations are time-major [rows, channels] bf16, so the 8 consecutive K values an MFMA lane needs
// are 16 contiguous bytes and a tap is a row offset into the same LDS tile (staged once per channel
// chunk, halo rows included, Snake applied while staging, rows outside the window read as zero).
// Accumulation is fp32 in a fixed order (chunk-major, then tap, then channel), independent of where
// the tile sits in the window, so a windowed decode reproduces the full decode bit for bit.
#include <algorithm>

#include "device_common.h"

namespace demon {

constexpr int MAXSPAN = 64;    // largest (max tap offset - min tap offset) the LDS tile is sized for

// The residual stream h is kept in fp32 in HBM (rounding it to bf16 after every layer alone would use
// up the error budget of the bf16 path); only MFMA operands are bf16: Snake(h) is rounded while it is
// staged into LDS, and the activated output of the dilated conv is stored as bf16.
// Split operands: where the rounding of an activation operand to bf16 costs too much accuracy (the
// wide, low-rate levels, whose branch gain is about one), the operand is carried as hi + lo with
// hi = bf16(v), lo = bf16(v - hi), and every k-step issues two MFMAs against the same weight
// fragment.  SPLIT_IN: the B operand is split (staged from fp32 by the kernel itself, or read as two
// bf16 planes in MODE_RES).  SPLIT_OUT (MODE_ACT): the activated output is stored as two planes.
enum { MODE_ACT = 0,   // fp32 in, Snake on input;  bias + Snake on output, bf16 out   (dilated conv of a residual unit)
       MODE_RES = 1,   // bf16 in (already activated); bias + fp32 residual add, fp32 out (1x1 conv of a residual unit)
       MODE_UP  = 2 }; // fp32 in, Snake on input;  bias, polyphase scatter, fp32 out  (ConvTranspose1d)

struct MfmaParams {
    const void* x; void* y; const float* res; const uint16_t* w;
    const float* bias;
    const float* in_alpha; const float* in_inv_beta;
    const float* out_alpha; const float* out_inv_beta;
    const Slot* slots;
    int r_in, cin, cout, ntaps, tap0, tap_step, stride, nchunks, margin;
    long long in_lo_off, out_lo_off;     // element offset of the lo plane of a split bf16 tensor
};

struct Variant { int MT, NT, KC; };
static const Variant kVariants[3] = {{128, 128, 64}, {64, 256, 64}, {32, 128, 16}};

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

// Packed layout: [M/MT][chunk][tap] blocks of MT x KC bf16 (row-major), the order the kernel walks them.
size_t packed_bf16_count(int cin, int cout, int ntaps, int stride, int variant)
{
    (void)variant;
    const size_t M = stride > 0 ? (size_t)stride * cout : (size_t)cout;
    return M * (size_t)ntaps * cin;
}

void pack_bf16(const float* w, int cin, int cout, int ntaps, int stride, int variant, uint16_t* dst)
{
    const Variant v = kVariants[variant];
    const int M = stride > 0 ? stride * cout : cout;
    const int nch = cin / v.KC;
    size_t pos = 0;
    for (int mt = 0; mt < M / v.MT; ++mt)
        for (int c = 0; c < nch; ++c)
            for (int t = 0; t < ntaps; ++t)
                for (int i = 0; i < v.MT; ++i)
                    for (int e = 0; e < v.KC; ++e) {
                        const int mu = mt * v.MT + i, ci = c * v.KC + e;
                        float val;
                        if (stride == 0) {
                            val = w[((size_t)mu * cin + ci) * ntaps + t];
                        } else {
                            const int phi = mu / cout, o = mu - phi * cout;
                            val = w[((size_t)ci * cout + o) * (2 * stride) + phi + t * stride];
                        }
                        dst[pos++] = f32_to_bf16_rne(val);
                    }
}

template <int MT, int NT, int KC, int WM, int WN, int MODE, bool SPLIT_IN, bool SPLIT_OUT>
__global__ __launch_bounds__(256) void conv_mfma_kernel(MfmaParams p)
{
    constexpr int LDK = KC + 8;                 // padded LDS row (bf16 elements): 16-byte multiple, bank-spread
    constexpr int XR_MAX = NT + MAXSPAN;
    constexpr int WTM = MT / WM, WTN = NT / WN; // tile of one wave
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int SEGS = KC / 8;                // 16-byte segments per row
    constexpr int RPP = 256 / SEGS;             // rows staged per pass
    constexpr int A_CH = MT * SEGS;             // 16-byte chunks of an A block
    constexpr int A_ITERS = (A_CH + 255) / 256;
    constexpr int X_ITERS = (XR_MAX + RPP - 1) / RPP;
    constexpr bool SNAKE_IN = (MODE != MODE_RES);     // these modes read the fp32 residual stream
    constexpr int XV = (SNAKE_IN || SPLIT_IN) ? 2 : 1; // 16-byte loads per staged 8-channel segment
    constexpr int NP = SPLIT_IN ? 2 : 1;              // operand planes (hi, lo)
    static_assert(WM * WN == 4, "four waves per workgroup");

    __shared__ __attribute__((aligned(16))) uint16_t As[2][MT * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Xs[NP][XR_MAX * LDK];

    const Slot s = p.slots[blockIdx.y];
    const int nrows = s.len * p.r_in;                       // valid input rows of this window
    // output rows that later layers read: the interior widened by `margin`, clamped to the window
    const int r_out = (MODE == MODE_UP) ? p.r_in * p.stride : p.r_in;
    const int nrows_o = s.len * r_out;
    const int out_lo = max(0, s.crop * r_out - p.margin);
    const int out_hi = min(nrows_o, (s.crop + s.n_int) * r_out + p.margin);
    // GEMM columns: output rows (conv) or input positions m whose s outputs m s - p .. m s - p + s - 1 touch them
    const int col_lo = (MODE == MODE_UP) ? (out_lo + p.stride / 2) / p.stride : out_lo;
    const int ncols = (MODE == MODE_UP) ? (out_hi - 1 + p.stride / 2) / p.stride + 1 : out_hi;
    const int n0 = col_lo + blockIdx.x * NT;
    if (n0 >= ncols) return;
    const int m0 = blockIdx.z * MT;
    const long long rowbase = (long long)s.row0 * p.r_in;

    const int last_off = p.tap0 + (p.ntaps - 1) * p.tap_step;
    const int minoff = min(p.tap0, last_off);
    const int XR = NT + max(p.tap0, last_off) - minoff;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS, xr0 = tid / SEGS;

    const int nstages = p.nchunks * p.ntaps;
    const u32x4* wblk = reinterpret_cast<const u32x4*>(p.w) + (size_t)blockIdx.z * nstages * (A_CH);

    u32x4 ra[A_ITERS];
    u32x4 rx[X_ITERS][XV];
    float al[8], ib[8];

    auto load_a = [&](int stage) __attribute__((always_inline)) {
        const u32x4* src = wblk + (size_t)stage * A_CH;
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) {
            const int q = tid + it * 256;
            if (A_CH % 256 == 0 || q < A_CH) ra[it] = src[q];
        }
    };
    auto store_a = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) {
            const int q = tid + it * 256;
            if (A_CH % 256 == 0 || q < A_CH)
                *reinterpret_cast<u32x4*>(&As[buf][(q / SEGS) * LDK + (q % SEGS) * 8]) = ra[it];
        }
    };
    auto load_x = [&](int chunk) __attribute__((always_inline)) {
        const int cbase = chunk * KC + seg * 8;
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            const int srow = n0 + minoff + xr;
            const bool ok = xr < XR && srow >= 0 && srow < nrows;
            const size_t e0 = (size_t)(rowbase + srow) * p.cin + cbase;
#pragma unroll
            for (int q = 0; q < XV; ++q) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = SNAKE_IN ? reinterpret_cast<const u32x4*>(static_cast<const float*>(p.x) + e0)[q]
                                     : *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.x) + e0 + (q ? p.in_lo_off : 0));
                rx[it][q] = v;
            }
        }
        if (SNAKE_IN) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { al[e] = p.in_alpha[cbase + e]; ib[e] = p.in_inv_beta[cbase + e]; }
        }
    };
    auto store_x = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            if (xr >= XR_MAX) continue;
            u32x4 v = rx[it][0], vlo = rx[it][XV - 1];
            if (SNAKE_IN) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float e0 = __uint_as_float(rx[it][q >> 1][(2 * q) & 3]), e1 = __uint_as_float(rx[it][q >> 1][(2 * q + 1) & 3]);
                    e0 = snake_fast(e0, al[2 * q], ib[2 * q]);
                    e1 = snake_fast(e1, al[2 * q + 1], ib[2 * q + 1]);
                    const uint32_t h0 = f32_to_bf16_bits(e0), h1 = f32_to_bf16_bits(e1);
                    v[q] = h0 | (h1 << 16);
                    if (SPLIT_IN) {
                        const float r0 = e0 - __uint_as_float(h0 << 16), r1 = e1 - __uint_as_float(h1 << 16);
                        vlo[q] = (uint32_t)f32_to_bf16_bits(r0) | ((uint32_t)f32_to_bf16_bits(r1) << 16);
                    }
                }
            }
            *reinterpret_cast<u32x4*>(&Xs[0][xr * LDK + seg * 8]) = v;
            if (SPLIT_IN) *reinterpret_cast<u32x4*>(&Xs[NP - 1][xr * LDK + seg * 8]) = vlo;
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

    int chunk = 0, tap = 0;
    for (int stage = 0; stage < nstages; ++stage) {
        int ntap = tap + 1, nchunk = chunk;
        if (ntap == p.ntaps) { ntap = 0; ++nchunk; }
        const bool more = stage + 1 < nstages;
        const bool new_chunk = more && nchunk != chunk;
        if (more) load_a(stage + 1);
        if (new_chunk) load_x(nchunk);

        const int off = p.tap0 + tap * p.tap_step - minoff;
        const uint16_t* abase = &As[stage & 1][(wm * WTM + j) * LDK + h * 8];
        const int xoff = (wn * WTN + j + off) * LDK + h * 8;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            bf16x8 af[TM], bfr[NP][TN];
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const bf16x8*>(abase + mi * 32 * LDK + ks * 16);
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    bfr[pl][ni] = *reinterpret_cast<const bf16x8*>(&Xs[pl][xoff + ni * 32 * LDK + ks * 16]);
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                    for (int pl = 0; pl < NP; ++pl)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[pl][ni], acc[mi][ni], 0, 0, 0);
        }

        if (more) {
            if (new_chunk) {
                __syncthreads();              // every wave is done with the old X tile
                store_x();
            }
            store_a((stage + 1) & 1);
            __syncthreads();
        }
        tap = ntap; chunk = nchunk;
    }

    // ---- epilogue: lane (j, h) of a 32x32 tile holds column j, rows 8g + 4h + {0..3}, g = 0..3 ----
    const int s_up = p.stride, p_up = p.stride / 2;
    const long long nrows_out = (long long)nrows * (MODE == MODE_UP ? s_up : 1);
    const long long rowbase_out = rowbase * (MODE == MODE_UP ? s_up : 1);
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int mu = m0 + wm * WTM + mi * 32 + 8 * g + 4 * h;
            int o = mu, phi = 0;
            if (MODE == MODE_UP) { phi = mu / p.cout; o = mu - phi * p.cout; }
            const float4 b4 = *reinterpret_cast<const float4*>(p.bias + o);
            float4 oa = make_float4(0, 0, 0, 0), ob = oa;
            if (MODE == MODE_ACT) {
                oa = *reinterpret_cast<const float4*>(p.out_alpha + o);
                ob = *reinterpret_cast<const float4*>(p.out_inv_beta + o);
            }
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
                const int col = n0 + wn * WTN + ni * 32 + j;
                if (col >= ncols) continue;
                float v0 = acc[mi][ni][4 * g + 0] + b4.x, v1 = acc[mi][ni][4 * g + 1] + b4.y;
                float v2 = acc[mi][ni][4 * g + 2] + b4.z, v3 = acc[mi][ni][4 * g + 3] + b4.w;
                long long n = col;
                if (MODE == MODE_UP) {
                    n = (long long)col * s_up - p_up + phi;
                    if (n < 0 || n >= nrows_out) continue;
                }
                const size_t idx = (size_t)(rowbase_out + n) * p.cout + o;
                if (MODE == MODE_ACT) {
                    v0 = snake_fast(v0, oa.x, ob.x); v1 = snake_fast(v1, oa.y, ob.y);
                    v2 = snake_fast(v2, oa.z, ob.z); v3 = snake_fast(v3, oa.w, ob.w);
                }
                if (MODE == MODE_RES) {
                    const float4 r = *reinterpret_cast<const float4*>(p.res + idx);
                    v0 += r.x; v1 += r.y; v2 += r.z; v3 += r.w;
                }
                if (MODE == MODE_ACT) {
                    const uint32_t h0 = f32_to_bf16_bits(v0), h1 = f32_to_bf16_bits(v1);
                    const uint32_t h2 = f32_to_bf16_bits(v2), h3 = f32_to_bf16_bits(v3);
                    uint2 st;
                    st.x = h0 | (h1 << 16);
                    st.y = h2 | (h3 << 16);
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.y) + idx) = st;
                    if (SPLIT_OUT) {
                        st.x = (uint32_t)f32_to_bf16_bits(v0 - __uint_as_float(h0 << 16)) |
                               ((uint32_t)f32_to_bf16_bits(v1 - __uint_as_float(h1 << 16)) << 16);
                        st.y = (uint32_t)f32_to_bf16_bits(v2 - __uint_as_float(h2 << 16)) |
                               ((uint32_t)f32_to_bf16_bits(v3 - __uint_as_float(h3 << 16)) << 16);
                        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.y) + p.out_lo_off + idx) = st;
                    }
                } else {
                    *reinterpret_cast<float4*>(static_cast<float*>(p.y) + idx) = make_float4(v0, v1, v2, v3);
                }
            }
        }
    }
}

template <int MT, int NT, int KC, int WM, int WN>
static hipError_t launch_variant(const MfmaParams& p, int mode, bool split_in, bool split_out, dim3 grid, hipStream_t stream)
{
#define DEMON_LAUNCH(MODE_, SI_, SO_) \
    hipLaunchKernelGGL((conv_mfma_kernel<MT, NT, KC, WM, WN, MODE_, SI_, SO_>), grid, dim3(256), 0, stream, p)
    if (mode == MODE_ACT) {
        if (split_in) { if (split_out) DEMON_LAUNCH(MODE_ACT, true, true); else DEMON_LAUNCH(MODE_ACT, true, false); }
        else          { if (split_out) DEMON_LAUNCH(MODE_ACT, false, true); else DEMON_LAUNCH(MODE_ACT, false, false); }
    } else if (mode == MODE_RES) {
        if (split_in) DEMON_LAUNCH(MODE_RES, true, false); else DEMON_LAUNCH(MODE_RES, false, false);
    } else {
        if (split_in) DEMON_LAUNCH(MODE_UP, true, false); else DEMON_LAUNCH(MODE_UP, false, false);
    }
#undef DEMON_LAUNCH
    return hipGetLastError();
}

hipError_t launch_conv_bf16(const ConvArgs& a, int variant, hipStream_t stream)
{
    if (variant < 0 || variant > 2) return hipErrorInvalidValue;
    const Variant v = kVariants[variant];
    const int M = a.stride > 0 ? a.stride * a.cout : a.cout;
    MfmaParams p;
    p.x = a.x; p.y = a.y; p.res = (const float*)a.res; p.w = (const uint16_t*)a.w;
    p.bias = a.bias;
    p.in_alpha = a.in_alpha; p.in_inv_beta = a.in_inv_beta;
    p.out_alpha = a.out_alpha; p.out_inv_beta = a.out_inv_beta;
    p.slots = a.slots;
    p.r_in = a.r_in; p.cin = a.cin; p.cout = a.cout; p.ntaps = a.ntaps; p.stride = a.stride;
    p.nchunks = a.cin / v.KC; p.margin = a.margin;
    p.in_lo_off = a.in_lo_off; p.out_lo_off = a.out_lo_off;
    int mode;
    if (a.stride > 0) { p.tap0 = 0; p.tap_step = -1; mode = MODE_UP; }
    else { p.tap0 = -((a.ntaps - 1) / 2) * a.dil; p.tap_step = a.dil; mode = a.res ? MODE_RES : MODE_ACT; }
    const int span = (a.ntaps - 1) * (a.stride > 0 ? 1 : a.dil);
    // shape checks: everything the kernel's indexing assumes
    if (span > MAXSPAN || M % v.MT != 0 || a.cin % v.KC != 0 || a.cout % 4 != 0) return hipErrorInvalidValue;
    if (mode == MODE_ACT && (!a.in_alpha || !a.out_alpha)) return hipErrorInvalidValue;
    if (mode == MODE_UP && !a.in_alpha) return hipErrorInvalidValue;
    if (a.split_out && mode != MODE_ACT) return hipErrorInvalidValue;
    if ((long long)a.max_len * a.r_in * (a.stride > 0 ? a.stride : 1) > 0x3fffffffll || a.margin < 0) return hipErrorInvalidValue;
    // most columns any window needs: interior plus margins, never more than the longest window
    const long long r_out = (long long)a.r_in * (a.stride > 0 ? a.stride : 1);
    long long out_rows = std::min((long long)a.max_int * r_out + 2ll * a.margin, (long long)a.max_len * r_out);
    const long long ncols = a.stride > 0 ? out_rows / a.stride + 2 : out_rows;
    dim3 grid((unsigned)((ncols + v.NT - 1) / v.NT), (unsigned)a.n_slots, (unsigned)(M / v.MT));
    switch (variant) {
        case 0: return launch_variant<128, 128, 64, 2, 2>(p, mode, a.split_in, a.split_out, grid, stream);
        case 1: return launch_variant<64, 256, 64, 1, 4>(p, mode, a.split_in, a.split_out, grid, stream);
        default: return launch_variant<32, 128, 16, 1, 4>(p, mode, a.split_in, a.split_out, grid, stream);
    }
}

}  // namespace demon
