// Window gather, output head, crop/stitch and the debug tap (HBM-bound kernels).
//
// gather : step 1 of the windowed decode of paper section 3.6 (extend each window by its margins):
//          copies latent frames [lo, hi) of every window into its slot, transposing to time-major.
// head   : Snake -> Conv1d(k, C -> out_channels) -> tanh, the last layer of the decoder.
// stitch : step 3 (trim the margins, keep the frame-aligned interior) plus the side-by-side write
//          of the interiors into the clip's waveform.
#include <algorithm>

#include "device_common.h"

namespace demon {

template <typename T> __device__ __forceinline__ float load_act(const T* p);
template <> __device__ __forceinline__ float load_act<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_act<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }
template <> __device__ __forceinline__ float load_act<_Float16>(const _Float16* p) { return (float)*p; }

// ---------------------------------------------------------------------------------- gather
// The latent is [clip, channel, frame] (frames fastest), the slots are time-major [frame, channel]: a workgroup moves a
// tile of 64 frames x 64 channels through LDS, reading runs of consecutive frames of one channel and writing runs of
// consecutive channels of one frame, so both sides are coalesced.  With `xa` (bf16 path) it writes the first layer's
// MFMA operand directly, snake(latent) in operand format fmt, instead of the fp32 copy.
constexpr int GATHER_TILE = 64;

template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(const T* __restrict__ latent, float* __restrict__ x0,
                                                     uint16_t* __restrict__ xa, int fmt, long long lo_off,
                                                     const float* __restrict__ alpha, const float* __restrict__ inv_beta,
                                                     int c0, int n_frames, const Slot* __restrict__ slots)
{
    fp16_saturate_on();
    __shared__ float tile[GATHER_TILE][GATHER_TILE + 1];
    const Slot s = slots[blockIdx.y];
    const int r0 = blockIdx.x * GATHER_TILE, cbase = blockIdx.z * GATHER_TILE;
    if (r0 >= s.len) return;
    const int lane = threadIdx.x % GATHER_TILE, sub = threadIdx.x / GATHER_TILE;      // 4 rows of 64 threads
    for (int cc = sub; cc < GATHER_TILE; cc += 256 / GATHER_TILE) {
        const int c = cbase + cc, r = r0 + lane;
        if (c < c0 && r < s.len) tile[cc][lane] = load_act<T>(latent + ((size_t)s.clip * c0 + c) * n_frames + s.lo + r);
    }
    __syncthreads();
    const int c = cbase + lane;
    if (c >= c0) return;
    const float al = xa ? alpha[c] : 0.f, ib = xa ? inv_beta[c] : 0.f;
    for (int rr = sub; rr < GATHER_TILE; rr += 256 / GATHER_TILE) {
        const int r = r0 + rr;
        if (r >= s.len) break;
        const float raw = tile[lane][rr];
        const size_t idx = ((size_t)s.row0 + r) * c0 + c;
        if (!xa) { x0[idx] = raw; continue; }
        const float v = snake_fast(raw, al, ib);
        if (fmt == OP_F16) {
            xa[idx] = __builtin_bit_cast(uint16_t, (_Float16)v);
        } else {
            const uint16_t hi = f32_to_bf16_bits(v);
            xa[idx] = hi;
            if (fmt == OP_BF16X2) xa[lo_off + idx] = f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
        }
    }
}

hipError_t launch_gather(const void* latent, float* x0, int c0, int n_frames, bool bf16,
                         const Slot* slots, int n_slots, int max_len, hipStream_t stream,
                         uint16_t* xa, int xa_fmt, long long xa_lo_off, const float* alpha, const float* inv_beta)
{
    if (xa && (!alpha || !inv_beta)) return hipErrorInvalidValue;
    dim3 grid((unsigned)((max_len + GATHER_TILE - 1) / GATHER_TILE), (unsigned)n_slots, (unsigned)((c0 + GATHER_TILE - 1) / GATHER_TILE));
    if (bf16)
        hipLaunchKernelGGL(gather_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t*)latent, x0, xa, xa_fmt, xa_lo_off, alpha, inv_beta, c0, n_frames, slots);
    else
        hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(256), 0, stream, (const float*)latent, x0, xa, xa_fmt, xa_lo_off, alpha, inv_beta, c0, n_frames, slots);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- encoder stem
// First layer of the encoder (the mirror of the head): Conv1d(k, channels -> C) + bias straight from the planar fp32
// waveform of every extended window into the time-major residual stream, and with `ya` the activated operand of the
// next layer as well.  Samples outside the window read as zero (the convolution's zero padding: the window is encoded
// as if it were a whole clip).  A thread owns one row: it loads its k x channels samples once (consecutive threads,
// consecutive samples) and walks the C output channels in groups of 8, whose weights are the same for every thread
// (scalar loads); K = k x channels is tiny (14 for stereo, k = 7), so this is bound by the store of the C-channel rows.
constexpr int STEM_MAXK = 15 * 8;                 // taps x channels held in registers

template <typename TY, int KCH>
__global__ __launch_bounds__(256) void stem_kernel(const float* __restrict__ wave, TY* __restrict__ y, uint16_t* __restrict__ ya,
                                                   int ya_fmt, const float* __restrict__ w /*[k][ch][C]*/,
                                                   const float* __restrict__ bias, const float* __restrict__ alpha,
                                                   const float* __restrict__ inv_beta, int ch, int C, int k, int S,
                                                   int n_frames, int margin, const Slot* __restrict__ slots)
{
    if (sizeof(TY) == 2) fp16_saturate_on();
    const Slot s = slots[blockIdx.y];
    const long long nrows = (long long)s.len * S;
    const long long out_lo = max(0ll, (long long)s.crop * S - margin);
    const long long out_hi = min(nrows, (long long)(s.crop + s.n_int) * S + margin);
    const long long n = out_lo + (long long)blockIdx.x * 256 + threadIdx.x;
    if (n >= out_hi) return;
    const int half = (k - 1) / 2;
    const float* clip = wave + (size_t)s.clip * ch * ((size_t)n_frames * S) + (long long)s.lo * S;
    float xv[KCH];                                 // [tap][channel]
#pragma unroll
    for (int q = 0; q < KCH; ++q) {
        const int t = q / ch, c = q - t * ch;
        const long long m = n + t - half;
        xv[q] = (q < k * ch && m >= 0 && m < nrows) ? clip[(size_t)c * ((size_t)n_frames * S) + m] : 0.f;
    }
    const size_t row = ((size_t)s.row0 * S + n) * C;
    for (int g = 0; g < C / 8; ++g) {
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = bias[8 * g + e];
#pragma unroll
        for (int q = 0; q < KCH; ++q) {
            if (q >= k * ch) break;                // uniform
            const float* wt = w + (size_t)q * C + 8 * g;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(wt[e], xv[q], acc[e]);
        }
        const size_t idx = row + 8 * g;
        if constexpr (sizeof(TY) == 4) {
            *reinterpret_cast<float4*>(&y[idx]) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            *reinterpret_cast<float4*>(&y[idx + 4]) = make_float4(acc[4], acc[5], acc[6], acc[7]);
        } else {
            f16x8 hv;
#pragma unroll
            for (int e = 0; e < 8; ++e) hv[e] = (_Float16)acc[e];
            *reinterpret_cast<f16x8*>(&y[idx]) = hv;
            if (ya) {
                // the next layer's operand is Snake of the STORED value
                u32x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float a0 = keep_f32(snake_fast((float)hv[2 * q], alpha[8 * g + 2 * q], inv_beta[8 * g + 2 * q]));
                    const float a1 = keep_f32(snake_fast((float)hv[2 * q + 1], alpha[8 * g + 2 * q + 1], inv_beta[8 * g + 2 * q + 1]));
                    o[q] = ya_fmt == OP_F16 ? pack_f16x2(a0, a1) : pack_bf16x2(a0, a1);
                }
                *reinterpret_cast<u32x4*>(&ya[idx]) = o;
            }
        }
    }
}

hipError_t launch_stem(const float* wave, void* y, bool y_half, uint16_t* ya, int ya_fmt, const float* w, const float* bias,
                       const float* alpha, const float* inv_beta, int ch, int C, int k, int S, int n_frames, int margin,
                       const Slot* slots, int n_slots, int max_len, int max_int, hipStream_t stream)
{
    if (C % 8 != 0 || k < 1 || (k & 1) == 0 || margin < 0 || k * ch > STEM_MAXK) return hipErrorInvalidValue;
    if (ya && (ya_fmt == OP_BF16X2 || !alpha || !inv_beta || !y_half)) return hipErrorInvalidValue;
    const long long rows = std::min((long long)max_int * S + 2ll * margin, (long long)max_len * S);
    dim3 grid((unsigned)((rows + 255) / 256), (unsigned)n_slots);
    // stereo with a 7-tap stem holds 14 samples per thread; anything up to 15 taps x 8 channels takes the large form
#define DEMON_STEM(TY_, KCH_) hipLaunchKernelGGL((stem_kernel<TY_, KCH_>), grid, dim3(256), 0, stream, wave, (TY_*)y, ya, ya_fmt, w, bias, alpha, \
                                                 inv_beta, ch, C, k, S, n_frames, margin, slots)
    if (y_half) { if (k * ch <= 16) DEMON_STEM(hres_t, 16); else DEMON_STEM(hres_t, STEM_MAXK); }
    else { if (k * ch <= 16) DEMON_STEM(float, 16); else DEMON_STEM(float, STEM_MAXK); }
#undef DEMON_STEM
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- encoder: sampling step + trim + scatter
// Last step of the windowed encode: of every window's moments [rows = frames, 2 C0] (mean | log-variance) keep the
// interior frames, write them to moments_out [clip, 2 C0, n_frames] (fp32) and the sampled latent
// z = mean + exp(logvar / 2) eps (the sampling step on the output moments of Table III; eps drawn by the caller, z = mean
// without eps) to latent_out [clip, C0, n_frames] in the path's latent type.  Either output may be absent.
template <typename TM, typename TZ>
__global__ __launch_bounds__(256) void sample_kernel(const TM* __restrict__ m, const float* __restrict__ eps,
                                                     float* __restrict__ moments_out, TZ* __restrict__ latent_out,
                                                     int C0, int n_frames, const Slot* __restrict__ slots)
{
    const Slot s = slots[blockIdx.y];
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= s.n_int * C0) return;
    const int fi = e / C0, c = e - fi * C0;
    const size_t row = (size_t)s.row0 + s.crop + fi;
    const int f = s.begin + fi;
    const float mean = load_act<TM>(m + row * (2 * C0) + c);
    const float lv = load_act<TM>(m + row * (2 * C0) + C0 + c);
    if (moments_out) {
        moments_out[((size_t)s.clip * 2 * C0 + c) * n_frames + f] = mean;
        moments_out[((size_t)s.clip * 2 * C0 + C0 + c) * n_frames + f] = lv;
    }
    if (latent_out) {
        const size_t zi = ((size_t)s.clip * C0 + c) * n_frames + f;
        const float z = eps ? fmaf(expf(0.5f * lv), eps[zi], mean) : mean;
        if constexpr (sizeof(TZ) == 2) latent_out[zi] = f32_to_bf16_bits(z);
        else latent_out[zi] = z;
    }
}

hipError_t launch_sample(const void* m, bool m_half, const float* eps, float* moments_out, void* latent_out, bool latent_bf16,
                         int C0, int n_frames, const Slot* slots, int n_slots, int max_int, hipStream_t stream)
{
    dim3 grid((unsigned)(((size_t)max_int * C0 + 255) / 256), (unsigned)n_slots);
    if (m_half && latent_bf16)
        hipLaunchKernelGGL((sample_kernel<_Float16, uint16_t>), grid, dim3(256), 0, stream, (const _Float16*)m, eps, moments_out, (uint16_t*)latent_out, C0, n_frames, slots);
    else if (!m_half && !latent_bf16)
        hipLaunchKernelGGL((sample_kernel<float, float>), grid, dim3(256), 0, stream, (const float*)m, eps, moments_out, (float*)latent_out, C0, n_frames, slots);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- head
// Only the interior rows of every window are produced (the halo is trimmed right after).  Rows outside
// the window read as zero (the conv's zero padding at a clip edge); Snake is applied while staging.
//
// Fast kernel (OC output channels, K taps as template arguments): a workgroup owns HEAD_NT = 1024
// consecutive samples, each thread 4 of them.  Channels go through LDS in chunks of 16, transposed to
// [channel][row] so that a thread's 4 + K - 1 input rows are consecutive words (three 16-byte reads per
// channel for K = 7) and feed 4*K*OC FMAs; the weights are wave-uniform (scalar loads).  The row
// length HEAD_LDR = 4 mod 16 keeps both the transposing stores and the reads free of bank conflicts.
constexpr int HEAD_SPT = 4;                    // samples per thread
constexpr int HEAD_NT = 256 * HEAD_SPT;
constexpr int HEAD_KC = 16;
constexpr int HEAD_MAXK = 15;
constexpr int HEAD_MAXOC = 8;
constexpr int HEAD_LDR = 1044;                 // >= HEAD_NT + HEAD_MAXK - 1, = 4 (mod 16)

template <typename TX, bool FAST, int OC, int K>
__global__ __launch_bounds__(256) void head_fast_kernel(const TX* __restrict__ x, float* __restrict__ y,
                                                        const float* __restrict__ w, const float* __restrict__ bias,
                                                        const float* __restrict__ alpha, const float* __restrict__ inv_beta,
                                                        int cin, int r, long long total_rows,
                                                        const Slot* __restrict__ slots)
{
    __shared__ __attribute__((aligned(16))) float xs[HEAD_KC * HEAD_LDR];
    constexpr int HALF = (K - 1) / 2;
    constexpr int XR = HEAD_NT + K - 1;
    constexpr int NV = (HEAD_SPT + K - 1 + 3) / 4;          // float4 reads per channel
    const Slot s = slots[blockIdx.y];
    const long long nrows = (long long)s.len * r;
    const long long lo = (long long)s.crop * r, hi = (long long)(s.crop + s.n_int) * r;
    const long long n0 = lo + (long long)blockIdx.x * HEAD_NT;
    if (n0 >= hi) return;
    const long long rowbase = (long long)s.row0 * r;
    const int tid = threadIdx.x;
    const int q = tid & 3, r0 = tid >> 2;                   // staging: 4 lanes per row, 4 channels each

    float acc[HEAD_SPT][OC];
#pragma unroll
    for (int i = 0; i < HEAD_SPT; ++i)
#pragma unroll
        for (int o = 0; o < OC; ++o) acc[i][o] = 0.f;

    for (int c0 = 0; c0 < cin; c0 += HEAD_KC) {
        const float4 al = *reinterpret_cast<const float4*>(alpha + c0 + 4 * q);
        const float4 ib = *reinterpret_cast<const float4*>(inv_beta + c0 + 4 * q);
        __syncthreads();
        for (int row = r0; row < XR; row += 64) {
            const long long n = n0 - HALF + row;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n >= 0 && n < nrows) {
                const TX* src = x + (size_t)(rowbase + n) * cin + c0 + 4 * q;
                if (sizeof(TX) == 4) {
                    v = *reinterpret_cast<const float4*>(src);
                } else {
                    const f16x4 hv = *reinterpret_cast<const f16x4*>(src);
                    v = make_float4((float)hv[0], (float)hv[1], (float)hv[2], (float)hv[3]);
                }
                if (FAST) {
                    v.x = snake_fast(v.x, al.x, ib.x); v.y = snake_fast(v.y, al.y, ib.y);
                    v.z = snake_fast(v.z, al.z, ib.z); v.w = snake_fast(v.w, al.w, ib.w);
                } else {
                    v.x = snake_precise(v.x, al.x, ib.x); v.y = snake_precise(v.y, al.y, ib.y);
                    v.z = snake_precise(v.z, al.z, ib.z); v.w = snake_precise(v.w, al.w, ib.w);
                }
            }
            xs[(4 * q + 0) * HEAD_LDR + row] = v.x;
            xs[(4 * q + 1) * HEAD_LDR + row] = v.y;
            xs[(4 * q + 2) * HEAD_LDR + row] = v.z;
            xs[(4 * q + 3) * HEAD_LDR + row] = v.w;
        }
        __syncthreads();
#pragma unroll 4
        for (int c = 0; c < HEAD_KC; ++c) {
            float xv[NV * 4];
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const float4 t4 = *reinterpret_cast<const float4*>(&xs[c * HEAD_LDR + HEAD_SPT * tid + 4 * i]);
                xv[4 * i] = t4.x; xv[4 * i + 1] = t4.y; xv[4 * i + 2] = t4.z; xv[4 * i + 3] = t4.w;
            }
#pragma unroll
            for (int t = 0; t < K; ++t)
#pragma unroll
                for (int o = 0; o < OC; ++o) {
                    const float wv = w[((size_t)t * cin + c0 + c) * OC + o];
#pragma unroll
                    for (int i = 0; i < HEAD_SPT; ++i) acc[i][o] = fmaf(wv, xv[i + t], acc[i][o]);
                }
        }
    }
    const long long n = n0 + HEAD_SPT * tid;
#pragma unroll
    for (int o = 0; o < OC; ++o) {
        const float b = bias[o];
        float* dst = y + (size_t)o * total_rows + rowbase + n;
        if (n + HEAD_SPT <= hi && (r % 4) == 0) {
            *reinterpret_cast<float4*>(dst) = make_float4(tanhf(acc[0][o] + b), tanhf(acc[1][o] + b),
                                                          tanhf(acc[2][o] + b), tanhf(acc[3][o] + b));
        } else {
#pragma unroll
            for (int i = 0; i < HEAD_SPT; ++i)
                if (n + i < hi) dst[i] = tanhf(acc[i][o] + b);
        }
    }
}

// Generic kernel (any out_channels <= 8, any odd kernel <= 15, any channel count): one sample per
// thread, channels staged through LDS in chunks of 32.
constexpr int HEADG_NT = 256;
constexpr int HEADG_KC = 32;

template <typename TX, bool FAST>
__global__ __launch_bounds__(256) void head_generic_kernel(const TX* __restrict__ x, float* __restrict__ y,
                                                           const float* __restrict__ w, const float* __restrict__ bias,
                                                           const float* __restrict__ alpha, const float* __restrict__ inv_beta,
                                                           int cin, int oc, int k, int r, long long total_rows,
                                                           const Slot* __restrict__ slots)
{
    __shared__ float xs[(HEADG_NT + HEAD_MAXK - 1) * (HEADG_KC + 1)];
    const Slot s = slots[blockIdx.y];
    const long long nrows = (long long)s.len * r;
    const long long lo = (long long)s.crop * r, hi = (long long)(s.crop + s.n_int) * r;
    const long long n0 = lo + (long long)blockIdx.x * HEADG_NT;
    if (n0 >= hi) return;
    const long long rowbase = (long long)s.row0 * r;
    const int half = (k - 1) / 2;
    const int xr = HEADG_NT + k - 1;

    float acc[HEAD_MAXOC];
#pragma unroll
    for (int o = 0; o < HEAD_MAXOC; ++o) acc[o] = 0.f;

    for (int c0 = 0; c0 < cin; c0 += HEADG_KC) {
        const int kc = min(HEADG_KC, cin - c0);
        __syncthreads();
        for (int e = threadIdx.x; e < xr * HEADG_KC; e += 256) {
            const int row = e / HEADG_KC, c = e - row * HEADG_KC;
            const long long n = n0 - half + row;
            float v = 0.f;
            if (c < kc && n >= 0 && n < nrows) {
                v = load_act<TX>(x + (size_t)(rowbase + n) * cin + c0 + c);
                v = FAST ? snake_fast(v, alpha[c0 + c], inv_beta[c0 + c]) : snake_precise(v, alpha[c0 + c], inv_beta[c0 + c]);
            }
            xs[row * (HEADG_KC + 1) + c] = v;
        }
        __syncthreads();
        for (int t = 0; t < k; ++t) {
            const float* xrow = xs + (threadIdx.x + t) * (HEADG_KC + 1);
            const float* wt = w + ((size_t)t * cin + c0) * oc;
            for (int c = 0; c < kc; ++c) {
                const float v = xrow[c];
#pragma unroll
                for (int o = 0; o < HEAD_MAXOC; ++o)
                    if (o < oc) acc[o] = fmaf(wt[c * oc + o], v, acc[o]);
            }
        }
    }
    const long long n = n0 + threadIdx.x;
    if (n < hi) {
#pragma unroll
        for (int o = 0; o < HEAD_MAXOC; ++o)
            if (o < oc) y[(size_t)o * total_rows + rowbase + n] = tanhf(acc[o] + bias[o]);
    }
}

// MFMA head for the bf16 path (half-precision residual stream in, out_channels <= 32).
// GEMM with rows = time, columns = output channel (padded to 32), K = (tap, channel):
//     D[n, o] = sum_t sum_c snake(h[n + t - (K-1)/2, c]) W[o, c, t]
// on v_mfma_f32_32x32x16_f16: operands in IEEE half (their rounding is an order of magnitude below that of
// the bf16 operands elsewhere), fp32 accumulation.  The A operand is the activation tile: whole 128-byte
// rows are read once from HBM, Snake is applied in fp32, the tile sits row-major in LDS and a tap is a row
// offset.  The B operand (the weights, zero beyond out_channels) is packed at create in fragment order and
// staged into LDS once per workgroup.  A lane with column index < out_channels holds the results.
constexpr int HM_NT = 256;                     // rows per sub-tile: 4 waves x 64 rows
constexpr int HM_SUB = 4;                      // sub-tiles per workgroup (the weights are staged once)
constexpr int HM_MAXFRAG = 40;                 // taps * channels / 16

size_t head_mfma_frag_count(int cin, int k) { return (size_t)k * (cin / 16); }

// [tap][k-step][lane][8]: lane (j, h) of k-step ks holds W[o = j][c = 16 ks + 8 h + e][tap], e = 0..7
void pack_head_mfma(const float* w /*[oc][cin][k]*/, int cin, int oc, int k, uint16_t* dst)
{
    size_t pos = 0;
    for (int t = 0; t < k; ++t)
        for (int ks = 0; ks < cin / 16; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 8; ++e) {
                    const int j = lane & 31, h = lane >> 5, c = 16 * ks + 8 * h + e;
                    const _Float16 v = (j < oc) ? (_Float16)w[((size_t)j * cin + c) * k + t] : (_Float16)0.f;
                    uint16_t bits;
                    __builtin_memcpy(&bits, &v, 2);
                    dst[pos++] = bits;
                }
}

typedef _Float16 f16x8v __attribute__((ext_vector_type(8)));

// OCP: output channels kept in LDS per weight fragment (8 when oc <= 8, else 32): the other lanes of the fragment are
// zero padding and are not stored, which with the unpadded-weights tile leaves room for three workgroups per CU.
template <int CIN, int OCP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OCP == 8 ? 3 : 2, OCP == 8 ? 3 : 2)))
void head_mfma_kernel(const _Float16* __restrict__ x, float* __restrict__ y,
                                                        const uint16_t* __restrict__ wfrag, const float* __restrict__ bias,
                                                        const float* __restrict__ alpha, const float* __restrict__ inv_beta,
                                                        int oc, int k, int r, long long total_rows,
                                                        const Slot* __restrict__ slots)
{
    fp16_saturate_on();
    constexpr int LDX = CIN + 8;                           // padded LDS row (halfs)
    constexpr int XR_MAX = HM_NT + HEAD_MAXK - 1;
    constexpr int SEGS = CIN / 8, RPP = 256 / SEGS;
    constexpr int X_ITERS = (XR_MAX + RPP - 1) / RPP;
    constexpr int KS = CIN / 16;
    __shared__ __attribute__((aligned(16))) _Float16 Xs[XR_MAX * LDX];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[HM_MAXFRAG * 2 * OCP * 8];       // [fragment][h][channel < OCP][8 halves]

    const Slot s = slots[blockIdx.y];
    const int nrows = s.len * r;
    const int lo = s.crop * r, hi = (s.crop + s.n_int) * r;
    const int half = (k - 1) / 2;
    const int XR = HM_NT + k - 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, j = lane & 31, h = lane >> 5;
    const int seg = tid % SEGS, xr0 = tid / SEGS;
    const long long rowbase = (long long)s.row0 * r;
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(x + rowbase * CIN, (unsigned)nrows * CIN * 2u);
    if (lo + (int)blockIdx.x * (HM_NT * HM_SUB) >= hi) return;

    // weights -> LDS once
    {
        const u32x4* src = reinterpret_cast<const u32x4*>(wfrag);             // [fragment][lane = h * 32 + channel][8 halves]
        for (int q = tid; q < k * KS * 2 * OCP; q += 256)
            reinterpret_cast<u32x4*>(Ws)[q] = src[(q / OCP) * 32 + q % OCP];
    }
    float al[8], ib[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { al[e] = alpha[seg * 8 + e]; ib[e] = inv_beta[seg * 8 + e]; }
    // accumulator register 4g + q of lane (j, h) is output channel 8g + 4h + q: with OCP = 8 only g = 0 holds channels
    constexpr int NB = OCP == 8 ? 4 : 16;
    float b[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int c = 8 * (q >> 2) + 4 * h + (q & 3);
        b[q] = (c < oc) ? bias[c] : 0.f;
    }

    // The raw rows of a sub-tile are fetched one sub-tile ahead, so that their latency hides behind the MFMAs and the
    // tanh epilogue of the previous one.  Rows outside the window are out of range of the descriptor and read as
    // zero = the convolution's zero padding.
    u32x4 raw[X_ITERS];
    auto load_rows = [&](int n0) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            if (it * RPP >= XR) break;                         // uniform
            raw[it] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, (unsigned)((n0 - half + xr0 + it * RPP) * CIN + seg * 8) * 2u, 0, 0);
        }
    };
    load_rows(lo + (int)blockIdx.x * (HM_NT * HM_SUB));
    for (int sub = 0; sub < HM_SUB; ++sub) {
        const int n0 = lo + ((int)blockIdx.x * HM_SUB + sub) * HM_NT;
        if (n0 >= hi) break;                                   // uniform
        __syncthreads();                                       // the previous sub-tile's reads are done
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            const int xr = xr0 + it * RPP;
            if (it * RPP >= XR) break;                         // uniform
            if (xr >= XR_MAX) continue;
            const f16x8v hv = __builtin_bit_cast(f16x8v, raw[it]);
            f16x8v ov;
#pragma unroll
            for (int e = 0; e < 8; ++e) ov[e] = (_Float16)keep_f32(snake_fast((float)hv[e], al[e], ib[e]));
            *reinterpret_cast<f16x8v*>(&Xs[xr * LDX + seg * 8]) = ov;
        }
        __syncthreads();
        if (sub + 1 < HM_SUB && n0 + HM_NT < hi) load_rows(n0 + HM_NT);

        f32x16 acc[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[mi][q] = q < NB ? b[q] : 0.f;
        for (int t = 0; t < k; ++t) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                f16x8v bw = {0, 0, 0, 0, 0, 0, 0, 0};
                if (j < OCP) bw = *reinterpret_cast<const f16x8v*>(&Ws[(((t * KS + ks) * 2 + h) * OCP + j) * 8]);
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    const f16x8v av = *reinterpret_cast<const f16x8v*>(&Xs[(wave * 64 + mi * 32 + j + t) * LDX + ks * 16 + h * 8]);
                    // weights as the row operand: the accumulator tile is [output channel][time]
                    acc[mi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bw, av, acc[mi], 0, 0, 0);
                }
            }
        }
        // lane (j, h) holds time column j and output channels 8g + 4h + {0..3}: with a few output channels the tanh work
        // sits in the first registers of half of the lanes, and a channel's 32 samples are one contiguous store
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const int n = n0 + wave * 64 + mi * 32 + j;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (8 * g >= oc) break;                        // uniform
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = 8 * g + 4 * h + q;
                    if (c < oc && n < hi) y[(size_t)c * total_rows + rowbase + n] = tanhf(acc[mi][4 * g + q]);
                }
            }
        }
    }
}

hipError_t launch_head_mfma(const void* x, float* y, const uint16_t* wfrag, const float* bias, const float* alpha,
                            const float* inv_beta, int cin, int oc, int k, int r, long long total_rows,
                            const Slot* slots, int n_slots, int max_len, int max_int, hipStream_t stream)
{
    if (oc > 32 || k > HEAD_MAXK || (cin != 64 && cin != 32) || head_mfma_frag_count(cin, k) > HM_MAXFRAG) return hipErrorInvalidValue;
    if ((long long)max_len * r * cin * 2 > 0xf0000000ll) return hipErrorInvalidValue;
    const long long rows = (long long)max_int * r;
    dim3 grid((unsigned)((rows + HM_NT * HM_SUB - 1) / (HM_NT * HM_SUB)), (unsigned)n_slots);
#define DEMON_HEAD(CIN_, OCP_) hipLaunchKernelGGL((head_mfma_kernel<CIN_, OCP_>), grid, dim3(256), 0, stream, (const _Float16*)x, y, wfrag, bias, alpha, inv_beta, oc, k, r, total_rows, slots)
    if (cin == 64) { if (oc <= 8) DEMON_HEAD(64, 8); else DEMON_HEAD(64, 32); }
    else { if (oc <= 8) DEMON_HEAD(32, 8); else DEMON_HEAD(32, 32); }
#undef DEMON_HEAD
    return hipGetLastError();
}

hipError_t launch_head(const void* x, bool x_half, float* y, const float* w, const float* bias, const float* alpha,
                       const float* inv_beta, int cin, int oc, int k, int r, long long total_rows,
                       bool fast, const Slot* slots, int n_slots, int max_int, hipStream_t stream)
{
    if (k > HEAD_MAXK || oc > HEAD_MAXOC || (x_half && !fast)) return hipErrorInvalidValue;
    const long long rows = (long long)max_int * r;
    if (oc == 2 && k == 7 && cin % HEAD_KC == 0) {
        dim3 grid((unsigned)((rows + HEAD_NT - 1) / HEAD_NT), (unsigned)n_slots);
        if (x_half)
            hipLaunchKernelGGL((head_fast_kernel<_Float16, true, 2, 7>), grid, dim3(256), 0, stream, (const _Float16*)x, y, w, bias, alpha, inv_beta, cin, r, total_rows, slots);
        else if (fast)
            hipLaunchKernelGGL((head_fast_kernel<float, true, 2, 7>), grid, dim3(256), 0, stream, (const float*)x, y, w, bias, alpha, inv_beta, cin, r, total_rows, slots);
        else
            hipLaunchKernelGGL((head_fast_kernel<float, false, 2, 7>), grid, dim3(256), 0, stream, (const float*)x, y, w, bias, alpha, inv_beta, cin, r, total_rows, slots);
        return hipGetLastError();
    }
    dim3 grid((unsigned)((rows + HEADG_NT - 1) / HEADG_NT), (unsigned)n_slots);
    if (x_half)
        hipLaunchKernelGGL((head_generic_kernel<_Float16, true>), grid, dim3(256), 0, stream, (const _Float16*)x, y, w, bias, alpha, inv_beta, cin, oc, k, r, total_rows, slots);
    else if (fast)
        hipLaunchKernelGGL((head_generic_kernel<float, true>), grid, dim3(256), 0, stream, (const float*)x, y, w, bias, alpha, inv_beta, cin, oc, k, r, total_rows, slots);
    else
        hipLaunchKernelGGL((head_generic_kernel<float, false>), grid, dim3(256), 0, stream, (const float*)x, y, w, bias, alpha, inv_beta, cin, oc, k, r, total_rows, slots);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- stitch
// grid (chunks of the interior, slots, output channels).  VEC = 4 when S % 4 == 0 (then every
// interior starts on a 16-byte boundary in both buffers), else 1.
template <int VEC>
__global__ __launch_bounds__(256) void stitch_kernel(const float* __restrict__ y, float* __restrict__ out,
                                                     int oc, int S, int n_frames, long long total_rows,
                                                     const Slot* __restrict__ slots)
{
    const Slot s = slots[blockIdx.y];
    const int c = blockIdx.z;
    const long long n = (long long)s.n_int * S;
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (i >= n) return;
    const float* src = y + (size_t)c * total_rows + ((long long)s.row0 + s.crop) * S + i;
    float* dst = out + ((size_t)s.clip * oc + c) * ((size_t)n_frames * S) + (long long)s.begin * S + i;
    if (VEC == 4) *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(src);
    else *dst = *src;
}

hipError_t launch_stitch(const float* y, float* out, int oc, int S, int n_frames, long long total_rows,
                         const Slot* slots, int n_slots, int max_int, hipStream_t stream)
{
    const bool vec = (S % 4 == 0) && ((reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(out)) % 16 == 0);
    const long long per = (long long)max_int * S;
    if (vec) {
        dim3 grid((unsigned)((per / 4 + 255) / 256), (unsigned)n_slots, (unsigned)oc);
        hipLaunchKernelGGL(stitch_kernel<4>, grid, dim3(256), 0, stream, y, out, oc, S, n_frames, total_rows, slots);
    } else {
        dim3 grid((unsigned)((per + 255) / 256), (unsigned)n_slots, (unsigned)oc);
        hipLaunchKernelGGL(stitch_kernel<1>, grid, dim3(256), 0, stream, y, out, oc, S, n_frames, total_rows, slots);
    }
    return hipGetLastError();
}

// 16-bit render fused into the stitch: q = rint(32767 * clamp(y, -1, 1)) in fp32 (round half to even), channels
// interleaved per sample: pcm[clip][sample][channel].  One thread quantises VEC consecutive samples of all channels.
template <int VEC, int OC>
__global__ __launch_bounds__(256) void stitch_pcm16_kernel(const float* __restrict__ y, int16_t* __restrict__ pcm,
                                                           int oc, int S, int n_frames, long long total_rows,
                                                           const Slot* __restrict__ slots)
{
    const Slot s = slots[blockIdx.y];
    const long long n = (long long)s.n_int * S;
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (i >= n) return;
    const float* src = y + ((long long)s.row0 + s.crop) * S + i;
    int16_t* dst = pcm + ((size_t)s.clip * ((size_t)n_frames * S) + (size_t)s.begin * S + i) * oc;
    auto quant = [](float v) -> int16_t {
        v = fminf(fmaxf(v, -1.0f), 1.0f);
        return (int16_t)__float2int_rn(v * 32767.0f);
    };
    if (OC == 2 && VEC == 4) {
        const float4 l = *reinterpret_cast<const float4*>(src);
        const float4 r = *reinterpret_cast<const float4*>(src + total_rows);
        const float lv[4] = {l.x, l.y, l.z, l.w}, rv[4] = {r.x, r.y, r.z, r.w};
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = (uint32_t)(uint16_t)quant(lv[e]) | ((uint32_t)(uint16_t)quant(rv[e]) << 16);
        *reinterpret_cast<u32x4*>(dst) = o;
    } else {
        for (int e = 0; e < VEC && i + e < n; ++e)
            for (int c = 0; c < oc; ++c) dst[(size_t)e * oc + c] = quant(src[(size_t)c * total_rows + e]);
    }
}

hipError_t launch_stitch_pcm16(const float* y, int16_t* pcm, int oc, int S, int n_frames, long long total_rows,
                               const Slot* slots, int n_slots, int max_int, hipStream_t stream)
{
    // 16-byte stores need 4 stereo samples per thread at a 16-byte aligned address: S % 4 == 0 keeps every window start aligned
    const bool vec = oc == 2 && (S % 4 == 0) && (total_rows % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(y) % 16 == 0) && (reinterpret_cast<uintptr_t>(pcm) % 16 == 0);
    const long long per = (long long)max_int * S;
    if (vec) {
        dim3 grid((unsigned)((per / 4 + 255) / 256), (unsigned)n_slots);
        hipLaunchKernelGGL((stitch_pcm16_kernel<4, 2>), grid, dim3(256), 0, stream, y, pcm, oc, S, n_frames, total_rows, slots);
    } else {
        dim3 grid((unsigned)((per + 255) / 256), (unsigned)n_slots);
        hipLaunchKernelGGL((stitch_pcm16_kernel<1, 0>), grid, dim3(256), 0, stream, y, pcm, oc, S, n_frames, total_rows, slots);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- decode gate
// Copy of a window table in which the windows of skipped clips are empty (no rows, no interior): every kernel of the
// decode derives its work from the table, so those clips cost (almost) nothing and their output is left untouched.
__global__ __launch_bounds__(256) void gate_slots_kernel(const Slot* __restrict__ src, Slot* __restrict__ dst, int n,
                                                         const int* __restrict__ skip)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    Slot s = src[i];
    if (skip[s.clip] != 0) { s.len = 0; s.n_int = 0; s.crop = 0; }
    dst[i] = s;
}

hipError_t launch_gate_slots(const Slot* src, Slot* dst, int n, const int* skip, hipStream_t stream)
{
    hipLaunchKernelGGL(gate_slots_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, src, dst, n, skip);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- window table on the device
// The window grid of section 3.6 written by a kernel: window k of a clip covers frames [begin + k window, ...), is
// extended by the halo and clamped to the clip; its workspace rows follow those of the windows before it (the windows
// from `split` on form a second group whose rows count from the group's first).  One thread per window; the prefix
// sum over the earlier windows of the clip is a short loop (at most 4096 windows per call).
__global__ __launch_bounds__(256) void plan_slots_kernel(Slot* __restrict__ dst, int n, int per_clip, int clip_frames,
                                                         int n_frames, int fb, int fe, int window, int halo, int split, int split_row0)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int clip = i / per_clip, k = i - clip * per_clip;
    auto extent = [&](int kk, int* lo, int* hi, int* b, int* e) {
        *b = fb + kk * window;
        *e = min(*b + window, fe);
        *lo = max(0, *b - halo);
        *hi = min(n_frames, *e + halo);
    };
    int row = clip * clip_frames;
    for (int kk = 0; kk < k; ++kk) {
        int lo, hi, b, e;
        extent(kk, &lo, &hi, &b, &e);
        row += hi - lo;
    }
    int lo, hi, b, e;
    extent(k, &lo, &hi, &b, &e);
    Slot s;
    s.row0 = i >= split ? row - split_row0 : row; s.len = hi - lo; s.clip = clip; s.lo = lo; s.crop = b - lo; s.n_int = e - b; s.begin = b; s.pad = 0;
    dst[i] = s;
}

hipError_t launch_plan_slots(Slot* dst, int n_clips, int per_clip, int clip_frames, int n_frames, int frame_begin,
                             int frame_end, int window, int halo, int split, int split_row0, hipStream_t stream)
{
    const long long n = (long long)n_clips * per_clip;
    if (n < 1 || n > 65536) return hipErrorInvalidValue;
    hipLaunchKernelGGL(plan_slots_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, dst, (int)n, per_clip, clip_frames,
                       n_frames, frame_begin, frame_end, window, halo, split, split_row0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- latent similarity filter
// One workgroup per clip: squared differences accumulate in double in a fixed order (thread-strided partial sums, then a
// tree over the workgroup), so the result does not depend on scheduling.  mse and the gate go out as fp32 / int.
template <typename T>
__global__ __launch_bounds__(1024) void latent_mse_kernel(const T* __restrict__ a, const T* __restrict__ b, long long n,
                                                          float threshold, float* __restrict__ mse, int* __restrict__ unchanged)
{
    __shared__ double part[16];
    const T* pa = a + (size_t)blockIdx.x * n;
    const T* pb = b + (size_t)blockIdx.x * n;
    double acc = 0.0;
    for (long long i = threadIdx.x; i < n; i += 1024) {
        const double d = (double)load_act<T>(pa + i) - (double)load_act<T>(pb + i);
        acc += d * d;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += part[w];
        const float m = (float)(t / (double)n);
        if (mse) mse[blockIdx.x] = m;
        if (unchanged) unchanged[blockIdx.x] = m < threshold ? 1 : 0;
    }
}

hipError_t launch_latent_mse(const void* a, const void* b, int n_clips, long long n, bool bf16, float threshold,
                             float* mse, int* unchanged, hipStream_t stream)
{
    if (bf16)
        hipLaunchKernelGGL(latent_mse_kernel<uint16_t>, dim3(n_clips), dim3(1024), 0, stream,
                           (const uint16_t*)a, (const uint16_t*)b, n, threshold, mse, unchanged);
    else
        hipLaunchKernelGGL(latent_mse_kernel<float>, dim3(n_clips), dim3(1024), 0, stream,
                           (const float*)a, (const float*)b, n, threshold, mse, unchanged);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- equal-power crossfade
// out[c][i] = cos(theta_i) * tail[c][i] + sin(theta_i) * head[c][i], theta_i = (pi/2)(i + 1/2)/n.  Element-wise, so out may
// alias head or tail.
__global__ __launch_bounds__(256) void crossfade_kernel(const float* __restrict__ tail, long long tail_stride,
                                                        const float* __restrict__ head, long long head_stride,
                                                        float* out, long long out_stride, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int c = blockIdx.y;
    const float theta = 1.57079632679489662f * (((float)i + 0.5f) / (float)n);
    float sn, cs;
    sincosf(theta, &sn, &cs);
    out[c * out_stride + i] = cs * tail[c * tail_stride + i] + sn * head[c * head_stride + i];
}

hipError_t launch_crossfade(const float* tail, long long tail_stride, const float* head, long long head_stride,
                            float* out, long long out_stride, int n_planes, int n, hipStream_t stream)
{
    dim3 grid((unsigned)((n + 255) / 256), (unsigned)n_planes);
    hipLaunchKernelGGL(crossfade_kernel, grid, dim3(256), 0, stream, tail, tail_stride, head, head_stride, out, out_stride, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- debug tap
template <typename T>
__global__ __launch_bounds__(256) void to_f32_kernel(const T* __restrict__ x, float* __restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = load_act<T>(x + i);
}

hipError_t launch_to_f32(const void* x, float* dst, size_t n, int src_type, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + 255) / 256));
    if (src_type == 1) hipLaunchKernelGGL(to_f32_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t*)x, dst, n);
    else if (src_type == 2) hipLaunchKernelGGL(to_f32_kernel<_Float16>, grid, dim3(256), 0, stream, (const _Float16*)x, dst, n);
    else hipLaunchKernelGGL(to_f32_kernel<float>, grid, dim3(256), 0, stream, (const float*)x, dst, n);
    return hipGetLastError();
}

}  // namespace demon
