// Window gather, output head, crop/stitch and the debug tap (HBM-bound kernels).
//
// gather : step 1 of the windowed decode of paper section 3.6 (extend each window by its margins):
//          copies latent frames [lo, hi) of every window into its slot, transposing to time-major.
// head   : Snake -> Conv1d(k, C -> out_channels) -> tanh, the last layer of the decoder.
// stitch : step 3 (trim the margins, keep the frame-aligned interior) plus the side-by-side write
//          of the interiors into the clip's waveform.
#include "device_common.h"

namespace demon {

template <typename T> __device__ __forceinline__ float load_act(const T* p);
template <> __device__ __forceinline__ float load_act<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_act<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// ---------------------------------------------------------------------------------- gather
template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(const T* __restrict__ latent, float* __restrict__ x0,
                                                     int c0, int n_frames, const Slot* __restrict__ slots)
{
    const Slot s = slots[blockIdx.y];
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= s.len * c0) return;
    const int r = e / c0, c = e - r * c0;
    x0[((size_t)s.row0 + r) * c0 + c] = load_act<T>(latent + ((size_t)s.clip * c0 + c) * n_frames + s.lo + r);
}

hipError_t launch_gather(const void* latent, float* x0, int c0, int n_frames, bool bf16,
                         const Slot* slots, int n_slots, int max_len, hipStream_t stream)
{
    dim3 grid((unsigned)(((size_t)max_len * c0 + 255) / 256), (unsigned)n_slots);
    if (bf16)
        hipLaunchKernelGGL(gather_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t*)latent, x0, c0, n_frames, slots);
    else
        hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(256), 0, stream, (const float*)latent, x0, c0, n_frames, slots);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- head
// One workgroup = 256 consecutive samples of one slot.  Channels are staged through LDS in chunks
// of HEAD_KC (Snake applied while staging, rows outside the slot read as zero = the conv's zero
// padding); each thread then owns one sample and all output channels.
constexpr int HEAD_NT = 256;
constexpr int HEAD_KC = 32;
constexpr int HEAD_MAXK = 15;
constexpr int HEAD_MAXOC = 8;

template <bool FAST>
__global__ __launch_bounds__(256) void head_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                   const float* __restrict__ w, const float* __restrict__ bias,
                                                   const float* __restrict__ alpha, const float* __restrict__ inv_beta,
                                                   int cin, int oc, int k, int r, long long total_rows,
                                                   const Slot* __restrict__ slots)
{
    __shared__ float xs[(HEAD_NT + HEAD_MAXK - 1) * (HEAD_KC + 1)];
    const Slot s = slots[blockIdx.y];
    const long long nrows = (long long)s.len * r;
    const long long n0 = (long long)blockIdx.x * HEAD_NT;
    if (n0 >= nrows) return;
    const long long rowbase = (long long)s.row0 * r;
    const int half = (k - 1) / 2;
    const int xr = HEAD_NT + k - 1;

    float acc[HEAD_MAXOC];
#pragma unroll
    for (int o = 0; o < HEAD_MAXOC; ++o) acc[o] = 0.f;

    for (int c0 = 0; c0 < cin; c0 += HEAD_KC) {
        const int kc = min(HEAD_KC, cin - c0);
        __syncthreads();
        for (int e = threadIdx.x; e < xr * HEAD_KC; e += 256) {
            const int row = e / HEAD_KC, c = e - row * HEAD_KC;
            const long long n = n0 - half + row;
            float v = 0.f;
            if (c < kc && n >= 0 && n < nrows) {
                v = x[(size_t)(rowbase + n) * cin + c0 + c];
                v = FAST ? snake_fast(v, alpha[c0 + c], inv_beta[c0 + c]) : snake_precise(v, alpha[c0 + c], inv_beta[c0 + c]);
            }
            xs[row * (HEAD_KC + 1) + c] = v;
        }
        __syncthreads();
        for (int t = 0; t < k; ++t) {
            const float* xrow = xs + (threadIdx.x + t) * (HEAD_KC + 1);
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
    if (n < nrows) {
#pragma unroll
        for (int o = 0; o < HEAD_MAXOC; ++o)
            if (o < oc) y[(size_t)o * total_rows + rowbase + n] = tanhf(acc[o] + bias[o]);
    }
}

hipError_t launch_head(const float* x, float* y, const float* w, const float* bias, const float* alpha,
                       const float* inv_beta, int cin, int oc, int k, int r, long long total_rows,
                       bool fast, const Slot* slots, int n_slots, int max_len, hipStream_t stream)
{
    if (k > HEAD_MAXK || oc > HEAD_MAXOC) return hipErrorInvalidValue;
    dim3 grid((unsigned)(((long long)max_len * r + HEAD_NT - 1) / HEAD_NT), (unsigned)n_slots);
    if (fast)
        hipLaunchKernelGGL(head_kernel<true>, grid, dim3(256), 0, stream, x, y, w, bias, alpha, inv_beta, cin, oc, k, r, total_rows, slots);
    else
        hipLaunchKernelGGL(head_kernel<false>, grid, dim3(256), 0, stream, x, y, w, bias, alpha, inv_beta, cin, oc, k, r, total_rows, slots);
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

// ---------------------------------------------------------------------------------- debug tap
template <typename T>
__global__ __launch_bounds__(256) void to_f32_kernel(const T* __restrict__ x, float* __restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = load_act<T>(x + i);
}

hipError_t launch_to_f32(const void* x, float* dst, size_t n, bool bf16, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + 255) / 256));
    if (bf16) hipLaunchKernelGGL(to_f32_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t*)x, dst, n);
    else hipLaunchKernelGGL(to_f32_kernel<float>, grid, dim3(256), 0, stream, (const float*)x, dst, n);
    return hipGetLastError();
}

}  // namespace demon
