// fp32 reference-precision path: plain FMA kernels, one thread per output element.
// Same layer semantics as the bf16 path (decoder layers of the benchmark description):
//   conv  : y[n, o] = b[o] + sum_t sum_i W[o,i,t] x[n + (t - (k-1)/2) d, i]      (x = 0 outside the slot)
//   convT : y[m s - p + phi, o] = b[o] + sum_j sum_i W[i,o,phi + j s] x[m - j, i],  j in {0,1}, p = s/2
//   convS : y[n, o] = b[o] + sum_t sum_i W[o,i,t] x[n s - p + t, i],  t in 0..2s-1, p = s/2   (the encoder's strided conv)
#include <algorithm>

#include "device_common.h"

namespace demon {

__global__ __launch_bounds__(256) void snake_f32_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                        const float* __restrict__ alpha,
                                                        const float* __restrict__ inv_beta, int C, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int c = (int)(i % (size_t)C);
    y[i] = snake_precise(x[i], alpha[c], inv_beta[c]);
}

hipError_t launch_snake_f32(const float* x, float* y, const float* alpha, const float* inv_beta, int C,
                            size_t n, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(snake_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, x, y, alpha, inv_beta, C, n);
    return hipGetLastError();
}

// Weights packed as [tap][cin][M] (M fastest) so that consecutive lanes read consecutive words.
// M = cout for Conv1d, s*cout (row mu = phi*cout + o) for ConvTranspose1d.
size_t packed_f32_count(int cin, int cout, int ntaps, int stride)
{
    const size_t M = stride > 0 ? (size_t)stride * cout : (size_t)cout;
    return (size_t)ntaps * cin * M;
}

void pack_f32(const float* w, int cin, int cout, int ntaps, int stride, float* dst)
{
    if (stride == 0) {
        for (int t = 0; t < ntaps; ++t)
            for (int i = 0; i < cin; ++i)
                for (int o = 0; o < cout; ++o)
                    dst[((size_t)t * cin + i) * cout + o] = w[((size_t)o * cin + i) * ntaps + t];
    } else {
        const int s = stride, M = s * cout;
        for (int j = 0; j < 2; ++j)
            for (int i = 0; i < cin; ++i)
                for (int phi = 0; phi < s; ++phi)
                    for (int o = 0; o < cout; ++o)
                        dst[((size_t)j * cin + i) * M + phi * cout + o] = w[((size_t)i * cout + o) * (2 * s) + phi + j * s];
    }
}

// grid: (ceil(ncols*M/256), n_slots); thread -> (col, mu), mu fastest.
__global__ __launch_bounds__(256) void conv_f32_kernel(ConvArgs a)
{
    const Slot s = a.slots[blockIdx.y];
    const int M = a.stride > 0 ? a.stride * a.cout : a.cout;
    const long long nrows_in = (long long)s.len * a.r_in;
    // output rows that later layers read: the interior widened by `margin`, clamped to the window
    const long long r_out = a.stride > 0 ? (long long)a.r_in * a.stride : a.down > 0 ? a.r_in / a.down : a.r_in;
    const long long out_lo = max(0ll, s.crop * r_out - a.margin);
    const long long out_hi = min(s.len * r_out, (s.crop + s.n_int) * r_out + a.margin);
    if (out_hi <= out_lo) return;                        // an empty window (a gated clip)
    const long long col_lo = a.stride > 0 ? (out_lo + a.stride / 2) / a.stride : out_lo;
    const long long col_hi = a.stride > 0 ? (out_hi - 1 + a.stride / 2) / a.stride + 1 : out_hi;
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= (col_hi - col_lo) * M) return;
    const long long col = col_lo + e / M;
    const int mu = (int)(e % M);
    const long long rowbase_in = (long long)s.row0 * a.r_in;
    const float* __restrict__ x = (const float*)a.x;
    const float* __restrict__ w = (const float*)a.w;

    float acc = 0.f;
    const int half = (a.ntaps - 1) / 2;
    for (int t = 0; t < a.ntaps; ++t) {
        const long long r = a.stride > 0 ? col - t : a.down > 0 ? col * a.down - a.down / 2 + t : col + (long long)(t - half) * a.dil;
        if (r < 0 || r >= nrows_in) continue;
        const float* xr = x + (size_t)(rowbase_in + r) * a.cin;
        const float* wt = w + (size_t)t * a.cin * M + mu;
        for (int i = 0; i < a.cin; ++i) acc = fmaf(wt[(size_t)i * M], xr[i], acc);
    }

    int o = mu;
    long long n = col;
    long long rowbase_out = a.down > 0 ? (long long)s.row0 * r_out : rowbase_in;
    if (a.stride > 0) {
        const int phi = mu / a.cout;
        o = mu - phi * a.cout;
        n = col * a.stride - a.stride / 2 + phi;
        if (n < 0 || n >= nrows_in * a.stride) return;
        rowbase_out = rowbase_in * a.stride;
    }
    float v = acc + a.bias[o];
    if (a.out_alpha) v = snake_precise(v, a.out_alpha[o], a.out_inv_beta[o]);
    const size_t idx = (size_t)(rowbase_out + n) * a.cout + o;
    if (a.res) v += ((const float*)a.res)[idx];
    ((float*)a.y)[idx] = v;
}

hipError_t launch_conv_f32(const ConvArgs& a, hipStream_t stream)
{
    const long long M = a.stride > 0 ? (long long)a.stride * a.cout : a.cout;
    if (a.down > 0 && (a.stride != 0 || a.ntaps != 2 * a.down || a.r_in % a.down != 0 || a.res)) return hipErrorInvalidValue;
    const long long r_out = a.down > 0 ? (long long)a.r_in / a.down : (long long)a.r_in * (a.stride > 0 ? a.stride : 1);
    const long long out_rows = std::min((long long)a.max_int * r_out + 2ll * a.margin, (long long)a.max_len * r_out);
    const long long ncols = a.stride > 0 ? out_rows / a.stride + 2 : out_rows;
    const long long blocks = (ncols * M + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_f32_kernel, dim3((unsigned)blocks, (unsigned)a.n_slots), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace demon
