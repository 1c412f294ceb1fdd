/*
 * CPU oracle of the VAE audio decoder behind the windowed decode (paper section 3.6).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, direct-sum loops over the textbook
 * definitions, in planar [channels, time] layout, no tiling, no windows, no code
 * shared with the HIP library.  Compiled twice: REAL=double (the parity oracle) and
 * REAL=float (the same loops in fp32, timed as the CPU baseline).
 *
 * The paper does not list the decoder's layers; the stack follows the benchmark
 * description: per upsample block Snake -> ConvTranspose1d(kernel 2s, stride s,
 * padding s/2) -> residual units [Snake -> Conv1d(k, dilation d) -> Snake ->
 * Conv1d(1) -> add]; head Snake -> Conv1d(k) -> tanh.
 *
 * Definitions (x is zero outside [0, L)):
 *   snake : y[c,n] = x[c,n] + sin(alpha_c x[c,n])^2 / (beta_c + 1e-9)
 *   conv  : y[o,n] = b[o] + sum_i sum_k W[o,i,k] x[i, n + (k - (K-1)/2) d]
 *   convT : y[o,n] = b[o] + sum_i sum_k W[i,o,k] x[i,m]  over (m,k) with m s - p + k = n,
 *           output length (L-1) s - 2p + K
 *   convS : y[o,n] = b[o] + sum_i sum_k W[o,i,k] x[i, n s - p + k],  output length floor((L + 2p - K)/s) + 1
 *           (the strided convolution of the encoder, the mirror of convT)
 *
 * The encoder (section 3.7 names separate encode and decode engines; Table III times the encode) is
 * the decoder's mirror: stem Conv1d(k) from the waveform, then per block, from the audio rate down,
 * the residual units followed by Snake -> strided Conv1d(kernel 2s, stride s, padding s/2); the last
 * strided convolution produces the moments (mean, log-variance) of the latent.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#if defined(ORACLE_F32)
typedef float REAL;
#define SFX(name) name##_f32
#define SIN sinf
#define TANH tanhf
#else
typedef double REAL;
#define SFX(name) name##_f64
#define SIN sin
#define TANH tanh
#endif

void SFX(oracle_snake)(const REAL* x, int C, long L, const REAL* alpha, const REAL* beta, REAL* y)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const REAL a = alpha[c];
        const REAL inv = (REAL)1 / (beta[c] + (REAL)1e-9);
        for (long n = 0; n < L; ++n) {
            const REAL v = x[(size_t)c * L + n];
            const REAL s = SIN(a * v);
            y[(size_t)c * L + n] = v + s * s * inv;
        }
    }
}

/* Conv1d, odd kernel K, dilation d, zero padding d (K-1)/2 on both sides: output length L. */
void SFX(oracle_conv1d)(const REAL* x, int Cin, long L, const REAL* W, const REAL* b,
                        int Cout, int K, int d, REAL* y)
{
    const int half = (K - 1) / 2;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Cout; ++o) {
        REAL* yo = y + (size_t)o * L;
        for (long n = 0; n < L; ++n) yo[n] = b ? b[o] : (REAL)0;
        for (int i = 0; i < Cin; ++i) {
            const REAL* xi = x + (size_t)i * L;
            for (int k = 0; k < K; ++k) {
                const REAL w = W[((size_t)o * Cin + i) * K + k];
                const long off = (long)(k - half) * d;     /* input index = n + off */
                long n0 = off < 0 ? -off : 0;
                long n1 = off > 0 ? L - off : L;
                for (long n = n0; n < n1; ++n) yo[n] += w * xi[n + off];
            }
        }
    }
}

/* ConvTranspose1d: weight [Cin, Cout, K], stride s, padding p; output length (L-1) s - 2p + K. */
void SFX(oracle_convT1d)(const REAL* x, int Cin, long L, const REAL* W, const REAL* b,
                         int Cout, int K, int s, int p, REAL* y)
{
    const long Lout = (L - 1) * s - 2 * p + K;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Cout; ++o) {
        REAL* yo = y + (size_t)o * Lout;
        for (long n = 0; n < Lout; ++n) yo[n] = b ? b[o] : (REAL)0;
        for (int i = 0; i < Cin; ++i) {
            const REAL* xi = x + (size_t)i * L;
            for (int k = 0; k < K; ++k) {
                const REAL w = W[((size_t)i * Cout + o) * K + k];
                for (long m = 0; m < L; ++m) {
                    const long n = m * s - p + k;
                    if (n >= 0 && n < Lout) yo[n] += w * xi[m];
                }
            }
        }
    }
}

void SFX(oracle_tanh)(const REAL* x, size_t n, REAL* y)
{
    for (size_t i = 0; i < n; ++i) y[i] = TANH(x[i]);
}

/*
 * Full decode of one clip.  `w` is the flat parameter array in the canonical order
 * (per block: up.alpha, up.beta, up.weight, up.bias, then per residual unit
 * a1.alpha, a1.beta, c1.weight, c1.bias, a2.alpha, a2.beta, c2.weight, c2.bias;
 * then head.alpha, head.beta, head.weight, head.bias).
 * latent [C0, T] -> out [out_channels, T * prod(strides)].  Returns 0, or -1 on a bad argument.
 */
int SFX(oracle_decode)(int C0, int nb, const int* strides, const int* widths,
                       int nres, const int* dilations, int res_kernel, int head_kernel,
                       int out_channels, const REAL* w, const REAL* latent, long T, REAL* out)
{
    if (nb <= 0 || T <= 0 || (res_kernel & 1) == 0 || (head_kernel & 1) == 0) return -1;
    for (int l = 0; l < nb; ++l) if (strides[l] <= 0 || (strides[l] & 1)) return -1;

    int C = C0;
    long L = T;
    REAL* h = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
    memcpy(h, latent, sizeof(REAL) * (size_t)C * L);

    for (int l = 0; l < nb; ++l) {
        const int s = strides[l], Cn = widths[l];
        const REAL* alpha = w;  w += C;
        const REAL* beta = w;   w += C;
        const REAL* Wt = w;     w += (size_t)C * Cn * 2 * s;
        const REAL* bt = w;     w += Cn;
        REAL* a = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
        SFX(oracle_snake)(h, C, L, alpha, beta, a);
        const long Ln = L * s;                      /* (L-1)s - 2(s/2) + 2s */
        REAL* hn = (REAL*)malloc(sizeof(REAL) * (size_t)Cn * Ln);
        SFX(oracle_convT1d)(a, C, L, Wt, bt, Cn, 2 * s, s, s / 2, hn);
        free(a); free(h);
        h = hn; C = Cn; L = Ln;

        REAL* t1 = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
        REAL* t2 = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
        for (int j = 0; j < nres; ++j) {
            const REAL* a1 = w;  w += C;
            const REAL* b1 = w;  w += C;
            const REAL* W1 = w;  w += (size_t)C * C * res_kernel;
            const REAL* c1 = w;  w += C;
            const REAL* a2 = w;  w += C;
            const REAL* b2 = w;  w += C;
            const REAL* W2 = w;  w += (size_t)C * C;
            const REAL* c2 = w;  w += C;
            SFX(oracle_snake)(h, C, L, a1, b1, t1);
            SFX(oracle_conv1d)(t1, C, L, W1, c1, C, res_kernel, dilations[j], t2);
            SFX(oracle_snake)(t2, C, L, a2, b2, t1);
            SFX(oracle_conv1d)(t1, C, L, W2, c2, C, 1, 1, t2);
            const size_t tot = (size_t)C * L;
            for (size_t e = 0; e < tot; ++e) h[e] = h[e] + t2[e];
        }
        free(t1); free(t2);
    }

    const REAL* ah = w;  w += C;
    const REAL* bh = w;  w += C;
    const REAL* Wh = w;  w += (size_t)out_channels * C * head_kernel;
    const REAL* ch = w;
    REAL* a = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
    SFX(oracle_snake)(h, C, L, ah, bh, a);
    SFX(oracle_conv1d)(a, C, L, Wh, ch, out_channels, head_kernel, 1, out);
    SFX(oracle_tanh)(out, (size_t)out_channels * L, out);
    free(a); free(h);
    return 0;
}

/* Strided Conv1d: weight [Cout, Cin, K], stride s, zero padding p on both sides;
 * output length floor((L + 2p - K)/s) + 1. */
void SFX(oracle_conv1d_strided)(const REAL* x, int Cin, long L, const REAL* W, const REAL* b,
                                int Cout, int K, int s, int p, REAL* y)
{
    const long Lout = (L + 2 * p - K) / s + 1;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Cout; ++o) {
        REAL* yo = y + (size_t)o * Lout;
        for (long n = 0; n < Lout; ++n) yo[n] = b ? b[o] : (REAL)0;
        for (int i = 0; i < Cin; ++i) {
            const REAL* xi = x + (size_t)i * L;
            for (int k = 0; k < K; ++k) {
                const REAL w = W[((size_t)o * Cin + i) * K + k];
                for (long n = 0; n < Lout; ++n) {
                    const long m = n * s - p + k;
                    if (m >= 0 && m < L) yo[n] += w * xi[m];
                }
            }
        }
    }
}

/*
 * Full encode of one clip to the moments of the latent.  The layer description is the decoder's
 * (strides, widths, dilations of its blocks 1..nb); the encoder walks it backwards.  `w` is the flat
 * parameter array in processing order: stem.weight [C_nb, in_channels, stem_kernel], stem.bias;
 * then for l = nb .. 1: per residual unit a1.alpha, a1.beta, c1.weight [C_l, C_l, res_kernel], c1.bias,
 * a2.alpha, a2.beta, c2.weight [C_l, C_l, 1], c2.bias; then down.alpha [C_l], down.beta [C_l],
 * down.weight [C_out, C_l, 2 s_l], down.bias [C_out] with C_out = C_{l-1}, and 2 C0 for l = 1.
 * wave [in_channels, T * prod(strides)] -> moments [2 C0, T] (rows 0..C0-1 mean, C0..2C0-1 log-variance).
 * Returns 0, or -1 on a bad argument.
 */
int SFX(oracle_encode)(int C0, int nb, const int* strides, const int* widths,
                       int nres, const int* dilations, int res_kernel, int stem_kernel,
                       int in_channels, const REAL* w, const REAL* wave, long T, REAL* moments)
{
    if (nb <= 0 || T <= 0 || (res_kernel & 1) == 0 || (stem_kernel & 1) == 0) return -1;
    long L = T;
    for (int l = 0; l < nb; ++l) { if (strides[l] <= 0 || (strides[l] & 1)) return -1; L *= strides[l]; }

    int C = widths[nb - 1];
    REAL* h = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
    {
        const REAL* Ws = w;  w += (size_t)C * in_channels * stem_kernel;
        const REAL* bs = w;  w += C;
        SFX(oracle_conv1d)(wave, in_channels, L, Ws, bs, C, stem_kernel, 1, h);
    }
    for (int l = nb - 1; l >= 0; --l) {
        const int s = strides[l];
        const int Cn = l > 0 ? widths[l - 1] : 2 * C0;
        REAL* t1 = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
        REAL* t2 = (REAL*)malloc(sizeof(REAL) * (size_t)C * L);
        for (int j = 0; j < nres; ++j) {
            const REAL* a1 = w;  w += C;
            const REAL* b1 = w;  w += C;
            const REAL* W1 = w;  w += (size_t)C * C * res_kernel;
            const REAL* c1 = w;  w += C;
            const REAL* a2 = w;  w += C;
            const REAL* b2 = w;  w += C;
            const REAL* W2 = w;  w += (size_t)C * C;
            const REAL* c2 = w;  w += C;
            SFX(oracle_snake)(h, C, L, a1, b1, t1);
            SFX(oracle_conv1d)(t1, C, L, W1, c1, C, res_kernel, dilations[j], t2);
            SFX(oracle_snake)(t2, C, L, a2, b2, t1);
            SFX(oracle_conv1d)(t1, C, L, W2, c2, C, 1, 1, t2);
            const size_t tot = (size_t)C * L;
            for (size_t e = 0; e < tot; ++e) h[e] = h[e] + t2[e];
        }
        const REAL* ad = w;  w += C;
        const REAL* bd = w;  w += C;
        const REAL* Wd = w;  w += (size_t)Cn * C * 2 * s;
        const REAL* cd = w;  w += Cn;
        SFX(oracle_snake)(h, C, L, ad, bd, t1);
        const long Ln = L / s;                      /* floor((L + s - 2s)/s) + 1 for s | L */
        REAL* hn = l > 0 ? (REAL*)malloc(sizeof(REAL) * (size_t)Cn * Ln) : moments;
        SFX(oracle_conv1d_strided)(t1, C, L, Wd, cd, Cn, 2 * s, s, s / 2, hn);
        free(t1); free(t2); free(h);
        h = hn; C = Cn; L = Ln;
    }
    return 0;
}
