// Host-side logic of libdemon_vae that needs no GPU: layer-stack validation, the analytic
// receptive field, the window grid and the thread-local error message.
#include <stdarg.h>
#include <stdio.h>

#include "internal.h"

namespace demon {

static thread_local char g_err[512] = "";

demon_status fail(demon_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

void clear_error() { g_err[0] = 0; }

demon_status stack_from_config(const demon_vae_config* cfg, Stack* out)
{
    if (!cfg) return fail(DEMON_ERR_INVALID_ARG, "config is NULL");
    if (cfg->latent_channels < 1) return fail(DEMON_ERR_INVALID_ARG, "latent_channels must be >= 1");
    if (cfg->n_blocks < 1 || cfg->n_blocks > 16) return fail(DEMON_ERR_INVALID_ARG, "n_blocks must be in 1..16");
    if (!cfg->strides || !cfg->widths) return fail(DEMON_ERR_INVALID_ARG, "strides/widths is NULL");
    if (cfg->n_res < 0 || cfg->n_res > 8) return fail(DEMON_ERR_INVALID_ARG, "n_res must be in 0..8");
    if (cfg->n_res > 0 && !cfg->dilations) return fail(DEMON_ERR_INVALID_ARG, "dilations is NULL");
    if (cfg->res_kernel < 1 || (cfg->res_kernel & 1) == 0) return fail(DEMON_ERR_INVALID_ARG, "res_kernel must be odd");
    if (cfg->head_kernel < 1 || (cfg->head_kernel & 1) == 0) return fail(DEMON_ERR_INVALID_ARG, "head_kernel must be odd");
    if (cfg->out_channels < 1 || cfg->out_channels > 8) return fail(DEMON_ERR_INVALID_ARG, "out_channels must be in 1..8");
    Stack st;
    st.c0 = cfg->latent_channels;
    long long total = 1;
    for (int l = 0; l < cfg->n_blocks; ++l) {
        const int s = cfg->strides[l], c = cfg->widths[l];
        if (s < 2 || (s & 1)) return fail(DEMON_ERR_INVALID_ARG, "stride %d of block %d must be even and >= 2 (padding s/2)", s, l);
        if (c < 1) return fail(DEMON_ERR_INVALID_ARG, "width of block %d must be >= 1", l);
        total *= s;
        if (total > (1 << 20)) return fail(DEMON_ERR_INVALID_ARG, "total upsampling factor too large");
        st.strides.push_back(s);
        st.widths.push_back(c);
    }
    for (int j = 0; j < cfg->n_res; ++j) {
        if (cfg->dilations[j] < 1) return fail(DEMON_ERR_INVALID_ARG, "dilation %d must be >= 1", j);
        st.dilations.push_back(cfg->dilations[j]);
    }
    st.res_kernel = cfg->res_kernel;
    st.head_kernel = cfg->head_kernel;
    st.out_channels = cfg->out_channels;
    *out = st;
    return DEMON_OK;
}

size_t stack_weight_count(const Stack& st)
{
    size_t n = 0;
    size_t cin = (size_t)st.c0;
    for (size_t l = 0; l < st.strides.size(); ++l) {
        const size_t c = (size_t)st.widths[l], s = (size_t)st.strides[l];
        n += 2 * cin + cin * c * 2 * s + c;
        n += st.dilations.size() * (2 * c + c * c * (size_t)st.res_kernel + c + 2 * c + c * c + c);
        cin = c;
    }
    n += 2 * cin + (size_t)st.out_channels * cin * (size_t)st.head_kernel + (size_t)st.out_channels;
    return n;
}

// Encoder (the decoder's mirror): stem conv [C_nb, channels, k] + bias; per block, from the audio rate down, the residual
// units of width C_l and Snake + strided conv [C_out, C_l, 2 s_l] + bias, C_out = C_{l-1}, and 2 C0 (the moments) for l = 1.
size_t stack_encoder_weight_count(const Stack& st)
{
    const size_t nb = st.strides.size();
    size_t n = (size_t)st.widths[nb - 1] * st.out_channels * st.head_kernel + (size_t)st.widths[nb - 1];
    for (size_t l = nb; l-- > 0;) {
        const size_t c = (size_t)st.widths[l], s = (size_t)st.strides[l];
        const size_t cn = l > 0 ? (size_t)st.widths[l - 1] : 2 * (size_t)st.c0;
        n += st.dilations.size() * (2 * c + c * c * (size_t)st.res_kernel + c + 2 * c + c * c + c);
        n += 2 * c + cn * c * 2 * s + cn;
    }
    return n;
}

static long long floor_div(long long a, long long b) { long long q = a / b; return (a % b != 0 && ((a < 0) != (b < 0))) ? q - 1 : q; }
static long long ceil_div(long long a, long long b) { return -floor_div(-a, b); }

// Backward interval propagation, last layer first.
static void backward(const Stack& st, long long a, long long b, long long* lo, long long* hi)
{
    const long long rh = (st.head_kernel - 1) / 2;
    a -= rh; b += rh;
    for (int l = (int)st.strides.size() - 1; l >= 0; --l) {
        for (int j = (int)st.dilations.size() - 1; j >= 0; --j) {
            const long long r = (long long)st.dilations[j] * ((st.res_kernel - 1) / 2);
            a -= r; b += r;
        }
        const long long s = st.strides[l], k = 2 * s, p = s / 2;
        // output n takes input m when 0 <= n + p - m s <= k - 1
        a = ceil_div(a + p - k + 1, s);
        b = floor_div(b + p, s);
    }
    *lo = a; *hi = b;
}

void stack_receptive_field(const Stack& st, int* left, int* right)
{
    const long long S = st.total_stride();
    const long long f = 4096;                     // any frame: the stack is shift-invariant
    long long lo, hi;
    backward(st, f * S, (f + 1) * S - 1, &lo, &hi);
    *left = (int)(f - lo);
    *right = (int)(hi - f);
}

// Waveform samples [*lo, *hi] that latent frames [a, b] of the encoder depend on: backwards from the moments, a strided
// conv (kernel 2s, stride s, padding s/2) reads inputs n s - s/2 .. n s + 3s/2 - 1 for output n, an odd conv of
// dilation d reaches d (k-1)/2 further on both sides.
static void encoder_backward(const Stack& st, long long a, long long b, long long* lo, long long* hi)
{
    for (size_t l = 0; l < st.strides.size(); ++l) {
        const long long s = st.strides[l];
        a = a * s - s / 2;
        b = b * s + 3 * s / 2 - 1;
        for (int d : st.dilations) {
            const long long r = (long long)d * ((st.res_kernel - 1) / 2);
            a -= r; b += r;
        }
    }
    const long long rh = (st.head_kernel - 1) / 2;
    *lo = a - rh; *hi = b + rh;
}

void stack_encoder_receptive_field(const Stack& st, int* left, int* right, long long* samples_left, long long* samples_right)
{
    const long long S = st.total_stride();
    const long long f = 4096;
    long long lo, hi;
    encoder_backward(st, f, f, &lo, &hi);
    const long long sl = f * S - lo, sr = hi - (f * S + S - 1);       // samples before the frame's first / after its last
    if (samples_left) *samples_left = sl;
    if (samples_right) *samples_right = sr;
    *left = (int)((sl + S - 1) / S);
    *right = (int)((sr + S - 1) / S);
}

void stack_forward_support(const Stack& st, long long a, long long b, long long* lo, long long* hi)
{
    for (size_t l = 0; l < st.strides.size(); ++l) {
        const long long s = st.strides[l], k = 2 * s, p = s / 2;
        a = a * s - p;
        b = b * s - p + k - 1;
        for (int d : st.dilations) {
            const long long r = (long long)d * ((st.res_kernel - 1) / 2);
            a -= r; b += r;
        }
    }
    const long long rh = (st.head_kernel - 1) / 2;
    *lo = a - rh; *hi = b + rh;
}

}  // namespace demon

using namespace demon;

extern "C" {

const char* demon_vae_last_error(void) { return g_err; }

size_t demon_vae_weight_count(const demon_vae_config* cfg)
{
    Stack st;
    if (stack_from_config(cfg, &st) != DEMON_OK) return 0;
    return stack_weight_count(st);
}

size_t demon_vae_encoder_weight_count(const demon_vae_config* cfg)
{
    Stack st;
    if (stack_from_config(cfg, &st) != DEMON_OK) return 0;
    return stack_encoder_weight_count(st);
}

demon_status demon_vae_encoder_rf_from_config(const demon_vae_config* cfg, int* halo_left, int* halo_right,
                                              long long* samples_left, long long* samples_right)
{
    if (!halo_left || !halo_right) return fail(DEMON_ERR_INVALID_ARG, "output pointer is NULL");
    Stack st;
    demon_status rc = stack_from_config(cfg, &st);
    if (rc != DEMON_OK) return rc;
    stack_encoder_receptive_field(st, halo_left, halo_right, samples_left, samples_right);
    return DEMON_OK;
}

demon_status demon_vae_rf_from_config(const demon_vae_config* cfg, int* halo_left, int* halo_right)
{
    if (!halo_left || !halo_right) return fail(DEMON_ERR_INVALID_ARG, "output pointer is NULL");
    Stack st;
    demon_status rc = stack_from_config(cfg, &st);
    if (rc != DEMON_OK) return rc;
    stack_receptive_field(st, halo_left, halo_right);
    return DEMON_OK;
}

demon_status demon_vae_forward_support(const demon_vae_config* cfg, int frame_a, int frame_b,
                                       long long* lo, long long* hi)
{
    if (!lo || !hi) return fail(DEMON_ERR_INVALID_ARG, "output pointer is NULL");
    if (frame_b < frame_a) return fail(DEMON_ERR_INVALID_ARG, "frame_b < frame_a");
    Stack st;
    demon_status rc = stack_from_config(cfg, &st);
    if (rc != DEMON_OK) return rc;
    stack_forward_support(st, frame_a, frame_b, lo, hi);
    return DEMON_OK;
}

demon_status demon_vae_plan_windows(int n_clips, int n_frames, int frame_begin, int frame_end,
                                    int window, int halo, demon_window* out, int capacity,
                                    int* n_windows)
{
    if (!n_windows) return fail(DEMON_ERR_INVALID_ARG, "n_windows is NULL");
    if (n_clips < 1) return fail(DEMON_ERR_INVALID_ARG, "n_clips must be >= 1");
    if (n_frames < 1) return fail(DEMON_ERR_INVALID_ARG, "n_frames must be >= 1");
    if (frame_begin < 0) return fail(DEMON_ERR_INVALID_ARG, "frame_begin must be >= 0");
    if (frame_end > n_frames) return fail(DEMON_ERR_INVALID_ARG, "frame_end %d exceeds n_frames %d", frame_end, n_frames);
    if (frame_begin >= frame_end) return fail(DEMON_ERR_INVALID_ARG, "empty frame range [%d, %d)", frame_begin, frame_end);
    if (window < 1) return fail(DEMON_ERR_INVALID_ARG, "window must be >= 1");
    if (halo < 0) return fail(DEMON_ERR_INVALID_ARG, "halo must be >= 0");
    long long count = 0;
    for (int c = 0; c < n_clips; ++c) {
        for (long long b = frame_begin; b < frame_end; b += window) {
            const long long e = b + window < frame_end ? b + window : frame_end;
            if (out && count < capacity) {
                demon_window w;
                w.clip = c;
                w.begin = (int)b;
                w.end = (int)e;
                w.lo = (int)(b - halo > 0 ? b - halo : 0);
                w.hi = (int)(e + halo < n_frames ? e + halo : n_frames);
                out[count] = w;
            }
            ++count;
            if (count > (1ll << 30)) return fail(DEMON_ERR_INVALID_ARG, "too many windows");
        }
    }
    *n_windows = (int)count;
    return DEMON_OK;
}

}  // extern "C"
