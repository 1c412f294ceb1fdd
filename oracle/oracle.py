"""Python face of the CPU oracle (ctypes over oracle/liboracle.so).  TEST INFRASTRUCTURE ONLY.

Everything is planar [channels, time].  `dtype=np.float64` (default) is the parity
oracle; `np.float32` runs the same loops in single precision (the timed CPU baseline).

Windowed decode follows the three steps of paper section 3.6: extend the target
window by a margin on both sides, decode the extended region as if it were a whole
clip, trim the margins so that only the frame-aligned interior remains
(prod(strides) samples per latent frame; 1920 at 48 kHz).

The receptive field is derived analytically by propagating index intervals through
the layer stack (the paper measures it empirically for the trained model; section
3.6 gives 8.3 frames for that model, which has a different stack).
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Tuple

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = ctypes.CDLL(path)
    return _LIB


def omp_threads() -> int:
    """Number of OpenMP threads the oracle's loops will use."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    return len(os.sched_getaffinity(0))


def _sfx(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float64:
        return "_f64", ctypes.c_double
    if dtype == np.float32:
        return "_f32", ctypes.c_float
    raise TypeError(dtype)


def _ptr(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def snake(x, alpha, beta, dtype=np.float64):
    sfx, ct = _sfx(dtype)
    x = np.ascontiguousarray(x, dtype=dtype)
    alpha = np.ascontiguousarray(alpha, dtype=dtype)
    beta = np.ascontiguousarray(beta, dtype=dtype)
    C, L = x.shape
    y = np.empty_like(x)
    getattr(_lib(), "oracle_snake" + sfx)(_ptr(x, ct), C, ctypes.c_long(L), _ptr(alpha, ct),
                                          _ptr(beta, ct), _ptr(y, ct))
    return y


def conv1d(x, W, b, dilation=1, dtype=np.float64):
    """Conv1d with odd kernel and zero 'same' padding; W [Cout, Cin, K]."""
    sfx, ct = _sfx(dtype)
    x = np.ascontiguousarray(x, dtype=dtype)
    W = np.ascontiguousarray(W, dtype=dtype)
    b = None if b is None else np.ascontiguousarray(b, dtype=dtype)
    Cin, L = x.shape
    Cout, Cin2, K = W.shape
    assert Cin == Cin2 and K % 2 == 1
    y = np.empty((Cout, L), dtype=dtype)
    getattr(_lib(), "oracle_conv1d" + sfx)(_ptr(x, ct), Cin, ctypes.c_long(L), _ptr(W, ct), _ptr(b, ct),
                                           Cout, K, int(dilation), _ptr(y, ct))
    return y


def convT1d(x, W, b, stride, padding, dtype=np.float64):
    """ConvTranspose1d; W [Cin, Cout, K]; output length (L-1) stride - 2 padding + K."""
    sfx, ct = _sfx(dtype)
    x = np.ascontiguousarray(x, dtype=dtype)
    W = np.ascontiguousarray(W, dtype=dtype)
    b = None if b is None else np.ascontiguousarray(b, dtype=dtype)
    Cin, L = x.shape
    Cin2, Cout, K = W.shape
    assert Cin == Cin2
    Lout = (L - 1) * stride - 2 * padding + K
    y = np.empty((Cout, Lout), dtype=dtype)
    getattr(_lib(), "oracle_convT1d" + sfx)(_ptr(x, ct), Cin, ctypes.c_long(L), _ptr(W, ct), _ptr(b, ct),
                                            Cout, K, int(stride), int(padding), _ptr(y, ct))
    return y


def conv1d_strided(x, W, b, stride, padding, dtype=np.float64):
    """Strided Conv1d; W [Cout, Cin, K]; output length floor((L + 2 padding - K) / stride) + 1."""
    sfx, ct = _sfx(dtype)
    x = np.ascontiguousarray(x, dtype=dtype)
    W = np.ascontiguousarray(W, dtype=dtype)
    b = None if b is None else np.ascontiguousarray(b, dtype=dtype)
    Cin, L = x.shape
    Cout, Cin2, K = W.shape
    assert Cin == Cin2 and L + 2 * padding >= K
    Lout = (L + 2 * padding - K) // stride + 1
    y = np.empty((Cout, Lout), dtype=dtype)
    getattr(_lib(), "oracle_conv1d_strided" + sfx)(_ptr(x, ct), Cin, ctypes.c_long(L), _ptr(W, ct), _ptr(b, ct),
                                                   Cout, K, int(stride), int(padding), _ptr(y, ct))
    return y


def decode(spec, weights, latent, dtype=np.float64):
    """Full decode.  latent [C0, T] or [n_clips, C0, T] -> [.., out_channels, T * S]."""
    latent = np.asarray(latent)
    if latent.ndim == 3:
        return np.stack([decode(spec, weights, z, dtype) for z in latent])
    sfx, ct = _sfx(dtype)
    w = np.ascontiguousarray(weights, dtype=dtype)
    z = np.ascontiguousarray(latent, dtype=dtype)
    C0, T = z.shape
    assert C0 == spec.latent_channels
    S = spec.total_stride
    out = np.empty((spec.out_channels, T * S), dtype=dtype)
    IntArr = lambda v: (ctypes.c_int * len(v))(*v)
    rc = getattr(_lib(), "oracle_decode" + sfx)(
        C0, len(spec.strides), IntArr(spec.strides), IntArr(spec.widths),
        len(spec.dilations), IntArr(spec.dilations), spec.res_kernel, spec.head_kernel,
        spec.out_channels, _ptr(w, ct), _ptr(z, ct), ctypes.c_long(T), _ptr(out, ct))
    if rc != 0:
        raise ValueError("oracle_decode rejected the decoder description")
    return out


def window_grid(frame_begin: int, frame_end: int, window: int) -> List[Tuple[int, int]]:
    """Windows start at frame_begin and step by `window`; the last may be short."""
    return [(b, min(b + window, frame_end)) for b in range(frame_begin, frame_end, window)]


def decode_windowed(spec, weights, latent, window, halo, frame_begin=0, frame_end=None,
                    dtype=np.float64):
    """Windowed decode of frames [frame_begin, frame_end): returns [.., out_channels, (end-begin) S]."""
    latent = np.asarray(latent)
    if latent.ndim == 3:
        return np.stack([decode_windowed(spec, weights, z, window, halo, frame_begin, frame_end, dtype)
                         for z in latent])
    T = latent.shape[1]
    if frame_end is None:
        frame_end = T
    S = spec.total_stride
    pieces = []
    for b, e in window_grid(frame_begin, frame_end, window):
        lo, hi = max(0, b - halo), min(T, e + halo)          # step 1: extend by the margins
        y = decode(spec, weights, latent[:, lo:hi], dtype)   # step 2: decode the extended region
        pieces.append(y[:, (b - lo) * S:(e - lo) * S])       # step 3: trim to the frame-aligned interior
    return np.concatenate(pieces, axis=1)


# ---------------------------------------------------------------- receptive field (analytic)

def _layers(spec):
    """(kind, kernel, stride_or_dilation, padding) of every layer that moves indices, input to output."""
    out = []
    for s in spec.strides:
        out.append(("convT", 2 * s, s, s // 2))
        for d in spec.dilations:
            out.append(("conv", spec.res_kernel, d, 0))
    out.append(("conv", spec.head_kernel, 1, 0))
    return out


def backward_interval(spec, a: int, b: int) -> Tuple[int, int]:
    """Latent frames [lo, hi] that output samples [a, b] depend on (clip edges ignored)."""
    for kind, K, sd, p in reversed(_layers(spec)):
        if kind == "conv":
            r = sd * (K - 1) // 2
            a, b = a - r, b + r
        else:
            # output n takes input m when 0 <= n + p - m s <= K - 1
            a, b = -((-(a + p - K + 1)) // sd), (b + p) // sd
    return a, b


def forward_interval(spec, a: int, b: int) -> Tuple[int, int]:
    """Output samples [lo, hi] that latent frames [a, b] can influence (clip edges ignored)."""
    for kind, K, sd, p in _layers(spec):
        if kind == "conv":
            r = sd * (K - 1) // 2
            a, b = a - r, b + r
        else:
            a, b = a * sd - p, b * sd - p + K - 1
    return a, b


def receptive_field(spec) -> Tuple[int, int]:
    """(halo_left, halo_right) in latent frames: context one output frame needs on each side."""
    S = spec.total_stride
    f = 1000                                   # any frame; the stack is shift-invariant
    lo, hi = backward_interval(spec, f * S, (f + 1) * S - 1)
    return f - lo, hi - f


def pcm16(y, dtype=np.float32):
    """16-bit render of a planar waveform y [channels, samples] -> int16 [samples, channels] (interleaved).

    Section 3.6 judges the windowed decode on its 16-bit PCM render.  The paper does not print the quantiser;
    the reading taken here is the symmetric one, q = round_half_even(32767 * clamp(y, -1, 1)), evaluated in
    single precision by default because the product's rounding decides the integer.
    """
    y = np.asarray(y).astype(dtype)
    v = np.clip(y, dtype(-1), dtype(1)) * dtype(32767)
    return np.rint(v).astype(np.int16).T.copy()


def latent_mse(curr, prev):
    """Mean squared difference of two latents of equal shape, in double precision: the quantity the latent
    similarity filter (section 3.5) compares with its threshold."""
    a = np.asarray(curr, dtype=np.float64)
    b = np.asarray(prev, dtype=np.float64)
    assert a.shape == b.shape and a.size > 0
    d = a - b
    return float(np.sum(d * d) / d.size)


def latent_unchanged(curr, prev, threshold=1e-3):
    """Gate of the similarity filter: True means the decode is skipped and the previous audio is reused."""
    return latent_mse(curr, prev) < threshold


def decode_gated(spec, weights, curr, prev, prev_audio, window, halo, threshold=1e-3):
    """The decode behind the similarity filter (section 3.5), clip by clip: a clip whose latent moved by less than
    the threshold keeps its previous audio, every other clip is decoded (windowed, section 3.6).
    curr, prev: [n_clips, C, T]; prev_audio: [n_clips, out_channels, T * total_stride].  Returns (audio, skipped)."""
    out = np.array(prev_audio, dtype=np.float64, copy=True)
    skipped = []
    for c in range(len(curr)):
        skip = latent_unchanged(curr[c], prev[c], threshold)
        skipped.append(bool(skip))
        if not skip:
            out[c] = decode_windowed(spec, weights, curr[c], window=window, halo=halo)
    return out, skipped


def crossfade(prev_tail, next_head):
    """Equal-power crossfade of two [channels, N] segments that overlap in time (the chunk boundary of the
    playback stream; the paper names a 50 ms equal-power crossfade without printing the gain curve).  Reading
    taken here: quarter-sine gains sampled at the sample midpoints, theta_n = (pi/2)(n + 1/2)/N,
    out = cos(theta) * prev_tail + sin(theta) * next_head, so that the squared gains sum to one everywhere."""
    a = np.asarray(prev_tail, dtype=np.float64)
    b = np.asarray(next_head, dtype=np.float64)
    assert a.shape == b.shape and a.ndim == 2
    n = a.shape[1]
    theta = (np.pi / 2) * (np.arange(n) + 0.5) / n
    return np.cos(theta)[None, :] * a + np.sin(theta)[None, :] * b


# ---------------------------------------------------------------- encoder (the mirror path)

def encode_moments(spec, enc_weights, wave, dtype=np.float64):
    """Full encode to the latent's moments.  wave [channels, T * S] or [n_clips, channels, T * S] ->
    [.., 2 C0, T]: rows 0..C0-1 the mean, rows C0..2C0-1 the log-variance.  The encoder is the decoder's mirror
    (section 3.7 only names the encode engine): stem conv from the waveform, then per block from the audio rate
    down the residual units and Snake -> strided conv (kernel 2s, stride s, padding s/2)."""
    wave = np.asarray(wave)
    if wave.ndim == 3:
        return np.stack([encode_moments(spec, enc_weights, x, dtype) for x in wave])
    sfx, ct = _sfx(dtype)
    w = np.ascontiguousarray(enc_weights, dtype=dtype)
    x = np.ascontiguousarray(wave, dtype=dtype)
    ch, n = x.shape
    S = spec.total_stride
    assert ch == spec.out_channels and n % S == 0 and n > 0
    T = n // S
    out = np.empty((2 * spec.latent_channels, T), dtype=dtype)
    IntArr = lambda v: (ctypes.c_int * max(len(v), 1))(*v)
    rc = getattr(_lib(), "oracle_encode" + sfx)(
        spec.latent_channels, len(spec.strides), IntArr(spec.strides), IntArr(spec.widths),
        len(spec.dilations), IntArr(spec.dilations), spec.res_kernel, spec.head_kernel,
        spec.out_channels, _ptr(w, ct), _ptr(x, ct), ctypes.c_long(T), _ptr(out, ct))
    if rc != 0:
        raise ValueError("oracle_encode rejected the encoder description")
    return out


def sample_latent(moments, eps):
    """The sampling step on the output moments (Table III's note names it, no formula is printed).  Reading taken
    here, the usual diagonal-Gaussian posterior: z = mean + exp(logvar / 2) * eps, eps ~ N(0, 1) drawn by the caller."""
    m = np.asarray(moments, dtype=np.float64)
    c0 = m.shape[-2] // 2
    mean, logvar = m[..., :c0, :], m[..., c0:, :]
    return mean + np.exp(0.5 * logvar) * np.asarray(eps, dtype=np.float64)


def encode_moments_windowed(spec, enc_weights, wave, window, halo, frame_begin=0, frame_end=None, dtype=np.float64):
    """Windowed encode of latent frames [frame_begin, frame_end): the three steps of section 3.6 in the other
    direction -- extend the window's samples by `halo` frames of samples on both sides (clamped to the clip), encode
    the extended region as if it were a whole clip, trim the halo frames.  Returns [.., 2 C0, frame_end - frame_begin]."""
    wave = np.asarray(wave)
    if wave.ndim == 3:
        return np.stack([encode_moments_windowed(spec, enc_weights, x, window, halo, frame_begin, frame_end, dtype)
                         for x in wave])
    S = spec.total_stride
    T = wave.shape[1] // S
    if frame_end is None:
        frame_end = T
    pieces = []
    for b, e in window_grid(frame_begin, frame_end, window):
        lo, hi = max(0, b - halo), min(T, e + halo)
        m = encode_moments(spec, enc_weights, wave[:, lo * S:hi * S], dtype)
        pieces.append(m[:, b - lo:e - lo])
    return np.concatenate(pieces, axis=1)


def _encoder_layers(spec):
    """(kind, kernel, stride_or_dilation, padding) of the encoder's index-moving layers, input to output."""
    out = [("conv", spec.head_kernel, 1, 0)]
    for s in reversed(spec.strides):
        for d in spec.dilations:
            out.append(("conv", spec.res_kernel, d, 0))
        out.append(("convS", 2 * s, s, s // 2))
    return out


def encoder_backward_interval(spec, a: int, b: int) -> Tuple[int, int]:
    """Waveform samples [lo, hi] that latent frames [a, b] depend on (clip edges ignored): a strided conv reads
    inputs n s - p .. n s - p + K - 1 for output n, an odd conv of dilation d reaches d (K-1)/2 further."""
    for kind, K, sd, p in reversed(_encoder_layers(spec)):
        if kind == "conv":
            r = sd * (K - 1) // 2
            a, b = a - r, b + r
        else:
            a, b = a * sd - p, b * sd - p + K - 1
    return a, b


def encoder_forward_interval(spec, a: int, b: int) -> Tuple[int, int]:
    """Latent frames [lo, hi] that waveform samples [a, b] can influence (clip edges ignored)."""
    for kind, K, sd, p in _encoder_layers(spec):
        if kind == "conv":
            r = sd * (K - 1) // 2
            a, b = a - r, b + r
        else:
            # output n reads input m when 0 <= m - n s + p <= K - 1
            a, b = -((-(a + p - K + 1)) // sd), (b + p) // sd
    return a, b


def encoder_receptive_field(spec) -> Tuple[int, int]:
    """(halo_left, halo_right) of the windowed encode in latent frames: how many frames' worth of samples before and
    after a frame its moments depend on."""
    S = spec.total_stride
    f = 1000
    lo, hi = encoder_backward_interval(spec, f, f)
    return -((lo - f * S) // S), (hi - (f * S + S - 1) + S - 1) // S
