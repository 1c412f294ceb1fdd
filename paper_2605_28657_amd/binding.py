"""Thin ctypes binding of include/demon_vae.h: argument marshalling only.

Every step of the decode runs in the HIP library; PyTorch supplies device memory and
streams.  There is no fallback: if libdemon_vae.so cannot be loaded (and cannot be
built because hipcc is absent) importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdemon_vae.so")

DEMON_OK, DEMON_ERR_INVALID_ARG, DEMON_ERR_UNSUPPORTED, DEMON_ERR_WORKSPACE, DEMON_ERR_HIP = range(5)
DEMON_F32, DEMON_BF16 = 0, 1
_STATUS_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE", 4: "HIP"}


class DemonError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"demon_vae: {_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


class _Config(ctypes.Structure):
    _fields_ = [("latent_channels", ctypes.c_int), ("n_blocks", ctypes.c_int),
                ("strides", ctypes.POINTER(ctypes.c_int)), ("widths", ctypes.POINTER(ctypes.c_int)),
                ("n_res", ctypes.c_int), ("dilations", ctypes.POINTER(ctypes.c_int)),
                ("res_kernel", ctypes.c_int), ("head_kernel", ctypes.c_int), ("out_channels", ctypes.c_int),
                ("dtype", ctypes.c_int), ("max_frames", ctypes.c_int), ("max_clips", ctypes.c_int),
                ("max_extended_frames", ctypes.c_longlong),
                ("wide_operands", ctypes.c_int), ("flags", ctypes.c_int), ("small_tile_wgs", ctypes.c_int)]

DEMON_VAE_FLAG_NO_FUSED, DEMON_VAE_FLAG_ONE_STREAM, DEMON_VAE_FLAG_NO_WIDE_TILE, DEMON_VAE_FLAG_NO_HEAD_FUSION = 1, 2, 4, 8


class _Window(ctypes.Structure):
    _fields_ = [("clip", ctypes.c_int), ("begin", ctypes.c_int), ("end", ctypes.c_int),
                ("lo", ctypes.c_int), ("hi", ctypes.c_int)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libdemon_vae.so (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER
    lib.demon_vae_weight_count.restype = ctypes.c_size_t
    lib.demon_vae_weight_count.argtypes = [P(_Config)]
    lib.demon_vae_rf_from_config.argtypes = [P(_Config), P(ctypes.c_int), P(ctypes.c_int)]
    lib.demon_vae_forward_support.argtypes = [P(_Config), ctypes.c_int, ctypes.c_int, P(ctypes.c_longlong), P(ctypes.c_longlong)]
    lib.demon_vae_plan_windows.argtypes = [ctypes.c_int] * 6 + [P(_Window), ctypes.c_int, P(ctypes.c_int)]
    lib.demon_vae_create.argtypes = [P(_Config), P(ctypes.c_float), ctypes.c_size_t, P(ctypes.c_void_p)]
    lib.demon_vae_destroy.argtypes = [ctypes.c_void_p]
    lib.demon_vae_destroy.restype = None
    lib.demon_vae_receptive_field.argtypes = [ctypes.c_void_p, P(ctypes.c_int), P(ctypes.c_int)]
    lib.demon_vae_decode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.demon_vae_decode_windowed.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p]
    lib.demon_vae_decode_windowed_pcm16.argtypes = lib.demon_vae_decode_windowed.argtypes
    lib.demon_vae_decode_windowed_static.argtypes = lib.demon_vae_decode_windowed.argtypes
    lib.demon_vae_decode_windowed_gated.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 6 + [ctypes.c_void_p] * 3
    lib.demon_vae_encoder_weight_count.restype = ctypes.c_size_t
    lib.demon_vae_encoder_weight_count.argtypes = [P(_Config)]
    lib.demon_vae_encoder_rf_from_config.argtypes = [P(_Config), P(ctypes.c_int), P(ctypes.c_int), P(ctypes.c_longlong), P(ctypes.c_longlong)]
    lib.demon_vae_create_encoder.argtypes = lib.demon_vae_create.argtypes
    lib.demon_vae_encode_windowed.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 6 + [ctypes.c_void_p] * 4
    lib.demon_vae_encode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int] + [ctypes.c_void_p] * 4
    lib.demon_vae_latent_similarity.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_int,
                                                ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.demon_vae_crossfade.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p, ctypes.c_longlong,
                                        ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    lib.demon_vae_debug_tap.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t]
    lib.demon_vae_set_timing.argtypes = [ctypes.c_void_p, ctypes.c_int]
    lib.demon_vae_get_timing.argtypes = [ctypes.c_void_p, P(ctypes.c_float), ctypes.c_int, P(ctypes.c_int)]
    lib.demon_vae_last_error.restype = ctypes.c_char_p
    lib.demon_vae_last_error.argtypes = []
    _lib = lib
    return lib


def demon_vae_last_error() -> str:
    return load_library().demon_vae_last_error().decode()


def _check(status: int):
    if status != DEMON_OK:
        raise DemonError(status, demon_vae_last_error())


def _make_config(latent_channels: int, strides: Sequence[int], widths: Sequence[int], dilations: Sequence[int],
                 res_kernel: int, head_kernel: int, out_channels: int, dtype: int = DEMON_F32,
                 max_frames: int = 1, max_clips: int = 1, max_extended_frames: int = 0,
                 wide_operands: int = 0, flags: int = 0, small_tile_wgs: int = 0):
    """Returns (config struct, keep-alive tuple of the int arrays it points to)."""
    s = (ctypes.c_int * max(len(strides), 1))(*strides)
    w = (ctypes.c_int * max(len(widths), 1))(*widths)
    d = (ctypes.c_int * max(len(dilations), 1))(*dilations)
    if len(strides) != len(widths):
        raise ValueError("strides and widths differ in length")
    cfg = _Config(latent_channels, len(strides), s, w, len(dilations), d, res_kernel, head_kernel, out_channels,
                  dtype, max_frames, max_clips, max_extended_frames, wide_operands, flags, small_tile_wgs)
    return cfg, (s, w, d)


def config_from_spec(spec, dtype: int = DEMON_F32, max_frames: int = 1, max_clips: int = 1,
                     max_extended_frames: int = 0, wide_operands: int = 0, flags: int = 0, small_tile_wgs: int = 0):
    """Config from any object with latent_channels/strides/widths/dilations/res_kernel/head_kernel/out_channels."""
    return _make_config(spec.latent_channels, spec.strides, spec.widths, spec.dilations, spec.res_kernel,
                        spec.head_kernel, spec.out_channels, dtype, max_frames, max_clips, max_extended_frames,
                        wide_operands, flags, small_tile_wgs)


def demon_vae_weight_count(spec) -> int:
    cfg, _keep = config_from_spec(spec)
    return int(load_library().demon_vae_weight_count(ctypes.byref(cfg)))


def demon_vae_rf_from_config(spec) -> Tuple[int, int]:
    cfg, _keep = config_from_spec(spec)
    l, r = ctypes.c_int(), ctypes.c_int()
    _check(load_library().demon_vae_rf_from_config(ctypes.byref(cfg), ctypes.byref(l), ctypes.byref(r)))
    return l.value, r.value


def demon_vae_forward_support(spec, frame_a: int, frame_b: int) -> Tuple[int, int]:
    cfg, _keep = config_from_spec(spec)
    lo, hi = ctypes.c_longlong(), ctypes.c_longlong()
    _check(load_library().demon_vae_forward_support(ctypes.byref(cfg), frame_a, frame_b, ctypes.byref(lo), ctypes.byref(hi)))
    return lo.value, hi.value


def demon_vae_plan_windows(n_clips: int, n_frames: int, frame_begin: int, frame_end: int, window: int,
                           halo: int) -> List[dict]:
    lib = load_library()
    n = ctypes.c_int()
    _check(lib.demon_vae_plan_windows(n_clips, n_frames, frame_begin, frame_end, window, halo, None, 0, ctypes.byref(n)))
    arr = (_Window * max(n.value, 1))()
    _check(lib.demon_vae_plan_windows(n_clips, n_frames, frame_begin, frame_end, window, halo, arr, n.value, ctypes.byref(n)))
    return [dict(clip=w.clip, begin=w.begin, end=w.end, lo=w.lo, hi=w.hi) for w in arr[:n.value]]


def demon_vae_create(spec, weights: np.ndarray, dtype: int, max_frames: int, max_clips: int = 1,
                     max_extended_frames: int = 0, wide_operands: int = 0, flags: int = 0, small_tile_wgs: int = 0) -> int:
    """Returns the opaque handle (an integer address).  `weights`: flat fp32 host array, canonical order."""
    cfg, _keep = config_from_spec(spec, dtype, max_frames, max_clips, max_extended_frames, wide_operands, flags, small_tile_wgs)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    handle = ctypes.c_void_p()
    _check(load_library().demon_vae_create(ctypes.byref(cfg), w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                           w.size, ctypes.byref(handle)))
    return handle.value


def demon_vae_encoder_weight_count(spec) -> int:
    cfg, _keep = config_from_spec(spec)
    return int(load_library().demon_vae_encoder_weight_count(ctypes.byref(cfg)))


def demon_vae_encoder_rf_from_config(spec) -> Tuple[int, int, int, int]:
    """(halo_left, halo_right) in latent frames and (samples_left, samples_right)."""
    cfg, _keep = config_from_spec(spec)
    l, r = ctypes.c_int(), ctypes.c_int()
    sl, sr = ctypes.c_longlong(), ctypes.c_longlong()
    _check(load_library().demon_vae_encoder_rf_from_config(ctypes.byref(cfg), ctypes.byref(l), ctypes.byref(r),
                                                           ctypes.byref(sl), ctypes.byref(sr)))
    return l.value, r.value, sl.value, sr.value


def demon_vae_create_encoder(spec, weights: np.ndarray, dtype: int, max_frames: int, max_clips: int = 1,
                             max_extended_frames: int = 0, wide_operands: int = 0, flags: int = 0, small_tile_wgs: int = 0) -> int:
    """Returns the opaque handle of an encoder.  `weights`: flat fp32 host array in the encoder's order."""
    cfg, _keep = config_from_spec(spec, dtype, max_frames, max_clips, max_extended_frames, wide_operands, flags, small_tile_wgs)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    handle = ctypes.c_void_p()
    _check(load_library().demon_vae_create_encoder(ctypes.byref(cfg), w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                                   w.size, ctypes.byref(handle)))
    return handle.value


def demon_vae_encode_windowed(handle: int, d_wave: int, n_clips: int, n_frames: int, frame_begin: int, frame_end: int,
                              window: int, halo: int, d_eps: int, d_moments: int, d_latent: int, stream: int = 0):
    _check(load_library().demon_vae_encode_windowed(handle, d_wave, n_clips, n_frames, frame_begin, frame_end, window, halo,
                                                    d_eps, d_moments, d_latent, stream))


def demon_vae_encode(handle: int, d_wave: int, n_clips: int, n_frames: int, d_eps: int, d_moments: int, d_latent: int,
                     stream: int = 0):
    _check(load_library().demon_vae_encode(handle, d_wave, n_clips, n_frames, d_eps, d_moments, d_latent, stream))


def demon_vae_destroy(handle: Optional[int]):
    if handle:
        load_library().demon_vae_destroy(handle)


def demon_vae_receptive_field(handle: int) -> Tuple[int, int]:
    l, r = ctypes.c_int(), ctypes.c_int()
    _check(load_library().demon_vae_receptive_field(handle, ctypes.byref(l), ctypes.byref(r)))
    return l.value, r.value


def demon_vae_decode(handle: int, d_latent: int, n_clips: int, n_frames: int, d_out: int, stream: int = 0):
    """d_latent / d_out are device addresses (tensor.data_ptr()); stream is a hipStream_t address."""
    _check(load_library().demon_vae_decode(handle, d_latent, n_clips, n_frames, d_out, stream))


def demon_vae_decode_windowed(handle: int, d_latent: int, n_clips: int, n_frames: int, frame_begin: int,
                              frame_end: int, window: int, halo: int, d_out: int, stream: int = 0):
    _check(load_library().demon_vae_decode_windowed(handle, d_latent, n_clips, n_frames, frame_begin, frame_end,
                                                    window, halo, d_out, stream))


def demon_vae_decode_windowed_static(handle: int, d_latent: int, n_clips: int, n_frames: int, frame_begin: int,
                                     frame_end: int, window: int, halo: int, d_out: int, stream: int = 0):
    _check(load_library().demon_vae_decode_windowed_static(handle, d_latent, n_clips, n_frames, frame_begin, frame_end,
                                                           window, halo, d_out, stream))


def demon_vae_decode_windowed_pcm16(handle: int, d_latent: int, n_clips: int, n_frames: int, frame_begin: int,
                                    frame_end: int, window: int, halo: int, d_pcm: int, stream: int = 0):
    _check(load_library().demon_vae_decode_windowed_pcm16(handle, d_latent, n_clips, n_frames, frame_begin,
                                                          frame_end, window, halo, d_pcm, stream))


def demon_vae_decode_windowed_gated(handle: int, d_latent: int, n_clips: int, n_frames: int, frame_begin: int,
                                    frame_end: int, window: int, halo: int, d_skip: int, d_out: int, stream: int = 0):
    _check(load_library().demon_vae_decode_windowed_gated(handle, d_latent, n_clips, n_frames, frame_begin, frame_end,
                                                          window, halo, d_skip, d_out, stream))


def demon_vae_latent_similarity(d_curr: int, d_prev: int, n_clips: int, elems_per_clip: int, dtype: int,
                                threshold: float, d_mse: int, d_unchanged: int, stream: int = 0):
    _check(load_library().demon_vae_latent_similarity(d_curr, d_prev, n_clips, elems_per_clip, dtype, threshold,
                                                      d_mse, d_unchanged, stream))


def demon_vae_crossfade(d_prev_tail: int, prev_stride: int, d_next_head: int, next_stride: int, d_out: int,
                        out_stride: int, n_planes: int, n_samples: int, stream: int = 0):
    _check(load_library().demon_vae_crossfade(d_prev_tail, prev_stride, d_next_head, next_stride, d_out, out_stride,
                                              n_planes, n_samples, stream))


def latent_similarity(curr, prev, threshold: float = 1e-3):
    """(mse, unchanged) device tensors of shape [n_clips] for two latents [n_clips, C, T] (or [C, T])."""
    import torch
    if curr.dim() == 2:
        curr, prev = curr[None], prev[None]
    assert curr.is_cuda and prev.is_cuda and curr.shape == prev.shape and curr.dtype == prev.dtype
    assert curr.is_contiguous() and prev.is_contiguous()
    dtype = {torch.bfloat16: DEMON_BF16, torch.float32: DEMON_F32}[curr.dtype]
    n = curr.shape[0]
    mse = torch.empty(n, dtype=torch.float32, device=curr.device)
    flag = torch.empty(n, dtype=torch.int32, device=curr.device)
    demon_vae_latent_similarity(curr.data_ptr(), prev.data_ptr(), n, curr[0].numel(), dtype, threshold,
                                mse.data_ptr(), flag.data_ptr(), torch.cuda.current_stream().cuda_stream)
    return mse, flag


def crossfade(prev_tail, next_head, out=None):
    """Equal-power crossfade of two fp32 device tensors [..., n]; the last dimension must be contiguous and the
    leading dimensions must collapse to one plane stride (views into planar waveforms are fine)."""
    import torch

    def planes(t):
        t2 = t.reshape(-1, t.shape[-1]) if t.is_contiguous() else t
        assert t2.dim() == 2 and t2.stride(1) == 1 and t2.dtype == torch.float32 and t2.is_cuda
        return t2

    if out is None:
        out = torch.empty(prev_tail.shape, dtype=torch.float32, device=prev_tail.device)
    a, b, o = planes(prev_tail), planes(next_head), planes(out)
    assert a.shape == b.shape == o.shape
    demon_vae_crossfade(a.data_ptr(), a.stride(0), b.data_ptr(), b.stride(0), o.data_ptr(), o.stride(0),
                        a.shape[0], a.shape[1], torch.cuda.current_stream().cuda_stream)
    return out


def demon_vae_debug_tap(handle: int, layer: int, d_dst: int, capacity: int):
    _check(load_library().demon_vae_debug_tap(handle, layer, d_dst, capacity))


def demon_vae_set_timing(handle: int, level: int):
    _check(load_library().demon_vae_set_timing(handle, level))


def demon_vae_get_timing(handle: int) -> List[float]:
    lib = load_library()
    n = ctypes.c_int()
    _check(lib.demon_vae_get_timing(handle, None, 0, ctypes.byref(n)))
    arr = (ctypes.c_float * max(n.value, 1))()
    _check(lib.demon_vae_get_timing(handle, arr, n.value, ctypes.byref(n)))
    return [float(x) for x in arr[:n.value]]


class DemonVAE:
    """Convenience wrapper: owns a handle, marshals torch tensors.  No arithmetic happens here."""

    def __init__(self, spec, weights: np.ndarray, dtype: str = "bf16", max_frames: int = 1500, max_clips: int = 1,
                 max_extended_frames: int = 0, wide_operands: int = 0, flags: int = 0, small_tile_wgs: int = 0):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("DemonVAE needs a HIP device; there is no CPU fallback")
        self.spec = spec
        self.dtype = {"bf16": DEMON_BF16, "f32": DEMON_F32}[dtype]
        self.torch_dtype = torch.bfloat16 if self.dtype == DEMON_BF16 else torch.float32
        self.S = 1
        for s in spec.strides:
            self.S *= s
        self.handle = demon_vae_create(spec, weights, self.dtype, max_frames, max_clips, max_extended_frames,
                                       wide_operands, flags, small_tile_wgs)

    def close(self):
        if getattr(self, "handle", None):
            import torch
            torch.cuda.synchronize()
            demon_vae_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def receptive_field(self) -> Tuple[int, int]:
        return demon_vae_receptive_field(self.handle)

    def _prep(self, latent, out):
        import torch
        if latent.dim() == 2:
            latent = latent[None]
        assert latent.is_cuda and latent.dtype == self.torch_dtype and latent.is_contiguous()
        n_clips, c, t = latent.shape
        assert c == self.spec.latent_channels
        if out is None:
            out = torch.empty((n_clips, self.spec.out_channels, t * self.S), dtype=torch.float32, device=latent.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == (n_clips, self.spec.out_channels, t * self.S)
        return latent, out, n_clips, t, torch.cuda.current_stream().cuda_stream

    def decode(self, latent, out=None):
        latent, out, n_clips, t, stream = self._prep(latent, out)
        demon_vae_decode(self.handle, latent.data_ptr(), n_clips, t, out.data_ptr(), stream)
        return out

    def decode_windowed(self, latent, window: int, halo: int = -1, frame_begin: int = 0,
                        frame_end: Optional[int] = None, out=None):
        latent, out, n_clips, t, stream = self._prep(latent, out)
        if frame_end is None:
            frame_end = t
        demon_vae_decode_windowed(self.handle, latent.data_ptr(), n_clips, t, frame_begin, frame_end, window, halo,
                                  out.data_ptr(), stream)
        return out

    def decode_windowed_static(self, latent, window: int, halo: int = -1, frame_begin: int = 0,
                               frame_end: Optional[int] = None, out=None):
        """The windowed decode in the library's static scratch array (allocates nothing); `out` should be given."""
        latent, out, n_clips, t, stream = self._prep(latent, out)
        if frame_end is None:
            frame_end = t
        demon_vae_decode_windowed_static(self.handle, latent.data_ptr(), n_clips, t, frame_begin, frame_end, window, halo,
                                         out.data_ptr(), stream)
        return out

    def decode_windowed_gated(self, latent, skip, out, window: int, halo: int = -1, frame_begin: int = 0,
                              frame_end: Optional[int] = None):
        """skip: int32 device tensor [n_clips]; clips with a non-zero flag keep what `out` holds."""
        import torch
        latent, out, n_clips, t, stream = self._prep(latent, out)
        assert skip.is_cuda and skip.dtype == torch.int32 and skip.is_contiguous() and skip.numel() == n_clips
        if frame_end is None:
            frame_end = t
        demon_vae_decode_windowed_gated(self.handle, latent.data_ptr(), n_clips, t, frame_begin, frame_end, window, halo,
                                        skip.data_ptr(), out.data_ptr(), stream)
        return out

    def decode_windowed_pcm16(self, latent, window: int, halo: int = -1, frame_begin: int = 0,
                              frame_end: Optional[int] = None, out=None):
        """out: int16 [n_clips, n_frames * S, out_channels], channel-interleaved."""
        import torch
        if latent.dim() == 2:
            latent = latent[None]
        assert latent.is_cuda and latent.dtype == self.torch_dtype and latent.is_contiguous()
        n_clips, c, t = latent.shape
        assert c == self.spec.latent_channels
        if out is None:
            out = torch.zeros((n_clips, t * self.S, self.spec.out_channels), dtype=torch.int16, device=latent.device)
        assert out.is_cuda and out.dtype == torch.int16 and out.is_contiguous()
        assert tuple(out.shape) == (n_clips, t * self.S, self.spec.out_channels)
        if frame_end is None:
            frame_end = t
        demon_vae_decode_windowed_pcm16(self.handle, latent.data_ptr(), n_clips, t, frame_begin, frame_end, window,
                                        halo, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        return out

    def set_timing(self, level: int):
        demon_vae_set_timing(self.handle, level)

    def get_timing(self) -> List[float]:
        return demon_vae_get_timing(self.handle)

    def tap(self, layer: int, dst=None):
        demon_vae_debug_tap(self.handle, layer, dst.data_ptr() if dst is not None else 0,
                            dst.numel() if dst is not None else 0)


class DemonVAEEncoder:
    """Convenience wrapper of an encoder handle: marshals torch tensors.  No arithmetic happens here."""

    def __init__(self, spec, weights: np.ndarray, dtype: str = "bf16", max_frames: int = 1500, max_clips: int = 1,
                 max_extended_frames: int = 0, flags: int = 0, small_tile_wgs: int = 0):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("DemonVAEEncoder needs a HIP device; there is no CPU fallback")
        self.spec = spec
        self.dtype = {"bf16": DEMON_BF16, "f32": DEMON_F32}[dtype]
        self.latent_dtype = torch.bfloat16 if self.dtype == DEMON_BF16 else torch.float32
        self.S = 1
        for s in spec.strides:
            self.S *= s
        self.handle = demon_vae_create_encoder(spec, weights, self.dtype, max_frames, max_clips, max_extended_frames,
                                               0, flags, small_tile_wgs)

    def close(self):
        if getattr(self, "handle", None):
            import torch
            torch.cuda.synchronize()
            demon_vae_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def receptive_field(self) -> Tuple[int, int]:
        return demon_vae_receptive_field(self.handle)

    def set_timing(self, level: int):
        demon_vae_set_timing(self.handle, level)

    def get_timing(self) -> List[float]:
        return demon_vae_get_timing(self.handle)

    def tap(self, layer: int, dst=None):
        demon_vae_debug_tap(self.handle, layer, dst.data_ptr() if dst is not None else 0,
                            dst.numel() if dst is not None else 0)

    def encode_windowed(self, wave, window: int, halo: int = -1, frame_begin: int = 0, frame_end: Optional[int] = None,
                        eps=None, moments=None, latent=None):
        """wave: fp32 [n_clips, channels, T * S] (or [channels, T * S]).  Returns (moments, latent); pass the tensors
        to write into, or get new ones (zero outside the encoded range)."""
        import torch
        if wave.dim() == 2:
            wave = wave[None]
        assert wave.is_cuda and wave.dtype == torch.float32 and wave.is_contiguous()
        n_clips, ch, n = wave.shape
        assert ch == self.spec.out_channels and n % self.S == 0
        t = n // self.S
        c0 = self.spec.latent_channels
        if moments is None:
            moments = torch.zeros((n_clips, 2 * c0, t), dtype=torch.float32, device=wave.device)
        if latent is None:
            latent = torch.zeros((n_clips, c0, t), dtype=self.latent_dtype, device=wave.device)
        assert moments.is_contiguous() and moments.dtype == torch.float32 and tuple(moments.shape) == (n_clips, 2 * c0, t)
        assert latent.is_contiguous() and latent.dtype == self.latent_dtype and tuple(latent.shape) == (n_clips, c0, t)
        if eps is not None:
            assert eps.is_cuda and eps.dtype == torch.float32 and eps.is_contiguous() and tuple(eps.shape) == (n_clips, c0, t)
        if frame_end is None:
            frame_end = t
        demon_vae_encode_windowed(self.handle, wave.data_ptr(), n_clips, t, frame_begin, frame_end, window, halo,
                                  eps.data_ptr() if eps is not None else 0, moments.data_ptr(), latent.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream)
        return moments, latent

    def encode(self, wave, eps=None):
        if wave.dim() == 2:
            wave = wave[None]
        t = wave.shape[2] // self.S
        return self.encode_windowed(wave, window=t, halo=0, eps=eps)
