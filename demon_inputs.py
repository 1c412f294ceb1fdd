"""Seeded synthetic inputs for the windowed VAE decode (decoder specs, weights, latents).

This module is the only code shared by the CPU oracle and the HIP path.  It holds
no arithmetic of the method: it describes the decoder's layer stack, fixes the
canonical order of the parameter tensors in the flat weight array, and draws
seeded random values.  Both sides parse the flat array on their own.

The paper (section 3.6) only says the audio VAE decoder is a stack of dilated 1-D
convolutions mapping a 25 Hz, 64-channel latent to 48 kHz stereo (1920 samples per
latent frame); the concrete synthetic stacks below stand in for the trained model,
which is not available.

Canonical parameter order (all fp32, each tensor C-contiguous):
  for each upsample block l = 0..nb-1 (C_in = widths[l-1] or latent_channels, C = widths[l], s = strides[l]):
      up.alpha[C_in], up.beta[C_in]                      Snake parameters (positive)
      up.weight[C_in, C, 2*s], up.bias[C]               ConvTranspose1d(kernel 2s, stride s, padding s/2)
      for each residual unit j (dilation dilations[j]):
          a1.alpha[C], a1.beta[C]
          c1.weight[C, C, res_kernel], c1.bias[C]       Conv1d(kernel res_kernel, dilation d, zero "same" padding)
          a2.alpha[C], a2.beta[C]
          c2.weight[C, C, 1], c2.bias[C]                Conv1d(kernel 1)
  head.alpha[C_last], head.beta[C_last]
  head.weight[out_channels, C_last, head_kernel], head.bias[out_channels]
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class DecoderSpec:
    latent_channels: int
    strides: Tuple[int, ...]
    widths: Tuple[int, ...]
    dilations: Tuple[int, ...] = (1, 3, 9)
    res_kernel: int = 7
    head_kernel: int = 7
    out_channels: int = 2

    @property
    def total_stride(self) -> int:
        s = 1
        for v in self.strides:
            s *= v
        return s


# configs[0]: tiny fp32 decoder (x32); configs[1..4]: 48 kHz stereo decoder (x1920).
TINY = DecoderSpec(latent_channels=16, strides=(4, 4, 2), widths=(128, 64, 32))
FULL = DecoderSpec(latent_channels=64, strides=(10, 6, 4, 4, 2), widths=(1024, 512, 256, 128, 64))


def weight_layout(spec: DecoderSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the parameter tensors in canonical order."""
    out: List[Tuple[str, Tuple[int, ...]]] = []
    cin = spec.latent_channels
    for l, (s, c) in enumerate(zip(spec.strides, spec.widths)):
        out += [(f"b{l}.up.alpha", (cin,)), (f"b{l}.up.beta", (cin,)),
                (f"b{l}.up.weight", (cin, c, 2 * s)), (f"b{l}.up.bias", (c,))]
        for j in range(len(spec.dilations)):
            p = f"b{l}.r{j}"
            out += [(f"{p}.a1.alpha", (c,)), (f"{p}.a1.beta", (c,)),
                    (f"{p}.c1.weight", (c, c, spec.res_kernel)), (f"{p}.c1.bias", (c,)),
                    (f"{p}.a2.alpha", (c,)), (f"{p}.a2.beta", (c,)),
                    (f"{p}.c2.weight", (c, c, 1)), (f"{p}.c2.bias", (c,))]
        cin = c
    out += [("head.alpha", (cin,)), ("head.beta", (cin,)),
            ("head.weight", (spec.out_channels, cin, spec.head_kernel)),
            ("head.bias", (spec.out_channels,))]
    return out


def n_weights(spec: DecoderSpec) -> int:
    return int(sum(int(np.prod(shape)) for _, shape in weight_layout(spec)))


def split_weights(spec: DecoderSpec, flat: np.ndarray) -> dict:
    """Views of the flat array, by tensor name (no copies, no arithmetic)."""
    out = {}
    pos = 0
    for name, shape in weight_layout(spec):
        n = int(np.prod(shape))
        out[name] = flat[pos:pos + n].reshape(shape)
        pos += n
    if pos != flat.size:
        raise ValueError(f"flat weight array has {flat.size} values, layout needs {pos}")
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16-representable value (ties to even), kept as fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already bf16-representable (uint16, for device upload)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    if np.any(u & 0xFFFF):
        raise ValueError("values are not bf16-representable; call round_to_bf16 first")
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def make_weights(spec: DecoderSpec, seed: int = 0, std: float = 0.02, bf16: bool = False,
                 snake: str = "lognormal", zero_bias: bool = False,
                 positive: bool = False) -> np.ndarray:
    """Flat fp32 parameter array.

    Convolution weights and biases are N(0, std).  Snake alpha/beta are exp(N(0, std))
    ("lognormal", close to 1) or U[0.5, 2] ("uniform", a test variant that makes a
    per-channel indexing mistake visible).  `positive` replaces every conv weight by
    |w| scaled to 1/fan_in (used to measure impulse-response support without
    cancellation); `zero_bias` zeroes all biases.
    """
    rng = np.random.default_rng(seed)
    parts = []
    for name, shape in weight_layout(spec):
        n = int(np.prod(shape))
        if name.endswith(".alpha") or name.endswith(".beta"):
            if snake == "lognormal":
                v = np.exp(rng.standard_normal(n, dtype=np.float32) * np.float32(std))
            elif snake == "uniform":
                v = rng.uniform(0.5, 2.0, n).astype(np.float32)
            else:
                raise ValueError(snake)
        elif name.endswith(".bias"):
            v = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
            if zero_bias:
                v[:] = 0
        else:
            v = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
            if positive:
                # fan-in: taps that reach one output times input channels
                if ".up." in name:
                    fan = shape[0] * 2
                else:
                    fan = shape[1] * shape[2]
                v = (np.abs(v) / np.float32(std) + np.float32(0.5)) / np.float32(fan)
        parts.append(v.astype(np.float32))
    flat = np.concatenate(parts)
    return round_to_bf16(flat) if bf16 else flat


def make_latent(channels: int, frames: int, seed: int, bf16: bool = False) -> np.ndarray:
    """Latent [channels, frames], N(0,1), fp32 (bf16-representable if bf16=True)."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((channels, frames), dtype=np.float32)
    return round_to_bf16(z) if bf16 else z


# ---------------------------------------------------------------- encoder (the decoder's mirror)

def encoder_weight_layout(spec: DecoderSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the encoder's parameter tensors in processing order: stem conv from the waveform, then per
    block from the audio rate down (decoder block index l = nb-1 .. 0) its residual units and the strided conv to the
    next width (the last one to 2 x latent_channels: mean and log-variance)."""
    nb = len(spec.strides)
    c = spec.widths[-1]
    out: List[Tuple[str, Tuple[int, ...]]] = [("stem.weight", (c, spec.out_channels, spec.head_kernel)), ("stem.bias", (c,))]
    for l in range(nb - 1, -1, -1):
        c, s = spec.widths[l], spec.strides[l]
        cn = spec.widths[l - 1] if l > 0 else 2 * spec.latent_channels
        for j in range(len(spec.dilations)):
            p = f"e{l}.r{j}"
            out += [(f"{p}.a1.alpha", (c,)), (f"{p}.a1.beta", (c,)),
                    (f"{p}.c1.weight", (c, c, spec.res_kernel)), (f"{p}.c1.bias", (c,)),
                    (f"{p}.a2.alpha", (c,)), (f"{p}.a2.beta", (c,)),
                    (f"{p}.c2.weight", (c, c, 1)), (f"{p}.c2.bias", (c,))]
        out += [(f"e{l}.down.alpha", (c,)), (f"e{l}.down.beta", (c,)),
                (f"e{l}.down.weight", (cn, c, 2 * s)), (f"e{l}.down.bias", (cn,))]
    return out


def split_encoder_weights(spec: DecoderSpec, flat: np.ndarray) -> dict:
    """Views of the flat encoder array, by tensor name (no copies, no arithmetic)."""
    out = {}
    pos = 0
    for name, shape in encoder_weight_layout(spec):
        n = int(np.prod(shape))
        out[name] = flat[pos:pos + n].reshape(shape)
        pos += n
    if pos != flat.size:
        raise ValueError(f"flat encoder weight array has {flat.size} values, layout needs {pos}")
    return out


def make_encoder_weights(spec: DecoderSpec, seed: int = 100, std: float = 0.02, bf16: bool = False,
                         snake: str = "lognormal", zero_bias: bool = False, positive: bool = False) -> np.ndarray:
    """Flat fp32 encoder parameters, drawn like the decoder's (make_weights): conv weights and biases N(0, std), Snake
    parameters exp(N(0, std)) or U[0.5, 2]; `positive`: |w| scaled to 1/fan-in, for exact support measurements."""
    rng = np.random.default_rng(seed)
    parts = []
    for name, shape in encoder_weight_layout(spec):
        n = int(np.prod(shape))
        if name.endswith(".alpha") or name.endswith(".beta"):
            if snake == "lognormal":
                v = np.exp(rng.standard_normal(n, dtype=np.float32) * np.float32(std))
            elif snake == "uniform":
                v = rng.uniform(0.5, 2.0, n).astype(np.float32)
            else:
                raise ValueError(snake)
        elif name.endswith(".bias"):
            v = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
            if zero_bias:
                v[:] = 0
        else:
            v = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
            if positive:
                v = (np.abs(v) / np.float32(std) + np.float32(0.5)) / np.float32(shape[1] * shape[2])
        parts.append(v.astype(np.float32))
    flat = np.concatenate(parts)
    return round_to_bf16(flat) if bf16 else flat


def make_waveform(channels: int, samples: int, seed: int, bf16: bool = False) -> np.ndarray:
    """Waveform [channels, samples], N(0, 0.25) clipped to [-1, 1], fp32: the stand-in for audio at the encoder's input."""
    rng = np.random.default_rng(seed)
    x = np.clip(rng.standard_normal((channels, samples), dtype=np.float32) * np.float32(0.25), -1.0, 1.0).astype(np.float32)
    return round_to_bf16(x) if bf16 else x


def make_noise(channels: int, frames: int, seed: int) -> np.ndarray:
    """The N(0, 1) draw of the encoder's sampling step, [channels, frames] fp32: an input of the method, not its arithmetic."""
    return np.random.default_rng(seed).standard_normal((channels, frames), dtype=np.float32)


@dataclass(frozen=True)
class Workload:
    """One of the benchmark configurations: decoder, latent shape, window grid, seeds."""
    name: str
    spec: DecoderSpec
    bf16: bool
    n_clips: int
    n_frames: int
    window: int
    latent_seeds: Tuple[int, ...]
    weight_seed: int = 0


WORKLOADS = {
    "tiny_2s_fp32": Workload("tiny_2s_fp32", TINY, False, 1, 50, 16, (0,)),
    "full_10s_bf16": Workload("full_10s_bf16", FULL, True, 1, 250, 64, (1,)),
    "full_60s_bf16": Workload("full_60s_bf16", FULL, True, 1, 1500, 64, (2,)),
    "full_4x60s_bf16": Workload("full_4x60s_bf16", FULL, True, 4, 1500, 64, (10, 11, 12, 13)),
    "full_240s_bf16": Workload("full_240s_bf16", FULL, True, 1, 6000, 64, (20,)),
}


def workload_inputs(w: Workload):
    """(flat weights, latents [n_clips, C, T]) of a workload, fp32 arrays."""
    weights = make_weights(w.spec, seed=w.weight_seed, bf16=w.bf16)
    lat = np.stack([make_latent(w.spec.latent_channels, w.n_frames, s, bf16=w.bf16)
                    for s in w.latent_seeds])
    return weights, lat
