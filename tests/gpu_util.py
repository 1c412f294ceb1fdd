"""Helpers of the GPU parity tests (marshalling and error metrics only)."""
import numpy as np
import torch

import demon_inputs as di
from paper_2605_28657_amd import DemonVAE

# Tolerances of the parity bar: (max-abs, relative L2) against the f64 oracle.
TOL = {"f32": (1e-4, 1e-4), "bf16": (2e-2, 1e-2)}
# GPU windowed decode against GPU full decode (max-abs).
TOL_WINDOWED_VS_FULL = 1e-3


def to_device(z: np.ndarray, dtype: str):
    t = torch.from_numpy(np.ascontiguousarray(z)).to("cuda:0")
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t


def make(spec, dtype, T, n_clips=1, weight_seed=0, latent_seed=1, snake="lognormal", std=0.02, **kw):
    bf = dtype == "bf16"
    w = di.make_weights(spec, seed=weight_seed, bf16=bf, snake=snake, std=std)
    z = np.stack([di.make_latent(spec.latent_channels, T, latent_seed + i, bf16=bf) for i in range(n_clips)])
    vae = DemonVAE(spec, w, dtype=dtype, max_frames=T, max_clips=n_clips, **kw)
    return vae, w, z


def errors(g, ref):
    g = np.asarray(g, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(g - ref).max()), float(np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-300))


def assert_close(g, ref, dtype, what=""):
    ma, rl = errors(g, ref)
    tma, trl = TOL[dtype]
    assert ma <= tma and rl <= trl, f"{what}: max-abs {ma:.3e} (tol {tma}), rel-L2 {rl:.3e} (tol {trl})"
    return ma, rl


def pcm16(y):
    return np.round(32767.0 * np.asarray(y, dtype=np.float64)).astype(np.int32)
