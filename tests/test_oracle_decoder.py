"""Pins of the oracle's full decoder, its windowed decode and the analytic receptive field.  No GPU."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import demon_inputs as di
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

SMALL = di.DecoderSpec(latent_channels=4, strides=(4, 2), widths=(8, 6), dilations=(1, 3), res_kernel=7)


def paper_constants():
    out = {}
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = int(v)
    return out


def torch_decode(spec, weights, latent):
    """The decoder assembled from PyTorch's own conv routines (float64): an independent composition."""
    p = {k: torch.from_numpy(np.array(v, dtype=np.float64)) for k, v in di.split_weights(spec, weights).items()}

    def snake(h, name):
        a = p[name + ".alpha"][None, :, None]; b = p[name + ".beta"][None, :, None]
        return h + torch.sin(a * h) ** 2 / (b + 1e-9)

    h = torch.from_numpy(np.array(latent, dtype=np.float64))[None]
    for l, s in enumerate(spec.strides):
        h = F.conv_transpose1d(snake(h, f"b{l}.up"), p[f"b{l}.up.weight"], p[f"b{l}.up.bias"], stride=s, padding=s // 2)
        for j, d in enumerate(spec.dilations):
            q = f"b{l}.r{j}"
            r = F.conv1d(snake(h, q + ".a1"), p[q + ".c1.weight"], p[q + ".c1.bias"],
                         dilation=d, padding=d * (spec.res_kernel - 1) // 2)
            r = F.conv1d(snake(r, q + ".a2"), p[q + ".c2.weight"], p[q + ".c2.bias"])
            h = h + r
    h = F.conv1d(snake(h, "head"), p["head.weight"], p["head.bias"], padding=(spec.head_kernel - 1) // 2)
    return torch.tanh(h)[0].numpy()


def test_paper_constants_and_output_length():
    c = paper_constants()
    assert di.FULL.total_stride == c["samples_per_latent_frame"] == c["sample_rate_hz"] // c["latent_rate_hz"]
    assert di.FULL.latent_channels == c["latent_channels"] and di.FULL.out_channels == c["audio_channels"]
    assert di.WORKLOADS["full_60s_bf16"].n_frames == c["frames_per_60s"] == 60 * c["latent_rate_hz"]
    assert di.WORKLOADS["full_240s_bf16"].n_frames == c["frames_per_240s"]
    w = di.make_weights(di.TINY)
    for T in (1, 3, 50):
        assert oracle.decode(di.TINY, w, di.make_latent(16, T, 0)).shape == (2, T * 32)
    y = oracle.decode(di.FULL, di.make_weights(di.FULL), di.make_latent(64, 2, 0))
    assert y.shape == (2, 2 * 1920)


@pytest.mark.parametrize("spec,T,snake", [(SMALL, 11, "uniform"), (di.TINY, 50, "lognormal"), (di.TINY, 7, "uniform")])
def test_decode_vs_torch_composition(spec, T, snake):
    w = di.make_weights(spec, seed=3, std=0.3 if spec is SMALL else 0.02, snake=snake)
    z = di.make_latent(spec.latent_channels, T, 5)
    y = oracle.decode(spec, w, z)
    ref = torch_decode(spec, w, z)
    assert np.abs(ref).max() > 1e-3
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_decode_full_stack_vs_torch_composition():
    """The x1920 stack on a short latent (bf16-representable inputs, as the GPU path consumes)."""
    w = di.make_weights(di.FULL, seed=0, bf16=True)
    z = di.make_latent(64, 3, 1, bf16=True)
    np.testing.assert_allclose(oracle.decode(di.FULL, w, z), torch_decode(di.FULL, w, z), rtol=0, atol=1e-11)


def test_decode_f32_close_to_f64():
    w = di.make_weights(di.TINY); z = di.make_latent(16, 50, 0)
    y64 = oracle.decode(di.TINY, w, z)
    y32 = oracle.decode(di.TINY, w, z, dtype=np.float32)
    assert np.abs(y64 - y32).max() < 1e-6


# ------------------------------------------------------------------ receptive field

def test_receptive_field_values():
    """Hand-derivable values: each conv7 of dilation d widens by 3d samples at its level, each convT
    maps [a,b] -> [ceil((a+p-k+1)/s), floor((b+p)/s)]."""
    assert oracle.receptive_field(di.TINY) == (15, 15)
    assert oracle.receptive_field(di.FULL) == (6, 6)
    assert oracle.forward_interval(di.TINY, 0, 0) == (-453, 484)
    assert oracle.forward_interval(di.FULL, 0, 0) == (-10245, 12164)
    # a single conv7, dilation 9: +-27 samples; a single convT stride 4: frame 0 reaches samples [-2, 5]
    one = di.DecoderSpec(latent_channels=1, strides=(4,), widths=(1,), dilations=(), head_kernel=1)
    assert oracle.forward_interval(one, 0, 0) == (-2, 5)
    assert oracle.backward_interval(one, 0, 3) == (-1, 1)


@pytest.mark.parametrize("spec,T,frame", [(SMALL, 40, 20), (di.TINY, 40, 20), (di.TINY, 40, 3), (di.TINY, 40, 38)])
def test_receptive_field_equals_impulse_support(spec, T, frame):
    """Zero biases and zero base latent give D(0) = 0 exactly; with positive weights nothing cancels,
    so the non-zero support of the response to a one-frame impulse is the exact forward cone."""
    w = di.make_weights(spec, seed=1, zero_bias=True, positive=True)
    C0, S = spec.latent_channels, spec.total_stride
    assert np.all(oracle.decode(spec, w, np.zeros((C0, T))) == 0.0)
    z = np.zeros((C0, T)); z[:, frame] = 1.0
    y = oracle.decode(spec, w, z)
    nz = np.nonzero(np.any(y != 0.0, axis=0))[0]
    lo, hi = oracle.forward_interval(spec, frame, frame)
    assert nz[0] == max(lo, 0) and nz[-1] == min(hi, T * S - 1)
    assert len(nz) == nz[-1] - nz[0] + 1
    # the backward cone is the transpose of the forward cone
    hl, hr = oracle.receptive_field(spec)
    first_frame, last_frame = nz[0] // S, nz[-1] // S
    if lo >= 0 and hi < T * S:
        assert frame - first_frame == hr and last_frame - frame == hl


def test_full_stack_impulse_support():
    spec, T, frame = di.FULL, 15, 7
    w = di.make_weights(spec, seed=1, zero_bias=True, positive=True)
    z = np.zeros((64, T)); z[:, frame] = 1.0
    y = oracle.decode(spec, w, z)
    nz = np.nonzero(np.any(y != 0.0, axis=0))[0]
    lo, hi = oracle.forward_interval(spec, frame, frame)
    assert (nz[0], nz[-1]) == (lo, hi) == (frame * 1920 - 10245, frame * 1920 + 12164)
    assert len(nz) == hi - lo + 1


def test_perturbation_support_within_cone():
    """Seeded signed weights, f64: perturbing one latent frame changes nothing outside the analytic cone
    and reaches close to both of its edges (the outermost taps are products of many small weights and
    drown in rounding, which is why the exact test above uses positive weights)."""
    spec, T, frame = di.TINY, 48, 24
    w = di.make_weights(spec, seed=0, std=0.2)
    z = di.make_latent(16, T, 9)
    z2 = z.copy(); z2[:, frame] += 1.0
    d = np.abs(oracle.decode(spec, w, z2) - oracle.decode(spec, w, z)).max(axis=0)
    lo, hi = oracle.forward_interval(spec, frame, frame)
    assert np.all(d[:lo] == 0) and np.all(d[hi + 1:] == 0)
    nz = np.nonzero(d)[0]
    S = spec.total_stride
    assert nz[0] // S - lo // S <= 4 and hi // S - nz[-1] // S <= 4


# ------------------------------------------------------------------ windowed == full

@pytest.mark.parametrize("spec,T,window", [(di.TINY, 50, 16), (SMALL, 37, 5), (di.TINY, 50, 50), (di.TINY, 33, 1)])
def test_windowed_equals_full_bit_exact(spec, T, window):
    w = di.make_weights(spec, seed=0, std=0.2, snake="uniform")
    z = di.make_latent(spec.latent_channels, T, 0)
    H = max(oracle.receptive_field(spec))
    full = oracle.decode(spec, w, z)
    assert np.array_equal(oracle.decode_windowed(spec, w, z, window, H), full)
    assert np.array_equal(oracle.decode_windowed(spec, w, z, window, H + 3), full)


def test_window_grid_and_partial_span():
    assert oracle.window_grid(0, 1500, 64)[-1] == (1472, 1500) and len(oracle.window_grid(0, 1500, 64)) == 24
    assert len(oracle.window_grid(0, 250, 64)) == 4 and oracle.window_grid(0, 250, 64)[-1] == (192, 250)
    assert len(oracle.window_grid(0, 6000, 64)) == 94 and oracle.window_grid(0, 6000, 64)[-1] == (5952, 6000)
    assert oracle.window_grid(0, 50, 16) == [(0, 16), (16, 32), (32, 48), (48, 50)]
    spec = di.TINY
    w = di.make_weights(spec, seed=0, std=0.2)
    z = di.make_latent(16, 50, 0)
    full = oracle.decode(spec, w, z)
    part = oracle.decode_windowed(spec, w, z, 8, 15, frame_begin=11, frame_end=37)
    assert np.array_equal(part, full[:, 11 * 32:37 * 32])


def test_windowed_with_short_halo_differs():
    spec = di.TINY; S = 32; H = 15
    # exact variant: positive weights, zero biases, a latent that is zero except in frame 1, which is
    # exactly H frames left of the window starting at frame 16.  Its cone ends at sample 32 + 484 = 516.
    w = di.make_weights(spec, seed=1, zero_bias=True, positive=True)
    z = np.zeros((16, 50)); z[:, 1] = 1.0
    full = oracle.decode(spec, w, z)
    assert np.all(full[:, 16 * S:517] > 0) and np.all(full[:, 517:] == 0)
    assert np.array_equal(oracle.decode_windowed(spec, w, z, 16, H), full)
    short = oracle.decode_windowed(spec, w, z, 16, H - 1)
    bad = np.nonzero(np.any(short != full, axis=0))[0]
    assert bad[0] == 16 * S and bad[-1] == 516            # one frame short: the window's first samples differ
    # seeded signed weights: no halo at all differs grossly at every interior join
    w = di.make_weights(spec, seed=0, std=0.2)
    z = di.make_latent(16, 50, 0)
    full = oracle.decode(spec, w, z)
    d0 = np.abs(oracle.decode_windowed(spec, w, z, 16, 0) - full)
    assert d0.max() > 1e-2 * np.abs(full).max()
    for j in (16, 32, 48):
        assert d0[:, j * S - 8:j * S + 8].max() > 1e-3 * np.abs(full).max()


def test_partial_redecode_splice_equals_full_redecode():
    """Replacing latent frames [c0,c1) dirties output frames [c0-H, c1+H); re-decoding the windows that
    cover that span and splicing equals a full decode of the new latent."""
    spec = di.TINY; H = 15; S = 32; window = 8
    w = di.make_weights(spec, seed=0, std=0.2)
    z = di.make_latent(16, 120, 0)
    buf = oracle.decode(spec, w, z)
    z2 = z.copy(); z2[:, 50:57] = di.make_latent(16, 7, 21)
    fb = ((50 - H) // window) * window; fe = -((-(57 + H)) // window) * window
    assert (fb, fe) == (32, 72)
    buf[:, fb * S:fe * S] = oracle.decode_windowed(spec, w, z2, window, H, frame_begin=fb, frame_end=fe)
    assert np.array_equal(buf, oracle.decode(spec, w, z2))


# ------------------------------------------------------------------ structure

def test_shift_equivariance():
    spec = di.TINY; S = 32; H = 15
    w = di.make_weights(spec, seed=0, std=0.2)
    z = di.make_latent(16, 60, 4)
    zs = np.zeros_like(z); zs[:, 1:] = z[:, :-1]
    y, ys = oracle.decode(spec, w, z), oracle.decode(spec, w, zs)
    a, b = (H + 1) * S, (60 - H - 1) * S
    np.testing.assert_allclose(ys[:, a + S:b], y[:, a:b - S], rtol=0, atol=1e-13)
    assert not np.allclose(ys[:, a:b], y[:, a:b], atol=1e-6)


def test_affine_when_snake_is_identity():
    """With beta huge, Snake is the identity and the pre-tanh decoder is affine in the latent."""
    spec = SMALL
    w = di.make_weights(spec, seed=2, std=0.1)
    parts = di.split_weights(spec, w)
    for k, v in parts.items():
        if k.endswith(".beta"):
            v[:] = 1e30
    D = lambda z: np.arctanh(oracle.decode(spec, w, z))
    z1, z2 = di.make_latent(4, 9, 1).astype(np.float64) * 0.1, di.make_latent(4, 9, 2).astype(np.float64) * 0.1
    d0 = D(np.zeros((4, 9)))
    lhs = D(0.3 * z1 - 0.7 * z2) - d0
    rhs = 0.3 * (D(z1) - d0) - 0.7 * (D(z2) - d0)
    assert np.abs(lhs).max() > 1e-3
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-12)


def test_gated_decode_keeps_or_replaces_whole_clips():
    """Section 3.5's gate composed with the decode: pinned by its two limits (nothing below the threshold: the plain
    windowed decode; everything below: the previous audio, whatever it holds) and by a mixed case clip by clip."""
    spec = di.TINY
    w = di.make_weights(spec, 3)
    T, S = 12, spec.total_stride
    hl = max(oracle.receptive_field(spec))
    prev = np.stack([di.make_latent(spec.latent_channels, T, 60 + c) for c in range(3)])
    old = np.full((3, spec.out_channels, T * S), 7.0)
    curr = prev + 1.0                                             # mse 1: every clip decoded
    out, skipped = oracle.decode_gated(spec, w, curr, prev, old, window=5, halo=hl)
    assert skipped == [False] * 3 and np.array_equal(out, oracle.decode_windowed(spec, w, curr, 5, hl))
    out, skipped = oracle.decode_gated(spec, w, prev, prev, old, window=5, halo=hl)
    assert skipped == [True] * 3 and np.array_equal(out, old)
    curr = prev.copy()
    curr[1] += 0.01                                               # mse 1e-4 < 1e-3: kept
    curr[2] += 0.1                                                # mse 1e-2: decoded
    out, skipped = oracle.decode_gated(spec, w, curr, prev, old, window=5, halo=hl)
    assert skipped == [True, True, False]
    assert np.array_equal(out[:2], old[:2]) and np.array_equal(out[2], oracle.decode(spec, w, curr[2]))
    out, skipped = oracle.decode_gated(spec, w, curr, prev, old, window=5, halo=hl, threshold=1e-5)
    assert skipped == [True, False, False]
