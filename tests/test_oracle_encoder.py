"""Pins of the oracle's encoder (the decoder's mirror), its windowed encode, the sampling step and the encoder's
analytic receptive field.  No GPU."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import demon_inputs as di
import oracle

SMALL = di.DecoderSpec(latent_channels=4, strides=(4, 2), widths=(8, 6), dilations=(1, 3), res_kernel=7)


# ------------------------------------------------------------------ the strided convolution

def brute_conv1d_strided(x, W, b, s, p):
    """The index definition written out: y[o, n] = b[o] + sum_i sum_k W[o, i, k] x[i, n s - p + k]."""
    Cin, L = x.shape
    Cout, _, K = W.shape
    Lout = (L + 2 * p - K) // s + 1
    y = np.zeros((Cout, Lout))
    for o, n in itertools.product(range(Cout), range(Lout)):
        acc = b[o]
        for i, k in itertools.product(range(Cin), range(K)):
            m = n * s - p + k
            if 0 <= m < L:
                acc += W[o, i, k] * x[i, m]
        y[o, n] = acc
    return y


@pytest.mark.parametrize("s", [2, 4, 6, 10])
@pytest.mark.parametrize("L", [1, 3])
def test_strided_conv_vs_brute_force_and_torch(s, L):
    """Every (kernel 2s, stride s, padding s/2) of the benchmark stacks, on lengths that are multiples of s."""
    rng = np.random.default_rng(s * 10 + L)
    Cin, Cout, n = 3, 2, L * s
    x = rng.standard_normal((Cin, n)); W = rng.standard_normal((Cout, Cin, 2 * s)); b = rng.standard_normal(Cout)
    y = oracle.conv1d_strided(x, W, b, s, s // 2)
    assert y.shape == (Cout, L)                                    # length / s exactly
    np.testing.assert_allclose(y, brute_conv1d_strided(x, W, b, s, s // 2), rtol=0, atol=1e-12)
    ref = F.conv1d(torch.from_numpy(x)[None], torch.from_numpy(W), torch.from_numpy(b), stride=s, padding=s // 2)[0].numpy()
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("K,s,p,L", [(3, 1, 1, 9), (5, 2, 0, 11), (4, 3, 2, 10), (7, 5, 3, 23)])
def test_strided_conv_general_shapes_vs_torch(K, s, p, L):
    rng = np.random.default_rng(K + s + p + L)
    x = rng.standard_normal((2, L)); W = rng.standard_normal((3, 2, K)); b = rng.standard_normal(3)
    ref = F.conv1d(torch.from_numpy(x)[None], torch.from_numpy(W), torch.from_numpy(b), stride=s, padding=p)[0].numpy()
    np.testing.assert_allclose(oracle.conv1d_strided(x, W, b, s, p), ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv1d_strided(x, W, b, s, p), brute_conv1d_strided(x, W, b, s, p), rtol=0, atol=1e-12)


@pytest.mark.parametrize("s", [2, 4, 10])
def test_strided_conv_is_the_adjoint_of_the_transposed_conv(s):
    """<convS(x; W), y> = <x, convT(y; W)> with the same weight array (Conv1d [out, in, k] is ConvTranspose1d
    [in, out, k] read the other way): ties the new primitive to the decoder's transposed conv, which has its own pins."""
    rng = np.random.default_rng(s)
    Cin, Cout, Lo = 3, 4, 5
    x = rng.standard_normal((Cin, Lo * s)); y = rng.standard_normal((Cout, Lo)); W = rng.standard_normal((Cout, Cin, 2 * s))
    lhs = np.sum(oracle.conv1d_strided(x, W, None, s, s // 2) * y)
    back = oracle.convT1d(y, W, None, s, s // 2)
    assert back.shape == x.shape
    assert abs(lhs - np.sum(x * back)) < 1e-10 * max(1.0, abs(lhs))


# ------------------------------------------------------------------ the whole encoder

def torch_encode(spec, weights, wave):
    """The encoder assembled from PyTorch's own conv routines (float64): an independent composition."""
    p = {k: torch.from_numpy(np.array(v, dtype=np.float64)) for k, v in di.split_encoder_weights(spec, weights).items()}

    def snake(h, name):
        a = p[name + ".alpha"][None, :, None]; b = p[name + ".beta"][None, :, None]
        return h + torch.sin(a * h) ** 2 / (b + 1e-9)

    h = torch.from_numpy(np.array(wave, dtype=np.float64))[None]
    h = F.conv1d(h, p["stem.weight"], p["stem.bias"], padding=(spec.head_kernel - 1) // 2)
    for l in range(len(spec.strides) - 1, -1, -1):
        s = spec.strides[l]
        for j, d in enumerate(spec.dilations):
            q = f"e{l}.r{j}"
            r = F.conv1d(snake(h, q + ".a1"), p[q + ".c1.weight"], p[q + ".c1.bias"], dilation=d, padding=d * (spec.res_kernel - 1) // 2)
            r = F.conv1d(snake(r, q + ".a2"), p[q + ".c2.weight"], p[q + ".c2.bias"])
            h = h + r
        h = F.conv1d(snake(h, f"e{l}.down"), p[f"e{l}.down.weight"], p[f"e{l}.down.bias"], stride=s, padding=s // 2)
    return h[0].numpy()


def test_layout_and_output_shape():
    names = [n for n, _ in di.encoder_weight_layout(di.FULL)]
    assert names[0] == "stem.weight" and names[-1] == "e0.down.bias" and names[2].startswith("e4.r0")
    shapes = dict(di.encoder_weight_layout(di.FULL))
    assert shapes["stem.weight"] == (64, 2, 7) and shapes["e4.down.weight"] == (128, 64, 4)
    assert shapes["e0.down.weight"] == (128, 1024, 20)            # the moments: 2 x 64 channels
    for T in (1, 3, 50):
        w = di.make_encoder_weights(di.TINY)
        assert oracle.encode_moments(di.TINY, w, di.make_waveform(2, T * 32, 0)).shape == (32, T)
    m = oracle.encode_moments(di.FULL, di.make_encoder_weights(di.FULL), di.make_waveform(2, 2 * 1920, 0))
    assert m.shape == (128, 2)                                    # 1920 samples per latent frame, 25 Hz at 48 kHz


@pytest.mark.parametrize("spec,T,snake", [(SMALL, 11, "uniform"), (di.TINY, 50, "lognormal"), (di.TINY, 7, "uniform")])
def test_encode_vs_torch_composition(spec, T, snake):
    w = di.make_encoder_weights(spec, seed=3, std=0.3 if spec is SMALL else 0.02, snake=snake)
    x = di.make_waveform(spec.out_channels, T * spec.total_stride, 5)
    m = oracle.encode_moments(spec, w, x)
    ref = torch_encode(spec, w, x)
    assert np.abs(ref).max() > 1e-3
    np.testing.assert_allclose(m, ref, rtol=0, atol=1e-12)


def test_encode_full_stack_vs_torch_composition():
    w = di.make_encoder_weights(di.FULL, bf16=True)
    x = di.make_waveform(2, 3 * 1920, 1)
    np.testing.assert_allclose(oracle.encode_moments(di.FULL, w, x), torch_encode(di.FULL, w, x), rtol=0, atol=1e-10)


def test_encode_f32_close_to_f64():
    w = di.make_encoder_weights(di.TINY); x = di.make_waveform(2, 50 * 32, 0)
    assert np.abs(oracle.encode_moments(di.TINY, w, x) - oracle.encode_moments(di.TINY, w, x, dtype=np.float32)).max() < 1e-6


def test_shift_equivariance():
    """Shifting the waveform by one latent frame's worth of samples shifts the moments by one frame, away from the edges."""
    spec, T = di.TINY, 60
    S = spec.total_stride
    w = di.make_encoder_weights(spec, seed=2)
    x = di.make_waveform(2, T * S, 9)
    xs = np.zeros_like(x); xs[:, S:] = x[:, :-S]
    m, ms = oracle.encode_moments(spec, w, x), oracle.encode_moments(spec, w, xs)
    hl, hr = oracle.encoder_receptive_field(spec)
    np.testing.assert_allclose(ms[:, hl + 2:T - hr], m[:, hl + 1:T - hr - 1], rtol=0, atol=1e-13)


def test_affine_when_snake_is_the_identity():
    """With beta huge Snake is the identity and the encoder is affine: E(a x1 + b x2) - E(0) = a (E(x1) - E(0)) + b (E(x2) - E(0))."""
    spec = SMALL
    w = di.make_encoder_weights(spec, seed=4, std=0.3)
    for name, t in di.split_encoder_weights(spec, w).items():
        if name.endswith(".beta"):
            t[:] = 1e30
    n = 9 * spec.total_stride
    x1, x2 = di.make_waveform(2, n, 1).astype(np.float64), di.make_waveform(2, n, 2).astype(np.float64)
    e0 = oracle.encode_moments(spec, w, np.zeros((2, n)))
    f = lambda x: oracle.encode_moments(spec, w, x) - e0
    np.testing.assert_allclose(f(0.7 * x1 - 1.9 * x2), 0.7 * f(x1) - 1.9 * f(x2), rtol=1e-13, atol=1e-11)


# ------------------------------------------------------------------ receptive field

def test_encoder_receptive_field_values():
    """The mirror has the decoder's cone read the other way: latent frame 0 depends on the samples that frame 0's
    impulse reaches in the decoder."""
    assert oracle.encoder_backward_interval(di.FULL, 0, 0) == oracle.forward_interval(di.FULL, 0, 0) == (-10245, 12164)
    assert oracle.encoder_backward_interval(di.TINY, 0, 0) == oracle.forward_interval(di.TINY, 0, 0) == (-453, 484)
    assert oracle.encoder_receptive_field(di.FULL) == (6, 6) and oracle.encoder_receptive_field(di.TINY) == (15, 15)
    # one strided conv, stride 4: frame 0 reads samples [-2, 5]; samples [0, 3] reach frames [-1, 1]
    one = di.DecoderSpec(latent_channels=1, strides=(4,), widths=(1,), dilations=(), head_kernel=1)
    assert oracle.encoder_backward_interval(one, 0, 0) == (-2, 5)
    assert oracle.encoder_forward_interval(one, 0, 3) == (-1, 1)


@pytest.mark.parametrize("spec,T,frame", [(SMALL, 40, 20), (di.TINY, 40, 20), (di.TINY, 40, 3), (di.TINY, 40, 38)])
def test_encoder_receptive_field_equals_impulse_support(spec, T, frame):
    """Zero biases and a zero waveform give E(0) = 0 exactly (snake(0) = 0); with positive weights nothing cancels, so
    the set of samples whose impulse moves the moments of `frame` is the exact backward cone: impulses on its first and
    last sample reach the frame, impulses one sample outside do not, and the frames one impulse reaches are the forward cone."""
    w = di.make_encoder_weights(spec, seed=1, zero_bias=True, positive=True)
    S = spec.total_stride
    n = T * S
    assert np.all(oracle.encode_moments(spec, w, np.zeros((2, n))) == 0.0)
    lo, hi = oracle.encoder_backward_interval(spec, frame, frame)

    def reaches(sample):
        x = np.zeros((2, n)); x[:, sample] = 1.0
        return np.nonzero(np.any(oracle.encode_moments(spec, w, x) != 0.0, axis=0))[0]

    for sample, inside in ((lo, True), (hi, True), (lo - 1, False), (hi + 1, False)):
        if 0 <= sample < n:
            assert (frame in reaches(sample)) == inside, (sample, inside)
    mid = min(max(frame * S + S // 2, 0), n - 1)
    nz = reaches(mid)
    flo, fhi = oracle.encoder_forward_interval(spec, mid, mid)
    assert nz[0] == max(flo, 0) and nz[-1] == min(fhi, T - 1) and len(nz) == nz[-1] - nz[0] + 1


def test_full_stack_encoder_cone_edges():
    spec, T, frame = di.FULL, 14, 7
    w = di.make_encoder_weights(spec, seed=1, zero_bias=True, positive=True)
    S = spec.total_stride
    lo, hi = oracle.encoder_backward_interval(spec, frame, frame)
    assert (lo - frame * S, hi - frame * S) == (-10245, 12164)
    for sample, inside in ((lo, True), (hi, True), (lo - 1, False), (hi + 1, False)):
        x = np.zeros((2, T * S)); x[:, sample] = 1.0
        m = oracle.encode_moments(spec, w, x)
        assert bool(np.any(m[:, frame] != 0.0)) == inside, (sample, inside)


# ------------------------------------------------------------------ windowed encode

@pytest.mark.parametrize("spec,T,window", [(di.TINY, 50, 16), (SMALL, 23, 5), (di.TINY, 17, 17), (di.TINY, 40, 1)])
def test_windowed_encode_equals_full_encode_for_halo_at_least_rf(spec, T, window):
    w = di.make_encoder_weights(spec, seed=5, std=0.3 if spec is SMALL else 0.02)
    x = di.make_waveform(2, T * spec.total_stride, 11)
    full = oracle.encode_moments(spec, w, x)
    H = max(oracle.encoder_receptive_field(spec))
    for halo in (H, H + 3):
        assert np.array_equal(oracle.encode_moments_windowed(spec, w, x, window, halo), full)
    part = oracle.encode_moments_windowed(spec, w, x, window, H, frame_begin=3, frame_end=T - 2)
    assert np.array_equal(part, full[:, 3:T - 2])


def test_windowed_encode_with_a_short_halo_differs_where_the_cone_says():
    spec, T, window = di.TINY, 64, 16
    w = di.make_encoder_weights(spec, seed=5)
    x = di.make_waveform(2, T * spec.total_stride, 11)
    full = oracle.encode_moments(spec, w, x)
    hl, hr = oracle.encoder_receptive_field(spec)
    H = max(hl, hr)
    short = oracle.encode_moments_windowed(spec, w, x, window, H - 1)
    bad = np.nonzero(np.any(short != full, axis=0))[0]
    assert len(bad) > 0
    # only frames whose cone crosses a cut of the extended region can differ: within one frame of an interior window edge
    edges = [b for b in range(window, T, window)]
    assert all(any(f in (e - 1, e) for e in edges) for f in bad), bad
    none = oracle.encode_moments_windowed(spec, w, x, window, 0)
    assert np.abs(none - full).max() > 100 * np.abs(short - full).max()


# ------------------------------------------------------------------ sampling step

def test_sampling_step_closed_forms():
    rng = np.random.default_rng(0)
    C0, T = 4, 7
    mean = rng.standard_normal((C0, T))
    eps = rng.standard_normal((C0, T))
    zero = np.zeros((C0, T))
    assert np.array_equal(oracle.sample_latent(np.concatenate([mean, zero]), zero), mean)             # eps = 0: the mean
    assert np.array_equal(oracle.sample_latent(np.concatenate([mean, zero]), eps), mean + eps)        # logvar = 0: unit variance
    lv = np.full((C0, T), 2.0 * np.log(3.0))
    np.testing.assert_allclose(oracle.sample_latent(np.concatenate([mean, lv]), eps), mean + 3.0 * eps, rtol=1e-15)
    lv = np.full((C0, T), -2.0 * np.log(4.0))
    np.testing.assert_allclose(oracle.sample_latent(np.concatenate([zero, lv]), eps), eps / 4.0, rtol=1e-15)
    # batch axis
    m3 = np.stack([np.concatenate([mean, zero]), np.concatenate([zero, zero])])
    assert np.array_equal(oracle.sample_latent(m3, np.stack([eps, eps])), np.stack([mean + eps, eps]))
    # the sampled latent has the posterior's moments
    big = oracle.sample_latent(np.concatenate([np.full((1, 200000), 1.5), np.full((1, 200000), np.log(0.25))]),
                               rng.standard_normal((1, 200000)))
    assert abs(big.mean() - 1.5) < 5e-3 and abs(big.std() - 0.5) < 5e-3
