"""Pins of the oracle's primitives: brute force over the index definitions, library
cross-checks (PyTorch CPU), and closed forms.  No GPU."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def brute_conv(x, W, b, d):
    """y[o,n] = b[o] + sum_i sum_k W[o,i,k] x[i, n + (k - (K-1)/2) d], x = 0 outside."""
    Cin, L = x.shape
    Cout, _, K = W.shape
    y = np.zeros((Cout, L))
    for o in range(Cout):
        for n in range(L):
            acc = b[o]
            for i in range(Cin):
                for k in range(K):
                    m = n + (k - (K - 1) // 2) * d
                    if 0 <= m < L:
                        acc += W[o, i, k] * x[i, m]
            y[o, n] = acc
    return y


def brute_convT(x, W, b, s, p):
    """Gather form: y[o,n] = b[o] + sum_i sum_{k : (n+p-k) % s == 0, 0 <= (n+p-k)/s < L} W[i,o,k] x[i,(n+p-k)/s]."""
    Cin, L = x.shape
    _, Cout, K = W.shape
    Lout = (L - 1) * s - 2 * p + K
    y = np.zeros((Cout, Lout))
    for o in range(Cout):
        for n in range(Lout):
            acc = b[o]
            for i in range(Cin):
                for k in range(K):
                    t = n + p - k
                    if t % s == 0 and 0 <= t // s < L:
                        acc += W[i, o, k] * x[i, t // s]
            y[o, n] = acc
    return y


@pytest.mark.parametrize("K,d", [(7, 1), (7, 3), (7, 9), (1, 1), (3, 2)])
@pytest.mark.parametrize("L", [1, 5, 16, 61])
def test_conv1d_brute_force(K, d, L):
    rng = np.random.default_rng(K * 100 + d * 10 + L)
    x = rng.standard_normal((3, L))
    W = rng.standard_normal((4, 3, K))
    b = rng.standard_normal(4)
    np.testing.assert_allclose(oracle.conv1d(x, W, b, d), brute_conv(x, W, b, d), rtol=0, atol=1e-12)


@pytest.mark.parametrize("s", [2, 4, 6, 10])
@pytest.mark.parametrize("L", [1, 2, 7, 16])
def test_convT1d_brute_force(s, L):
    rng = np.random.default_rng(s * 100 + L)
    x = rng.standard_normal((3, L))
    W = rng.standard_normal((3, 2, 2 * s))
    b = rng.standard_normal(2)
    y = oracle.convT1d(x, W, b, s, s // 2)
    assert y.shape == (2, L * s)          # kernel 2s, padding s/2: exact xs upsampling
    np.testing.assert_allclose(y, brute_convT(x, W, b, s, s // 2), rtol=0, atol=1e-12)


@pytest.mark.parametrize("s,K,p", [(3, 5, 1), (2, 4, 0), (4, 8, 3)])
def test_convT1d_brute_force_general_padding(s, K, p):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 9))
    W = rng.standard_normal((2, 3, K))
    b = rng.standard_normal(3)
    np.testing.assert_allclose(oracle.convT1d(x, W, b, s, p), brute_convT(x, W, b, s, p), rtol=0, atol=1e-12)


@pytest.mark.parametrize("Cin,Cout,K,d,L", [(16, 8, 7, 1, 100), (8, 8, 7, 3, 100), (8, 16, 7, 9, 257),
                                            (32, 32, 1, 1, 64), (64, 2, 7, 1, 333)])
def test_conv1d_vs_torch(Cin, Cout, K, d, L):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((Cin, L)); W = rng.standard_normal((Cout, Cin, K)); b = rng.standard_normal(Cout)
    ref = F.conv1d(torch.from_numpy(x)[None], torch.from_numpy(W), torch.from_numpy(b),
                   padding=d * (K - 1) // 2, dilation=d)[0].numpy()
    np.testing.assert_allclose(oracle.conv1d(x, W, b, d), ref, rtol=0, atol=1e-11)


@pytest.mark.parametrize("s", [2, 4, 6, 10])
def test_convT1d_vs_torch(s):
    rng = np.random.default_rng(2)
    Cin, Cout, L = 12, 5, 37
    x = rng.standard_normal((Cin, L)); W = rng.standard_normal((Cin, Cout, 2 * s)); b = rng.standard_normal(Cout)
    ref = F.conv_transpose1d(torch.from_numpy(x)[None], torch.from_numpy(W), torch.from_numpy(b),
                             stride=s, padding=s // 2)[0].numpy()
    np.testing.assert_allclose(oracle.convT1d(x, W, b, s, s // 2), ref, rtol=0, atol=1e-11)


def test_snake_closed_forms():
    alpha = np.array([0.5, 1.0, 2.0]); beta = np.array([2.0, 1.0, 0.25])
    # snake(0) = 0
    assert np.all(oracle.snake(np.zeros((3, 4)), alpha, beta) == 0.0)
    # at x = pi / (2 alpha): sin^2 = 1  ->  x + 1/(beta + 1e-9)
    x = (math.pi / (2 * alpha))[:, None] * np.ones((3, 2))
    np.testing.assert_allclose(oracle.snake(x, alpha, beta), x + (1.0 / (beta + 1e-9))[:, None], atol=1e-14)
    # at x = pi / alpha: sin^2 = 0  ->  x
    x = (math.pi / alpha)[:, None] * np.ones((3, 2))
    np.testing.assert_allclose(oracle.snake(x, alpha, beta), x, atol=1e-14)
    # generic values against the formula evaluated with Python's math module, element by element
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 17)) * 3
    y = oracle.snake(x, alpha, beta)
    for c, n in itertools.product(range(3), range(17)):
        assert abs(y[c, n] - (x[c, n] + math.sin(alpha[c] * x[c, n]) ** 2 / (beta[c] + 1e-9))) < 1e-14
    # snake is not odd: snake(-x) + snake(x) = 2 sin^2 / beta  (catches sin(x)^2 vs sin(x^2) style slips)
    np.testing.assert_allclose(oracle.snake(-x, alpha, beta) + y,
                               2 * np.sin(alpha[:, None] * x) ** 2 / (beta[:, None] + 1e-9), atol=1e-13)


def test_conv_constant_input_interior():
    """Constant input: interior of conv = const * sum(W) + b; convT with all-ones weights = 2 Cin const."""
    rng = np.random.default_rng(4)
    W = rng.standard_normal((3, 5, 7)); b = rng.standard_normal(3)
    x = np.full((5, 80), 0.7)
    y = oracle.conv1d(x, W, b, 3)
    np.testing.assert_allclose(y[:, 9:-9], (0.7 * W.sum(axis=(1, 2)) + b)[:, None] * np.ones((1, 62)), atol=1e-13)
    assert not np.allclose(y[:, 0], 0.7 * W.sum(axis=(1, 2)) + b)     # the edge sees the zero padding
    for s in (2, 4, 6, 10):
        Wt = np.ones((5, 3, 2 * s))
        yt = oracle.convT1d(x, Wt, np.zeros(3), s, s // 2)
        np.testing.assert_allclose(yt[:, s:-s], 2 * 5 * 0.7, atol=1e-13)


def test_f32_build_matches_f64():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((8, 200)); W = rng.standard_normal((8, 8, 7)) * 0.1; b = rng.standard_normal(8)
    y64 = oracle.conv1d(x, W, b, 3)
    y32 = oracle.conv1d(x, W, b, 3, dtype=np.float32)
    assert y32.dtype == np.float32
    np.testing.assert_allclose(y32, y64, atol=2e-5)


# ------------------------------------------------------------------ 16-bit render (section 3.6)
def test_pcm16_fixed_points_ties_and_clamp():
    y = np.array([[0.0, 1.0, -1.0, 0.5 / 32767, 1.5 / 32767, 2.5 / 32767, -0.5 / 32767, -1.5 / 32767, 1.7, -3.0,
                   100 / 32767, -100 / 32767]])
    q = oracle.pcm16(y, dtype=np.float64)
    assert q.dtype == np.int16 and q.shape == (12, 1)
    assert q[:, 0].tolist() == [0, 32767, -32767, 0, 2, 2, 0, -2, 32767, -32767, 100, -100]


def test_pcm16_interleaves_channels():
    y = np.array([[0.1, 0.2, 0.3], [-0.1, -0.2, -0.3]])
    q = oracle.pcm16(y)
    assert q.shape == (3, 2) and q.flags["C_CONTIGUOUS"]
    assert np.all(q[:, 0] > 0) and np.all(q[:, 1] < 0) and np.array_equal(q[:, 0], -q[:, 1])


def test_pcm16_single_precision_matches_exact_rational_arithmetic():
    """Brute force: the fp32 product is rounded once from the exact rational product (39 significant bits fit a
    double), then rounded half-to-even to an integer with Python's rational round()."""
    from fractions import Fraction
    rng = np.random.default_rng(5)
    y = np.concatenate([rng.uniform(-1.2, 1.2, 400), (np.arange(-40, 40) + 0.5) / 32767.0]).astype(np.float32)
    q = oracle.pcm16(y[None], dtype=np.float32)[:, 0]
    for yi, qi in zip(y, q):
        c = min(max(Fraction(float(yi)), Fraction(-1)), Fraction(1))
        prod32 = np.float32(float(c * 32767))                    # exact in double, one rounding to single
        assert int(qi) == round(Fraction(float(prod32)))
    # and the quantisation error bound of a mid-tread quantiser
    inside = np.abs(y) <= 1
    assert np.all(np.abs(q[inside] / 32767.0 - y[inside]) <= 0.5 / 32767 + 1e-7)


# ------------------------------------------------------------------ latent similarity filter (section 3.5)
def test_latent_mse_closed_forms():
    rng = np.random.default_rng(11)
    a = rng.standard_normal((64, 50))
    assert oracle.latent_mse(a, a) == 0.0
    assert oracle.latent_mse(a + 0.25, a) == pytest.approx(0.0625, rel=1e-12)
    b = a.copy(); b[3, 7] += 2.0                       # one differing element: 4 / size
    assert oracle.latent_mse(a, b) == pytest.approx(4.0 / a.size, rel=1e-12)
    assert oracle.latent_mse(a, b) == oracle.latent_mse(b, a)
    assert oracle.latent_mse(3 * a, 3 * b) == pytest.approx(9 * oracle.latent_mse(a, b), rel=1e-12)
    # independent unit normals differ by variance 2
    c = rng.standard_normal((64, 4000)); d = rng.standard_normal((64, 4000))
    assert oracle.latent_mse(c, d) == pytest.approx(2.0, rel=2e-2)


def test_latent_mse_brute_force_and_library():
    from sklearn.metrics import mean_squared_error
    rng = np.random.default_rng(12)
    a = rng.standard_normal((5, 9)); b = rng.standard_normal((5, 9))
    acc = 0.0
    for i in range(5):
        for j in range(9):
            acc += (a[i, j] - b[i, j]) ** 2
    assert oracle.latent_mse(a, b) == pytest.approx(acc / 45, rel=1e-13)
    assert oracle.latent_mse(a, b) == pytest.approx(mean_squared_error(a.ravel(), b.ravel()), rel=1e-13)


def test_latent_gate_uses_the_papers_threshold():
    a = np.zeros((64, 10))
    assert oracle.latent_unchanged(a + 0.03, a)              # 9e-4 < 1e-3
    assert not oracle.latent_unchanged(a + 0.032, a)         # 1.024e-3
    assert not oracle.latent_unchanged(a + np.sqrt(1e-3) * 1.0001, a)
    assert oracle.latent_unchanged(a + 0.5, a, threshold=0.3)


# ------------------------------------------------------------------ equal-power crossfade of the chunk boundary
@pytest.mark.parametrize("n", [1, 2, 7, 2400])
def test_crossfade_gains_are_equal_power_and_mirror_images(n):
    one = np.ones((1, n)); zero = np.zeros((1, n))
    g_out = oracle.crossfade(one, zero)[0]
    g_in = oracle.crossfade(zero, one)[0]
    np.testing.assert_allclose(g_out ** 2 + g_in ** 2, 1.0, atol=1e-14)
    np.testing.assert_allclose(g_out, g_in[::-1], atol=1e-15)
    assert np.all(np.diff(g_in) > 0) and np.all(np.diff(g_out) < 0)
    assert 0 < g_in[0] <= np.sqrt(0.5) + 1e-15 and g_in[0] == pytest.approx(np.sin(np.pi / (4 * n)), rel=1e-12)
    if n % 2 == 1:
        assert g_in[n // 2] == pytest.approx(np.sqrt(0.5), rel=1e-14)


def test_crossfade_is_linear_and_keeps_the_power_of_uncorrelated_signals():
    rng = np.random.default_rng(13)
    a = rng.standard_normal((2, 2400)); b = rng.standard_normal((2, 2400))
    y = oracle.crossfade(a, b)
    np.testing.assert_allclose(oracle.crossfade(2 * a, -3 * b), 2 * oracle.crossfade(a, 0 * b) - 3 * oracle.crossfade(0 * a, b), atol=1e-13)
    assert np.mean(y ** 2) == pytest.approx(1.0, rel=0.1)
    # a signal crossfaded with itself is boosted by cos+sin (at most sqrt 2 in the middle), never attenuated
    s = oracle.crossfade(a, a) / a
    assert np.all(s >= 1.0 - 1e-12) and s.max() == pytest.approx(np.sqrt(2), rel=1e-6)
    # channels are independent
    np.testing.assert_array_equal(oracle.crossfade(a[:1], b[:1])[0], y[0])
