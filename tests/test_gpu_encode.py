"""GPU parity of the windowed VAE encode (the mirror path) through the C ABI against the CPU oracle, element by
element on seeded inputs: moments and sampled latent, windowed against full, edge cases, the benchmark shape on
sampled frames.  Bars: fp32 path 1e-4; bf16 path relative L2 1e-2 and max-abs 2e-2 of the moments' range (the
decode's bars, stated for a waveform in [-1, 1], scaled to the range of the compared tensor)."""
import numpy as np
import pytest
import torch

import demon_inputs as di
import oracle
import paper_2605_28657_amd as pa
from gpu_util import errors

pytestmark = pytest.mark.gpu

TOL_REL = {"f32": 1e-4, "bf16": 1e-2}
TOL_ABS = {"f32": 1e-4, "bf16": 2e-2}

STACK_V0 = di.DecoderSpec(64, (2,), (128,), (1, 3, 9))
STACK_V1 = di.DecoderSpec(64, (4,), (64,), (1, 3, 9))
STACK_V2 = di.DecoderSpec(16, (4, 2), (96, 32), (1, 3, 9))
STACK_SPLIT = di.DecoderSpec(64, (2, 2), (512, 128), (1, 9))
STACK_ODD = di.DecoderSpec(32, (6, 2), (64, 32), (2, 5), 5, 3, 3)
STACK_WIDE = di.DecoderSpec(64, (2, 2), (256, 64), (1, 3, 9))
STACK_NORES = di.DecoderSpec(32, (2, 4, 2), (256, 128, 64), ())


def assert_close(g, ref, dtype, what):
    ma, rl = errors(g, ref)
    scale = max(1.0, float(np.abs(ref).max()))
    assert rl <= TOL_REL[dtype] and ma <= TOL_ABS[dtype] * scale, \
        f"{what}: max-abs {ma:.3e} (tol {TOL_ABS[dtype] * scale:.3e}), rel-L2 {rl:.3e} (tol {TOL_REL[dtype]})"
    return ma, rl


def make(spec, dtype, T, n_clips=1, weight_seed=100, wave_seed=40, snake="lognormal", **kw):
    bf = dtype == "bf16"
    w = di.make_encoder_weights(spec, seed=weight_seed, bf16=bf, snake=snake)
    x = np.stack([di.make_waveform(spec.out_channels, T * spec.total_stride, wave_seed + i) for i in range(n_clips)])
    eps = np.stack([di.make_noise(spec.latent_channels, T, 70 + i) for i in range(n_clips)])
    enc = pa.DemonVAEEncoder(spec, w, dtype=dtype, max_frames=T, max_clips=n_clips, **kw)
    return enc, w, x, eps


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def latent_np(t):
    return t.float().cpu().numpy()


def test_tiny_fp32_full_and_windowed():
    spec, T = di.TINY, 50
    enc, w, x, eps = make(spec, "f32", T)
    assert enc.receptive_field() == (15, 15)
    ref = oracle.encode_moments(spec, w, x)
    xt, et = dev(x), dev(eps)
    m_full, z_full = enc.encode(xt, eps=et)
    m_win, z_win = enc.encode_windowed(xt, window=16, halo=-1, eps=et)
    assert_close(m_full.cpu().numpy(), ref, "f32", "moments, full")
    assert_close(m_win.cpu().numpy(), ref, "f32", "moments, windowed")
    assert torch.equal(m_win, m_full) and torch.equal(z_win, z_full)          # same kernels, same summation order
    assert_close(z_win.cpu().numpy(), oracle.sample_latent(ref, eps), "f32", "sampled latent")
    _, z_mean = enc.encode_windowed(xt, window=16, halo=-1)                    # no noise: the mean
    assert torch.equal(z_mean, m_win[:, :spec.latent_channels])
    enc.close()


def test_fp32_path_on_the_x1920_stack():
    spec, T = di.FULL, 5
    enc, w, x, eps = make(spec, "f32", T, max_extended_frames=40)
    ref = oracle.encode_moments(spec, w, x)
    m, _ = enc.encode(dev(x))
    assert_close(m.cpu().numpy(), ref, "f32", "full")
    m2, _ = enc.encode_windowed(dev(x), window=2, halo=-1)
    assert_close(m2.cpu().numpy(), ref, "f32", "windowed")
    enc.close()


def test_bf16_x1920_stack_full_and_windowed():
    spec, T = di.FULL, 24
    enc, w, x, eps = make(spec, "bf16", T, max_extended_frames=100)
    assert enc.receptive_field() == (6, 6)
    ref = oracle.encode_moments(spec, w, x)
    xt, et = dev(x), dev(eps)
    m_full, z_full = enc.encode(xt, eps=et)
    m_win, z_win = enc.encode_windowed(xt, window=7, halo=-1, eps=et)         # 4 windows, the last one 3 frames
    ma, rl = assert_close(m_full.cpu().numpy(), ref, "bf16", "moments, full")
    print(f"bf16 x1920 encode T={T}: moments max-abs {ma:.3e} rel-L2 {rl:.3e} (range {np.abs(ref).max():.2f})")
    assert_close(m_win.cpu().numpy(), ref, "bf16", "moments, windowed")
    assert torch.equal(m_win, m_full) and torch.equal(z_win, z_full)
    assert z_win.dtype == torch.bfloat16
    # the sampling step itself, on the GPU's own moments: exact up to the bf16 rounding of z and fp32 exp
    zr = oracle.sample_latent(m_win.cpu().numpy().astype(np.float64), eps)
    assert np.abs(latent_np(z_win) - zr).max() <= 2.0 ** -8 * np.abs(zr).max()
    assert_close(latent_np(z_win), oracle.sample_latent(ref, eps), "bf16", "sampled latent")
    enc.close()


@pytest.mark.parametrize("spec,T,window", [(STACK_V0, 300, 64), (STACK_V1, 150, 37), (STACK_V2, 40, 9), (STACK_SPLIT, 80, 16),
                                           (STACK_ODD, 70, 11), (STACK_WIDE, 70, 16), (STACK_NORES, 60, 13)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_stacks_with_distinct_snake_parameters(spec, T, window, dtype):
    enc, w, x, eps = make(spec, dtype, T, snake="uniform", max_extended_frames=8 * T + 64)
    ref = oracle.encode_moments(spec, w, x)
    xt = dev(x)
    m_full, _ = enc.encode(xt)
    m_win, _ = enc.encode_windowed(xt, window=window, halo=-1)
    ma, rl = assert_close(m_full.cpu().numpy(), ref, dtype, "full")
    print(f"{spec.widths} {dtype}: max-abs {ma:.3e} rel-L2 {rl:.3e} (range {np.abs(ref).max():.2f})")
    assert torch.equal(m_win, m_full)
    enc.close()


@pytest.mark.parametrize("dtype,spec", [("f32", di.TINY), ("bf16", STACK_V1)])
def test_edge_cases(dtype, spec):
    T = 33
    enc, w, x, eps = make(spec, dtype, T, n_clips=2, max_extended_frames=64 * T)
    ref = oracle.encode_moments(spec, w, x)
    xt = dev(x)
    C0 = spec.latent_channels
    # a partial range writes only its frames, of both outputs
    m = torch.full((2, 2 * C0, T), -7.0, device="cuda:0")
    z = torch.full((2, C0, T), -7.0, device="cuda:0", dtype=enc.latent_dtype)
    enc.encode_windowed(xt, window=5, halo=-1, frame_begin=9, frame_end=22, moments=m, latent=z)
    torch.cuda.synchronize()
    assert_close(m[:, :, 9:22].cpu().numpy(), ref[:, :, 9:22], dtype, "partial range")
    assert bool((m[:, :, :9] == -7.0).all()) and bool((m[:, :, 22:] == -7.0).all())
    assert bool((z[:, :, :9] == -7.0).all()) and bool((z[:, :, 22:] == -7.0).all())
    # window 1 (every frame its own window), window > T, halo larger than the clip, halo 0 (inexact but legal)
    full, _ = enc.encode(xt)
    for window, halo in ((1, -1), (T + 5, -1), (4, T + 3)):
        mw, _ = enc.encode_windowed(xt, window=window, halo=halo)
        assert torch.equal(mw, full), (window, halo)
    m0, _ = enc.encode_windowed(xt, window=4, halo=0)
    assert not torch.equal(m0, full)
    assert np.array_equal(m0.cpu().numpy()[:, :, :1].shape, (2, 2 * C0, 1))
    ref0 = oracle.encode_moments_windowed(spec, w, x, 4, 0)
    assert_close(m0.cpu().numpy(), ref0, dtype, "halo 0 follows the oracle's windowed encode")
    # one frame
    x1 = np.ascontiguousarray(x[:1, :, :spec.total_stride])
    m1, _ = enc.encode(dev(x1))
    assert_close(m1.cpu().numpy(), oracle.encode_moments(spec, w, x1), dtype, "one frame")
    enc.close()


def test_random_small_stacks():
    """Ten seeded random encoder stacks (1-3 blocks, strides 2/4/6, widths that are multiples of 32, 1-3 dilations, odd kernels,
    1-3 waveform channels, 1-2 clips, windows from one frame to longer than the clip): parity with the oracle and
    windowed == full, in both precisions."""
    rng = np.random.default_rng(4048)
    done = 0
    while done < 10:
        nb = int(rng.integers(1, 4))
        strides = tuple(int(rng.choice([2, 4, 6])) for _ in range(nb))
        widths = tuple(int(rng.choice([32, 64, 96, 128, 160, 192, 256, 320, 512])) for _ in range(nb))
        c0 = int(rng.choice([16, 32, 48, 64]))
        dil = tuple(int(v) for v in rng.choice([1, 2, 3, 5, 9], size=int(rng.integers(1, 4))))
        rk, hk, oc = int(rng.choice([3, 5, 7])), int(rng.choice([3, 7])), int(rng.choice([1, 2, 3]))
        T, ncl = int(rng.integers(3, 30)), int(rng.integers(1, 3))
        window = int(rng.integers(1, T + 3))
        spec = di.DecoderSpec(c0, strides, widths, dil, rk, hk, oc)
        if (rk - 1) * max(dil) > 64 or T * spec.total_stride * max(widths) > 8e6:
            continue
        H = max(oracle.encoder_receptive_field(spec))
        for dtype in ("bf16", "f32"):
            enc, w, x, eps = make(spec, dtype, T, n_clips=ncl, snake="uniform",
                                  max_extended_frames=ncl * (T + 2 * H) * (T // window + 2))
            xt = dev(x)
            full, _ = enc.encode(xt)
            assert_close(full.cpu().numpy(), oracle.encode_moments(spec, w, x), dtype, f"{spec} T={T} clips={ncl}")
            win, _ = enc.encode_windowed(xt, window=window, halo=-1)
            assert torch.equal(win, full), (spec, T, window)
            enc.close()
        done += 1


def oracle_encoder_layers(spec, w, x):
    """Activations after every residual unit and strided conv of the encoder, from the oracle's primitives, [rows, channels]."""
    p = di.split_encoder_weights(spec, np.asarray(w, dtype=np.float64))
    h = oracle.conv1d(np.asarray(x, dtype=np.float64), p["stem.weight"], p["stem.bias"], 1)
    outs = []
    for l in range(len(spec.strides) - 1, -1, -1):
        s = spec.strides[l]
        for j, d in enumerate(spec.dilations):
            q = f"e{l}.r{j}"
            r = oracle.conv1d(oracle.snake(h, p[q + ".a1.alpha"], p[q + ".a1.beta"]), p[q + ".c1.weight"], p[q + ".c1.bias"], d)
            r = oracle.conv1d(oracle.snake(r, p[q + ".a2.alpha"], p[q + ".a2.beta"]), p[q + ".c2.weight"], p[q + ".c2.bias"], 1)
            h = h + r
            outs.append(h.T.copy())
        h = oracle.conv1d_strided(oracle.snake(h, p[f"e{l}.down.alpha"], p[f"e{l}.down.beta"]), p[f"e{l}.down.weight"],
                                  p[f"e{l}.down.bias"], s, s // 2)
        outs.append(h.T.copy())
    return outs


@pytest.mark.parametrize("dtype,spec", [("f32", di.TINY), ("bf16", STACK_V2), ("bf16", STACK_SPLIT), ("bf16", STACK_WIDE),
                                        ("bf16", di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9)))])
def test_every_layer_against_oracle_primitives(dtype, spec):
    """Reads each layer's activation back through the debug tap (full encode, one window per clip)."""
    T = 21
    enc, w, x, eps = make(spec, dtype, T, snake="uniform")
    refs = oracle_encoder_layers(spec, w, x[0])
    xt = dev(x)
    for i, ref in enumerate(refs):
        dst = torch.full((ref.size,), float("nan"), device="cuda:0")
        enc.tap(i, dst)
        enc.encode(xt)
        torch.cuda.synchronize()
        got = dst.cpu().numpy().reshape(ref.shape)
        ma, rl = errors(got, ref)
        tol = 1e-5 if dtype == "f32" else 1e-2
        tol_abs = (1e-4 if dtype == "f32" else 2e-2) * max(1.0, float(np.abs(ref).max()))
        assert rl <= tol and ma <= tol_abs, f"layer {i}: rel-L2 {rl:.3e} (tol {tol}), max-abs {ma:.3e} (tol {tol_abs:.3e})"
    enc.tap(-1)
    enc.close()


def test_four_clips_in_one_call_and_graph_replay():
    """A batch of clips equals clip-by-clip encodes bit for bit; an encode recorded into a HIP graph (two window groups on
    two streams, a grid never seen before the capture) replays to the eager result, also after the waveform changed in place."""
    spec, T = di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9)), 40
    enc, w, x, eps = make(spec, "bf16", T, n_clips=4, max_extended_frames=4 * 5 * T)
    xt, et = dev(x), dev(eps)
    m_all, z_all = enc.encode_windowed(xt, window=9, halo=-1, eps=et)
    for c in (0, 3):
        m1, z1 = enc.encode_windowed(xt[c:c + 1].contiguous(), window=9, halo=-1, eps=et[c:c + 1].contiguous())
        assert torch.equal(m1[0], m_all[c]) and torch.equal(z1[0], z_all[c])
    assert_close(m_all.cpu().numpy(), oracle.encode_moments(spec, w, x), "bf16", "four clips")
    m_g = torch.zeros_like(m_all); z_g = torch.zeros_like(z_all)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enc.encode_windowed(xt, window=11, halo=-1, eps=et, moments=m_g, latent=z_g)
    for rep in range(3):
        if rep == 1:
            xt.copy_(dev(np.stack([di.make_waveform(2, T * spec.total_stride, 90 + i) for i in range(4)])))
        m_e, z_e = enc.encode_windowed(xt, window=11, halo=-1, eps=et)
        m_g.zero_(); z_g.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(m_g, m_e) and torch.equal(z_g, z_e), rep
    enc.close()


def test_argument_errors_and_handle_kinds():
    spec = di.TINY
    enc, w, x, eps = make(spec, "f32", 10)
    xt = dev(x)
    m = torch.zeros((1, 32, 10), device="cuda:0")
    h = enc.handle

    def status(fn):
        try:
            fn()
            return pa.DEMON_OK
        except pa.DemonError as e:
            return e.status

    for args in [(1, 10, -1, 10, 4, 1), (1, 10, 0, 11, 4, 1), (1, 10, 5, 5, 4, 1), (1, 10, 0, 10, 0, 1), (1, 10, 0, 10, 4, -2), (0, 10, 0, 10, 4, 1)]:
        assert status(lambda: pa.demon_vae_encode_windowed(h, xt.data_ptr(), *args, 0, m.data_ptr(), 0)) == pa.DEMON_ERR_INVALID_ARG
    assert status(lambda: pa.demon_vae_encode_windowed(h, xt.data_ptr(), 1, 10, 0, 10, 4, 1, 0, 0, 0)) == pa.DEMON_ERR_INVALID_ARG   # no output
    assert status(lambda: pa.demon_vae_encode_windowed(h, xt.data_ptr(), 1, 11, 0, 11, 4, 1, 0, m.data_ptr(), 0)) == pa.DEMON_ERR_WORKSPACE
    assert status(lambda: pa.demon_vae_encode_windowed(h, xt.data_ptr(), 2, 10, 0, 10, 4, 1, 0, m.data_ptr(), 0)) == pa.DEMON_ERR_WORKSPACE
    # an encoder is not a decoder and the other way round
    out = torch.zeros((1, 2, 320), device="cuda:0")
    assert status(lambda: pa.demon_vae_decode_windowed(h, xt.data_ptr(), 1, 10, 0, 10, 4, 1, out.data_ptr())) == pa.DEMON_ERR_INVALID_ARG
    assert "encoder" in pa.demon_vae_last_error()
    dec = pa.DemonVAE(spec, di.make_weights(spec), dtype="f32", max_frames=10)
    assert status(lambda: pa.demon_vae_encode_windowed(dec.handle, xt.data_ptr(), 1, 10, 0, 10, 4, 1, 0, m.data_ptr(), 0)) == pa.DEMON_ERR_INVALID_ARG
    # wrong weight count; hi + lo operands are a decoder option
    with pytest.raises(pa.DemonError) as e:
        pa.demon_vae_create_encoder(spec, w[:-1], pa.DEMON_F32, 10)
    assert e.value.status == pa.DEMON_ERR_INVALID_ARG
    with pytest.raises(pa.DemonError) as e:
        pa.demon_vae_create_encoder(di.FULL, di.make_encoder_weights(di.FULL), pa.DEMON_BF16, 4, wide_operands=2)
    assert e.value.status == pa.DEMON_ERR_UNSUPPORTED
    dec.close()
    enc.close()


def test_encode_then_decode_round_trip_layouts():
    """The sampled latent comes out in the layout and type the decoder reads: encoder and decoder chain on the device."""
    spec, T = di.FULL, 12
    enc, w, x, eps = make(spec, "bf16", T, max_extended_frames=60)
    dec = pa.DemonVAE(spec, di.make_weights(spec, bf16=True), dtype="bf16", max_frames=T, max_extended_frames=60)
    _, z = enc.encode_windowed(dev(x), window=5, halo=-1, eps=dev(eps))
    y = dec.decode_windowed(z, window=5, halo=-1)
    torch.cuda.synchronize()
    ref = oracle.decode(spec, di.make_weights(spec, bf16=True), latent_np(z)[0])
    ma, rl = errors(y[0].cpu().numpy(), ref)
    assert ma <= 2e-2 and rl <= 1e-2
    dec.close(); enc.close()


def test_60s_windowed_encode_on_sampled_frames():
    """The benchmark shape of the encode (60 s of 48 kHz stereo, 24 windows of 64 frames + the 6-frame halo, one batch):
    the oracle's own windowed encode on sampled blocks of frames; windowed == full bit for bit over the whole clip."""
    spec, T, window, H, BLOCK = di.FULL, 1500, 64, 6, 4
    w = di.make_encoder_weights(spec, bf16=True)
    x = di.make_waveform(2, T * spec.total_stride, 41)[None]
    eps = di.make_noise(64, T, 71)[None]
    enc = pa.DemonVAEEncoder(spec, w, dtype="bf16", max_frames=T, max_extended_frames=24 * (window + 2 * H))
    xt = dev(x)
    m_win, z_win = enc.encode_windowed(xt, window=window, halo=-1, eps=dev(eps))
    m_full, z_full = enc.encode(xt, eps=dev(eps))
    assert torch.equal(m_win, m_full) and torch.equal(z_win, z_full)
    g = m_win[0].cpu().numpy()
    assert np.all(np.isfinite(g))
    for b in (0, 62, 749, 1496):
        ref = oracle.encode_moments_windowed(spec, w, x[0], window=BLOCK, halo=H, frame_begin=b, frame_end=b + BLOCK)
        ma, rl = assert_close(g[:, b:b + BLOCK], ref, "bf16", f"frames {b}..{b + BLOCK}")
        print(f"60 s encode, frames {b}..{b + BLOCK}: max-abs {ma:.3e} rel-L2 {rl:.3e}")
    enc.close()
