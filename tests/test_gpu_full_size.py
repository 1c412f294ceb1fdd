"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (window 64,
analytic halo, all windows in one batch).  The oracle cannot decode whole clips in seconds, so it is
evaluated on sampled blocks of output frames through its own windowed decode (whose equality with the
full decode is pinned on the CPU); the rest is covered by properties that hold at any size: windowed ==
full bit for bit, batch of clips == clip by clip, partial re-decode + splice == full re-decode."""
import numpy as np
import pytest
import torch

import demon_inputs as di
import oracle
from gpu_util import TOL_WINDOWED_VS_FULL, assert_close, to_device
from paper_2605_28657_amd import DemonVAE, DEMON_VAE_FLAG_NO_FUSED, DEMON_VAE_FLAG_ONE_STREAM

pytestmark = pytest.mark.gpu

SPEC = di.FULL
S = SPEC.total_stride
H = 6
BLOCK = 4          # output frames per oracle sample


def oracle_blocks(weights, z, starts):
    """{start: oracle output of frames [start, start+BLOCK)} from the oracle's windowed decode."""
    return {b: oracle.decode_windowed(SPEC, weights, z, window=BLOCK, halo=H, frame_begin=b, frame_end=b + BLOCK)
            for b in starts}


def check_blocks(gpu_out, refs, what):
    g = np.concatenate([gpu_out[:, b * S:(b + BLOCK) * S] for b in refs], axis=1)
    r = np.concatenate([refs[b] for b in refs], axis=1)
    ma, rl = assert_close(g, r, "bf16", what)
    print(f"{what}: max-abs {ma:.3e} rel-L2 {rl:.3e} over {g.size} samples")


def make_vae(wl, extra=0):
    weights, lat = di.workload_inputs(wl)
    n_windows = wl.n_clips * -(-wl.n_frames // wl.window)
    vae = DemonVAE(SPEC, weights, dtype="bf16", max_frames=wl.n_frames, max_clips=wl.n_clips,
                   max_extended_frames=n_windows * (wl.window + 2 * H) + extra)
    return vae, weights, lat


@pytest.mark.parametrize("name,starts", [("full_10s_bf16", (0, 62, 123, 246)), ("full_60s_bf16", (0, 638, 1470, 1496))])
def test_single_clip_windowed_full_and_oracle_samples(name, starts):
    wl = di.WORKLOADS[name]
    vae, weights, lat = make_vae(wl)
    assert vae.receptive_field() == (H, H)
    zt = to_device(lat, "bf16")
    win = vae.decode_windowed(zt, window=wl.window, halo=-1)
    full = vae.decode(zt)
    assert float((win - full).abs().max()) <= TOL_WINDOWED_VS_FULL
    assert torch.equal(win, full)
    g = win[0].cpu().numpy()
    assert g.shape == (2, wl.n_frames * S) and np.all(np.isfinite(g)) and np.abs(g).max() <= 1.0
    check_blocks(g, oracle_blocks(weights, lat[0], starts), name)
    vae.close()


def test_10s_clip_whole_against_the_oracle_with_every_kernel_variant():
    """configs[1] element by element over the whole clip (the f64 oracle decodes 10 s in seconds), for the default
    kernels and for each alternative the config selects: hi + lo bf16 operands on the wide levels, unfused residual
    units, one stream, no small tiles.  Each variant also reproduces its own full decode bit for bit."""
    wl = di.WORKLOADS["full_10s_bf16"]
    weights, lat = di.workload_inputs(wl)
    ref = oracle.decode(SPEC, weights, lat[0])
    zt = to_device(lat, "bf16")
    n_windows = -(-wl.n_frames // wl.window)
    base = None
    for name, kw in [("default", {}), ("bf16x2", dict(wide_operands=2)), ("unfused", dict(flags=DEMON_VAE_FLAG_NO_FUSED)),
                     ("one stream", dict(flags=DEMON_VAE_FLAG_ONE_STREAM)), ("large tiles only", dict(small_tile_wgs=-1))]:
        vae = DemonVAE(SPEC, weights, dtype="bf16", max_frames=wl.n_frames, max_extended_frames=n_windows * (wl.window + 2 * H), **kw)
        win = vae.decode_windowed(zt, window=wl.window, halo=-1)
        full = vae.decode(zt)
        assert torch.equal(win, full), name
        g = win[0].cpu().numpy()
        ma, rl = assert_close(g, ref, "bf16", name)
        print(f"10 s clip, {name}: max-abs {ma:.3e} rel-L2 {rl:.3e} over {g.size} samples")
        if name == "default":
            base = win.clone()
        elif name in ("one stream", "large tiles only"):
            assert torch.equal(win, base), name              # same kernels and K order: the same bits
        vae.close()


def test_four_clips_in_one_call():
    wl = di.WORKLOADS["full_4x60s_bf16"]
    vae, weights, lat = make_vae(wl)
    zt = to_device(lat, "bf16")
    win = vae.decode_windowed(zt, window=wl.window, halo=-1)
    assert win.shape == (4, 2, 1500 * S)
    for c, b in enumerate((0, 63, 700, 1496)):          # one oracle block per clip
        check_blocks(win[c].cpu().numpy(), oracle_blocks(weights, lat[c], (b,)), f"clip {c}")
    # the batch of 96 windows equals clip-by-clip decodes
    for c in (0, 3):
        one = vae.decode_windowed(zt[c:c + 1].contiguous(), window=wl.window, halo=-1)
        assert torch.equal(one[0], win[c])
    vae.close()


def test_240s_partial_redecode_equals_full_redecode():
    wl = di.WORKLOADS["full_240s_bf16"]
    vae, weights, lat = make_vae(wl)
    zt = to_device(lat, "bf16")
    buf = vae.decode_windowed(zt, window=wl.window, halo=-1)
    # latent frames 2000..2099 replaced; dirty output frames [1994, 2106) snap to windows 31-32 = [1984, 2112)
    lat2 = lat.copy()
    lat2[0][:, 2000:2100] = di.make_latent(64, 100, 21, bf16=True)
    fb = ((2000 - H) // wl.window) * wl.window
    fe = -((-(2100 + H)) // wl.window) * wl.window
    assert (fb, fe) == (1984, 2112)
    zt2 = to_device(lat2, "bf16")
    before = buf.clone()
    vae.decode_windowed(zt2, window=wl.window, halo=-1, frame_begin=fb, frame_end=fe, out=buf)
    assert torch.equal(buf[:, :, :fb * S], before[:, :, :fb * S]) and torch.equal(buf[:, :, fe * S:], before[:, :, fe * S:])
    redone = vae.decode_windowed(zt2, window=wl.window, halo=-1)
    assert torch.equal(buf, redone)                       # whole 240 s buffer, bit for bit
    assert not torch.equal(before, redone)
    g = buf[0].cpu().numpy()
    check_blocks(g, oracle_blocks(weights, lat2[0], (1994, 2046, 2102)), "dirty span")
    check_blocks(g, oracle_blocks(weights, lat2[0], (5996,)), "clip end")
    vae.close()


def test_60s_playback_window_and_pcm16_render():
    """The single 3 s playback window of the latency figure (frames 712..787 of the 60 s clip) and the 16-bit render
    of the whole clip, in the launch configurations bench.py uses."""
    wl = di.WORKLOADS["full_60s_bf16"]
    vae, weights, lat = make_vae(wl)
    zt = to_device(lat, "bf16")
    whole = vae.decode_windowed(zt, window=wl.window, halo=-1)
    pb, pw = (wl.n_frames - 75) // 2, 75
    buf = torch.full_like(whole, 3.0)
    vae.decode_windowed(zt, window=pw, halo=-1, frame_begin=pb, frame_end=pb + pw, out=buf)
    assert torch.equal(buf[:, :, pb * S:(pb + pw) * S], whole[:, :, pb * S:(pb + pw) * S])      # bit for bit
    assert float((buf[:, :, :pb * S] - 3.0).abs().max()) == 0.0 and float((buf[:, :, (pb + pw) * S:] - 3.0).abs().max()) == 0.0
    check_blocks(buf[0].cpu().numpy(), oracle_blocks(weights, lat[0], (pb, pb + 36, pb + pw - BLOCK)), "playback window")
    pcm = vae.decode_windowed_pcm16(zt, window=wl.window, halo=-1)
    assert pcm.shape == (1, wl.n_frames * S, 2) and pcm.dtype == torch.int16
    y = whole[0].cpu().numpy()
    assert np.array_equal(pcm[0].cpu().numpy(), oracle.pcm16(y))                                 # the fp32 decision, bit for bit
    for b, ref in oracle_blocks(weights, lat[0], (0, 749, 1496)).items():                        # and close to the oracle's render
        d = pcm[0, b * S:(b + BLOCK) * S].cpu().numpy().astype(np.int32) - oracle.pcm16(ref, dtype=np.float64).astype(np.int32)
        assert np.abs(d).max() <= 32767 * 2e-2 + 1
    vae.close()
