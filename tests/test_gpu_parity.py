"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on seeded
inputs; windowed against full decode; edge cases.  Sizes are chosen so that the oracle takes seconds
while every kernel still sees several tiles and a ragged tail."""
import numpy as np
import pytest
import torch

import demon_inputs as di
import oracle
import paper_2605_28657_amd as pa
from gpu_util import TOL_WINDOWED_VS_FULL, assert_close, errors, make, pcm16, to_device

pytestmark = pytest.mark.gpu

# small stacks that select each MFMA tile variant: (128x128, K64), (64x256, K64), (32x128, K16)
STACK_V0 = di.DecoderSpec(64, (2,), (128,), (1, 3, 9))
STACK_V1 = di.DecoderSpec(64, (4,), (64,), (1, 3, 9))
STACK_V2 = di.DecoderSpec(16, (4, 2), (96, 32), (1, 3, 9))
STACK_SPLIT = di.DecoderSpec(64, (2, 2), (512, 128), (1, 9))      # first block wide enough for the wide operand format
STACK_ODD = di.DecoderSpec(32, (6, 2), (64, 32), (2, 5), 5, 3, 3)  # other kernels, dilations, 3 output channels
STACK_WIDE = di.DecoderSpec(64, (2, 2), (256, 64), (1, 3, 9))      # 256 channels: the fused unit that streams its 1x1 weights
STACK_GROW = di.DecoderSpec(32, (2, 2, 2), (128, 256, 512), (1, 3))  # fused units whose block feeds a transposed conv with wide operands


def test_config0_tiny_fp32_full_and_windowed():
    vae, w, z = make(di.TINY, "f32", 50, latent_seed=0)
    ref = oracle.decode(di.TINY, w, z)
    zt = to_device(z, "f32")
    full = vae.decode(zt).cpu().numpy()
    win = vae.decode_windowed(zt, window=16, halo=-1).cpu().numpy()
    assert vae.receptive_field() == (15, 15)
    assert_close(full, ref, "f32", "full")
    assert_close(win, ref, "f32", "windowed")
    assert np.abs(win - full).max() <= TOL_WINDOWED_VS_FULL
    assert np.array_equal(win, full)                      # same kernels, same summation order
    assert np.array_equal(pcm16(win), pcm16(full))        # the paper's criterion (section 4.5): 16-bit identity
    vae.close()


def test_fp32_path_on_the_x1920_stack():
    vae, w, z = make(di.FULL, "f32", 5, max_extended_frames=40)
    ref = oracle.decode(di.FULL, w, z)
    zt = to_device(z, "f32")
    assert_close(vae.decode(zt).cpu().numpy(), ref, "f32", "full")
    assert_close(vae.decode_windowed(zt, window=2, halo=-1).cpu().numpy(), ref, "f32", "windowed")
    vae.close()


def test_bf16_x1920_stack_full_and_windowed():
    T = 24
    vae, w, z = make(di.FULL, "bf16", T, max_extended_frames=100)
    ref = oracle.decode(di.FULL, w, z)
    zt = to_device(z, "bf16")
    full = vae.decode(zt).cpu().numpy()
    win = vae.decode_windowed(zt, window=7, halo=-1).cpu().numpy()       # 4 windows, the last one 3 frames
    ma, rl = assert_close(full, ref, "bf16", "full")
    print(f"bf16 x1920 T={T}: max-abs {ma:.3e} rel-L2 {rl:.3e}")
    assert_close(win, ref, "bf16", "windowed")
    assert np.abs(win - full).max() <= TOL_WINDOWED_VS_FULL
    assert np.array_equal(win, full)
    # other window sizes move every tile boundary of every kernel: an element's value must not depend on where in a
    # tile it is computed
    for window in (5, 11, 12):
        assert np.array_equal(vae.decode_windowed(zt, window=window, halo=-1).cpu().numpy(), full), window
    vae.close()


@pytest.mark.parametrize("spec,T,window", [(STACK_V0, 300, 64), (STACK_V1, 150, 37), (STACK_V2, 40, 9),
                                           (STACK_SPLIT, 70, 16), (STACK_ODD, 33, 8), (STACK_WIDE, 150, 37),
                                           (STACK_GROW, 21, 6)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_stacks_with_distinct_snake_parameters(spec, T, window, dtype):
    """alpha, beta ~ U[0.5, 2] per channel: a wrong channel index is far outside the tolerance."""
    vae, w, z = make(spec, dtype, T, snake="uniform", max_extended_frames=8 * T)
    ref = oracle.decode(spec, w, z)
    zt = to_device(z, dtype)
    full = vae.decode(zt).cpu().numpy()
    win = vae.decode_windowed(zt, window=window, halo=-1).cpu().numpy()
    assert_close(full, ref, dtype, "full")
    assert np.array_equal(win, full)
    vae.close()


def test_random_small_stacks():
    """Seeded random layer stacks (widths that select every tile variant and fusion, odd kernels, several dilations,
    1-3 output channels, 1-2 clips, windows from one frame to longer than the clip): parity with the oracle and
    windowed == full, in both precisions."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 10:
        nb = int(rng.integers(1, 4))
        strides = tuple(int(rng.choice([2, 4, 6])) for _ in range(nb))
        widths = tuple(int(rng.choice([32, 64, 96, 128, 160, 192, 256, 320, 512])) for _ in range(nb))
        c0 = int(rng.choice([16, 32, 48, 64]))
        dil = tuple(int(x) for x in rng.choice([1, 2, 3, 5, 9], size=int(rng.integers(1, 4))))
        rk, hk, oc = int(rng.choice([3, 5, 7])), int(rng.choice([3, 7])), int(rng.choice([1, 2, 3]))
        T, ncl = int(rng.integers(3, 30)), int(rng.integers(1, 3))
        window = int(rng.integers(1, T + 3))
        spec = di.DecoderSpec(c0, strides, widths, dil, rk, hk, oc)
        if (rk - 1) * max(dil) > 64 or T * spec.total_stride * max(widths) > 8e6:
            continue
        H = max(oracle.receptive_field(spec))
        for dtype in ("bf16", "f32"):
            vae, w, z = make(spec, dtype, T, n_clips=ncl, snake="uniform",
                             max_extended_frames=ncl * (T + 2 * H) * (T // window + 2))
            zt = to_device(z, dtype)
            full = vae.decode(zt).cpu().numpy()
            assert_close(full, oracle.decode(spec, w, z), dtype, f"{spec} T={T} clips={ncl}")
            assert np.array_equal(vae.decode_windowed(zt, window=window, halo=-1).cpu().numpy(), full), (spec, T, window)
            vae.close()
        done += 1


def oracle_layers(spec, w, z):
    """Activations after every up / residual layer, from the oracle's primitives, [rows, channels]."""
    p = di.split_weights(spec, np.asarray(w, dtype=np.float64))
    h = np.asarray(z, dtype=np.float64)
    outs = []
    for l, s in enumerate(spec.strides):
        h = oracle.convT1d(oracle.snake(h, p[f"b{l}.up.alpha"], p[f"b{l}.up.beta"]), p[f"b{l}.up.weight"],
                           p[f"b{l}.up.bias"], s, s // 2)
        outs.append(h.T.copy())
        for j, d in enumerate(spec.dilations):
            q = f"b{l}.r{j}"
            r = oracle.conv1d(oracle.snake(h, p[q + ".a1.alpha"], p[q + ".a1.beta"]), p[q + ".c1.weight"], p[q + ".c1.bias"], d)
            r = oracle.conv1d(oracle.snake(r, p[q + ".a2.alpha"], p[q + ".a2.beta"]), p[q + ".c2.weight"], p[q + ".c2.bias"], 1)
            h = h + r
            outs.append(h.T.copy())
    return outs


@pytest.mark.parametrize("dtype,spec", [("f32", di.TINY), ("bf16", STACK_V2), ("bf16", STACK_SPLIT), ("bf16", STACK_WIDE),
                                        ("bf16", di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9)))])
def test_every_layer_against_oracle_primitives(dtype, spec):
    """Reads each layer's activation back through the debug tap (full decode, one window per clip)."""
    T = 21
    vae, w, z = make(spec, dtype, T, snake="uniform")
    refs = oracle_layers(spec, w, z[0])
    zt = to_device(z, dtype)
    for i, ref in enumerate(refs):
        dst = torch.full((ref.size,), float("nan"), device="cuda:0")
        vae.tap(i, dst)
        vae.decode(zt)
        torch.cuda.synchronize()
        got = dst.cpu().numpy().reshape(ref.shape)
        ma, rl = errors(got, ref)
        tol = 1e-5 if dtype == "f32" else 1e-2
        # max-abs against the layer's own magnitude: the output bar (2e-2 at |y| <= 1) scaled to the activation's range
        tol_abs = (1e-4 if dtype == "f32" else 2e-2) * max(1.0, float(np.abs(ref).max()))
        assert rl <= tol and ma <= tol_abs, f"layer {i}: rel-L2 {rl:.3e} (tol {tol}), max-abs {ma:.3e} (tol {tol_abs:.3e})"
    vae.tap(-1)
    vae.close()


@pytest.mark.parametrize("dtype,spec", [("f32", di.TINY), ("bf16", STACK_V1)])
def test_edge_cases(dtype, spec):
    T = 19
    H = max(oracle.receptive_field(spec))
    vae, w, z = make(spec, dtype, T, n_clips=3, max_extended_frames=3 * T * (2 * H + 1))
    zt = to_device(z, dtype)
    ref = oracle.decode(spec, w, z)
    full = vae.decode(zt).cpu().numpy()
    assert_close(full, ref, dtype, "3 clips full")
    S = spec.total_stride
    # window of one frame, window longer than the clip, halo longer than the clip
    for window, halo in ((1, -1), (T + 5, -1), (4, 10 * T)):
        win = vae.decode_windowed(zt, window=window, halo=halo).cpu().numpy()
        assert np.array_equal(win, full), (window, halo)
    # a short halo is legal: it must equal the oracle's windowed decode with the same halo, not the full decode
    for halo in (0, H - 1):
        win = vae.decode_windowed(zt, window=5, halo=halo).cpu().numpy()
        assert_close(win, oracle.decode_windowed(spec, w, z, 5, halo), dtype, f"halo {halo}")
    assert np.abs(vae.decode_windowed(zt, window=5, halo=0).cpu().numpy() - full).max() > 1e-4      # and it does differ
    # a partial range writes only its own samples
    out = torch.full((3, spec.out_channels, T * S), 7.0, device="cuda:0")
    vae.decode_windowed(zt, window=3, halo=-1, frame_begin=4, frame_end=12, out=out)
    got = out.cpu().numpy()
    assert np.all(got[:, :, :4 * S] == 7.0) and np.all(got[:, :, 12 * S:] == 7.0)
    assert np.array_equal(got[:, :, 4 * S:12 * S], full[:, :, 4 * S:12 * S])
    # single playback window (frame range no longer than the window)
    out.fill_(7.0)
    vae.decode_windowed(zt, window=8, halo=-1, frame_begin=9, frame_end=15, out=out)
    assert np.array_equal(out.cpu().numpy()[:, :, 9 * S:15 * S], full[:, :, 9 * S:15 * S])
    vae.close()
    # one-frame clip
    vae, w, z = make(spec, dtype, 1)
    assert_close(vae.decode(to_device(z, dtype)).cpu().numpy(), oracle.decode(spec, w, z), dtype, "T=1")
    vae.close()


@pytest.mark.parametrize("dtype,spec", [("f32", di.TINY), ("bf16", di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9)))])
def test_partial_redecode_splices_into_existing_waveform(dtype, spec):
    T, window = 120, 8
    H = max(oracle.receptive_field(spec))
    S = spec.total_stride
    vae, w, z = make(spec, dtype, T, max_extended_frames=6 * T)
    zt = to_device(z, dtype)
    buf = vae.decode_windowed(zt, window=window, halo=-1)
    z2 = z.copy()
    z2[0][:, 50:57] = di.make_latent(spec.latent_channels, 7, 21, bf16=(dtype == "bf16"))
    fb = max(0, ((50 - H) // window) * window); fe = min(T, -((-(57 + H)) // window) * window)
    zt2 = to_device(z2, dtype)
    vae.decode_windowed(zt2, window=window, halo=-1, frame_begin=fb, frame_end=fe, out=buf)
    redone = vae.decode_windowed(zt2, window=window, halo=-1)
    assert torch.equal(buf, redone)                                   # whole buffer, bit for bit
    ref = oracle.decode(spec, w, z2)
    assert_close(buf.cpu().numpy()[:, :, fb * S:fe * S], ref[:, :, fb * S:fe * S], dtype, "dirty span")
    assert_close(buf.cpu().numpy(), ref, dtype, "whole clip")
    vae.close()


@pytest.mark.parametrize("dtype,spec,T,window", [("f32", di.TINY, 50, 16), ("bf16", STACK_V1, 37, 8),
                                                 ("f32", STACK_ODD, 23, 5), ("bf16", di.FULL, 9, 4)])
def test_pcm16_render_fused_into_the_stitch(dtype, spec, T, window):
    """The integer decision is taken in fp32 on both sides: the int16 output must equal the oracle's quantiser
    applied to the fp32 output of the same decode, bit for bit; against the oracle's own decode it may differ by the
    floating-point tolerance expressed in 16-bit steps."""
    S = spec.total_stride
    vae, w, z = make(spec, dtype, T, n_clips=2, max_extended_frames=8 * T)
    zt = to_device(z, dtype)
    y = vae.decode_windowed(zt, window=window, halo=-1).cpu().numpy()
    q = vae.decode_windowed_pcm16(zt, window=window, halo=-1).cpu().numpy()
    assert q.dtype == np.int16 and q.shape == (2, T * S, spec.out_channels)
    for c in range(2):
        assert np.array_equal(q[c], oracle.pcm16(y[c]))
        ref = oracle.pcm16(oracle.decode(spec, w, z[c]), dtype=np.float64)
        tol = 32767 * (2e-2 if dtype == "bf16" else 1e-4) + 1
        assert np.abs(q[c].astype(np.int32) - ref.astype(np.int32)).max() <= tol
    # a partial range writes only its own samples, and the full-clip render equals the windowed one
    out = torch.full((2, T * S, spec.out_channels), 1234, dtype=torch.int16, device="cuda:0")
    fb, fe = 3, min(T, 3 + window + 2)
    vae.decode_windowed_pcm16(zt, window=window, halo=-1, frame_begin=fb, frame_end=fe, out=out)
    got = out.cpu().numpy()
    assert np.all(got[:, :fb * S] == 1234) and np.all(got[:, fe * S:] == 1234)
    assert np.array_equal(got[:, fb * S:fe * S], q[:, fb * S:fe * S])
    whole = vae.decode_windowed_pcm16(zt, window=T, halo=0).cpu().numpy()
    assert np.array_equal(whole, q)
    vae.close()


def test_runs_are_deterministic_and_plans_are_reused():
    vae, w, z = make(STACK_V1, "bf16", 64, max_extended_frames=1200)
    zt = to_device(z, "bf16")
    a = vae.decode_windowed(zt, window=16, halo=-1).clone()
    for window in (3, 5, 7, 9, 11, 13, 15, 17, 19):      # more shapes than the plan cache holds
        vae.decode_windowed(zt, window=window, halo=-1)
    b = vae.decode_windowed(zt, window=16, halo=-1)
    assert torch.equal(a, b)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        c = vae.decode_windowed(zt, window=16, halo=-1)
    s.synchronize()
    assert torch.equal(a, c)
    vae.close()


def test_workspace_and_argument_errors():
    vae, w, z = make(STACK_V2, "bf16", 10, max_extended_frames=30)
    zt = to_device(z, "bf16")
    long_z = to_device(np.zeros((1, 16, 11), dtype=np.float32), "bf16")
    two = to_device(np.zeros((2, 16, 10), dtype=np.float32), "bf16")
    out = torch.empty((1, 2, 10 * 8), device="cuda:0")

    def status(fn):
        try:
            fn()
        except pa.DemonError as e:
            return e.status
        return pa.DEMON_OK

    h = vae.handle
    assert status(lambda: pa.demon_vae_decode(h, long_z.data_ptr(), 1, 11, out.data_ptr())) == pa.DEMON_ERR_WORKSPACE
    assert status(lambda: pa.demon_vae_decode(h, two.data_ptr(), 2, 10, out.data_ptr())) == pa.DEMON_ERR_WORKSPACE
    # window 1 with the full halo: 10 windows of up to 10 frames = more than 30 extended frames
    assert status(lambda: pa.demon_vae_decode_windowed(h, zt.data_ptr(), 1, 10, 0, 10, 1, -1, out.data_ptr())) == pa.DEMON_ERR_WORKSPACE
    assert "workspace" in pa.demon_vae_last_error()
    for args in ((0, 10, 0, 10, 4, 1), (1, 10, -1, 10, 4, 1), (1, 10, 0, 11, 4, 1), (1, 10, 5, 5, 4, 1),
                 (1, 10, 0, 10, 0, 1), (1, 10, 0, 10, 4, -2)):
        assert status(lambda: pa.demon_vae_decode_windowed(h, zt.data_ptr(), *args, out.data_ptr())) == pa.DEMON_ERR_INVALID_ARG
    assert status(lambda: pa.demon_vae_decode(h, 0, 1, 10, out.data_ptr())) == pa.DEMON_ERR_INVALID_ARG
    # the handle still works after errors
    vae.decode(zt, out=out)
    torch.cuda.synchronize()
    vae.close()


def test_unfused_kernels_for_64_128_and_256_channels_in_a_subprocess():
    """DEMON_VAE_NO_FUSED=1 (read when the library loads) keeps the 64-, 128- and 256-channel residual units on the
    two-kernel path; same parity bar, and bit-identical windowed == full there too."""
    import os
    import subprocess
    import sys
    code = r'''
import sys, os
sys.path.insert(0, os.path.join(os.getcwd(), "tests")); sys.path.insert(0, os.getcwd())
import numpy as np
import demon_inputs as di, oracle
from gpu_util import make, to_device, assert_close
for spec, T in ((di.DecoderSpec(64, (2,), (128,), (1, 3, 9)), 150), (di.DecoderSpec(64, (4,), (64,), (1, 3, 9)), 150),
                (di.DecoderSpec(64, (2, 2), (256, 64), (1, 3, 9)), 150)):
    vae, w, z = make(spec, "bf16", T, snake="uniform", max_extended_frames=8 * T)
    zt = to_device(z, "bf16")
    full = vae.decode(zt).cpu().numpy()
    win = vae.decode_windowed(zt, window=37, halo=-1).cpu().numpy()
    assert_close(full, oracle.decode(spec, w, z), "bf16", "unfused")
    assert np.array_equal(win, full)
    vae.close()
print("ok")
'''
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, DEMON_VAE_NO_FUSED="1")
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=240)
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr


def test_small_grid_tile_is_bit_identical_to_the_large_tile(tmp_path):
    """Launches with few workgroups use a 64 x 64 tile on the same packed weights (here: every generic launch, the
    inputs are short); DEMON_VAE_SMALL_TILE_WGS=0 in a subprocess keeps the 128 x 128 tile.  Same K order, so the two
    decodes must agree bit for bit."""
    import os
    import subprocess
    import sys
    code = r'''
import sys, os
sys.path.insert(0, os.path.join(os.getcwd(), "tests")); sys.path.insert(0, os.getcwd())
import numpy as np
import demon_inputs as di
from gpu_util import make, to_device
outs = []
for spec, T in ((di.DecoderSpec(64, (2, 2), (512, 128), (1, 9)), 60), (di.DecoderSpec(64, (10, 6, 2), (1024, 512, 64), (1, 3, 9)), 12),
                (di.DecoderSpec(64, (2, 2), (256, 128), (1, 3)), 50)):
    vae, w, z = make(spec, "bf16", T, n_clips=2, max_extended_frames=8 * T)
    outs.append(vae.decode_windowed(to_device(z, "bf16"), window=T // 2 + 1, halo=-1).cpu().numpy().ravel())
    vae.close()
np.save(sys.argv[1], np.concatenate(outs))
print("ok")
'''
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    got = {}
    for name, wgs in (("small", None), ("large", "0")):
        env = dict(os.environ)
        env.pop("DEMON_VAE_SMALL_TILE_WGS", None)
        if wgs is not None:
            env["DEMON_VAE_SMALL_TILE_WGS"] = wgs
        path = str(tmp_path / (name + ".npy"))
        r = subprocess.run([sys.executable, "-c", code, path], cwd=root, env=env, capture_output=True, text=True, timeout=240)
        assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr
        got[name] = np.load(path)
    assert got["small"].shape == got["large"].shape and np.array_equal(got["small"], got["large"])
    assert np.all(np.isfinite(got["small"])) and np.abs(got["small"]).max() > 1e-3


def test_wide_column_tile_is_bit_identical_to_the_square_tile():
    """Dilated convs with many columns run a 128 x 256 tile on the same packed weights, in the same K order: a long clip
    on a stack with a 512-channel level selects it (one window: 2 x 17000 rows, 4 row tiles), the flag switches it off."""
    spec = di.DecoderSpec(64, (2, 2), (512, 64), (1, 9))
    T = 17000
    vae, w, z = make(spec, "bf16", T, max_extended_frames=T)
    ref_vae = pa.DemonVAE(spec, w, dtype="bf16", max_frames=T, max_extended_frames=T, flags=pa.DEMON_VAE_FLAG_NO_WIDE_TILE)
    zt = to_device(z, "bf16")
    a = vae.decode(zt)
    b = ref_vae.decode(zt)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    # and against the oracle on the first frames (a clip edge and the interior of the first tiles)
    ref = oracle.decode_windowed(spec, w, z[0], window=24, halo=max(oracle.receptive_field(spec)), frame_begin=0, frame_end=24)
    assert_close(a[0, :, :24 * spec.total_stride].cpu().numpy(), ref, "bf16", "first frames")
    vae.close(); ref_vae.close()


def test_wide_levels_with_hi_lo_bf16_operands_in_a_subprocess():
    """DEMON_VAE_WIDE_OPERANDS=bf16x2 (read when the library loads) carries the operands of the levels that are at least
    512 channels wide as hi + lo bf16 pairs instead of half; same parity bar, bit-identical windowed == full, also on
    the first two levels of the x1920 stack and on a stack whose width grows into the wide range."""
    import os
    import subprocess
    import sys
    code = r'''
import sys, os
sys.path.insert(0, os.path.join(os.getcwd(), "tests")); sys.path.insert(0, os.getcwd())
import numpy as np
import demon_inputs as di, oracle
from gpu_util import make, to_device, assert_close
for spec, T, window in ((di.DecoderSpec(64, (2, 2), (512, 128), (1, 9)), 60, 23),
                        (di.DecoderSpec(32, (2, 2, 2), (128, 256, 512), (1, 3)), 40, 17),
                        (di.DecoderSpec(64, (10, 6, 2), (1024, 512, 64), (1, 3, 9)), 12, 5)):
    vae, w, z = make(spec, "bf16", T, max_extended_frames=8 * T)
    zt = to_device(z, "bf16")
    full = vae.decode(zt).cpu().numpy()
    win = vae.decode_windowed(zt, window=window, halo=-1).cpu().numpy()
    assert_close(full, oracle.decode(spec, w, z), "bf16", "hi + lo operands")
    assert np.array_equal(win, full)
    vae.close()
print("ok")
'''
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, DEMON_VAE_WIDE_OPERANDS="bf16x2")
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=240)
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr


# ------------------------------------------------------------------ latent similarity filter and crossfade
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("C,T", [(64, 1500), (16, 50), (64, 1), (3, 1025)])
def test_latent_similarity_filter(dtype, C, T):
    bf = dtype == "bf16"
    prev = np.stack([di.make_latent(C, T, 40 + i, bf16=bf) for i in range(5)])
    curr = prev.copy()
    rng = np.random.default_rng(41)
    curr[1] = di.make_latent(C, T, 50, bf16=bf)                                        # unrelated latent: mse ~ 2
    curr[2] = di.round_to_bf16(prev[2] + 0.02 * rng.standard_normal((C, T)).astype(np.float32)) if bf else \
        prev[2] + np.float32(0.02) * rng.standard_normal((C, T)).astype(np.float32)    # small drift: mse ~ 4e-4
    curr[3] = di.round_to_bf16(prev[3] + 0.06 * rng.standard_normal((C, T)).astype(np.float32)) if bf else \
        prev[3] + np.float32(0.06) * rng.standard_normal((C, T)).astype(np.float32)    # larger drift: mse ~ 3.6e-3
    curr[4, C // 2, T // 2] += 1.0                                                      # one element
    if bf:
        curr[4] = di.round_to_bf16(curr[4])
    mse, flag = pa.latent_similarity(to_device(curr, dtype), to_device(prev, dtype), 1e-3)
    mse = mse.cpu().numpy(); flag = flag.cpu().numpy()
    for c in range(5):
        ref = oracle.latent_mse(curr[c], prev[c])
        assert mse[c] == pytest.approx(ref, rel=1e-6, abs=1e-30), (c, mse[c], ref)
        if abs(ref - 1e-3) > 1e-8:                       # away from the threshold the gate is unique
            assert bool(flag[c]) == oracle.latent_unchanged(curr[c], prev[c], 1e-3)
        assert bool(flag[c]) == bool(np.float32(mse[c]) < np.float32(1e-3))     # the decision as taken in fp32
    assert mse[0] == 0.0 and flag[0] == 1 and flag[1] == 0
    # a 2-D latent is one clip; another threshold
    m1, f1 = pa.latent_similarity(to_device(curr[1], dtype), to_device(prev[1], dtype), 10.0)
    assert m1.shape == (1,) and float(m1[0]) == mse[1] and int(f1[0]) == 1


@pytest.mark.parametrize("n", [1, 7, 2400, 5003])
def test_equal_power_crossfade(n):
    rng = np.random.default_rng(60 + n)
    a = rng.uniform(-1, 1, (2, n)).astype(np.float32); b = rng.uniform(-1, 1, (2, n)).astype(np.float32)
    ref = oracle.crossfade(a, b)
    got = pa.crossfade(to_device(a, "f32"), to_device(b, "f32")).cpu().numpy()
    assert np.abs(got - ref).max() <= 1e-6
    # segments inside larger planar waveforms, written in place over the head of the next chunk
    S = 3 * n + 11
    prev_wave = torch.from_numpy(rng.uniform(-1, 1, (2, S)).astype(np.float32)).to("cuda:0")
    next_wave = torch.from_numpy(rng.uniform(-1, 1, (2, S)).astype(np.float32)).to("cuda:0")
    before = next_wave.clone()
    tail, head = prev_wave[:, S - n:], next_wave[:, :n]
    ref2 = oracle.crossfade(tail.cpu().numpy(), head.cpu().numpy())
    pa.crossfade(tail, head, out=head)
    assert np.abs(next_wave[:, :n].cpu().numpy() - ref2).max() <= 1e-6
    assert torch.equal(next_wave[:, n:], before[:, n:])


def test_filter_and_crossfade_argument_errors():
    lib = pa.load_library()
    x = torch.zeros(8, device="cuda:0")
    p = x.data_ptr()
    assert lib.demon_vae_latent_similarity(p, p, 0, 8, pa.DEMON_F32, 1e-3, p, None, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_latent_similarity(p, p, 1, 0, pa.DEMON_F32, 1e-3, p, None, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_latent_similarity(p, p, 1, 8, 7, 1e-3, p, None, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_latent_similarity(p, p, 1, 8, pa.DEMON_F32, -1.0, p, None, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_latent_similarity(p, p, 1, 8, pa.DEMON_F32, 1e-3, None, None, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_latent_similarity(None, p, 1, 8, pa.DEMON_F32, 1e-3, p, None, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_crossfade(p, 4, p, 4, p, 4, 1, 0, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_crossfade(p, 4, p, 4, p, 2, 2, 4, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_crossfade(None, 4, p, 4, p, 4, 1, 4, None) == pa.DEMON_ERR_INVALID_ARG
    assert lib.demon_vae_crossfade(p, -4, p, 4, p, 4, 1, 4, None) == pa.DEMON_ERR_INVALID_ARG
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,spec,T,window", [("f32", di.TINY, 40, 16), ("bf16", STACK_WIDE, 70, 16),
                                                 ("bf16", STACK_V0, 33, 33)])
def test_gated_decode_skips_unchanged_clips_without_a_host_round_trip(dtype, spec, T, window):
    """Filter and decode issued back to back to one stream: the flags never visit the host.  A skipped clip keeps
    what the output buffer held (its previous audio), a decoded clip equals the ungated decode bit for bit, and the
    whole result meets the oracle's gated decode."""
    bf = dtype == "bf16"
    S, C, n = spec.total_stride, spec.latent_channels, 5
    vae, w, prev = make(spec, dtype, T, n_clips=n, max_extended_frames=8 * n * T)
    rng = np.random.default_rng(5)
    drift = lambda z, a: (di.round_to_bf16(z + a * rng.standard_normal(z.shape).astype(np.float32)) if bf
                          else z + np.float32(a) * rng.standard_normal(z.shape).astype(np.float32))
    curr = prev.copy()
    curr[0] = di.make_latent(C, T, 91, bf16=bf)            # new content
    curr[2] = drift(prev[2], 0.01)                         # mse ~ 1e-4: kept
    curr[3] = drift(prev[3], 0.1)                          # mse ~ 1e-2: decoded
    zp, zc = to_device(prev, dtype), to_device(curr, dtype)
    old = vae.decode_windowed(zp, window=window, halo=-1)
    plain = vae.decode_windowed(zc, window=window, halo=-1)
    buf = old.clone()
    mse, flag = pa.latent_similarity(zc, zp, 1e-3)
    vae.decode_windowed_gated(zc, flag, buf, window=window, halo=-1)
    expect_skip = [False, True, True, False, True]
    assert flag.cpu().numpy().astype(bool).tolist() == expect_skip
    for c in range(n):
        assert torch.equal(buf[c], old[c] if expect_skip[c] else plain[c]), c
    hl = max(oracle.receptive_field(spec))
    ref, skipped = oracle.decode_gated(spec, w, curr, prev, old.cpu().numpy(), window=window, halo=hl)
    assert skipped == expect_skip
    assert_close(buf.cpu().numpy(), ref, dtype, "gated decode")
    # all clips skipped: nothing is written; none skipped: the ungated decode; a partial range composes with the gate
    buf.fill_(5.0)
    vae.decode_windowed_gated(zc, torch.ones(n, dtype=torch.int32, device="cuda:0"), buf, window=window, halo=-1)
    assert float((buf - 5.0).abs().max()) == 0.0
    vae.decode_windowed_gated(zc, torch.zeros(n, dtype=torch.int32, device="cuda:0"), buf, window=window, halo=-1)
    assert torch.equal(buf, plain)
    buf.fill_(5.0)
    fb, fe = 2, min(T, 2 + window + 3)
    vae.decode_windowed_gated(zc, flag, buf, window=window, halo=-1, frame_begin=fb, frame_end=fe)
    for c in range(n):
        if expect_skip[c]:
            assert float((buf[c] - 5.0).abs().max()) == 0.0
        else:
            assert torch.equal(buf[c, :, fb * S:fe * S], plain[c, :, fb * S:fe * S])
            assert bool(torch.all(buf[c, :, :fb * S] == 5.0)) and bool(torch.all(buf[c, :, fe * S:] == 5.0))
    # the ungated entry points are not affected by an earlier gated call on the same window grid
    assert torch.equal(vae.decode_windowed(zc, window=window, halo=-1), plain)
    with pytest.raises(pa.DemonError):
        pa.demon_vae_decode_windowed_gated(vae.handle, zc.data_ptr(), n, T, 0, T, window, -1, 0, buf.data_ptr(), 0)
    vae.close()


def test_filter_and_gated_decode_replay_from_one_hip_graph():
    """Similarity filter and gated decode captured together: which clips are decoded is decided on the device at every
    replay from the latents then in the buffers."""
    spec = di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9))
    T, S, n = 40, spec.total_stride, 3
    vae, w, prev = make(spec, "bf16", T, n_clips=n, max_extended_frames=4 * n * T)
    zp = to_device(prev, "bf16")
    zc = zp.clone()
    args = dict(window=13, halo=-1)
    audio = vae.decode_windowed(zp, **args).clone()             # the previous audio; also caches the plan
    mse = torch.empty(n, dtype=torch.float32, device="cuda:0")
    flag = torch.empty(n, dtype=torch.int32, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    elems = spec.latent_channels * T
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cs = torch.cuda.current_stream().cuda_stream
        pa.demon_vae_latent_similarity(zc.data_ptr(), zp.data_ptr(), n, elems, pa.DEMON_BF16, 1e-3,
                                       mse.data_ptr(), flag.data_ptr(), cs)
        vae.decode_windowed_gated(zc, flag, audio, **args)
    for rep, changed in enumerate(([1], [], [0, 2], [0, 1, 2])):
        before = audio.clone()
        for c in changed:
            zc[c].copy_(to_device(di.make_latent(spec.latent_channels, T, 200 + 10 * rep + c, bf16=True), "bf16"))
        expect = vae.decode_windowed(zc, **args).clone()        # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert flag.cpu().numpy().tolist() == [0 if c in changed else 1 for c in range(n)], rep
        for c in range(n):
            assert torch.equal(audio[c], expect[c] if c in changed else before[c]), (rep, c)
        zp.copy_(zc)                                            # the streaming loop: current becomes previous
    ref = oracle.decode(spec, w, zc.float().cpu().numpy())
    assert_close(audio.cpu().numpy(), ref, "bf16", "after the last replay")
    vae.close()


def test_playback_window_decode_replays_from_a_hip_graph():
    """The decode allocates nothing and records no memset once its window plan is cached, so a caller may capture it
    (the playback-window call of a streaming loop) and replay it; every replay is checked against the eager result,
    with eager work and synchronisations in between, also after the latent changed in place."""
    spec = di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9))
    T, S = 90, spec.total_stride
    vae, w, z = make(spec, "bf16", T, max_extended_frames=3 * T)
    zt = to_device(z, "bf16")
    out_eager = torch.zeros((1, spec.out_channels, T * S), device="cuda:0")
    out_graph = torch.zeros_like(out_eager)
    # two windows: the two halves of the layer sequence run on two streams, forked from and joined into the captured one
    args = dict(window=13, halo=-1, frame_begin=30, frame_end=55)
    vae.decode_windowed(zt, out=out_eager, **args)              # also caches the plan (its slot table is uploaded here)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        vae.decode_windowed(zt, out=out_graph, **args)
    for rep in range(4):
        if rep == 2:                                            # new latent content, same buffers
            z2 = np.stack([di.make_latent(spec.latent_channels, T, 77, bf16=True)])
            zt.copy_(to_device(z2, "bf16"))
            vae.decode_windowed(zt, out=out_eager, **args)
        out_graph.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_graph, out_eager), rep
        assert float(out_graph[:, :, :30 * S].abs().max()) == 0.0 and float(out_graph[:, :, 55 * S:].abs().max()) == 0.0
        _ = vae.decode(zt)                                      # unrelated eager work between replays
        torch.cuda.synchronize()
    ref = oracle.decode(spec, w, z2)
    assert_close(out_graph.cpu().numpy()[:, :, 30 * S:55 * S], ref[:, :, 30 * S:55 * S], "bf16", "graph replay")
    vae.close()


def test_sliding_playback_window_cycles_the_plan_cache():
    """A playback window that moves every call is a new window grid every call: more grids than the cache holds,
    back to back without synchronising in between, each written into the same waveform buffer."""
    spec = STACK_V1
    T, S = 64, spec.total_stride
    vae, w, z = make(spec, "bf16", T, max_extended_frames=2 * T)
    zt = to_device(z, "bf16")
    full = vae.decode(zt)
    buf = torch.zeros_like(full)
    for begin in range(0, T, 3):                             # 22 different grids, 8 cache entries
        vae.decode_windowed(zt, window=3, halo=-1, frame_begin=begin, frame_end=min(T, begin + 3), out=buf)
    torch.cuda.synchronize()
    assert torch.equal(buf, full)
    for begin in (30, 0, 61, 30):                            # revisits and a short last window
        buf[:, :, begin * S:].zero_()
        vae.decode_windowed(zt, window=7, halo=-1, frame_begin=begin, frame_end=min(T, begin + 7), out=buf)
        e = min(T, begin + 7)
        assert torch.equal(buf[:, :, begin * S:e * S], full[:, :, begin * S:e * S])
        buf.copy_(full)
    torch.cuda.synchronize()
    vae.close()


def test_a_recorded_grid_survives_any_number_of_other_grids():
    """A call recorded into a graph holds the address of its grid's window table.  The entry is pinned: eager calls
    on more other grids than the cache holds do not evict it, and replays keep decoding the recorded window.  A grid
    seen for the first time while recording is fine too (its table is written by a kernel inside the graph).  When all
    entries are pinned a further recorded grid is refused with WORKSPACE."""
    spec = STACK_V1
    T, S = 64, spec.total_stride
    vae, w, z = make(spec, "bf16", T, max_extended_frames=2 * T)
    zt = to_device(z, "bf16")
    full = vae.decode(zt)
    out_graph = torch.zeros_like(full)
    buf = torch.zeros_like(full)
    rec = dict(window=5, halo=-1, frame_begin=11, frame_end=21)          # two windows, never seen before the capture
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        vae.decode_windowed(zt, out=out_graph, **rec)
    # a second graph on the same grid must not depend on the first one having been replayed: the kernel that writes the
    # grid's table has only been recorded so far, so it is recorded again
    out_graph2 = torch.zeros_like(full)
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2):
        vae.decode_windowed(zt, out=out_graph2, **rec)
    g2.replay()
    torch.cuda.synchronize()
    assert torch.equal(out_graph2[:, :, 11 * S:21 * S], full[:, :, 11 * S:21 * S])
    # nor may an eager call on the recorded grid rely on a replay having written the table
    vae2, _, _ = make(spec, "bf16", T, max_extended_frames=2 * T)
    g3 = torch.cuda.CUDAGraph()
    out3 = torch.zeros_like(full)
    with torch.cuda.graph(g3):
        vae2.decode_windowed(zt, out=out3, **rec)
    vae2.decode_windowed(zt, out=buf, **rec)
    torch.cuda.synchronize()
    assert torch.equal(buf[:, :, 11 * S:21 * S], full[:, :, 11 * S:21 * S])
    g3.replay()
    torch.cuda.synchronize()
    assert torch.equal(out3[:, :, 11 * S:21 * S], full[:, :, 11 * S:21 * S])
    del g3
    vae2.close()
    for rep in range(3):
        for begin in range(0, T - 3, 3):                                  # 21 other grids, 16 cache entries
            vae.decode_windowed(zt, window=3, halo=-1, frame_begin=begin, frame_end=begin + 3, out=buf)
        out_graph.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_graph[:, :, 11 * S:21 * S], full[:, :, 11 * S:21 * S]), rep
        assert float(out_graph[:, :, :11 * S].abs().max()) == 0.0 and float(out_graph[:, :, 21 * S:].abs().max()) == 0.0
        assert torch.equal(buf[:, :, :(T - 4) // 3 * 3 * S], full[:, :, :(T - 4) // 3 * 3 * S])
    # fill the cache with recorded grids: the 16th distinct recorded grid still fits (one entry is taken above), the next does not
    graphs = []
    for i in range(16):
        gi = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            gi.capture_begin()
            try:
                if i < 15:
                    vae.decode_windowed(zt, window=2, halo=-1, frame_begin=2 * i, frame_end=2 * i + 2, out=buf)
                else:
                    with pytest.raises(pa.DemonError) as ei:
                        vae.decode_windowed(zt, window=2, halo=-1, frame_begin=2 * i, frame_end=2 * i + 2, out=buf)
            finally:
                gi.capture_end()
        torch.cuda.current_stream().wait_stream(s)
        graphs.append(gi)
    assert ei.value.status == pa.DEMON_ERR_WORKSPACE and "graph" in ei.value.message
    # eager calls on cached (pinned) grids still work; a new eager grid has no entry left either
    vae.decode_windowed(zt, out=out_graph, **rec)
    with pytest.raises(pa.DemonError) as ei:
        vae.decode_windowed(zt, window=4, halo=-1, frame_begin=40, frame_end=44, out=buf)
    assert ei.value.status == pa.DEMON_ERR_WORKSPACE
    torch.cuda.synchronize()
    vae.close()


@pytest.mark.parametrize("spec", [STACK_V1, STACK_SPLIT, STACK_WIDE])
def test_values_beyond_the_half_range_saturate(spec):
    """Weights large enough to push the residual stream (IEEE half in memory) and the half operands of the wide levels
    far beyond 65504: conversions to half clamp instead of producing infinities, which Snake's sine would turn into
    NaNs.  There is no parity to check out there (the oracle does not clip); the output must be finite and in tanh's range."""
    w = di.make_weights(spec, seed=0, bf16=True)
    for name, t in di.split_weights(spec, w).items():
        if name.endswith(".weight") and not name.startswith("head."):
            t *= np.float32(2.0 ** 17)                       # exact in bf16; Snake parameters and biases stay as they are
    z = np.stack([di.make_latent(spec.latent_channels, 20, 1, bf16=True)])
    vae = pa.DemonVAE(spec, w, dtype="bf16", max_frames=20)
    y = vae.decode_windowed(to_device(z, "bf16"), window=8, halo=-1)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y).all())
    assert float(y.abs().max()) <= 1.0 and float(y.abs().max()) > 0.0
    vae.close()


def test_transposed_conv_feeding_wide_operands_without_residual_units():
    """No residual units and widths rising across 512 channels: a transposed conv with plain bf16 input emits the wide
    operand format of the next block itself."""
    spec = di.DecoderSpec(32, (2, 2, 2), (256, 512, 64), ())
    for wide in (1, 2):
        vae, w, z = make(spec, "bf16", 40, wide_operands=wide)
        ref = oracle.decode(spec, w, z)
        zt = to_device(z, "bf16")
        full = vae.decode(zt).cpu().numpy()
        win = vae.decode_windowed(zt, window=9, halo=-1).cpu().numpy()
        assert_close(full, ref, "bf16", f"wide_operands={wide}")
        assert np.array_equal(win, full)
        vae.close()


@pytest.mark.parametrize("spec,T,window", [(di.DecoderSpec(64, (4, 2), (128, 64), (1, 3, 9)), 45, 11), (STACK_V1, 100, 37),
                                           (di.DecoderSpec(64, (2,), (64,), (1, 3, 9), 7, 5, 1), 120, 64)])
def test_head_inside_the_last_unit_is_bit_identical_to_the_head_kernel(spec, T, window):
    """When the last layer is the fused 64-channel unit, the head runs inside its kernel (the unit's output never goes
    to memory): the same operands in the same order as the head kernel, so the same bits -- full and windowed, at clip
    edges, with ragged windows, two clips, partial ranges -- and the oracle's values.  The library does this for calls of at
    most 256 extended frames (the calls below, except the window-1 grids, which take the head kernel on both sides)."""
    vae, w, z = make(spec, "bf16", T, n_clips=2, max_extended_frames=100 * T)
    ref_vae = pa.DemonVAE(spec, w, dtype="bf16", max_frames=T, max_clips=2, max_extended_frames=100 * T,
                          flags=pa.DEMON_VAE_FLAG_NO_HEAD_FUSION)
    zt = to_device(z, "bf16")
    S = spec.total_stride
    for kw in (dict(window=T, halo=0), dict(window=window, halo=-1), dict(window=7, halo=-1, frame_begin=5, frame_end=T - 3), dict(window=1, halo=-1)):
        a = torch.full((2, spec.out_channels, T * S), -5.0, device="cuda:0")
        b = torch.full((2, spec.out_channels, T * S), -5.0, device="cuda:0")
        vae.decode_windowed(zt, out=a, **kw)
        ref_vae.decode_windowed(zt, out=b, **kw)
        torch.cuda.synchronize()
        assert torch.equal(a, b), kw
    assert_close(vae.decode(zt).cpu().numpy(), oracle.decode(spec, w, z), "bf16", "head inside the unit")
    pcm_a = vae.decode_windowed_pcm16(zt, window=window, halo=-1)
    pcm_b = ref_vae.decode_windowed_pcm16(zt, window=window, halo=-1)
    assert torch.equal(pcm_a, pcm_b)
    vae.close(); ref_vae.close()
