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
STACK_SPLIT = di.DecoderSpec(64, (2, 2), (512, 128), (1, 9))      # first block wide enough for split operands
STACK_ODD = di.DecoderSpec(32, (6, 2), (64, 32), (2, 5), 5, 3, 3)  # other kernels, dilations, 3 output channels


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
    vae.close()


@pytest.mark.parametrize("spec,T,window", [(STACK_V0, 300, 64), (STACK_V1, 150, 37), (STACK_V2, 40, 9),
                                           (STACK_SPLIT, 70, 16), (STACK_ODD, 33, 8)])
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


@pytest.mark.parametrize("dtype,spec", [("f32", di.TINY), ("bf16", STACK_V2), ("bf16", STACK_SPLIT),
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
        assert rl <= tol, f"layer {i}: rel-L2 {rl:.3e}, max-abs {ma:.3e}"
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


def test_unfused_kernels_for_64_and_128_channels_in_a_subprocess():
    """DEMON_VAE_NO_FUSED=1 (read when the library loads) keeps the 64- and 128-channel residual units on the
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
for spec, T in ((di.DecoderSpec(64, (2,), (128,), (1, 3, 9)), 150), (di.DecoderSpec(64, (4,), (64,), (1, 3, 9)), 150)):
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
