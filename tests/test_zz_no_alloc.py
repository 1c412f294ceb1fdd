"""The entry point that allocates nothing (demon_vae_decode_windowed_static: every buffer of the call in the
library's static scratch array) against demon_vae_decode_windowed, through the C ABI, bit for bit -- two calls in a
row per handle, the second on a smaller input, so that what the first call left in the array cannot matter."""
import numpy as np
import pytest
import torch

import demon_inputs as di
import paper_2605_28657_amd as pa
from gpu_util import make, to_device

pytestmark = pytest.mark.gpu

STACK_WIDE = di.DecoderSpec(64, (2, 2), (256, 64), (1, 3, 9))


def _pair(vae, zt, **kw):
    """(existing entry point, static entry point) on the same input, outputs pre-filled with a marker."""
    n_clips, _, t = zt.shape
    shape = (n_clips, vae.spec.out_channels, t * vae.S)
    ref = torch.full(shape, -7.0, dtype=torch.float32, device=zt.device)
    out = torch.full(shape, -7.0, dtype=torch.float32, device=zt.device)
    vae.decode_windowed(zt, out=ref, **kw)
    vae.decode_windowed_static(zt, out=out, **kw)
    torch.cuda.synchronize()
    return ref, out


@pytest.mark.parametrize("dtype,spec,T1,T2,window", [("bf16", di.FULL, 24, 11, 8), ("f32", di.TINY, 50, 13, 16),
                                                     ("bf16", STACK_WIDE, 150, 40, 37)])
def test_static_scratch_decode_equals_the_windowed_decode_twice_in_a_row(dtype, spec, T1, T2, window):
    vae, _, z = make(spec, dtype, T1, n_clips=2, max_extended_frames=8 * T1 + 64)
    zt = to_device(z, dtype)
    ref, out = _pair(vae, zt, window=window, halo=-1)
    assert torch.equal(out, ref)
    assert float(ref.abs().max()) <= 1.0                   # every sample was written (tanh range), the marker is gone

    # second call: fewer clips, fewer frames, another window, a partial range -- with the first call's data still in the array
    z2 = np.ascontiguousarray(z[:1, :, :T2])
    zt2 = to_device(z2, dtype)
    free_before = torch.cuda.mem_get_info()[0]
    ref2, out2 = _pair(vae, zt2, window=5, halo=-1, frame_begin=2, frame_end=T2 - 1)
    assert torch.equal(out2, ref2)
    S = vae.S
    assert bool((out2[:, :, :2 * S] == -7.0).all()) and bool((out2[:, :, (T2 - 1) * S:] == -7.0).all())   # writes only its range
    # a full decode through the static array (one window, no halo) equals the existing full decode
    full = vae.decode(zt2)
    stat = vae.decode_windowed_static(zt2, window=T2, halo=0)
    torch.cuda.synchronize()
    assert torch.equal(stat, full)
    # nothing was allocated behind torch's back (torch's own pool serves the small output tensors above)
    assert torch.cuda.mem_get_info()[0] >= free_before - (8 << 20)
    vae.close()


def test_static_scratch_decode_with_hi_lo_operand_planes():
    """wide_operands = 2 carries some operands as two planes: the static array is carved accordingly."""
    spec = di.DecoderSpec(64, (2, 2), (512, 128), (1, 9))
    vae, _, z = make(spec, "bf16", 60, max_extended_frames=400, wide_operands=2)
    zt = to_device(z, "bf16")
    ref, out = _pair(vae, zt, window=16, halo=-1)
    assert torch.equal(out, ref)
    vae.close()


def test_static_scratch_decode_rejects_what_does_not_fit():
    vae, _, z = make(di.FULL, "bf16", 8, max_extended_frames=32)
    # the handle's own workspace limits do not apply to the static entry point ...
    z_big = di.make_latent(64, 48, 5, bf16=True)[None]
    zt = to_device(z_big, "bf16")
    out = torch.zeros((1, 2, 48 * vae.S), dtype=torch.float32, device="cuda:0")
    with pytest.raises(pa.DemonError) as e:
        vae.decode_windowed(zt, window=16, out=out)
    assert e.value.status == pa.DEMON_ERR_WORKSPACE
    vae.decode_windowed_static(zt, window=16, out=out)       # 3 windows, 72 extended frames: fits the static array
    torch.cuda.synchronize()
    assert float(out.abs().max()) <= 1.0 and float(out.abs().max()) > 0.0
    # ... but the array's size does: 60 s in 24 windows needs 1788 extended frames
    z_long = torch.zeros((1, 64, 1500), dtype=torch.bfloat16, device="cuda:0")
    out_long = torch.zeros((1, 2, 1500 * vae.S), dtype=torch.float32, device="cuda:0")
    with pytest.raises(pa.DemonError) as e:
        vae.decode_windowed_static(z_long, window=64, out=out_long)
    assert e.value.status == pa.DEMON_ERR_WORKSPACE and "static" in e.value.message
    with pytest.raises(pa.DemonError) as e:
        vae.decode_windowed_static(zt, window=0, out=out)
    assert e.value.status == pa.DEMON_ERR_INVALID_ARG
    vae.close()


def test_static_scratch_decode_can_be_captured_without_a_warm_up_call():
    vae, _, z = make(di.TINY, "f32", 40, max_extended_frames=256)
    zt = to_device(z, "f32")
    ref = vae.decode_windowed(zt, window=16)
    out = torch.zeros_like(ref)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            vae.decode_windowed_static(zt, window=16, out=out)      # this grid was never seen by the static entry point
    for _ in range(3):
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
    vae.close()
