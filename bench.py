#!/usr/bin/env python3
"""Benchmark of the windowed VAE decode on one MI355X.

One step = one windowed decode (gather -> transposed/dilated/1x1 convolutions -> head -> stitch) of the
60 s, 48 kHz stereo workload: a 64 x 1500 latent cut into 24 windows of 64 frames plus a 6-frame halo,
all windows in one batch.  Inputs are synthetic (seeded) and resident in HBM before the timed region.
Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def measured_traffic(workload):
    """HBM bytes per step of the convolution kernels from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy; not collectable inside this process), or None.  The summary
    names the source revision it was measured on; a kernel change makes it stale until the profile is taken again."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("MFMA convolution kernels, bytes per step:"):
                return int(line.split(":")[1].split()[0])
    except (OSError, ValueError):
        pass
    return None


def mfma_probe_rates(seconds=1.0):
    """What the MFMA units of this GPU sustain on operands that toggle like activations (the probe beside the library):
    on register operands, and in the stage loop of the 128 x 128 tile (weights global -> LDS, barriers, fragment reads).
    The published peak is only reached on constant operands; the board's power limit caps everything else."""
    import re
    import subprocess
    exe = os.path.join(ROOT, "paper_2605_28657_amd", "mfma_probe")
    out = {}
    if not os.path.exists(exe):
        return None
    for name, mode in (("register_operands", "0"), ("stage_loop_128x128", "5")):
        try:
            r = subprocess.run([exe, mode, str(seconds), "1"], capture_output=True, text=True, timeout=60)
            m = re.search(r"sustained\s+([0-9.]+)\s+TFLOP/s", r.stdout)
            out[name] = {"TFLOP/s": float(m.group(1)), "frac_of_published_peak": float(m.group(1)) / PEAK_BF16_TFLOPS} if m else None
        except (OSError, subprocess.SubprocessError):
            out[name] = None
    return out


def conv_flops_per_frame(spec):
    """Algorithmic FLOPs (2 x MAC, no halo, no tile padding) per latent frame: (convolutions, head)."""
    cin, rate, conv = spec.latent_channels, 1, 0
    for s, c in zip(spec.strides, spec.widths):
        rate *= s
        conv += rate * 2 * cin * c                                   # transposed conv: 2 taps reach each output
        conv += rate * len(spec.dilations) * (spec.res_kernel * c * c + c * c)
        cin = c
    head = rate * spec.head_kernel * cin * spec.out_channels
    return 2 * conv, 2 * head


def layer_table(spec, wl, launch_ms):
    """Per layer of the decoder (a residual unit = its two convolutions, whichever kernels run them): serialized time of
    one step on one stream, algorithmic FLOPs (2 x MAC, halo-free), algorithmic HBM bytes of a one-kernel-per-layer data
    flow (read the input tensor once, write the output tensor once, 16-bit activations), and both as fractions of peak."""
    frames = wl.n_clips * wl.n_frames
    rows, cin, rate = [], spec.latent_channels, 1
    for l, (s_, c) in enumerate(zip(spec.strides, spec.widths)):
        t = launch_ms.get(f"b{l}.up", 0.0)
        rate_in, rate = rate, rate * s_
        rows.append((f"b{l}.up {cin}->{c} x{s_}", t, 2.0 * rate * 2 * cin * c * frames, 2.0 * (rate_in * cin + rate * c) * frames))
        for j in range(len(spec.dilations)):
            t = launch_ms.get(f"b{l}.r{j}.conv{spec.res_kernel}", 0.0) + launch_ms.get(f"b{l}.r{j}.conv1", 0.0)
            rows.append((f"b{l}.r{j} C={c} d={spec.dilations[j]}", t, 2.0 * rate * (spec.res_kernel + 1) * c * c * frames,
                         2.0 * 2 * rate * c * frames))
        cin = c
    out = []
    for name, ms, flop, byt in rows:
        if ms <= 0:
            continue
        out.append({"layer": name, "ms": round(ms, 4), "GFLOP": round(flop / 1e9, 1), "MB": round(byt / 1e6, 1),
                    "mfma_frac": round(flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 3),
                    "hbm_frac": round(byt / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)})
    return out


def sustained_power(step, torch, seconds=3.0):
    """Back-to-back steps for `seconds` while a thread reads the socket power from hwmon and, once, the shader clocks
    from amd-smi.  The board holds this workload at its power cap by lowering the clock, so both belong beside the rate."""
    import glob
    import subprocess
    import threading
    pfiles = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") + \
        glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
    cfiles = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")
    watts, clocks, stop = [], [], threading.Event()

    def read_int(path):
        try:
            return int(open(path).read().strip())
        except (OSError, ValueError):
            return None

    def sampler():
        t_start = time.perf_counter()
        asked = False
        while not stop.is_set():
            if time.perf_counter() - t_start > 0.8 and pfiles:
                v = read_int(pfiles[0])
                if v:
                    watts.append(v / 1e6)
            if time.perf_counter() - t_start > 1.2 and not asked:
                asked = True
                try:
                    o = subprocess.run(["amd-smi", "metric", "-c"], capture_output=True, text=True, timeout=10).stdout
                    for line in o.splitlines():
                        f = line.split()
                        if len(f) >= 3 and f[0] == "CLK:" and f[1].isdigit() and len(clocks) < 8:
                            clocks.append(int(f[1]))             # the first 8 entries are the GFX (XCD) clocks
                except (OSError, subprocess.SubprocessError):
                    pass
            time.sleep(0.1)

    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        n += 10
    dt = time.perf_counter() - t0
    stop.set()
    th.join()
    cap = read_int(cfiles[0]) if cfiles else None
    return {"ms_per_step_sustained": dt * 1e3 / n, "steps": n,
            "socket_w_mean": sum(watts) / len(watts) if watts else None, "socket_w_max": max(watts) if watts else None,
            "cap_w": cap / 1e6 if cap else None,
            "gfx_clk_mhz_mean": sum(clocks) / len(clocks) if clocks else None, "gfx_clk_mhz_max_state": 2400}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="full_60s_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="add per-launch timings (one extra instrumented step)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the playback-window / similarity-filter / crossfade timings (profiling runs: only the decode steps)")
    ap.add_argument("--power", action="store_true",
                    help="add 3 s of back-to-back steps with the socket power (hwmon) and shader clock (amd-smi) read beside them")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus N with N > 1 is not supported "
                 "(windows and clips shard without communication, see DESIGN.md)")

    import numpy as np
    import torch
    import demon_inputs as di
    from paper_2605_28657_amd import DemonVAE

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    wl = di.WORKLOADS[args.workload]
    spec = wl.spec
    dtype = "bf16" if wl.bf16 else "f32"
    weights, lat = di.workload_inputs(wl)
    S = spec.total_stride
    halo = 6 if spec is di.FULL else 15
    n_windows = wl.n_clips * -(-wl.n_frames // wl.window)
    ext = n_windows * (wl.window + 2 * halo)
    vae = DemonVAE(spec, weights, dtype=dtype, max_frames=wl.n_frames, max_clips=wl.n_clips,
                   max_extended_frames=max(ext, wl.n_frames * wl.n_clips))
    assert max(vae.receptive_field()) == halo
    z = torch.from_numpy(lat).to("cuda:0")
    z = z.to(torch.bfloat16).contiguous() if wl.bf16 else z.contiguous()
    out = torch.empty((wl.n_clips, spec.out_channels, wl.n_frames * S), dtype=torch.float32, device="cuda:0")

    def step():
        vae.decode_windowed(z, window=wl.window, halo=-1, out=out)

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst

    # group-level HIP events (5 per step, on the decode stream) stay on during the timed region
    vae.set_timing(1)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    vae.get_timing()                                   # drop the warm-up steps from the event average
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    groups = np.array(vae.get_timing())                # average over the timed steps (the last 32 at most)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    audio_s = wl.n_clips * wl.n_frames / 25.0

    conv_f, head_f = conv_flops_per_frame(spec)
    frames = wl.n_clips * wl.n_frames
    n_conv_launches = sum(1 + 2 * len(spec.dilations) for _ in spec.strides)
    conv_ms = float(groups[1])
    achieved = conv_f * frames / (conv_ms * 1e-3) / 1e12
    result = {
        "metric": "audio_seconds_decoded_per_second",
        "value": audio_s / (ms_per_step * 1e-3),
        "unit": "audio-s/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_60s_clip": ms_per_step * 60.0 / audio_s,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": args.workload, "latent": [wl.n_clips, spec.latent_channels, wl.n_frames],
                   "window": wl.window, "halo": halo, "n_windows": n_windows,
                   "strides": list(spec.strides), "widths": list(spec.widths),
                   # the 16-bit formats of the bf16 path (bf16 and f16 MFMA have the same peak rate)
                   "operands": ("weights: bf16 values; activation operands: bf16 below 512 channels, IEEE half from 512 "
                                "channels on (f16 MFMA); fp32 accumulation; residual stream stored as IEEE half")
                   if wl.bf16 else "fp32"},
        "roofline": {
            "kernel": "MFMA convolution kernels (conv_mfma_kernel, res_unit_wide_kernel, res_unit_fused_kernel): all %d "
                      "convolution layers of a step, launched once per window group (two groups on two streams)" % n_conv_launches,
            "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_TFLOPS,
            # L2 miss traffic of these kernels per step from rocprofv3 FETCH_SIZE + WRITE_SIZE (bytes, scaled by a plain
            # copy), read from profiles/<workload>_hbm_traffic.txt; null where no such profile is committed
            "traffic": measured_traffic(args.workload),
            "algorithmic_flop": conv_f * frames,
            "time_ms": conv_ms,
        },
        "stage_ms": {"gather": float(groups[0]), "convolutions": conv_ms, "head": float(groups[2]),
                     "stitch": float(groups[3])},
    }
    # HBM-bound kernels: algorithmic bytes = what must be read plus what must be written.  The head reads the
    # interior rows of the last residual stream (half precision on the bf16 path) once and writes the window waveforms.
    rows = frames * S
    head_bytes = rows * spec.widths[-1] * (2 if wl.bf16 else 4) + rows * spec.out_channels * 4
    stitch_bytes = 2 * rows * spec.out_channels * 4
    result["hbm_kernels"] = {
        "stitch": {"GB/s": stitch_bytes / (groups[3] * 1e-3) / 1e9, "frac": stitch_bytes / (groups[3] * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }
    if groups[2] > 2e-2:
        result["hbm_kernels"]["head"] = {"GB/s": head_bytes / (groups[2] * 1e-3) / 1e9,
                                         "frac": head_bytes / (groups[2] * 1e-3) / 1e9 / PEAK_HBM_GBS}
    else:
        # calls of a few windows run the head inside the last residual unit's kernel: no launch of its own
        result["hbm_kernels"]["head"] = {"note": "ran inside the last 64-channel unit's kernel (counted under convolutions)"}

    if args.detail:
        vae.set_timing(2)
        step()
        torch.cuda.synchronize()
        t = vae.get_timing()
        names = ["gather"]
        for l in range(len(spec.strides)):
            names.append(f"b{l}.up")
            for j in range(len(spec.dilations)):
                names += [f"b{l}.r{j}.conv{spec.res_kernel}", f"b{l}.r{j}.conv1"]
        names += ["head", "stitch"]
        result["launch_ms"] = dict(zip(names, [round(x, 4) for x in t]))
        result["layers"] = layer_table(spec, wl, result["launch_ms"])
    vae.set_timing(0)

    if not args.no_extras:
        # every step on its own (synchronised before and after): median and fastest of 20
        singles = []
        for _ in range(20):
            torch.cuda.synchronize()
            s0 = time.perf_counter()
            step()
            torch.cuda.synchronize()
            singles.append((time.perf_counter() - s0) * 1e3)
        result["ms_per_step_single"] = {"median": float(np.median(singles)), "min": float(np.min(singles))}
        # what a plain device copy reaches on this GPU (256 MiB read + 256 MiB written per call): the HBM fractions above
        # can be read against it as well as against the published 8 TB/s
        src = torch.empty(1 << 26, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        s0 = time.perf_counter()
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        copy_gbs = 20 * 2 * src.numel() * 4 / (time.perf_counter() - s0) / 1e9
        result["hbm_kernels"]["device_copy_256MiB"] = {"GB/s": copy_gbs, "frac": copy_gbs / PEAK_HBM_GBS}
        del src, dst

        # Latency of re-decoding one playback window (3 s = 75 latent frames in the middle of the clip, analytic halo)
        # into the resident waveform buffer: the call the paper's 8x windowed-decode figure is about (section 3.6).
        pw = min(75, wl.n_frames)
        pb = max(0, (wl.n_frames - pw) // 2)
        for _ in range(3):
            vae.decode_windowed(z, window=pw, halo=-1, frame_begin=pb, frame_end=pb + pw, out=out)
        torch.cuda.synchronize()
        reps = 50
        p0 = time.perf_counter()
        for _ in range(reps):
            vae.decode_windowed(z, window=pw, halo=-1, frame_begin=pb, frame_end=pb + pw, out=out)
        torch.cuda.synchronize()
        pw_ms = (time.perf_counter() - p0) * 1e3 / reps
        result["playback_window"] = {"frames": pw, "audio_s": pw / 25.0, "ms": pw_ms,
                                     "speedup_vs_whole_clip_decode": ms_per_step / wl.n_clips / pw_ms}
        # a window that moves by one frame per call: a new window grid (table upload on the stream) every call
        p0 = time.perf_counter()
        for i in range(reps):
            b = (pb + i) % max(1, wl.n_frames - pw)
            vae.decode_windowed(z, window=pw, halo=-1, frame_begin=b, frame_end=b + pw, out=out)
        torch.cuda.synchronize()
        result["playback_window"]["ms_moving_window"] = (time.perf_counter() - p0) * 1e3 / reps
        # the same call captured once into a HIP graph and replayed (31 launches per replay, no host work in between)
        vae.decode_windowed(z, window=pw, halo=-1, frame_begin=pb, frame_end=pb + pw, out=out)     # its grid must be cached
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            vae.decode_windowed(z, window=pw, halo=-1, frame_begin=pb, frame_end=pb + pw, out=out)
        graph.replay()
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        result["playback_window"]["ms_graph_replay"] = (time.perf_counter() - p0) * 1e3 / reps
        del graph

        # the two small kernels around the playback-window decode: similarity gate on the whole latent, 50 ms crossfade
        import paper_2605_28657_amd as pa
        z_prev = z.clone()
        tail = out[0, :, :2400]
        headv = out[0, :, 2400:4800]
        xf = torch.empty((spec.out_channels, 2400), dtype=torch.float32, device="cuda:0")
        small = {}
        for name, fn in (("similarity_filter", lambda: pa.latent_similarity(z, z_prev, 1e-3)),
                         ("crossfade_50ms", lambda: pa.crossfade(tail, headv, out=xf))):
            fn(); torch.cuda.synchronize()
            q0 = time.perf_counter()
            for _ in range(200):
                fn()
            torch.cuda.synchronize()
            small[name + "_ms"] = (time.perf_counter() - q0) * 1e3 / 200
        # the playback-window decode behind the gate, flags read on the device: decoded (flag 0) and skipped (flag 1)
        for name, flags in (("gated_decoded", torch.zeros(wl.n_clips, dtype=torch.int32, device="cuda:0")),
                            ("gated_skipped", torch.ones(wl.n_clips, dtype=torch.int32, device="cuda:0"))):
            fn = lambda: vae.decode_windowed_gated(z, flags, out, window=pw, halo=-1, frame_begin=pb, frame_end=pb + pw)
            fn(); torch.cuda.synchronize()
            q0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            small[name + "_ms"] = (time.perf_counter() - q0) * 1e3 / reps
        result["playback_window"].update(small)

    if not args.no_extras and wl.bf16:
        # the alternative that stays within bf16 operands on the wide levels (hi + lo pairs, two MFMAs per k-step there)
        v2 = DemonVAE(spec, weights, dtype=dtype, max_frames=wl.n_frames, max_clips=wl.n_clips,
                      max_extended_frames=max(ext, wl.n_frames * wl.n_clips), wide_operands=2)
        v2.set_timing(1)
        for _ in range(3):
            v2.decode_windowed(z, window=wl.window, halo=-1, out=out)
        torch.cuda.synchronize()
        v2.get_timing()
        q0 = time.perf_counter()
        for _ in range(args.steps):
            v2.decode_windowed(z, window=wl.window, halo=-1, out=out)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - q0) * 1e3 / args.steps
        conv2 = float(v2.get_timing()[1])
        result["operands_bf16x2"] = {"ms_per_step": ms2, "conv_ms": conv2,
                                     "roofline_frac": conv_f * frames / (conv2 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                     "note": "wide_operands = 2: hi + lo bf16 pairs instead of IEEE half operands from 512 channels on"}
        v2.close()
        step(); torch.cuda.synchronize()               # `out` holds the default path's waveform again

        # the mirror path: windowed encode of the same shape (waveform -> moments + sampled latent), section 3.7 / Table III
        from paper_2605_28657_amd import DemonVAEEncoder
        enc_w = di.make_encoder_weights(spec, bf16=True)
        enc = DemonVAEEncoder(spec, enc_w, dtype=dtype, max_frames=wl.n_frames, max_clips=wl.n_clips,
                              max_extended_frames=max(ext, wl.n_frames * wl.n_clips))
        wave = torch.from_numpy(np.stack([di.make_waveform(spec.out_channels, wl.n_frames * S, 40 + i) for i in range(wl.n_clips)])).to("cuda:0")
        eps = torch.from_numpy(np.stack([di.make_noise(spec.latent_channels, wl.n_frames, 70 + i) for i in range(wl.n_clips)])).to("cuda:0")
        mom = torch.empty((wl.n_clips, 2 * spec.latent_channels, wl.n_frames), dtype=torch.float32, device="cuda:0")
        zl = torch.empty((wl.n_clips, spec.latent_channels, wl.n_frames), dtype=enc.latent_dtype, device="cuda:0")
        enc.set_timing(1)
        for _ in range(3):
            enc.encode_windowed(wave, window=wl.window, halo=-1, eps=eps, moments=mom, latent=zl)
        torch.cuda.synchronize()
        enc.get_timing()
        q0 = time.perf_counter()
        for _ in range(args.steps):
            enc.encode_windowed(wave, window=wl.window, halo=-1, eps=eps, moments=mom, latent=zl)
        torch.cuda.synchronize()
        ems = (time.perf_counter() - q0) * 1e3 / args.steps
        eg = enc.get_timing()
        # the encoder's convolutions: the decoder's, with the first transposed conv (C0 -> C1) replaced by a strided conv to 2 C0
        enc_f = conv_f + 2 * spec.strides[0] * 2 * spec.latent_channels * spec.widths[0]
        result["encode"] = {"ms_per_step": ems, "audio_s_per_s": audio_s / (ems * 1e-3),
                            "stage_ms": {"stem": float(eg[0]), "convolutions": float(eg[1]), "sampling_step": float(eg[2])},
                            "roofline_frac": enc_f * frames / (float(eg[1]) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                            "algorithmic_flop": enc_f * frames,
                            "config": "windowed encode of the same shape: %d windows of %d frames + halo 6, one batch" % (n_windows, wl.window)}
        if args.detail:
            enc.set_timing(2)
            enc.encode_windowed(wave, window=wl.window, halo=-1, eps=eps, moments=mom, latent=zl)
            torch.cuda.synchronize()
            names = ["stem"]
            for l in range(len(spec.strides) - 1, -1, -1):
                for j in range(len(spec.dilations)):
                    names += [f"e{l}.r{j}.conv{spec.res_kernel}", f"e{l}.r{j}.conv1"]
                names.append(f"e{l}.down")
            names.append("sampling_step")
            result["encode"]["launch_ms"] = dict(zip(names, [round(x, 4) for x in enc.get_timing()]))
        enc.close()
        del wave, eps, mom, zl

    if not args.no_extras:
        result["mfma_probe"] = mfma_probe_rates()

    if args.power:
        result["power"] = sustained_power(step, torch)

    if not args.no_cpu_baseline:
        # The oracle (fp32 build, as it stands) beside the GPU, on a bounded sample of this workload's own inputs: the
        # whole 10 s clip of the same decoder (configs[1]) on all host cores, and a 2 s clip on one thread.
        import oracle
        os.environ.pop("OMP_DYNAMIC", None)
        wl1 = di.WORKLOADS["full_10s_bf16"] if spec is di.FULL else wl
        w1, lat1 = di.workload_inputs(wl1)
        c0 = time.perf_counter()
        ref = oracle.decode(wl1.spec, w1, lat1[0], dtype=np.float32)
        c1 = time.perf_counter()
        secs = wl1.n_frames / 25.0
        cb = {"value": secs / (c1 - c0), "unit": "audio-s/s", "cores": oracle.omp_threads(), "kind": "oracle",
              "sample": f"fp32 oracle, full decode of the whole {secs:.0f} s clip ({wl1.name}: latent {wl1.spec.latent_channels} x "
                        f"{wl1.n_frames}) in {c1 - c0:.2f} s on {oracle.omp_threads()} threads",
              "GFLOP/s": (conv_flops_per_frame(wl1.spec)[0] + conv_flops_per_frame(wl1.spec)[1]) * wl1.n_frames / (c1 - c0) / 1e9}
        if wl1 is not wl and wl.n_clips == 1:
            # the GPU's result on the same frames of this run's clip differs from the 10 s clip's (another latent): compare on
            # the first second of THIS workload instead
            e1 = min(25, wl.n_frames)
            r1 = oracle.decode(spec, weights, lat[0][:, :min(wl.n_frames, e1 + halo)], dtype=np.float32)
            cb["gpu_vs_oracle_max_abs_on_first_second"] = float(np.abs(out[0, :, :e1 * S].cpu().numpy() - r1[:, :e1 * S]).max())
        # one thread, 2 s of audio (ctypes releases the GIL but the loops are OpenMP: a fresh process with one thread)
        import subprocess
        code = ("import time, numpy as np, demon_inputs as di, oracle\n"
                f"wl = di.WORKLOADS[{wl1.name!r}]; w, lat = di.workload_inputs(wl)\n"
                "z = lat[0][:, :50]\n"
                "t = time.perf_counter(); oracle.decode(wl.spec, w, z, dtype=np.float32); print(time.perf_counter() - t)\n")
        try:
            r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=dict(os.environ, OMP_NUM_THREADS="1"),
                               capture_output=True, text=True, timeout=300)
            t1 = float(r.stdout.strip().splitlines()[-1])
            cb["one_thread"] = {"value": 2.0 / t1, "unit": "audio-s/s", "sample": f"the first 2 s of the same clip in {t1:.2f} s on 1 thread"}
        except Exception as ex:                                       # noqa: BLE001 -- the baseline is a report, not a gate
            cb["one_thread"] = {"error": str(ex)[:200]}
        result["cpu_baseline"] = cb
    vae.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
