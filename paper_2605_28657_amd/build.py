"""Builds libdemon_vae.so in-tree with hipcc for gfx950."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdemon_vae.so")
PROBE = os.path.join(HERE, "mfma_probe")        # stand-alone measurement aid (sustained MFMA rate), see csrc/mfma_probe.hip
SOURCES = ["host_plan.cpp", "api.hip", "kernels_io.hip", "kernels_f32.hip", "kernels_bf16.hip", "kernels_bf16_fused.hip", "kernels_bf16_wide.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-fvisibility=hidden", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA accumulators in ordinary VGPRs: the epilogues work on them with VALU instructions
         "-mllvm", "-amdgpu-mfma-vgpr-form"]


def _compile(src):
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc"] + FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build() -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    for o in objs:
        os.remove(o)
    build_probe()
    return LIB


def build_probe() -> str:
    cmd = ["hipcc"] + [f for f in FLAGS if f != "-fPIC"] + [os.path.join(CSRC, "mfma_probe.hip"), "-o", PROBE]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on mfma_probe.hip:\n" + r.stderr)
    return PROBE


if __name__ == "__main__":
    print(build())
