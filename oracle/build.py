"""Builds oracle/liboracle.so (gcc, both precisions in one library).  Test infrastructure."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "demon_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    objs = []
    for tag, flag in (("f64", []), ("f32", ["-DORACLE_F32"])):
        obj = os.path.join(HERE, f"demon_oracle_{tag}.o")
        subprocess.check_call(["gcc", "-O2", "-ftree-vectorize", "-fno-fast-math", "-ffp-contract=off",
                               "-fopenmp", "-fPIC", "-std=c11", "-Wall", "-c", SRC, "-o", obj] + flag)
        objs.append(obj)
    subprocess.check_call(["gcc", "-shared", "-fopenmp", "-o", LIB] + objs + ["-lm"])
    for o in objs:
        os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
