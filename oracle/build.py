"""Compile the CPU oracle (plain C, fp64) into oracle/libvgg_ref.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "vgg_ref.c")
    out = os.path.join(HERE, "libvgg_ref.so")
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", out, src, "-lm"])
    return out


if __name__ == "__main__":
    print(build())
