"""Compile the C oracle into oracle/libpvref_f64.so and oracle/libpvref_f32.so (gcc, OpenMP)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path(real="f64"):
    return os.path.join(HERE, f"libpvref_{real}.so")


def build(force=True):
    src = os.path.join(HERE, "ref_decoder.c")
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(real)
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
            subprocess.check_call(["gcc", "-O2", "-march=native", "-fopenmp", "-fno-fast-math",
                                   "-shared", "-fPIC", f"-DPV_REAL={ctype}", "-o", out, src, "-lm"])


if __name__ == "__main__":
    build()
