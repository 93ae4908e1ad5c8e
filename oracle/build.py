"""Compile the C part of the CPU oracle (test infrastructure) with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(HERE, "_build")
SRC = os.path.join(HERE, "ens_oracle.c")


def lib_path(real):
    return os.path.join(OUT, "libens_oracle_%s.so" % real)


def build(force=False):
    os.makedirs(OUT, exist_ok=True)
    for real, ctype in (("f32", "float"), ("f64", "double")):
        dst = lib_path(real)
        if not force and os.path.exists(dst) and os.path.getmtime(dst) >= os.path.getmtime(SRC):
            continue
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-DREAL=" + ctype, SRC, "-o", dst, "-lm"])


if __name__ == "__main__":
    build(force=True)
