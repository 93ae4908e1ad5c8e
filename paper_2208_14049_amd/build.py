"""Builds the HIP library in-tree: hipcc for gfx950, one shared object next to this file."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libens_mi355x.so")
SOURCES = ["conv_mfma.hip", "conv_halo.hip", "conv_taps.hip", "conv_stempool.hip", "conv_wreg.hip", "conv_bneck.hip", "conv_pw.hip", "conv_dense.hip", "conv_regstage.hip", "layers.hip", "fc_mfma.hip", "static_scratch.hip", "member.cpp", "planner.cpp", "seedgen.cpp", "engine.cpp"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose=False):
    objs = []
    procs = []
    out_dir = os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(out_dir, src + ".o")
        cmd = ["hipcc"] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out = p.communicate()[0].decode()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write("hipcc failed on %s:\n%s\n" % (src, out))
        elif verbose and out.strip():
            print(src + ":\n" + out)
    if failed:
        raise RuntimeError("building the HIP library failed")
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-Wl,--no-undefined", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
