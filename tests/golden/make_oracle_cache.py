"""Writes the CPU oracle's per-member logits of the full-size parity cases (configurations 2-5).

Calls only `oracle/` (the forward pass and the resize) and `synth/` (the seeded inputs); no GPU
code is imported or run.  One file per configuration, `oracle_full_size/config<k>_logits.npy`:
float32 [members][n][classes], the oracle's fp32 logits as they are (it computes in fp32, so the
cast loses nothing).  The GPU parity tests load these files instead of re-running the oracle
(minutes per configuration) and recompute them in place when a file is missing.

    python tests/golden/make_oracle_cache.py [config ...]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle                                   # noqa: E402
from synth import requests as R                 # noqa: E402

OUT_DIR = os.path.join(HERE, "oracle_full_size")


def cache_path(cfg):
    return os.path.join(OUT_DIR, "config%d_logits.npy" % cfg)


def oracle_logits(nets, blobs, imgs, chunk=16, progress=None):
    """float32 [members][n][classes]: every member's fp32 logits on the request images, each member
    fed the images resized to its own resolution."""
    n = imgs.shape[0]
    out = np.zeros((len(nets), n, nets[0].classes), dtype=np.float32)
    for m, (net, blob) in enumerate(zip(nets, blobs)):
        t0 = time.time()
        for a in range(0, n, chunk):
            x = oracle.resize_bilinear(imgs[a:a + chunk], net.in_h, net.in_w)
            out[m, a:a + chunk] = oracle.forward_logits(net, blob, x, real="f32").astype(np.float32)
        if progress:
            progress("member %d (%s): %d images in %.0f s" % (m, net.name, n, time.time() - t0))
    return out


def load_or_make(cfg, write=False, progress=None):
    """The cached logits of configuration `cfg`, computed (and optionally stored) when absent."""
    path = cache_path(cfg)
    nets, blobs, imgs = R.full_size_case(cfg)
    if os.path.exists(path):
        z = np.load(path, allow_pickle=False)
        assert z.shape == (len(nets), imgs.shape[0], nets[0].classes) and z.dtype == np.float32, z.shape
        return nets, blobs, imgs, z
    z = oracle_logits(nets, blobs, imgs, progress=progress)
    if write:
        os.makedirs(OUT_DIR, exist_ok=True)
        np.save(path, z)
    return nets, blobs, imgs, z


def main():
    cfgs = [int(a) for a in sys.argv[1:]] or sorted(R.FULL_SIZE_N)
    for cfg in cfgs:
        if os.path.exists(cache_path(cfg)):
            os.remove(cache_path(cfg))
        t0 = time.time()
        say = lambda s: print("config %d: %s" % (cfg, s), flush=True)    # noqa: E731
        _, _, _, z = load_or_make(cfg, write=True, progress=say)
        say("wrote %s %s in %.0f s, logit std %.3f" % (cache_path(cfg), z.shape, time.time() - t0, float(z.std())))


if __name__ == "__main__":
    main()
