"""Throughput of the ensemble hot path on one MI355X.

A step is one pass of the whole hot path (input staging, every member's forward pass on its
worker streams, fused softmax-and-mean) over one request of n synthetic images resident in HBM.
Prints one JSON line: images per second, the roofline figures of the dominant kernel (measured
with HIP events on the worker streams) and the CPU oracle's rate on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
os.environ.setdefault("GPU_MAX_HW_QUEUES", "8")   # one hardware queue per worker stream (before HIP starts)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised
# in profiles/bench_resnet18x3_b32.md (scaled by the plain-copy calibration given there).  They
# describe the kernel sources with the digest below; with any other sources the figure is withheld.
TRAFFIC = {
    "kernel": "conv3x3_halo_bf16<128,64,c64>",
    "bytes_per_launch": 80.4e6,
    "sources": ("conv_halo.hip", "conv_common.h", "kernels.h"),
    "sha256": "4c78a285f36902f3fcec5f9b15c63a10e0b3cac99aba0bd07050e84f26cebdf5",
}


def sources_digest(names):
    import hashlib
    h = hashlib.sha256()
    for name in names:
        with open(os.path.join(ROOT, "paper_2208_14049_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--images", type=int, default=1024)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--instances", type=int, default=2, help="workers per member (rows of the allocation matrix)")
    ap.add_argument("--cpu-sample", type=int, default=16, help="images the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path uses no second device (run with --gpus 1)")

    import numpy as np
    import torch
    import paper_2208_14049_amd as ens
    import synth
    from synth import nets as N, weights as W
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    ens.lib()

    nets = N.config_members(2)                                  # 3 x ResNet-18-shaped, bf16
    blobs = [W.quantise_weights_bf16(n, W.make_blob(n, synth.BASE_SEED, i)) for i, n in enumerate(nets)]
    E = ens.Ensemble(nets, blobs)
    alloc = [[args.batch] * len(nets) for _ in range(args.instances)]
    E.ens_set_alloc(alloc)
    n = args.images
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + 1000)
    images = torch.randn((n, 224, 224, 3), generator=g, device="cuda", dtype=torch.float32)
    out = torch.empty((n, E.classes), device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                                          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        E.ens_predict(images, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        E.ens_predict(images, out)                              # synchronous: returns when Y is complete
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = n * args.steps / dt

    # per-kernel durations: same launches, each bracketed by HIP events on its worker stream
    E.ens_set_profiling(1)
    prof = {}
    psteps = max(1, min(3, args.steps))
    tp0 = time.perf_counter()
    for _ in range(psteps):
        E.ens_predict(images, out)
        for c in E.ens_profile():
            if not c["launches"]:
                continue                             # a class some other batch size or pairing would use
            p = prof.setdefault(c["name"], dict(ms=0.0, launches=0, flop=0.0, bytes=0.0))
            for k in ("ms", "launches", "flop", "bytes"):
                p[k] += c[k]
    E.ens_set_profiling(0)
    profiled_ms_per_step = (time.perf_counter() - tp0) / psteps * 1e3
    dom_name, dom = max(prof.items(), key=lambda kv: kv[1]["ms"])
    achieved = dom["flop"] / (dom["ms"] * 1e-3) / 1e12 if dom["ms"] > 0 else 0.0
    traffic = None
    if dom_name == TRAFFIC["kernel"] and sources_digest(TRAFFIC["sources"]) == TRAFFIC["sha256"]:
        traffic = TRAFFIC["bytes_per_launch"]
    # The worker rows run on separate streams: with more than one row two launches share the GPU
    # and each takes longer than it would alone.  The same kernel timed with one row (its launches
    # alone on the GPU) is reported next to it.
    one_row = None
    if args.instances > 1:
        E.ens_set_alloc([[args.batch] * len(nets)])
        E.ens_predict(images, out)
        t1 = time.perf_counter()
        E.ens_predict(images, out)
        dt1 = time.perf_counter() - t1
        E.ens_set_profiling(1)
        E.ens_predict(images, out)
        for c in E.ens_profile():
            if c["name"] == dom_name and c["ms"] > 0:
                a1 = c["flop"] / (c["ms"] * 1e-3) / 1e12
                one_row = dict(achieved=round(a1, 2), frac=round(a1 / PEAK_BF16_TFLOPS, 4),
                               avg_launch_us=round(c["ms"] * 1e3 / max(1, c["launches"]), 2),
                               images_per_s=round(n / dt1, 1))
        E.ens_set_profiling(0)
    roofline = dict(bound="mfma", kernel=dom_name, achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / PEAK_BF16_TFLOPS, 4), traffic=traffic,
                    flop_per_launch=round(dom["flop"] / max(1, dom["launches"]), 0),
                    bytes_per_launch=round(dom["bytes"] / max(1, dom["launches"]), 0),
                    avg_launch_us=round(dom["ms"] * 1e3 / max(1, dom["launches"]), 2), one_row=one_row,
                    launches_per_step=dom["launches"] // psteps, profiled_ms_per_step=round(profiled_ms_per_step, 3),
                    kernels={k: dict(ms_per_step=round(v["ms"] / psteps, 4), launches=v["launches"] // psteps,
                                     tflops=round(v["flop"] / max(v["ms"], 1e-9) / 1e9, 2),
                                     gbs=round(v["bytes"] / max(v["ms"], 1e-9) / 1e6, 1)) for k, v in prof.items()})

    cpu = None
    if args.cpu_sample > 0:
        import oracle
        ns = args.cpu_sample
        x = images[:ns].cpu().numpy()
        oracle.forward_logits(nets[0], blobs[0], x[:1])          # loads the oracle library
        t0 = time.perf_counter()
        oracle.ensemble_predict(nets, blobs, x, real="f32")
        cdt = time.perf_counter() - t0
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = dict(value=round(ns / cdt, 3), unit="images/s", cores=cores, kind="oracle",
                   sample="%d of the %d request images through all %d members" % (ns, n, len(nets)))
    E.close()

    print(json.dumps({
        "metric": "ensemble images/sec on 1 MI355X", "value": round(value, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "3 x ResNet-18-shaped ensemble, 1000 classes, 224x224x3 N(0,1) images, "
                               "batch %d per member, mean of softmax" % args.batch,
                   "request_images": n, "allocation": alloc, "input": "fp32 NHWC resident in HBM"},
        "roofline": roofline, "cpu_baseline": cpu,
    }))


if __name__ == "__main__":
    main()
