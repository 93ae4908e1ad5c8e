"""Throughput of the ensemble hot path on one MI355X.

A step is one pass of the whole hot path (input staging, every member's forward pass on its
worker streams, fused softmax-and-mean) over one request of n synthetic images resident in HBM.
The headline workload is the heavy 12-member ensemble (the largest of the workload configurations
that one GPU holds); the other bf16 configurations are measured in the same run as sub-records.
Prints one JSON line: images per second (whole K steps), median and relative standard deviation of
the single steps, the rate with the images coming from pinned host memory, the roofline figures of
the dominant kernel (durations from HIP events attached to the dispatches on the worker streams),
per-kernel-class rates, and the CPU oracle's rate on the host cores.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

WORKLOADS = {
    2: "3 x ResNet-18-shaped ensemble",
    3: "heterogeneous 4-member ensemble: ResNet-50 (224), Inception-v3-shaped (299, resized in the library), "
       "EfficientNet-B0-shaped, DenseNet-121-shaped",
    4: "heavy 12-member ensemble co-located on one GPU: ResNet-50/101/152, EfficientNet-B0/B2/B4-shaped, "
       "DenseNet-121/169/201, 3 x Inception-v3-shaped",
    5: "single ResNet-50 served by data-parallel instances",
}
CPU_SAMPLE = {2: 16, 3: 16, 4: 12, 5: 16}      # images the oracle is timed on (about 10-30 s of CPU work)

# HBM bytes per launch of a kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised under
# profiles/ (scaled by the plain-copy calibration given there).  An entry describes the kernel sources
# with the digest recorded with it; with any other sources the figure is withheld (null).
TRAFFIC = {
    (4, "conv1x1_direct_bf16<128x128>"): dict(
        bytes_per_launch=97.2e6,                 # read + written (profiles/bench_config4_12members_b128.md)
        sources=["conv_pw.hip", "conv_direct.h", "conv_common.h", "kernels.h"],
        sha256="5119a20acf9c0b64cb2ad90a1e8a33ccbd2747c48b7645bd7fba83864d033d63"),
}


def sources_digest(names):
    import hashlib
    h = hashlib.sha256()
    for name in names:
        with open(os.path.join(ROOT, "paper_2208_14049_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_conv(name):
    return name.startswith(("conv", "bottleneck", "dense_layer", "stem"))


def progress(msg):
    """One line on stderr per finished phase (stdout carries the JSON line only)."""
    print("[bench] " + msg, file=sys.stderr, flush=True)


def measure(ens, cfg, n, steps, warmup, profile_steps, host_steps, matrix=None, segment=None):
    """Loads configuration `cfg`, installs its kept allocation and times `steps` requests of n images."""
    import torch
    import synth
    from synth import nets as N, weights as W
    nets = N.config_members(cfg)
    blobs = [W.quantise_weights_bf16(net, W.make_blob(net, synth.BASE_SEED, i)) for i, net in enumerate(nets)]
    with open(os.path.join(ROOT, "paper_2208_14049_amd", "allocations.json")) as f:
        kept = json.load(f)[str(cfg)]
    matrix = matrix or kept["matrix"]
    segment = segment or kept["segment"]
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc(matrix, segment)
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + 1000)
    images = torch.randn((n, 224, 224, 3), generator=g, device="cuda", dtype=torch.float32)
    out = torch.empty((n, E.classes), device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    for _ in range(warmup):
        E.ens_predict(images, out)
    torch.cuda.synchronize()
    progress("config %d: %d members loaded, %d warm-up steps done" % (cfg, len(nets), warmup))
    per_step = []
    t0 = time.perf_counter()
    for _ in range(steps):
        t1 = time.perf_counter()
        E.ens_predict(images, out)                              # synchronous: returns when Y is complete
        per_step.append(time.perf_counter() - t1)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    progress("config %d: %d timed steps, %.1f images/s" % (cfg, steps, n * steps / dt))
    rec = dict(workload=WORKLOADS[cfg], members=[net.name for net in nets], request_images=n, allocation=matrix,
               segment_size=segment, allocation_source=kept["source"],
               value=round(n * steps / dt, 1), ms_per_step=round(dt / steps * 1e3, 3),
               median_ms_per_step=round(statistics.median(per_step) * 1e3, 3),
               rsd_percent=round(100.0 * statistics.pstdev(per_step) / statistics.mean(per_step), 2) if steps > 1 else None)

    # images in pinned host memory, probabilities returned to host memory (PCIe-inclusive; never `value`)
    if host_steps > 0:
        h_img = torch.empty(images.shape, dtype=torch.float32, pin_memory=True)
        h_img.copy_(images)
        h_out = torch.empty(out.shape, dtype=torch.float32, pin_memory=True)
        E.ens_predict(h_img, h_out)
        ts = []
        for _ in range(host_steps):
            t1 = time.perf_counter()
            E.ens_predict(h_img, h_out)
            ts.append(time.perf_counter() - t1)
        rec["host_input_images_per_s"] = round(n / statistics.median(ts), 1)
        del h_img, h_out

    # per-kernel durations: the same launches, each with HIP events attached to its dispatch
    E.ens_set_profiling(1)
    prof = {}
    tp0 = time.perf_counter()
    for i in range(profile_steps):
        E.ens_predict(images, out)
        progress("config %d: profiled step %d of %d" % (cfg, i + 1, profile_steps))
        for c in E.ens_profile():
            if not c["launches"]:
                continue                             # a class some other batch size or pairing would use
            p = prof.setdefault(c["name"], dict(ms=0.0, launches=0, flop=0.0, bytes=0.0))
            for k in ("ms", "launches", "flop", "bytes"):
                p[k] += c[k]
    rec["profiled_ms_per_step"] = round((time.perf_counter() - tp0) / max(1, profile_steps) * 1e3, 3)
    # the same launches once more with every worker on one stream: each kernel alone on the GPU
    E.ens_debug_one_stream(1)
    E.ens_predict(images, out)
    alone = {c["name"]: c for c in E.ens_profile() if c["launches"]}
    E.ens_debug_one_stream(0)
    E.ens_set_profiling(0)
    total_ms = sum(v["ms"] for v in prof.values()) or 1.0
    conv_ms = sum(v["ms"] for k, v in prof.items() if is_conv(k)) or 1.0
    conv_flop = sum(v["flop"] for k, v in prof.items() if is_conv(k))
    rec["kernels"] = {
        k: dict(ms_per_step=round(v["ms"] / profile_steps, 4), launches=v["launches"] // profile_steps,
                share_of_kernel_time=round(v["ms"] / total_ms, 4),
                tflops=round(v["flop"] / max(v["ms"], 1e-9) / 1e9, 2),
                mfma_frac=round(v["flop"] / max(v["ms"], 1e-9) / 1e9 / PEAK_BF16_TFLOPS, 4) if is_conv(k) else None,
                gbs=round(v["bytes"] / max(v["ms"], 1e-9) / 1e6, 1),
                hbm_frac=round(v["bytes"] / max(v["ms"], 1e-9) / 1e6 / PEAK_HBM_GBS, 4),
                alone=None if k not in alone else dict(
                    avg_launch_us=round(alone[k]["ms"] * 1e3 / alone[k]["launches"], 2),
                    tflops=round(alone[k]["flop"] / max(alone[k]["ms"], 1e-9) / 1e9, 2),
                    gbs=round(alone[k]["bytes"] / max(alone[k]["ms"], 1e-9) / 1e6, 1)))
        for k, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"])}
    # all convolution launches together, on the sum of their own durations, and on the step's wall time
    rec["conv_mfma_frac_of_kernel_time"] = round(conv_flop / (conv_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
    rec["conv_mfma_frac_of_step"] = round(conv_flop / profile_steps / (dt / steps) / 1e12 / PEAK_BF16_TFLOPS, 4)
    dom_name, dom = max(prof.items(), key=lambda kv: kv[1]["ms"])
    # which roof bounds the dominant kernel: the matrix cores when its launches' algorithmic intensity
    # (flop per byte) lies above the ridge of the two peaks, HBM below it
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    intensity = dom["flop"] / max(dom["bytes"], 1.0)
    one = alone.get(dom_name)
    if is_conv(dom_name) and intensity >= ridge:
        achieved = dom["flop"] / (dom["ms"] * 1e-3) / 1e12
        roof = dict(bound="mfma", kernel=dom_name, achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_BF16_TFLOPS, 4))
        if one:
            a1 = one["flop"] / (one["ms"] * 1e-3) / 1e12
            roof["alone"] = dict(achieved=round(a1, 2), frac=round(a1 / PEAK_BF16_TFLOPS, 4),
                                 avg_launch_us=round(one["ms"] * 1e3 / one["launches"], 2))
    else:
        achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roof = dict(bound="hbm", kernel=dom_name, achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(achieved / PEAK_HBM_GBS, 4))
        if one:
            a1 = one["bytes"] / (one["ms"] * 1e-3) / 1e9
            roof["alone"] = dict(achieved=round(a1, 1), frac=round(a1 / PEAK_HBM_GBS, 4),
                                 avg_launch_us=round(one["ms"] * 1e3 / one["launches"], 2))
    roof["flop_per_byte"] = round(intensity, 1)
    traffic = None
    t = TRAFFIC.get((cfg, dom_name))
    if t and sources_digest(t["sources"]) == t["sha256"]:
        traffic = t["bytes_per_launch"]
    roof.update(traffic=traffic, flop_per_launch=round(dom["flop"] / max(1, dom["launches"]), 0),
                bytes_per_launch=round(dom["bytes"] / max(1, dom["launches"]), 0),
                avg_launch_us=round(dom["ms"] * 1e3 / max(1, dom["launches"]), 2),
                launches_per_step=dom["launches"] // profile_steps,
                share_of_kernel_time=round(dom["ms"] / total_ms, 4))
    rec["roofline"] = roof
    E.close()
    del images, out
    torch.cuda.empty_cache()
    return rec, nets, blobs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--images", type=int, default=1024)
    ap.add_argument("--config", type=int, default=4, choices=sorted(WORKLOADS), help="headline workload configuration")
    ap.add_argument("--others", default="2,3,5", help="configurations measured as sub-records ('' = none)")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="images the CPU oracle is timed on (0 = skip, -1 = the configuration's default)")
    ap.add_argument("--host-steps", type=int, default=3, help="extra steps with the images in pinned host memory (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path uses no second device (run with --gpus 1)")

    import torch
    import paper_2208_14049_amd as ens
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    ens.lib()
    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                                          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    psteps = max(1, min(3, args.steps))
    main_rec, nets, blobs = measure(ens, args.config, args.images, args.steps, args.warmup, psteps, args.host_steps)
    cpu = None
    ns = CPU_SAMPLE[args.config] if args.cpu_sample < 0 else args.cpu_sample
    if ns > 0:
        import oracle
        import synth
        from synth import weights as W
        x = W.make_images(synth.BASE_SEED + 1000, ns, 224, 224)
        oracle.forward_logits(nets[0], blobs[0], oracle.resize_bilinear(x[:1], nets[0].in_h, nets[0].in_w))   # loads the oracle library
        t0 = time.perf_counter()
        oracle.ensemble_predict(nets, blobs, x, real="f32")
        cdt = time.perf_counter() - t0
        progress("CPU oracle: %d images in %.1f s" % (ns, cdt))
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = dict(value=round(ns / cdt, 3), unit="images/s", cores=cores, kind="oracle",
                   sample="%d images of the request's distribution through all %d members" % (ns, len(nets)))
    del nets, blobs
    others = {}
    for c in [int(v) for v in args.others.split(",") if v.strip()]:
        if c == args.config:
            continue
        rec, _, _ = measure(ens, c, args.images, max(3, args.steps // 2), 1, 2, 2 if args.host_steps else 0)
        others[str(c)] = rec

    roofline = main_rec.pop("roofline")
    line = {
        "metric": "ensemble images/sec on 1 MI355X", "value": main_rec.pop("value"), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_rec.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config %d: %s; bf16, 1000 classes, 224x224x3 N(0,1) images, mean of softmax"
                               % (args.config, main_rec.pop("workload")),
                   "request_images": main_rec.pop("request_images"), "allocation": main_rec.pop("allocation"),
                   "segment_size": main_rec.pop("segment_size"), "allocation_source": main_rec.pop("allocation_source"),
                   "members": main_rec.pop("members"), "input": "fp32 NHWC resident in HBM",
                   "gpu_max_hw_queues": os.environ.get("GPU_MAX_HW_QUEUES", "unset (HIP default: 4)")},
        "median_ms_per_step": main_rec.pop("median_ms_per_step"), "rsd_percent": main_rec.pop("rsd_percent"),
        "host_input_images_per_s": main_rec.pop("host_input_images_per_s", None),
        "roofline": roofline, "cpu_baseline": cpu,
        "conv_mfma_frac_of_kernel_time": main_rec.pop("conv_mfma_frac_of_kernel_time"),
        "conv_mfma_frac_of_step": main_rec.pop("conv_mfma_frac_of_step"),
        "profiled_ms_per_step": main_rec.pop("profiled_ms_per_step"),
        "kernels": main_rec.pop("kernels"),
        "other_configs": others,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
