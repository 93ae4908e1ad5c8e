"""Allocation report for one of the synthetic ensemble configurations on one MI355X.

    python -m paper_2208_14049_amd.report --config 3

Plans the allocation matrix three ways, as the paper's evaluation does (section "Experimental results"):
the baseline that only tunes each member's batch size with one worker per member (BBS), Algorithm 1
alone (worst-fit-decreasing at the default batch size) and Algorithm 1 followed by Algorithm 2 (bounded
greedy over instances and batch sizes).  Every matrix is then timed again on the same request
(images resident in HBM) and, for the planned one, with host-resident images (the PCIe-inclusive
rate), and the latency of single small requests (1 to 128 images) under the planned matrix.  Prints one
JSON object per line.  With --member M only that member runs, alone at --batch, and its kernel classes
are listed.  With --grid (config 5: one ResNet-50) it also times every
cell of the instances x batch-size grid.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def matrix_of(alloc):
    return [[alloc.batch[r][c] for c in range(alloc.cols)] for r in range(alloc.rows)]


def timed_predict(E, images, out, repeats):
    import torch
    E.ens_predict(images, out)
    torch.cuda.synchronize()
    times = []
    for _ in range(repeats):
        t0 = time.perf_counter()
        E.ens_predict(images, out)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    times.sort()
    return images.shape[0] / times[len(times) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2, help="configuration 2..9 (7, 8, 9: the paper's IMN1, IMN4, IMN12 ensembles as shapes)")
    ap.add_argument("--images", type=int, default=1024)
    ap.add_argument("--slots", type=int, default=2, help="instance slots (rows of the matrix) the greedy search may use")
    ap.add_argument("--max-neighs", type=int, default=32)
    ap.add_argument("--max-iter", type=int, default=6)
    ap.add_argument("--default-batch", type=int, default=0,
                    help="batch size Algorithm 1 places every member at (0: the smallest of the domain)")
    ap.add_argument("--n-calib", type=int, default=512)
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--grid", action="store_true", help="time every (instances, batch size) cell (single-member configs)")
    ap.add_argument("--member", type=int, default=-1,
                    help="run only this member of the configuration, alone, at --batch, and print its per-kernel times")
    ap.add_argument("--batch", type=int, default=64)
    args = ap.parse_args()

    import torch
    import paper_2208_14049_amd as ens
    import synth
    from synth import nets as N, weights as W
    assert torch.cuda.is_available(), "the report needs the GPU"
    ens.lib()

    nets = N.config_members(args.config)
    if args.member >= 0:
        nets = [nets[args.member]]
    blobs = [W.quantise_weights_bf16(n, W.make_blob(n, synth.BASE_SEED, i)) if n.dtype == "bf16"
             else W.make_blob(n, synth.BASE_SEED, i) for i, n in enumerate(nets)]
    E = ens.Ensemble(nets, blobs)
    E.set_base_size(224, 224)
    n = args.images
    g = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + 1000)
    images = torch.randn((n, 224, 224, 3), generator=g, device="cuda", dtype=torch.float32)
    out = torch.empty((n, E.classes), device="cuda", dtype=torch.float32)
    common = dict(n_calib=args.n_calib, repeats=2, verbose=1)
    say = lambda **kw: print(json.dumps(kw), flush=True)
    say(config=args.config, members=[m.name for m in nets], images=n)
    if args.member >= 0:                                         # one member alone: throughput and kernel classes
        E.ens_set_alloc([[args.batch]])
        ips = timed_predict(E, images, out, args.repeats)
        say(member=nets[0].name, batch=args.batch, images_per_s=round(ips, 1),
            tflops=round(2.0 * nets[0].macs() * ips / 1e12, 1))
        E.ens_set_profiling(1)
        E.ens_predict(images, out)
        for c in sorted(E.ens_profile(), key=lambda c: -c["ms"]):
            if c["launches"]:
                say(kernel=c["name"], ms=round(c["ms"], 3), launches=c["launches"],
                    us_per_launch=round(1e3 * c["ms"] / c["launches"], 1),
                    tflops=round(c["flop"] / max(c["ms"], 1e-9) / 1e9, 1), gbs=round(c["bytes"] / max(c["ms"], 1e-9) / 1e6, 1))
        E.close()
        return

    results = {}
    db = dict(default_batch=args.default_batch) if args.default_batch > 0 else {}
    for label, opts in (("bbs", dict(strategy=2)),
                        ("wfd", dict(strategy=1, **db)),
                        ("greedy", dict(strategy=0, slots=args.slots, max_neighs=args.max_neighs,
                                        max_iter=args.max_iter, seed=synth.BASE_SEED, **db))):
        t0 = time.perf_counter()
        a = E.ens_plan(0, **opts, **common)
        plan_s = time.perf_counter() - t0
        m = matrix_of(a)
        ips = timed_predict(E, images, out, args.repeats)
        results[label] = ips
        say(strategy=label, allocation=m, planner_score=round(a.score, 1), benchmarks=a.n_bench,
            planning_seconds=round(plan_s, 1), device_bytes=a.bytes, images_per_s=round(ips, 1))
    host_images = images.cpu().pin_memory()
    host_out = torch.empty((n, E.classes), dtype=torch.float32).pin_memory()
    ips_host = timed_predict(E, host_images, host_out, args.repeats)
    say(strategy="greedy", input="host (pinned), output to host", images_per_s=round(ips_host, 1))
    # the paper's overhead experiment: every forward pass replaced by a prediction of zeros
    E.ens_debug_fake_predictor(1)
    ips_fake = timed_predict(E, images, out, args.repeats)
    E.ens_debug_fake_predictor(0)
    say(strategy="greedy", fake_predictor_seconds=round(n / ips_fake, 5), true_seconds=round(n / results["greedy"], 5),
        overhead_share=round(results["greedy"] / ips_fake, 4))
    say(allocation_speedup_vs_bbs=round(results["greedy"] / results["bbs"], 3),
        wfd_vs_bbs=round(results["wfd"] / results["bbs"], 3))
    # deploy mode on small requests (no request batching in front of the system): latency of one call
    for small in (1, 8, 32, 128):
        if small > n:
            break
        xs, ys = images[:small], out[:small]
        E.ens_predict(xs, ys)
        torch.cuda.synchronize()
        lat = []
        for _ in range(7):
            t0 = time.perf_counter()
            E.ens_predict(xs, ys)
            torch.cuda.synchronize()
            lat.append(time.perf_counter() - t0)
        lat.sort()
        say(strategy="greedy", request_images=small, latency_ms=round(1e3 * lat[len(lat) // 2], 3),
            images_per_s=round(small / lat[len(lat) // 2], 1))

    if args.grid:
        best = (0.0, None)
        for k in (1, 2, 4, 8):
            for b in (1, 4, 16, 64, 256):
                ips = E.ens_bench([[b] * len(nets) for _ in range(k)], n_calib=max(args.n_calib, 4 * b), repeats=2)
                say(instances=k, batch=b, images_per_s=round(ips, 1))
                if k == 1 and ips > best[0]:
                    best = (ips, b)
        say(best_single_instance_batch=best[1], images_per_s=round(best[0], 1),
            greedy_vs_best_single_instance=round(results["greedy"] / best[0], 3))
    E.close()


if __name__ == "__main__":
    main()
