#!/usr/bin/env python3
"""Benchmark of the fused OD-SGD step on one MI355X.

A "step" is one pass of the whole update path over the resident state: W-way
gradient reduce + global momentum-SGD update + W local compensated updates, in
one launch (odsgd_step).  Inputs (weights, momentum, W gradient buffers) are in
HBM before the timed region starts.  The headline workload is the largest
parameter set, VGG-16-shaped with W = 16 (19.9 GB moved per step).

Prints ONE JSON line:
  value        params updated per second (N / wall time per step) on the headline set
  roofline     the headline set: algorithmic bytes 8*(W+2)*N per launch / mean
               kernel duration (HIP events on the launch stream, same K steps)
               against the 8 TB/s HBM peak
  roofline_by_workload   the same for each of the three roofline sets, back-to-back
               and with a cold last-level cache, and which of the two is the HBM rate
  cpu_baseline the CPU oracle timed on this host on a bounded sample
"""
import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
LAST_LEVEL_CACHE_BYTES = 256 << 20   # MI355X Infinity Cache
ROOFLINE_SETS = ("vgg16", "resnet50", "alexnet")
KERNEL_SOURCE = os.path.join(ROOT, "paper_2005_06728_amd", "csrc", "odsgd.hip")

PAPER_CONTEXT = {
    "note": "the paper reports end-to-end training speed only, never the update path; other hardware, context only",
    "resnet50_imagenet_90_epochs_4x(4xV100)_IB56": {"SSGD_hours": 10.5, "OD-SGD_hours": 9.2},
    "resnet18v2_cifar10_4_workers_K80_IB56_samples_per_s": {"SSGD": 236.78, "OD-SGD": 309.782},
    "mobilenet_mnist_4_workers_K80_10GbE_samples_per_s": {"SSGD": 236.63, "OD-SGD": 401.395},
}


def algorithmic_bytes(n_params, W):
    return 8 * (W + 2) * n_params


def device_code_sha256():
    """Hash of the device part of the kernel source file (everything above its "host side"
    marker): what a counter summary under profiles/ is valid for."""
    text = open(KERNEL_SOURCE, "rb").read()
    cut = text.find(b"\n// host side\n")
    return hashlib.sha256(text if cut < 0 else text[:cut]).hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch from the rocprofv3 counter summary under profiles/, if that summary
    was made from the kernel source this run times; otherwise null with the reason."""
    rel = os.path.join("profiles", "odsgd_step_%s.md" % workload)
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, "no counter summary %s" % rel
    text = open(path).read()
    m = re.search(r"measured HBM traffic per launch: ([0-9.eE+]+) bytes", text)
    sha = re.search(r"device code sha256: ([0-9a-f]{64})", text)
    if not m or not sha:
        return None, "%s holds no traffic figure" % rel
    now = device_code_sha256()
    if sha.group(1) != now:
        return None, "%s was measured on other device code (sha256 %s...)" % (rel, sha.group(1)[:12])
    return float(m.group(1)), "%s: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, scaled by the same counters on " \
                              "the 1 GiB copy probe; same device code (sha256 %s...)" % (rel, now[:12])


def launch_stats(ms, nbytes):
    mean = sum(ms) / len(ms)
    med = statistics.median(ms)
    return {"launches": len(ms), "kernel_ms_mean": mean, "kernel_ms_median": med, "kernel_ms_min": min(ms),
            "achieved": nbytes / (mean * 1e-3) / 1e9, "frac": nbytes / (mean * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "frac_at_median": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS}


def timed_launches(torch, fn, steps, warmup):
    """K back-to-back calls bracketed by synchronisation; HIP events on the launch stream around every call.
    Returns (wall ms per step, [kernel ms])."""
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        fn(stream)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events[0].record(stream)
    for i in range(steps):
        fn(stream)
        events[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, [events[i].elapsed_time(events[i + 1]) for i in range(steps)]


def cold_launches(torch, fn, steps=10, warmup=2):
    """Each launch timed alone after 2 GiB of unrelated device traffic, which evicts whatever
    the previous step left in the last-level cache: what a step sees when forward/backward
    ran in between."""
    stream = torch.cuda.current_stream()
    a, b = torch.zeros(1 << 28, device="cuda:0"), torch.zeros(1 << 28, device="cuda:0")
    out = []
    for i in range(warmup + steps):
        b.copy_(a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn(stream)
        e1.record(stream)
        torch.cuda.synchronize()
        if i >= warmup:
            out.append(e0.elapsed_time(e1))
    return out


def measure_workload(wl_mod, B, torch, name, steps, warmup, layout="separate", cold=True, probe=True):
    """Fused step on one parameter set: back-to-back, cold cache, and the arithmetic-free
    probe of the same access shape.  layout="separate": one torch allocation per tensor per
    role; layout="arena": each role packed into one flat bucket with tile-aligned tensor starts."""
    w = wl_mod.WORKLOADS[name]
    st = wl_mod.allocate(w, "cuda:0", layout=layout, skew_bytes=0, align_elems=256)
    wl_mod.fill_all_grads_(st, w, 0)
    eng = B.Engine(st["w"], st["v"], st["g"], st["u"])
    hy = B.odsgd_hyper(*w.hyper)
    N, W = wl_mod.total_params(w), w.num_workers
    nbytes = algorithmic_bytes(N, W)
    wall_ms, ms = timed_launches(torch, lambda s: eng.step(hy, s), steps, warmup)
    fits = 8 * N <= LAST_LEVEL_CACHE_BYTES
    r = {"workload": name, "tensors": len(w.tensors), "params": N, "workers": W,
         "algorithmic_bytes_per_launch": nbytes, "ms_per_step": wall_ms, "params_per_s": N / (wall_ms * 1e-3),
         "back_to_back": launch_stats(ms, nbytes),
         "w_and_momentum_bytes": 8 * N, "w_and_momentum_fit_last_level_cache": fits}
    if cold:
        r["cold_cache"] = launch_stats(cold_launches(torch, lambda s: eng.step(hy, s)), nbytes)
        r["cold_cache"]["how"] = "2 GiB device copy between launches, each launch timed alone"
    # which figure is an HBM rate: back-to-back steps re-read w and momentum (loaded through the
    # cache) from the 256 MB last-level cache when they fit, so only the cold figure is one then
    r["hbm_frac"] = r["cold_cache"]["frac"] if (fits and cold) else r["back_to_back"]["frac"]
    r["hbm_frac_is"] = "cold_cache" if (fits and cold) else "back_to_back"
    if probe:
        _, pms = timed_launches(torch, lambda s: eng.probe_streams(s), max(5, min(steps, 20)), 2)
        r["same_shape_copy_probe"] = launch_stats(pms, nbytes)
        r["frac_of_same_shape_copy_probe"] = r["back_to_back"]["achieved"] / r["same_shape_copy_probe"]["achieved"]
    eng.close()
    return r, st


def time_entry_points(wl_mod, B, torch, name, st, steps=15, warmup=3):
    """The other entry points and local updaters on the same resident state, each against its
    own algorithmic bytes per parameter, and the two halves of an iteration run on two streams."""
    w = wl_mod.WORKLOADS[name]
    W, N = w.num_workers, wl_mod.total_params(w)
    hy = B.odsgd_hyper(*w.hyper)
    state = [[torch.zeros_like(t) for t in st["w"]] for _ in range(W)]
    eng = B.Engine(st["w"], st["v"], st["g"], st["u"])
    cases = [
        ("odsgd_local_update(-1) sgd", 4 * (2 * W + 1), None, lambda s: eng.local_update(-1, hy, s)),
        ("odsgd_global_update", 4 * (W + 4), None, lambda s: eng.global_update(hy, s)),
        ("odsgd_ssgd_step", 8 * (W + 2), None, lambda s: eng.ssgd_step(hy, s)),
        ("odsgd_step dcasgd_c", 4 * (3 * W + 4), (B.ODSGD_LOCAL_DCASGD_C, 0.04, 0.0, 0.0, None),
         lambda s: eng.step(hy, s)),
        ("odsgd_step dcasgd_a", 4 * (5 * W + 4), (B.ODSGD_LOCAL_DCASGD_A, 2.0, 0.95, 1e-7, state),
         lambda s: eng.step(hy, s)),
        ("odsgd_step local momentum", 4 * (4 * W + 4), (B.ODSGD_LOCAL_SGD_MOMENTUM, 0.0, 0.0, 0.0, state),
         lambda s: eng.step(hy, s)),
    ]
    out = {}
    for label, bpp, rule, fn in cases:
        if rule is not None:
            eng.set_local_rule(rule[0], lam=rule[1], ms_decay=rule[2], epsilon=rule[3], mean_square=rule[4],
                               local_momentum=0.9)
        _, ms = timed_launches(torch, fn, steps, warmup)
        out[label] = dict(launch_stats(ms, bpp * N), bytes_per_param=bpp)
    eng.close()
    del state

    # split path: serial on one stream, then the two kernels on two streams at once
    # (out-of-place global update), each iteration against the split total 4*(3W+5) B/param
    eng = B.Engine(st["w"], st["v"], st["g"], st["u"])
    bpp = 4 * (3 * W + 5)

    def serial(s):
        eng.local_update(-1, hy, s)
        eng.global_update(hy, s)

    _, ms = timed_launches(torch, serial, steps, warmup)
    out["split, one stream: local_update(-1) then global_update"] = dict(launch_stats(ms, bpp * N), bytes_per_param=bpp)
    alt_w = [torch.empty_like(t) for t in st["w"]]
    alt_v = [torch.empty_like(t) for t in st["v"]]
    eng.set_double_buffer(alt_w, alt_v)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def concurrent(s):
        sa.wait_stream(s)
        sb.wait_stream(s)
        eng.local_update(-1, hy, sa)
        eng.global_update(hy, sb)
        s.wait_stream(sa)
        s.wait_stream(sb)

    _, ms = timed_launches(torch, concurrent, steps, warmup)
    out["split, two streams at once (out-of-place global update)"] = dict(launch_stats(ms, bpp * N),
                                                                          bytes_per_param=bpp)
    torch.cuda.synchronize()
    if eng.current_buffers:   # leave the current weights where the caller's tensors are
        eng.global_update(hy, main)
        torch.cuda.synchronize()
    eng.close()
    return out


def time_small(wl_mod, B, torch, name, steps=200, graph_len=20):
    """Launch-bound, cache-resident parameter sets: per-step time launched eagerly and
    as a captured HIP graph of graph_len steps.  The GB/s figure is effective (the
    whole state fits in on-chip cache), not an HBM rate."""
    w = wl_mod.WORKLOADS[name]
    st = wl_mod.allocate(w, "cuda:0")
    wl_mod.fill_all_grads_(st, w, 0)
    eng = B.Engine(st["w"], st["v"], st["g"], st["u"])
    hy = B.odsgd_hyper(*w.hyper)
    N, W = wl_mod.total_params(w), w.num_workers
    side = torch.cuda.Stream()
    out = {"params": N, "workers": W}
    with torch.cuda.stream(side):
        for _ in range(10):
            eng.step(hy, side)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        side.synchronize()
        ev[0].record(side)
        for _ in range(steps):
            eng.step(hy, side)
        ev[1].record(side)
        side.synchronize()
        out["eager_us_per_step"] = ev[0].elapsed_time(ev[1]) * 1e3 / steps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(graph_len):
                eng.step(hy, side)
        graph.replay()
        side.synchronize()
        ev[0].record(side)
        for _ in range(steps // graph_len):
            graph.replay()
        ev[1].record(side)
        side.synchronize()
        out["graph_us_per_step"] = ev[0].elapsed_time(ev[1]) * 1e3 / (steps // graph_len * graph_len)
    best = min(out["eager_us_per_step"], out["graph_us_per_step"])
    out["effective_gbps_not_hbm"] = algorithmic_bytes(N, W) / (best * 1e-6) / 1e9
    out["params_per_s"] = N / (best * 1e-6)
    eng.close()
    return out


def time_copy_probe(B, torch, steps, warmup, gib=1.0):
    """Plain copy of `gib` GiB (read) + `gib` GiB (write) per launch, one contiguous 1 KiB tile per wavefront."""
    n = int(gib * (1 << 30)) // 4
    src = torch.empty(n, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    _, ms = timed_launches(torch, lambda s: B.odsgd_probe_copy(dst, src, s), steps, warmup)
    assert torch.equal(dst, src)
    mean = sum(ms) / len(ms)
    return {"bytes_per_launch": 8 * n, "kernel_ms_mean": mean, "gbps": 8 * n / (mean * 1e-3) / 1e9}


def cpu_baseline(wl_mod, name, st, iterations=3):
    """Time the oracle, as it stands, on host copies of the same state: single thread (the
    reference definition), then the same routine over a static split of the flat element
    range, one thread per host core."""
    import numpy as np
    from oracle import odsgd_oracle as oracle
    w = wl_mod.WORKLOADS[name]
    hs = {k: [t.cpu().numpy() for t in st[k]] for k in ("w", "v")}
    hs["g"] = [[t.cpu().numpy() for t in r] for r in st["g"]]
    hs["u"] = [[t.cpu().numpy() for t in r] for r in st["u"]]
    hy = [float(np.float32(x)) for x in w.hyper]
    N, W = wl_mod.total_params(w), w.num_workers

    def timed(fn):
        t0 = time.perf_counter()
        fn()
        return time.perf_counter() - t0

    single = lambda: oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], *hy)
    timed(single)  # page in
    times = [timed(single) for _ in range(iterations)]
    t = statistics.median(times)
    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    multi = lambda: oracle.od_step_threads(hs["w"], hs["v"], hs["g"], hs["u"], *hy, threads=threads)
    timed(multi)
    times_mt = [timed(multi) for _ in range(max(3, iterations))]
    t_mt = statistics.median(times_mt)
    nbytes = algorithmic_bytes(N, W)
    return {"value": N / t, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": "%d full OD-SGD steps of the %s parameter set (N=%d, W=%d) after one untimed step, single "
                      "thread, median %.2f s each" % (iterations, name, N, W, t),
            "gbps": nbytes / t / 1e9,
            "all_cores": {"value": N / t_mt, "unit": "params/s", "cores": threads, "gbps": nbytes / t_mt / 1e9,
                          "speedup_over_one_core": t / t_mt,
                          "sample": "same step, flat element range split statically over %d POSIX threads "
                                    "(oracle/threads.c), median of %d" % (threads, len(times_mt))}}


def brief(r):
    keep = ("workload", "tensors", "params", "workers", "algorithmic_bytes_per_launch", "ms_per_step", "params_per_s",
            "back_to_back", "cold_cache", "hbm_frac", "hbm_frac_is", "w_and_momentum_bytes",
            "w_and_momentum_fit_last_level_cache", "same_shape_copy_probe", "frac_of_same_shape_copy_probe")
    return {k: r[k] for k in keep if k in r}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16")
    ap.add_argument("--others", default=None,
                    help="comma list of further roofline sets measured in the same run (default: the other "
                         "two of vgg16, resnet50, alexnet; '' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline workload's timed steps and the copy probe (what the rocprofv3 runs "
                         "use): no other workloads, layouts, entry points, cold-cache or CPU measurements")
    ap.add_argument("--with-cold", action="store_true",
                    help="with --headline-only: also time the headline workload with a cold last-level cache")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only the plain copy kernel of known traffic (counter calibration)")
    args = ap.parse_args()
    if args.others is None:
        args.others = ",".join(x for x in ROOFLINE_SETS if x != args.workload)
    if args.headline_only:
        args.others, args.no_cpu_baseline = "", True
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the W workers are W gradient buffers in "
                 "one HBM); --gpus %d is not supported, no multi-GPU figure exists" % args.gpus)

    import torch
    from paper_2005_06728_amd import binding as B
    from paper_2005_06728_amd import workloads as wl_mod
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    B.lib()  # fail loudly if the extension is missing

    if args.copy_probe:
        r = time_copy_probe(B, torch, args.steps, args.warmup)
        r["frac_of_peak"] = r["gbps"] / HBM_PEAK_GBPS
        print(json.dumps({"copy_probe": r}))
        return

    full = not args.headline_only
    head, st = measure_workload(wl_mod, B, torch, args.workload, args.steps, args.warmup,
                                cold=full or args.with_cold, probe=full)
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl_mod, args.workload, st)
    by_workload = {args.workload: brief(head)}
    entry_points = {}
    if full:
        entry_points[args.workload] = time_entry_points(wl_mod, B, torch, args.workload, st)
    del st
    torch.cuda.empty_cache()

    for name in [x for x in args.others.split(",") if x and x != args.workload]:
        r, st2 = measure_workload(wl_mod, B, torch, name, max(5, min(args.steps, 30)), args.warmup)
        by_workload[name] = brief(r)
        if name == "resnet50":
            entry_points[name] = time_entry_points(wl_mod, B, torch, name, st2)
        del st2
        torch.cuda.empty_cache()

    # the same fused step with every role packed into one flat bucket (the usual
    # gradient-bucket layout) instead of one allocation per tensor
    buckets = {}
    for name in ([] if not full else [args.workload] + [x for x in args.others.split(",") if x and x != args.workload]):
        r, st2 = measure_workload(wl_mod, B, torch, name, max(5, min(args.steps, 20)), args.warmup, layout="arena",
                                  cold=False, probe=False)
        del st2
        torch.cuda.empty_cache()
        buckets[name] = r["back_to_back"]

    small = {n: time_small(wl_mod, B, torch, n) for n in ("lenet5", "resnet20")} if full else {}
    probe = time_copy_probe(B, torch, 20, 3)
    w = wl_mod.WORKLOADS[args.workload]
    b2b = head["back_to_back"]
    traffic, traffic_source = measured_traffic(args.workload)
    line = {
        "metric": "params updated/sec per OD-SGD step (and achieved HBM GB/s, see roofline)",
        "value": head["params_per_s"],
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s-shaped parameter set" % args.workload, "tensors": head["tensors"],
                   "params": head["params"], "workers": head["workers"],
                   "hyper": dict(w.hyper._asdict()), "entry_point": "odsgd_step (fused, one launch)"},
        "roofline": {"bound": "hbm", "achieved": b2b["achieved"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": b2b["frac"],
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": head["algorithmic_bytes_per_launch"],
                     "kernel_ms_mean": b2b["kernel_ms_mean"], "kernel_ms_median": b2b["kernel_ms_median"],
                     "kernel_ms_min": b2b["kernel_ms_min"],
                     "plain_copy_gbps_same_box": probe["gbps"],
                     "note": "timed region = the K back-to-back steps; mean kernel duration from HIP events around "
                             "every launch on the launch stream. w and momentum of this set (%.0f MB) %s the 256 MB "
                             "last-level cache, so this back-to-back figure %s an HBM rate; see "
                             "roofline_by_workload for the cold-cache figures"
                             % (head["w_and_momentum_bytes"] / 1e6,
                                "fit" if head["w_and_momentum_fit_last_level_cache"] else "do not fit",
                                "is cache-assisted, not" if head["w_and_momentum_fit_last_level_cache"] else "is")},
        "roofline_by_workload": by_workload,
        "cpu_baseline": cpu,
        "other_entry_points": entry_points,
        "flat_bucket_layout": buckets,
        "launch_bound_workloads": small,
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
