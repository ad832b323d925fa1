"""Launch-shape sweep for the update kernels on the GPU at hand.

    python -m paper_2005_06728_amd.tune --workload vgg16 --entry step --waves 0,2,3,4,5,6,8,-1

For each setting it re-creates the handle (the tuning variables are read by
odsgd_init), times the chosen entry point with HIP events and prints achieved
GB/s against the entry point's algorithmic bytes.  ODSGD_WAVES_PER_CU = 0 is
the library's own choice, -1 no residency cap.  Results never depend on these
settings, only speed does.
"""
import argparse
import itertools
import os

import torch

from . import binding as B
from . import workloads as wl

BYTES_PER_PARAM = {
    "step": lambda W: 8 * (W + 2),
    "ssgd": lambda W: 8 * (W + 2),
    "global": lambda W: 4 * (W + 4),
    "local": lambda W: 4 * (2 * W + 1),
}


def _call(eng, entry, hy, stream):
    if entry == "step":
        eng.step(hy, stream)
    elif entry == "ssgd":
        eng.ssgd_step(hy, stream)
    elif entry == "global":
        eng.global_update(hy, stream)
    else:
        eng.local_update(-1, hy, stream)


def time_entry(eng, entry, hy, steps, warmup):
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        _call(eng, entry, hy, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(steps):
        _call(eng, entry, hy, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="resnet50", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--workers", type=int, default=0, help="override the workload's worker count")
    ap.add_argument("--entry", default="step", choices=sorted(BYTES_PER_PARAM))
    ap.add_argument("--waves", default="0,2,3,4,5,6,8,12,-1", help="ODSGD_WAVES_PER_CU values")
    ap.add_argument("--chunks", default="256", help="ODSGD_CHUNK_ELEMS values")
    ap.add_argument("--layout", default="separate", choices=["separate", "arena"])
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    args = ap.parse_args()

    w = wl.WORKLOADS[args.workload]
    W = args.workers or w.num_workers
    st = wl.allocate(w, "cuda:0", num_workers=W, layout=args.layout, skew_bytes=0, align_elems=256)
    wl.fill_all_grads_(st, w, 0)
    hy = B.odsgd_hyper(*w.hyper)
    nbytes = BYTES_PER_PARAM[args.entry](W) * wl.total_params(w)
    saved = {k: os.environ.get(k) for k in ("ODSGD_WAVES_PER_CU", "ODSGD_CHUNK_ELEMS")}
    print("%s W=%d entry=%s layout=%s: %.4g algorithmic bytes per launch"
          % (args.workload, W, args.entry, args.layout, nbytes))
    try:
        for chunk, waves in itertools.product(args.chunks.split(","), args.waves.split(",")):
            os.environ["ODSGD_CHUNK_ELEMS"], os.environ["ODSGD_WAVES_PER_CU"] = chunk, waves
            eng = B.Engine(st["w"], st["v"], st["g"], st["u"])
            ms = time_entry(eng, args.entry, hy, args.steps, args.warmup)
            eng.close()
            print("chunk_elems=%-6s waves_per_cu=%-3s  %.4f ms  %7.1f GB/s  %.3f of 8 TB/s"
                  % (chunk, waves, ms, nbytes / ms / 1e6, nbytes / ms / 8e9), flush=True)
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


if __name__ == "__main__":
    main()
