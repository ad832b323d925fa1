"""Shared machinery of the GPU parity tests: run the HIP path (through the C ABI
binding) and the CPU oracle side by side on the same seeded inputs and compare
every output element."""
import numpy as np
import torch

from helpers import max_rel_err, same_bits
from oracle import odsgd_oracle as oracle
from paper_2005_06728_amd import binding as B

TOL = 1e-6  # max relative error bar for fp32 (the arithmetic is order-fixed, so bitwise equality is expected)


def to_host(lst):
    return [t.detach().cpu().numpy().copy() for t in lst]


def host_state(st):
    return {"w": to_host(st["w"]), "v": to_host(st["v"]),
            "g": [to_host(r) for r in st["g"]], "u": [to_host(r) for r in st["u"]]}


def refresh_host_grads(st, hs):
    for m in range(len(st["g"])):
        for k in range(len(st["g"][m])):
            hs["g"][m][k][...] = st["g"][m][k].cpu().numpy()


def compare(st, hs, what=("w", "v", "u"), label=""):
    """Element-by-element comparison GPU vs oracle. Returns (mismatching elements, max rel err)."""
    torch.cuda.synchronize()
    bad, worst = 0, 0.0
    pairs = []
    if "w" in what:
        pairs += list(zip(st["w"], hs["w"]))
    if "v" in what:
        pairs += list(zip(st["v"], hs["v"]))
    if "u" in what:
        for m in range(len(st["u"])):
            pairs += list(zip(st["u"][m], hs["u"][m]))
    for t, ref in pairs:
        x = t.cpu().numpy()
        if not same_bits(x, ref):
            nan_both = np.isnan(x) & np.isnan(ref)
            bad += int(np.sum((x.view(np.uint32) != ref.view(np.uint32)) & ~nan_both))
            finite = np.isfinite(ref) & np.isfinite(x)
            if np.any(finite):
                worst = max(worst, max_rel_err(x[finite], ref[finite]))
            if np.any(~finite & ~nan_both & (x != ref)):
                worst = float("inf")
    assert worst <= TOL, "%s max rel err %g (%d differing elements)" % (label, worst, bad)
    return bad, worst


def make_engine(st, warmup_steps=0):
    return B.Engine(st["w"], st["v"], st["g"], st["u"], warmup_steps=warmup_steps)


def hyper_tuple(h):
    return (h.lr, h.local_lr, h.momentum, h.weight_decay, h.grad_scale)


def f32(x):
    return float(np.float32(x))


def oracle_hyper(h):
    """The C ABI takes floats; hand the oracle the same binary32 values."""
    return dict(lr=f32(h[0]), local_lr=f32(h[1]), momentum=f32(h[2]),
                weight_decay=f32(h[3]), grad_scale=f32(h[4]))
