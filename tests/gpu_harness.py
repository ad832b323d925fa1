"""Shared machinery of the GPU parity tests: run the HIP path (through the C ABI
binding) and the CPU oracle side by side on the same seeded inputs and compare
every output element."""
import numpy as np
import torch

from helpers import max_rel_err, same_bits
from oracle import odsgd_oracle as oracle
from paper_2005_06728_amd import binding as B

DEV = "cuda:0"
CANARY = 1234.5
TOL = 1e-6  # max relative error bar for fp32 (the arithmetic is order-fixed, so bitwise equality is expected)


def say(msg):
    print(msg, flush=True)


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


# ---------------------------------------------------------------------------
# custom tensor lists inside guarded arenas
# ---------------------------------------------------------------------------
class Arena:
    """One flat buffer per role; tensors are views separated by canary gaps."""

    def __init__(self, sizes, shift=0, gap=64, block_phase=None):
        """block_phase: if given, the arena's layout starts at an address that is block_phase
        bytes past a 64 KiB boundary, so that arenas of equal layout put every tensor at the
        same offset from such a boundary (the condition for two-half tiles)."""
        offs, o = [], gap + shift
        for n in sizes:
            offs.append(o)
            o += ((n + 3) // 4) * 4 + gap  # next view starts 16-byte aligned (+ shift elements)
        total = o + gap + (16384 if block_phase is not None else 0)
        self.buf = torch.full((total,), CANARY, dtype=torch.float32, device=DEV)
        skip = 0
        if block_phase is not None:
            assert block_phase % 4 == 0 and self.buf.data_ptr() % 4 == 0
            skip = ((block_phase - self.buf.data_ptr()) % 65536) // 4
        self.views = [self.buf[skip + a:skip + a + n] for a, n in zip(offs, sizes)]
        self.mask = torch.ones(total, dtype=torch.bool, device=DEV)
        for a, n in zip(offs, sizes):
            self.mask[skip + a:skip + a + n] = False

    def intact(self):
        return bool(torch.all(self.buf[self.mask] == CANARY))


def custom_state(sizes, W, seed, shifts=None, wstd=0.05, gstd=1e-3, block_phase=None):
    """shifts: per-role element shift (0 = 16-byte aligned views, 1..3 = only 4-byte aligned).
    block_phase: see Arena."""
    shifts = shifts or {}
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    mk = lambda role: Arena(sizes, shifts.get(role, 0), block_phase=block_phase)
    arenas = {"w": mk("w"), "v": mk("v"), "g": [mk("g") for _ in range(W)], "u": [mk("u") for _ in range(W)]}
    st = {"w": arenas["w"].views, "v": arenas["v"].views,
          "g": [a.views for a in arenas["g"]], "u": [a.views for a in arenas["u"]]}
    for t in st["w"]:
        t.normal_(0, wstd, generator=gen)
    for t in st["v"]:
        t.normal_(0, 1e-3, generator=gen)
    for m in range(W):
        for t in st["g"][m]:
            t.normal_(0, gstd, generator=gen)
    return st, arenas, gen


def arenas_intact(arenas):
    return (arenas["w"].intact() and arenas["v"].intact()
            and all(a.intact() for a in arenas["g"]) and all(a.intact() for a in arenas["u"]))


def regen_grads(st, gen, gstd=1e-3):
    for r in st["g"]:
        for t in r:
            t.normal_(0, gstd, generator=gen)


RAGGED = [0, 1, 3, 4, 5, 255, 256, 257, 1023, 1024, 1025, 4096, 4097, 8191, 3 * 4096 + 7, 20000]
