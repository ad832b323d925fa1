"""Randomised (seeded) configurations of the whole boundary against the oracle: tensor lists,
worker counts, alignments, local updaters, warm-up lengths, hyper-parameters and the mix of
entry points are drawn per seed; every output element is compared after every call."""
import numpy as np
import pytest
import torch

from gpu_harness import (DEV, Arena, arenas_intact, compare, custom_state, f32, host_state, oracle_hyper,
                         refresh_host_grads, regen_grads, say, to_host)
from helpers import same_bits
from oracle import odsgd_oracle as oracle
from paper_2005_06728_amd import binding as B

pytestmark = pytest.mark.gpu


def draw_sizes(rng):
    kinds = [lambda: int(rng.integers(0, 6)), lambda: int(rng.integers(6, 300)), lambda: int(rng.integers(300, 5000)),
             lambda: int(rng.integers(5000, 40000)), lambda: 16384 * int(rng.integers(1, 4)) + int(rng.integers(0, 600)),
             lambda: 256 * int(rng.integers(1, 40))]
    return [kinds[int(rng.integers(0, len(kinds)))]() for _ in range(int(rng.integers(1, 7)))]


@pytest.mark.parametrize("seed", range(36))
def test_random_configuration(seed):
    rng = np.random.default_rng(9000 + seed)
    sizes = draw_sizes(rng)
    if sum(sizes) == 0:
        sizes.append(17)
    W = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16, 19, 33]))
    layout = rng.choice(["plain", "blocks", "blocks_off", "shifted"])
    block_phase = None if layout in ("plain", "shifted") else int(rng.choice([0, 512, 1024, 4096, 48 * 1024 + 16]))
    shifts = {r: int(rng.integers(0, 4)) for r in ("w", "v", "g", "u")} if layout == "shifted" else None
    rule = rng.choice(["sgd", "c", "a", "m"])
    wp = int(rng.integers(0, 3))
    hy = (float(rng.choice([0.01, 0.1, 0.5])), float(rng.choice([0.01, 0.05, 0.3])), float(rng.choice([0.0, 0.5, 0.9])),
          float(rng.choice([0.0, 1e-4, 1e-2])), float(rng.choice([0.0, 1.0, 0.125])))
    say("seed %d: sizes=%s W=%d layout=%s phase=%s shifts=%s rule=%s wp=%d hyper=%s"
        % (seed, sizes, W, layout, block_phase, shifts, rule, wp, hy))
    st, arenas, gen = custom_state(sizes, W, seed=9000 + seed, shifts=shifts, block_phase=block_phase)
    for m in range(W):
        for k, t in enumerate(st["u"][m]):
            t.copy_(st["w"][k])
    state_phase = block_phase if layout == "blocks" else (None if block_phase is None else (block_phase + 2048) % 65536)
    ms_arenas = [Arena(sizes, block_phase=state_phase) for _ in range(W)] if rule in ("a", "m") else []
    ms = [a.views for a in ms_arenas]
    for r in ms:
        for t in r:
            t.zero_()
    hs = host_state(st)
    ms_h = [to_host(r) for r in ms]
    eng = B.Engine(st["w"], st["v"], st["g"], st["u"], warmup_steps=wp, static_plan=bool(rng.integers(0, 2)))
    orule = None
    if rule == "c":
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_C, lam=0.04)
        orule = ("dcasgd_c", f32(0.04))
    elif rule == "a":
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=2.0, ms_decay=0.95, epsilon=1e-7, mean_square=ms)
        orule = ("dcasgd_a", f32(2.0), f32(0.95), f32(1e-7), ms_h)
    elif rule == "m":
        eng.set_local_rule(B.ODSGD_LOCAL_SGD_MOMENTUM, local_momentum=0.9, local_velocity=ms)
        orule = ("momentum", f32(0.9), ms_h)
    oh = oracle_hyper(hy)

    def check(label):
        assert compare(st, hs, label="seed %d %s" % (seed, label))[0] == 0
        for m in range(len(ms)):
            for t, ref in zip(ms[m], ms_h[m]):
                assert same_bits(t.cpu().numpy(), ref), "seed %d %s: per-worker state" % (seed, label)

    for it in range(5):
        split = it >= wp and bool(rng.integers(0, 2))
        if split:
            order = list(rng.permutation(W)) if rng.integers(0, 2) else None
            if order is None:
                eng.local_update(-1, hy)
            else:
                for m in order:
                    eng.local_update(int(m), hy)
            eng.global_update(hy)
        else:
            eng.step(hy)
        kw = dict(rule=orule) if orule else {}
        oracle.step(it, wp, hs["w"], hs["v"], hs["g"], hs["u"], **kw, **oh)
        check("it %d (%s)" % (it, "split" if split else "fused"))
        regen_grads(st, gen, gstd=1e-2)
        refresh_host_grads(st, hs)
    assert eng.iteration == 5
    assert arenas_intact(arenas) and all(a.intact() for a in ms_arenas)
    eng.close()
