"""odsgd_init_static (chunk and pointer tables in the library's static device
array, nothing allocated) against odsgd_init (tables in a caller workspace):
the same seeded inputs go through both registrations and every output must be
bitwise equal, on two registrations in a row, the second with a smaller input
that leaves most of the previous tables behind in the array."""
import ctypes

import pytest
import torch

from gpu_harness import (RAGGED, Arena, arenas_intact, compare, custom_state, host_state, oracle_hyper,
                         refresh_host_grads, regen_grads, say)
from oracle import odsgd_oracle as oracle
from paper_2005_06728_amd import binding as B

pytestmark = pytest.mark.gpu

HY = (0.05, 0.02, 0.9, 1e-3, 0.0)


def equal_states(a, b):
    """Every output of the two registrations, element by element, bit for bit."""
    torch.cuda.synchronize()
    pairs = list(zip(a["w"], b["w"])) + list(zip(a["v"], b["v"]))
    for ra, rb in zip(a["u"], b["u"]):
        pairs += list(zip(ra, rb))
    return all(torch.equal(x.view(torch.int32), y.view(torch.int32)) for x, y in pairs)


def run_pair(sizes, W, seed):
    """All entry points on a workspace handle and on a static handle side by side;
    returns after closing both."""
    say("static vs workspace plan: W=%d sizes=%s" % (W, sizes))
    sa, arenas_a, gen_a = custom_state(sizes, W, seed=seed)
    sb, arenas_b, gen_b = custom_state(sizes, W, seed=seed)
    hs = host_state(sa)
    ea = B.Engine(sa["w"], sa["v"], sa["g"], sa["u"])
    eb = B.Engine(sb["w"], sb["v"], sb["g"], sb["u"], static_plan=True)
    assert eb.workspace is None
    oh = oracle_hyper(HY)

    def both(fn):
        fn(ea)
        fn(eb)

    def fresh_grads():
        regen_grads(sa, gen_a)
        regen_grads(sb, gen_b)

    both(lambda e: e.step(HY))
    assert equal_states(sa, sb), "fused step"
    # the workspace handle itself is checked against the oracle elsewhere; once here
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(sb, hs, label="static plan vs oracle")[0] == 0
    fresh_grads()
    both(lambda e: e.step(HY))
    assert equal_states(sa, sb), "second fused step"
    fresh_grads()
    both(lambda e: (e.local_update(-1, HY), e.global_update(HY)))
    assert equal_states(sa, sb), "local(all) + global"
    fresh_grads()
    both(lambda e: ([e.local_update(m, HY) for m in range(W)], e.global_update(HY)))
    assert equal_states(sa, sb), "local(m) + global"
    fresh_grads()
    both(lambda e: e.ssgd_step(HY))
    assert equal_states(sa, sb), "warm-up step"
    assert ea.iteration == eb.iteration == 5
    assert arenas_intact(arenas_a) and arenas_intact(arenas_b)
    ea.close()
    eb.close()


def test_two_static_registrations_in_a_row_second_one_smaller():
    run_pair(RAGGED + [300000], 8, seed=901)   # 1200 tiles, templated kernel
    run_pair([5000, 17, 1], 3, seed=902)       # a few tiles, generic worker loop, old tables left behind
    run_pair([70000, 255], 16, seed=903)       # larger again, widest pointer rows


def test_static_plan_with_per_worker_state():
    """odsgd_set_local_rule writes the state columns of the pointer table: into the static array here."""
    W, sizes = 4, [9000, 33]
    res = []
    for static in (False, True):
        st, _, gen = custom_state(sizes, W, seed=911)
        for m in range(W):
            for k, t in enumerate(st["u"][m]):
                t.copy_(st["w"][k])
        ms = [[torch.zeros_like(t) for t in st["w"]] for _ in range(W)]
        eng = B.Engine(st["w"], st["v"], st["g"], st["u"], static_plan=static)
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=2.0, ms_decay=0.95, epsilon=1e-7, mean_square=ms)
        for _ in range(3):
            eng.step(HY)
            regen_grads(st, gen, gstd=1e-2)
        torch.cuda.synchronize()
        eng.close()
        res.append((st, ms))
    assert equal_states(res[0][0], res[1][0])
    for ra, rb in zip(res[0][1], res[1][1]):
        for x, y in zip(ra, rb):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32))


def test_earlier_static_handle_goes_stale_and_launches_nothing():
    s1, _, _ = custom_state([4096, 10], 2, seed=921)
    s2, _, _ = custom_state([100], 2, seed=922)
    e1 = B.Engine(s1["w"], s1["v"], s1["g"], s1["u"], static_plan=True)
    e1.step(HY)
    torch.cuda.synchronize()
    before = [t.clone() for t in s1["w"]]
    e2 = B.Engine(s2["w"], s2["v"], s2["g"], s2["u"], static_plan=True)
    hy = B.odsgd_hyper(*HY)
    L, s = B.lib(), torch.cuda.current_stream().cuda_stream
    assert L.odsgd_step(e1.handle, ctypes.byref(hy), s) == B.ODSGD_ESTALE
    assert L.odsgd_local_update(e1.handle, -1, ctypes.byref(hy), s) == B.ODSGD_ESTALE
    assert L.odsgd_global_update(e1.handle, ctypes.byref(hy), s) == B.ODSGD_ESTALE
    with pytest.raises(B.OdsgdError) as err:
        e1.set_local_rule(B.ODSGD_LOCAL_DCASGD_C, lam=0.04)
    assert err.value.code == B.ODSGD_ESTALE
    assert B.odsgd_strerror(B.ODSGD_ESTALE) not in ("", "unknown error code")
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(before, s1["w"]))
    assert e1.iteration == 1
    e2.step(HY)   # the live one works
    torch.cuda.synchronize()
    assert e2.iteration == 1
    # a workspace handle is never affected
    e3 = B.Engine(s1["w"], s1["v"], s1["g"], s1["u"])
    e3.step(HY)
    e1.close()
    e2.close()
    e3.close()


def test_static_plan_rejects_what_does_not_fit():
    """Beyond ODSGD_STATIC_PLAN_BYTES of tables: ODSGD_ENOSPC, checked before any device work
    (the made-up addresses are never dereferenced)."""
    n = 1 << 29   # 2^21 chunks of 16 bytes = 32 MiB of chunk table
    assert B.odsgd_workspace_bytes([n], 1) > B.ODSGD_STATIC_PLAN_BYTES
    with pytest.raises(B.OdsgdError) as err:
        B.odsgd_init_static([n], [1 << 40], [2 << 40], [[3 << 40]], [[4 << 40]], 1)
    assert err.value.code == B.ODSGD_ENOSPC
