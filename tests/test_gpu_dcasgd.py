"""GPU parity for the other local updaters (DC-ASGD-c, DC-ASGD-a, local momentum
SGD): HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from gpu_harness import compare, f32, host_state, hyper_tuple, make_engine, oracle_hyper, refresh_host_grads, to_host
from helpers import same_bits
from oracle import odsgd_oracle as oracle
from paper_2005_06728_amd import binding as B
from paper_2005_06728_amd import workloads as wl
from gpu_harness import RAGGED, Arena, arenas_intact, custom_state, regen_grads, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# values the paper runs with (Section 4.3 / 4.4); epsilon is never stated there
LAMBDA_C = 0.04
LAMBDA_A, DECAY_A, EPS_A = 2.0, 0.95, 1e-7
LOCAL_MOMENTUM = 0.9


def install_rule(eng, rule, state, state_host):
    """Set the local updater on the engine; return the matching oracle rule tuple."""
    if rule == "c":
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_C, lam=LAMBDA_C)
        return ("dcasgd_c", f32(LAMBDA_C))
    if rule == "a":
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=LAMBDA_A, ms_decay=DECAY_A, epsilon=EPS_A, mean_square=state)
        return ("dcasgd_a", f32(LAMBDA_A), f32(DECAY_A), f32(EPS_A), state_host)
    eng.set_local_rule(B.ODSGD_LOCAL_SGD_MOMENTUM, local_momentum=LOCAL_MOMENTUM, local_velocity=state)
    return ("momentum", f32(LOCAL_MOMENTUM), state_host)


def compare_ms(ms_dev, ms_host):
    torch.cuda.synchronize()
    bad = 0
    for m in range(len(ms_dev)):
        for t, ref in zip(ms_dev[m], ms_host[m]):
            x = t.cpu().numpy()
            if not same_bits(x, ref):
                bad += int(np.sum(x.view(np.uint32) != ref.view(np.uint32)))
                rel = np.max(np.abs(x.astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-30))
                assert rel <= 1e-6, rel
    return bad


def test_hand_expanded_literals_on_gpu(golden_dcasgd):
    gd = golden_dcasgd
    t = lambda x: torch.tensor(np.array(x, np.float32), device=DEV)
    c = gd["rule_c"]
    st = {"w": [t(gd["c_w"])], "v": [torch.zeros(3, device=DEV)], "g": [[t(gd["c_g"])]], "u": [[t(gd["c_u_old"])]]}
    eng = make_engine(st)
    eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_C, lam=c["lambda"])
    eng.local_update(-1, (0.0, c["local_lr"], 0.0, c["weight_decay"], 1.0))
    torch.cuda.synchronize()
    assert st["u"][0][0].cpu().numpy().tolist() == gd["c_u_new"]
    eng.close()
    a = gd["rule_a"]
    st = {"w": [t(gd["a_w"])], "v": [torch.zeros(3, device=DEV)], "g": [[t(gd["a_g"])]], "u": [[t(gd["a_u_old"])]]}
    ms = [[t(gd["a_ms_old"])]]
    eng = make_engine(st)
    eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=a["lambda"], ms_decay=a["ms_decay"], epsilon=a["epsilon"],
                       mean_square=ms)
    eng.local_update(0, (0.0, a["local_lr"], 0.0, a["weight_decay"], 1.0))
    torch.cuda.synchronize()
    assert st["u"][0][0].cpu().numpy().tolist() == gd["a_u_new"]
    assert ms[0][0].cpu().numpy().tolist() == gd["a_ms_new"]
    eng.close()


@pytest.mark.parametrize("rule", ["c", "a", "m"])
@pytest.mark.parametrize("W", [1, 3, 4, 6, 8, 9, 12, 13, 16, 18])
def test_rules_ragged_sizes_schedule_and_split_calls(rule, W):
    say("rule=%s W=%d" % (rule, W))
    st, arenas, gen = custom_state(RAGGED, W, seed=300 + W)
    for m in range(W):                       # previous local weights: near the global ones
        for k, t in enumerate(st["u"][m]):
            t.copy_(st["w"][k] + 1e-3 * torch.randn(t.shape, generator=gen, device=DEV))
    ms_arenas = [Arena(RAGGED) for _ in range(W)]
    ms = [a.views for a in ms_arenas]
    for r in ms:
        for t in r:
            t.zero_()
    hs = host_state(st)
    ms_h = [to_host(r) for r in ms]
    wp = 2
    eng = make_engine(st, warmup_steps=wp)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    orule = install_rule(eng, rule, ms, ms_h)
    for it in range(5):                      # two warm-up iterations, then fused one-step-delay iterations
        eng.step(hy)
        oracle.step(it, wp, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
        assert compare(st, hs, label="fused it %d" % it)[0] == 0
        assert compare_ms(ms, ms_h) == 0
        regen_grads(st, gen, gstd=1e-2)
        refresh_host_grads(st, hs)
    # split: all workers, then one at a time
    eng.local_update(-1, hy)
    eng.global_update(hy)
    oracle.step(5, wp, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
    assert compare(st, hs, label="local(all)+global")[0] == 0 and compare_ms(ms, ms_h) == 0
    regen_grads(st, gen, gstd=1e-2)
    refresh_host_grads(st, hs)
    for m in range(W):
        eng.local_update(m, hy)
    eng.global_update(hy)
    oracle.step(6, wp, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
    assert compare(st, hs, label="local(m)+global")[0] == 0 and compare_ms(ms, ms_h) == 0
    assert arenas_intact(arenas) and all(a.intact() for a in ms_arenas)
    eng.close()


@pytest.mark.parametrize("name,rule,iters", [("resnet20", "c", 20), ("resnet20", "a", 20), ("lenet5", "m", 10),
                                             ("resnet50", "a", 2), ("resnet50", "m", 2), ("vgg16", "c", 1)])
def test_workloads_with_rules(name, rule, iters):
    w = wl.WORKLOADS[name]
    say("workload %s rule %s iterations %d" % (name, rule, iters))
    st = wl.allocate(w, DEV)
    ms = [[torch.zeros_like(t) for t in st["w"]] for _ in range(w.num_workers)] if rule in "am" else None
    hs = host_state(st)
    ms_h = [to_host(r) for r in ms] if ms else None
    eng = make_engine(st, warmup_steps=1)
    hy = hyper_tuple(w.hyper)
    oh = oracle_hyper(hy)
    orule = install_rule(eng, rule, ms, ms_h)
    for it in range(iters + 1):
        wl.fill_all_grads_(st, w, it)
        refresh_host_grads(st, hs)
        eng.step(hy)
        oracle.step(it, 1, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
        assert compare(st, hs, label="%s it %d" % (name, it))[0] == 0
        if ms:
            assert compare_ms(ms, ms_h) == 0
    eng.close()


@pytest.mark.parametrize("rule", ["c", "a", "m"])
@pytest.mark.parametrize("W,state_phase", [(4, 512), (16, 512), (13, 512), (8, 1536)])
def test_rules_on_two_half_tiles(rule, W, state_phase):
    """Tensors longer than a 64 KiB block, every array 512 bytes past a block boundary: the rules run
    on two-half tiles.  With the per-worker state at a different offset (1536) the registration
    moves those tensors back to contiguous tiles; the results are the same either way."""
    sizes = [16384 * 2 + 300, 16384, 700]
    say("rule=%s W=%d state_phase=%d" % (rule, W, state_phase))
    st, arenas, gen = custom_state(sizes, W, seed=420 + W, block_phase=512)
    for m in range(W):
        for k, t in enumerate(st["u"][m]):
            t.copy_(st["w"][k] + 1e-3 * torch.randn(t.shape, generator=gen, device=DEV))
    ms_arenas = [Arena(sizes, block_phase=state_phase) for _ in range(W)]
    ms = [a.views for a in ms_arenas]
    for r in ms:
        for t in r:
            t.zero_()
    hs = host_state(st)
    ms_h = [to_host(r) for r in ms]
    eng = make_engine(st, warmup_steps=1)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    orule = install_rule(eng, rule, ms, ms_h)
    for it in range(4):
        eng.step(hy)
        oracle.step(it, 1, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
        assert compare(st, hs, label="fused it %d" % it)[0] == 0 and compare_ms(ms, ms_h) == 0
        regen_grads(st, gen, gstd=1e-2)
        refresh_host_grads(st, hs)
    eng.local_update(-1, hy)
    eng.global_update(hy)
    oracle.step(4, 1, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
    assert compare(st, hs, label="local(all)+global")[0] == 0 and compare_ms(ms, ms_h) == 0
    assert arenas_intact(arenas) and all(a.intact() for a in ms_arenas)
    eng.close()


@pytest.mark.parametrize("rule", ["a", "m"])
def test_state_that_is_only_4_byte_aligned_moves_the_tensor_to_the_32_bit_path(rule):
    W, sizes = 3, [1000, 7, 4096]
    st, arenas, gen = custom_state(sizes, W, seed=390)
    for m in range(W):
        for k, t in enumerate(st["u"][m]):
            t.copy_(st["w"][k])
    ms_arenas = [Arena(sizes, shift=1 + m) for m in range(W)]     # views 4, 8, 12 bytes past a 16-byte boundary
    ms = [a.views for a in ms_arenas]
    assert all(t.data_ptr() % 16 for r in ms for t in r)
    for r in ms:
        for t in r:
            t.zero_()
    hs = host_state(st)
    ms_h = [to_host(r) for r in ms]
    eng = make_engine(st)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    orule = install_rule(eng, rule, ms, ms_h)
    for it in range(3):
        eng.step(hy)
        oracle.step(it, 0, hs["w"], hs["v"], hs["g"], hs["u"], rule=orule, **oh)
        assert compare(st, hs, label="it %d" % it)[0] == 0 and compare_ms(ms, ms_h) == 0
        regen_grads(st, gen, gstd=1e-2)
        refresh_host_grads(st, hs)
    assert arenas_intact(arenas) and all(a.intact() for a in ms_arenas)
    eng.close()


def test_rule_error_paths():
    n = 1024
    t = lambda: torch.zeros(n, device=DEV)
    st = {"w": [t()], "v": [t()], "g": [[t()], [t()]], "u": [[t()], [t()]]}
    eng = make_engine(st)
    with pytest.raises(B.OdsgdError) as e:
        eng.set_local_rule(7)
    assert e.value.code == B.ODSGD_EINVAL
    with pytest.raises(B.OdsgdError) as e:
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=2.0)          # state missing
    assert e.value.code == B.ODSGD_EINVAL
    with pytest.raises(B.OdsgdError) as e:                            # state aliases local weights
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=2.0, mean_square=[[st["u"][0][0]], [t()]])
    assert e.value.code == B.ODSGD_EALIAS
    with pytest.raises(B.OdsgdError) as e:                            # same state for two workers
        shared = t()
        eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=2.0, mean_square=[[shared], [shared]])
    assert e.value.code == B.ODSGD_EALIAS
    big, other = torch.zeros(n + 4, device=DEV), t()
    with pytest.raises(B.OdsgdError) as e:                            # state not even 4-byte aligned
        B.odsgd_set_local_rule(eng.handle, B.ODSGD_LOCAL_DCASGD_A, lam=2.0,
                               state_ptrs=[[big.data_ptr() + 2], [other.data_ptr()]])
    assert e.value.code == B.ODSGD_EALIGN
    # a failed registration leaves the SGD rule in place and the engine usable
    eng.step((0.1, 0.1, 0.9, 0.0, 0.0))
    eng.set_local_rule(B.ODSGD_LOCAL_DCASGD_A, lam=2.0, ms_decay=0.5, epsilon=1e-7, mean_square=[[t()], [t()]])
    eng.step((0.1, 0.1, 0.9, 0.0, 0.0))
    eng.set_local_rule(B.ODSGD_LOCAL_SGD)
    eng.step((0.1, 0.1, 0.9, 0.0, 0.0))
    with pytest.raises(B.OdsgdError) as e:
        eng.set_local_rule(B.ODSGD_LOCAL_SGD_MOMENTUM, local_momentum=0.9)   # state missing
    assert e.value.code == B.ODSGD_EINVAL
    eng.set_local_rule(B.ODSGD_LOCAL_SGD_MOMENTUM, local_momentum=0.9, local_velocity=[[t()], [t()]])
    eng.step((0.1, 0.1, 0.9, 0.0, 0.0))
    torch.cuda.synchronize()
    assert eng.iteration == 4
    eng.close()
