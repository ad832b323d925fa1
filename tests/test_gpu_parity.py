"""GPU parity: the HIP path (called through the C ABI) against the CPU oracle,
element by element, on the same seeded inputs.  Run with -m gpu on an MI355X."""
import os

import numpy as np
import pytest
import torch

from gpu_harness import (CANARY, DEV, RAGGED, TOL, arenas_intact, compare, custom_state, f32, host_state,
                         hyper_tuple, make_engine, oracle_hyper, refresh_host_grads, regen_grads, say, to_host)
from helpers import cat, same_bits, split
from oracle import odsgd_oracle as oracle
from paper_2005_06728_amd import binding as B
from paper_2005_06728_amd import workloads as wl

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------
# hand-expanded literals on the GPU
# ---------------------------------------------------------------------------
def test_hand_expanded_sequence_on_gpu(golden_w2):
    gd = golden_w2
    h = gd["hyper"]
    sizes = gd["tensors"]
    mk = lambda flat: [torch.tensor(a, device=DEV) for a in split(flat, sizes)]
    st = {"w": mk(gd["w_init"]), "v": mk(gd["v_init"]),
          "g": [mk([0, 0, 0]), mk([0, 0, 0])], "u": [mk([0, 0, 0]), mk([0, 0, 0])]}
    eng = make_engine(st)
    hy = (h["lr"], h["local_lr"], h["momentum"], h["weight_decay"], h["grad_scale"])
    for it in gd["iters"]:
        for m, key in enumerate(("g0", "g1")):
            for t, a in zip(st["g"][m], split(it[key], sizes)):
                t.copy_(torch.tensor(a))
        eng.step(hy)
        torch.cuda.synchronize()
        assert cat(to_host(st["w"])).tolist() == it["w"]
        assert cat(to_host(st["v"])).tolist() == it["v"]
        assert cat(to_host(st["u"][0])).tolist() == it["u0"]
        assert cat(to_host(st["u"][1])).tolist() == it["u1"]
    assert eng.iteration == 3
    eng.close()


# ---------------------------------------------------------------------------
# the five parameter sets, fused step, all outputs compared after every iteration
# ---------------------------------------------------------------------------
def run_workload(name, iterations, warmup=0, layout="separate", every_output=None, threads=1):
    """every_output(it) -> compare w, momentum and all local weights after iteration `it`
    (default: always); otherwise only w and momentum, which carry the accumulated state --
    the local weights are rewritten from scratch by every iteration.  threads > 1 runs the
    oracle's one-step-delay iteration with its element range split over that many host
    threads (the same C routine per piece; the split is pinned against the unsplit call in
    the host-only tests), which keeps the full-length runs of the large sets short."""
    w = wl.WORKLOADS[name]
    say("workload %s: K=%d N=%d W=%d iterations=%d warmup=%d" %
        (name, len(w.tensors), wl.total_params(w), w.num_workers, iterations, warmup))
    st = wl.allocate(w, DEV, layout=layout)
    hs = host_state(st)
    eng = make_engine(st, warmup_steps=warmup)
    hy = hyper_tuple(w.hyper)
    oh = oracle_hyper(hy)
    total_bad = 0
    for it in range(iterations):
        wl.fill_all_grads_(st, w, it)
        refresh_host_grads(st, hs)
        eng.step(hy)
        if threads > 1 and it >= warmup:
            oracle.od_step_threads(hs["w"], hs["v"], hs["g"], hs["u"], threads=threads, **oh)
        else:
            oracle.step(it, warmup, hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        what = ("w", "v", "u") if every_output is None or every_output(it) else ("w", "v")
        bad, worst = compare(st, hs, what=what, label="%s it %d" % (name, it))
        total_bad += bad
        say("  %s iteration %d of %d compared (%s)" % (name, it + 1, iterations, "+".join(what)))
    say("  %s: %d elements differ bitwise from the oracle" % (name, total_bad))
    eng.close()
    return total_bad


HOST_THREADS = min(16, os.cpu_count() or 1)


def ends_only(iterations):
    """All outputs after the first two and the last iteration; w and momentum after every one."""
    return lambda it: it < 2 or it == iterations - 1


def test_lenet5_full_run():
    assert run_workload("lenet5", wl.WORKLOADS["lenet5"].iterations) == 0


def test_resnet20_full_run_heavy_tailed_gradients():
    assert run_workload("resnet20", wl.WORKLOADS["resnet20"].iterations) == 0


def test_resnet50_full_size_full_run():
    n = wl.WORKLOADS["resnet50"].iterations
    assert n == 50 and run_workload("resnet50", n, every_output=ends_only(n), threads=HOST_THREADS) == 0


def test_alexnet_full_size_full_run():
    n = wl.WORKLOADS["alexnet"].iterations
    assert n == 20 and run_workload("alexnet", n, every_output=ends_only(n), threads=HOST_THREADS) == 0


def test_vgg16_full_size_full_run_with_exact_zero_gradients():
    n = wl.WORKLOADS["vgg16"].iterations
    assert n == 10 and run_workload("vgg16", n, every_output=ends_only(n), threads=HOST_THREADS) == 0


def test_resnet20_with_warmup_schedule():
    assert run_workload("resnet20", 8, warmup=3) == 0


def test_lenet5_packed_buckets_layout():
    """All tensors of a role packed back to back in one flat bucket (the usual
    gradient-bucket layout): neighbours are other tensors, not padding."""
    assert run_workload("lenet5", 4, layout="arena") == 0


def test_probe_copy():
    src = torch.randn(1 << 20, device=DEV)
    dst = torch.zeros_like(src)
    B.odsgd_probe_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    a, b = torch.randn(1000, device=DEV), torch.zeros(1000, device=DEV)
    B.odsgd_probe_copy(b[:996], a[:996])
    torch.cuda.synchronize()
    assert torch.equal(b[:996], a[:996]) and torch.all(b[996:] == 0)
    with pytest.raises(B.OdsgdError):
        B.odsgd_probe_copy(b[:998], a[:998])  # not a multiple of 4


# ---------------------------------------------------------------------------
# worker counts (templated and generic kernels), ragged sizes, guard bands
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 12, 13, 15, 16, 17, 64])
def test_worker_counts_ragged_sizes_all_entry_points(W):
    say("W=%d sizes=%s" % (W, RAGGED))
    st, arenas, gen = custom_state(RAGGED, W, seed=100 + W)
    hs = host_state(st)
    eng = make_engine(st)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0 if W % 2 else 1.0 / W)
    oh = oracle_hyper(hy)
    # fused step
    eng.step(hy)
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs, label="fused")[0] == 0
    # local(all) then global
    regen_grads(st, gen)
    refresh_host_grads(st, hs)
    eng.local_update(-1, hy)
    eng.global_update(hy)
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs, label="local(all)+global")[0] == 0
    # one worker at a time, then global
    regen_grads(st, gen)
    refresh_host_grads(st, hs)
    for m in range(W):
        eng.local_update(m, hy)
    eng.global_update(hy)
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs, label="local(m)+global")[0] == 0
    # a single worker's local update touches only its own row
    regen_grads(st, gen)
    refresh_host_grads(st, hs)
    eng.local_update(W - 1, hy)
    oracle.local_update(hs["w"], hs["g"], hs["u"], oh["local_lr"], oh["weight_decay"], worker=W - 1)
    assert compare(st, hs, label="local(W-1)")[0] == 0
    # warm-up step
    eng.ssgd_step(hy)
    oracle.ssgd_step(hs["w"], hs["v"], hs["g"], hs["u"], oh["lr"], oh["momentum"],
                     oh["weight_decay"], oh["grad_scale"])
    assert compare(st, hs, label="ssgd")[0] == 0
    assert eng.iteration == 4
    assert arenas_intact(arenas)
    eng.close()


BLOCKY = [16384 * 3 + 77, 5, 16384, 16383, 20000, 16384 * 2, 1, 70000]


@pytest.mark.parametrize("block_phase", [0, 512, 1040, 65536 - 16, 32768 + 256])
@pytest.mark.parametrize("W", [2, 8, 16, 5, 13, 20])
def test_two_half_tiles_all_entry_points(W, block_phase):
    """Every array of a tensor at the same offset from a 64 KiB boundary: the blocks inside
    take two-half tiles, the pieces before and after them contiguous ones; the oracle knows
    nothing of either."""
    say("W=%d block_phase=%d sizes=%s" % (W, block_phase, BLOCKY))
    st, arenas, gen = custom_state(BLOCKY, W, seed=600 + W, block_phase=block_phase)
    ptrs = lambda lst: [t.data_ptr() for t in lst]
    rows, chunks = B.odsgd_plan_host(BLOCKY, ptrs(st["w"]), ptrs(st["v"]), [ptrs(r) for r in st["g"]],
                                     [ptrs(r) for r in st["u"]], W)
    assert sum(1 for c in chunks if c[4]) >= 64 * 5, "expected two-half tiles in this layout"
    hs = host_state(st)
    eng = make_engine(st)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    eng.step(hy)
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs, label="fused")[0] == 0
    regen_grads(st, gen)
    refresh_host_grads(st, hs)
    eng.local_update(-1, hy)
    eng.global_update(hy)
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs, label="local(all)+global")[0] == 0
    regen_grads(st, gen)
    refresh_host_grads(st, hs)
    eng.local_update(W // 2, hy)
    oracle.local_update(hs["w"], hs["g"], hs["u"], oh["local_lr"], oh["weight_decay"], worker=W // 2)
    assert compare(st, hs, label="local(m)")[0] == 0
    eng.ssgd_step(hy)
    oracle.ssgd_step(hs["w"], hs["v"], hs["g"], hs["u"], oh["lr"], oh["momentum"],
                     oh["weight_decay"], oh["grad_scale"])
    assert compare(st, hs, label="ssgd")[0] == 0
    assert arenas_intact(arenas)
    eng.close()


def test_probe_streams_moves_the_same_arrays_and_changes_nothing_else():
    W = 8
    st, arenas, gen = custom_state(BLOCKY, W, seed=650, block_phase=0)
    before = host_state(st)
    eng = make_engine(st)
    eng.probe_streams()
    torch.cuda.synchronize()
    after = host_state(st)
    for k in range(len(BLOCKY)):
        assert same_bits(after["w"][k], before["w"][k]) and same_bits(after["v"][k], before["v"][k])
        for m in range(W):
            assert same_bits(after["g"][m][k], before["g"][m][k])
            assert same_bits(after["u"][m][k], before["g"][m][k])   # local weights received the gradients
    assert eng.iteration == 0 and arenas_intact(arenas)
    eng.close()


@pytest.mark.parametrize("shifts", [{"w": 1}, {"g": 2}, {"u": 3}, {"w": 1, "v": 1, "g": 1, "u": 1}])
def test_pointers_only_4_byte_aligned_take_the_scalar_path(shifts):
    say("shifts=%s" % shifts)
    W = 4
    st, arenas, gen = custom_state(RAGGED, W, seed=7, shifts=shifts)
    assert any(t.data_ptr() % 16 for t in st["w"] + st["v"] + st["g"][0] + st["u"][0] if t.numel())
    hs = host_state(st)
    eng = make_engine(st)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    for _ in range(2):
        eng.step(hy)
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        assert compare(st, hs)[0] == 0
        regen_grads(st, gen)
        refresh_host_grads(st, hs)
    eng.local_update(-1, hy)
    eng.global_update(hy)
    oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs)[0] == 0
    assert arenas_intact(arenas)
    eng.close()


@pytest.mark.parametrize("env", [{"ODSGD_PAIR_BIT": "0"}, {"ODSGD_PAIR_BIT": "12"}, {"ODSGD_PAIR_BIT": "17"},
                                 {"ODSGD_BLOCKS_PER_CU": "1"}, {"ODSGD_BLOCKS_PER_CU": "8"},
                                 {"ODSGD_PAIR_BIT": "0", "ODSGD_BLOCKS_PER_CU": "2"},
                                 {"ODSGD_WAVES_PER_CU": "-1"}, {"ODSGD_WAVES_PER_CU": "2"},
                                 {"ODSGD_WAVES_PER_CU": "7", "ODSGD_PAIR_BIT": "13"}])
def test_launch_shape_does_not_change_results(env):
    """Tile shape, grid size and residency are tuning only: outputs are bitwise the same."""
    say("env=%s" % env)
    sizes = RAGGED + [300000]
    W = 8
    old = {k: os.environ.get(k) for k in env}
    os.environ.update(env)
    try:
        st, arenas, gen = custom_state(sizes, W, seed=11, block_phase=528)
        hs = host_state(st)
        eng = make_engine(st)
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    for _ in range(3):
        eng.step(hy)
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        assert compare(st, hs)[0] == 0
        regen_grads(st, gen)
        refresh_host_grads(st, hs)
    assert arenas_intact(arenas)
    eng.close()


# ---------------------------------------------------------------------------
# special values, resume, error paths with real device memory
# ---------------------------------------------------------------------------
def test_special_values_on_gpu():
    sub = np.float32(1e-41)
    W = 2
    wv = np.array([1.0, -0.0, 0.5, 2.0, sub, 3.0, 0.0, 1.0], np.float32)
    g0 = np.array([0.0, 0.0, np.nan, 1.0, 0.0, np.inf, 2.0 ** -120, -0.0], np.float32)
    g1 = np.array([0.0, -0.0, 1.0, 1.0, 0.0, 1.0, 2.0 ** -120, -0.0], np.float32)
    st = {"w": [torch.tensor(wv, device=DEV)], "v": [torch.zeros(8, device=DEV)],
          "g": [[torch.tensor(g0, device=DEV)], [torch.tensor(g1, device=DEV)]],
          "u": [[torch.zeros(8, device=DEV)], [torch.zeros(8, device=DEV)]]}
    hs = host_state(st)
    eng = make_engine(st)
    for hy in ((0.5, 0.5, 0.0, 0.0, 0.0), (2.0 ** -20, 2.0 ** -20, 0.5, 0.25, 1.0)):
        eng.step(hy)
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oracle_hyper(hy))
        torch.cuda.synchronize()
        for a, b in ((st["w"][0], hs["w"][0]), (st["v"][0], hs["v"][0]),
                     (st["u"][0][0], hs["u"][0][0]), (st["u"][1][0], hs["u"][1][0])):
            assert same_bits(a.cpu().numpy(), b), (a.cpu().numpy(), b)
    # subnormal results were produced and kept (not flushed to zero)
    assert hs["u"][0][0][4] != 0.0 and abs(hs["u"][0][0][4]) < 1.2e-38
    eng.close()


def test_resume_from_caller_owned_state():
    """All state lives in the caller's buffers: 6 steps == 3 steps, destroy, re-init, 3 steps."""
    sizes = [5000, 17]
    W = 4
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    results = []
    for split_at in (None, 3):
        st, _, gen = custom_state(sizes, W, seed=21)
        eng = make_engine(st, warmup_steps=2)
        for it in range(6):
            if split_at is not None and it == split_at:
                eng.close()
                eng = make_engine(st, warmup_steps=2)
                B.odsgd_set_iteration(eng.handle, it)
            eng.step(hy)
            regen_grads(st, gen)
        torch.cuda.synchronize()
        results.append(host_state(st))
        eng.close()
    for key in ("w", "v"):
        for a, b in zip(results[0][key], results[1][key]):
            assert same_bits(a, b)
    for m in range(W):
        for a, b in zip(results[0]["u"][m], results[1]["u"][m]):
            assert same_bits(a, b)


def test_error_paths_with_device_memory():
    n = 1024
    t = lambda: torch.zeros(n, device=DEV)
    w, v, g, u = [t()], [t()], [[t()], [t()]], [[t()], [t()]]
    nbytes = B.odsgd_workspace_bytes([n], 2)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    ptr = lambda lst: [x.data_ptr() for x in lst]

    def init(**kw):
        args = dict(numel=[n], w_ptrs=ptr(w), mom_ptrs=ptr(v), grad_ptrs=[ptr(r) for r in g],
                    local_ptrs=[ptr(r) for r in u], num_workers=2, workspace_ptr=ws.data_ptr(),
                    workspace_bytes=nbytes, stream=torch.cuda.current_stream().cuda_stream)
        args.update(kw)
        return B.odsgd_init(**args)

    for code, kw in ((B.ODSGD_ENOSPC, dict(workspace_bytes=nbytes - 1)),
                     (B.ODSGD_EALIAS, dict(local_ptrs=[ptr(w), ptr(u[1])])),
                     (B.ODSGD_EALIAS, dict(local_ptrs=[ptr(u[0]), ptr(u[0])])),
                     (B.ODSGD_EALIAS, dict(grad_ptrs=[ptr(v), ptr(g[1])])),
                     (B.ODSGD_EALIGN, dict(mom_ptrs=[v[0].data_ptr() + 2])),
                     (B.ODSGD_EINVAL, dict(w_ptrs=[0]))):
        with pytest.raises(B.OdsgdError) as e:
            init(**kw)
        assert e.value.code == code, kw
    # the same gradient buffer registered for both workers is legal
    h = init(grad_ptrs=[ptr(g[0]), ptr(g[0])])
    hy = B.odsgd_hyper(0.1, 0.1, 0.9, 0.0, 0.0)
    import ctypes
    L = B.lib()
    s = torch.cuda.current_stream().cuda_stream
    assert L.odsgd_local_update(h, 2, ctypes.byref(hy), s) == B.ODSGD_EINVAL
    assert L.odsgd_local_update(h, -2, ctypes.byref(hy), s) == B.ODSGD_EINVAL
    assert L.odsgd_step(h, None, s) == B.ODSGD_EINVAL
    assert L.odsgd_set_warmup(h, -1) == B.ODSGD_EINVAL
    assert B.odsgd_get_iteration(h) == 0
    B.odsgd_step(h, hy)
    torch.cuda.synchronize()
    assert B.odsgd_get_iteration(h) == 1
    B.odsgd_destroy(h)


def test_all_tensors_empty_is_a_no_op():
    z = lambda: torch.zeros(0, device=DEV)
    st = {"w": [z()], "v": [z()], "g": [[z()]], "u": [[z()]]}
    eng = make_engine(st)
    eng.step((0.1, 0.1, 0.9, 0.0, 0.0))
    torch.cuda.synchronize()
    assert eng.iteration == 1
    eng.close()


def test_non_default_stream():
    sizes = [10000, 33]
    W = 4
    st, arenas, gen = custom_state(sizes, W, seed=31)
    hs = host_state(st)
    eng = make_engine(st)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        eng.step(hy)
    eng.step(hy, stream=s)
    s.synchronize()
    for _ in range(2):
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oracle_hyper(hy))
    assert compare(st, hs)[0] == 0
    eng.close()


def test_hip_graph_replay_matches_eager():
    """The step is a single kernel launch and nothing else, so it can be captured.
    Replay the graph several times with eager work and synchronisation in between
    and compare every replay with the oracle (the iteration counter is host state
    and advances at capture time only, so the schedule must not change mid-graph)."""
    w = wl.WORKLOADS["resnet20"]
    st = wl.allocate(w, DEV)
    hs = host_state(st)
    eng = make_engine(st)
    hy = hyper_tuple(w.hyper)
    oh = oracle_hyper(hy)
    wl.fill_all_grads_(st, w, 0)
    refresh_host_grads(st, hs)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(3):
            eng.step(hy, side)
    torch.cuda.synchronize()
    steps_done = 0
    for rep in range(4):
        graph.replay()
        torch.cuda.synchronize()
        for _ in range(3):
            oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        steps_done += 3
        assert compare(st, hs, label="replay %d" % rep)[0] == 0
        # eager work between replays: new gradients, one eager step
        wl.fill_all_grads_(st, w, rep + 1)
        refresh_host_grads(st, hs)
        eng.step(hy)
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        assert compare(st, hs, label="eager after replay %d" % rep)[0] == 0
    eng.close()


def test_tensor_beyond_32_bit_element_offsets():
    """One tensor of 2^32 + 70,003 elements (W = 1): chunk offsets need the high word
    of the 64-bit element offset and byte offsets exceed 2^34.  Four arrays of 17 GB
    each stay on the GPU; the oracle checks a sample: both ends, the region around
    element 2^32, and a million random positions."""
    n = (1 << 32) + 70003
    free, _ = torch.cuda.mem_get_info()
    if free < 5 * 4 * n:
        pytest.skip("needs about 86 GB of free device memory")
    say("huge tensor: n=%d" % n)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    mk = lambda: torch.empty(n, dtype=torch.float32, device=DEV)
    w, v, g, u = mk(), mk(), mk(), mk()
    step = 1 << 28
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        w[lo:hi].normal_(0, 0.05, generator=gen)
        v[lo:hi].normal_(0, 1e-3, generator=gen)
        g[lo:hi].normal_(0, 1e-3, generator=gen)
    u.fill_(CANARY)
    idx = torch.cat([torch.arange(0, 5000, device=DEV), torch.arange(n - 5000, n, device=DEV),
                     torch.arange((1 << 32) - 3000, (1 << 32) + 3000, device=DEV),
                     torch.arange((1 << 31) - 1000, (1 << 31) + 1000, device=DEV),
                     torch.randint(0, n, (1 << 20,), device=DEV, generator=gen)])
    hw, hv, hg = (t[idx].cpu().numpy().copy() for t in (w, v, g))
    hu = np.zeros_like(hw)
    eng = B.Engine([w], [v], [[g]], [[u]])
    hy = (0.05, 0.02, 0.9, 1e-3, 1.0)
    eng.step(hy)
    torch.cuda.synchronize()
    oracle.od_step([hw], [hv], [[hg]], [[hu]], **oracle_hyper(hy))
    assert same_bits(w[idx].cpu().numpy(), hw)
    assert same_bits(v[idx].cpu().numpy(), hv)
    assert same_bits(u[idx].cpu().numpy(), hu)
    # every element was written exactly once: no canary left in the local weights
    for lo in range(0, n, step):
        assert not bool(torch.any(u[lo:min(n, lo + step)] == CANARY))
    eng.close()


def test_thousands_of_tiny_tensors():
    """K = 3000 tensors of 1..300 elements: one ragged chunk (or two) each, a 3000-row pointer table."""
    rng = np.random.default_rng(5)
    sizes = [int(x) for x in rng.integers(1, 300, 3000)]
    W = 2
    st, arenas, gen = custom_state(sizes, W, seed=41)
    hs = host_state(st)
    eng = make_engine(st)
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    for _ in range(2):
        eng.step(hy)
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
    assert compare(st, hs)[0] == 0
    assert arenas_intact(arenas)
    eng.close()


def test_two_handles_on_two_streams_are_independent():
    states, engines, hosts, streams = [], [], [], []
    for seed, sizes, W in ((51, [30000, 77, 4096], 4), (52, [12345, 1000], 8)):
        st, _, _ = custom_state(sizes, W, seed=seed)
        states.append(st)
        hosts.append(host_state(st))
        engines.append(make_engine(st))
        streams.append(torch.cuda.Stream())
    torch.cuda.synchronize()
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    for _ in range(5):
        for eng, s in zip(engines, streams):
            eng.step(hy, stream=s)
    for s in streams:
        s.synchronize()
    for st, hs, eng in zip(states, hosts, engines):
        for _ in range(5):
            oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oracle_hyper(hy))
        assert compare(st, hs)[0] == 0
        eng.close()


# ---------------------------------------------------------------------------
# the whole loop of Alg. 2 closed on the GPU: gradients computed from the weights
# each worker was handed, warm-up, switching and training stages in one run
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("wp", [0, 1, 3])
def test_closed_training_loop_on_gpu_follows_the_oracle(wp):
    """Worker m minimises 0.5*a*(x - c_m)^2 per coordinate: its gradient is a*(x_m - c_m) at the
    weights x_m it was handed -- the exact global weights during warm-up, its compensated local
    weights afterwards.  The same loop runs on the host with the oracle; the gradient is two
    separately rounded binary32 operations on both sides, so every iteration must agree bit for bit."""
    W, sizes, steps = 4, [1000, 3, 16384 * 2 + 5], 12
    a = 0.5
    st, arenas, gen = custom_state(sizes, W, seed=800 + wp, wstd=1.0, block_phase=0)
    centres = [[torch.randn(n, device=DEV, generator=gen) for n in sizes] for _ in range(W)]
    for k, t in enumerate(st["v"]):
        t.zero_()
    for m in range(W):
        for k, t in enumerate(st["u"][m]):
            t.copy_(st["w"][k])            # workers pull w_0 before the first iteration
    hs = host_state(st)
    hc = [to_host(r) for r in centres]
    eng = make_engine(st, warmup_steps=wp)
    hy = (0.25, 0.375, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    for it in range(steps):
        for m in range(W):
            for k in range(len(sizes)):
                torch.mul(torch.sub(st["u"][m][k], centres[m][k]), a, out=st["g"][m][k])
                hs["g"][m][k][...] = (hs["u"][m][k] - hc[m][k]) * np.float32(a)
        eng.step(hy)
        oracle.step(it, wp, hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        assert compare(st, hs, label="closed loop wp=%d it %d" % (wp, it))[0] == 0
        handed_equals_global = all(torch.equal(st["u"][m][k], st["w"][k]) for m in range(W) for k in range(len(sizes)))
        assert handed_equals_global == (it < wp), "iteration %d" % it
    # and the loop does what training is for: the weights move towards the mean of the workers' centres
    mean_c = [sum(centres[m][k] for m in range(W)) / W for k in range(len(sizes))]
    dist = sum(float(torch.sum((w_ - c) ** 2)) for w_, c in zip(st["w"], mean_c))
    start = sum(float(torch.sum(c ** 2)) for c in mean_c) + sum(sizes)   # E|w_0 - c|^2 with w_0 ~ N(0, 1)
    assert dist < 0.5 * start
    assert arenas_intact(arenas)
    eng.close()


@pytest.mark.parametrize("W", [3, 16, 20])
def test_global_update_that_streams_its_state(W):
    """Weights plus momentum larger than the last-level cache make odsgd_global_update load them
    non-temporally (another kernel variant); forced here by declaring the cache empty."""
    old = os.environ.get("ODSGD_LLC_BYTES")
    os.environ["ODSGD_LLC_BYTES"] = "0"
    try:
        st, arenas, gen = custom_state(BLOCKY, W, seed=850 + W, block_phase=0)
        hs = host_state(st)
        eng = make_engine(st)
    finally:
        if old is None:
            os.environ.pop("ODSGD_LLC_BYTES")
        else:
            os.environ["ODSGD_LLC_BYTES"] = old
    hy = (0.05, 0.02, 0.9, 1e-3, 0.0)
    oh = oracle_hyper(hy)
    for it in range(3):
        eng.local_update(-1, hy)
        eng.global_update(hy)
        oracle.od_step(hs["w"], hs["v"], hs["g"], hs["u"], **oh)
        assert compare(st, hs, label="it %d" % it)[0] == 0
        regen_grads(st, gen)
        refresh_host_grads(st, hs)
    # global update alone: local weights untouched
    before_u = [to_host(r) for r in st["u"]]
    eng.global_update(hy)
    oracle.global_update(hs["w"], hs["v"], hs["g"], oh["lr"], oh["momentum"], oh["weight_decay"], oh["grad_scale"])
    assert compare(st, hs, what=("w", "v"))[0] == 0
    for m in range(W):
        for a, b in zip(to_host(st["u"][m]), before_u[m]):
            assert same_bits(a, b)
    assert arenas_intact(arenas)
    eng.close()
