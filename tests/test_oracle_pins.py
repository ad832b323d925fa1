"""Pins for the CPU oracle: each test ties it to something other than itself --
a hand-expanded sequence, a closed form, a library optimiser, an invariant the
update rules imply, or the dataflow of Algorithm 2.  No GPU needed."""
from fractions import Fraction as F

import numpy as np
import pytest
import torch

from oracle import odsgd_oracle as oracle
from helpers import bits, cat, copy_list, max_rel_err, same_bits, split, zeros_like_list

F32 = np.float32


def _rand_state(rng, sizes, W, dtype=F32, wstd=0.05, gstd=1e-3):
    w = [rng.normal(0, wstd, n).astype(dtype) for n in sizes]
    v = [rng.normal(0, 1e-3, n).astype(dtype) for n in sizes]
    g = [[rng.normal(0, gstd, n).astype(dtype) for n in sizes] for _ in range(W)]
    u = [[np.full(n, 7.0, dtype) for n in sizes] for _ in range(W)]
    return w, v, g, u


# --------------------------------------------------------------------------
# hand-expanded sequence (Alg. 1 server step + Alg. 2 worker step, <=16 params)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_hand_expanded_sequence_exact(golden_w2, dtype):
    gd = golden_w2
    h = gd["hyper"]
    sizes = gd["tensors"]
    w = split(gd["w_init"], sizes, dtype)
    v = split(gd["v_init"], sizes, dtype)
    u = [zeros_like_list(w) for _ in range(2)]
    for it in gd["iters"]:
        g = [split(it["g0"], sizes, dtype), split(it["g1"], sizes, dtype)]
        oracle.od_step(w, v, g, u, h["lr"], h["local_lr"], h["momentum"],
                       h["weight_decay"], h["grad_scale"])
        # exact: every literal is representable, so == is the right comparison
        assert cat(w).tolist() == it["w"]
        assert cat(v).tolist() == it["v"]
        assert cat(u[0]).tolist() == it["u0"]
        assert cat(u[1]).tolist() == it["u1"]


def test_hand_expanded_split_calls_and_warmup(golden_w2):
    """local(all) then global reproduces the same table; a warm-up iteration
    hands the new weights to both workers and leaves w, v as in the table."""
    gd = golden_w2
    h = gd["hyper"]
    sizes = gd["tensors"]
    w = split(gd["w_init"], sizes)
    v = split(gd["v_init"], sizes)
    u = [zeros_like_list(w) for _ in range(2)]
    w2, v2, u2 = copy_list(w), copy_list(v), [zeros_like_list(w) for _ in range(2)]
    for i, it in enumerate(gd["iters"]):
        g = [split(it["g0"], sizes), split(it["g1"], sizes)]
        oracle.local_update(w, g, u, h["local_lr"], h["weight_decay"], worker=0)
        oracle.local_update(w, g, u, h["local_lr"], h["weight_decay"], worker=1)
        oracle.global_update(w, v, g, h["lr"], h["momentum"], h["weight_decay"], h["grad_scale"])
        assert cat(w).tolist() == it["w"] and cat(v).tolist() == it["v"]
        assert cat(u[0]).tolist() == it["u0"] and cat(u[1]).tolist() == it["u1"]
        # schedule with wp = 1
        oracle.step(i, 1, w2, v2, g, u2, h["lr"], h["local_lr"], h["momentum"],
                    h["weight_decay"], h["grad_scale"])
        assert cat(w2).tolist() == it["w"] and cat(v2).tolist() == it["v"]
        if i == 0:
            assert cat(u2[0]).tolist() == it["w"] and cat(u2[1]).tolist() == it["w"]
        else:
            assert cat(u2[0]).tolist() == it["u0"] and cat(u2[1]).tolist() == it["u1"]


# --------------------------------------------------------------------------
# one worker, zero delay, local_lr = 0  ==>  textbook momentum SGD
# --------------------------------------------------------------------------
def _quadratic_grad(x, a, c):
    return a * (x - c)


@pytest.mark.parametrize("wd", [0.0, 1e-2])
def test_reduces_to_library_momentum_sgd(wd):
    """W=1, grad_scale=1, local_lr=0, gradient taken at the current global
    weights: the w sequence is momentum SGD.  Cross-checked against
    torch.optim.SGD in float64 (its buffer b relates to ours by v = -lr*b)."""
    rng = np.random.default_rng(1)
    n, lr, mu = 13, 0.05, 0.9
    a = rng.uniform(0.5, 2.0, n)
    c = rng.normal(0, 1, n)
    w0 = rng.normal(0, 1, n)

    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd, dampening=0.0, nesterov=False)

    w = [w0.copy()]
    v = [np.zeros(n)]
    u = [[np.zeros(n)]]
    w32, v32, u32 = [w0.astype(F32)], [np.zeros(n, F32)], [[np.zeros(n, F32)]]
    for it in range(25):
        g = _quadratic_grad(w[0], a, c)
        w_before = w[0].copy()
        oracle.od_step(w, v, [[g]], u, lr, 0.0, mu, wd, 1.0)
        # local_lr = 0: the local weights are exactly the pulled w_t
        assert same_bits(u[0][0], w_before)

        p.grad = torch.tensor(_quadratic_grad(p.detach().numpy(), a, c))
        opt.step()
        assert max_rel_err(w[0], p.detach().numpy()) < 1e-12
        buf = opt.state[p]["momentum_buffer"].numpy()
        assert np.allclose(v[0], -lr * buf, rtol=1e-12, atol=1e-15)

        g32 = _quadratic_grad(w32[0].astype(np.float64), a, c).astype(F32)
        oracle.od_step(w32, v32, [[g32]], u32, lr, 0.0, mu, wd, 1.0)
        assert np.max(np.abs(w32[0] - w[0])) < 2e-6  # fp32 run tracks the fp64 one


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
def test_constant_gradient_closed_form():
    """wd=0, v_0=0, constant g: v_t = -lr*g*(1-mu^t)/(1-mu),
    w_t = w_0 - lr*g*sum_{j=1..t}(1-mu^j)/(1-mu)."""
    lr, mu, g0, w0 = F(1, 100), F(9, 10), F(3, 8), F(5, 4)
    w = [np.array([float(w0)])]
    v = [np.zeros(1)]
    g = [[np.array([float(g0)])], [np.array([float(g0)])]]  # W=2, mean of equal grads
    u = [[np.zeros(1)], [np.zeros(1)]]
    acc = F(0)
    for t in range(1, 31):
        oracle.od_step(w, v, g, u, float(lr), 0.3, float(mu), 0.0, 0.0)
        vt = -lr * g0 * (1 - mu ** t) / (1 - mu)
        acc += (1 - mu ** t) / (1 - mu)
        wt = w0 - lr * g0 * acc
        assert abs(v[0][0] - float(vt)) < 1e-15
        assert abs(w[0][0] - float(wt)) < 1e-14


def test_pure_weight_decay_closed_form():
    """g=0, mu=0: w_t = w_0 (1 - lr*wd)^t; local weights u = w_t (1 - local_lr*wd)."""
    lr, ll, wd = F(1, 4), F(1, 8), F(1, 2)
    w0 = F(3)
    w = [np.array([float(w0)])]
    v = [np.zeros(1)]
    g = [[np.zeros(1)] for _ in range(3)]
    u = [[np.zeros(1)] for _ in range(3)]
    for t in range(1, 15):
        oracle.od_step(w, v, g, u, float(lr), float(ll), 0.0, float(wd), 0.0)
        assert w[0][0] == float(w0 * (1 - lr * wd) ** t)  # dyadic: exact in fp64
        for m in range(3):
            assert u[m][0][0] == float(w0 * (1 - lr * wd) ** (t - 1) * (1 - ll * wd))


# --------------------------------------------------------------------------
# invariants the update rules imply
# --------------------------------------------------------------------------
def test_single_worker_compensation_is_exact():
    """W=1, mu=0, local_lr=lr, grad_scale=1: the local update performs the same
    operations as the global one, so u_0 == w_{t+1} bitwise."""
    rng = np.random.default_rng(2)
    sizes = [5, 64, 7]
    w, v, g, u = _rand_state(rng, sizes, 1)
    v = zeros_like_list(v)
    for _ in range(4):
        oracle.od_step(w, v, g, u, 0.3, 0.3, 0.0, 1e-3, 1.0)
        for k in range(len(sizes)):
            assert same_bits(u[0][k], w[k])
        g = [[rng.normal(0, 1e-3, n).astype(F32) for n in sizes]]


@pytest.mark.parametrize("W", [2, 4, 8, 16])
def test_identical_gradients_every_local_equals_new_global(W):
    """mu=0, local_lr=lr, mean aggregation, W a power of two and all workers
    holding the same gradient: the W-way sum is exact, so u_m == w_{t+1} bitwise."""
    rng = np.random.default_rng(3)
    sizes = [9, 33]
    w, v, g, u = _rand_state(rng, sizes, W)
    v = zeros_like_list(v)
    g = [copy_list(g[0]) for _ in range(W)]
    oracle.od_step(w, v, g, u, 0.125, 0.125, 0.0, 5e-4, 0.0)
    for m in range(W):
        for k in range(len(sizes)):
            assert same_bits(u[m][k], w[k])


def test_mean_of_locals_is_new_global_in_exact_arithmetic():
    """mu=0, local_lr=lr, grad_scale=1/W: (1/W) sum_m u_m = w_{t+1} (fp64 twin, 1e-15)."""
    rng = np.random.default_rng(4)
    sizes = [17]
    W = 5
    w, v, g, u = _rand_state(rng, sizes, W, dtype=np.float64)
    v = zeros_like_list(v)
    oracle.od_step(w, v, g, u, 0.2, 0.2, 0.0, 1e-3, 0.0)
    mean_u = sum(u[m][0] for m in range(W)) / W
    assert max_rel_err(mean_u, w[0]) < 1e-14


def test_worker_permutation():
    """Permuting workers permutes the rows of u and leaves w, v unchanged:
    bitwise when the gradient sums are exact (small integers * 2^-10)."""
    rng = np.random.default_rng(5)
    sizes = [11, 4]
    W = 8
    w, v, _, u = _rand_state(rng, sizes, W)
    g = [[(rng.integers(-64, 64, n) / 1024.0).astype(F32) for n in sizes] for _ in range(W)]
    perm = rng.permutation(W)
    w2, v2 = copy_list(w), copy_list(v)
    u2 = [zeros_like_list(w) for _ in range(W)]
    g2 = [g[p] for p in perm]
    oracle.od_step(w, v, g, u, 0.1, 0.05, 0.9, 1e-3, 0.0)
    oracle.od_step(w2, v2, g2, u2, 0.1, 0.05, 0.9, 1e-3, 0.0)
    for k in range(len(sizes)):
        assert same_bits(w[k], w2[k]) and same_bits(v[k], v2[k])
        for j, p in enumerate(perm):
            assert same_bits(u2[j][k], u[p][k])


def test_worker_permutation_fp64_general_values():
    rng = np.random.default_rng(6)
    sizes = [29]
    W = 12
    w, v, g, u = _rand_state(rng, sizes, W, dtype=np.float64)
    w2, v2, u2 = copy_list(w), copy_list(v), [zeros_like_list(w) for _ in range(W)]
    oracle.od_step(w, v, g, u, 0.1, 0.05, 0.9, 1e-3, 0.0)
    oracle.od_step(w2, v2, g[::-1], u2, 0.1, 0.05, 0.9, 1e-3, 0.0)
    assert max_rel_err(w2[0], w[0]) < 1e-13 and max_rel_err(v2[0], v[0]) < 1e-10


def test_reduction_is_sequential_in_ascending_worker_order():
    """((g0 + g1) + g2) in binary32: 1e8 + 1 rounds back to 1e8."""
    big = F32(1e8)
    for grads, expect_sum in (([big, 1.0, -big], 0.0), ([big, -big, 1.0], 1.0),
                              ([1.0, big, -big], 0.0)):
        w, v = [np.zeros(1, F32)], [np.zeros(1, F32)]
        g = [[np.array([x], F32)] for x in grads]
        oracle.global_update(w, v, g, 1.0, 0.0, 0.0, 1.0)
        assert w[0][0] == -expect_sum


def test_default_grad_scale_is_reciprocal_of_worker_count():
    for W in (1, 3, 4, 7, 16):
        w, v = [np.zeros(1, F32)], [np.zeros(1, F32)]
        g = [[np.array([1.0], F32)] for _ in range(W)]
        oracle.global_update(w, v, g, 1.0, 0.0, 0.0, 0.0)
        expect = F32(W) * (F32(1.0) / F32(W))
        assert v[0][0] == -expect and w[0][0] == -expect
        w, v = [np.zeros(1, F32)], [np.zeros(1, F32)]
        oracle.global_update(w, v, g, 1.0, 0.0, 0.0, 1.0)  # explicit raw sum
        assert w[0][0] == -F32(W)


def test_structure_independence():
    """u_m - w_t depends only on (g_m, w_t, local_lr, wd); w, v do not depend on local_lr."""
    rng = np.random.default_rng(7)
    sizes = [21, 3]
    W = 4
    w, v, g, u = _rand_state(rng, sizes, W)
    wa, va, ua = copy_list(w), copy_list(v), [zeros_like_list(w) for _ in range(W)]
    wb, vb, ub = copy_list(w), copy_list(v), [zeros_like_list(w) for _ in range(W)]
    oracle.od_step(wa, va, g, ua, 0.1, 0.05, 0.9, 1e-3, 0.0)
    g_other = [g[0]] + [[x * F32(3.0) for x in g[m]] for m in range(1, W)]
    oracle.od_step(wb, vb, g_other, ub, 0.7, 0.05, 0.3, 1e-3, 0.25)
    for k in range(len(sizes)):
        assert same_bits(ua[0][k], ub[0][k])          # worker 0 saw the same g_0 and w_t
        assert not same_bits(wa[k], wb[k])
    wc, vc, uc = copy_list(w), copy_list(v), [zeros_like_list(w) for _ in range(W)]
    oracle.od_step(wc, vc, g, uc, 0.1, 0.9, 0.9, 1e-3, 0.0)  # only local_lr changed
    for k in range(len(sizes)):
        assert same_bits(wa[k], wc[k]) and same_bits(va[k], vc[k])
        assert not same_bits(ua[1][k], uc[1][k])


def test_local_update_single_worker_touches_only_that_row():
    rng = np.random.default_rng(8)
    sizes = [10]
    w, v, g, u = _rand_state(rng, sizes, 3)
    w_before = copy_list(w)
    oracle.local_update(w, g, u, 0.1, 1e-3, worker=1)
    assert np.all(u[0][0] == 7.0) and np.all(u[2][0] == 7.0)
    assert not np.any(u[1][0] == 7.0)
    assert same_bits(w[0], w_before[0])
    # value: separately rounded binary32 operations
    r = F32(1e-3) * w[0]
    expect = w[0] - F32(0.1) * (g[1][0] + r)
    assert same_bits(u[1][0], expect.astype(F32))


# --------------------------------------------------------------------------
# delay dataflow of Algorithm 2 (which weights the local update reads, and when
# the first local update happens), on a closed-loop scalar problem
# --------------------------------------------------------------------------
def _closed_loop(wp, steps, a, lr, ll, y0):
    """One worker, gradient g = a*(x - c) with c = 0 taken at the weights x the
    worker was handed; returns the sequence of handed weights x_0..x_steps."""
    w, v, u = [np.array([y0])], [np.zeros(1)], [[np.array([y0])]]
    xs = [y0]
    for i in range(steps):
        x = u[0][0][0]
        g = [[np.array([a * x])]]
        oracle.step(i, wp, w, v, g, u, lr, ll, 0.0, 0.0, 1.0)
        xs.append(u[0][0][0])
    return xs


@pytest.mark.parametrize("wp", [0, 1, 3])
def test_one_step_delay_recurrence(wp):
    """Expanding Alg. 2 by hand for one worker, mu=0, wd=0 (e = w - c, y = x - c):
       warm-up   i <  wp:  y_{i+1} = (1 - lr a) y_i              (x is the exact w)
       training  i >= wp:  e_{i+1} = e_i - lr a y_i,  y_{i+1} = e_i - ll a y_i
       hence for i >= wp:  y_{i+2} = (1 - ll a) y_{i+1} + (ll - lr) a y_i.
    The two other candidate dataflows (local update applied to the *new* global
    weights; no delay at all) give different numbers, so this pins the reading."""
    a, lr, ll, y0 = F(1, 2), F(1, 4), F(3, 8), F(1)
    steps = 9
    xs = _closed_loop(wp, steps, float(a), float(lr), float(ll), float(y0))

    y = [y0]
    e = y0
    for i in range(steps):
        if i < wp:
            e = e - lr * a * y[i]
            y.append(e)
        else:
            e_new = e - lr * a * y[i]
            y.append(e - ll * a * y[i])
            e = e_new
    assert [float(t) for t in y] == xs  # dyadic values: exact in fp64

    for i in range(wp, steps - 1):
        assert y[i + 2] == (1 - ll * a) * y[i + 1] + (ll - lr) * a * y[i]

    # the rejected readings really differ on this problem
    alt_new, alt_nodelay = [y0], [y0]
    e1 = e2 = y0
    for i in range(steps):
        e1 = e1 - lr * a * alt_new[i]
        alt_new.append(e1 if i < wp else e1 - ll * a * alt_new[i])
        e2 = e2 - lr * a * alt_nodelay[i]
        alt_nodelay.append(e2)
    assert [float(t) for t in alt_new] != xs and [float(t) for t in alt_nodelay] != xs


def test_first_local_update_happens_at_iteration_wp():
    """Before iteration wp the handed weights equal the global ones; from wp on they differ."""
    rng = np.random.default_rng(9)
    sizes, W, wp = [6], 2, 3
    w, v, g, u = _rand_state(rng, sizes, W)
    for i in range(6):
        g = [[rng.normal(0, 1e-2, n).astype(F32) for n in sizes] for _ in range(W)]
        w_before = copy_list(w)
        oracle.step(i, wp, w, v, g, u, 0.1, 0.1, 0.9, 0.0, 0.0)
        if i < wp:
            assert same_bits(u[0][0], w[0]) and same_bits(u[1][0], w[0])
        else:
            assert not same_bits(u[0][0], w[0])
            # derived from the pre-update weights: u_m - w_t = -local_lr * g_m
            expect = w_before[0] - F32(0.1) * (g[1][0] + F32(0.0) * w_before[0])
            assert same_bits(u[1][0], expect.astype(F32))


# --------------------------------------------------------------------------
# special values and arithmetic mode
# --------------------------------------------------------------------------
def test_special_values():
    sub = np.float32(1e-41)  # subnormal
    w = [np.array([1.0, -0.0, 0.5, 2.0, sub, 3.0], F32)]
    v = [np.zeros(6, F32)]
    g0 = np.array([0.0, 0.0, np.nan, 1.0, 0.0, np.inf], F32)
    g1 = np.array([0.0, -0.0, 1.0, 1.0, 0.0, 1.0], F32)
    u = [[np.zeros(6, F32)], [np.zeros(6, F32)]]
    oracle.od_step(w, v, [[g0], [g1]], u, 0.5, 0.5, 0.0, 0.0, 0.0)
    assert w[0][0] == 1.0 and u[0][0][0] == 1.0        # zero gradient: nothing moves
    assert np.isnan(w[0][2]) and np.isnan(v[0][2])     # NaN poisons the global weight ...
    assert np.isnan(u[0][0][2]) and u[1][0][2] == 0.0  # ... and only the owner's local weight
    assert w[0][3] == 1.5
    assert w[0][4] == sub and u[0][0][4] == sub        # subnormal weight survives
    assert w[0][5] == -np.inf and u[0][0][5] == -np.inf and u[1][0][5] == 2.5
    # subnormal product is kept, not flushed: lr * g with both tiny
    w, v = [np.zeros(1, F32)], [np.zeros(1, F32)]
    oracle.global_update(w, v, [[np.array([2.0 ** -120], F32)]], 2.0 ** -20, 0.0, 0.0, 1.0)
    assert w[0][0] == -np.float32(2.0 ** -140) and w[0][0] != 0.0


def test_no_fused_multiply_add_and_fp32_rounding():
    """Each operation rounds separately to binary32.  Compared against numpy
    float32 element-wise operations (which never contract) on random data,
    and on a case built so that a fused a*b-c would give a different bit."""
    rng = np.random.default_rng(10)
    sizes = [1000]
    W = 5
    w, v, g, u = _rand_state(rng, sizes, W, wstd=1.0, gstd=1.0)
    lr, ll, mu, wd = F32(0.37), F32(0.11), F32(0.9), F32(0.013)
    w0, v0 = w[0].copy(), v[0].copy()
    oracle.od_step(w, v, g, u, lr, ll, mu, wd, 0.0)
    s = g[0][0].copy()
    for m in range(1, W):
        s = s + g[m][0]
    gb = s * (F32(1.0) / F32(W))
    r = wd * w0
    v1 = mu * v0 - lr * (gb + r)
    assert v1.dtype == F32
    assert same_bits(v[0], v1) and same_bits(w[0], w0 + v1)
    for m in range(W):
        assert same_bits(u[m][0], w0 - ll * (g[m][0] + r))
    # a = 1+2^-12, b = 1+2^-12: a*b = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11;
    # an FMA computing a*b - (1+2^-11) exactly would give 2^-24, separate rounding gives 0.
    a = F32(1.0 + 2.0 ** -12)
    w, v = [np.array([0.0], F32)], [np.array([a], F32)]
    gval = F32(1.0 + 2.0 ** -11)
    oracle.global_update(w, v, [[np.array([gval], F32)]], 1.0, a, 0.0, 1.0)
    assert v[0][0] == 0.0


def test_fp32_run_tracks_fp64_twin():
    rng = np.random.default_rng(11)
    sizes = [257, 30]
    W = 8
    w, v, g, u = _rand_state(rng, sizes, W)
    w64 = [x.astype(np.float64) for x in w]
    v64 = [x.astype(np.float64) for x in v]
    u64 = [[x.astype(np.float64) for x in um] for um in u]
    for it in range(20):
        g = [[rng.normal(0, 1e-3, n).astype(F32) for n in sizes] for _ in range(W)]
        g64 = [[x.astype(np.float64) for x in gm] for gm in g]
        oracle.od_step(w, v, g, u, 0.01, 0.01, 0.9, 5e-4, 0.0)
        oracle.od_step(w64, v64, g64, u64, float(F32(0.01)), float(F32(0.01)),
                       float(F32(0.9)), float(F32(5e-4)), 0.0)
    assert max_rel_err(cat(w), cat(w64)) < 1e-5
    assert np.max(np.abs(cat(v) - cat(v64))) < 1e-8


def test_empty_tensor_is_a_no_op():
    w, v = [np.zeros(0, F32), np.ones(2, F32)], [np.zeros(0, F32), np.zeros(2, F32)]
    g = [[np.zeros(0, F32), np.ones(2, F32)]]
    u = [[np.zeros(0, F32), np.zeros(2, F32)]]
    oracle.od_step(w, v, g, u, 0.5, 0.25, 0.0, 0.0, 1.0)
    assert w[1].tolist() == [0.5, 0.5] and u[0][1].tolist() == [0.75, 0.75]


def test_static_thread_split_is_the_single_thread_oracle_bit_for_bit():
    """oracle/threads.c only cuts the flat element range into contiguous parts and calls the
    oracle's own routine on each: any thread count must reproduce od_step exactly."""
    rng = np.random.default_rng(11)
    sizes = [5, 1000, 0, 77777, 3, 1]
    M = 3
    mk = lambda: [rng.standard_normal(n).astype(np.float32) for n in sizes]
    w, v, g, u = mk(), mk(), [mk() for _ in range(M)], [mk() for _ in range(M)]
    ref = ([a.copy() for a in w], [a.copy() for a in v], [[a.copy() for a in r] for r in u])
    oracle.od_step(ref[0], ref[1], g, ref[2], 0.1, 0.05, 0.9, 1e-3, 0.0)
    for threads in (1, 2, 7, 16, 200):
        w2, v2, u2 = [a.copy() for a in w], [a.copy() for a in v], [[a.copy() for a in r] for r in u]
        oracle.od_step_threads(w2, v2, g, u2, 0.1, 0.05, 0.9, 1e-3, 0.0, threads=threads)
        assert all(same_bits(a, b) for a, b in zip(w2, ref[0]))
        assert all(same_bits(a, b) for a, b in zip(v2, ref[1]))
        assert all(same_bits(a, b) for r, s in zip(u2, ref[2]) for a, b in zip(r, s))
