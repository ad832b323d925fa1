"""Pins for the delay-compensated local updaters of the oracle (Section 3.3
equations): hand-expanded literals, reductions to the SGD updater, the
exact-curvature case in which the compensation recovers the zero-delay gradient,
and the closed form of the MeanSquare recurrence.  No GPU needed."""
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import odsgd_oracle as oracle
from helpers import copy_list, max_rel_err, same_bits

F32 = np.float32


def arr(x, dtype=F32):
    return np.array(x, dtype=dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_hand_expanded_literals(golden_dcasgd, dtype):
    gd = golden_dcasgd
    c = gd["rule_c"]
    u = [[arr(gd["c_u_old"], dtype)]]
    oracle.local_update_dcasgd_c([arr(gd["c_w"], dtype)], [[arr(gd["c_g"], dtype)]], u,
                                 c["local_lr"], c["weight_decay"], c["lambda"])
    assert u[0][0].tolist() == gd["c_u_new"]
    a = gd["rule_a"]
    u = [[arr(gd["a_u_old"], dtype)]]
    ms = [[arr(gd["a_ms_old"], dtype)]]
    oracle.local_update_dcasgd_a([arr(gd["a_w"], dtype)], [[arr(gd["a_g"], dtype)]], u, ms,
                                 a["local_lr"], a["weight_decay"], a["lambda"], a["ms_decay"], a["epsilon"])
    assert u[0][0].tolist() == gd["a_u_new"]
    assert ms[0][0].tolist() == gd["a_ms_new"]


def _rand(rng, n, W, dtype=F32):
    w = [rng.normal(0, 0.05, n).astype(dtype)]
    g = [[rng.normal(0, 1e-2, n).astype(dtype)] for _ in range(W)]
    u = [[(w[0] + rng.normal(0, 1e-3, n)).astype(dtype)] for _ in range(W)]
    ms = [[np.abs(rng.normal(0, 1e-4, n)).astype(dtype)] for _ in range(W)]
    return w, g, u, ms


def test_zero_lambda_or_zero_delay_reduces_to_sgd_updater_bitwise():
    rng = np.random.default_rng(1)
    w, g, u, ms = _rand(rng, 50, 3)
    ref = [[np.zeros(50, F32)] for _ in range(3)]
    oracle.local_update(w, g, ref, 0.3, 1e-3)
    for rule in ("c", "a"):
        # lambda = 0
        uu = [copy_list(r) for r in u]
        if rule == "c":
            oracle.local_update_dcasgd_c(w, g, uu, 0.3, 1e-3, 0.0)
        else:
            oracle.local_update_dcasgd_a(w, g, uu, [copy_list(r) for r in ms], 0.3, 1e-3, 0.0, 0.95, 1e-7)
        for m in range(3):
            assert same_bits(uu[m][0], ref[m][0])
        # no delay: the gradient was taken at the very weights being updated
        uu = [[w[0].copy()] for _ in range(3)]
        if rule == "c":
            oracle.local_update_dcasgd_c(w, g, uu, 0.3, 1e-3, 0.04)
        else:
            oracle.local_update_dcasgd_a(w, g, uu, [copy_list(r) for r in ms], 0.3, 1e-3, 2.0, 0.95, 1e-7)
        for m in range(3):
            assert same_bits(uu[m][0], ref[m][0])


def test_exact_curvature_recovers_the_zero_delay_step():
    """Quadratic loss f(x) = a x^2 / 2: the gradient taken at the stale point u_old is
    g = a*u_old, the true gradient at w is a*w = g + a*(w - u_old).  The compensation
    term lambda*g*g*(w - u_old) equals a*(w - u_old) when lambda = a/g^2, so the
    update must land on w - lr*a*w."""
    rng = np.random.default_rng(2)
    n = 40
    a = rng.uniform(0.5, 2.0, n)
    w = rng.normal(0, 1, n)
    u_old = w + rng.normal(0, 0.1, n)
    g = a * u_old
    lr = 0.1
    for i in range(n):  # lambda is a scalar hyper-parameter: one element at a time
        u = [[arr([u_old[i]], np.float64)]]
        oracle.local_update_dcasgd_c([arr([w[i]], np.float64)], [[arr([g[i]], np.float64)]], u,
                                     lr, 0.0, a[i] / g[i] ** 2)
        assert abs(u[0][0][0] - (w[i] - lr * a[i] * w[i])) < 1e-14
        # adaptive rule with ms_decay = 0, eps = 0: MeanSquare = g^2, lambda_eff = lambda/|g|
        u = [[arr([u_old[i]], np.float64)]]
        ms = [[arr([123.0], np.float64)]]
        oracle.local_update_dcasgd_a([arr([w[i]], np.float64)], [[arr([g[i]], np.float64)]], u, ms,
                                     lr, 0.0, a[i] / abs(g[i]), 0.0, 0.0)
        assert abs(u[0][0][0] - (w[i] - lr * a[i] * w[i])) < 1e-14
        assert abs(ms[0][0][0] - g[i] ** 2) < 1e-18


def test_mean_square_recurrence_closed_form():
    """Constant gradient g from MeanSquare_0 = 0: MeanSquare_t = g^2 (1 - m^t)."""
    m, g = F(3, 4), F(3, 2)
    w = [arr([1.0], np.float64)]
    u = [[arr([1.0], np.float64)]]
    ms = [[arr([0.0], np.float64)]]
    for t in range(1, 20):
        oracle.local_update_dcasgd_a(w, [[arr([float(g)], np.float64)]], u, ms, 0.0, 0.0, 2.0,
                                     float(m), 1e-7)
        assert abs(ms[0][0][0] - float(g * g * (1 - m ** t))) < 1e-15
        assert u[0][0][0] == 1.0  # local_lr = 0 keeps the pulled weights


def test_sign_and_structure():
    """The compensation pulls along +(w - u_old) scaled by g^2 >= 0: flipping the sign of the
    delay flips the correction; flipping the sign of g flips the plain term but not the correction."""
    w = [arr([1.0], np.float64)]
    lr, lam, g = 0.5, 0.25, 2.0
    out = {}
    for du in (+0.5, -0.5):
        for sg in (+1, -1):
            u = [[arr([1.0 - du], np.float64)]]
            oracle.local_update_dcasgd_c(w, [[arr([sg * g], np.float64)]], u, lr, 0.0, lam)
            out[(du, sg)] = u[0][0][0]
    for du in (+0.5, -0.5):
        for sg in (+1, -1):
            assert out[(du, sg)] == 1.0 - lr * (sg * g + lam * g * g * du)
    # workers are independent; a single-worker call touches only its row
    rng = np.random.default_rng(3)
    w, g, u, ms = _rand(rng, 10, 3)
    u_all = [copy_list(r) for r in u]
    oracle.local_update_dcasgd_c(w, g, u_all, 0.1, 1e-3, 0.04)
    u_one = [copy_list(r) for r in u]
    oracle.local_update_dcasgd_c(w, g, u_one, 0.1, 1e-3, 0.04, worker=1)
    assert same_bits(u_one[1][0], u_all[1][0])
    assert same_bits(u_one[0][0], u[0][0]) and same_bits(u_one[2][0], u[2][0])


def test_fp32_operation_order_matches_separately_rounded_numpy():
    rng = np.random.default_rng(4)
    w, g, u, ms = _rand(rng, 500, 2)
    lr, wd, lam, dec, eps = F32(0.37), F32(0.013), F32(2.0), F32(0.95), F32(1e-7)
    u0 = [copy_list(r) for r in u]
    ms0 = [copy_list(r) for r in ms]
    oracle.local_update_dcasgd_a(w, g, u, ms, lr, wd, lam, dec, eps)
    for m in range(2):
        gm, w0 = g[m][0], w[0]
        gg = gm * gm
        msq = dec * ms0[m][0] + (F32(1) - dec) * gg
        den = np.sqrt(msq + eps)
        c2 = (gg * (w0 - u0[m][0])) * (lam / den)
        expect = w0 - lr * ((gm + wd * w0) + c2)
        assert msq.dtype == F32 and expect.dtype == F32
        assert same_bits(ms[m][0], msq) and same_bits(u[m][0], expect)
    uc = [copy_list(r) for r in u0]
    oracle.local_update_dcasgd_c(w, g, uc, lr, wd, F32(0.04))
    for m in range(2):
        gm, w0 = g[m][0], w[0]
        expect = w0 - lr * ((gm + wd * w0) + ((gm * gm) * (w0 - u0[m][0])) * F32(0.04))
        assert same_bits(uc[m][0], expect)


def test_schedule_with_rule_first_compensated_update_at_wp():
    """Through warm-up the handed weights are the global ones, so at iteration wp the delay term is zero
    and the first compensated update equals the plain SGD one; from wp+1 on it differs."""
    rng = np.random.default_rng(5)
    n, W, wp = 12, 2, 2
    w = [rng.normal(0, 1, n).astype(F32)]
    v = [np.zeros(n, F32)]
    u = [[w[0].copy()] for _ in range(W)]
    w2, v2, u2 = copy_list(w), copy_list(v), [copy_list(r) for r in u]
    for i in range(5):
        g = [[rng.normal(0, 0.1, n).astype(F32)] for _ in range(W)]
        oracle.step(i, wp, w, v, g, u, 0.1, 0.1, 0.9, 0.0, 0.0, rule=("dcasgd_c", 0.5))
        oracle.step(i, wp, w2, v2, g, u2, 0.1, 0.1, 0.9, 0.0, 0.0)
        assert same_bits(w[0], w2[0]) and same_bits(v[0], v2[0])  # server side never depends on the rule
        if i <= wp:
            assert same_bits(u[0][0], u2[0][0])
        else:
            assert not same_bits(u[0][0], u2[0][0])
        u2 = [copy_list(r) for r in u]  # keep the two runs' worker state aligned for the next comparison


# --------------------------------------------------------------------------
# local momentum-SGD updater (Section 4.2: local SGD with the server's momentum)
# --------------------------------------------------------------------------
def test_local_momentum_zero_is_plain_sgd_updater_bitwise():
    rng = np.random.default_rng(6)
    w, g, u, _ = _rand(rng, 40, 3)
    lv = [[rng.normal(0, 1e-3, 40).astype(F32)] for _ in range(3)]
    ref = [[np.zeros(40, F32)] for _ in range(3)]
    oracle.local_update(w, g, ref, 0.3, 1e-3)
    oracle.local_update_momentum(w, g, u, lv, 0.3, 1e-3, 0.0)
    for m in range(3):
        assert same_bits(u[m][0], ref[m][0])
        # the stored velocity is the step just taken: u = w + lv
        assert same_bits((w[0] + lv[m][0]).astype(F32), u[m][0])


def test_single_worker_local_velocity_tracks_the_server_bitwise():
    """W=1, grad_scale=1, local_lr=lr, local momentum = server momentum, both velocities
    zero at the start and the gradient fed independent of the weights: worker and server
    perform the same operations, so u_0 == w_{t+1} and lv_0 == v after every iteration."""
    rng = np.random.default_rng(7)
    n = 30
    w = [rng.normal(0, 1, n).astype(F32)]
    v = [np.zeros(n, F32)]
    u = [[w[0].copy()]]
    lv = [[np.zeros(n, F32)]]
    for i in range(6):
        g = [[rng.normal(0, 0.1, n).astype(F32)]]
        oracle.step(i, 0, w, v, g, u, 0.1, 0.1, 0.9, 1e-3, 1.0, rule=("momentum", 0.9, lv))
        assert same_bits(u[0][0], w[0]) and same_bits(lv[0][0], v[0])


def test_local_momentum_constant_gradient_closed_form():
    """Constant g, wd = 0, lv_0 = 0: lv_t = -ll g (1 - mu^t)/(1 - mu); u_t = w + lv_t."""
    ll, mu, g0 = F(1, 8), F(1, 2), F(3, 4)
    w = [arr([2.0], np.float64)]
    u = [[arr([0.0], np.float64)]]
    lv = [[arr([0.0], np.float64)]]
    for t in range(1, 12):
        oracle.local_update_momentum(w, [[arr([float(g0)], np.float64)]], u, lv, float(ll), 0.0, float(mu))
        expect = -ll * g0 * (1 - mu ** t) / (1 - mu)
        assert lv[0][0][0] == float(expect) and u[0][0][0] == float(2 + expect)  # dyadic: exact


def test_local_momentum_against_library_momentum_sgd():
    """A worker whose pulled weights are its own previous result (server frozen out:
    w := u after every step) runs textbook momentum SGD; cross-check with torch.optim.SGD."""
    import torch
    rng = np.random.default_rng(8)
    n, ll, mu, wd = 9, 0.05, 0.9, 1e-2
    a = rng.uniform(0.5, 2.0, n)
    x0 = rng.normal(0, 1, n)
    p = torch.nn.Parameter(torch.tensor(x0))
    opt = torch.optim.SGD([p], lr=ll, momentum=mu, weight_decay=wd)
    w = [x0.copy()]
    u = [[np.zeros(n)]]
    lv = [[np.zeros(n)]]
    for _ in range(20):
        g = a * w[0]
        oracle.local_update_momentum(w, [[g]], u, lv, ll, wd, mu)
        w[0][...] = u[0][0]
        p.grad = torch.tensor(a * p.detach().numpy())
        opt.step()
        assert max_rel_err(w[0], p.detach().numpy()) < 1e-12
