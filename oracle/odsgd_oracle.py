"""ctypes front end of the C oracle (oracle/odsgd_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this module.  It holds no arithmetic of
its own -- every number comes from the C loops -- and imports nothing from the
GPU package.

State is a plain dict of numpy arrays, one flat array per parameter tensor:
    w[k], v[k]          global weights / momentum (updated in place)
    u[m][k]             worker m's local weights (overwritten)
    g[m][k]             worker m's gradient (read only)
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build()
        _LIB = ctypes.CDLL(path)
    return _LIB


_CT = {np.dtype(np.float32): (ctypes.c_float, "f32"),
       np.dtype(np.float64): (ctypes.c_double, "f64")}


def _ptr_array(arrs, ctype):
    pp = ctypes.POINTER(ctype)
    return (pp * len(arrs))(*[a.ctypes.data_as(pp) for a in arrs])


def _check(arrs, dtype, n):
    for a in arrs:
        assert isinstance(a, np.ndarray) and a.dtype == dtype, (type(a), getattr(a, "dtype", None))
        assert a.ndim == 1 and a.shape[0] == n and a.flags.c_contiguous


def local_update(w, g, u, local_lr, weight_decay, worker=-1):
    """Worker-side local update, tensor list form. w: [K], g/u: [M][K]."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        uk = [u[m][k] for m in range(M)]
        _check([w[k]] + gk + uk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_local_" + sfx)
        fn.restype = None
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(ctypes.POINTER(ct)),
           _ptr_array(gk, ct), _ptr_array(uk, ct), ctypes.c_int(worker),
           ct(local_lr), ct(weight_decay))


def local_update_dcasgd_c(w, g, u, local_lr, weight_decay, lam, worker=-1):
    """Local update, constant delay compensation. u[m] holds the weights the
    gradient was taken at on entry and the new local weights on return."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        uk = [u[m][k] for m in range(M)]
        _check([w[k]] + gk + uk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_local_dcasgd_c_" + sfx)
        fn.restype = None
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(ctypes.POINTER(ct)),
           _ptr_array(gk, ct), _ptr_array(uk, ct), ctypes.c_int(worker),
           ct(local_lr), ct(weight_decay), ct(lam))


def local_update_dcasgd_a(w, g, u, ms, local_lr, weight_decay, lam, ms_decay, epsilon, worker=-1):
    """Local update, adaptive delay compensation; ms[m][k] is the MeanSquare state."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        uk = [u[m][k] for m in range(M)]
        mk = [ms[m][k] for m in range(M)]
        _check([w[k]] + gk + uk + mk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_local_dcasgd_a_" + sfx)
        fn.restype = None
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(ctypes.POINTER(ct)),
           _ptr_array(gk, ct), _ptr_array(uk, ct), _ptr_array(mk, ct), ctypes.c_int(worker),
           ct(local_lr), ct(weight_decay), ct(lam), ct(ms_decay), ct(epsilon))


def local_update_momentum(w, g, u, lv, local_lr, weight_decay, local_momentum, worker=-1):
    """Local momentum-SGD updater; lv[m][k] is worker m's local velocity."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        uk = [u[m][k] for m in range(M)]
        lk = [lv[m][k] for m in range(M)]
        _check([w[k]] + gk + uk + lk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_local_momentum_" + sfx)
        fn.restype = None
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(ctypes.POINTER(ct)),
           _ptr_array(gk, ct), _ptr_array(uk, ct), _ptr_array(lk, ct), ctypes.c_int(worker),
           ct(local_lr), ct(weight_decay), ct(local_momentum))


def global_update(w, v, g, lr, momentum, weight_decay, grad_scale=0.0):
    """Server-side global update, tensor list form. w, v: [K], g: [M][K]."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        _check([w[k], v[k]] + gk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_global_" + sfx)
        fn.restype = None
        P = ctypes.POINTER(ct)
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(P), v[k].ctypes.data_as(P),
           _ptr_array(gk, ct), ct(lr), ct(momentum), ct(weight_decay), ct(grad_scale))


def od_step(w, v, g, u, lr, local_lr, momentum, weight_decay, grad_scale=0.0):
    """One training-stage OD-SGD iteration over a tensor list."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        uk = [u[m][k] for m in range(M)]
        _check([w[k], v[k]] + gk + uk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_od_step_" + sfx)
        fn.restype = None
        P = ctypes.POINTER(ct)
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(P), v[k].ctypes.data_as(P),
           _ptr_array(gk, ct), _ptr_array(uk, ct), ct(lr), ct(local_lr), ct(momentum),
           ct(weight_decay), ct(grad_scale))


def ssgd_step(w, v, g, u, lr, momentum, weight_decay, grad_scale=0.0):
    """One warm-up (synchronous SGD) iteration over a tensor list."""
    M = len(g)
    for k in range(len(w)):
        dt = w[k].dtype
        ct, sfx = _CT[dt]
        n = w[k].shape[0]
        gk = [g[m][k] for m in range(M)]
        uk = [u[m][k] for m in range(M)]
        _check([w[k], v[k]] + gk + uk, dt, n)
        fn = getattr(lib(), "odsgd_oracle_ssgd_step_" + sfx)
        fn.restype = None
        P = ctypes.POINTER(ct)
        fn(ctypes.c_int64(n), ctypes.c_int(M), w[k].ctypes.data_as(P), v[k].ctypes.data_as(P),
           _ptr_array(gk, ct), _ptr_array(uk, ct), ct(lr), ct(momentum),
           ct(weight_decay), ct(grad_scale))


def step(i, warmup_steps, w, v, g, u, lr, local_lr, momentum, weight_decay, grad_scale=0.0,
         rule=None):
    """Iteration i of the whole schedule of Alg. 2: synchronous SGD while
    i < warmup_steps, one-step-delay iteration from i == warmup_steps on.

    rule: None for the SGD local updater, ("dcasgd_c", lam) or
    ("dcasgd_a", lam, ms_decay, epsilon, ms) for the delay-compensated ones,
    ("momentum", local_momentum, lv) for the local momentum-SGD updater.  By
    definition the OD iteration is the local update followed by the global one."""
    if i < warmup_steps:
        ssgd_step(w, v, g, u, lr, momentum, weight_decay, grad_scale)
    elif rule is None:
        od_step(w, v, g, u, lr, local_lr, momentum, weight_decay, grad_scale)
    else:
        if rule[0] == "dcasgd_c":
            local_update_dcasgd_c(w, g, u, local_lr, weight_decay, rule[1])
        elif rule[0] == "dcasgd_a":
            local_update_dcasgd_a(w, g, u, rule[4], local_lr, weight_decay, rule[1], rule[2], rule[3])
        elif rule[0] == "momentum":
            local_update_momentum(w, g, u, rule[2], local_lr, weight_decay, rule[1])
        else:
            raise ValueError(rule[0])
        global_update(w, v, g, lr, momentum, weight_decay, grad_scale)


def od_step_threads(w, v, g, u, lr, local_lr, momentum, weight_decay, grad_scale=0.0, threads=1):
    """od_step (float32 only) with the flat element range split statically over `threads`
    POSIX threads by oracle/threads.c; every piece runs the same C routine as od_step."""
    M, K = len(g), len(w)
    f = ctypes.c_float
    P = ctypes.POINTER(f)
    for k in range(K):
        n = w[k].shape[0]
        _check([w[k], v[k]] + [g[m][k] for m in range(M)] + [u[m][k] for m in range(M)], np.dtype(np.float32), n)
    tl = ctypes.CDLL(_build.build_threads())
    fn = lib().odsgd_oracle_od_step_f32
    numel = (ctypes.c_int64 * K)(*[a.shape[0] for a in w])
    flat = lambda rows: _ptr_array([rows[m][k] for m in range(M) for k in range(K)], f)
    tl.odsgd_oracle_threads_od_step_f32.restype = ctypes.c_int
    rc = tl.odsgd_oracle_threads_od_step_f32(
        ctypes.cast(fn, ctypes.c_void_p), ctypes.c_int(threads), ctypes.c_int(K), numel,
        _ptr_array(w, f), _ptr_array(v, f), flat(g), flat(u), ctypes.c_int(M),
        f(lr), f(local_lr), f(momentum), f(weight_decay), f(grad_scale))
    if rc != 0:
        raise RuntimeError("odsgd_oracle_threads_od_step_f32 failed")
