"""ctypes binding of libodsgd.so (C ABI declared in include/odsgd.h).

Argument marshalling only: every arithmetic step runs in the HIP kernels.
PyTorch supplies device memory (tensors -> data_ptr) and the current stream.
There is no fallback: if the library has not been built the first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

ODSGD_OK = 0
ODSGD_EINVAL = -1
ODSGD_EALIGN = -2
ODSGD_EALIAS = -3
ODSGD_ENOSPC = -4
ODSGD_EHIP = -5
ODSGD_ERANGE = -6
ODSGD_ESTALE = -7
ODSGD_STATIC_PLAN_BYTES = 16 << 20
ODSGD_MAX_WORKERS = 64
ODSGD_LOCAL_SGD = 0
ODSGD_LOCAL_DCASGD_C = 1
ODSGD_LOCAL_DCASGD_A = 2
ODSGD_LOCAL_SGD_MOMENTUM = 3


class odsgd_hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("local_lr", ctypes.c_float),
                ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float)]


class odsgd_local_rule(ctypes.Structure):
    _fields_ = [("rule", ctypes.c_int), ("lambda_", ctypes.c_float),
                ("ms_decay", ctypes.c_float), ("epsilon", ctypes.c_float),
                ("local_momentum", ctypes.c_float)]


class OdsgdError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, odsgd_strerror(code)))


def library_path():
    return os.environ.get("ODSGD_LIB", os.path.join(_HERE, "libodsgd.so"))


def lib():
    """Load libodsgd.so (once) and declare the C signatures."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(
            "%s not found: build it first (python -m paper_2005_06728_amd.build); "
            "there is no CPU fallback" % path)
    L = ctypes.CDLL(path)
    vp, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)
    hp = ctypes.POINTER(odsgd_hyper)
    L.odsgd_workspace_bytes.restype = ctypes.c_size_t
    L.odsgd_workspace_bytes.argtypes = [ctypes.c_int, i64p, ctypes.c_int]
    L.odsgd_init.restype = ctypes.c_int
    L.odsgd_init.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, vp, vp, vp, vp,
                             ctypes.c_int, vp, ctypes.c_size_t, vp]
    L.odsgd_init_static.restype = ctypes.c_int
    L.odsgd_init_static.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, vp, vp, vp, vp, ctypes.c_int, vp]
    L.odsgd_plan_host.restype = ctypes.c_int
    L.odsgd_plan_host.argtypes = [ctypes.c_int, i64p, vp, vp, vp, vp, ctypes.c_int, vp, ctypes.c_size_t,
                                  ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                  ctypes.POINTER(ctypes.c_size_t)]
    L.odsgd_plan_residency.restype = ctypes.c_int
    L.odsgd_plan_residency.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                                       ctypes.c_size_t, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int),
                                       ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_int)]
    L.odsgd_set_double_buffer.restype = ctypes.c_int
    L.odsgd_set_double_buffer.argtypes = [vp, vp, vp, vp]
    L.odsgd_current_buffers.restype = ctypes.c_int
    L.odsgd_current_buffers.argtypes = [vp]
    L.odsgd_probe_streams.restype = ctypes.c_int
    L.odsgd_probe_streams.argtypes = [vp, vp]
    L.odsgd_local_update.restype = ctypes.c_int
    L.odsgd_local_update.argtypes = [vp, ctypes.c_int, hp, vp]
    for name in ("odsgd_global_update", "odsgd_step", "odsgd_ssgd_step"):
        fn = getattr(L, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [vp, hp, vp]
    L.odsgd_set_local_rule.restype = ctypes.c_int
    L.odsgd_set_local_rule.argtypes = [vp, ctypes.POINTER(odsgd_local_rule), vp, vp]
    L.odsgd_set_warmup.restype = ctypes.c_int
    L.odsgd_set_warmup.argtypes = [vp, ctypes.c_int64]
    L.odsgd_get_iteration.restype = ctypes.c_int64
    L.odsgd_get_iteration.argtypes = [vp]
    L.odsgd_set_iteration.restype = ctypes.c_int
    L.odsgd_set_iteration.argtypes = [vp, ctypes.c_int64]
    L.odsgd_probe_copy.restype = ctypes.c_int
    L.odsgd_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.odsgd_destroy.restype = ctypes.c_int
    L.odsgd_destroy.argtypes = [vp]
    L.odsgd_strerror.restype = ctypes.c_char_p
    L.odsgd_strerror.argtypes = [ctypes.c_int]
    _LIB = L
    return L


def odsgd_strerror(code):
    return lib().odsgd_strerror(int(code)).decode()


def _i64_array(vals):
    return (ctypes.c_int64 * len(vals))(*[int(v) for v in vals])


def _ptr_row(ptrs):
    return (ctypes.c_void_p * len(ptrs))(*[ctypes.c_void_p(int(p)) for p in ptrs])


def _ptr_rows(rows):
    """[W][K] integers -> (array of W pointers to arrays of K pointers, keep-alive list)."""
    keep = [_ptr_row(r) for r in rows]
    top = (ctypes.c_void_p * len(rows))(*[ctypes.cast(r, ctypes.c_void_p) for r in keep])
    return top, keep


def odsgd_workspace_bytes(numel, num_workers):
    return int(lib().odsgd_workspace_bytes(len(numel), _i64_array(numel), int(num_workers)))


def odsgd_init(numel, w_ptrs, mom_ptrs, grad_ptrs, local_ptrs, num_workers,
               workspace_ptr, workspace_bytes, stream=0):
    """Raw form: integers in, handle (int) out.  grad_ptrs/local_ptrs are [W][K]."""
    out = ctypes.c_void_p()
    g_top, g_keep = _ptr_rows(grad_ptrs)
    u_top, u_keep = _ptr_rows(local_ptrs)
    w_row, m_row, n_arr = _ptr_row(w_ptrs), _ptr_row(mom_ptrs), _i64_array(numel)
    rc = lib().odsgd_init(ctypes.byref(out), len(numel), n_arr,
                          ctypes.cast(w_row, ctypes.c_void_p), ctypes.cast(m_row, ctypes.c_void_p),
                          ctypes.cast(g_top, ctypes.c_void_p), ctypes.cast(u_top, ctypes.c_void_p),
                          int(num_workers), ctypes.c_void_p(int(workspace_ptr)),
                          int(workspace_bytes), ctypes.c_void_p(int(stream)))
    del g_keep, u_keep, w_row, m_row, n_arr
    if rc != ODSGD_OK:
        raise OdsgdError(rc, "odsgd_init")
    return out.value


def odsgd_init_static(numel, w_ptrs, mom_ptrs, grad_ptrs, local_ptrs, num_workers, stream=0):
    """odsgd_init without a workspace: the tables go into the library's static device array."""
    out = ctypes.c_void_p()
    g_top, g_keep = _ptr_rows(grad_ptrs)
    u_top, u_keep = _ptr_rows(local_ptrs)
    w_row, m_row, n_arr = _ptr_row(w_ptrs), _ptr_row(mom_ptrs), _i64_array(numel)
    rc = lib().odsgd_init_static(ctypes.byref(out), len(numel), n_arr,
                                 ctypes.cast(w_row, ctypes.c_void_p), ctypes.cast(m_row, ctypes.c_void_p),
                                 ctypes.cast(g_top, ctypes.c_void_p), ctypes.cast(u_top, ctypes.c_void_p),
                                 int(num_workers), ctypes.c_void_p(int(stream)))
    del g_keep, u_keep, w_row, m_row, n_arr
    if rc != ODSGD_OK:
        raise OdsgdError(rc, "odsgd_init_static")
    return out.value


ROW_ELEMS = 1 << 29  # elements per pointer-table row (see odsgd_plan_host in odsgd.h)


def odsgd_plan_host(numel, w_ptrs, mom_ptrs, grad_ptrs, local_ptrs, num_workers):
    """Host-only: the tables odsgd_init would upload.  Returns (pointer_rows, chunks)
    with pointer_rows[r] = list of 4 + 3W addresses and chunks = list of
    (row, vec, count, offset, second_half)."""
    import struct
    nbytes = odsgd_workspace_bytes(numel, num_workers)
    if nbytes == 0:
        raise OdsgdError(ODSGD_EINVAL, "odsgd_workspace_bytes")
    buf = ctypes.create_string_buffer(nbytes)
    g_top, g_keep = _ptr_rows(grad_ptrs)
    u_top, u_keep = _ptr_rows(local_ptrs)
    w_row, m_row, n_arr = _ptr_row(w_ptrs), _ptr_row(mom_ptrs), _i64_array(numel)
    nrows, nch, off = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_size_t()
    rc = lib().odsgd_plan_host(len(numel), n_arr, ctypes.cast(w_row, ctypes.c_void_p),
                               ctypes.cast(m_row, ctypes.c_void_p), ctypes.cast(g_top, ctypes.c_void_p),
                               ctypes.cast(u_top, ctypes.c_void_p), int(num_workers), buf, nbytes,
                               ctypes.byref(nrows), ctypes.byref(nch), ctypes.byref(off))
    del g_keep, u_keep
    if rc != ODSGD_OK:
        raise OdsgdError(rc, "odsgd_plan_host")
    stride = 4 + 3 * num_workers
    raw = buf.raw
    rows = [list(struct.unpack_from("<%dQ" % stride, raw, r * stride * 8)) for r in range(nrows.value)]
    chunks = []
    for c in range(nch.value):
        t, cnt, o, second = struct.unpack_from("<4I", raw, off.value + 16 * c)
        chunks.append((t & 0x7fffffff, bool(t >> 31), cnt, o, second))
    return rows, chunks


def chunk_elements(chunk):
    """Element ranges (start, stop) inside its row that a chunk tuple of odsgd_plan_host covers."""
    _, _, cnt, off, second = chunk
    if second == 0:
        return [(off, off + cnt)]
    assert cnt == 256
    return [(off, off + 128), (off + 4 * (32 + second), off + 4 * (32 + second) + 128)]


ODSGD_ENTRY_STEP, ODSGD_ENTRY_SSGD_STEP, ODSGD_ENTRY_GLOBAL_UPDATE, ODSGD_ENTRY_LOCAL_UPDATE = 0, 1, 2, 3


def odsgd_plan_residency(entry, rule, num_workers, waves_override=0, lds_per_cu=160 * 1024, lds_granule=1280,
                         max_request=64 * 1024):
    """Host-only: (waves wanted, LDS bytes requested, waves achieved) for a CU of the given LDS geometry."""
    wanted, lds, got = ctypes.c_int(), ctypes.c_size_t(), ctypes.c_int()
    _call("odsgd_plan_residency",
          lib().odsgd_plan_residency(int(entry), int(rule), int(num_workers), int(waves_override), int(lds_per_cu),
                                     int(lds_granule), int(max_request), ctypes.byref(wanted), ctypes.byref(lds),
                                     ctypes.byref(got)))
    return wanted.value, lds.value, got.value


def _hyper(h):
    if isinstance(h, odsgd_hyper):
        return h
    return odsgd_hyper(*[float(x) for x in h])


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _call(name, rc):
    if rc != ODSGD_OK:
        raise OdsgdError(rc, name)


def odsgd_local_update(handle, worker, hyper, stream=None):
    _call("odsgd_local_update",
          lib().odsgd_local_update(handle, int(worker), ctypes.byref(_hyper(hyper)), _stream(stream)))


def odsgd_global_update(handle, hyper, stream=None):
    _call("odsgd_global_update",
          lib().odsgd_global_update(handle, ctypes.byref(_hyper(hyper)), _stream(stream)))


def odsgd_step(handle, hyper, stream=None):
    _call("odsgd_step", lib().odsgd_step(handle, ctypes.byref(_hyper(hyper)), _stream(stream)))


def odsgd_ssgd_step(handle, hyper, stream=None):
    _call("odsgd_ssgd_step",
          lib().odsgd_ssgd_step(handle, ctypes.byref(_hyper(hyper)), _stream(stream)))


def odsgd_set_local_rule(handle, rule, lam=0.0, ms_decay=0.0, epsilon=0.0, state_ptrs=None,
                         stream=None, local_momentum=0.0):
    """rule: ODSGD_LOCAL_*; state_ptrs: [W][K] integers (DCASGD_A: MeanSquare, SGD_MOMENTUM: velocity)."""
    r = odsgd_local_rule(int(rule), float(lam), float(ms_decay), float(epsilon), float(local_momentum))
    top, keep = (None, None) if state_ptrs is None else _ptr_rows(state_ptrs)
    rc = lib().odsgd_set_local_rule(handle, ctypes.byref(r),
                                    None if top is None else ctypes.cast(top, ctypes.c_void_p),
                                    _stream(stream))
    del keep
    _call("odsgd_set_local_rule", rc)


def odsgd_set_double_buffer(handle, w_alt_ptrs, mom_alt_ptrs, stream=None):
    """Register the second (w, mom) buffer pair: odsgd_global_update becomes out of place."""
    a, b = _ptr_row(w_alt_ptrs), _ptr_row(mom_alt_ptrs)
    _call("odsgd_set_double_buffer",
          lib().odsgd_set_double_buffer(handle, ctypes.cast(a, ctypes.c_void_p), ctypes.cast(b, ctypes.c_void_p),
                                        _stream(stream)))


def odsgd_current_buffers(handle):
    return int(lib().odsgd_current_buffers(handle))


def odsgd_probe_streams(handle, stream=None):
    _call("odsgd_probe_streams", lib().odsgd_probe_streams(handle, _stream(stream)))


def odsgd_set_warmup(handle, warmup_steps):
    _call("odsgd_set_warmup", lib().odsgd_set_warmup(handle, int(warmup_steps)))


def odsgd_get_iteration(handle):
    return int(lib().odsgd_get_iteration(handle))


def odsgd_set_iteration(handle, iteration):
    _call("odsgd_set_iteration", lib().odsgd_set_iteration(handle, int(iteration)))


def odsgd_probe_copy(dst, src, stream=None):
    """Copy tensor src into dst (contiguous fp32 CUDA tensors of equal size)."""
    assert dst.numel() == src.numel() and dst.dtype == src.dtype == torch.float32
    _call("odsgd_probe_copy", lib().odsgd_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel(),
                                                     _stream(stream)))


def odsgd_destroy(handle):
    _call("odsgd_destroy", lib().odsgd_destroy(handle))


class Engine:
    """Convenience owner of a handle: keeps the registered tensors and the
    workspace alive and forwards to the C entry points of the same name."""

    def __init__(self, w, mom, grads, local_w, warmup_steps=0, stream=None, static_plan=False):
        """static_plan=True registers through odsgd_init_static (no workspace tensor)."""
        self.w, self.mom, self.grads, self.local_w = w, mom, grads, local_w
        W = len(grads)
        for t in list(w) + list(mom) + [x for r in grads for x in r] + [x for r in local_w for x in r]:
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
                raise ValueError("tensors must be contiguous fp32 CUDA tensors")
        numel = [t.numel() for t in w]
        ptrs = ([t.data_ptr() for t in w], [t.data_ptr() for t in mom],
                [[t.data_ptr() for t in r] for r in grads], [[t.data_ptr() for t in r] for r in local_w])
        self.handle = None
        if static_plan:
            self.workspace = None
            self.handle = odsgd_init_static(numel, *ptrs, W, _stream(stream))
        else:
            nbytes = odsgd_workspace_bytes(numel, W)
            if nbytes == 0:
                raise OdsgdError(ODSGD_EINVAL, "odsgd_workspace_bytes")
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=w[0].device)
            self.handle = odsgd_init(numel, *ptrs, W, self.workspace.data_ptr(), nbytes, _stream(stream))
        if warmup_steps:
            odsgd_set_warmup(self.handle, warmup_steps)

    def set_local_rule(self, rule, lam=0.0, ms_decay=0.0, epsilon=0.0, mean_square=None, stream=None,
                       local_momentum=0.0, local_velocity=None):
        """mean_square / local_velocity: [W][K] fp32 CUDA tensors holding the per-worker
        state of DCASGD_A / SGD_MOMENTUM."""
        state = mean_square if mean_square is not None else local_velocity
        self.local_state = state
        ptrs = None if state is None else [[t.data_ptr() for t in r] for r in state]
        odsgd_set_local_rule(self.handle, rule, lam, ms_decay, epsilon, ptrs, stream, local_momentum)

    def set_double_buffer(self, w_alt, mom_alt, stream=None):
        """w_alt / mom_alt: [K] fp32 CUDA tensors, the second buffer pair of the out-of-place global update."""
        self.w_alt, self.mom_alt = w_alt, mom_alt
        odsgd_set_double_buffer(self.handle, [t.data_ptr() for t in w_alt], [t.data_ptr() for t in mom_alt], stream)

    @property
    def current_buffers(self):
        return odsgd_current_buffers(self.handle)

    def current_w(self):
        return self.w_alt if self.current_buffers else self.w

    def current_mom(self):
        return self.mom_alt if self.current_buffers else self.mom

    def probe_streams(self, stream=None):
        odsgd_probe_streams(self.handle, stream)

    def step(self, hyper, stream=None):
        odsgd_step(self.handle, hyper, stream)

    def ssgd_step(self, hyper, stream=None):
        odsgd_ssgd_step(self.handle, hyper, stream)

    def local_update(self, worker, hyper, stream=None):
        odsgd_local_update(self.handle, worker, hyper, stream)

    def global_update(self, hyper, stream=None):
        odsgd_global_update(self.handle, hyper, stream)

    @property
    def iteration(self):
        return odsgd_get_iteration(self.handle)

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            odsgd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
