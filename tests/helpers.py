"""Small array helpers shared by the tests (no update arithmetic here)."""
import numpy as np


def split(flat, sizes, dtype=np.float32):
    """Flat list of numbers -> list of 1-D arrays with the given sizes."""
    flat = np.asarray(flat, dtype=dtype)
    out, o = [], 0
    for n in sizes:
        out.append(np.ascontiguousarray(flat[o:o + n]))
        o += n
    assert o == flat.shape[0]
    return out


def cat(arrs):
    return np.concatenate([np.asarray(a).ravel() for a in arrs])


def bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint32 if a.dtype == np.float32 else np.uint64)


def same_bits(a, b):
    """Bitwise equality, except that any NaN equals any NaN."""
    a, b = np.asarray(a), np.asarray(b)
    if a.shape != b.shape or a.dtype != b.dtype:
        return False
    both_nan = np.isnan(a) & np.isnan(b)
    return bool(np.all((bits(a) == bits(b)) | both_nan))


def max_rel_err(x, ref):
    """max_i |x_i - ref_i| / max(|ref_i|, 1e-30)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if x.size == 0:
        return 0.0
    return float(np.max(np.abs(x - ref) / np.maximum(np.abs(ref), 1e-30)))


def zeros_like_list(lst):
    return [np.zeros_like(a) for a in lst]


def copy_list(lst):
    return [a.copy() for a in lst]
