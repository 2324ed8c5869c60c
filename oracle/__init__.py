"""ctypes access to the CPU oracle (oracle/wash_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py.  The product package never imports this.
All arrays are host numpy arrays; nothing here touches a GPU.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None
MAX_N = 32


class Segment(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_uint64), ("length", ctypes.c_uint64), ("p", ctypes.c_double)]


def _bind(L):
    """Declare the argument and result types of every oracle entry point on a loaded library."""
    u32, u64, dbl = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_double
    vp = ctypes.c_void_p
    L.wash_ref_philox4x32_10.argtypes = [vp, vp, vp]
    L.wash_ref_philox4x32_10.restype = None
    L.wash_ref_threshold.argtypes = [dbl]
    L.wash_ref_threshold.restype = u64
    L.wash_ref_mask_word.argtypes = [u64, u64, u64]
    L.wash_ref_mask_word.restype = u32
    L.wash_ref_perm_words.argtypes = [u64, u64, u64, u32, vp]
    L.wash_ref_perm_words.restype = None
    L.wash_ref_fisher_yates.argtypes = [vp, u32, vp]
    L.wash_ref_fisher_yates.restype = None
    L.wash_ref_permutation.argtypes = [u64, u64, u64, u32, vp]
    L.wash_ref_permutation.restype = ctypes.c_int
    L.wash_layer_probs_ref.argtypes = [dbl, u32, ctypes.c_int, vp]
    L.wash_layer_probs_ref.restype = ctypes.c_int
    L.wash_shuffle_ref_window.argtypes = [vp, vp, u32, u64, u64, u64, u64, vp, u32, u64, u64, vp]
    L.wash_shuffle_ref_window.restype = ctypes.c_int
    L.wash_shuffle_ref.argtypes = [vp, vp, u32, u64, vp, u32, u64, u64, vp]
    L.wash_shuffle_ref.restype = ctypes.c_int
    L.wash_shuffle_ref_mt.argtypes = [vp, vp, u32, u64, vp, u32, u64, u64, vp, u32]
    L.wash_shuffle_ref_mt.restype = ctypes.c_int
    L.wash_ref_log2.argtypes = [dbl]
    L.wash_ref_log2.restype = dbl
    L.wash_ref_gap_scale.argtypes = [dbl]
    L.wash_ref_gap_scale.restype = dbl
    L.wash_ref_gap_uniform.argtypes = [u64, u64, u64, u32]
    L.wash_ref_gap_uniform.restype = u64
    L.wash_ref_gap.argtypes = [u64, dbl]
    L.wash_ref_gap.restype = u32
    L.wash_shuffle_gap_ref_window.argtypes = [vp, vp, u32, u64, u64, u64, u64, vp, u32, u64, u64, vp]
    L.wash_shuffle_gap_ref_window.restype = ctypes.c_int
    L.wash_shuffle_gap_ref.argtypes = [vp, vp, u32, u64, vp, u32, u64, u64, vp]
    L.wash_shuffle_gap_ref.restype = ctypes.c_int
    L.wash_shuffle_gap_ref_mt.argtypes = [vp, vp, u32, u64, vp, u32, u64, u64, vp, u32]
    L.wash_shuffle_gap_ref_mt.restype = ctypes.c_int
    L.wash_ref_gap_mask.argtypes = [vp, u64, vp, u32, u64, u64]
    L.wash_ref_gap_mask.restype = ctypes.c_int
    L.wash_consensus_sqdist_ref.argtypes = [vp, u32, u64, u64, u64, vp]
    L.wash_consensus_sqdist_ref.restype = ctypes.c_int
    L.wash_weighted_average_ref.argtypes = [vp, vp, vp, u32, u64]
    L.wash_weighted_average_ref.restype = ctypes.c_int
    L.wash_average_ref.argtypes = [vp, vp, u32, u64]
    L.wash_average_ref.restype = ctypes.c_int
    L.papa_ema_ref.argtypes = [vp, u32, u64, ctypes.c_float]
    L.papa_ema_ref.restype = ctypes.c_int
    return L


def lib():
    global _LIB
    if _LIB is None:
        _LIB = _bind(ctypes.CDLL(_build.build(force=False)))
    return _LIB


def use_library(path):
    """Point every wrapper of this module at another build of the oracle (None = the regular
    one).  For tests that plant a mistake in a copy of the source and check that the pins notice."""
    global _LIB
    _LIB = None if path is None else _bind(ctypes.CDLL(path))


def _segarray(segs):
    arr = (Segment * max(len(segs), 1))()
    for k, (off, length, p) in enumerate(segs):
        arr[k].offset, arr[k].length, arr[k].p = int(off), int(length), float(p)
    return arr


def _check_pop(a, name):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.ndim == 2 and a.flags.c_contiguous):
        raise TypeError(f"{name}: need a C-contiguous float32 [N, P] numpy array")


def philox(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    o = np.zeros(4, dtype=np.uint32)
    lib().wash_ref_philox4x32_10(c.ctypes.data, k.ctypes.data, o.ctypes.data)
    return tuple(int(v) for v in o)


def threshold(p):
    return int(lib().wash_ref_threshold(float(p)))


def mask_word(seed, step, g):
    return int(lib().wash_ref_mask_word(seed, step, g))


def perm_words(seed, step, g, N):
    w = np.zeros(max(N - 1, 1), dtype=np.uint32)
    lib().wash_ref_perm_words(seed, step, g, N, w.ctypes.data)
    return w[: N - 1]


def fisher_yates(words, N):
    w = np.ascontiguousarray(np.asarray(words, dtype=np.uint32))
    if w.size < N - 1:
        raise ValueError("need N-1 words")
    w = np.concatenate([w, np.zeros(1, np.uint32)])
    perm = np.zeros(N, dtype=np.uint32)
    lib().wash_ref_fisher_yates(w.ctypes.data, N, perm.ctypes.data)
    return perm


def permutation(seed, step, g, N):
    perm = np.zeros(N, dtype=np.uint32)
    rc = lib().wash_ref_permutation(seed, step, g, N, perm.ctypes.data)
    if rc != 0:
        raise ValueError("wash_ref_permutation failed")
    return perm


def layer_probs(p, L, schedule=0):
    out = np.zeros(max(L, 1), dtype=np.float64)
    rc = lib().wash_layer_probs_ref(float(p), int(L), int(schedule), out.ctypes.data)
    if rc != 0:
        raise ValueError("wash_layer_probs_ref: invalid argument")
    return out[:L]


def log2(x):
    return float(lib().wash_ref_log2(float(x)))


def gap_scale(p):
    return float(lib().wash_ref_gap_scale(float(p)))


def gap_uniform(seed, step, s, d):
    return int(lib().wash_ref_gap_uniform(seed, step, s, d))


def gap(U, inv):
    return int(lib().wash_ref_gap(int(U), float(inv)))


def gap_mask(P, segs, seed, step):
    """uint8 [P]: 1 where the gap stream selects the coordinate."""
    mask = np.zeros(P, dtype=np.uint8)
    sa = _segarray(segs)
    rc = lib().wash_ref_gap_mask(mask.ctypes.data, P, ctypes.addressof(sa), len(segs), seed, step)
    if rc != 0:
        raise ValueError("wash_ref_gap_mask: invalid argument")
    return mask


def shuffle(params, momentum, segs, seed, step, threads=1, stream="v1"):
    """In-place shuffle of a whole [N, P] population. Returns the selected count.
    stream: "v1" (one mask word per coordinate) or "gap" (geometric gap sampling)."""
    _check_pop(params, "params")
    N, P = params.shape
    if momentum is not None:
        _check_pop(momentum, "momentum")
        assert momentum.shape == params.shape
    sa = _segarray(segs)
    cnt = ctypes.c_uint64(0)
    mom = momentum.ctypes.data if momentum is not None else None
    if stream not in ("v1", "gap"):
        raise ValueError("stream must be 'v1' or 'gap'")
    one = lib().wash_shuffle_ref if stream == "v1" else lib().wash_shuffle_gap_ref
    many = lib().wash_shuffle_ref_mt if stream == "v1" else lib().wash_shuffle_gap_ref_mt
    if threads <= 1:
        rc = one(params.ctypes.data, mom, N, P, ctypes.addressof(sa), len(segs), seed, step, ctypes.addressof(cnt))
    else:
        rc = many(params.ctypes.data, mom, N, P, ctypes.addressof(sa), len(segs), seed, step,
                  ctypes.addressof(cnt), threads)
    if rc != 0:
        raise ValueError(f"wash_shuffle_ref: invalid argument (rc={rc})")
    return cnt.value


def shuffle_window(win, mom_win, P, g_begin, segs, seed, step, stream="v1"):
    """In-place shuffle of a window holding columns [g_begin, g_begin + W) of a
    population with P columns; win is a contiguous [N, W] array.  For the gap
    stream the window must start and end on multiples of 1024 (or at P)."""
    _check_pop(win, "win")
    N, W = win.shape
    if mom_win is not None:
        _check_pop(mom_win, "mom_win")
        assert mom_win.shape == win.shape
    sa = _segarray(segs)
    cnt = ctypes.c_uint64(0)
    mom = mom_win.ctypes.data if mom_win is not None else None
    fn = lib().wash_shuffle_ref_window if stream == "v1" else lib().wash_shuffle_gap_ref_window
    rc = fn(win.ctypes.data, mom, N, P, W, g_begin, g_begin + W,
            ctypes.addressof(sa), len(segs), seed, step, ctypes.addressof(cnt))
    if rc != 0:
        raise ValueError(f"wash_shuffle_ref_window: invalid argument (rc={rc})")
    return cnt.value


def average(params):
    _check_pop(params, "params")
    N, P = params.shape
    out = np.empty(P, dtype=np.float32)
    rc = lib().wash_average_ref(params.ctypes.data, out.ctypes.data, N, P)
    if rc != 0:
        raise ValueError("wash_average_ref: invalid argument")
    return out


def ema(params, alpha):
    """In-place PAPA EMA of a whole [N, P] population."""
    _check_pop(params, "params")
    N, P = params.shape
    rc = lib().papa_ema_ref(params.ctypes.data, N, P, float(alpha))
    if rc != 0:
        raise ValueError("papa_ema_ref: invalid argument")
    return params


def consensus_sqdist(params, g_begin=0, g_end=None):
    """float64 [N]: sum over coordinates [g_begin, g_end) of (theta_n - mean)^2."""
    _check_pop(params, "params")
    N, P = params.shape
    if g_end is None:
        g_end = P
    out = np.zeros(N, dtype=np.float64)
    rc = lib().wash_consensus_sqdist_ref(params.ctypes.data, N, P, int(g_begin), int(g_end), out.ctypes.data)
    if rc != 0:
        raise ValueError("wash_consensus_sqdist_ref: invalid argument")
    return out


def weighted_average(params, weights):
    _check_pop(params, "params")
    N, P = params.shape
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.float64))
    if w.shape != (N,):
        raise ValueError("need N weights")
    out = np.empty(P, dtype=np.float32)
    rc = lib().wash_weighted_average_ref(params.ctypes.data, w.ctypes.data, out.ctypes.data, N, P)
    if rc != 0:
        raise ValueError("wash_weighted_average_ref: invalid argument")
    return out
