"""CPU oracle for the LowDiff differential-checkpoint hot path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes front end over ``lowdiff_oracle.cpp`` (numpy arrays in, numpy arrays
out).  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg
of ``bench.py`` may import this package; the product path never does, and this
package never imports the product.

Functions (all operate on host memory, single threaded):

* ``topk_ef(g, r, seg_off, seg_k, select=False)`` - per-segment top-k with an
  error-feedback residual (Comp of Algorithm 1, Sec. IV-B; rho of Sec. VII-A).
* ``merge_sparse(w, idx_list, val_list, lr)`` - ordered replay of sparse diffs
  (Recovery of Algorithm 1; Eq. (6); batched-write semantics of Sec. IV-C).
* ``snapshot(src)`` - bit copy of a bf16 layer (Snapshot of Algorithm 2).
* ``adam_replay(w, m, v, grads, step0, lr, beta1, beta2, eps)`` - dense Adam
  merge (Algorithm 2 "Merge in CPU", Eq. (4)).
* ``combine_sparse(idx_list, val_list, n, scale)`` - N per-worker record lists
  combined into one (Sync of Algorithm 1, Eq. (3)): values at equal indices added
  in worker order.
* ``sparse_adam_replay(w, m, v, idx_list, val_list, step0, lr, beta1, beta2, eps)``
  - sparse diffs replayed through Adam (Recovery of Algorithm 1 with the update
  the paper names there).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lowdiff_oracle.cpp")
# LOWDIFF_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (host code only); the process must then have been started with the
# sanitizer runtime preloaded (tests/test_oracle_sanitized.py does that in a child process).
SANITIZED = os.environ.get("LOWDIFF_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "liblowdiff_oracle_san.so" if SANITIZED else "liblowdiff_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-fno-omit-frame-pointer"] if SANITIZED else ["-O2"]
        cmd = ["g++"] + opt + ["-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-o", _LIB + ".tmp", _SRC]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        lib.oracle_topk_ef.argtypes = [p, p, p, p, ctypes.c_int32, p, p]
        lib.oracle_topk_ef.restype = ctypes.c_int
        lib.oracle_topk_select.argtypes = [p, p, p, p, ctypes.c_int32, p, p]
        lib.oracle_topk_select.restype = ctypes.c_int
        lib.oracle_merge_sparse.argtypes = [p, ctypes.c_int64, p, p, p, ctypes.c_int32,
                                            ctypes.c_float]
        lib.oracle_merge_sparse.restype = ctypes.c_int
        lib.oracle_snapshot.argtypes = [p, p, ctypes.c_int64]
        lib.oracle_snapshot.restype = None
        lib.oracle_adam_replay.argtypes = [p, p, p, ctypes.c_int64, p, ctypes.c_int32,
                                           ctypes.c_int64, ctypes.c_float, ctypes.c_float,
                                           ctypes.c_float, ctypes.c_float]
        lib.oracle_adam_replay.restype = None
        lib.oracle_sparse_adam_replay.argtypes = [p, p, p, ctypes.c_int64, p, p, p, ctypes.c_int32,
                                                  ctypes.c_int64, ctypes.c_float, ctypes.c_float,
                                                  ctypes.c_float, ctypes.c_float]
        lib.oracle_sparse_adam_replay.restype = ctypes.c_int
        lib.oracle_combine_sparse.argtypes = [p, p, p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, p, p]
        lib.oracle_combine_sparse.restype = ctypes.c_int64
        lib.oracle_check_diff.argtypes = [p, p, ctypes.c_int64, ctypes.c_int64, p]
        lib.oracle_check_diff.restype = None
        d = ctypes.c_double
        lib.oracle_wasted_time.argtypes = [d] * 10
        lib.oracle_wasted_time.restype = d
        lib.oracle_critical_interval.argtypes = [d] * 6
        lib.oracle_critical_interval.restype = d
        _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def topk_ef(g, r, seg_off, seg_k, select: bool = False):
    """Returns (idx int32[K], val float32[K], r_new float32[n]); inputs are not modified.

    ``select=False`` finds the k first elements by a full sort (the definition);
    ``select=True`` uses nth_element with the same comparator.
    """
    g = _c(g, np.float32)
    r_new = np.array(r, dtype=np.float32, copy=True, order="C")
    seg_off = _c(seg_off, np.int64)
    seg_k = _c(seg_k, np.int32)
    n_seg = int(seg_k.shape[0])
    assert seg_off.shape[0] == n_seg + 1 and g.shape == r_new.shape
    assert int(seg_off[0]) == 0 and int(seg_off[-1]) == g.shape[0]
    K = int(seg_k.astype(np.int64).sum())
    idx = np.empty(K, dtype=np.int32)
    val = np.empty(K, dtype=np.float32)
    fn = _load().oracle_topk_select if select else _load().oracle_topk_ef
    rc = fn(_ptr(g), _ptr(r_new), _ptr(seg_off), _ptr(seg_k), n_seg, _ptr(idx), _ptr(val))
    if rc != 0:
        raise ValueError(f"oracle_topk: malformed segment table (rc={rc})")
    return idx, val, r_new


def merge_sparse(w, idx_list, val_list, lr: float) -> np.ndarray:
    """Returns the merged copy of ``w`` after replaying the diffs in list order."""
    w_new = np.array(w, dtype=np.float32, copy=True, order="C")
    W = len(idx_list)
    assert len(val_list) == W
    idxs = [_c(a, np.int32) for a in idx_list]
    vals = [_c(a, np.float32) for a in val_list]
    K = np.array([a.shape[0] for a in idxs], dtype=np.int64)
    for a, b in zip(idxs, vals):
        assert a.shape == b.shape
    ip = (ctypes.c_void_p * max(W, 1))(*[a.ctypes.data for a in idxs])
    vp = (ctypes.c_void_p * max(W, 1))(*[a.ctypes.data for a in vals])
    rc = _load().oracle_merge_sparse(_ptr(w_new), w_new.shape[0], ip, vp, _ptr(K), W,
                                     ctypes.c_float(lr))
    if rc != 0:
        raise ValueError("oracle_merge_sparse: index out of range")
    return w_new


def snapshot(src) -> np.ndarray:
    """Bit copy of a bf16 layer given as uint16 bit patterns."""
    src = _c(src, np.uint16)
    dst = np.empty_like(src)
    _load().oracle_snapshot(_ptr(src), _ptr(dst), src.shape[0])
    return dst


def adam_replay(w, m, v, grads, step0: int, lr: float, beta1: float, beta2: float, eps: float):
    """Replays ``grads`` (list of uint16 bf16 bit patterns) as Adam steps step0+1..step0+W.

    Returns new (w, m, v) float32 arrays; inputs are not modified.
    """
    w2 = np.array(w, dtype=np.float32, copy=True, order="C")
    m2 = np.array(m, dtype=np.float32, copy=True, order="C")
    v2 = np.array(v, dtype=np.float32, copy=True, order="C")
    gs = [_c(a, np.uint16) for a in grads]
    for a in gs:
        assert a.shape == w2.shape
    W = len(gs)
    gp = (ctypes.c_void_p * max(W, 1))(*[a.ctypes.data for a in gs])
    _load().oracle_adam_replay(_ptr(w2), _ptr(m2), _ptr(v2), w2.shape[0], gp, W, int(step0),
                               ctypes.c_float(lr), ctypes.c_float(beta1),
                               ctypes.c_float(beta2), ctypes.c_float(eps))
    return w2, m2, v2


def sparse_adam_replay(w, m, v, idx_list, val_list, step0: int, lr: float, beta1: float, beta2: float,
                       eps: float):
    """Replays sparse diffs as Adam steps step0+1..step0+W (gradient zero off the records).

    Returns new (w, m, v) float32 arrays; inputs are not modified.
    """
    w2 = np.array(w, dtype=np.float32, copy=True, order="C")
    m2 = np.array(m, dtype=np.float32, copy=True, order="C")
    v2 = np.array(v, dtype=np.float32, copy=True, order="C")
    W = len(idx_list)
    assert len(val_list) == W
    idxs = [_c(a, np.int32) for a in idx_list]
    vals = [_c(a, np.float32) for a in val_list]
    K = np.array([a.shape[0] for a in idxs], dtype=np.int64)
    for a, b in zip(idxs, vals):
        assert a.shape == b.shape
    ip = (ctypes.c_void_p * max(W, 1))(*[a.ctypes.data for a in idxs])
    vp = (ctypes.c_void_p * max(W, 1))(*[a.ctypes.data for a in vals])
    rc = _load().oracle_sparse_adam_replay(_ptr(w2), _ptr(m2), _ptr(v2), w2.shape[0], ip, vp, _ptr(K), W,
                                           int(step0), ctypes.c_float(lr), ctypes.c_float(beta1),
                                           ctypes.c_float(beta2), ctypes.c_float(eps))
    if rc != 0:
        raise ValueError("oracle_sparse_adam_replay: index out of range")
    return w2, m2, v2


def combine_sparse(idx_list, val_list, n: int, scale: float = 1.0):
    """Combines per-worker record lists; returns (idx int32[Kout], val float32[Kout])."""
    N = len(idx_list)
    assert len(val_list) == N
    idxs = [_c(a, np.int32) for a in idx_list]
    vals = [_c(a, np.float32) for a in val_list]
    K = np.array([a.shape[0] for a in idxs], dtype=np.int64)
    for a, b in zip(idxs, vals):
        assert a.shape == b.shape
    total = int(K.sum())
    out_i = np.empty(max(total, 1), dtype=np.int32)
    out_v = np.empty(max(total, 1), dtype=np.float32)
    ip = (ctypes.c_void_p * max(N, 1))(*[a.ctypes.data for a in idxs])
    vp = (ctypes.c_void_p * max(N, 1))(*[a.ctypes.data for a in vals])
    cnt = _load().oracle_combine_sparse(ip, vp, _ptr(K), N, int(n), ctypes.c_float(scale), _ptr(out_i), _ptr(out_v))
    if cnt < 0:
        raise ValueError("oracle_combine_sparse: index out of range or not ascending")
    return out_i[:cnt].copy(), out_v[:cnt].copy()


def check_diff(idx, val, n: int):
    """(out of range, not ascending, NaN) counts of one differential; `val` may be None."""
    i = _c(idx, np.int32)
    v = None if val is None else _c(val, np.float32)
    out = np.zeros(3, dtype=np.int64)
    _load().oracle_check_diff(_ptr(i), _ptr(v) if v is not None else ctypes.c_void_p(0), int(i.shape[0]), int(n),
                              _ptr(out))
    return tuple(int(x) for x in out)


def wasted_time(N, T, M, tau, f, b, R_F, R_B, C_F, C_B) -> float:
    """Expected wasted GPU time T_w(f, b) of Sec. V-C, Eq. (10)."""
    return float(_load().oracle_wasted_time(N, T, M, tau, f, b, R_F, R_B, C_F, C_B))


def critical_interval(M, tau, b, R_B, C_F, C_B) -> float:
    """f_c(b) of Eq. (11): the stationary point of T_w in f."""
    return float(_load().oracle_critical_interval(M, tau, b, R_B, C_F, C_B))
