"""ctypes front end of the CPU oracle (``rcd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library never calls
it and it never calls the GPU library.

Every function here only marshals numpy arrays into the C routines; the
arithmetic lives in ``rcd_oracle.c`` where each routine cites the passage of
the paper (arXiv 2211.00839) it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rcd_oracle.c")
_LIB = os.path.join(_HERE, "librcd_oracle.so")

F32 = 0
BF16 = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no OpenMP, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fno-fast-math", "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    c = ctypes
    vp, i64, i32, dbl = c.c_void_p, c.c_int64, c.c_int, c.c_double
    lib.oracle_similarity.restype = i32
    lib.oracle_similarity.argtypes = [vp, i32, i64, i64, i64, dbl, vp, vp]
    lib.oracle_quota.restype = i32
    lib.oracle_quota.argtypes = [i64, vp, i32, vp]
    lib.oracle_f.restype = dbl
    lib.oracle_f.argtypes = [vp, i64, i64, vp, i64]
    lib.oracle_gain_row.restype = i32
    lib.oracle_gain_row.argtypes = [vp, i64, i64, vp, vp, vp]
    lib.oracle_partition_class.restype = i64
    lib.oracle_partition_class.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.oracle_lockstep.restype = i32
    lib.oracle_lockstep.argtypes = [vp, i64, i64, i32, vp, vp, vp, i64, vp, dbl, vp, vp]
    lib.oracle_bruteforce.restype = i64
    lib.oracle_bruteforce.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.oracle_f_gc.restype = dbl
    lib.oracle_f_gc.argtypes = [vp, i64, i64, vp, i64]
    lib.oracle_partition_class_gc.restype = i64
    lib.oracle_partition_class_gc.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.oracle_worker_shards.restype = i32
    lib.oracle_worker_shards.argtypes = [vp, i64, i32, vp, vp]
    lib.oracle_batch_sizes.restype = i32
    lib.oracle_batch_sizes.argtypes = [i64, vp, i32, vp]
    lib.oracle_bandwidth.restype = dbl
    lib.oracle_bandwidth.argtypes = [vp, i32, i64, i64, i64]
    lib.oracle_lockstep_gc.restype = i32
    lib.oracle_lockstep_gc.argtypes = [vp, i64, i64, i32, vp, vp, vp, i64, vp, dbl, dbl, vp, vp]
    lib.oracle_partition_dataset.restype = i32
    lib.oracle_partition_dataset.argtypes = [vp, i32, i64, i64, i64, vp, i32, vp, i32, dbl, vp, vp, vp]
    _lib = lib
    return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _features(X):
    """float32 array -> (array, F32); uint16 array holding bf16 bit patterns -> (array, BF16)."""
    X = np.ascontiguousarray(X)
    if X.dtype == np.float32:
        return X, F32
    if X.dtype == np.uint16:
        return X, BF16
    raise TypeError("features must be float32, or uint16 holding bf16 bit patterns")


def _sim_matrix(S):
    S = np.ascontiguousarray(S, dtype=np.float32)
    if S.ndim != 2 or S.shape[0] > S.shape[1]:
        raise ValueError("S must be n x ld with ld >= n")
    return S


def similarity(X, sigma2: float, want64: bool = False):
    """Gaussian-kernel similarity of the rows of X.  Returns float32 (n,n), or
    (float32, float64) if want64."""
    X, dt = _features(X)
    n, d = X.shape
    S32 = np.empty((n, n), dtype=np.float32)
    S64 = np.empty((n, n), dtype=np.float64) if want64 else None
    rc = _load().oracle_similarity(_ptr(X), dt, n, d, d, float(sigma2), _ptr(S64), _ptr(S32))
    if rc != 0:
        raise ValueError("oracle_similarity rejected its arguments")
    return (S32, S64) if want64 else S32


def worker_shards(assign, K: int):
    """Per-worker ascending index lists of an assignment (-1 = in no list).  Returns (index[:total], offset[K+1])."""
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    N = len(assign)
    index = np.full(max(N, 1), -1, dtype=np.int32)
    offset = np.zeros(K + 1, dtype=np.int64)
    if _load().oracle_worker_shards(_ptr(assign), N, int(K), _ptr(index), _ptr(offset)) != 0:
        raise ValueError("oracle_worker_shards rejected its arguments")
    return index[: offset[K]], offset


def batch_sizes(B: int, r) -> np.ndarray:
    """Batch size per worker: B r_i / r_1 to the nearest integer, at least 1."""
    r = np.ascontiguousarray(r, dtype=np.int64)
    out = np.zeros(len(r), dtype=np.int64)
    if _load().oracle_batch_sizes(int(B), _ptr(r), len(r), _ptr(out)) != 0:
        raise ValueError("oracle_batch_sizes rejected its arguments")
    return out


def bandwidth(X) -> float:
    """The paper's kernel bandwidth: mean L2 distance over all n^2 ordered pairs of rows of X."""
    X, dt = _features(X)
    n, d = X.shape
    sigma = _load().oracle_bandwidth(_ptr(X), dt, n, d, d)
    if sigma < 0:
        raise ValueError("oracle_bandwidth rejected its arguments")
    return float(sigma)


def quota(n_l: int, r) -> np.ndarray:
    r = np.ascontiguousarray(r, dtype=np.int64)
    cap = np.empty(len(r), dtype=np.int64)
    if _load().oracle_quota(int(n_l), _ptr(r), len(r), _ptr(cap)) != 0:
        raise ValueError("oracle_quota rejected its arguments")
    return cap


def f_value(S, members, objective: str = "fl") -> float:
    """f(A) from the definition: facility location ("fl") or graph cut ("gc")."""
    S = _sim_matrix(S)
    mem = np.ascontiguousarray(members, dtype=np.int32)
    fn = _load().oracle_f if objective == "fl" else _load().oracle_f_gc
    return float(fn(_ptr(S), S.shape[1], S.shape[0], _ptr(mem), len(mem)))


def gain_row(S, cov, assign=None) -> np.ndarray:
    S = _sim_matrix(S)
    n = S.shape[0]
    cov = np.ascontiguousarray(cov, dtype=np.float64)
    assert cov.shape == (n,)
    a = None if assign is None else np.ascontiguousarray(assign, dtype=np.int32)
    g = np.empty(n, dtype=np.float64)
    if _load().oracle_gain_row(_ptr(S), S.shape[1], n, _ptr(cov), _ptr(a), _ptr(g)) != 0:
        raise ValueError("oracle_gain_row rejected its arguments")
    return g


def partition_class(S, cap, trace: bool = False, objective: str = "fl"):
    """Algorithm 1 on one class with the facility-location ("fl") or graph-cut ("gc") function.
    Returns dict(assign, order, obj, fsum, steps[, tr_block, tr_elem, tr_gain])."""
    S = _sim_matrix(S)
    n = S.shape[0]
    cap = np.ascontiguousarray(cap, dtype=np.int64)
    K = len(cap)
    assign = np.empty(n, dtype=np.int32)
    order = np.empty(n, dtype=np.int32)
    obj = np.empty(K, dtype=np.float64)
    fsum = np.empty(K, dtype=np.float64)
    tb = te = tg = None
    if trace:
        tb = np.full(max(n, 1), -1, dtype=np.int32)
        te = np.full(max(n, 1), -1, dtype=np.int32)
        tg = np.zeros(max(n, 1), dtype=np.float64)
    fn = _load().oracle_partition_class if objective == "fl" else _load().oracle_partition_class_gc
    steps = fn(_ptr(S), S.shape[1], n, K, _ptr(cap), _ptr(assign), _ptr(order), _ptr(obj), _ptr(fsum),
               _ptr(tb), _ptr(te), _ptr(tg))
    if steps < 0:
        raise ValueError("oracle_partition_class rejected its arguments")
    out = dict(assign=assign, order=order, obj=obj, fsum=fsum, steps=int(steps))
    if trace:
        out.update(tr_block=tb[:steps], tr_elem=te[:steps], tr_gain=tg[:steps])
    return out


def lockstep(S, cap, order, assign, rel_tol: float = 1e-5, check=None, objective: str = "fl", abs_tol: float = 0.0):
    """Referee a foreign trace against Algorithm 1 (see oracle_lockstep in the C
    file; abs_tol is the graph-cut referee's absolute element window).  Returns dict(rc, checked, exact, near_block, near_elem, violations,
    first_violation, worst_elem_gap, worst_block_gap)."""
    S = _sim_matrix(S)
    n = S.shape[0]
    cap = np.ascontiguousarray(cap, dtype=np.int64)
    order = np.ascontiguousarray(order, dtype=np.int32)
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    steps = int((order >= 0).sum())
    chk = None
    if check is not None:
        chk = np.zeros(max(steps, 1), dtype=np.uint8)
        idx = np.asarray(check, dtype=np.int64)
        chk[idx[idx < steps]] = 1
    stats = np.zeros(6, dtype=np.int64)
    worst = np.zeros(2, dtype=np.float64)
    fn = _load().oracle_lockstep if objective == "fl" else _load().oracle_lockstep_gc
    tol = (float(rel_tol),) if objective == "fl" else (float(rel_tol), float(abs_tol))
    rc = fn(_ptr(S), S.shape[1], n, len(cap), _ptr(cap), _ptr(order), _ptr(assign), steps, _ptr(chk),
            *tol, _ptr(stats), _ptr(worst))
    return dict(rc=int(rc), checked=int(stats[0]), exact=int(stats[1]), near_block=int(stats[2]),
                near_elem=int(stats[3]), violations=int(stats[4]), first_violation=int(stats[5]),
                worst_elem_gap=float(worst[0]), worst_block_gap=float(worst[1]), steps=steps)


def bruteforce(S, cap):
    """Exhaustive optimum for tiny n.  Returns (max sum_k f_k, max min_k f_k, visited)."""
    S = _sim_matrix(S)
    cap = np.ascontiguousarray(cap, dtype=np.int64)
    best = np.zeros(2, dtype=np.float64)
    visited = _load().oracle_bruteforce(_ptr(S), S.shape[1], S.shape[0], len(cap), _ptr(cap), _ptr(best))
    if visited < 0:
        raise ValueError("oracle_bruteforce rejected its arguments")
    return float(best[0]), float(best[1]), int(visited)


def partition_dataset(X, labels, L: int, r, sigma2: float):
    """Algorithm 1 on a labelled data set.  Returns dict(assign, order, obj[L,K])."""
    X, dt = _features(X)
    N, d = X.shape
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    r = np.ascontiguousarray(r, dtype=np.int64)
    K = len(r)
    assign = np.full(N, -1, dtype=np.int32)
    order = np.full(N, -1, dtype=np.int32)
    obj = np.zeros((L, K), dtype=np.float64)
    rc = _load().oracle_partition_dataset(_ptr(X), dt, N, d, d, _ptr(labels), L, _ptr(r), K,
                                          float(sigma2), _ptr(assign), _ptr(order), _ptr(obj))
    if rc != 0:
        raise ValueError("oracle_partition_dataset rejected its arguments")
    return dict(assign=assign, order=order, obj=obj)
