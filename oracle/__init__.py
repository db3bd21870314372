"""CPU oracle for exact kNN -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The GPU library never does, and the two
share no code: this binding loads ``libknn_oracle.so`` (plain C, fp64, built
from ``knn_oracle.c`` by :func:`build`) and nothing else.

What the oracle computes is the problem statement of the paper's Sect. 3
written out (all distances of a row, full sort by (distance, index), first k);
see the header of ``knn_oracle.c`` for the readings of the paper it fixes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "knn_oracle.c")
_LIB = os.path.join(_HERE, "libknn_oracle.so")

METRICS = {"sqeuclidean": 0, "cosine": 1, "hellinger": 2, "l1": 3, "linf": 4, "kl": 5}

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (IEEE semantics kept: no fast-math)."""
    if force or not os.path.exists(_LIB):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-fno-fast-math", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build(force=True)
        lib = ctypes.CDLL(_LIB)
        lib.knn_oracle_search.restype = ctypes.c_int32
        lib.knn_oracle_search.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.knn_oracle_delta.restype = ctypes.c_double
        lib.knn_oracle_delta.argtypes = [ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_int32, ctypes.c_int32]
        lib.knn_oracle_pair_dists.restype = ctypes.c_int32
        lib.knn_oracle_pair_dists.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
            ctypes.c_void_p]
        lib.knn_oracle_select.restype = ctypes.c_int32
        lib.knn_oracle_select.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p,
                                          ctypes.c_void_p]
        lib.knn_oracle_threads.restype = ctypes.c_int32
        lib.knn_oracle_threads.argtypes = []
        _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads the oracle's row loop uses."""
    return int(_load().knn_oracle_threads())


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float32)
    if a.ndim != 2:
        raise ValueError("expected a 2-D array")
    return a


def search(Q, R, k: int, metric: str = "sqeuclidean", self_idx=None):
    """k nearest references of every query row (Sect. 3 of the paper).

    Q[nq, d], R[nr, d]: fp32 host arrays.  ``self_idx[i]`` is the reference
    index that is query i itself (skipped), or -1; ``None`` skips nothing.
    Returns ``(idx int32 [nq,k], dist float64 [nq,k], next_dist float64 [nq])``
    where ``next_dist`` is the (k+1)-th distance of the sorted row (+inf if
    there is none).
    """
    lib = _load()
    Q = _f32(Q)
    R = _f32(R)
    nq, d = Q.shape
    nr, d2 = R.shape
    if d != d2:
        raise ValueError("Q and R differ in dimension")
    if self_idx is not None:
        self_arr = np.ascontiguousarray(np.asarray(self_idx), dtype=np.int64)
        if self_arr.shape != (nq,):
            raise ValueError("self_idx must have one entry per query")
        self_ptr = self_arr.ctypes.data
    else:
        self_arr = None
        self_ptr = None
    idx = np.empty((nq, k), dtype=np.int32)
    dist = np.empty((nq, k), dtype=np.float64)
    nxt = np.empty((nq,), dtype=np.float64)
    rc = lib.knn_oracle_search(Q.ctypes.data, nq, R.ctypes.data, nr, d, k,
                               METRICS[metric], self_ptr,
                               idx.ctypes.data, dist.ctypes.data, nxt.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"knn_oracle_search failed with code {rc}")
    return idx, dist, nxt


def build_knn(X, k: int, metric: str = "sqeuclidean"):
    """All-pairs self kNN of the rows of X, each row excluding itself."""
    X = _f32(X)
    return search(X, X, k, metric, self_idx=np.arange(X.shape[0], dtype=np.int64))


def delta(u, v, metric: str = "sqeuclidean") -> float:
    """One distance, in double, from fp32 inputs."""
    lib = _load()
    u = np.ascontiguousarray(np.asarray(u), dtype=np.float32).ravel()
    v = np.ascontiguousarray(np.asarray(v), dtype=np.float32).ravel()
    if u.shape != v.shape:
        raise ValueError("vectors differ in length")
    return float(lib.knn_oracle_delta(u.ctypes.data, v.ctypes.data,
                                      u.shape[0], METRICS[metric]))


def pair_dists(Q, R, idx, metric: str = "sqeuclidean") -> np.ndarray:
    """out[i, r] = delta(Q[i], R[idx[i, r]]) in double; NaN for a bad index."""
    lib = _load()
    Q = _f32(Q)
    R = _f32(R)
    idx = np.ascontiguousarray(np.asarray(idx), dtype=np.int32)
    nq, d = Q.shape
    if idx.ndim != 2 or idx.shape[0] != nq:
        raise ValueError("idx must be [nq, k]")
    out = np.empty(idx.shape, dtype=np.float64)
    rc = lib.knn_oracle_pair_dists(Q.ctypes.data, nq, R.ctypes.data, R.shape[0], d,
                                   idx.shape[1], METRICS[metric],
                                   idx.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"knn_oracle_pair_dists failed with code {rc}")
    return out


def select(A, k: int):
    """k smallest entries of every row of A (Sect. 6 of the paper), ascending, ties to the
    lower column.  Returns (idx int32 [m,k], val float32 [m,k])."""
    lib = _load()
    A = _f32(A)
    m, n = A.shape
    idx = np.empty((m, k), dtype=np.int32)
    val = np.empty((m, k), dtype=np.float32)
    rc = lib.knn_oracle_select(A.ctypes.data, m, n, n, k, idx.ctypes.data, val.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"knn_oracle_select failed with code {rc}")
    return idx, val
