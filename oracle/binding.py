"""ctypes binding of the fp64 CPU oracle (oracle/blr_oracle.cpp).

Test infrastructure: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this. It shares nothing with the GPU library.
All arrays are numpy float64, C-contiguous, host memory.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "blr_oracle.cpp")
_LIB = os.path.join(_HERE, "libblr_oracle.so")
_lib = None

OUT_INTERLEAVED, OUT_BLOCKED = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread",
                               _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # BLR_ORACLE_LIB: a library built from a deliberately altered copy of the source; only the test
        # that checks that the pins notice such alterations sets it (in a child process)
        override = os.environ.get("BLR_ORACLE_LIB")
        if not override:
            build()
        _lib = ctypes.CDLL(override or _LIB)
        for name in ("blr_oracle_dense_forward", "blr_oracle_monarch_forward", "blr_oracle_blast_forward",
                     "blr_oracle_materialize_monarch", "blr_oracle_materialize_blast",
                     "blr_oracle_monarch_middle_perm", "blr_oracle_lowrank_forward",
                     "blr_oracle_materialize_lowrank", "blr_oracle_monarch_rect_forward"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def default_threads() -> int:
    return len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)


def dense_forward(X, W, nthreads=None):
    X, W = _f64(X), _f64(W)
    T, n_in = X.shape
    n_out = W.shape[0]
    assert W.shape == (n_out, n_in)
    Y = np.empty((T, n_out), dtype=np.float64)
    rc = _load().blr_oracle_dense_forward(_p(X), _p(W), _p(Y), ctypes.c_int64(T), n_in, n_out,
                                          nthreads or default_threads())
    if rc:
        raise ValueError("oracle: invalid argument")
    return Y


def monarch_forward(X, R, L, out_order=OUT_INTERLEAVED, nthreads=None, return_macs=False):
    X, R, L = _f64(X), _f64(R), _f64(L)
    T, n_in = X.shape
    nblocks, r, p = R.shape
    q = L.shape[1]
    assert L.shape == (nblocks, q, r) and nblocks * p == n_in
    n_out = nblocks * q
    Y = np.empty((T, n_out), dtype=np.float64)
    macs = ctypes.c_int64(0)
    rc = _load().blr_oracle_monarch_forward(_p(X), _p(R), _p(L), _p(Y), ctypes.c_int64(T), n_in, n_out,
                                            nblocks, r, out_order, nthreads or default_threads(),
                                            ctypes.byref(macs))
    if rc:
        raise ValueError("oracle: invalid argument")
    return (Y, macs.value) if return_macs else Y


def monarch_rect_forward(X, R, L, b1, b2, out_order=OUT_INTERLEAVED, nthreads=None, return_macs=False):
    """Monarch with b1 input blocks and b2 output blocks: R[b1][r'*b2][n_in/b1], L[b2][n_out/b2][b1*r']."""
    X, R, L = _f64(X), _f64(R), _f64(L)
    T, n_in = X.shape
    p = R.shape[2]
    q = L.shape[1]
    rp = R.shape[1] // b2
    assert R.shape == (b1, rp * b2, p) and L.shape == (b2, q, b1 * rp) and b1 * p == n_in
    n_out = b2 * q
    Y = np.empty((T, n_out), dtype=np.float64)
    macs = ctypes.c_int64(0)
    rc = _load().blr_oracle_monarch_rect_forward(_p(X), _p(R), _p(L), _p(Y), ctypes.c_int64(T), n_in, n_out,
                                                 b1, b2, rp, out_order, nthreads or default_threads(), ctypes.byref(macs))
    if rc:
        raise ValueError("oracle: invalid argument")
    return (Y, macs.value) if return_macs else Y


def blast_forward(X, U, S, V, nthreads=None, return_macs=False):
    X, U, S, V = _f64(X), _f64(U), _f64(S), _f64(V)
    T, n_in = X.shape
    b, p, r = U.shape
    q = V.shape[1]
    assert V.shape == (b, q, r) and S.shape == (b, b, r) and b * q == n_in
    n_out = b * p
    Y = np.empty((T, n_out), dtype=np.float64)
    macs = ctypes.c_int64(0)
    rc = _load().blr_oracle_blast_forward(_p(X), _p(U), _p(S), _p(V), _p(Y), ctypes.c_int64(T), n_in, n_out,
                                          b, r, nthreads or default_threads(), ctypes.byref(macs))
    if rc:
        raise ValueError("oracle: invalid argument")
    return (Y, macs.value) if return_macs else Y


def lowrank_forward(X, V, U, nthreads=None, return_macs=False):
    """Y = (X V^T) U^T with V[r][n_in], U[n_out][r]."""
    X, V, U = _f64(X), _f64(V), _f64(U)
    T, n_in = X.shape
    r = V.shape[0]
    n_out = U.shape[0]
    assert V.shape == (r, n_in) and U.shape == (n_out, r)
    Y = np.empty((T, n_out), dtype=np.float64)
    macs = ctypes.c_int64(0)
    rc = _load().blr_oracle_lowrank_forward(_p(X), _p(V), _p(U), _p(Y), ctypes.c_int64(T), n_in, n_out, r,
                                            nthreads or default_threads(), ctypes.byref(macs))
    if rc:
        raise ValueError("oracle: invalid argument")
    return (Y, macs.value) if return_macs else Y


def materialize_lowrank(V, U):
    V, U = _f64(V), _f64(U)
    r, n_in = V.shape
    n_out = U.shape[0]
    W = np.empty((n_out, n_in), dtype=np.float64)
    rc = _load().blr_oracle_materialize_lowrank(_p(V), _p(U), _p(W), n_in, n_out, r)
    if rc:
        raise ValueError("oracle: invalid argument")
    return W


def materialize_monarch(R, L, out_order=OUT_INTERLEAVED):
    R, L = _f64(R), _f64(L)
    nblocks, r, p = R.shape
    q = L.shape[1]
    W = np.empty((nblocks * q, nblocks * p), dtype=np.float64)
    rc = _load().blr_oracle_materialize_monarch(_p(R), _p(L), _p(W), nblocks * p, nblocks * q, nblocks, r, out_order)
    if rc:
        raise ValueError("oracle: invalid argument")
    return W


def materialize_blast(U, S, V):
    U, S, V = _f64(U), _f64(S), _f64(V)
    b, p, r = U.shape
    q = V.shape[1]
    W = np.empty((b * p, b * q), dtype=np.float64)
    rc = _load().blr_oracle_materialize_blast(_p(U), _p(S), _p(V), _p(W), b * q, b * p, b, r)
    if rc:
        raise ValueError("oracle: invalid argument")
    return W


def monarch_middle_perm(nblocks, r):
    perm = np.empty(nblocks * r, dtype=np.int64)
    rc = _load().blr_oracle_monarch_middle_perm(nblocks, r, _p(perm))
    if rc:
        raise ValueError("oracle: invalid argument")
    return perm
