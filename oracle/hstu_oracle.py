"""ctypes binding of the CPU fp64 oracle (``hstu_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's cpu_baseline leg.  The product path never touches this module.
All arrays are float64, laid out [T, H, d]; see the C file for the definitions.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hstu_oracle.c")
_LIB = os.path.join(_HERE, "libhstu_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_count_pairs.restype = ctypes.c_int64
    return _lib


def num_threads() -> int:
    """Threads the OpenMP runtime will use for the oracle's parallel loops."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_get_max_threads.restype = ctypes.c_int
    return int(omp.omp_get_max_threads())


def _f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def _p(x):
    return None if x is None else x.ctypes.data_as(ctypes.c_void_p)


def _desc(offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, H, d):
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    nt = None if num_targets is None else np.ascontiguousarray(num_targets, dtype=np.int32)
    tb = None if table is None else _f64(table)
    bd = None if bounds is None else np.ascontiguousarray(bounds, dtype=np.int32)
    nb = 0 if bd is None else int(bd.shape[0])
    if tb is not None:
        assert tb.shape == (H, nb) and bd[0] == 0
    keep = (offsets, nt, tb, bd)
    args = (ctypes.c_int(offsets.shape[0] - 1), ctypes.c_int(H), ctypes.c_int(d), _p(offsets), _p(nt),
            ctypes.c_int(K1), ctypes.c_int(K2), ctypes.c_double(alpha), ctypes.c_double(inv_n),
            _p(tb), _p(bd), ctypes.c_int(nb))
    return args, keep


def attn_fwd(q, k, v, offsets, *, num_targets=None, K1=-1, K2=0, alpha=1.0, inv_n=1.0, table=None, bounds=None,
             rows=None):
    """A = ((SiLU(alpha QK^T + bias)/N) * M) V.  With ``rows`` (global token indices) only those rows."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    T, H, d = q.shape
    args, keep = _desc(offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, H, d)
    assert int(keep[0][-1]) == T
    lib = _load()
    if rows is None:
        out = np.empty_like(q)
        lib.oracle_attn_fwd(*args, _p(q), _p(k), _p(v), _p(out))
        return out
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    out = np.empty((rows.shape[0], H, d), dtype=np.float64)
    lib.oracle_attn_fwd_rows(*args, _p(q), _p(k), _p(v), ctypes.c_int(rows.shape[0]), _p(rows), _p(out))
    return out


def attn_bwd(q, k, v, dout, offsets, *, num_targets=None, K1=-1, K2=0, alpha=1.0, inv_n=1.0, table=None,
             bounds=None, rows=None):
    """dQ, dK, dV of ``attn_fwd`` for upstream gradient ``dout``.  With ``rows`` only those token rows."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    T, H, d = q.shape
    args, keep = _desc(offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, H, d)
    assert int(keep[0][-1]) == T
    lib = _load()
    if rows is None:
        dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
        lib.oracle_attn_bwd(*args, _p(q), _p(k), _p(v), _p(dout), _p(dq), _p(dk), _p(dv))
        return dq, dk, dv
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    shp = (rows.shape[0], H, d)
    dq, dk, dv = np.empty(shp), np.empty(shp), np.empty(shp)
    lib.oracle_attn_bwd_rows(*args, _p(q), _p(k), _p(v), _p(dout), ctypes.c_int(rows.shape[0]), _p(rows),
                             _p(dq), _p(dk), _p(dv))
    return dq, dk, dv


def attn_bwd_bias(q, k, v, dout, offsets, *, num_targets=None, K1=-1, K2=0, alpha=1.0, inv_n=1.0, table=None,
                  bounds=None):
    """Gradient of the relative-bias table [H, num_buckets] for upstream gradient ``dout`` of ``attn_fwd``."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    T, H, d = q.shape
    args, keep = _desc(offsets, num_targets, K1, K2, alpha, inv_n, table, bounds, H, d)
    assert int(keep[0][-1]) == T and table is not None
    dtable = np.empty((H, np.asarray(bounds).shape[0]), dtype=np.float64)
    _load().oracle_attn_bwd_bias(*args, _p(q), _p(k), _p(v), _p(dout), _p(dtable))
    return dtable


def mask(L, M=0, K1=-1, K2=0):
    """Dense visibility matrix (bool [L, L]) and bias distances (int32, -1 where masked) of one sequence."""
    m = np.zeros((L, L), dtype=np.uint8)
    dist = np.zeros((L, L), dtype=np.int32)
    _load().oracle_mask(ctypes.c_int(L), ctypes.c_int(M), ctypes.c_int(K1), ctypes.c_int(K2), _p(m), _p(dist))
    return m.astype(bool), dist


def count_pairs(lengths, num_targets=None, K1=-1, K2=0) -> int:
    """Visible (query, key) pairs per head, summed over the batch."""
    lib = _load()
    total = 0
    for b, L in enumerate(lengths):
        M = 0 if num_targets is None else int(num_targets[b])
        total += int(lib.oracle_count_pairs(ctypes.c_int(int(L)), ctypes.c_int(M), ctypes.c_int(K1), ctypes.c_int(K2)))
    return total


def gated_norm_fwd(a, u, gamma, beta=None, eps=1e-5):
    """Y = (LayerNorm(A) gamma + beta) * U over the flattened H*d features; returns Y, mean, rstd."""
    a, u = _f64(a), _f64(u)
    T = a.shape[0]
    D = int(np.prod(a.shape[1:]))
    gamma = _f64(gamma)
    beta = None if beta is None else _f64(beta)
    y = np.empty_like(a)
    mean, rstd = np.empty(T), np.empty(T)
    _load().oracle_gated_norm_fwd(ctypes.c_int64(T), ctypes.c_int(D), _p(a), _p(u), _p(gamma), _p(beta),
                                  ctypes.c_double(eps), _p(y), _p(mean), _p(rstd))
    return y, mean, rstd


def gated_norm_bwd(dy, a, u, gamma, beta=None, eps=1e-5):
    """dA, dU, dgamma, dbeta of ``gated_norm_fwd``."""
    dy, a, u = _f64(dy), _f64(a), _f64(u)
    T = a.shape[0]
    D = int(np.prod(a.shape[1:]))
    gamma = _f64(gamma)
    beta_ = None if beta is None else _f64(beta)
    da, du = np.empty_like(a), np.empty_like(a)
    dgamma, dbeta = np.empty(D), np.empty(D)
    _load().oracle_gated_norm_bwd(ctypes.c_int64(T), ctypes.c_int(D), _p(dy), _p(a), _p(u), _p(gamma), _p(beta_),
                                  ctypes.c_double(eps), _p(da), _p(du), _p(dgamma), _p(dbeta))
    return da, du, dgamma, dbeta
