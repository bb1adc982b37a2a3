"""fp64 CPU oracle of SPT's sparse multi-head attention (ctypes wrapper of mha_oracle.c).

TEST INFRASTRUCTURE ONLY: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg
may import this.  Follows section 4.1 (Eq. 6, Algorithm 1) and section 5.1 (Algorithms 2, 3) of
the paper; the readings taken where the text is silent are listed at the top of mha_oracle.c.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mha_oracle.c")
_LIB = os.path.join(_HERE, "libmha_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"],
                       check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def pq_assign(X, C, with_error: bool = False):
    """X[S,n,dh], C[H,M,E,dp] -> codes[S,n,M] uint8, margin[S,n,M] (second best - best squared
    distance) and, with_error, err[S,n,M] (Euclidean distance to the chosen codeword)."""
    X = _f32(X); C = _f32(C)
    S, n, dh = X.shape
    H, M, E, dp = C.shape
    assert M * dp == dh and S % H == 0 and E <= 256
    codes = np.empty((S, n, M), dtype=np.uint8)
    margin = np.empty((S, n, M), dtype=np.float64)
    err = np.empty((S, n, M), dtype=np.float64) if with_error else None
    _load().mha_oracle_pq_assign(_p(X), _p(C), S, H, n, dh, M, E, _p(codes), _p(margin), _p(err))
    return (codes, margin, err) if with_error else (codes, margin)


def topl(cq, ck, L: int):
    """Algorithm 3: idx[S,n,L] int32 (-1 = no key) from the codes of queries and keys."""
    cq = np.ascontiguousarray(cq, dtype=np.uint8); ck = np.ascontiguousarray(ck, dtype=np.uint8)
    S, n, M = cq.shape
    idx = np.empty((S, n, L), dtype=np.int32)
    _load().mha_oracle_topl(_p(cq), _p(ck), S, n, M, L, _p(idx))
    return idx


def attn_fwd(Q, K, V, idx, scale: float):
    Q = _f32(Q); K = _f32(K); V = _f32(V)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    S, n, dh = Q.shape
    L = idx.shape[2]
    A = np.empty((S, n, L), dtype=np.float64)
    Y = np.empty((S, n, dh), dtype=np.float64)
    _load().mha_oracle_attn_fwd(_p(Q), _p(K), _p(V), _p(idx), S, n, dh, L, ctypes.c_double(scale), _p(A), _p(Y))
    return A, Y


def attn_bwd(Q, K, V, dY, idx, A, scale: float):
    Q = _f32(Q); K = _f32(K); V = _f32(V); dY = _f32(dY)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    A = np.ascontiguousarray(A, dtype=np.float64)
    S, n, dh = Q.shape
    L = idx.shape[2]
    dQ = np.empty((S, n, dh), dtype=np.float64)
    dK = np.empty((S, n, dh), dtype=np.float64)
    dV = np.empty((S, n, dh), dtype=np.float64)
    _load().mha_oracle_attn_bwd(_p(Q), _p(K), _p(V), _p(dY), _p(idx), _p(A), S, n, dh, L,
                                ctypes.c_double(scale), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV
