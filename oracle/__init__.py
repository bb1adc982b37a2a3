"""fp64 CPU oracle for the routed FFN -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy wrapper over `spt_oracle.c` (plain C, double precision, one
token and one hidden unit at a time).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the product path never
does, and this package imports nothing from the product.

All tensor arguments are numpy arrays: bf16/fp32 inputs are given as float32
(exact widenings), results come back as float64 / int32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spt_oracle.c")
_LIB = os.path.join(_HERE, "libspt_oracle.so")
_lib = None

ACT_GELU = 0
ACT_RELU = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (baseline x86-64-v3 ISA so the library also
    runs on a host other than the one that built it)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.spt_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().spt_oracle_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def act(z: np.ndarray, kind: int = ACT_GELU) -> Tuple[np.ndarray, np.ndarray]:
    """Activation and its derivative, elementwise, in fp64."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    out = np.empty_like(z)
    grad = np.empty_like(z)
    _load().spt_oracle_act(_p(z), ctypes.c_int64(z.size), ctypes.c_int(kind), _p(out), _p(grad))
    return out, grad


def router_logits(X, W_r, b_r=None) -> np.ndarray:
    """L[T,N] = X @ W_r (+ b_r) in fp64."""
    X = _f32(X); W_r = _f32(W_r)
    T, d = X.shape
    N = W_r.shape[1]
    assert W_r.shape[0] == d
    b = None if b_r is None else _f32(b_r)
    L = np.empty((T, N), dtype=np.float64)
    _load().spt_oracle_router_logits(_p(X), _p(W_r), _p(b), T, d, N, _p(L))
    return L


def topk(L: np.ndarray, k: int, flags: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """idx[T,k] (ascending block ids of the k largest fp32 keys, ties to the lower
    index) and margin[T] (k-th minus (k+1)-th largest fp64 key)."""
    L = np.ascontiguousarray(L, dtype=np.float64)
    T, N = L.shape
    assert 1 <= k <= N
    idx = np.empty((T, k), dtype=np.int32)
    margin = np.empty(T, dtype=np.float64)
    _load().spt_oracle_topk(_p(L), T, N, k, flags, _p(idx), _p(margin))
    return idx, margin


def route(X, W_r, b_r, k: int, flags: int = 0):
    L = router_logits(X, W_r, b_r)
    idx, margin = topk(L, k, flags)
    return idx, margin, L


def bucket(idx: np.ndarray, N: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """offsets[N+1], perm[T*k], inv[T*k] of the stable sort of pairs by block id."""
    idx = _i32(idx)
    T, k = idx.shape
    offsets = np.empty(N + 1, dtype=np.int32)
    perm = np.empty(T * k, dtype=np.int32)
    inv = np.empty(T * k, dtype=np.int32)
    _load().spt_oracle_bucket(_p(idx), T, N, k, _p(offsets), _p(perm), _p(inv))
    return offsets, perm, inv


def _tok(tokens, T):
    if tokens is None:
        return None, T
    tok = _i32(tokens)
    return tok, int(tok.size)


def ffn_fwd(X, W1, W2, idx, act_kind: int = ACT_GELU, tokens: Optional[Sequence[int]] = None):
    """Y[nt,d] and Hpre[nt,k,Bs] for the listed tokens (all tokens if None)."""
    X = _f32(X); W1 = _f32(W1); W2 = _f32(W2); idx = _i32(idx)
    T, d = X.shape
    N, Bs, d2 = W1.shape
    assert d2 == d and W2.shape == W1.shape
    k = idx.shape[1]
    tok, nt = _tok(tokens, T)
    Y = np.empty((nt, d), dtype=np.float64)
    Hpre = np.empty((nt, k, Bs), dtype=np.float64)
    _load().spt_oracle_ffn_fwd(_p(X), _p(W1), _p(W2), _p(idx), T, d, N, Bs, k, act_kind,
                               _p(tok), nt, _p(Y), _p(Hpre))
    return Y, Hpre


def ffn_bwd_dx(X, W1, W2, dY, idx, act_kind: int = ACT_GELU, tokens=None):
    """dX[nt,d] and dHpre[nt,k,Bs] for the listed tokens."""
    X = _f32(X); W1 = _f32(W1); W2 = _f32(W2); dY = _f32(dY); idx = _i32(idx)
    T, d = X.shape
    N, Bs, _ = W1.shape
    k = idx.shape[1]
    tok, nt = _tok(tokens, T)
    dX = np.empty((nt, d), dtype=np.float64)
    dHpre = np.empty((nt, k, Bs), dtype=np.float64)
    _load().spt_oracle_ffn_bwd_dx(_p(X), _p(W1), _p(W2), _p(dY), _p(idx), T, d, N, Bs, k,
                                  act_kind, _p(tok), nt, _p(dX), _p(dHpre))
    return dX, dHpre


def ffn_bwd_dw(X, W1, W2, dY, idx, act_kind: int = ACT_GELU, blocks=None):
    """dW1[nb,Bs,d], dW2[nb,Bs,d] for the listed blocks (all blocks if None)."""
    X = _f32(X); W1 = _f32(W1); W2 = _f32(W2); dY = _f32(dY); idx = _i32(idx)
    T, d = X.shape
    N, Bs, _ = W1.shape
    k = idx.shape[1]
    if blocks is None:
        blk, nb = None, N
    else:
        blk = _i32(blocks); nb = int(blk.size)
    dW1 = np.empty((nb, Bs, d), dtype=np.float64)
    dW2 = np.empty((nb, Bs, d), dtype=np.float64)
    _load().spt_oracle_ffn_bwd_dw(_p(X), _p(W1), _p(W2), _p(dY), _p(idx), T, d, N, Bs, k,
                                  act_kind, _p(blk), nb, _p(dW1), _p(dW2))
    return dW1, dW2


def to_bucket_order(per_pair: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """Reorder a [T,k,...] per-pair array into bucket (sorted) order [T*k,...]."""
    flat = per_pair.reshape((-1,) + per_pair.shape[2:])
    return flat[perm]


def lora_fwd(X, W1, W2, A1, C1, B2, C2, idx, act_kind: int = ACT_GELU, tokens=None):
    """Low-rank adapted routed FFN (section 2.2 on top of section 4.2): Y[nt,d], Hpre[nt,k,Bs].
    Adapters: A1[d,r], C1[r,N*Bs], B2[N*Bs,r], C2[r,d]."""
    X = _f32(X); W1 = _f32(W1); W2 = _f32(W2); idx = _i32(idx)
    A1 = _f32(A1); C1 = _f32(C1); B2 = _f32(B2); C2 = _f32(C2)
    T, d = X.shape
    N, Bs, _ = W1.shape
    k = idx.shape[1]
    r = A1.shape[1]
    assert A1.shape == (d, r) and C1.shape == (r, N * Bs) and B2.shape == (N * Bs, r) and C2.shape == (r, d)
    tok, nt = _tok(tokens, T)
    Y = np.empty((nt, d), dtype=np.float64)
    Hpre = np.empty((nt, k, Bs), dtype=np.float64)
    _load().spt_oracle_lora_fwd(_p(X), _p(W1), _p(W2), _p(A1), _p(C1), _p(B2), _p(C2), _p(idx),
                                T, d, N, Bs, k, r, act_kind, _p(tok), nt, _p(Y), _p(Hpre))
    return Y, Hpre


def lora_bwd(X, W1, W2, A1, C1, B2, C2, dY, idx, act_kind: int = ACT_GELU):
    """Gradients of lora_fwd with W1, W2 frozen and routing fixed, over all tokens:
    dX[T,d], dA1[d,r], dC1[r,N*Bs], dB2[N*Bs,r], dC2[r,d]."""
    X = _f32(X); W1 = _f32(W1); W2 = _f32(W2); dY = _f32(dY); idx = _i32(idx)
    A1 = _f32(A1); C1 = _f32(C1); B2 = _f32(B2); C2 = _f32(C2)
    T, d = X.shape
    N, Bs, _ = W1.shape
    k = idx.shape[1]
    r = A1.shape[1]
    D = N * Bs
    dX = np.empty((T, d), dtype=np.float64)
    dA1 = np.empty((d, r), dtype=np.float64)
    dC1 = np.empty((r, D), dtype=np.float64)
    dB2 = np.empty((D, r), dtype=np.float64)
    dC2 = np.empty((r, d), dtype=np.float64)
    _load().spt_oracle_lora_bwd(_p(X), _p(W1), _p(W2), _p(A1), _p(C1), _p(B2), _p(C2), _p(dY), _p(idx),
                                T, d, N, Bs, k, r, act_kind, _p(dX), _p(dA1), _p(dC1), _p(dB2), _p(dC2))
    return dX, dA1, dC1, dB2, dC2


def router_balance(X, W_r, b_r, idx, N: int):
    """Load-balancing loss of the route network and its gradient (section 4.2 names such a loss
    but prints no formula; this is the standard one for top-k routers, chosen for this build):
        f_b    = (number of (token, slot) pairs routed to block b) / (T k)      [treated as constant]
        p_t    = softmax over blocks of the token's logits x_t W_r + b_r
        pbar_b = mean_t p_t[b]
        loss   = N * sum_b f_b * pbar_b          (= 1 when the soft assignment is uniform)
    Gradient through pbar only:
        dlogit[t][c] = (N / T) * p_t[c] * (f_c - sum_b f_b p_t[b]),
        dW_r = X^T dlogit,  db_r = sum_t dlogit[t].
    Plain numpy in float64 on the exact fp64 logits; returns loss, f, dW_r, db_r, dlogit.
    Pins: tests/test_oracle_pins.py (torch autograd of the same loss, finite differences, the
    uniform closed form)."""
    X = np.asarray(X, dtype=np.float64)
    W_r = np.asarray(W_r, dtype=np.float64)
    T, _ = X.shape
    L = X @ W_r
    if b_r is not None:
        L = L + np.asarray(b_r, dtype=np.float64)[None, :]
    idx = _i32(idx)
    f = np.bincount(idx.ravel(), minlength=N).astype(np.float64) / float(idx.size)
    z = L - L.max(axis=1, keepdims=True)
    e = np.exp(z)
    p = e / e.sum(axis=1, keepdims=True)
    pbar = p.mean(axis=0)
    loss = float(N * np.dot(f, pbar))
    c = p @ f
    dlogit = (float(N) / T) * p * (f[None, :] - c[:, None])
    return loss, f, X.T @ dlogit, dlogit.sum(axis=0), dlogit
