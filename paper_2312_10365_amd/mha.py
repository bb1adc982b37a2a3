"""ctypes binding of the sparse multi-head attention entry points of libspt (include/spt_mha.h):
argument marshalling only.  Tensors live on the GPU; nothing is computed here or by torch."""
from __future__ import annotations

import ctypes
from typing import Optional

import torch

from . import spt

EXPORTS = ("spt_mha_pq_assign", "spt_mha_topl", "spt_mha_attn_fwd", "spt_mha_attn_bwd",
           "spt_mha_workspace_bytes")


class MhaShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("S", "H", "n", "dh", "M", "E", "L")] + [("scale", ctypes.c_float)]


_ready = False


def lib() -> ctypes.CDLL:
    global _ready
    L = spt.lib()
    if not _ready:
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        shp = ctypes.POINTER(MhaShape)
        L.spt_mha_workspace_bytes.restype = sz
        L.spt_mha_workspace_bytes.argtypes = [shp]
        L.spt_mha_pq_assign.restype = i32
        L.spt_mha_pq_assign.argtypes = [shp, vp, vp, vp, vp, vp]
        L.spt_mha_topl.restype = i32
        L.spt_mha_topl.argtypes = [shp, vp, vp, vp, vp]
        L.spt_mha_attn_fwd.restype = i32
        L.spt_mha_attn_fwd.argtypes = [shp] + [vp] * 7
        L.spt_mha_attn_bwd.restype = i32
        L.spt_mha_attn_bwd.argtypes = [shp] + [vp] * 10 + [sz, vp]
        _ready = True
    return L


def make_shape(S, H, n, dh, L, E=16, M=None, scale=1.0) -> MhaShape:
    return MhaShape(S, H, n, dh, dh // 8 if M is None else M, E, L, scale)


def workspace_bytes(shape: MhaShape) -> int:
    return int(lib().spt_mha_workspace_bytes(ctypes.byref(shape)))


def alloc_workspace(shape: MhaShape, device="cuda") -> torch.Tensor:
    n = workspace_bytes(shape)
    if n == 0:
        raise spt.SptError(-2, "spt_mha_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


_ptr, _check, _stream = spt._ptr, spt._check, spt._stream


def pq_assign(shape: MhaShape, X, C, codes: Optional[torch.Tensor] = None,
              err: Optional[torch.Tensor] = None) -> torch.Tensor:
    s = shape
    rows = s.S * s.n
    if codes is None:
        codes = torch.empty((s.S, s.n, s.M), dtype=torch.uint8, device=X.device)
    rc = lib().spt_mha_pq_assign(ctypes.byref(s), _ptr(X, torch.bfloat16, rows * s.dh, "X"),
                                 _ptr(C, torch.float32, s.H * s.M * s.E * (s.dh // max(s.M, 1)), "C"),
                                 _ptr(codes, torch.uint8, rows * s.M, "codes"),
                                 _ptr(err, torch.float32, rows * s.M, "err"), _stream())
    _check(rc, "spt_mha_pq_assign")
    return codes


def topl(shape: MhaShape, cq, ck, idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    s = shape
    rows = s.S * s.n
    if idx is None:
        idx = torch.empty((s.S, s.n, s.L), dtype=torch.int32, device=cq.device)
    rc = lib().spt_mha_topl(ctypes.byref(s), _ptr(cq, torch.uint8, rows * s.M, "cq"),
                            _ptr(ck, torch.uint8, rows * s.M, "ck"),
                            _ptr(idx, torch.int32, rows * s.L, "idx"), _stream())
    _check(rc, "spt_mha_topl")
    return idx


def attn_fwd(shape: MhaShape, Q, K, V, idx, A=None, Y=None):
    s = shape
    rows = s.S * s.n
    if A is None:
        A = torch.empty((s.S, s.n, s.L), dtype=torch.float32, device=Q.device)
    if Y is None:
        Y = torch.empty((s.S, s.n, s.dh), dtype=torch.bfloat16, device=Q.device)
    bf = torch.bfloat16
    rc = lib().spt_mha_attn_fwd(ctypes.byref(s), _ptr(Q, bf, rows * s.dh, "Q"), _ptr(K, bf, rows * s.dh, "K"),
                                _ptr(V, bf, rows * s.dh, "V"), _ptr(idx, torch.int32, rows * s.L, "idx"),
                                _ptr(A, torch.float32, rows * s.L, "A"), _ptr(Y, bf, rows * s.dh, "Y"), _stream())
    _check(rc, "spt_mha_attn_fwd")
    return A, Y


def attn_bwd(shape: MhaShape, Q, K, V, dY, idx, A, ws=None, dQ=None, dK=None, dV=None):
    s = shape
    rows = s.S * s.n
    bf = torch.bfloat16
    if ws is None:
        ws = alloc_workspace(s, Q.device)
    outs = []
    for t in (dQ, dK, dV):
        outs.append(torch.empty((s.S, s.n, s.dh), dtype=bf, device=Q.device) if t is None else t)
    dQ, dK, dV = outs
    rc = lib().spt_mha_attn_bwd(ctypes.byref(s), _ptr(Q, bf, rows * s.dh, "Q"), _ptr(K, bf, rows * s.dh, "K"),
                                _ptr(V, bf, rows * s.dh, "V"), _ptr(dY, bf, rows * s.dh, "dY"),
                                _ptr(idx, torch.int32, rows * s.L, "idx"), _ptr(A, torch.float32, rows * s.L, "A"),
                                _ptr(dQ, bf, rows * s.dh, "dQ"), _ptr(dK, bf, rows * s.dh, "dK"),
                                _ptr(dV, bf, rows * s.dh, "dV"), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "spt_mha_attn_bwd")
    return dQ, dK, dV
