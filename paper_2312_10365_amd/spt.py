"""ctypes binding of libspt (see include/spt.h): argument marshalling only.

Every function here takes torch tensors that live on the GPU, checks dtype /
shape / contiguity, and passes raw device pointers plus the current HIP stream
to the C ABI.  No step of the routed FFN is computed in Python or by torch.
The library must have been built (``__graft_entry__.build()``); loading fails
loudly otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspt.so")

ACT_GELU, ACT_RELU = 0, 1
FLAG_ABS_LOGIT = 1
WS_BUCKET, WS_FWD, WS_BWD, WS_ROUTER, WS_LORA_FWD, WS_LORA_BWD, WS_BALANCE, WS_SCHEDULE = 0, 1, 2, 3, 4, 5, 6, 7

EXPORTS = ("spt_workspace_bytes", "spt_router_topk", "spt_bucket_tokens", "spt_bucket_tokens_noalloc",
           "spt_routed_ffn_fwd", "spt_routed_ffn_bwd", "spt_build_schedule", "spt_routed_ffn_fwd_sched",
           "spt_routed_ffn_bwd_sched", "spt_lora_ffn_fwd", "spt_lora_ffn_bwd",
           "spt_router_balance", "spt_strerror",
           "spt_profile_enable", "spt_profile_slots", "spt_profile_slot_name", "spt_profile_read",
           "spt_calibrate_mfma", "spt_calibrate_stream")


class SptShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "N", "Bs", "k", "act", "flags")]


class SptError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(hipcc --offload-arch=gfx950); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        shp = ctypes.POINTER(SptShape)
        L.spt_workspace_bytes.restype = sz
        L.spt_workspace_bytes.argtypes = [shp, i32]
        L.spt_router_topk.restype = i32
        L.spt_router_topk.argtypes = [shp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.spt_bucket_tokens.restype = i32
        L.spt_bucket_tokens.argtypes = [shp, vp, vp, vp, vp, vp, sz, vp]
        L.spt_bucket_tokens_noalloc.restype = i32
        L.spt_bucket_tokens_noalloc.argtypes = [shp, vp, vp, vp, vp, vp]
        L.spt_routed_ffn_fwd.restype = i32
        L.spt_routed_ffn_fwd.argtypes = [shp] + [vp] * 9 + [sz, vp]
        L.spt_routed_ffn_bwd.restype = i32
        L.spt_routed_ffn_bwd.argtypes = [shp] + [vp] * 12 + [sz, vp]
        L.spt_build_schedule.restype = i32
        L.spt_build_schedule.argtypes = [shp, vp, vp, vp, sz, vp]
        L.spt_routed_ffn_fwd_sched.restype = i32
        L.spt_routed_ffn_fwd_sched.argtypes = [shp] + [vp] * 9 + [sz, vp, sz, vp]
        L.spt_routed_ffn_bwd_sched.restype = i32
        L.spt_routed_ffn_bwd_sched.argtypes = [shp] + [vp] * 12 + [sz, vp, sz, vp]
        L.spt_lora_ffn_fwd.restype = i32
        L.spt_lora_ffn_fwd.argtypes = [shp, i32] + [vp] * 13 + [sz, vp]
        L.spt_lora_ffn_bwd.restype = i32
        L.spt_lora_ffn_bwd.argtypes = [shp, i32] + [vp] * 18 + [sz, vp]
        L.spt_router_balance.restype = i32
        L.spt_router_balance.argtypes = [shp] + [vp] * 8 + [sz, vp]
        L.spt_strerror.restype = ctypes.c_char_p
        L.spt_strerror.argtypes = [i32]
        L.spt_profile_enable.restype = i32
        L.spt_profile_enable.argtypes = [i32]
        L.spt_profile_slots.restype = i32
        L.spt_profile_slot_name.restype = ctypes.c_char_p
        L.spt_profile_slot_name.argtypes = [i32]
        L.spt_profile_read.restype = i32
        L.spt_profile_read.argtypes = [vp, vp]
        L.spt_calibrate_mfma.restype = i32
        L.spt_calibrate_mfma.argtypes = [i32, i32, i32, vp, vp]
        L.spt_calibrate_stream.restype = i32
        L.spt_calibrate_stream.argtypes = [vp, vp, sz, i32, vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().spt_strerror(code).decode()


def make_shape(T, d, N, Bs, k, act=ACT_GELU, flags=0) -> SptShape:
    return SptShape(T, d, N, Bs, k, act, flags)


def workspace_bytes(shape: SptShape, which: int) -> int:
    return int(lib().spt_workspace_bytes(ctypes.byref(shape), which))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor], dtype, numel: int, name: str):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or t.numel() != numel:
        raise ValueError(f"{name}: need a contiguous cuda tensor of {dtype} with {numel} elements, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")
    return t.data_ptr()


def alloc_workspace(shape: SptShape, which: int, device="cuda") -> torch.Tensor:
    n = workspace_bytes(shape, which)
    if n == 0:
        raise SptError(-2, "spt_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _check(rc: int, where: str):
    if rc != 0:
        raise SptError(rc, where)


def router_topk(shape: SptShape, X, W_r, b_r=None, idx=None, logits=None, ws=None):
    """idx[T,k] int32 (and optionally the fp32 logits) for bf16 X[T,d], fp32 W_r[d,N]."""
    s = shape
    if idx is None:
        idx = torch.empty((s.T, s.k), dtype=torch.int32, device=X.device)
    if ws is None and logits is None:
        ws = alloc_workspace(s, WS_ROUTER, X.device)
    rc = lib().spt_router_topk(ctypes.byref(s), _ptr(X, torch.bfloat16, s.T * s.d, "X"),
                               _ptr(W_r, torch.float32, s.d * s.N, "W_r"),
                               _ptr(b_r, torch.float32, s.N, "b_r"),
                               _ptr(idx, torch.int32, s.T * s.k, "idx"),
                               _ptr(logits, torch.float32, s.T * s.N, "logits"),
                               None if ws is None else ws.data_ptr(),
                               0 if ws is None else ws.numel(), _stream())
    _check(rc, "spt_router_topk")
    return idx


def bucket_tokens(shape: SptShape, idx, ws=None, offsets=None, perm=None, inv=None):
    """offsets[N+1], perm[P], inv[P] (int32) of the stable sort of pairs by block id."""
    s = shape
    P = s.T * s.k
    dev = idx.device
    offsets = torch.empty(s.N + 1, dtype=torch.int32, device=dev) if offsets is None else offsets
    perm = torch.empty(P, dtype=torch.int32, device=dev) if perm is None else perm
    inv = torch.empty(P, dtype=torch.int32, device=dev) if inv is None else inv
    ws = alloc_workspace(s, WS_BUCKET, dev) if ws is None else ws
    rc = lib().spt_bucket_tokens(ctypes.byref(s), _ptr(idx, torch.int32, P, "idx"),
                                 _ptr(offsets, torch.int32, s.N + 1, "offsets"),
                                 _ptr(perm, torch.int32, P, "perm"), _ptr(inv, torch.int32, P, "inv"),
                                 ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "spt_bucket_tokens")
    return offsets, perm, inv


def bucket_tokens_noalloc(shape: SptShape, idx, offsets, perm, inv):
    """spt_bucket_tokens without a workspace: the library's fixed scratch is used instead.
    The caller passes every output; nothing is allocated here or in the library."""
    s = shape
    P = s.T * s.k
    rc = lib().spt_bucket_tokens_noalloc(ctypes.byref(s), _ptr(idx, torch.int32, P, "idx"),
                                         _ptr(offsets, torch.int32, s.N + 1, "offsets"),
                                         _ptr(perm, torch.int32, P, "perm"),
                                         _ptr(inv, torch.int32, P, "inv"), _stream())
    _check(rc, "spt_bucket_tokens_noalloc")
    return offsets, perm, inv


def build_schedule(shape: SptShape, offsets, perm, sched=None):
    """The launch tables of routed_ffn_fwd / routed_ffn_bwd for one bucketing, built once: pass the
    returned buffer to both as `sched`."""
    s = shape
    P = s.T * s.k
    sched = alloc_workspace(s, WS_SCHEDULE, offsets.device) if sched is None else sched
    rc = lib().spt_build_schedule(ctypes.byref(s), _ptr(offsets, torch.int32, s.N + 1, "offsets"),
                                  _ptr(perm, torch.int32, P, "perm"), sched.data_ptr(), sched.numel(), _stream())
    _check(rc, "spt_build_schedule")
    return sched


def routed_ffn_fwd(shape: SptShape, X, W1, W2, offsets, perm, inv, ws=None, Y=None, Hsave=None,
                   save_for_backward=True, sched=None):
    """Y[T,d] bf16 and (optionally) Hsave[P,Bs] bf16."""
    s = shape
    P = s.T * s.k
    dev = X.device
    Y = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=dev) if Y is None else Y
    if Hsave is None and save_for_backward:
        Hsave = torch.empty((P, s.Bs), dtype=torch.bfloat16, device=dev)
    ws = alloc_workspace(s, WS_FWD, dev) if ws is None else ws
    nw = s.N * s.Bs * s.d
    args = (ctypes.byref(s), _ptr(X, torch.bfloat16, s.T * s.d, "X"),
            _ptr(W1, torch.bfloat16, nw, "W1"), _ptr(W2, torch.bfloat16, nw, "W2"),
            _ptr(offsets, torch.int32, s.N + 1, "offsets"),
            _ptr(perm, torch.int32, P, "perm"), _ptr(inv, torch.int32, P, "inv"),
            _ptr(Y, torch.bfloat16, s.T * s.d, "Y"), _ptr(Hsave, torch.bfloat16, P * s.Bs, "Hsave"),
            ws.data_ptr(), ws.numel())
    if sched is None:
        rc = lib().spt_routed_ffn_fwd(*args, _stream())
    else:
        rc = lib().spt_routed_ffn_fwd_sched(*args, sched.data_ptr(), sched.numel(), _stream())
    _check(rc, "spt_routed_ffn_fwd")
    return Y, Hsave


def routed_ffn_bwd(shape: SptShape, X, W1, W2, dY, offsets, perm, inv, Hsave, ws=None,
                   dX=None, dW1=None, dW2=None, sched=None):
    """dX[T,d] bf16, dW1/dW2[N,Bs,d] fp32."""
    s = shape
    P = s.T * s.k
    dev = X.device
    nw = s.N * s.Bs * s.d
    dX = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=dev) if dX is None else dX
    dW1 = torch.empty((s.N, s.Bs, s.d), dtype=torch.float32, device=dev) if dW1 is None else dW1
    dW2 = torch.empty((s.N, s.Bs, s.d), dtype=torch.float32, device=dev) if dW2 is None else dW2
    ws = alloc_workspace(s, WS_BWD, dev) if ws is None else ws
    args = (ctypes.byref(s), _ptr(X, torch.bfloat16, s.T * s.d, "X"),
            _ptr(W1, torch.bfloat16, nw, "W1"), _ptr(W2, torch.bfloat16, nw, "W2"),
            _ptr(dY, torch.bfloat16, s.T * s.d, "dY"),
            _ptr(offsets, torch.int32, s.N + 1, "offsets"),
            _ptr(perm, torch.int32, P, "perm"), _ptr(inv, torch.int32, P, "inv"),
            _ptr(Hsave, torch.bfloat16, P * s.Bs, "Hsave"), _ptr(dX, torch.bfloat16, s.T * s.d, "dX"),
            _ptr(dW1, torch.float32, nw, "dW1"), _ptr(dW2, torch.float32, nw, "dW2"),
            ws.data_ptr(), ws.numel())
    if sched is None:
        rc = lib().spt_routed_ffn_bwd(*args, _stream())
    else:
        rc = lib().spt_routed_ffn_bwd_sched(*args, sched.data_ptr(), sched.numel(), _stream())
    _check(rc, "spt_routed_ffn_bwd")
    return dX, dW1, dW2


def router_balance(shape: SptShape, X, logits, offsets, ws=None, loss=None, frac=None, dW_r=None,
                   db_r=None):
    """Load-balancing loss of the route network and its gradient: returns (loss[1], frac[N],
    dW_r[d,N], db_r[N]) as fp32 device tensors."""
    s = shape
    dev = X.device
    f32 = lambda *sh: torch.empty(sh, dtype=torch.float32, device=dev)
    loss = f32(1) if loss is None else loss
    frac = f32(s.N) if frac is None else frac
    dW_r = f32(s.d, s.N) if dW_r is None else dW_r
    db_r = f32(s.N) if db_r is None else db_r
    ws = alloc_workspace(s, WS_BALANCE, dev) if ws is None else ws
    rc = lib().spt_router_balance(ctypes.byref(s), _ptr(X, torch.bfloat16, s.T * s.d, "X"),
                                  _ptr(logits, torch.float32, s.T * s.N, "logits"),
                                  _ptr(offsets, torch.int32, s.N + 1, "offsets"),
                                  _ptr(loss, torch.float32, 1, "loss"), _ptr(frac, torch.float32, s.N, "frac"),
                                  _ptr(dW_r, torch.float32, s.d * s.N, "dW_r"),
                                  _ptr(db_r, torch.float32, s.N, "db_r"),
                                  ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "spt_router_balance")
    return loss, frac, dW_r, db_r


def _adapter_ptrs(s: SptShape, r: int, A1, C1, B2, C2):
    D = s.N * s.Bs
    return (_ptr(A1, torch.bfloat16, s.d * r, "A1"), _ptr(C1, torch.bfloat16, r * D, "C1"),
            _ptr(B2, torch.bfloat16, D * r, "B2"), _ptr(C2, torch.bfloat16, r * s.d, "C2"))


def lora_ffn_fwd(shape: SptShape, r: int, X, W1, W2, A1, C1, B2, C2, offsets, perm, inv, ws=None,
                 Y=None, Hsave=None, save_for_backward=True):
    """Low-rank adapted forward: adapters A1[d,r], C1[r,N*Bs], B2[N*Bs,r], C2[r,d] (bf16).
    Returns Y[T,d] bf16 and Hsave[P,Bs] bf16 (pre-activations including the adapter term)."""
    s = shape
    P = s.T * s.k
    dev = X.device
    Y = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=dev) if Y is None else Y
    if Hsave is None and save_for_backward:
        Hsave = torch.empty((P, s.Bs), dtype=torch.bfloat16, device=dev)
    ws = alloc_workspace(s, WS_LORA_FWD, dev) if ws is None else ws
    nw = s.N * s.Bs * s.d
    rc = lib().spt_lora_ffn_fwd(ctypes.byref(s), r, _ptr(X, torch.bfloat16, s.T * s.d, "X"),
                                _ptr(W1, torch.bfloat16, nw, "W1"), _ptr(W2, torch.bfloat16, nw, "W2"),
                                *_adapter_ptrs(s, r, A1, C1, B2, C2),
                                _ptr(offsets, torch.int32, s.N + 1, "offsets"),
                                _ptr(perm, torch.int32, P, "perm"), _ptr(inv, torch.int32, P, "inv"),
                                _ptr(Y, torch.bfloat16, s.T * s.d, "Y"),
                                _ptr(Hsave, torch.bfloat16, P * s.Bs, "Hsave"),
                                ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "spt_lora_ffn_fwd")
    return Y, Hsave


def lora_ffn_bwd(shape: SptShape, r: int, X, W1, W2, A1, C1, B2, C2, dY, offsets, perm, inv, Hsave,
                 ws=None, dX=None, dA1=None, dC1=None, dB2=None, dC2=None):
    """Low-rank adapted backward with frozen W1, W2: dX[T,d] bf16 and the fp32 adapter gradients
    dA1[d,r], dC1[r,N*Bs], dB2[N*Bs,r], dC2[r,d]."""
    s = shape
    P = s.T * s.k
    D = s.N * s.Bs
    dev = X.device
    f32 = lambda *shape_: torch.empty(shape_, dtype=torch.float32, device=dev)
    dX = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=dev) if dX is None else dX
    dA1 = f32(s.d, r) if dA1 is None else dA1
    dC1 = f32(r, D) if dC1 is None else dC1
    dB2 = f32(D, r) if dB2 is None else dB2
    dC2 = f32(r, s.d) if dC2 is None else dC2
    ws = alloc_workspace(s, WS_LORA_BWD, dev) if ws is None else ws
    nw = s.N * s.Bs * s.d
    rc = lib().spt_lora_ffn_bwd(ctypes.byref(s), r, _ptr(X, torch.bfloat16, s.T * s.d, "X"),
                                _ptr(W1, torch.bfloat16, nw, "W1"), _ptr(W2, torch.bfloat16, nw, "W2"),
                                *_adapter_ptrs(s, r, A1, C1, B2, C2),
                                _ptr(dY, torch.bfloat16, s.T * s.d, "dY"),
                                _ptr(offsets, torch.int32, s.N + 1, "offsets"),
                                _ptr(perm, torch.int32, P, "perm"), _ptr(inv, torch.int32, P, "inv"),
                                _ptr(Hsave, torch.bfloat16, P * s.Bs, "Hsave"),
                                _ptr(dX, torch.bfloat16, s.T * s.d, "dX"),
                                _ptr(dA1, torch.float32, s.d * r, "dA1"), _ptr(dC1, torch.float32, r * D, "dC1"),
                                _ptr(dB2, torch.float32, D * r, "dB2"), _ptr(dC2, torch.float32, r * s.d, "dC2"),
                                ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "spt_lora_ffn_bwd")
    return dX, dA1, dC1, dB2, dC2


def bf16_tensor_from_bits(bits, device="cuda") -> torch.Tensor:
    """Upload uint16 bf16 patterns (numpy) as a torch.bfloat16 tensor, bit for bit."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def bf16_bits_to_numpy(t: torch.Tensor):
    """Download a bf16 tensor as uint16 patterns (numpy)."""
    import numpy as np
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def profile_enable(on: bool, only: Optional[str] = None) -> None:
    """Diagnostic: record HIP events around every kernel the library launches, or only around
    the kernel slot named `only`."""
    code = 1 if on else 0
    if on and only is not None:
        L = lib()
        names = [L.spt_profile_slot_name(i).decode() for i in range(L.spt_profile_slots())]
        code = 2 + names.index(only)
    _check(lib().spt_profile_enable(code), "spt_profile_enable")


def profile_read() -> dict:
    """{kernel slot name: (total ms, launches)} since the last read (waits for the events)."""
    L = lib()
    n = L.spt_profile_slots()
    ms = (ctypes.c_float * n)()
    cnt = (ctypes.c_int32 * n)()
    _check(L.spt_profile_read(ms, cnt), "spt_profile_read")
    return {L.spt_profile_slot_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


def calibrate_mfma(iters: int, workgroups: int, out, pattern: int = 0):
    """Enqueue the register-resident bf16 MFMA loop (pattern 0: trivial operands, 1: random
    values); returns the FLOP it performs."""
    _check(lib().spt_calibrate_mfma(iters, workgroups, pattern,
                                    _ptr(out, torch.float32, workgroups * 256, "out"), _stream()),
           "spt_calibrate_mfma")
    return workgroups * 4 * iters * 8 * 32768.0


def calibrate_stream(src, dst, mode: int):
    """Enqueue a streaming copy (0), read (1) or write (2) over the byte tensors src / dst."""
    n = dst.numel() if mode == 2 else src.numel()
    _check(lib().spt_calibrate_stream(None if src is None else src.data_ptr(), dst.data_ptr(), n, mode,
                                      _stream()), "spt_calibrate_stream")
    return n
