"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
function the header declares, sizes workspaces sensibly and rejects bad arguments
before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2312_10365_amd import spt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="spt.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spt_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert set(names) == set(spt.EXPORTS)
    L = spt.lib()
    for n in names:
        assert hasattr(L, n), n


def test_library_exports_every_declared_mha_function():
    from paper_2312_10365_amd import mha
    names = [n for n in declared_functions("spt_mha.h") if n.startswith("spt_mha_")]
    assert set(names) == set(mha.EXPORTS)
    L = mha.lib()
    for n in names:
        assert hasattr(L, n), n


def test_mha_validates_on_the_host():
    from paper_2312_10365_amd import mha
    L = mha.lib()
    ok = ctypes.c_void_p(0x1000)
    good = mha.make_shape(4, 2, 128, 64, 16)
    assert mha.workspace_bytes(good) >= 2 * 4 * 128 * 16 * 4 + 4 * 129 * 4
    assert mha.workspace_bytes(mha.make_shape(4, 2, 128, 80, 16)) == 0
    assert L.spt_mha_attn_fwd(ctypes.byref(good), None, ok, ok, ok, ok, ok, None) == -1
    assert L.spt_mha_attn_fwd(ctypes.byref(mha.make_shape(4, 3, 128, 64, 16)), ok, ok, ok, ok, ok, ok, None) == -1
    assert L.spt_mha_topl(ctypes.byref(mha.make_shape(4, 2, 128, 64, 129)), ok, ok, ok, None) == -1
    assert L.spt_mha_topl(ctypes.byref(mha.make_shape(4, 2, 128, 64, 16, E=17)), ok, ok, ok, None) == -2
    assert L.spt_mha_pq_assign(ctypes.byref(mha.make_shape(4, 2, 128, 64, 16, M=4)), ok, ok, ok, None, None) == -2
    assert L.spt_mha_attn_bwd(ctypes.byref(good), ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, 16, None) == -3


def test_strerror_and_codes():
    assert spt.strerror(0) == "success"
    for code in (-1, -2, -3, -4, -99):
        assert spt.strerror(code)


def test_workspace_sizes():
    s = spt.make_shape(8192, 4096, 128, 128, 32)
    P = 8192 * 32
    assert spt.workspace_bytes(s, spt.WS_BUCKET) >= (8192 // 128) * 128 * 4
    fwd = spt.workspace_bytes(s, spt.WS_FWD)
    bwd = spt.workspace_bytes(s, spt.WS_BWD)
    # narrow blocks: activated hidden values per pair, no per-pair partial output rows
    assert P * 128 * 2 <= fwd < P * 128 * 2 + (8 << 20)
    # backward: the second per-pair tensor, and staging for the weight-gradient pieces of buckets
    # larger than 1.5 x the mean (at most P / (1.5 P / N) blocks of Bs x d fp32)
    stage = (P // (3 * P // (2 * 128))) * 128 * 4096 * 4
    assert fwd + P * 128 * 2 + stage <= bwd < fwd + P * 128 * 2 + stage + (1 << 20)
    # wide blocks (more than 128 units) still stage per-pair partial rows
    wide = spt.make_shape(8192, 2048, 4, 2048, 2)
    assert spt.workspace_bytes(wide, spt.WS_FWD) >= 8192 * 2 * 2048 * 2 * 2
    # the schedule as a buffer of its own: the token id of every pair plus small tables
    sched = spt.workspace_bytes(s, spt.WS_SCHEDULE)
    assert P * 4 <= sched < P * 4 + (2 << 20)
    assert spt.workspace_bytes(s, 8) == 0
    assert spt.workspace_bytes(spt.make_shape(8, 100, 4, 32, 2), spt.WS_FWD) == 0   # d % 64


@pytest.mark.parametrize("shape,code", [
    ((0, 64, 4, 32, 2), -1), ((8, 64, 4, 32, 5), -1), ((8, 64, 4, 32, 0), -1),
    ((8, 100, 4, 32, 2), -2), ((8, 64, 4, 48, 2), -2), ((8, 64, 2048, 32, 2), -2),
])
def test_bad_shapes_are_rejected_before_any_launch(shape, code):
    s = spt.make_shape(*shape)
    L = spt.lib()
    fake = ctypes.c_void_p(4096)
    assert L.spt_router_topk(ctypes.byref(s), fake, fake, None, fake, None, fake, 1 << 30, None) == code
    assert L.spt_bucket_tokens(ctypes.byref(s), fake, fake, fake, fake, fake, 1 << 30, None) == code


def test_bad_pointers_and_workspace_are_rejected():
    s = spt.make_shape(64, 64, 4, 32, 2)
    L = spt.lib()
    ok = ctypes.c_void_p(1 << 20)
    odd = ctypes.c_void_p((1 << 20) + 2)
    assert L.spt_router_topk(ctypes.byref(s), None, ok, None, ok, None, ok, 1 << 30, None) == -1
    assert L.spt_router_topk(ctypes.byref(s), odd, ok, None, ok, None, ok, 1 << 30, None) == -1
    assert L.spt_router_topk(ctypes.byref(s), ok, ok, None, ok, None, ok, 16, None) == -3
    assert L.spt_bucket_tokens(ctypes.byref(s), ok, ok, ok, ok, ok, 0, None) == -3
    assert L.spt_routed_ffn_fwd(ctypes.byref(s), ok, ok, ok, ok, ok, ok, ok, None, ok, 16, None) == -3
    assert L.spt_routed_ffn_fwd(ctypes.byref(s), ok, ok, ok, ok, ok, ok, None, None, ok, 1 << 40, None) == -1
    assert L.spt_routed_ffn_bwd(ctypes.byref(s), ok, ok, ok, ok, ok, ok, ok, None, ok, ok, ok, ok, 1 << 40, None) == -1  # Hsave is required
    assert L.spt_routed_ffn_bwd(ctypes.byref(s), ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, 16, None) == -3
    # the schedule buffer: too small, misaligned, missing
    assert L.spt_build_schedule(ctypes.byref(s), ok, ok, ok, 16, None) == -3
    assert L.spt_build_schedule(ctypes.byref(s), ok, ok, odd, 1 << 30, None) == -1
    assert L.spt_build_schedule(ctypes.byref(s), ok, ok, None, 1 << 30, None) == -1
    assert L.spt_routed_ffn_fwd_sched(ctypes.byref(s), ok, ok, ok, ok, ok, ok, ok, None, ok, 1 << 40, ok, 16, None) == -3
    assert L.spt_routed_ffn_fwd_sched(ctypes.byref(s), ok, ok, ok, ok, ok, ok, ok, None, ok, 1 << 40, odd, 1 << 30, None) == -1
    assert L.spt_routed_ffn_bwd_sched(ctypes.byref(s), ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, 1 << 40, ok, 16, None) == -3
    bad_act = spt.make_shape(64, 64, 4, 32, 2, act=3)
    assert L.spt_router_topk(ctypes.byref(bad_act), ok, ok, None, ok, None, ok, 1 << 30, None) == -2
    bad_flag = spt.make_shape(64, 64, 4, 32, 2, flags=4)
    assert L.spt_router_topk(ctypes.byref(bad_flag), ok, ok, None, ok, None, ok, 1 << 30, None) == -2


def test_lora_entry_points_validate_on_the_host():
    s = spt.make_shape(64, 64, 4, 32, 2)
    L = spt.lib()
    ok = ctypes.c_void_p(1 << 20)
    assert spt.workspace_bytes(s, spt.WS_LORA_FWD) > spt.workspace_bytes(s, spt.WS_FWD)
    assert spt.workspace_bytes(s, spt.WS_LORA_BWD) > spt.workspace_bytes(s, spt.WS_BWD)
    fwd = lambda shape, r, ws_bytes, y=ok: L.spt_lora_ffn_fwd(
        ctypes.byref(shape), r, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, y, None, ok, ws_bytes, None)
    assert fwd(s, 0, 1 << 40) == -1 and fwd(s, 33, 1 << 40) == -1     # rank out of range
    assert fwd(s, 8, 16) == -3                                         # workspace too small
    assert fwd(s, 8, 1 << 40, None) == -1                              # null output
    bwd = L.spt_lora_ffn_bwd(ctypes.byref(s), 8, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, None,
                             ok, ok, ok, ok, ok, ok, 1 << 40, None)
    assert bwd == -1                                                   # Hsave is required


def test_router_balance_validates_on_the_host():
    s = spt.make_shape(64, 64, 4, 32, 2)
    L = spt.lib()
    ok = ctypes.c_void_p(1 << 20)
    assert spt.workspace_bytes(s, spt.WS_BALANCE) > 0
    call = lambda shape, loss, ws_bytes: L.spt_router_balance(ctypes.byref(shape), ok, ok, ok, loss, None, ok,
                                                              None, ok, ws_bytes, None)
    assert call(s, ok, 16) == -3
    assert call(s, None, 1 << 40) == -1
    assert call(spt.make_shape(64, 64, 4, 32, 2, spt.ACT_GELU, spt.FLAG_ABS_LOGIT), ok, 1 << 40) == -2
