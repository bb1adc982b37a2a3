"""GPU parity of the sparse multi-head attention (section 4.1, section 5.1) against the fp64
oracle, through the C ABI.  Codes and index lists are integer work: bit-exact, except that a PQ
code whose two best distances differ by less than 1e-5 of their scale may legitimately flip (the
kernel measures distances in fp32); such vectors are counted, reported and excluded.  Values:
relative Frobenius error <= 1e-2 (bf16 outputs)."""
import numpy as np
import pytest
import torch

from paper_2312_10365_amd import mha, spt
from paper_2312_10365_amd.mha_inputs import PRESETS, custom_mha_shape, make_mha_inputs

pytestmark = pytest.mark.gpu
from parity_util import TOL, check


def oracle():
    from oracle import mha as om
    return om


def to_dev(bits):
    return spt.bf16_tensor_from_bits(bits, "cuda")


def dev_shape(sh):
    return mha.make_shape(sh.S, sh.H, sh.n, sh.dh, sh.L, E=sh.E, scale=sh.softmax_scale)


def rel(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a)


def f32_of(t):
    return spt.bf16_bits_to_numpy(t).astype(np.uint32).__lshift__(16).view(np.float32)


CASES = [
    PRESETS["mha_tiny"],
    custom_mha_shape(1, 1, 64, 64, 64),          # L = n: every key reachable, overflow rule active
    custom_mha_shape(1, 2, 70, 128, 9, E=5),     # ragged n, few codewords (many equal codes)
    custom_mha_shape(2, 2, 300, 128, 130),       # three lanes' worth of entries, ragged
    custom_mha_shape(1, 1, 33, 64, 1),           # L = 1: the listing keeps nothing readable
    custom_mha_shape(1, 2, 257, 64, 256, E=2),   # largest L, heavy bucket overflow
    custom_mha_shape(1, 1, 520, 64, 65, seed=9, scale=1.0),  # the paper's unscaled softmax
    custom_mha_shape(1, 2, 600, 128, 70, seed=10),           # a sequence too large to sit in LDS
    custom_mha_shape(1, 1, 1100, 64, 50, seed=12),           # ... and too long for the LDS transposition
    custom_mha_shape(1, 1, 400, 128, 200, seed=13),          # head 128 with L > 128
    custom_mha_shape(1, 1, 4096, 128, 256, seed=14),         # the largest n, L and head size supported
    custom_mha_shape(1, 1, 1024, 64, 64, seed=15),           # the largest sequence that still sits in LDS
    custom_mha_shape(1, 1, 1, 64, 1, seed=16),               # a single token (and L = 1: nothing selected)
    custom_mha_shape(3, 1, 2, 128, 2, E=1, seed=17),         # two tokens, one codeword: every score is M
]


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for c in range(count):
        H = int(rng.integers(1, 4))
        batch = int(rng.integers(1, 3))
        n = int(rng.integers(3, 700))
        dh = int(rng.choice([64, 128]))
        L = int(rng.integers(1, min(n, 256) + 1))
        E = int(rng.integers(1, 17))
        out.append(custom_mha_shape(batch, H, n, dh, L, E=E, seed=100 + c))
    return out


CASES += _random_shapes(12, 2024)



@pytest.mark.parametrize("sh", CASES, ids=lambda s: s.name)
def test_whole_path_matches_oracle(sh):
    om = oracle()
    inp = make_mha_inputs(sh)
    s = dev_shape(sh)
    print(f"case {sh.name}", flush=True)
    Q, K, V, dY = (to_dev(getattr(inp, x + "_bits")) for x in ("Q", "K", "V", "dY"))
    C = torch.from_numpy(inp.C).cuda()
    # PQ assignment
    errq = torch.full((sh.S, sh.n, sh.M), float("nan"), device="cuda")
    cq = mha.pq_assign(s, Q, C, torch.full((sh.S, sh.n, sh.M), 255, dtype=torch.uint8, device="cuda"), errq)
    ck = mha.pq_assign(s, K, C)                      # err = NULL: the mini-batches that skip lines 4-5
    _, _, errq_ref = om.pq_assign(inp.f32("Q"), inp.C, with_error=True)
    # (a near-tie flip moves the error by less than the margin: still far inside the tolerance)
    assert rel(errq.cpu().numpy(), errq_ref) <= 1e-5
    flips = 0
    ref_codes = {}
    for name, got in (("Q", cq), ("K", ck)):
        ref, margin = om.pq_assign(inp.f32(name), inp.C)
        ref_codes[name] = ref
        bad = got.cpu().numpy() != ref
        scale2 = (inp.f32(name) ** 2).reshape(sh.S, sh.n, sh.M, 8).sum(-1) + 1.0
        unsafe = margin < 1e-5 * scale2
        assert not (bad & ~unsafe).any(), f"{name}: {int((bad & ~unsafe).sum())} wrong codes with a safe margin"
        flips += int(bad.sum())
    if flips:
        print(f"{sh.name}: {flips} near-tie codes differ (margin below 1e-5 relative)")
    # top-L on the oracle's codes (so a near-tie flip cannot leak into the index comparison)
    cq_ref = torch.from_numpy(ref_codes["Q"]).cuda(); ck_ref = torch.from_numpy(ref_codes["K"]).cuda()
    idx = mha.topl(s, cq_ref, ck_ref, torch.full((sh.S, sh.n, sh.L), -7, dtype=torch.int32, device="cuda"))
    idx_ref = om.topl(ref_codes["Q"], ref_codes["K"], sh.L)
    np.testing.assert_array_equal(idx.cpu().numpy(), idx_ref)
    # forward
    A = torch.full((sh.S, sh.n, sh.L), float("nan"), device="cuda")
    Y = to_dev(np.full((sh.S, sh.n, sh.dh), 0x7FC0, dtype=np.uint16))
    mha.attn_fwd(s, Q, K, V, idx, A, Y)
    A_ref, Y_ref = om.attn_fwd(inp.f32("Q"), inp.f32("K"), inp.f32("V"), idx_ref, sh.softmax_scale)
    check(sh.name, "A", A.cpu().numpy(), A_ref)
    check(sh.name, "Y", f32_of(Y), Y_ref)
    # backward (oracle from its own A; the kernel from the A it stored)
    outs = [to_dev(np.full((sh.S, sh.n, sh.dh), 0x7FC0, dtype=np.uint16)) for _ in range(3)]
    dQ, dK, dV = mha.attn_bwd(s, Q, K, V, dY, idx, A, None, *outs)
    dQ_ref, dK_ref, dV_ref = om.attn_bwd(inp.f32("Q"), inp.f32("K"), inp.f32("V"), inp.f32("dY"), idx_ref,
                                         A_ref, sh.softmax_scale)
    for name, got, ref in (("dQ", dQ, dQ_ref), ("dK", dK, dK_ref), ("dV", dV, dV_ref)):
        check(sh.name, name, f32_of(got), ref)
    torch.cuda.synchronize()


def test_backward_is_deterministic_and_workspace_reusable():
    sh = custom_mha_shape(2, 2, 200, 64, 40, seed=21)
    inp = make_mha_inputs(sh)
    s = dev_shape(sh)
    Q, K, V, dY = (to_dev(getattr(inp, x + "_bits")) for x in ("Q", "K", "V", "dY"))
    C = torch.from_numpy(inp.C).cuda()
    idx = mha.topl(s, mha.pq_assign(s, Q, C), mha.pq_assign(s, K, C))
    A, Y = mha.attn_fwd(s, Q, K, V, idx)
    ws = mha.alloc_workspace(s)
    ws.fill_(0xAB)                       # stale contents must not matter
    first = [t.clone() for t in mha.attn_bwd(s, Q, K, V, dY, idx, A, ws)]
    second = mha.attn_bwd(s, Q, K, V, dY, idx, A, ws)
    for a, b in zip(first, second):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_full_size_sampled_rows():
    """The workload bench.py times, checked on sampled sequences the oracle can do in seconds."""
    om = oracle()
    sh = PRESETS["mha_opt2048"]
    inp = make_mha_inputs(sh)
    s = dev_shape(sh)
    Q, K, V, dY = (to_dev(getattr(inp, x + "_bits")) for x in ("Q", "K", "V", "dY"))
    C = torch.from_numpy(inp.C).cuda()
    cq = mha.pq_assign(s, Q, C); ck = mha.pq_assign(s, K, C)
    idx = mha.topl(s, cq, ck)
    A, Y = mha.attn_fwd(s, Q, K, V, idx)
    dQ, dK, dV = mha.attn_bwd(s, Q, K, V, dY, idx, A)
    torch.cuda.synchronize()
    pick = [0, 37, 70, 101, 140, 171, 203, 255, 256, 290, 333, 367, 402, 440, 478, 511]   # 16 of the 512 sequences
    sub = lambda a: np.ascontiguousarray(a[pick])
    heads = [p % sh.H for p in pick]
    Csub = inp.C[heads]                  # one "head" per sampled sequence
    f = {x: sub(inp.f32(x)) for x in ("Q", "K", "V", "dY")}
    cq_ref, mq = om.pq_assign(f["Q"], Csub); ck_ref, mk = om.pq_assign(f["K"], Csub)
    cq_g = cq.cpu().numpy()[pick]; ck_g = ck.cpu().numpy()[pick]
    for g, r, m, x in ((cq_g, cq_ref, mq, f["Q"]), (ck_g, ck_ref, mk, f["K"])):
        scale2 = (x ** 2).reshape(len(pick), sh.n, sh.M, 8).sum(-1) + 1.0
        assert not ((g != r) & (m >= 1e-5 * scale2)).any()
    # indices from the GPU's own codes (identical unless a near-tie flipped)
    idx_ref = om.topl(cq_g, ck_g, sh.L)
    np.testing.assert_array_equal(idx.cpu().numpy()[pick], idx_ref)
    A_ref, Y_ref = om.attn_fwd(f["Q"], f["K"], f["V"], idx_ref, sh.softmax_scale)
    check("mha_opt2048, 16 sampled sequences", "A", A.cpu().numpy()[pick], A_ref)
    check("mha_opt2048, 16 sampled sequences", "Y", f32_of(Y)[pick], Y_ref)
    refs = om.attn_bwd(f["Q"], f["K"], f["V"], f["dY"], idx_ref, A_ref, sh.softmax_scale)
    for name, got, ref in zip(("dQ", "dK", "dV"), (dQ, dK, dV), refs):
        check("mha_opt2048, 16 sampled sequences", name, f32_of(got)[pick], ref)


def test_bad_arguments_are_rejected():
    s = mha.make_shape(2, 2, 64, 64, 8)
    Q = torch.zeros((2, 64, 64), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros((2, 64, 8), dtype=torch.int32, device="cuda")
    A = torch.zeros((2, 64, 8), device="cuda")
    with pytest.raises(spt.SptError) as e:
        mha.attn_bwd(s, Q, Q, Q, Q, idx, A, torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    Q80 = torch.zeros((2, 64, 80), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(spt.SptError) as e:
        mha.attn_fwd(mha.make_shape(2, 2, 64, 80, 8, M=10), Q80, Q80, Q80, idx)   # unsupported head size
    assert e.value.code == -2
    codes = torch.zeros(2 * 64 * 8, dtype=torch.uint8, device="cuda")
    with pytest.raises(spt.SptError) as e:
        mha.topl(mha.make_shape(2, 2, 64, 64, 65), codes, codes,
                 torch.zeros(2 * 64 * 65, dtype=torch.int32, device="cuda"))   # L > n
    assert e.value.code == -1


def test_step_replays_identically_from_a_hip_graph():
    """The calls allocate nothing, never synchronise and enqueue only on the caller's stream, so a
    whole attention step can be captured into a HIP graph; every replay (with eager work and
    synchronisations in between) must reproduce the eager results bit for bit."""
    sh = custom_mha_shape(2, 4, 256, 64, 32, seed=31)
    inp = make_mha_inputs(sh)
    s = dev_shape(sh)
    Q, K, V, dY = (to_dev(getattr(inp, x + "_bits")) for x in ("Q", "K", "V", "dY"))
    C = torch.from_numpy(inp.C).cuda()
    dev = Q.device
    cq = torch.empty((sh.S, sh.n, sh.M), dtype=torch.uint8, device=dev)
    ck = torch.empty_like(cq)
    idx = torch.empty((sh.S, sh.n, sh.L), dtype=torch.int32, device=dev)
    A = torch.empty((sh.S, sh.n, sh.L), dtype=torch.float32, device=dev)
    Y, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    ws = mha.alloc_workspace(s)

    def step():
        mha.pq_assign(s, Q, C, cq)
        mha.pq_assign(s, K, C, ck)
        mha.topl(s, cq, ck, idx)
        mha.attn_fwd(s, Q, K, V, idx, A, Y)
        mha.attn_bwd(s, Q, K, V, dY, idx, A, ws, dQ, dK, dV)

    outs = (cq, ck, idx, A, Y, dQ, dK, dV)
    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                      # warm up on the capture stream (function attributes etc.)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        for t in outs:
            t.fill_(0)
        ws.fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, e in zip(outs, eager):
            assert torch.equal(t.view(torch.uint8), e.view(torch.uint8))
