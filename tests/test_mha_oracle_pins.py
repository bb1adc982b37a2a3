"""Pins of the sparse multi-head attention oracle (oracle/mha.py) against things other than
itself: library routines (scipy cdist, numpy stable sort, torch dense masked attention and its
autograd), a hand-worked run of the paper's Algorithm 3, closed forms and brute force."""
import math
import os

import numpy as np
import pytest

import oracle.mha as mha

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *vals = line.split()
            out[name] = np.array([int(v) for v in vals])
    return out


def scores_of(cq, ck):
    """Eq. 6 by brute force: score[s, i, j] = number of codebooks where the codes agree."""
    return (cq[:, :, None, :] == ck[:, None, :, :]).sum(axis=3)


def test_pq_assign_is_cdist_argmin():
    from scipy.spatial.distance import cdist
    rng = np.random.default_rng(1)
    S, H, n, M, E, dp = 6, 3, 50, 4, 16, 8
    X = rng.standard_normal((S, n, M * dp)).astype(np.float32)
    C = rng.standard_normal((H, M, E, dp)).astype(np.float32)
    C[1, 2, 9] = C[1, 2, 4]                         # duplicate codeword: ties go to the lower index
    X[1, 7, 16:24] = C[1, 2, 4]                     # (sequence 1 belongs to head 1)
    codes, margin, err = mha.pq_assign(X, C, with_error=True)
    for s in range(S):
        for m in range(M):
            dist = cdist(X[s, :, m * dp:(m + 1) * dp].astype(np.float64), C[s % H, m].astype(np.float64), "sqeuclidean")
            assert np.array_equal(codes[s, :, m], dist.argmin(axis=1))
            part = np.partition(dist, 1, axis=1)
            np.testing.assert_allclose(margin[s, :, m], part[:, 1] - part[:, 0], atol=1e-12)
            # Alg. 2 lines 4-5: the quantisation error is the (plain Euclidean) distance to the chosen codeword
            plain = cdist(X[s, :, m * dp:(m + 1) * dp].astype(np.float64), C[s % H, m].astype(np.float64))
            np.testing.assert_allclose(err[s, :, m], plain.min(axis=1), rtol=1e-12, atol=1e-12)
    assert codes[1, 7, 2] == 4 and margin[1, 7, 2] == 0.0 and err[1, 7, 2] == 0.0


def test_topl_hand_worked_example():
    g = read_golden(os.path.join(GOLDEN, "topl_hand_example.txt"))
    ck = g["key_codes"].reshape(1, 7, 2).astype(np.uint8)
    cq = np.zeros((1, 7, 2), dtype=np.uint8)
    cq[0, 0] = g["query_code"]
    cq[0, 1] = g["query2_code"]
    idx = mha.topl(cq, ck, 3)
    assert np.array_equal(idx[0, 0], g["idx"])
    assert np.array_equal(idx[0, 1], g["idx2"])


def test_topl_without_overflow_is_a_stable_sort_by_score():
    rng = np.random.default_rng(2)
    S, n, M, L = 5, 90, 8, 24
    # 4 codewords per book keep every score bucket far below L - 1 = 23 keys ... except score 0-3,
    # so use many codewords for most books and check the no-overflow precondition explicitly
    cq = rng.integers(0, 3, (S, n, M)).astype(np.uint8)
    ck = rng.integers(0, 3, (S, n, M)).astype(np.uint8)
    sc = scores_of(cq, ck)
    idx = mha.topl(cq, ck, L)
    checked = 0
    for s in range(S):
        for i in range(n):
            counts = np.bincount(sc[s, i], minlength=M + 1)
            # buckets that are actually read before L keys are found
            need, ok = L, True
            for b in range(M, -1, -1):
                if need <= 0:
                    break
                if counts[b] > L - 1:
                    ok = False
                need -= min(counts[b], L - 1)
            if not ok:
                continue
            order = np.argsort(-sc[s, i], kind="stable")[:L]
            assert np.array_equal(idx[s, i], order)
            checked += 1
    assert checked > S * n // 2


def test_topl_overflow_and_exhaustion():
    n, M, L = 40, 4, 8
    ck = np.zeros((1, n, M), dtype=np.uint8)
    ck[0, 30:, 0] = 1                               # keys 30..39 agree with the query in 3 books, the rest in 4
    cq = np.zeros((1, n, M), dtype=np.uint8)
    idx = mha.topl(cq, ck, L)
    # score-4 bucket overflows: only its first L - 1 = 7 arrivals are read; then the score-3 bucket
    assert np.array_equal(idx[0, 0], [0, 1, 2, 3, 4, 5, 6, 30])
    # every key in ONE bucket and nothing else: L - 1 keys, then no key
    ck2 = np.zeros((1, n, M), dtype=np.uint8)
    idx2 = mha.topl(cq, ck2, L)
    assert np.array_equal(idx2[0, 5], [0, 1, 2, 3, 4, 5, 6, -1])
    # all entries are distinct keys (or -1) and in range
    rng = np.random.default_rng(3)
    cq3 = rng.integers(0, 16, (3, 64, 8)).astype(np.uint8)
    ck3 = rng.integers(0, 16, (3, 64, 8)).astype(np.uint8)
    idx3 = mha.topl(cq3, ck3, 8)
    for row in idx3.reshape(-1, 8):
        valid = row[row >= 0]
        assert len(set(valid.tolist())) == len(valid) and valid.max(initial=0) < 64
    # selected keys never score lower than an unselected key that arrived ... before the bucket cut:
    sc = scores_of(cq3, ck3)
    for s in range(3):
        for i in range(64):
            sel = idx3[s, i]
            assert np.all(np.diff(sc[s, i][sel[sel >= 0]]) <= 0)      # scores are non-increasing along the row


def dense_masked_attention(Q, K, V, idx, scale):
    import torch
    S, n, _ = Q.shape
    mask = np.zeros((S, n, n), dtype=bool)
    for s in range(S):
        for i in range(n):
            row = idx[s, i]
            mask[s, i, row[row >= 0]] = True
    tQ, tK, tV = (torch.tensor(a.astype(np.float64), requires_grad=True) for a in (Q, K, V))
    logits = scale * tQ @ tK.transpose(1, 2)
    logits = logits.masked_fill(~torch.from_numpy(mask), float("-inf"))
    A = torch.softmax(logits, dim=2)
    return tQ, tK, tV, A, A @ tV


@pytest.mark.parametrize("L", [5, 12])
def test_sparse_attention_is_dense_attention_restricted_to_the_selected_keys(L):
    import torch
    rng = np.random.default_rng(4)
    S, n, dh = 3, 12, 8
    Q, K, V, dY = (rng.standard_normal((S, n, dh)).astype(np.float32) for _ in range(4))
    if L == n:
        idx = np.tile(np.arange(n, dtype=np.int32), (S, n, 1))           # everything selected: textbook attention
    else:
        idx = np.stack([np.stack([rng.permutation(n)[:L] for _ in range(n)]) for _ in range(S)]).astype(np.int32)
        idx[0, 3, L - 1] = -1                                             # one exhausted entry
    scale = 1.0 / math.sqrt(dh)
    A, Y = mha.attn_fwd(Q, K, V, idx, scale)
    tQ, tK, tV, tA, tY = dense_masked_attention(Q, K, V, idx, scale)
    np.testing.assert_allclose(Y, tY.detach().numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(A.sum(axis=2), 1.0, atol=1e-14)
    tY.backward(torch.from_numpy(dY.astype(np.float64)))
    dQ, dK, dV = mha.attn_bwd(Q, K, V, dY, idx, A, scale)
    np.testing.assert_allclose(dQ, tQ.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, tK.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, tV.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_sparse_attention_with_one_key_per_query_copies_values():
    rng = np.random.default_rng(5)
    S, n, dh = 2, 6, 4
    Q, K, V, dY = (rng.standard_normal((S, n, dh)).astype(np.float32) for _ in range(4))
    idx = rng.integers(0, n, (S, n, 1)).astype(np.int32)
    A, Y = mha.attn_fwd(Q, K, V, idx, 0.7)
    assert np.array_equal(A, np.ones((S, n, 1)))
    for s in range(S):
        assert np.array_equal(Y[s], V[s][idx[s, :, 0]].astype(np.float64))
    dQ, dK, dV = mha.attn_bwd(Q, K, V, dY, idx, A, 0.7)
    assert not dQ.any() and not dK.any()          # a one-entry softmax is constant
    ref = np.zeros((S, n, dh))
    for s in range(S):
        np.add.at(ref[s], idx[s, :, 0], dY[s].astype(np.float64))
    np.testing.assert_allclose(dV, ref, atol=1e-15)
