"""The allocation-free bucketing entry point against the ordinary one (through the C ABI):
identical offsets / perm / inv, on two calls in a row, the second with a smaller input (the
fixed scratch keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2312_10365_amd import inputs as gen
from paper_2312_10365_amd import spt


def _random_idx(T, N, k, seed):
    rng = np.random.default_rng(seed)
    idx = np.stack([np.sort(rng.choice(N, size=k, replace=False)) for _ in range(T)]).astype(np.int32)
    return torch.from_numpy(idx).cuda()


@pytest.mark.gpu
def test_noalloc_bucketing_matches_twice_second_call_smaller():
    for (T, N, k, seed) in ((4096, 128, 32, 11), (700, 48, 5, 12)):
        shape = spt.make_shape(T, 256, N, 64, k)
        idx = _random_idx(T, N, k, seed)
        ref = spt.bucket_tokens(shape, idx)
        neg = lambda n: torch.full((n,), -1, dtype=torch.int32, device="cuda")
        out = (neg(N + 1), neg(T * k), neg(T * k))
        n_allocs = torch.cuda.memory_stats()["allocation.all.allocated"]
        got = spt.bucket_tokens_noalloc(shape, idx, *out)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == n_allocs   # no torch allocation in the call
        torch.cuda.synchronize()
        for name, a, b in zip(("offsets", "perm", "inv"), got, ref):
            assert torch.equal(a, b), f"T={T}: {name} differs from spt_bucket_tokens"


def test_noalloc_bucketing_rejects_sizes_beyond_its_scratch():
    L = spt.lib()
    fake = ctypes.c_void_p(4096)
    ok = spt.make_shape(262144, 64, 128, 32, 2)        # 2048 chunks x 128 blocks = 262144 entries: the limit
    too_big = spt.make_shape(262144 + 128, 64, 128, 32, 2)
    assert L.spt_bucket_tokens_noalloc(ctypes.byref(too_big), fake, fake, fake, fake, None) == -5
    assert "fixed scratch" in spt.strerror(-5)
    assert L.spt_bucket_tokens_noalloc(ctypes.byref(ok), None, fake, fake, fake, None) == -1   # size fine, null input
    bad = spt.make_shape(64, 100, 4, 32, 2)
    assert L.spt_bucket_tokens_noalloc(ctypes.byref(bad), fake, fake, fake, fake, None) == -2
