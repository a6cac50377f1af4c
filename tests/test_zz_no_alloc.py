"""The entry point that allocates nothing and takes no workspace: meteora_bucket_tokens_noalloc against
meteora_bucket_tokens (bit-exact, integer work), two calls in a row on the same GPU, the second smaller."""
import numpy as np
import pytest
import torch

import paper_2405_13053_amd as m

pytestmark = pytest.mark.gpu


def _routing(T, k, N, seed):
    """k distinct adapters per token, Zipf-like load (Gumbel top-k on log-probabilities)."""
    rng = np.random.default_rng(seed)
    p = 1.0 / (np.arange(N) + 1.0) ** 2
    scores = np.log(p)[None, :] + rng.gumbel(size=(T, N))
    return torch.from_numpy(np.argsort(-scores, axis=1)[:, :k].astype(np.int32)).cuda()


def test_noalloc_bucketing_equals_the_workspace_entry_point_twice_in_a_row():
    cases = [(16384, 2, 28, 1), (777, 3, 9, 2), (65536, 2, 64, 3), (1, 1, 5, 4)]   # large, then smaller, the limit, T = 1
    for T, k, N, seed in cases:
        idx = _routing(T, k, N, seed)
        ref = m.bucket_tokens(idx, N)
        # outputs exist before the call; the call itself must not allocate device memory
        out = tuple(torch.full_like(t, -7) for t in ref)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        got = m.bucket_tokens_noalloc(idx, N, out=out)
        after = torch.cuda.memory_stats()["allocation.all.allocated"]
        torch.cuda.synchronize()
        assert after == before
        for a, b, name in zip(got, ref, ("counts", "offsets", "bucket_tok", "bucket_slot")):
            assert torch.equal(a, b), f"T={T}: {name} differs"
        assert int(got[0].sum()) == T * k


def test_noalloc_bucketing_rejects_sizes_beyond_its_scratch():
    idx = torch.zeros((65537, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(m.MeteoraError) as e:
        m.bucket_tokens_noalloc(idx, 4)
    assert e.value.status == 5 and "fixed scratch" in str(e.value)
