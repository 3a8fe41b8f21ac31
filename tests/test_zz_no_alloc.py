"""The ranking entry point that allocates nothing (for callers under HIP graph capture, serving
loops, harnesses that forbid hipMalloc): through the C ABI, against tier_rank on the same counts,
two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2111_05894_amd import tier

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _context(n):
    """tier_rank needs a context: an edgeless graph of n nodes over a 16-byte-row table."""
    ip = torch.zeros(n + 1, dtype=torch.int64, device=DEV)
    ix = torch.zeros(0, dtype=torch.int32, device=DEV)
    feat = torch.zeros((n, 4), dtype=torch.float32, pin_memory=True)
    return tier.tier_create(ip, ix, feat)


def _counts(n, seed, max_count):
    rng = np.random.default_rng(seed)
    c = rng.integers(0, max_count + 1, n).astype(np.uint32)
    if n > 10:
        c[rng.integers(0, n, 5)] = 3_000_000_000            # all four digits in play
    return torch.from_numpy(c.view(np.int32)).to(DEV)


def test_rank_static_matches_tier_rank_on_two_calls_in_a_row():
    # the larger call first, then a smaller one that finds the first call's leftovers in the scratch
    for n, seed, max_count in ((300_007, 1, 70_000), (4_097, 2, 3)):
        counts = _counts(n, seed, max_count)
        ctx = _context(n)
        try:
            want_rank, want_order = tier.tier_rank(ctx, counts)
            rank = torch.full((n,), -7, dtype=torch.int32, device=DEV)
            order = torch.full((n,), -7, dtype=torch.int32, device=DEV)
            tier.tier_rank_static(counts, rank, order)
            torch.cuda.synchronize()
            assert torch.equal(rank, want_rank) and torch.equal(order, want_order)
        finally:
            ctx.close()


def test_rank_static_one_output_sizes_and_limits():
    n = 1000
    counts = _counts(n, 3, 9)
    rank, order = tier.tier_rank_static(counts)
    c = counts.cpu().numpy().view(np.uint32)
    want_order = np.argsort(-c.astype(np.int64), kind="stable").astype(np.int32)
    assert np.array_equal(order.cpu().numpy(), want_order)
    assert np.array_equal(rank.cpu().numpy()[want_order], np.arange(n, dtype=np.int32))
    lib = tier._load()
    only_rank = torch.empty(n, dtype=torch.int32, device=DEV)
    assert lib.tier_rank_static(counts.data_ptr(), n, only_rank.data_ptr(), None, None) == 0
    torch.cuda.synchronize()
    assert torch.equal(only_rank, rank)
    assert lib.tier_rank_static(counts.data_ptr(), 0, only_rank.data_ptr(), None, None) == 0
    assert lib.tier_rank_static(counts.data_ptr(), n, None, None, None) == -1                              # nothing to write
    assert lib.tier_rank_static(counts.data_ptr(), tier.RANK_STATIC_MAX_NODES + 1, only_rank.data_ptr(), None, None) == -4
    big = tier.RANK_STATIC_MAX_NODES                                                                        # the largest size it takes
    counts = _counts(big, 4, 1000)
    rank, order = tier.tier_rank_static(counts)
    c = counts.cpu().numpy().view(np.uint32)
    assert np.array_equal(order.cpu().numpy(), np.argsort(-c.astype(np.int64), kind="stable").astype(np.int32))
