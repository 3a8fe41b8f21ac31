"""GPU parity of the score functions (out degree: bit-exact; weighted reverse PageRank:
fp64 within 1e-12 relative, the bound of summing each node's pulls in any order) and of
the real-valued ranking (bit-exact on equal inputs)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2111_05894_amd import synth, tier

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-12     # each score is a sum of <= 2^31 non-negative fp64 terms: reordering moves it by a few ulp


def _ctx(ip, ix, dim=4):
    n = ip.numel() - 1
    feat = torch.zeros((n, dim), dtype=torch.float32).pin_memory()
    return tier.tier_create(ip.to(DEV), ix.to(DEV), feat), feat


@pytest.mark.parametrize("n,m,i64", [(500, 6000, True), (3001, 40_000, False), (200_000, 3_000_000, True)])
def test_scores_match_oracle(n, m, i64):
    ip, ix = synth.rmat_csr(n, m, 13, "cpu", i64_offsets=i64)
    ctx, _ = _ctx(ip, ix)
    ipn = ip.numpy().astype(np.int64); ixn = ix.numpy()
    deg = tier.tier_score_degree(ctx)
    assert np.array_equal(deg.cpu().numpy().view(np.uint32), orc.score_degree(ipn, ixn))
    train = synth.train_set(n, 0.1, 5)
    for iters, damp, tid in ((5, 0.85, train), (1, 0.5, train[:3]), (0, 0.85, train), (8, 0.85, train[:0])):
        got = tier.tier_score_wrpr(ctx, tid.to(DEV), iters, damp).cpu().numpy()
        want = orc.score_wrpr(ipn, ixn, tid.numpy(), iters, damp)
        assert np.allclose(got, want, rtol=RTOL, atol=0), (iters, damp, np.abs(got / want - 1).max())
        # the ranking the GPU derives is a valid descending order of the oracle's scores up to that bound
        rank, order = tier.tier_rank_scores(ctx, torch.from_numpy(got).to(DEV))
        o = order.cpu().numpy()
        assert np.array_equal(np.sort(o), np.arange(n))
        s = want[o]
        assert np.all(s[:-1] >= s[1:] * (1 - 4 * RTOL))
        # on identical inputs the ranking is exact (ties by id)
        assert np.array_equal(rank.cpu().numpy(), orc.rank_scores(got))
    with pytest.raises(tier.TierError):
        tier.tier_score_wrpr(ctx, torch.tensor([n], dtype=torch.int32, device=DEV), 1, 0.85)
    with pytest.raises(tier.TierError):
        tier.tier_score_wrpr(ctx, train.to(DEV), 1, 1.5)
    ctx.close()


def test_rank_scores_edge_values():
    n = 70_001
    ip = torch.zeros(n + 1, dtype=torch.int64); ix = torch.zeros(0, dtype=torch.int32)
    ctx, _ = _ctx(ip, ix)
    rng = np.random.default_rng(8)
    for s in (rng.choice([0.0, -0.0, 1.0, 1e-300, 5e-324, 2.5, 1e300, -3.0, -1e-9], n),       # ties, signs, denormals
              rng.random(n), np.zeros(n), -rng.random(n) * 1e-5, np.array([0.1, 0.4, 0.2, 0.3] + [0.0] * (n - 4))):
        s = s.astype(np.float64)
        rank, order = tier.tier_rank_scores(ctx, torch.from_numpy(s).to(DEV))
        want = orc.rank_scores(s)
        assert np.array_equal(rank.cpu().numpy(), want)
        assert np.array_equal(order.cpu().numpy()[want], np.arange(n))
    ctx.close()


def test_place_scores_and_degree_placement():
    ip, ix = synth.rmat_csr(20_000, 300_000, 21, "cpu")
    n = 20_000
    feat = torch.empty((n, 32), dtype=torch.float32, pin_memory=True)
    synth.fill_features(feat, "uniform", 2, "cpu")
    fb = feat.view(torch.uint8).numpy().reshape(n, -1)
    ctx = tier.tier_create(ip.to(DEV), ix.to(DEV), feat)
    ipn = ip.numpy().astype(np.int64); ixn = ix.numpy()
    train = synth.train_set(n, 0.1, 5)
    budget = 2000 * 128 + 5
    # degree score through the integer placement
    deg = tier.tier_score_degree(ctx)
    slot, n_hot = tier.tier_place(ctx, deg, budget)
    _, oslot, ohot = orc.place(orc.score_degree(ipn, ixn), 128, budget)
    assert n_hot == ohot == 2000 and np.array_equal(slot.cpu().numpy(), oslot)
    # weighted reverse PageRank through the real-valued placement (same scores on both sides)
    score = tier.tier_score_wrpr(ctx, train.to(DEV), 5, 0.85)
    slot, n_hot = tier.tier_place_scores(ctx, score, budget)
    orank = orc.rank_scores(score.cpu().numpy())
    want = np.where(orank < 2000, orank, -1)
    assert n_hot == 2000 and np.array_equal(slot.cpu().numpy(), want)
    ids = torch.from_numpy(np.random.default_rng(1).integers(0, n, 5000).astype(np.int32)).to(DEV)
    out, hit, miss = tier.tier_gather_features(ctx, ids, want_stats=True)
    assert np.array_equal(out.view(torch.uint8).cpu().numpy().reshape(5000, 128), fb[ids.cpu().numpy()])
    assert hit == int((want[ids.cpu().numpy()] >= 0).sum())
    ctx.close()
