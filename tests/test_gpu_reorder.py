"""GPU parity of the reordering path (Alg. 2) and of the boundary gather against the oracle."""
import time

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2111_05894_amd import synth, tier

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def _world(indptr, indices, dim, dtype=torch.float32):
    n = indptr.numel() - 1
    feat = torch.empty((n, dim), dtype=dtype, pin_memory=True)
    synth.fill_features(feat, "uniform", 5, "cpu")
    ctx = tier.tier_create(indptr.to(DEV), indices.to(DEV), feat)
    return ctx, feat


@pytest.mark.parametrize("n,m,i64,dim", [(2000, 30_000, True, 8), (3001, 40_000, False, 100), (70_000, 900_000, True, 32)])
def test_reorder_matches_oracle(n, m, i64, dim):
    ip, ix = synth.rmat_csr(n, m, 99, "cpu", i64_offsets=i64)
    ctx, feat = _world(ip, ix, dim)
    fb = feat.view(torch.uint8).numpy().reshape(n, -1)
    rb = fb.shape[1]
    ipn = ip.numpy().astype(np.int64); ixn = ix.numpy()
    rng = np.random.default_rng(n)
    counts = (rng.integers(0, 300, n) * (rng.random(n) < 0.5)).astype(np.uint32)
    cd = torch.from_numpy(counts.view(np.int32)).to(DEV)

    rank, order = tier.tier_rank(ctx, cd)
    orank, _, _ = orc.place(counts, rb, 0)
    assert np.array_equal(rank.cpu().numpy(), orank)
    assert np.array_equal(order.cpu().numpy()[orank], np.arange(n))

    ip2, ix2 = tier.tier_reorder_graph(ctx, rank, order)
    assert ip2.dtype == ip.dtype
    ond, oedg = orc.reorder_graph(ipn, ixn, orank)
    assert np.array_equal(ip2.cpu().numpy().astype(np.int64), ond)
    assert np.array_equal(ix2.cpu().numpy(), oedg)

    feat2 = torch.empty_like(feat).pin_memory()
    tier.tier_reorder_rows(ctx, rank, feat2)
    torch.cuda.synchronize()
    fb2 = feat2.view(torch.uint8).numpy().reshape(n, -1)
    assert np.array_equal(fb2, orc.reorder_rows(fb, orank))

    ids = torch.from_numpy(rng.integers(0, n, 777).astype(np.int32)).to(DEV)
    assert np.array_equal(tier.tier_relabel_ids(ctx, rank, ids).cpu().numpy(), orank[ids.cpu().numpy()])
    with pytest.raises(tier.TierError):
        tier.tier_relabel_ids(ctx, rank, torch.tensor([n], dtype=torch.int32, device=DEV))

    # a rank that is no permutation is refused before any kernel indexes with it
    broken = rank.clone(); broken[0] = broken[1]
    with pytest.raises(tier.TierError):
        tier.tier_reorder_graph(ctx, broken, order)
    with pytest.raises(tier.TierError):
        tier.tier_reorder_rows(ctx, broken, torch.empty_like(feat).pin_memory())
    broken[0] = n
    with pytest.raises(tier.TierError):
        tier.tier_reorder_rows(ctx, broken, torch.empty_like(feat).pin_memory())
    ip3, ix3 = tier.tier_reorder_graph(ctx, rank, order)                 # the context is still good
    assert torch.equal(ip3, ip2) and torch.equal(ix3, ix2)

    # a context on the reordered data: boundary placement, gather, and sampling
    ctx2 = tier.tier_create(ip2, ix2, feat2)
    for rows in (0, 1, n // 10, n):
        n_hot = tier.tier_place_boundary(ctx2, rows * rb + 3)
        assert n_hot == rows
        new_ids = rng.integers(0, n, 4001).astype(np.int32)
        out, hit, miss = tier.tier_gather_features(ctx2, torch.from_numpy(new_ids).to(DEV), want_stats=True)
        want, whit = orc.gather_boundary(fb2, rows, new_ids)
        assert (hit, miss) == (whit, len(new_ids) - whit)
        assert np.array_equal(out.view(torch.uint8).cpu().numpy().reshape(len(new_ids), rb), want)
    seeds = orank[rng.choice(n, 200, replace=False)].astype(np.int32)
    got = tier.tier_sample_minibatch(ctx2, torch.from_numpy(seeds).to(DEV), (5, 3), 17)
    want = orc.sample_minibatch(ond, oedg, seeds, (5, 3), 17)
    assert got.n_nodes == want["n_nodes"].tolist()
    assert np.array_equal(got.frontier().cpu().numpy(), want["nodes"])
    for l in range(2):
        assert np.array_equal(got.eid[l][: got.n_edges[l]].cpu().numpy(), want["eid"][l])
        assert np.array_equal(got.col[l][: got.n_edges[l]].cpu().numpy(), want["col"][l])
    ctx2.close(); ctx.close()


def test_reorder_cfg2_full_size():
    """Alg. 2 on the 2.4 M-node workload: same result as the oracle; times printed."""
    wl = synth.WORKLOADS["cfg2"]
    ip, ix, train = synth.make_graph(wl, DEV)
    n = ip.numel() - 1
    table = tier.tier_host_alloc(n, wl.dim, torch.float32)
    table2 = tier.tier_host_alloc(n, wl.dim, torch.float32)
    try:
        synth.fill_features(table.tensor, wl.dist, 7, DEV)
        ctx = tier.tier_create(ip, ix, table)
        counts = tier.tier_presample(ctx, train, wl.batch_size, wl.fanouts, 1, synth.PRESAMPLE_SEED)
        torch.cuda.synchronize(); t0 = time.time()
        rank, order = tier.tier_rank(ctx, counts)
        t1 = time.time()
        ip2, ix2 = tier.tier_reorder_graph(ctx, rank, order)
        t2 = time.time()
        tier.tier_reorder_rows(ctx, rank, table2)
        torch.cuda.synchronize(); t3 = time.time()
        say(f"cfg2 reorder on GPU: rank {1e3 * (t1 - t0):.2f} ms, graph {1e3 * (t2 - t1):.2f} ms, "
            f"rows {1e3 * (t3 - t2):.2f} ms")
        cn = counts.cpu().numpy().view(np.uint32)
        orank, _, _ = orc.place(cn, wl.row_bytes, 0)
        assert np.array_equal(rank.cpu().numpy(), orank)
        t4 = time.time()
        ond, oedg = orc.reorder_graph(ip.cpu().numpy(), ix.cpu().numpy(), orank)
        say(f"cfg2 reorder oracle (graph only, 1 thread): {time.time() - t4:.2f} s")
        assert np.array_equal(ip2.cpu().numpy(), ond) and np.array_equal(ix2.cpu().numpy(), oedg)
        fb = table.tensor.view(-1).view(torch.uint8).numpy().reshape(n, -1)
        fb2 = table2.tensor.view(-1).view(torch.uint8).numpy().reshape(n, -1)
        assert np.array_equal(fb2[orank], fb)
        ctx.close()
    finally:
        table.free(); table2.free()
