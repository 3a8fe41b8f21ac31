"""Pins of the CPU oracle against what the paper and the mathematics fix.

Everything here runs on the CPU.  Each test pins one function of
``oracle/tier_oracle.c`` to something other than itself: published known-answer
vectors, closed forms, brute-force enumeration, a separately written BFS, a
library sort, library fancy indexing, or a value the paper prints.
"""
import itertools
import os

import numpy as np
import pytest
from scipy import stats

from oracle import oracle as orc
from paper_2111_05894_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MASK32 = 0xFFFFFFFF


# ----------------------------------------------------------------------------
# random numbers
# ----------------------------------------------------------------------------
def _kat_rows():
    rows = []
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert orc.philox4x32_10(ctr, key).tolist() == want


def _philox_py(ctr, key, rounds=10):
    """Philox4x32 from the published description, on Python integers."""
    c = list(ctr); k = list(key)
    for _ in range(rounds):
        p0 = 0xD2511F53 * c[0]; p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK32, p1 & MASK32, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK32, p0 & MASK32]
        k = [(k[0] + 0x9E3779B9) & MASK32, (k[1] + 0xBB67AE85) & MASK32]
    return c


def test_philox_python_model_agrees_with_published_vectors_and_c():
    for ctr, key, want in _kat_rows():
        assert _philox_py(ctr, key) == want
    rng = np.random.default_rng(1)
    for _ in range(200):
        ctr = rng.integers(0, 2**32, 4).tolist(); key = rng.integers(0, 2**32, 2).tolist()
        assert orc.philox4x32_10(ctr, key).tolist() == _philox_py(ctr, key)


def test_bounded_closed_forms():
    top = 2**64 - 1
    for m in (1, 2, 3, 7, 1000, 2**31 - 1, 2**40 + 5):
        assert orc.bounded(0, m) == 0
        assert orc.bounded(top, m) == m - 1
    assert all(orc.bounded(r, 1) == 0 for r in (0, 1, 12345, top))
    rng = np.random.default_rng(2)
    rs = sorted(int(x) for x in rng.integers(0, 2**64, 500, dtype=np.uint64))
    for m in (5, 12, 2**33 + 1):
        vals = [orc.bounded(r, m) for r in rs]
        assert vals == sorted(vals)                         # monotone in r
        assert all(0 <= v < m for v in vals)
        assert vals == [(r * m) >> 64 for r in rs]          # exact 128-bit product
    # equal-width cells: the k-th value is reached first at ceil(k * 2^64 / m)
    m = 12
    for kk in range(1, m):
        edge = -(-kk * 2**64 // m)
        assert orc.bounded(edge, m) == kk and orc.bounded(edge - 1, m) == kk - 1


def test_batch_seed_keying():
    # words 0,1 of the block with counter (epoch, batch, 0, 2) and key = seed halves
    seed = 0x1234_5678_9ABC_DEF0
    for e, b in ((0, 0), (1, 0), (0, 1), (3, 77)):
        w = _philox_py([e, b, 0, 2], [seed & MASK32, seed >> 32])
        assert orc.batch_seed(seed, e, b) == (w[1] << 32) | w[0]
    assert len({orc.batch_seed(seed, e, b) for e in range(4) for b in range(50)}) == 200


# ----------------------------------------------------------------------------
# one node's draw
# ----------------------------------------------------------------------------
def test_draw_small_degree_takes_all_in_order():
    for d in range(0, 8):
        for k in (d, d + 1, 25):
            if k == 0:
                continue
            assert orc.draw_positions(7, 0, 3, d, k).tolist() == list(range(d))


def test_draw_distinct_and_in_range():
    rng = np.random.default_rng(3)
    for _ in range(300):
        d = int(rng.integers(2, 5000)); k = int(rng.integers(1, min(d, 64)))
        pos = orc.draw_positions(int(rng.integers(0, 2**63)), int(rng.integers(0, 8)), int(rng.integers(0, 2**31)), d, k)
        assert len(pos) == k and len(set(pos.tolist())) == k
        assert pos.min() >= 0 and pos.max() < d


def test_draw_follows_floyd_with_documented_keying():
    """Floyd's subset algorithm re-run on Python integers with the counter layout
    (node, draw, layer, 1): pins the addressing of every draw."""
    seed = 0xDEADBEEFCAFEF00D
    for (node, layer, d, k) in ((5, 0, 10, 3), (123456, 2, 1000, 25), (2**31 - 1, 7, 26, 25), (9, 1, 3, 2)):
        chosen = []
        for i in range(k):
            j = d - k + i
            w = _philox_py([node, i, layer, 1], [seed & MASK32, seed >> 32])
            t = (((w[1] << 32) | w[0]) * (j + 1)) >> 64
            chosen.append(j if t in chosen else t)
        assert orc.draw_positions(seed, layer, node, d, k).tolist() == chosen


def test_draw_uniform_over_subsets_chi_square():
    d, k, trials = 5, 2, 120_000
    subsets = {s: 0 for s in itertools.combinations(range(d), k)}
    incl = np.zeros(d)
    for s in range(trials):
        pos = orc.draw_positions(s * 2654435761 + 11, 1, 42, d, k)
        subsets[tuple(sorted(pos.tolist()))] += 1
        incl[pos] += 1
    obs = np.array(list(subsets.values()), float)
    assert stats.chisquare(obs).pvalue > 1e-3               # all 10 subsets equally likely
    assert np.all(np.abs(incl / trials - k / d) < 4 * np.sqrt(k / d * (1 - k / d) / trials))


def test_draw_uniform_over_nodes_and_layers():
    """Same law when the node id or the layer varies instead of the seed."""
    d, k = 6, 3
    for vary in ("node", "layer"):
        cnt = {s: 0 for s in itertools.combinations(range(d), k)}
        n = 40_000 if vary == "node" else 8
        for x in range(n):
            pos = orc.draw_positions(99, x % 8 if vary == "layer" else 0, x if vary == "node" else 5, d, k)
            cnt[tuple(sorted(pos.tolist()))] += 1
        if vary == "node":
            assert stats.chisquare(np.array(list(cnt.values()), float)).pvalue > 1e-3
        else:
            assert len([v for v in cnt.values() if v]) > 1   # layers give different draws


def test_draw_last_position_reachable_only_through_collision_rule():
    # k = d - 1: every subset misses exactly one position; all d choices equally likely
    d, k, trials = 4, 3, 60_000
    missing = np.zeros(d)
    for s in range(trials):
        pos = orc.draw_positions(s + 5, 0, 1, d, k)
        missing[list(set(range(d)) - set(pos.tolist()))[0]] += 1
    assert stats.chisquare(missing).pvalue > 1e-3


# ----------------------------------------------------------------------------
# mini-batch blocks
# ----------------------------------------------------------------------------
def _graph(n=400, m=3000, seed=7, kind="rmat"):
    return synth.small_graph(n, m, seed, kind)


def _check_blocks(indptr, indices, seeds, fanouts, out):
    L = len(fanouts)
    nodes = out["nodes"]
    assert len(set(nodes.tolist())) == len(nodes)                      # unique
    assert nodes[: len(seeds)].tolist() == list(seeds)                 # seeds first, given order
    for l in range(L):
        n_dst, n_src = int(out["n_nodes"][l]), int(out["n_nodes"][l + 1])
        new = nodes[n_dst:n_src]
        assert np.all(np.diff(new) > 0)                                # new nodes ascending
        rp, col, eid = out["row_ptr"][l], out["col"][l], out["eid"][l]
        assert rp[0] == 0 and rp[-1] == out["n_edges"][l] == len(col) == len(eid)
        seen_src = set()
        for i in range(n_dst):
            v = nodes[i]; beg, end = indptr[v], indptr[v + 1]
            cnt = rp[i + 1] - rp[i]
            assert cnt == min(fanouts[l], end - beg)                   # fixed number per node
            e = eid[rp[i]: rp[i + 1]]
            assert np.all((e >= beg) & (e < end))                      # a real neighbour of v
            assert len(set(e.tolist())) == cnt                         # without replacement
            if end - beg <= fanouts[l]:
                assert e.tolist() == list(range(beg, end))             # all, adjacency order
            c = col[rp[i]: rp[i + 1]]
            assert np.all((c >= 0) & (c < n_src))
            assert np.array_equal(nodes[c], indices[e])                # col names the sampled node
            seen_src.update(nodes[c].tolist())
        assert set(new.tolist()) <= seen_src                           # nothing unsampled is added
        assert seen_src <= set(nodes[:n_src].tolist())


def test_blocks_are_valid_samples():
    indptr, indices = _graph()
    rng = np.random.default_rng(5)
    for fan in ((3,), (4, 2), (5, 3, 2), (2, 2, 2, 2)):
        seeds = rng.choice(len(indptr) - 1, 17, replace=False).astype(np.int32)
        out = orc.sample_minibatch(indptr, indices, seeds, fan, 1234)
        _check_blocks(indptr, indices, seeds.tolist(), fan, out)


def test_blocks_depend_on_seed_only():
    indptr, indices = _graph()
    seeds = np.arange(0, 40, dtype=np.int32)
    a = orc.sample_minibatch(indptr, indices, seeds, (3, 3), 1)
    b = orc.sample_minibatch(indptr, indices, seeds, (3, 3), 1)
    c = orc.sample_minibatch(indptr, indices, seeds, (3, 3), 2)
    assert all(np.array_equal(x, y) for x, y in zip(a["eid"], b["eid"]))
    assert not all(np.array_equal(x, y) for x, y in zip(a["eid"], c["eid"]))


def _bfs_levels(indptr, indices, seeds, hops):
    """Textbook breadth-first closure: node sets reachable within 0..hops steps."""
    reached = set(seeds); levels = [set(reached)]
    for _ in range(hops):
        nxt = set(reached)
        for v in reached:
            nxt.update(indices[indptr[v]: indptr[v + 1]].tolist())
        reached = nxt; levels.append(set(reached))
    return levels


def test_full_fanout_equals_bfs_closure():
    indptr, indices = _graph(300, 1500, 11, "er")
    maxdeg = int(np.max(np.diff(indptr)))
    assert 1 < maxdeg <= 64
    fan = (maxdeg,) * 3
    seeds = np.array([3, 50, 51, 200], np.int32)
    out = orc.sample_minibatch(indptr, indices, seeds, fan, 99)
    levels = _bfs_levels(indptr, indices, seeds.tolist(), 3)
    for l in range(4):
        assert set(out["nodes"][: out["n_nodes"][l]].tolist()) == levels[l]
    for l in range(3):                                                 # every edge into frontier_l
        want = sorted(e for v in out["nodes"][: out["n_nodes"][l]] for e in range(indptr[v], indptr[v + 1]))
        assert sorted(out["eid"][l].tolist()) == want


def test_star_neighbours_equally_likely():
    """Hub with 7 in-neighbours, fanout 3, seen through the whole block builder."""
    d, k, trials = 7, 3, 30_000
    indptr = np.array([0, d] + [d] * d, np.int64)                      # node 0 <- nodes 1..7
    indices = np.arange(1, d + 1, dtype=np.int32)
    hits = np.zeros(d + 1)
    li = np.full(d + 1, -1, np.int32)
    for s in range(trials):
        out = orc.sample_minibatch(indptr, indices, np.array([0], np.int32), (k,), s, local_idx=li)
        assert out["n_nodes"][1] == 1 + k
        hits[out["nodes"][1:]] += 1
    assert np.all(li == -1)                                            # scratch restored
    assert stats.chisquare(hits[1:]).pvalue > 1e-3


def test_empty_and_degenerate_batches():
    indptr, indices = _graph()
    out = orc.sample_minibatch(indptr, indices, np.zeros(0, np.int32), (3, 2), 5)
    assert out["n_nodes"].tolist() == [0, 0, 0] and out["n_edges"].tolist() == [0, 0]
    iso = int(np.flatnonzero(np.diff(indptr) == 0)[0])                 # a node with no neighbours
    out = orc.sample_minibatch(indptr, indices, np.array([iso], np.int32), (3, 2), 5)
    assert out["n_nodes"].tolist() == [1, 1, 1] and out["n_edges"].tolist() == [0, 0]
    assert out["row_ptr"][0].tolist() == [0, 0]


# ----------------------------------------------------------------------------
# access counts
# ----------------------------------------------------------------------------
def test_counts_equal_histogram_of_batch_frontiers():
    indptr, indices = _graph(500, 4000, 13)
    train = synth.train_set(500, 0.3, 1).numpy()
    fan, bs, seed, epochs = (4, 3), 32, 77, 2
    counts, total, edges = orc.presample(indptr, indices, train, bs, fan, epochs, seed)
    want = np.zeros(500, np.int64); tot = 0; edg = 0
    nb = -(-len(train) // bs)
    for e in range(epochs):
        for b in range(nb):
            out = orc.sample_minibatch(indptr, indices, train[b * bs:(b + 1) * bs], fan, orc.batch_seed(seed, e, b))
            want[out["nodes"]] += 1; tot += len(out["nodes"]); edg += int(out["n_edges"].sum())
    assert np.array_equal(counts, want)
    assert counts.sum() == total == tot and edges == edg               # counts sum to the samples
    assert counts.max() <= epochs * nb
    assert np.all(counts[train] >= epochs)                             # a seed is always accessed
    c4, t4, e4 = orc.presample(indptr, indices, train, bs, fan, epochs, seed, threads=4)
    assert np.array_equal(c4, counts) and t4 == total and e4 == edges


def test_counts_full_fanout_equal_bfs_reach():
    indptr, indices = _graph(300, 1200, 17, "er")
    maxdeg = int(np.max(np.diff(indptr)))
    assert 1 < maxdeg <= 64
    train = synth.train_set(300, 0.2, 3).numpy()
    bs = 16
    counts, _, _ = orc.presample(indptr, indices, train, bs, (maxdeg, maxdeg), 1, 5)
    want = np.zeros(300, np.int64)
    for b in range(-(-len(train) // bs)):
        for v in _bfs_levels(indptr, indices, train[b * bs:(b + 1) * bs].tolist(), 2)[2]:
            want[v] += 1
    assert np.array_equal(counts, want)


def test_counts_one_hop_expectation():
    """One hop, closed form: a non-seed v is read by a batch with probability
    1 - prod over seeds u with v in adj(u) of (1 - min(1, k/deg u))."""
    indptr, indices = _graph(60, 400, 19)
    n = 60; k = 2; bs = 8
    train = np.arange(0, 24, dtype=np.int32)
    deg = np.diff(indptr)
    p = np.zeros(n)
    for b in range(3):
        seeds = train[b * bs:(b + 1) * bs]
        q = np.ones(n)
        for u in seeds:
            adj = indices[indptr[u]: indptr[u + 1]]
            if deg[u]:
                q[adj] *= 1 - min(1.0, k / deg[u])
        pb = 1 - q; pb[seeds] = 1.0
        p += pb
    runs = 3000
    acc = np.zeros(n)
    for s in range(runs):
        c, _, _ = orc.presample(indptr, indices, train, bs, (k,), 1, 1000 + s)
        acc += c
    mean = acc / runs
    sd = np.sqrt(np.maximum(p * 1.0, 1e-9) / runs) + 1e-9             # loose (variance <= mean)
    assert np.all(np.abs(mean - p) < 5 * sd + 1e-12)
    assert np.all(mean[p == 0] == 0)


def test_counts_empty_training_set():
    indptr, indices = _graph()
    counts, total, edges = orc.presample(indptr, indices, np.zeros(0, np.int32), 8, (3,), 1, 1)
    assert counts.sum() == 0 and total == 0 and edges == 0


# ----------------------------------------------------------------------------
# access counts, the other reading: every draw of a node counts
# ----------------------------------------------------------------------------
def test_draw_counts_equal_histogram_of_seeds_and_edge_sources():
    indptr, indices = _graph(500, 4000, 13)
    train = synth.train_set(500, 0.3, 1).numpy()
    fan, bs, seed, epochs = (4, 3), 32, 77, 2
    counts, draws = orc.presample_draws(indptr, indices, train, bs, fan, epochs, seed)
    by_eid = np.zeros(500, np.int64); by_col = np.zeros(500, np.int64); tot = 0
    nb = -(-len(train) // bs)
    for e in range(epochs):
        for b in range(nb):
            seeds = train[b * bs:(b + 1) * bs]
            out = orc.sample_minibatch(indptr, indices, seeds, fan, orc.batch_seed(seed, e, b))
            np.add.at(by_eid, seeds, 1); np.add.at(by_col, seeds, 1); tot += len(seeds)
            for l in range(len(fan)):
                np.add.at(by_eid, indices[out["eid"][l]], 1)            # the edge's source in the graph
                np.add.at(by_col, out["nodes"][out["col"][l]], 1)       # the same node through the block
                tot += len(out["eid"][l])
    assert np.array_equal(counts, by_eid) and np.array_equal(counts, by_col)
    assert counts.sum() == draws == tot                                 # counts sum to the samples
    frontier_counts, _, edges = orc.presample(indptr, indices, train, bs, fan, epochs, seed)
    assert draws == epochs * len(train) + edges
    assert np.all(counts >= frontier_counts)                            # a listed node was drawn or is a seed
    assert np.array_equal(counts > 0, frontier_counts > 0)
    c4, d4 = orc.presample_draws(indptr, indices, train, bs, fan, epochs, seed, threads=4)
    assert np.array_equal(c4, counts) and d4 == draws


def test_draw_counts_full_fanout_closed_form():
    """Fanouts above every degree: at hop l each node reached within l steps hands one count to each
    entry of its adjacency list (repeats included), and each seed gets one."""
    indptr, indices = _graph(300, 1200, 17, "er")
    maxdeg = int(np.max(np.diff(indptr)))
    assert 1 < maxdeg <= 64
    train = synth.train_set(300, 0.2, 3).numpy()
    bs, hops = 16, 2
    counts, _ = orc.presample_draws(indptr, indices, train, bs, (maxdeg,) * hops, 1, 5)
    want = np.zeros(300, np.int64)
    for b in range(-(-len(train) // bs)):
        seeds = train[b * bs:(b + 1) * bs].tolist()
        levels = _bfs_levels(indptr, indices, seeds, hops)
        for v in seeds:
            want[v] += 1
        for l in range(hops):
            for d in levels[l]:
                np.add.at(want, indices[indptr[d]: indptr[d + 1]], 1)
    assert np.array_equal(counts, want)


def test_draw_counts_one_hop_expectation():
    """One hop: the expected count of v is its seed occurrences plus, over the seeds u that list v,
    (entries of v in u's list) x min(1, k / deg u) -- exact, since every position is kept with that
    probability."""
    indptr, indices = _graph(60, 400, 19)
    n = 60; k = 2; bs = 8
    train = np.arange(0, 24, dtype=np.int32)
    deg = np.diff(indptr)
    mean_want = np.zeros(n)
    for u in train:
        mean_want[u] += 1
        if deg[u]:
            np.add.at(mean_want, indices[indptr[u]: indptr[u + 1]], min(1.0, k / deg[u]))
    runs = 3000
    acc = np.zeros(n)
    for s in range(runs):
        c, _ = orc.presample_draws(indptr, indices, train, bs, (k,), 1, 1000 + s)
        acc += c
    mean = acc / runs
    sd = np.sqrt(np.maximum(mean_want, 1e-9) / runs) + 1e-9            # loose (variance <= mean)
    assert np.all(np.abs(mean - mean_want) < 5 * sd + 1e-12)
    assert np.all(mean[mean_want == 0] == 0)


def test_draw_counts_empty_training_set():
    indptr, indices = _graph()
    counts, draws = orc.presample_draws(indptr, indices, np.zeros(0, np.int32), 8, (3,), 1, 1)
    assert counts.sum() == 0 and draws == 0


# ----------------------------------------------------------------------------
# placement
# ----------------------------------------------------------------------------
def test_rank_matches_papers_worked_example():
    lines = [l.split() for l in open(os.path.join(GOLD, "rank_example.txt")) if not l.startswith("#")]
    counts = [int(x) for x in lines[0][1:]]; want = [int(x) for x in lines[1][1:]]
    rank, slot, n_hot = orc.place(counts, 16, 16 * 4)
    assert rank.tolist() == want and slot.tolist() == want and n_hot == 4
    rank, slot, n_hot = orc.place(counts, 16, 16 * 2 + 15)              # room for two rows
    assert n_hot == 2 and slot.tolist() == [-1, 0, -1, 1]


def test_rank_equals_stable_library_sort():
    rng = np.random.default_rng(23)
    for n in (1, 2, 1000, 50_000):
        counts = rng.integers(0, 7, n).astype(np.uint32)                # many ties
        order = np.argsort(-counts.astype(np.int64), kind="stable")     # count desc, id asc
        want = np.empty(n, np.int64); want[order] = np.arange(n)
        rank, slot, n_hot = orc.place(counts, 400, 400 * (n // 3) + 399)
        assert np.array_equal(rank, want)
        assert n_hot == n // 3
        hot = slot >= 0
        assert np.array_equal(slot[hot], rank[hot]) and hot.sum() == n_hot and np.all(rank[~hot] >= n_hot)
        assert sorted(slot[hot].tolist()) == list(range(n_hot))         # bijection onto the cache
        if 0 < n_hot < n:
            assert counts[hot].min() >= counts[~hot].max()


def test_budget_edges():
    counts = np.array([5, 0, 9, 9, 1], np.uint32)
    assert orc.place(counts, 512, 0)[1].tolist() == [-1] * 5
    assert orc.place(counts, 512, 511)[2] == 0
    assert orc.place(counts, 512, 512)[1].tolist() == [-1, -1, 0, -1, -1]   # tie: lower id first
    r, s, h = orc.place(counts, 512, 10**12)
    assert h == 5 and s.tolist() == r.tolist() == [2, 4, 0, 1, 3]
    assert orc.place(np.zeros(4, np.uint32), 16, 32)[1].tolist() == [0, 1, -1, -1]  # zero counts fill by id


# ----------------------------------------------------------------------------
# gather
# ----------------------------------------------------------------------------
def test_gather_equals_fancy_indexing_for_any_budget():
    rng = np.random.default_rng(29)
    n, rb = 700, 400
    feat = rng.integers(0, 256, (n, rb), dtype=np.uint8)
    counts = rng.integers(0, 50, n).astype(np.uint32)
    ids = rng.integers(0, n, 5000).astype(np.int32)                    # with repeats
    for budget_rows in (0, 1, 70, 350, n, 2 * n):
        rank, slot, n_hot = orc.place(counts, rb, budget_rows * rb)
        cache = orc.fill_cache(feat, slot, n_hot)
        assert np.array_equal(cache[slot[slot >= 0]], feat[slot >= 0])  # cache rows byte-equal
        out, hit, miss = orc.gather(feat, cache, slot, ids)
        assert np.array_equal(out, feat[ids])                          # transparent to the model
        assert hit == int((slot[ids] >= 0).sum()) and hit + miss == len(ids)
    # the copy really comes from the cache for hot rows: poison the host copy of hot rows
    rank, slot, n_hot = orc.place(counts, rb, 100 * rb)
    cache = orc.fill_cache(feat, slot, n_hot)
    poisoned = feat.copy(); poisoned[slot >= 0] ^= 0xFF
    out, _, _ = orc.gather(poisoned, cache, slot, ids)
    assert np.array_equal(out, feat[ids])
    out, hit, miss = orc.gather(feat, cache, slot, np.zeros(0, np.int32))
    assert out.shape == (0, rb) and hit == 0 and miss == 0
