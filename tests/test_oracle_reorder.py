"""Pins of the oracle's graph / feature reordering (Alg. 2) and boundary gather."""
import os

import numpy as np
import scipy.sparse as sp

from oracle import oracle as orc
from paper_2111_05894_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold():
    d = {}
    for line in open(os.path.join(GOLD, "reorder_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        d[k] = np.array([int(x) for x in v])
    return d


def test_reorder_hand_worked_example():
    g = _gold()
    nd_new, edg_new = orc.reorder_graph(g["nd"], g["edg"], g["srt_idx"])
    assert nd_new.tolist() == g["nd_new"].tolist()
    assert edg_new.tolist() == g["edg_new"].tolist()


def _edges(indptr, indices):
    dst = np.repeat(np.arange(len(indptr) - 1), np.diff(indptr))
    return dst, indices


def test_reorder_is_a_relabelling():
    indptr, indices = synth.small_graph(500, 6000, 31)
    rng = np.random.default_rng(1)
    rank = rng.permutation(500).astype(np.int32)
    nd_new, edg_new = orc.reorder_graph(indptr, indices, rank)
    order = np.empty(500, np.int64); order[rank] = np.arange(500)
    # degrees follow their nodes; list order is kept, values renamed
    assert np.array_equal(np.diff(nd_new), np.diff(indptr)[order])
    for r in (0, 1, 17, 499):
        v = order[r]
        assert np.array_equal(edg_new[nd_new[r]: nd_new[r + 1]], rank[indices[indptr[v]: indptr[v + 1]]])
    # same edge set under the renaming
    d0, s0 = _edges(indptr, indices); d1, s1 = _edges(nd_new, edg_new)
    a = set(zip(rank[d0].tolist(), rank[s0].tolist())); b = set(zip(d1.tolist(), s1.tolist()))
    assert a == b and len(b) == len(indices)
    # library routine: P A P^T of the adjacency matrix
    A = sp.csr_matrix((np.ones(len(indices)), indices.copy(), indptr.copy()), shape=(500, 500))
    B = A[order][:, order]
    B.sort_indices()
    Bn = sp.csr_matrix((np.ones(len(edg_new)), edg_new.copy(), nd_new.copy()), shape=(500, 500)); Bn.sort_indices()
    assert np.array_equal(B.indptr, Bn.indptr) and np.array_equal(B.indices, Bn.indices)
    # identity and round trip
    i_nd, i_edg = orc.reorder_graph(indptr, indices, np.arange(500, dtype=np.int32))
    assert np.array_equal(i_nd, indptr) and np.array_equal(i_edg, indices)
    back_nd, back_edg = orc.reorder_graph(nd_new, edg_new, order.astype(np.int32))
    assert np.array_equal(back_nd, indptr) and np.array_equal(back_edg, indices)


def test_rows_follow_their_nodes_and_boundary_gather():
    rng = np.random.default_rng(2)
    n, rb = 300, 48
    feat = rng.integers(0, 256, (n, rb), dtype=np.uint8)
    counts = rng.integers(0, 9, n).astype(np.uint32)
    rank, _, _ = orc.place(counts, rb, 0)
    new = orc.reorder_rows(feat, rank)
    order = np.argsort(rank)
    assert np.array_equal(new, feat[order])                         # numpy fancy indexing
    assert np.array_equal(new[rank], feat)
    # after reordering, "hot" is a prefix: the boundary gather equals the slot-map gather
    ids_old = rng.integers(0, n, 2000).astype(np.int32)
    ids_new = rank[ids_old]
    for boundary in (0, 1, 77, n):
        out, hit = orc.gather_boundary(new, boundary, ids_new)
        assert np.array_equal(out, feat[ids_old])
        _, slot, n_hot = orc.place(counts, rb, boundary * rb)
        cache = orc.fill_cache(feat, slot, n_hot)
        out2, hit2, _ = orc.gather(feat, cache, slot, ids_old)
        assert np.array_equal(out, out2) and hit == hit2 == int((ids_new < boundary).sum())
        assert np.array_equal(cache, new[:boundary])                # the cache is the table's prefix
