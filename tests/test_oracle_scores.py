"""Pins of the oracle's score functions (Sec. 3.1, Alg. 1) and real-valued ranking."""
import numpy as np
import scipy.sparse as sp

from oracle import oracle as orc
from paper_2111_05894_amd import synth


def test_degree_is_a_bincount():
    indptr, indices = synth.small_graph(400, 5000, 3)
    assert np.array_equal(orc.score_degree(indptr, indices), np.bincount(indices, minlength=400))
    assert orc.score_degree(np.zeros(5, np.int64), np.zeros(0, np.int32)).tolist() == [0, 0, 0, 0]


def _pull_matrix(indptr, indices):
    """M[u, v] = 1 when u -> v: row u of M sums over the nodes u targets."""
    n = len(indptr) - 1
    dst = np.repeat(np.arange(n), np.diff(indptr))
    return sp.csr_matrix((np.ones(len(indices)), (indices, dst)), shape=(n, n))


def test_wrpr_hand_worked():
    # edges 0->1, 0->2, 1->2 ; rows list sources: row1=[0], row2=[0,1]; N=3, train={2}, d=0.5, one round
    indptr = np.array([0, 0, 1, 3], np.int64); indices = np.array([0, 0, 1], np.int32)
    s = orc.score_wrpr(indptr, indices, [2], 1, 0.5)
    # init [1/3, 1/3, 1]; divide by in-degree [-,1,2] -> [1/3, 1/3, 1/2]
    # pull: node0 targets 1,2 -> 1/3+1/2 ; node1 targets 2 -> 1/2 ; node2 targets nothing -> 0
    want = np.array([1 / 6 + 0.5 * (1 / 3 + 1 / 2), 1 / 6 + 0.5 * 0.5, 1 / 6])
    assert np.allclose(s, want, rtol=0, atol=1e-15)
    assert np.allclose(orc.score_wrpr(indptr, indices, [2], 0, 0.5), [1 / 3, 1 / 3, 1.0])
    assert np.allclose(orc.score_wrpr(indptr, indices, [], 0, 0.5), [1 / 3] * 3)


def test_wrpr_equals_sparse_matrix_iteration():
    indptr, indices = synth.small_graph(600, 7000, 5)
    n = 600
    train = synth.train_set(n, 0.1, 9).numpy()
    M = _pull_matrix(indptr, indices)
    indeg = np.diff(indptr).astype(float)
    for d, iters, tid in ((0.85, 5, train), (0.5, 3, train[:1]), (0.85, 20, np.zeros(0, np.int32))):
        s = np.full(n, 1.0 / n)
        if len(tid):
            s[tid] *= n / len(tid)
        for _ in range(iters):
            s = np.where(indeg > 0, s / np.maximum(indeg, 1), s)
            s = (1 - d) / n + d * (M @ s)                     # library sparse matrix-vector product
        got = orc.score_wrpr(indptr, indices, tid, iters, d)
        assert np.allclose(got, s, rtol=1e-12, atol=0)


def test_wrpr_invariants():
    n = 50                                                    # directed cycle: every node equal, forever
    indptr = np.arange(n + 1, dtype=np.int64); indices = ((np.arange(n) + 1) % n).astype(np.int32)
    s = orc.score_wrpr(indptr, indices, [], 7, 0.85)
    assert np.allclose(s, 1.0 / n, rtol=1e-14)
    # mass: what a node holds is pulled once per incoming edge after the division, so one round maps
    # total mass m to (1-d) + d * (mass on nodes with incoming edges)
    indptr, indices = synth.small_graph(300, 2500, 8)
    indeg = np.diff(indptr)
    s0 = orc.score_wrpr(indptr, indices, [5, 6, 7], 0, 0.7)
    s1 = orc.score_wrpr(indptr, indices, [5, 6, 7], 1, 0.7)
    assert np.isclose(s1.sum(), 0.3 + 0.7 * s0[indeg > 0].sum(), rtol=1e-12)
    # the training weight lifts the labelled nodes' own standing and what they target... sources of
    # edges into a labelled node gain: a node that targets a labelled node scores above its twin
    assert s1.min() >= 0.3 / 300 - 1e-18


def test_rank_scores_is_a_stable_descending_sort():
    rng = np.random.default_rng(4)
    s = rng.choice([0.0, 0.25, 0.5, 1e-9, 3.0], 5000) + 0.0
    order = np.argsort(-s, kind="stable")
    want = np.empty(5000, np.int64); want[order] = np.arange(5000)
    assert np.array_equal(orc.rank_scores(s), want)
    assert orc.rank_scores([0.1, 0.4, 0.2, 0.3]).tolist() == [3, 0, 2, 1]      # the paper's example, as printed
