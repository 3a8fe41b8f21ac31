"""ctypes front end of the C oracle (``tier_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays into the plain-C routines and returns numpy arrays; all
of the method's arithmetic lives in the C file.  ``build()`` compiles the C
file with gcc; every entry point builds on first use when the shared object is
missing or older than its source.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tier_oracle.c")
_LIB = os.path.join(_HERE, "libtier_oracle.so")
_lib = None

_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)
_u32p = C.POINTER(C.c_uint32)
_u8p = C.POINTER(C.c_uint8)


def build(force: bool = False) -> str:
    """Compile the oracle (plain C, -O2, no threads, no SIMD intrinsics)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                        "-ffp-contract=off", "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_bounded.restype = C.c_uint64
        _lib.orc_bounded.argtypes = [C.c_uint64, C.c_uint64]
        _lib.orc_batch_seed.restype = C.c_uint64
        _lib.orc_batch_seed.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        _lib.orc_philox4x32_10.restype = None
        _lib.orc_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        _lib.orc_draw_positions.restype = C.c_int
        _lib.orc_draw_positions.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_int64, C.c_int, _i64p]
        _lib.orc_sample_minibatch.restype = C.c_int
        _lib.orc_sample_minibatch.argtypes = [
            C.c_int64, _i64p, _i32p, _i32p, C.c_int64, _i32p, C.c_int, C.c_uint64,
            _i32p, _i32p, C.c_int64, _i32p, C.c_int64, _i32p, _i64p, C.c_int64, _i64p, _i64p]
        _lib.orc_presample.restype = C.c_int
        _lib.orc_presample.argtypes = [
            C.c_int64, _i64p, _i32p, _i32p, C.c_int64, C.c_int64, _i32p, C.c_int, C.c_int, C.c_uint64,
            C.c_int64, C.c_int64, _i32p, _i32p, C.c_int64, _u32p, _i64p, _i64p]
        _lib.orc_presample_draws.restype = C.c_int
        _lib.orc_presample_draws.argtypes = [
            C.c_int64, _i64p, _i32p, _i32p, C.c_int64, C.c_int64, _i32p, C.c_int, C.c_int, C.c_uint64,
            C.c_int64, C.c_int64, _i32p, _i32p, C.c_int64, _i64p, C.c_int64, _u32p, _i64p]
        _lib.orc_place.restype = C.c_int
        _lib.orc_place.argtypes = [_u32p, C.c_int64, C.c_int64, C.c_uint64, _i32p, _i32p, _i64p]
        _lib.orc_fill_cache.restype = None
        _lib.orc_fill_cache.argtypes = [_u8p, C.c_int64, C.c_int64, _i32p, _u8p]
        _lib.orc_gather.restype = None
        _lib.orc_gather.argtypes = [_u8p, _u8p, _i32p, C.c_int64, _i32p, C.c_int64, _u8p, _i64p, _i64p]
        _lib.orc_reorder_graph.restype = None
        _lib.orc_reorder_graph.argtypes = [C.c_int64, _i64p, _i32p, _i32p, _i64p, _i32p]
        _lib.orc_reorder_rows.restype = None
        _lib.orc_reorder_rows.argtypes = [_u8p, C.c_int64, C.c_int64, _i32p, _u8p]
        _lib.orc_gather_boundary.restype = None
        _lib.orc_gather_boundary.argtypes = [_u8p, _u8p, C.c_int64, C.c_int64, _i32p, C.c_int64, _u8p, _i64p]
        _f64p = C.POINTER(C.c_double)
        _lib.orc_score_degree.restype = None
        _lib.orc_score_degree.argtypes = [C.c_int64, _i64p, _i32p, _u32p]
        _lib.orc_score_wrpr.restype = None
        _lib.orc_score_wrpr.argtypes = [C.c_int64, _i64p, _i32p, _i32p, C.c_int64, C.c_int, C.c_double, _f64p]
        _lib.orc_rank_scores.restype = C.c_int
        _lib.orc_rank_scores.argtypes = [_f64p, C.c_int64, _i32p]
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t)


def _as(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def philox4x32_10(ctr, key):
    c = _as(ctr, np.uint32); k = _as(key, np.uint32); o = np.zeros(4, np.uint32)
    _load().orc_philox4x32_10(_p(c, _u32p), _p(k, _u32p), _p(o, _u32p))
    return o


def bounded(r: int, m: int) -> int:
    return int(_load().orc_bounded(r, m))


def batch_seed(seed: int, epoch: int, batch: int) -> int:
    return int(_load().orc_batch_seed(seed, epoch, batch))


def draw_positions(seed: int, layer: int, node: int, d: int, k: int):
    pos = np.zeros(max(k, d if d <= k else k, 1), np.int64)
    n = _load().orc_draw_positions(seed, layer, node, d, k, _p(pos, _i64p))
    return pos[:n].copy()


def frontier_bounds(n_seeds: int, fanouts, n_graph: int):
    """Upper bounds of |frontier_l| (l = 0..L) and of the edge count per hop."""
    nn = [min(n_seeds, n_graph)]
    ne = []
    for k in fanouts:
        ne.append(nn[-1] * k)
        nn.append(min(n_graph, nn[-1] * (1 + k)))
    return nn, ne


def sample_minibatch(indptr, indices, seeds, fanouts, seed, local_idx=None, want_blocks=True):
    indptr = _as(indptr, np.int64); indices = _as(indices, np.int32)
    seeds = _as(seeds, np.int32); fan = _as(fanouts, np.int32)
    n_graph = indptr.shape[0] - 1
    L = fan.shape[0]
    if local_idx is None:
        local_idx = np.full(n_graph, -1, np.int32)
    nn_b, ne_b = frontier_bounds(seeds.shape[0], fan.tolist(), n_graph)
    nodes = np.empty(max(nn_b[-1], 1), np.int32)
    cap_rp = sum(x + 1 for x in nn_b[:-1]); cap_e = max(sum(ne_b), 1)
    if want_blocks:
        rp = np.empty(max(cap_rp, 1), np.int32); col = np.empty(cap_e, np.int32); eid = np.empty(cap_e, np.int64)
        rp_p, col_p, eid_p = _p(rp, _i32p), _p(col, _i32p), _p(eid, _i64p)
    else:
        rp_p = col_p = eid_p = None
    n_nodes = np.zeros(L + 1, np.int64); n_edges = np.zeros(L, np.int64)
    rc = _load().orc_sample_minibatch(n_graph, _p(indptr, _i64p), _p(indices, _i32p), _p(seeds, _i32p),
                                      seeds.shape[0], _p(fan, _i32p), L, seed, _p(local_idx, _i32p),
                                      _p(nodes, _i32p), nodes.shape[0], rp_p, cap_rp, col_p, eid_p, cap_e,
                                      _p(n_nodes, _i64p), _p(n_edges, _i64p))
    if rc:
        raise RuntimeError("oracle capacity error")
    out = {"nodes": nodes[: n_nodes[L]].copy(), "n_nodes": n_nodes, "n_edges": n_edges}
    if want_blocks:
        out["row_ptr"], out["col"], out["eid"] = [], [], []
        rb = eb = 0
        for l in range(L):
            out["row_ptr"].append(rp[rb: rb + n_nodes[l] + 1].copy())
            out["col"].append(col[eb: eb + n_edges[l]].copy())
            out["eid"].append(eid[eb: eb + n_edges[l]].copy())
            rb += int(n_nodes[l]) + 1; eb += int(n_edges[l])
    return out


def presample(indptr, indices, train_ids, batch_size, fanouts, epochs, seed, threads=1):
    """Access counts.  ``threads`` > 1 splits the batches over host threads, each
    running the same single-threaded C routine on its share; the shares add."""
    indptr = _as(indptr, np.int64); indices = _as(indices, np.int32)
    train_ids = _as(train_ids, np.int32); fan = _as(fanouts, np.int32)
    n_graph = indptr.shape[0] - 1
    n_train = train_ids.shape[0]
    n_batches = (n_train + batch_size - 1) // batch_size
    nn_b, _ = frontier_bounds(min(batch_size, n_train), fan.tolist(), n_graph)
    lib = _load()

    def work(lo, hi):
        local_idx = np.full(n_graph, -1, np.int32)
        scratch = np.empty(max(nn_b[-1], 1), np.int32)
        counts = np.zeros(n_graph, np.uint32)
        tot = C.c_int64(0); edg = C.c_int64(0)
        rc = lib.orc_presample(n_graph, _p(indptr, _i64p), _p(indices, _i32p), _p(train_ids, _i32p), n_train,
                               batch_size, _p(fan, _i32p), fan.shape[0], epochs, seed, lo, hi,
                               _p(local_idx, _i32p), _p(scratch, _i32p), scratch.shape[0],
                               _p(counts, _u32p), C.byref(tot), C.byref(edg))
        if rc:
            raise RuntimeError("oracle capacity error")
        return counts, tot.value, edg.value

    threads = max(1, min(threads, n_batches if n_batches else 1))
    if threads == 1:
        return work(0, n_batches)
    cuts = [n_batches * t // threads for t in range(threads + 1)]
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda t: work(cuts[t], cuts[t + 1]), range(threads)))
    counts = parts[0][0]
    for c, _, _ in parts[1:]:
        counts += c
    return counts, sum(p[1] for p in parts), sum(p[2] for p in parts)


def presample_draws(indptr, indices, train_ids, batch_size, fanouts, epochs, seed, threads=1):
    """Counts of the other reading: one per seed and one per sampled edge's source.  Returns
    (counts, number of seeds + sampled edges); ``threads`` as in presample."""
    indptr = _as(indptr, np.int64); indices = _as(indices, np.int32)
    train_ids = _as(train_ids, np.int32); fan = _as(fanouts, np.int32)
    n_graph = indptr.shape[0] - 1
    n_train = train_ids.shape[0]
    n_batches = (n_train + batch_size - 1) // batch_size
    nn_b, ne_b = frontier_bounds(min(batch_size, n_train), fan.tolist(), n_graph)
    lib = _load()

    def work(lo, hi):
        local_idx = np.full(n_graph, -1, np.int32)
        scratch = np.empty(max(nn_b[-1], 1), np.int32)
        eids = np.empty(max(sum(ne_b), 1), np.int64)
        counts = np.zeros(n_graph, np.uint32)
        tot = C.c_int64(0)
        rc = lib.orc_presample_draws(n_graph, _p(indptr, _i64p), _p(indices, _i32p), _p(train_ids, _i32p), n_train,
                                     batch_size, _p(fan, _i32p), fan.shape[0], epochs, seed, lo, hi,
                                     _p(local_idx, _i32p), _p(scratch, _i32p), scratch.shape[0],
                                     _p(eids, _i64p), eids.shape[0], _p(counts, _u32p), C.byref(tot))
        if rc:
            raise RuntimeError("oracle capacity error")
        return counts, tot.value

    threads = max(1, min(threads, n_batches if n_batches else 1))
    if threads == 1:
        return work(0, n_batches)
    cuts = [n_batches * t // threads for t in range(threads + 1)]
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda t: work(cuts[t], cuts[t + 1]), range(threads)))
    counts = parts[0][0]
    for c, _ in parts[1:]:
        counts += c
    return counts, sum(p[1] for p in parts)


def place(counts, row_bytes: int, budget_bytes: int):
    counts = _as(counts, np.uint32)
    n = counts.shape[0]
    rank = np.empty(n, np.int32); slot = np.empty(n, np.int32); n_hot = C.c_int64(0)
    rc = _load().orc_place(_p(counts, _u32p), n, row_bytes, budget_bytes, _p(rank, _i32p), _p(slot, _i32p),
                           C.byref(n_hot))
    if rc:
        raise MemoryError
    return rank, slot, n_hot.value


def fill_cache(feat_bytes, slot, n_hot: int):
    """feat_bytes: uint8 array (N, row_bytes)."""
    assert feat_bytes.dtype == np.uint8 and feat_bytes.flags.c_contiguous
    n, rb = feat_bytes.shape
    cache = np.zeros((n_hot, rb), np.uint8)
    slot = _as(slot, np.int32)
    _load().orc_fill_cache(_p(feat_bytes, _u8p), n, rb, _p(slot, _i32p), _p(cache, _u8p))
    return cache


def gather(feat_bytes, cache, slot, ids):
    assert feat_bytes.dtype == np.uint8 and feat_bytes.flags.c_contiguous
    n, rb = feat_bytes.shape
    ids = _as(ids, np.int32); slot = _as(slot, np.int32)
    cache = np.ascontiguousarray(cache, np.uint8)
    out = np.empty((ids.shape[0], rb), np.uint8)
    hit = C.c_int64(0); miss = C.c_int64(0)
    _load().orc_gather(_p(feat_bytes, _u8p), _p(cache, _u8p), _p(slot, _i32p), rb, _p(ids, _i32p),
                       ids.shape[0], _p(out, _u8p), C.byref(hit), C.byref(miss))
    return out, hit.value, miss.value


def reorder_graph(indptr, indices, rank):
    """Alg. 2: returns (indptr_new int64, indices_new int32) with every node renamed to rank[node]."""
    indptr = _as(indptr, np.int64); indices = _as(indices, np.int32); rank = _as(rank, np.int32)
    n = indptr.shape[0] - 1
    nd_new = np.zeros(n + 1, np.int64); edg_new = np.empty(max(indices.shape[0], 1), np.int32)
    _load().orc_reorder_graph(n, _p(indptr, _i64p), _p(indices, _i32p), _p(rank, _i32p), _p(nd_new, _i64p),
                              _p(edg_new, _i32p))
    return nd_new, edg_new[: indices.shape[0]]


def reorder_rows(feat_bytes, rank):
    assert feat_bytes.dtype == np.uint8 and feat_bytes.flags.c_contiguous
    rank = _as(rank, np.int32)
    out = np.empty_like(feat_bytes)
    _load().orc_reorder_rows(_p(feat_bytes, _u8p), feat_bytes.shape[0], feat_bytes.shape[1], _p(rank, _i32p),
                             _p(out, _u8p))
    return out


def gather_boundary(feat_bytes_reordered, boundary: int, ids):
    """Hot tensor = rows [0, boundary), cold tensor = the rest, as two separate arrays."""
    fb = feat_bytes_reordered
    hot = np.ascontiguousarray(fb[:boundary]); cold = np.ascontiguousarray(fb[boundary:])
    ids = _as(ids, np.int32)
    out = np.empty((ids.shape[0], fb.shape[1]), np.uint8)
    hit = C.c_int64(0)
    _load().orc_gather_boundary(_p(hot, _u8p), _p(cold, _u8p), boundary, fb.shape[1], _p(ids, _i32p), ids.shape[0],
                                _p(out, _u8p), C.byref(hit))
    return out, hit.value


def score_degree(indptr, indices):
    indptr = _as(indptr, np.int64); indices = _as(indices, np.int32)
    n = indptr.shape[0] - 1
    deg = np.zeros(n, np.uint32)
    _load().orc_score_degree(n, _p(indptr, _i64p), _p(indices, _i32p), _p(deg, _u32p))
    return deg


def score_wrpr(indptr, indices, train_ids, iters: int, damp: float):
    """Weighted reverse PageRank (Alg. 1); no training ids = plain reverse PageRank."""
    indptr = _as(indptr, np.int64); indices = _as(indices, np.int32); tid = _as(train_ids, np.int32)
    n = indptr.shape[0] - 1
    score = np.zeros(max(n, 1), np.float64)
    _load().orc_score_wrpr(n, _p(indptr, _i64p), _p(indices, _i32p), _p(tid, _i32p), tid.shape[0], iters, damp,
                           _p(score, C.POINTER(C.c_double)))
    return score[:n]


def rank_scores(score):
    score = _as(score, np.float64)
    rank = np.empty(score.shape[0], np.int32)
    if _load().orc_rank_scores(_p(score, C.POINTER(C.c_double)), score.shape[0], _p(rank, _i32p)):
        raise MemoryError
    return rank
