"""ctypes binding of the C-ABI library (``include/tier.h``), same names.

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory (tensors) and the stream.  There is no
fallback: a missing library raises at load time.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

MAX_LAYERS = 8
MAX_FANOUT = 64
MAX_BATCHES = 64
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtier.so")
_lib = None

EXPORTS = (
    "tier_host_alloc", "tier_host_free", "tier_blocks_bounds", "tier_create", "tier_destroy",
    "tier_presample", "tier_presample_range", "tier_presample_draws", "tier_prefetch", "tier_batch_seed", "tier_place", "tier_sample_minibatch",
    "tier_sample_minibatches", "tier_max_batches", "tier_set_segment_words",
    "tier_score_degree", "tier_score_wrpr", "tier_rank_scores", "tier_place_scores",
    "tier_rank", "tier_rank_static", "tier_reorder_graph", "tier_reorder_rows", "tier_relabel_ids", "tier_place_boundary",
    "tier_gather_features", "tier_gather_minibatches", "tier_set_gather_stream", "tier_set_gather_dedup", "tier_set_gather_split",
    "tier_strerror", "tier_last_hip_error",
)


class TierError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {_load().tier_strerror(status).decode()} ({status})")


class _Csr(C.Structure):
    _fields_ = [("n_nodes", C.c_int64), ("n_edges", C.c_int64), ("indptr", C.c_void_p),
                ("indptr_is_i64", C.c_int32), ("indices", C.c_void_p)]


class _Feat(C.Structure):
    _fields_ = [("host_rows", C.c_void_p), ("row_bytes", C.c_int64)]


class _Blocks(C.Structure):
    _fields_ = [("nodes", C.c_void_p), ("cap_nodes", C.c_int64),
                ("row_ptr", C.c_void_p * MAX_LAYERS), ("col", C.c_void_p * MAX_LAYERS),
                ("eid", C.c_void_p * MAX_LAYERS),
                ("cap_dst", C.c_int64 * MAX_LAYERS), ("cap_edges", C.c_int64 * MAX_LAYERS),
                ("n_nodes", C.c_int64 * (MAX_LAYERS + 1)), ("n_edges", C.c_int64 * MAX_LAYERS)]


class _BlocksBatch(C.Structure):
    _fields_ = [("nodes", C.c_void_p), ("nodes_stride", C.c_int64),
                ("row_ptr", C.c_void_p * MAX_LAYERS), ("col", C.c_void_p * MAX_LAYERS),
                ("eid", C.c_void_p * MAX_LAYERS),
                ("row_ptr_stride", C.c_int64 * MAX_LAYERS), ("edge_stride", C.c_int64 * MAX_LAYERS),
                ("n_nodes", C.POINTER(C.c_int64)), ("n_edges", C.POINTER(C.c_int64))]


class _Stats(C.Structure):
    _fields_ = [("hit_rows", C.c_int64), ("miss_rows", C.c_int64), ("link_rows", C.c_int64)]


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2111_05894_amd.build`")
        lib = C.CDLL(LIB_PATH)
        i64p = C.POINTER(C.c_int64); i32p = C.POINTER(C.c_int32)
        lib.tier_host_alloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t]
        lib.tier_host_free.argtypes = [C.c_void_p]
        lib.tier_blocks_bounds.argtypes = [C.c_int64, C.c_int64, i32p, C.c_int32, i64p, i64p]
        lib.tier_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(_Csr), C.POINTER(_Feat), C.c_void_p]
        lib.tier_destroy.argtypes = [C.c_void_p]; lib.tier_destroy.restype = None
        lib.tier_presample.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, i32p, C.c_int32, C.c_int32,
                                       C.c_uint64, C.c_void_p, i64p, i64p]
        lib.tier_presample_range.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, i32p, C.c_int32, C.c_int32,
                                             C.c_uint64, C.c_int64, C.c_int64, C.c_int32, C.c_void_p]
        lib.tier_prefetch.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        lib.tier_presample_draws.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, i32p, C.c_int32, C.c_int32,
                                             C.c_uint64, C.c_void_p, i64p]
        lib.tier_batch_seed.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]; lib.tier_batch_seed.restype = C.c_uint64
        lib.tier_place.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, i64p]
        lib.tier_sample_minibatch.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, i32p, C.c_int32, C.c_uint64,
                                              C.POINTER(_Blocks)]
        lib.tier_sample_minibatches.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, i32p,
                                                C.c_int32, C.POINTER(C.c_uint64), C.POINTER(_BlocksBatch)]
        lib.tier_max_batches.argtypes = [C.c_void_p]
        lib.tier_set_segment_words.argtypes = [C.c_void_p, C.c_int32]
        lib.tier_score_degree.argtypes = [C.c_void_p, C.c_void_p]
        lib.tier_score_wrpr.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_double, C.c_void_p]
        lib.tier_rank_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.tier_place_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, i64p]
        lib.tier_rank.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.tier_rank_static.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.tier_reorder_graph.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.tier_reorder_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        lib.tier_relabel_ids.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        lib.tier_place_boundary.argtypes = [C.c_void_p, C.c_uint64, i64p]
        lib.tier_gather_features.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(_Stats)]
        lib.tier_gather_minibatches.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, i64p, i64p, C.c_int32, C.c_void_p,
                                                C.POINTER(_Stats)]
        lib.tier_set_gather_dedup.argtypes = [C.c_void_p, C.c_int]
        lib.tier_set_gather_split.argtypes = [C.c_void_p, C.c_int32, C.c_int64]
        lib.tier_set_gather_stream.argtypes = [C.c_void_p, C.c_void_p]
        lib.tier_strerror.argtypes = [C.c_int]; lib.tier_strerror.restype = C.c_char_p
        lib.tier_last_hip_error.argtypes = [C.c_void_p]
        _lib = lib
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise TierError(rc, what)


def _fan(fanouts):
    arr = (C.c_int32 * len(fanouts))(*[int(k) for k in fanouts])
    return arr, len(fanouts)


def _dev(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")
    return C.c_void_p(t.data_ptr())


# ------------------------------------------------------------------------------
# pinned host memory
# ------------------------------------------------------------------------------
class HostTable:
    """A (n_rows, dim) feature table in pinned, GPU-mapped host memory obtained
    from tier_host_alloc; ``tensor`` is a CPU view of it."""

    def __init__(self, n_rows: int, dim: int, dtype: torch.dtype):
        self.nbytes = n_rows * dim * torch.empty((), dtype=dtype).element_size()
        p = C.c_void_p()
        _check(_load().tier_host_alloc(C.byref(p), self.nbytes), "tier_host_alloc")
        self.ptr = p.value
        buf = (C.c_uint8 * self.nbytes).from_address(self.ptr) if self.nbytes else bytearray()
        self.tensor = torch.frombuffer(buf, dtype=dtype).view(n_rows, dim) if self.nbytes else torch.empty((n_rows, dim), dtype=dtype)

    def free(self):
        if self.ptr:
            self.tensor = None
            _check(_load().tier_host_free(C.c_void_p(self.ptr)), "tier_host_free")
            self.ptr = None


def tier_host_alloc(n_rows: int, dim: int, dtype: torch.dtype) -> HostTable:
    return HostTable(n_rows, dim, dtype)


def tier_host_free(table: HostTable):
    table.free()


# ------------------------------------------------------------------------------
# context
# ------------------------------------------------------------------------------
class Context:
    def __init__(self, handle, indptr, indices, feat, row_bytes, dim, dtype):
        self.handle = handle
        self._keep = (indptr, indices, feat)        # the library references these
        self.n_nodes = indptr.numel() - 1
        self.row_bytes = row_bytes
        self.dim = dim
        self.dtype = dtype

    def close(self):
        if self.handle:
            _load().tier_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tier_create(indptr: torch.Tensor, indices: torch.Tensor, feat, stream=None) -> Context:
    """indptr (int32/int64) and indices (int32) on the GPU; feat: a pinned CPU tensor
    (n_nodes, dim) or a HostTable."""
    table = feat.tensor if isinstance(feat, HostTable) else feat
    if indptr.dtype not in (torch.int32, torch.int64):
        raise TypeError("indptr: int32 or int64")
    if not isinstance(feat, HostTable) and not (table.is_pinned() or table.is_cuda):
        raise TypeError("feat: pinned host memory (or device memory) required")
    if table.dim() != 2 or not table.is_contiguous():
        raise TypeError("feat: contiguous (n_nodes, dim)")
    csr = _Csr(indptr.numel() - 1, indices.numel(), _dev(indptr, indptr.dtype, "indptr"),
               1 if indptr.dtype == torch.int64 else 0, _dev(indices, torch.int32, "indices"))
    row_bytes = table.shape[1] * table.element_size()
    if table.shape[0] != csr.n_nodes:
        raise ValueError("feat rows != graph nodes")
    ft = _Feat(C.c_void_p(table.data_ptr()), row_bytes)
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    h = C.c_void_p()
    _check(_load().tier_create(C.byref(h), C.byref(csr), C.byref(ft), C.c_void_p(stream)), "tier_create")
    return Context(h, indptr, indices, feat, row_bytes, table.shape[1], table.dtype)


def tier_destroy(ctx: Context):
    ctx.close()


def tier_blocks_bounds(n_graph_nodes: int, n_seeds: int, fanouts):
    fan, L = _fan(fanouts)
    cn = (C.c_int64 * (MAX_LAYERS + 1))(); ce = (C.c_int64 * MAX_LAYERS)()
    _check(_load().tier_blocks_bounds(n_graph_nodes, n_seeds, fan, L, cn, ce), "tier_blocks_bounds")
    return list(cn[: L + 1]), list(ce[:L])


def tier_batch_seed(seed: int, epoch: int, batch: int) -> int:
    return int(_load().tier_batch_seed(seed, epoch, batch))


def tier_presample(ctx: Context, train_ids: torch.Tensor, batch_size: int, fanouts, epochs: int, seed: int,
                   counts: torch.Tensor = None, want_totals: bool = False):
    """Returns counts (uint32 values in an int32 tensor), or (counts, rows, edges)."""
    fan, L = _fan(fanouts)
    if counts is None:
        counts = torch.empty(ctx.n_nodes, dtype=torch.int32, device=train_ids.device)
    tr = C.c_int64(0); te = C.c_int64(0)
    rc = _load().tier_presample(ctx.handle, _dev(train_ids, torch.int32, "train_ids"), train_ids.numel(),
                                batch_size, fan, L, epochs, seed, _dev(counts, torch.int32, "counts"),
                                C.byref(tr) if want_totals else None, C.byref(te) if want_totals else None)
    _check(rc, "tier_presample")
    return (counts, tr.value, te.value) if want_totals else counts


def tier_presample_range(ctx: Context, train_ids: torch.Tensor, batch_size: int, fanouts, epochs: int, seed: int,
                         first_batch: int, n_batches: int, counts: torch.Tensor = None, accumulate: bool = False):
    """Counts of the mini-batches [first_batch, first_batch + n_batches) of every epoch; with
    ``accumulate`` they are added to ``counts``."""
    fan, L = _fan(fanouts)
    if counts is None:
        if accumulate:
            raise ValueError("accumulate needs counts")
        counts = torch.empty(ctx.n_nodes, dtype=torch.int32, device=train_ids.device)
    rc = _load().tier_presample_range(ctx.handle, _dev(train_ids, torch.int32, "train_ids"), train_ids.numel(),
                                      batch_size, fan, L, epochs, seed, first_batch, n_batches, 1 if accumulate else 0,
                                      _dev(counts, torch.int32, "counts"))
    _check(rc, "tier_presample_range")
    return counts


def tier_prefetch(ctx: Context, counts: torch.Tensor, max_rows: int):
    _check(_load().tier_prefetch(ctx.handle, _dev(counts, torch.int32, "counts"), max_rows), "tier_prefetch")


def tier_presample_draws(ctx: Context, train_ids: torch.Tensor, batch_size: int, fanouts, epochs: int, seed: int,
                         counts: torch.Tensor = None, want_total: bool = False):
    """Returns counts (uint32 values in an int32 tensor), or (counts, seeds + sampled edges)."""
    fan, L = _fan(fanouts)
    if counts is None:
        counts = torch.empty(ctx.n_nodes, dtype=torch.int32, device=train_ids.device)
    td = C.c_int64(0)
    rc = _load().tier_presample_draws(ctx.handle, _dev(train_ids, torch.int32, "train_ids"), train_ids.numel(),
                                      batch_size, fan, L, epochs, seed, _dev(counts, torch.int32, "counts"),
                                      C.byref(td) if want_total else None)
    _check(rc, "tier_presample_draws")
    return (counts, td.value) if want_total else counts


def tier_place(ctx: Context, counts: torch.Tensor, budget_bytes: int, want_slot_map: bool = True):
    slot = torch.empty(ctx.n_nodes, dtype=torch.int32, device=counts.device) if want_slot_map else None
    n_hot = C.c_int64(0)
    rc = _load().tier_place(ctx.handle, _dev(counts, torch.int32, "counts"), budget_bytes,
                            _dev(slot, torch.int32, "slot_map") if want_slot_map else None, C.byref(n_hot))
    _check(rc, "tier_place")
    return slot, n_hot.value


def tier_score_degree(ctx: Context, device="cuda:0") -> torch.Tensor:
    deg = torch.empty(ctx.n_nodes, dtype=torch.int32, device=device)
    _check(_load().tier_score_degree(ctx.handle, _dev(deg, torch.int32, "degree")), "tier_score_degree")
    return deg


def tier_score_wrpr(ctx: Context, train_ids: torch.Tensor, iterations: int = 5, damp: float = 0.85) -> torch.Tensor:
    score = torch.empty(ctx.n_nodes, dtype=torch.float64, device=train_ids.device)
    _check(_load().tier_score_wrpr(ctx.handle, _dev(train_ids, torch.int32, "train_ids"), train_ids.numel(),
                                   iterations, damp, _dev(score, torch.float64, "score")), "tier_score_wrpr")
    return score


def tier_rank_scores(ctx: Context, scores: torch.Tensor):
    rank = torch.empty(ctx.n_nodes, dtype=torch.int32, device=scores.device)
    order = torch.empty_like(rank)
    _check(_load().tier_rank_scores(ctx.handle, _dev(scores, torch.float64, "scores"),
                                    _dev(rank, torch.int32, "rank"), _dev(order, torch.int32, "order")),
           "tier_rank_scores")
    return rank, order


def tier_place_scores(ctx: Context, scores: torch.Tensor, budget_bytes: int, want_slot_map: bool = True):
    slot = torch.empty(ctx.n_nodes, dtype=torch.int32, device=scores.device) if want_slot_map else None
    n_hot = C.c_int64(0)
    rc = _load().tier_place_scores(ctx.handle, _dev(scores, torch.float64, "scores"), budget_bytes,
                                   _dev(slot, torch.int32, "slot_map") if want_slot_map else None, C.byref(n_hot))
    _check(rc, "tier_place_scores")
    return slot, n_hot.value


def tier_rank(ctx: Context, counts: torch.Tensor):
    """Returns (rank, order): rank[v] = new id of v, order[r] = node of rank r."""
    rank = torch.empty(ctx.n_nodes, dtype=torch.int32, device=counts.device)
    order = torch.empty_like(rank)
    _check(_load().tier_rank(ctx.handle, _dev(counts, torch.int32, "counts"), _dev(rank, torch.int32, "rank"),
                             _dev(order, torch.int32, "order")), "tier_rank")
    return rank, order


RANK_STATIC_MAX_NODES = 1 << 20


def tier_rank_static(counts: torch.Tensor, rank: torch.Tensor = None, order: torch.Tensor = None, stream=None):
    """tier_rank without a context and without any allocation inside the library (see tier.h).
    The outputs are the caller's: pass them in to keep the call itself free of allocations."""
    n = counts.numel()
    if rank is None:
        rank = torch.empty(n, dtype=torch.int32, device=counts.device)
    if order is None:
        order = torch.empty(n, dtype=torch.int32, device=counts.device)
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(_load().tier_rank_static(_dev(counts, torch.int32, "counts"), n, _dev(rank, torch.int32, "rank"),
                                    _dev(order, torch.int32, "order"), C.c_void_p(stream)), "tier_rank_static")
    return rank, order


def tier_reorder_graph(ctx: Context, rank: torch.Tensor, order: torch.Tensor):
    """Alg. 2 on the context's graph: returns (indptr_new, indices_new)."""
    indptr, indices, _ = ctx._keep
    indptr_new = torch.empty_like(indptr); indices_new = torch.empty_like(indices)
    _check(_load().tier_reorder_graph(ctx.handle, _dev(rank, torch.int32, "rank"), _dev(order, torch.int32, "order"),
                                      C.c_void_p(indptr_new.data_ptr()), C.c_void_p(indices_new.data_ptr())),
           "tier_reorder_graph")
    return indptr_new, indices_new


def tier_reorder_rows(ctx: Context, rank: torch.Tensor, rows_new):
    """rows_new: a HostTable or a pinned / device tensor of the table's shape."""
    t = rows_new.tensor if isinstance(rows_new, HostTable) else rows_new
    if t.numel() * t.element_size() != ctx.n_nodes * ctx.row_bytes or not t.is_contiguous():
        raise TypeError("rows_new: contiguous, same size as the feature table")
    _check(_load().tier_reorder_rows(ctx.handle, _dev(rank, torch.int32, "rank"), C.c_void_p(t.data_ptr())),
           "tier_reorder_rows")
    return rows_new


def tier_relabel_ids(ctx: Context, rank: torch.Tensor, ids: torch.Tensor) -> torch.Tensor:
    out = torch.empty_like(ids)
    _check(_load().tier_relabel_ids(ctx.handle, _dev(rank, torch.int32, "rank"), _dev(ids, torch.int32, "ids"),
                                    ids.numel(), C.c_void_p(out.data_ptr())), "tier_relabel_ids")
    return out


def tier_place_boundary(ctx: Context, budget_bytes: int) -> int:
    n_hot = C.c_int64(0)
    _check(_load().tier_place_boundary(ctx.handle, budget_bytes, C.byref(n_hot)), "tier_place_boundary")
    return n_hot.value


class Blocks:
    """Device buffers of one mini-batch's blocks, sized to the upper bounds, plus
    the sizes the last tier_sample_minibatch call wrote."""

    def __init__(self, n_graph_nodes: int, n_seeds: int, fanouts, device):
        self.fanouts = tuple(int(k) for k in fanouts)
        L = len(self.fanouts)
        cn, ce = tier_blocks_bounds(n_graph_nodes, n_seeds, self.fanouts)
        self.cap_nodes, self.cap_edges = cn, ce
        self.nodes = torch.empty(max(cn[L], 1), dtype=torch.int32, device=device)
        self.row_ptr = [torch.empty(cn[l] + 1, dtype=torch.int32, device=device) for l in range(L)]
        self.col = [torch.empty(max(ce[l], 1), dtype=torch.int32, device=device) for l in range(L)]
        self.eid = [torch.empty(max(ce[l], 1), dtype=torch.int64, device=device) for l in range(L)]
        self.n_nodes = [0] * (L + 1)
        self.n_edges = [0] * L
        s = _Blocks()
        s.nodes = self.nodes.data_ptr(); s.cap_nodes = cn[L]
        for l in range(L):
            s.row_ptr[l] = self.row_ptr[l].data_ptr(); s.col[l] = self.col[l].data_ptr()
            s.eid[l] = self.eid[l].data_ptr(); s.cap_dst[l] = cn[l]; s.cap_edges[l] = ce[l]
        self._c = s

    def frontier(self, l: int = None) -> torch.Tensor:
        l = len(self.fanouts) if l is None else l
        return self.nodes[: self.n_nodes[l]]


def tier_sample_minibatch(ctx: Context, seeds: torch.Tensor, fanouts, seed: int, blocks: Blocks = None) -> Blocks:
    if blocks is None:
        blocks = Blocks(ctx.n_nodes, seeds.numel(), fanouts, seeds.device)
    fan, L = _fan(fanouts)
    rc = _load().tier_sample_minibatch(ctx.handle, _dev(seeds, torch.int32, "seeds"), seeds.numel(), fan, L, seed,
                                       C.byref(blocks._c))
    _check(rc, "tier_sample_minibatch")
    blocks.n_nodes = list(blocks._c.n_nodes[: L + 1])
    blocks.n_edges = list(blocks._c.n_edges[:L])
    return blocks


class BlocksBatch:
    """Device buffers for the blocks of up to ``n_batches`` mini-batches sampled by one
    call: every array has a leading mini-batch dimension, sized to the upper bounds."""

    def __init__(self, n_graph_nodes: int, batch_size: int, fanouts, n_batches: int, device):
        self.fanouts = tuple(int(k) for k in fanouts)
        self.n_batches = n_batches
        L = len(self.fanouts)
        cn, ce = tier_blocks_bounds(n_graph_nodes, batch_size, self.fanouts)
        self.cap_nodes, self.cap_edges = cn, ce
        B = n_batches
        self.nodes = torch.empty((B, max(cn[L], 1)), dtype=torch.int32, device=device)
        self.row_ptr = [torch.empty((B, cn[l] + 1), dtype=torch.int32, device=device) for l in range(L)]
        self.col = [torch.empty((B, max(ce[l], 1)), dtype=torch.int32, device=device) for l in range(L)]
        self.eid = [torch.empty((B, max(ce[l], 1)), dtype=torch.int64, device=device) for l in range(L)]
        self._nn = (C.c_int64 * (B * (MAX_LAYERS + 1)))()
        self._ne = (C.c_int64 * (B * MAX_LAYERS))()
        self.n_nodes = [[0] * (L + 1) for _ in range(B)]
        self.n_edges = [[0] * L for _ in range(B)]
        s = _BlocksBatch()
        s.nodes = self.nodes.data_ptr(); s.nodes_stride = self.nodes.shape[1]
        for l in range(L):
            s.row_ptr[l] = self.row_ptr[l].data_ptr(); s.col[l] = self.col[l].data_ptr()
            s.eid[l] = self.eid[l].data_ptr()
            s.row_ptr_stride[l] = self.row_ptr[l].shape[1]; s.edge_stride[l] = self.col[l].shape[1]
        s.n_nodes = C.cast(self._nn, C.POINTER(C.c_int64)); s.n_edges = C.cast(self._ne, C.POINTER(C.c_int64))
        self._c = s

    def frontier(self, b: int, l: int = None) -> torch.Tensor:
        l = len(self.fanouts) if l is None else l
        return self.nodes[b, : self.n_nodes[b][l]]


def tier_max_batches(ctx: Context) -> int:
    return int(_load().tier_max_batches(ctx.handle))


def tier_set_segment_words(ctx: Context, words: int):
    """Layout of the sampler's scratch: 1 or 32 bitmap words per segment (see tier.h)."""
    _check(_load().tier_set_segment_words(ctx.handle, words), "tier_set_segment_words")


def tier_sample_minibatches(ctx: Context, seeds: torch.Tensor, batch_size: int, batch_seeds, fanouts,
                            blocks: BlocksBatch = None) -> BlocksBatch:
    """Mini-batch s takes seeds[s*batch_size:(s+1)*batch_size] and samples with batch_seeds[s]."""
    B = len(batch_seeds)
    if blocks is None:
        blocks = BlocksBatch(ctx.n_nodes, batch_size, fanouts, B, seeds.device)
    if B > blocks.n_batches:
        raise ValueError("more mini-batches than the buffers hold")
    fan, L = _fan(fanouts)
    bs = (C.c_uint64 * B)(*[int(x) for x in batch_seeds])
    rc = _load().tier_sample_minibatches(ctx.handle, _dev(seeds, torch.int32, "seeds"), seeds.numel(), batch_size, B,
                                         fan, L, bs, C.byref(blocks._c))
    _check(rc, "tier_sample_minibatches")
    for s in range(B):
        blocks.n_nodes[s] = list(blocks._nn[s * (MAX_LAYERS + 1): s * (MAX_LAYERS + 1) + L + 1])
        blocks.n_edges[s] = list(blocks._ne[s * MAX_LAYERS: s * MAX_LAYERS + L])
    return blocks


def tier_gather_minibatches(ctx: Context, blocks: "BlocksBatch", n_batches: int, out: torch.Tensor = None,
                            want_stats: bool = False, first_batch: int = 0):
    """Rows of the final frontiers of n_batches mini-batches of ``blocks``, from mini-batch first_batch
    on, in one launch, packed back to back.  Returns (out, row_offsets) or (out, row_offsets, hit, miss)."""
    L = len(blocks.fanouts)
    if first_batch < 0 or n_batches < 1 or first_batch + n_batches > blocks.n_batches:
        raise ValueError("mini-batches outside the blocks")
    n_rows = [blocks.n_nodes[first_batch + b][L] for b in range(n_batches)]
    offs = [0] * n_batches
    for b in range(1, n_batches):
        offs[b] = offs[b - 1] + n_rows[b - 1]
    total = offs[-1] + n_rows[-1]
    if out is None:
        out = torch.empty((total, ctx.dim), dtype=ctx.dtype, device=blocks.nodes.device)
    if not (out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= total * ctx.row_bytes):
        raise TypeError("out: contiguous device tensor of sum(n_rows) * row_bytes bytes")
    nr = (C.c_int64 * n_batches)(*n_rows); of = (C.c_int64 * n_batches)(*offs)
    st = _Stats()
    rc = _load().tier_gather_minibatches(ctx.handle, C.c_void_p(blocks.nodes[first_batch].data_ptr()), blocks.nodes.shape[1],
                                         nr, of, n_batches, C.c_void_p(out.data_ptr()), C.byref(st) if want_stats else None)
    _check(rc, "tier_gather_minibatches")
    if want_stats:
        ctx.last_link_rows = st.link_rows
    return (out, offs, st.hit_rows, st.miss_rows) if want_stats else (out, offs)


def tier_set_gather_dedup(ctx: Context, on: bool):
    """Fetch every distinct cold row of a gather call over the host link once (see tier.h)."""
    _check(_load().tier_set_gather_dedup(ctx.handle, 1 if on else 0), "tier_set_gather_dedup")
    ctx.last_link_rows = None


def tier_set_gather_split(ctx: Context, link_blocks: int, min_rows: int = 0):
    """Copy the cold rows of every gather call of >= min_rows rows with a launch of link_blocks
    blocks of its own, beside the full-width launch for the hot rows (see tier.h); 0 = one launch."""
    _check(_load().tier_set_gather_split(ctx.handle, link_blocks, min_rows), "tier_set_gather_split")


def tier_set_gather_stream(ctx: Context, stream=None):
    """stream: a torch.cuda.Stream (kept alive by the context) or None for the context's own."""
    ctx._gather_stream = stream
    _check(_load().tier_set_gather_stream(ctx.handle, C.c_void_p(stream.cuda_stream if stream is not None else 0)),
           "tier_set_gather_stream")


def tier_gather_features(ctx: Context, ids: torch.Tensor, out: torch.Tensor = None, want_stats: bool = False):
    n = ids.numel()
    if out is None:
        out = torch.empty((n, ctx.dim), dtype=ctx.dtype, device=ids.device)
    if not (out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= n * ctx.row_bytes):
        raise TypeError("out: contiguous device tensor of n * row_bytes bytes")
    st = _Stats()
    rc = _load().tier_gather_features(ctx.handle, _dev(ids, torch.int32, "ids"), n, C.c_void_p(out.data_ptr()),
                                      C.byref(st) if want_stats else None)
    _check(rc, "tier_gather_features")
    if want_stats:
        ctx.last_link_rows = st.link_rows
    return (out, st.hit_rows, st.miss_rows) if want_stats else out
