"""Seeded synthetic inputs: graphs, training sets and feature tables.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds none of the method's arithmetic (no sampling, counting,
placement or gather): only the recipe for inputs shaped like the paper's
workloads (Table 1: 10^8-node power-law graphs with 512 B - 4 KB feature rows).

Every random choice comes from one counter-based 64-bit mixer evaluated with
integer tensor ops, so a (seed, index) pair gives the same value on the CPU and
on the GPU.  Feature values use torch's seeded generators (their values only
have to make rows distinguishable; the path copies bytes).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

_M1 = -4658895280553007687    # 0xBF58476D1CE4E5B9 as signed 64-bit
_M2 = -7723592293110705685    # 0x94D049BB133111EB
_GOLD = -7046029254386353131  # 0x9E3779B97F4A7C15


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 lanes (wrapping arithmetic)."""
    z = x + _GOLD
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def hash_u32(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """32 uniform bits (as int64 in [0, 2^32)) for (seed, stream, idx)."""
    base = mix64(torch.tensor([seed * 1000003 + stream], dtype=torch.int64, device=idx.device))
    return _lsr(mix64(idx ^ base), 32)


def hash_u63(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    base = mix64(torch.tensor([seed * 1000003 + stream], dtype=torch.int64, device=idx.device))
    return _lsr(mix64(idx ^ base), 1)


def random_order(n: int, seed: int, stream: int, device) -> torch.Tensor:
    """A seeded permutation of 0..n-1 (argsort of per-index hashes)."""
    h = hash_u63(seed, stream, torch.arange(n, dtype=torch.int64, device=device))
    return torch.sort(h, stable=True).indices


def _rmat_pairs(n_nodes: int, idx: torch.Tensor, seed: int, attempt: int, abcd) -> tuple:
    scale = max(1, math.ceil(math.log2(n_nodes)))
    a, b, c, _ = abcd
    ta = int(a * 2**32); tb = int((a + b) * 2**32); tc = int((a + b + c) * 2**32)
    src = torch.zeros_like(idx); dst = torch.zeros_like(idx)
    for level in range(scale):
        u = hash_u32(seed, 64 * attempt + level, idx)
        # quadrants: [0,a) -> (0,0); [a,a+b) -> (0,1); [a+b,a+b+c) -> (1,0); rest -> (1,1)
        sbit = (u >= tb).to(torch.int64)
        dbit = (((u >= ta) & (u < tb)) | (u >= tc)).to(torch.int64)
        src = (src << 1) | sbit
        dst = (dst << 1) | dbit
    return src, dst


def _pairs_to_csr(n_nodes: int, src: torch.Tensor, dst: torch.Tensor, i64_offsets: bool):
    """Drop duplicates, key rows by destination, sort each row ascending."""
    key = torch.sort(dst * n_nodes + src).values
    key = torch.unique_consecutive(key)
    d = torch.div(key, n_nodes, rounding_mode="floor")
    indices = (key - d * n_nodes).to(torch.int32)
    deg = torch.bincount(d, minlength=n_nodes)
    indptr = torch.zeros(n_nodes + 1, dtype=torch.int64, device=key.device)
    torch.cumsum(deg, 0, out=indptr[1:])
    if not i64_offsets:
        assert int(indptr[-1]) < 2**31
        indptr = indptr.to(torch.int32)
    return indptr, indices


def rmat_csr(n_nodes: int, n_draws: int, seed: int, device="cpu", abcd=(0.57, 0.19, 0.19, 0.05),
             i64_offsets=True, chunk=1 << 26):
    """R-MAT graph (Chakrabarti et al. 2004) as a CSR keyed by destination.

    ``n_draws`` edges are drawn; a draw with an endpoint >= n_nodes or a self
    loop is redrawn (up to 8 times, then dropped).  Node ids are then relabelled
    through a seeded permutation so that hub nodes are not the low ids, duplicate
    edges are dropped, and row v lists the sources of the edges into v ascending.
    Returns (indptr, indices) as tensors on ``device``.
    """
    dev = torch.device(device)
    srcs, dsts = [], []
    for lo in range(0, n_draws, chunk):
        idx = torch.arange(lo, min(n_draws, lo + chunk), dtype=torch.int64, device=dev)
        for attempt in range(8):
            s, d = _rmat_pairs(n_nodes, idx, seed, attempt, abcd)
            ok = (s < n_nodes) & (d < n_nodes) & (s != d)
            srcs.append(s[ok]); dsts.append(d[ok])
            idx = idx[~ok]
            if idx.numel() == 0:
                break
    src = torch.cat(srcs); dst = torch.cat(dsts)
    del srcs, dsts
    perm = random_order(n_nodes, seed, 9001, dev)
    src = perm[src]; dst = perm[dst]
    return _pairs_to_csr(n_nodes, src, dst, i64_offsets)


def erdos_renyi_csr(n_nodes: int, n_draws: int, seed: int, device="cpu", i64_offsets=True):
    """G(n, M)-style graph: ``n_draws`` directed edges with independent uniform
    endpoints, self loops redrawn once then dropped, duplicates dropped."""
    dev = torch.device(device)
    idx = torch.arange(n_draws, dtype=torch.int64, device=dev)
    src = hash_u63(seed, 1, idx) % n_nodes
    dst = hash_u63(seed, 2, idx) % n_nodes
    bad = src == dst
    dst = torch.where(bad, hash_u63(seed, 3, idx) % n_nodes, dst)
    ok = src != dst
    return _pairs_to_csr(n_nodes, src[ok], dst[ok], i64_offsets)


def train_set(n_nodes: int, fraction: float, seed: int, device="cpu") -> torch.Tensor:
    """``round(fraction * n_nodes)`` distinct node ids in seeded random order (int32)."""
    n_train = int(round(fraction * n_nodes))
    return random_order(n_nodes, seed, 9002, torch.device(device))[:n_train].to(torch.int32)


def fill_features(out: torch.Tensor, dist: str, seed: int, device="cpu", chunk_rows=1 << 20):
    """Fill a (N, D) tensor (any device, e.g. pinned host) with U(-1,1) or N(0,1)
    values generated on ``device`` in row chunks."""
    dev = torch.device(device)
    g = torch.Generator(device=dev); g.manual_seed(seed)
    n, d = out.shape
    for lo in range(0, n, chunk_rows):
        hi = min(n, lo + chunk_rows)
        if dist == "uniform":
            x = torch.rand((hi - lo, d), generator=g, device=dev, dtype=torch.float32) * 2 - 1
        elif dist == "normal":
            x = torch.randn((hi - lo, d), generator=g, device=dev, dtype=torch.float32)
        else:
            raise ValueError(dist)
        out[lo:hi].copy_(x.to(out.dtype))
    return out


@dataclass(frozen=True)
class Workload:
    """One of the benchmark configurations (shapes follow the paper's Table 1
    datasets and its sampling fanouts; the graphs themselves are synthetic)."""
    name: str
    graph: str            # "rmat" | "er"
    n_nodes: int
    n_draws: int
    i64_offsets: bool
    dim: int
    dtype: str            # "float32" | "float16"
    dist: str             # "uniform" | "normal"
    train_fraction: float
    fanouts: tuple
    batch_size: int
    budget: object        # float fraction of feature bytes, or int bytes

    @property
    def row_bytes(self) -> int:
        return self.dim * (4 if self.dtype == "float32" else 2)

    @property
    def feature_bytes(self) -> int:
        return self.n_nodes * self.row_bytes

    def budget_bytes(self, fraction=None) -> int:
        b = self.budget if fraction is None else fraction
        if isinstance(b, float):
            return int(math.floor(b * self.feature_bytes))
        return int(b)


GRAPH_SEED = 2111
PRESAMPLE_SEED = 5894
EPOCH_SEED = 5895

WORKLOADS = {
    "cfg1": Workload("cfg1", "rmat", 1 << 17, 2_000_000, False, 128, "float32", "uniform", 0.10, (10, 5), 1024, 0.10),
    "cfg2": Workload("cfg2", "rmat", 2_400_000, 62_000_000, True, 100, "float32", "normal", 0.08, (15, 10, 5), 1024, 0.20),
    "cfg3": Workload("cfg3", "rmat", 111_000_000, 1_600_000_000, True, 128, "float32", "normal", 0.01, (15, 10, 5), 1024, 0.10),
    "cfg4": Workload("cfg4", "rmat", 60_000_000, 1_200_000_000, True, 768, "float16", "normal", 0.01, (25, 15), 1024, 16 * 2**30),
    "cfg5": Workload("cfg5", "er", 10_000_000, 200_000_000, True, 256, "float32", "uniform", 0.05, (15, 10, 5), 2048, 0.10),
}


def make_graph(w: Workload, device="cpu", scale: float = 1.0):
    """Graph + training set of a workload; ``scale`` < 1 shrinks nodes and draws
    alike (same average degree and skew recipe) for quick tests."""
    n = max(64, int(w.n_nodes * scale)); m = max(256, int(w.n_draws * scale))
    if w.graph == "rmat":
        indptr, indices = rmat_csr(n, m, GRAPH_SEED, device, i64_offsets=w.i64_offsets)
    else:
        indptr, indices = erdos_renyi_csr(n, m, GRAPH_SEED, device, i64_offsets=w.i64_offsets)
    train = train_set(n, w.train_fraction, GRAPH_SEED + 1, device)
    return indptr, indices, train


def small_graph(n_nodes: int, n_draws: int, seed: int, kind="rmat"):
    """numpy CSR (int64 offsets, int32 indices) for CPU tests."""
    if kind == "rmat":
        ip, ix = rmat_csr(n_nodes, n_draws, seed, "cpu")
    else:
        ip, ix = erdos_renyi_csr(n_nodes, n_draws, seed, "cpu")
    return ip.numpy().astype(np.int64), ix.numpy().astype(np.int32)
