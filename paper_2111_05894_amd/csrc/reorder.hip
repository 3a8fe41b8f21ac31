// Graph and feature-table reordering by rank (Sec. 3.2, Alg. 2): every node takes its
// rank as its new id, so that "hot" becomes "id below the boundary" and the gather
// needs no node->slot map.
//
//   k_scatter_len   nd_new[rank[i] + 1] = length of node i's neighbour list
//   k_scan_*        prefix sum over nd_new (two launches)
//   k_relocate      one thread per position of the new edge list: the owning new node
//                   is found by bisection of nd_new (first for the block's span of
//                   positions, then inside that span), the value is read from the old
//                   list of the node that now has this id and renamed through rank[];
//                   writes are fully coalesced and hubs need no special case
//   k_permute_rows  rows_new[rank[i]] = rows[i], a lane group per row, the source read
//                   in order (the source is the pinned host table)
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kSpan = 2048;        // edge positions per block of k_relocate

// rank must be a permutation of 0..n-1 and order its inverse: everything below indexes
// with their values unchecked.
__global__ void k_check_permutation(const int32_t *__restrict__ rank, const int32_t *__restrict__ order, int64_t n,
                                    int64_t *__restrict__ meta)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t r = (uint32_t)rank[i];
        if (r >= (uint64_t)n || order[r] != (int32_t)i) bad = 1;      // order[rank[i]] == i for all i <=> bijection
    }
    if (bad) atomicOr((int *)&meta[META_ERROR], 1);
}

// without `order`: every rank in range and taken once (seen: n bits, zero on entry and on exit)
__global__ void k_check_rank_marks(const int32_t *__restrict__ rank, int64_t n, uint32_t *__restrict__ seen,
                                   int64_t *__restrict__ meta)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t r = (uint32_t)rank[i];
        if (r >= (uint64_t)n) bad = 1;
        else if (atomicOr(&seen[r >> 5], 1u << (r & 31)) & (1u << (r & 31))) bad = 1;
    }
    if (bad) atomicOr((int *)&meta[META_ERROR], 1);
}

__global__ void k_clear_words(uint32_t *__restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

template <typename OffT>
__global__ void k_scatter_len(const OffT *__restrict__ indptr, const int32_t *__restrict__ rank, int64_t n,
                              OffT *__restrict__ nd_new)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) nd_new[0] = 0;
    for (int64_t i = t; i < n; i += stride) nd_new[(int64_t)rank[i] + 1] = indptr[i + 1] - indptr[i];
}

template <typename T>
__device__ inline T block_sum_t(T x, T *s_wave)
{
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = x;
    __syncthreads();
    T t = 0;
    for (int i = 0; i < kBlock / 64; ++i) t += s_wave[i];
    return t;
}

__device__ inline void scan_range(int64_t n, int64_t &lo, int64_t &hi)
{
    int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    chunk = (chunk + kBlock - 1) / kBlock * kBlock;
    lo = (int64_t)blockIdx.x * chunk;
    if (lo > n) lo = n;
    hi = lo + chunk;
    if (hi > n) hi = n;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_scan_partial(const T *__restrict__ x, int64_t n, T *__restrict__ partial)
{
    __shared__ T s_wave[kBlock / 64];
    int64_t lo, hi;
    scan_range(n, lo, hi);
    T sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) sum += x[i];
    T tot = block_sum_t<T>(sum, s_wave);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

// inclusive prefix sum in place (grid <= 1024 blocks, same grid as k_scan_partial)
template <typename T>
__global__ __launch_bounds__(kBlock) void k_scan_inclusive(T *__restrict__ x, int64_t n, const T *__restrict__ partial)
{
    __shared__ T s_wave[kBlock / 64];
    int64_t lo, hi;
    scan_range(n, lo, hi);
    T before = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kBlock) before += partial[i];
    T carry = block_sum_t<T>(before, s_wave);
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        T incl = i < hi ? x[i] : (T)0;
        for (int d = 1; d < 64; d <<= 1) {
            T y = __shfl_up(incl, d);
            if (l >= d) incl += y;
        }
        __syncthreads();
        if (l == 63) s_wave[w] = incl;
        __syncthreads();
        T base = 0, tot = 0;
        for (int q = 0; q < kBlock / 64; ++q) {
            T t = s_wave[q];
            base += q < w ? t : (T)0;
            tot += t;
        }
        if (i < hi) x[i] = carry + base + incl;
        carry += tot;
    }
}

// largest r in [lo, hi] with nd[r] <= e   (nd non-decreasing, nd[lo] <= e)
template <typename OffT>
__device__ inline int64_t owner_of(const OffT *__restrict__ nd, int64_t lo, int64_t hi, int64_t e)
{
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if ((int64_t)nd[mid] <= e) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <typename OffT>
__global__ __launch_bounds__(kBlock) void k_relocate(const OffT *__restrict__ nd, const int32_t *__restrict__ edg,
                                                     const int32_t *__restrict__ rank,
                                                     const int32_t *__restrict__ order,
                                                     const OffT *__restrict__ nd_new, int64_t n, int64_t n_edges,
                                                     int32_t *__restrict__ edg_new)
{
    __shared__ int64_t s_span[2];
    for (int64_t first = (int64_t)blockIdx.x * kSpan; first < n_edges; first += (int64_t)gridDim.x * kSpan) {
        const int64_t last = (first + kSpan < n_edges ? first + kSpan : n_edges) - 1;
        __syncthreads();
        if (threadIdx.x < 2) s_span[threadIdx.x] = owner_of<OffT>(nd_new, 0, n - 1, threadIdx.x == 0 ? first : last);
        __syncthreads();
        const int64_t r_lo = s_span[0], r_hi = s_span[1];
        for (int64_t e = first + threadIdx.x; e <= last; e += kBlock) {
            const int64_t r = owner_of<OffT>(nd_new, r_lo, r_hi, e);
            const int32_t i = order[r];                               // the node that now has id r
            const int64_t j = e - (int64_t)nd_new[r];
            edg_new[e] = rank[edg[(int64_t)nd[i] + j]];
        }
    }
}

template <int LPR>
__global__ __launch_bounds__(kBlock) void k_permute_rows(const uint4 *__restrict__ rows,
                                                         const int32_t *__restrict__ rank, int64_t n, int cpr,
                                                         uint4 *__restrict__ rows_new)
{
    constexpr int kGroups = kBlock / LPR;
    const int lane = threadIdx.x % LPR;
    const int64_t stride = (int64_t)gridDim.x * kGroups;
    for (int64_t i = (int64_t)blockIdx.x * kGroups + threadIdx.x / LPR; i < n; i += stride) {
        const int64_t r = rank[i];
        for (int c = lane; c < cpr; c += LPR) rows_new[r * cpr + c] = rows[i * cpr + c];
    }
}

__global__ void k_relabel_ids(const int32_t *__restrict__ rank, const int32_t *__restrict__ ids, int64_t n,
                              int64_t n_nodes, int32_t *__restrict__ out, int64_t *__restrict__ meta)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int32_t v = ids[i];
        if ((uint32_t)v >= (uint64_t)n_nodes) {
            atomicOr((int *)&meta[META_ERROR], 1);
            out[i] = 0;
        } else {
            out[i] = rank[v];
        }
    }
}

int grid_for(int64_t n, int per_block, int cap)
{
    int64_t g = (n + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

template <typename OffT>
int reorder_graph(tier_ctx *c, const int32_t *rank, const int32_t *order, OffT *nd_new, int32_t *edg_new)
{
    const int64_t n = c->n_nodes, ne = c->n_edges;
    hipStream_t st = c->stream;
    k_check_permutation<<<grid_for(n, kBlock, 4096), kBlock, 0, st>>>(rank, order, n, c->meta);
    TIER_HIP(c, hipGetLastError());
    int rc = tier_sync_meta(c);
    if (rc != TIER_OK) return rc;
    rc = tier_ensure(c, (void **)&c->scan_partial, &c->scan_partial_cap, TIER_SCAN_BLOCKS * sizeof(int64_t));
    if (rc != TIER_OK) return rc;
    OffT *partial = (OffT *)c->scan_partial;      // kept by the context: no allocation after the first call
    k_scatter_len<OffT><<<grid_for(n, kBlock, 4096), kBlock, 0, st>>>((const OffT *)c->indptr, rank, n, nd_new);
    const int sg = grid_for(n + 1, 4 * kBlock, 1024);
    k_scan_partial<OffT><<<sg, kBlock, 0, st>>>(nd_new, n + 1, partial);
    k_scan_inclusive<OffT><<<sg, kBlock, 0, st>>>(nd_new, n + 1, partial);
    if (ne > 0 && n > 0)
        k_relocate<OffT><<<grid_for(ne, kSpan, 65536), kBlock, 0, st>>>((const OffT *)c->indptr, c->indices, rank,
                                                                        order, nd_new, n, ne, edg_new);
    TIER_HIP(c, hipGetLastError());
    TIER_HIP(c, hipStreamSynchronize(st));
    return TIER_OK;
}

}  // namespace

extern "C" {

int tier_reorder_graph(tier_ctx *ctx, const int32_t *rank, const int32_t *order, void *indptr_new,
                       int32_t *indices_new)
{
    if (!ctx || !rank || !order || !indptr_new || (!indices_new && ctx->n_edges > 0)) return TIER_EINVAL;
    if (ctx->indptr_i64) return reorder_graph<int64_t>(ctx, rank, order, (int64_t *)indptr_new, indices_new);
    return reorder_graph<int32_t>(ctx, rank, order, (int32_t *)indptr_new, indices_new);
}

int tier_reorder_rows(tier_ctx *ctx, const int32_t *rank, void *rows_new)
{
    if (!ctx || !rank || !rows_new || ((uintptr_t)rows_new & 15u)) return TIER_EINVAL;
    const int64_t n = ctx->n_nodes;
    if (n == 0) return TIER_OK;
    // the first slot's bitmap (all zero between sampling calls) marks the ranks seen
    k_check_rank_marks<<<grid_for(n, kBlock, 4096), kBlock, 0, ctx->stream>>>(rank, n, ctx->fresh, ctx->meta);
    k_clear_words<<<grid_for(ctx->n_words, kBlock, 4096), kBlock, 0, ctx->stream>>>(ctx->fresh, ctx->n_words);
    TIER_HIP(ctx, hipGetLastError());
    int rc = tier_sync_meta(ctx);
    if (rc != TIER_OK) return rc;
    const int cpr = (int)(ctx->row_bytes / 16);
    int lpr = 8;
    while (lpr < cpr && lpr < 64) lpr *= 2;
    const int grid = grid_for(n, kBlock / lpr, 65536);
    const uint4 *src = (const uint4 *)ctx->host_rows;
    switch (lpr) {
    case 8: k_permute_rows<8><<<grid, kBlock, 0, ctx->stream>>>(src, rank, n, cpr, (uint4 *)rows_new); break;
    case 16: k_permute_rows<16><<<grid, kBlock, 0, ctx->stream>>>(src, rank, n, cpr, (uint4 *)rows_new); break;
    case 32: k_permute_rows<32><<<grid, kBlock, 0, ctx->stream>>>(src, rank, n, cpr, (uint4 *)rows_new); break;
    default: k_permute_rows<64><<<grid, kBlock, 0, ctx->stream>>>(src, rank, n, cpr, (uint4 *)rows_new); break;
    }
    TIER_HIP(ctx, hipGetLastError());
    return TIER_OK;
}

int tier_relabel_ids(tier_ctx *ctx, const int32_t *rank, const int32_t *ids, int64_t n, int32_t *out)
{
    if (!ctx || !rank || n < 0 || (n > 0 && (!ids || !out))) return TIER_EINVAL;
    if (n == 0) return TIER_OK;
    k_relabel_ids<<<grid_for(n, kBlock, 4096), kBlock, 0, ctx->stream>>>(rank, ids, n, ctx->n_nodes, out, ctx->meta);
    TIER_HIP(ctx, hipGetLastError());
    return tier_sync_meta(ctx);
}

}  // extern "C"
