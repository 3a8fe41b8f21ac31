// Neighbour sampling of one mini-batch (Sec. 2.2) and the access counts built on
// it (Sec. 3.1, Sec. 5.2).
//
// One hop over the current frontier runs as a short chain of kernels on the
// context's stream; all sizes stay on the device (tier_internal.h, META_*):
//
//   k_hop_partial   per-block sums of min(fanout, degree) over the frontier
//   k_hop_sample    offsets of every dst's edges (scan of the sums above), then a
//                   group of G lanes per dst draws its neighbours: lane i owns
//                   draw i, the Floyd collision rule is resolved with in-group
//                   shuffles; every neighbour not yet in the frontier sets its
//                   bit in a bitmap over all nodes
//   k_bm_partial    popcounts of the bitmap
//   k_bm_emit       bitmap -> ascending list of new nodes appended to the
//                   frontier (dedup and sort in one pass), their frontier index
//                   recorded in local_idx[], bitmap cleared
//   k_relabel       col[e] = frontier index of the sampled neighbour
//
// tier_presample runs the same chain without materialising blocks (no offsets,
// no edge ids, no relabel) and ends every mini-batch with one atomic increment
// per frontier node.  Within a mini-batch the frontier nodes are distinct, so
// increments of one launch never collide; concurrent launches of one stream do
// not overlap either, hence plain global atomics (no LDS staging) suffice.
#include "rng.h"
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;

__device__ inline int wave_incl_scan(int x)
{
    const int l = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int y = __shfl_up(x, d);
        if (l >= d) x += y;
    }
    return x;
}

// Sum over the block's kBlock threads, returned to every thread.
__device__ inline int block_sum(int x, int *s_wave)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = x;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int i = 0; i < kBlock / 64; ++i) t += s_wave[i];
    return t;
}

// Exclusive prefix of x over the block's threads; total = sum over the block.
__device__ inline int block_excl_scan(int x, int &total, int *s_wave)
{
    const int incl = wave_incl_scan(x);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 63) s_wave[w] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kBlock / 64; ++i) {
        int t = s_wave[i];
        base += (i < w) ? t : 0;
        tot += t;
    }
    total = tot;
    return base + incl - x;
}

// Contiguous share of [0, n) for this block: a multiple of kBlock items.
__device__ inline void block_range(int64_t n, int64_t &lo, int64_t &hi)
{
    int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    chunk = (chunk + kBlock - 1) / kBlock * kBlock;
    lo = (int64_t)blockIdx.x * chunk;
    if (lo > n) lo = n;
    hi = lo + chunk;
    if (hi > n) hi = n;
}

// Sum of partial[0 .. blockIdx.x) and of all partials (gridDim.x <= TIER_SCAN_BLOCKS).
__device__ inline void partial_prefix(const int32_t *partial, int &before, int &all, int *s_wave)
{
    int b = 0, a = 0;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += kBlock) {
        int p = partial[i];
        a += p;
        b += (i < (int)blockIdx.x) ? p : 0;
    }
    before = block_sum(b, s_wave);
    all = block_sum(a, s_wave);
}

__global__ void k_init_seeds(const int32_t *__restrict__ seeds, int32_t n_seeds, int64_t n_nodes,
                             int32_t *__restrict__ nodes, int32_t *__restrict__ local_idx,
                             int64_t *__restrict__ meta)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) meta[META_NFRONT] = n_seeds;
    if (i < n_seeds) {
        int32_t v = seeds[i];
        if ((uint32_t)v >= (uint64_t)n_nodes) {
            atomicOr((int *)&meta[META_ERROR], 1);
            v = 0;                                  // keep every later index in range
        }
        nodes[i] = v;
        local_idx[v] = i;
    }
}

template <typename OffT>
__global__ __launch_bounds__(kBlock) void k_hop_partial(const OffT *__restrict__ indptr,
                                                        const int32_t *__restrict__ nodes,
                                                        const int64_t *__restrict__ meta, int layer, int k,
                                                        int32_t *__restrict__ partial)
{
    __shared__ int s_wave[kBlock / 64];
    int64_t lo, hi;
    block_range(meta[META_NFRONT + layer], lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
        int32_t v = nodes[i];
        int64_t d = (int64_t)(indptr[v + 1] - indptr[v]);
        sum += d < k ? (int)d : k;
    }
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

// One dst node, handled by a group of G consecutive lanes (G a power of two, k <= G).
// d <= k: all neighbours in adjacency order.  d > k: Floyd's subset algorithm, draw i
// on lane i: t_i uniform in [0, d-k+i]; position = t_i unless an earlier draw already
// took t_i, then d-k+i.
template <int G, bool BLOCKS, typename OffT>
__device__ inline void sample_one(int lane, int32_t v, OffT beg, int32_t d, int k, int layer, uint32_t key0,
                                  uint32_t key1, const int32_t *__restrict__ indices,
                                  const int32_t *__restrict__ local_idx, uint32_t *__restrict__ bitmap,
                                  int64_t *__restrict__ eid, int32_t *__restrict__ src_tmp, int32_t rp)
{
    const bool draw = d > k;
    const int cnt = draw ? k : d;
    int32_t pos = lane;
    const int32_t j = d - k + lane;
    int32_t t = -1;
    if (draw && lane < k) {
        uint64_t r = tier::philox_r64(key0, key1, (uint32_t)v, (uint32_t)lane, (uint32_t)layer, tier::kTagNeighbour);
        t = (int32_t)__umul64hi(r, (uint64_t)(uint32_t)(j + 1));
        pos = t;
    }
    if (draw) {
        bool taken = false;
        for (int i = 0; i + 1 < k; ++i) {
            int32_t p = __shfl(pos, i, G);          // final position of draw i
            taken = taken || (lane > i && t == p);
            if (lane == i + 1) pos = taken ? j : t;
        }
    }
    if (lane < cnt) {
        OffT e = beg + (OffT)pos;
        int32_t u = indices[e];
        if (BLOCKS) {
            eid[rp + lane] = (int64_t)e;
            src_tmp[rp + lane] = u;
        }
        if (local_idx[u] < 0) atomicOr(&bitmap[u >> 5], 1u << (u & 31));
    }
}

template <typename OffT, int G, bool BLOCKS>
__global__ __launch_bounds__(kBlock) void k_hop_sample(
    const OffT *__restrict__ indptr, const int32_t *__restrict__ indices, const int32_t *__restrict__ nodes,
    int64_t *__restrict__ meta, int layer, int k, uint32_t key0, uint32_t key1,
    const int32_t *__restrict__ partial, const int32_t *__restrict__ local_idx, uint32_t *__restrict__ bitmap,
    int32_t *__restrict__ row_ptr, int64_t *__restrict__ eid, int32_t *__restrict__ src_tmp)
{
    __shared__ int s_wave[kBlock / 64];
    __shared__ int32_t s_v[kBlock];
    __shared__ OffT s_beg[kBlock];
    __shared__ int32_t s_deg[kBlock];
    __shared__ int32_t s_rp[kBlock];
    constexpr int kGroups = kBlock / G;
    const int lane = threadIdx.x % G;
    const int group = threadIdx.x / G;

    const int64_t n = meta[META_NFRONT + layer];
    int64_t lo, hi;
    block_range(n, lo, hi);
    int carry = 0;
    if (BLOCKS) {
        int all;
        partial_prefix(partial, carry, all, s_wave);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            meta[META_NEDGES + layer] = all;
            row_ptr[n] = all;
        }
    }
    int edges = 0;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        int32_t v = 0, d = 0, cnt = 0;
        OffT beg = 0;
        if (i < hi) {
            v = nodes[i];
            beg = indptr[v];
            d = (int32_t)(indptr[v + 1] - beg);
            cnt = d < k ? d : k;
        }
        int rp = 0;
        if (BLOCKS) {
            int tot;
            rp = carry + block_excl_scan(cnt, tot, s_wave);
            if (i < hi) row_ptr[i] = rp;
            carry += tot;
        } else {
            edges += cnt;
            __syncthreads();
        }
        s_v[threadIdx.x] = v;
        s_beg[threadIdx.x] = beg;
        s_deg[threadIdx.x] = d;
        s_rp[threadIdx.x] = rp;
        __syncthreads();
        const int tile_n = (int)((hi - tile) < kBlock ? (hi - tile) : kBlock);
        for (int jj = group; jj < tile_n; jj += kGroups)
            sample_one<G, BLOCKS, OffT>(lane, s_v[jj], s_beg[jj], s_deg[jj], k, layer, key0, key1, indices,
                                        local_idx, bitmap, eid, src_tmp, s_rp[jj]);
        __syncthreads();
    }
    if (!BLOCKS) {
        int tot = block_sum(edges, s_wave);
        if (threadIdx.x == 0 && tot)
            atomicAdd((unsigned long long *)&meta[META_TOTAL_EDGES], (unsigned long long)tot);
    }
}

__global__ __launch_bounds__(kBlock) void k_bm_partial(const uint32_t *__restrict__ bitmap, int64_t n_words,
                                                       int32_t *__restrict__ partial)
{
    __shared__ int s_wave[kBlock / 64];
    int64_t lo, hi;
    block_range(n_words, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) sum += __popc(bitmap[i]);
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kBlock) void k_bm_emit(uint32_t *__restrict__ bitmap, int64_t n_words,
                                                    const int32_t *__restrict__ partial,
                                                    int64_t *__restrict__ meta, int layer,
                                                    int32_t *__restrict__ nodes, int32_t *__restrict__ local_idx)
{
    __shared__ int s_wave[kBlock / 64];
    int64_t lo, hi;
    block_range(n_words, lo, hi);
    int carry, all;
    partial_prefix(partial, carry, all, s_wave);
    const int64_t base = meta[META_NFRONT + layer];
    if (blockIdx.x == 0 && threadIdx.x == 0) meta[META_NFRONT + layer + 1] = base + all;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        uint32_t w = i < hi ? bitmap[i] : 0u;
        int tot;
        int64_t pos = base + carry + block_excl_scan(__popc(w), tot, s_wave);
        carry += tot;
        if (w) {
            bitmap[i] = 0u;
            while (w) {
                int b = __ffs(w) - 1;
                w &= w - 1;
                int32_t u = (int32_t)(i * 32 + b);
                nodes[pos] = u;
                local_idx[u] = (int32_t)pos;
                ++pos;
            }
        }
    }
}

__global__ void k_relabel(const int32_t *__restrict__ src_tmp, const int32_t *__restrict__ local_idx,
                          const int64_t *__restrict__ meta, int layer, int32_t *__restrict__ col)
{
    const int64_t n = meta[META_NEDGES + layer];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride)
        col[e] = local_idx[src_tmp[e]];
}

// End of a mini-batch: take its nodes out of local_idx[]; with COUNT, one access
// per node of the final frontier (the rows a gather for this mini-batch reads).
template <bool COUNT>
__global__ void k_finish(const int32_t *__restrict__ nodes, int64_t *__restrict__ meta, int n_layers,
                         int32_t *__restrict__ local_idx, uint32_t *__restrict__ counts)
{
    const int64_t n = meta[META_NFRONT + n_layers];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t; i < n; i += stride) {
        int32_t v = nodes[i];
        local_idx[v] = -1;
        if (COUNT) atomicAdd(&counts[v], 1u);
    }
    if (COUNT && t == 0) meta[META_TOTAL_ROWS] += n;
}

__global__ void k_fill_u32(uint32_t *__restrict__ p, int64_t n, uint32_t value)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = value;
}

__global__ void k_clear_totals(int64_t *meta)
{
    meta[META_TOTAL_ROWS] = 0;
    meta[META_TOTAL_EDGES] = 0;
}

int clamp_grid(int64_t items, int per_block, int cap)
{
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

struct batch_out {            // where one mini-batch's results go
    int32_t *nodes;
    int32_t *row_ptr[TIER_MAX_LAYERS];
    int32_t *col[TIER_MAX_LAYERS];
    int64_t *eid[TIER_MAX_LAYERS];
    bool blocks;              // false: frontier only (access counting)
    uint32_t *counts;         // non-null: count the final frontier
};

template <typename OffT, int G>
void launch_hop_sample(tier_ctx *c, int grid, int layer, int k, uint64_t seed, const batch_out &o)
{
    const OffT *ip = (const OffT *)c->indptr;
    if (o.blocks)
        k_hop_sample<OffT, G, true><<<grid, kBlock, 0, c->stream>>>(
            ip, c->indices, o.nodes, c->meta, layer, k, (uint32_t)seed, (uint32_t)(seed >> 32), c->partial_hop,
            c->local_idx, c->bitmap, o.row_ptr[layer], o.eid[layer], c->src_tmp);
    else
        k_hop_sample<OffT, G, false><<<grid, kBlock, 0, c->stream>>>(
            ip, c->indices, o.nodes, c->meta, layer, k, (uint32_t)seed, (uint32_t)(seed >> 32), c->partial_hop,
            c->local_idx, c->bitmap, nullptr, nullptr, nullptr);
}

template <typename OffT>
void launch_hop(tier_ctx *c, int grid, int layer, int k, uint64_t seed, const batch_out &o)
{
    if (o.blocks)
        k_hop_partial<OffT><<<grid, kBlock, 0, c->stream>>>((const OffT *)c->indptr, o.nodes, c->meta, layer, k,
                                                            c->partial_hop);
    if (k <= 4) launch_hop_sample<OffT, 4>(c, grid, layer, k, seed, o);
    else if (k <= 8) launch_hop_sample<OffT, 8>(c, grid, layer, k, seed, o);
    else if (k <= 16) launch_hop_sample<OffT, 16>(c, grid, layer, k, seed, o);
    else if (k <= 32) launch_hop_sample<OffT, 32>(c, grid, layer, k, seed, o);
    else launch_hop_sample<OffT, 64>(c, grid, layer, k, seed, o);
}

// Enqueue one mini-batch.  cap_nodes / cap_edges: the bounds of tier_blocks_bounds.
int enqueue_batch(tier_ctx *c, const int32_t *seeds, int32_t n_seeds, const int32_t *fanouts, int n_layers,
                  uint64_t seed, const int64_t *cap_nodes, const int64_t *cap_edges, const batch_out &o)
{
    k_init_seeds<<<clamp_grid(n_seeds, kBlock, 1 << 20), kBlock, 0, c->stream>>>(seeds, n_seeds, c->n_nodes, o.nodes,
                                                                                c->local_idx, c->meta);
    const int bm_grid = clamp_grid(c->n_words, 4 * kBlock, TIER_SCAN_BLOCKS);
    for (int l = 0; l < n_layers; ++l) {
        const int k = fanouts[l];
        const int grid = clamp_grid(cap_nodes[l], kBlock, TIER_SCAN_BLOCKS);
        if (c->indptr_i64) launch_hop<int64_t>(c, grid, l, k, seed, o);
        else launch_hop<int32_t>(c, grid, l, k, seed, o);
        k_bm_partial<<<bm_grid, kBlock, 0, c->stream>>>(c->bitmap, c->n_words, c->partial_bm);
        k_bm_emit<<<bm_grid, kBlock, 0, c->stream>>>(c->bitmap, c->n_words, c->partial_bm, c->meta, l, o.nodes,
                                                     c->local_idx);
        if (o.blocks)
            k_relabel<<<clamp_grid(cap_edges[l], kBlock, 4096), kBlock, 0, c->stream>>>(c->src_tmp, c->local_idx,
                                                                                       c->meta, l, o.col[l]);
    }
    const int fgrid = clamp_grid(cap_nodes[n_layers], kBlock, 4096);
    if (o.counts)
        k_finish<true><<<fgrid, kBlock, 0, c->stream>>>(o.nodes, c->meta, n_layers, c->local_idx, o.counts);
    else
        k_finish<false><<<fgrid, kBlock, 0, c->stream>>>(o.nodes, c->meta, n_layers, c->local_idx, nullptr);
    TIER_HIP(c, hipGetLastError());
    return TIER_OK;
}

int ensure_i32(tier_ctx *c, int32_t **buf, int64_t *cap, int64_t want)
{
    if (want <= *cap) return TIER_OK;
    TIER_HIP(c, hipStreamSynchronize(c->stream));
    if (*buf) TIER_HIP(c, hipFree(*buf));
    *buf = nullptr;
    *cap = 0;
    TIER_HIP(c, hipMalloc(buf, (size_t)want * sizeof(int32_t)));
    *cap = want;
    return TIER_OK;
}

int check_fanouts(const int32_t *fanouts, int n_layers)
{
    if (!fanouts || n_layers < 1 || n_layers > TIER_MAX_LAYERS) return TIER_EINVAL;
    for (int l = 0; l < n_layers; ++l)
        if (fanouts[l] < 1 || fanouts[l] > TIER_MAX_FANOUT) return TIER_EINVAL;
    return TIER_OK;
}

}  // namespace

extern "C" {

int tier_sample_minibatch(tier_ctx *ctx, const int32_t *seeds, int32_t n_seeds, const int32_t *fanouts,
                          int32_t n_layers, uint64_t seed, tier_blocks *out)
{
    if (!ctx || !out || n_seeds < 0 || (n_seeds > 0 && !seeds)) return TIER_EINVAL;
    int rc = check_fanouts(fanouts, n_layers);
    if (rc) return rc;
    int64_t cap_nodes[TIER_MAX_LAYERS + 1], cap_edges[TIER_MAX_LAYERS];
    rc = tier_blocks_bounds(ctx->n_nodes, n_seeds, fanouts, n_layers, cap_nodes, cap_edges);
    if (rc) return rc;
    if (n_seeds > ctx->n_nodes) return TIER_EINVAL;          // seeds are distinct
    if (!out->nodes || out->cap_nodes < cap_nodes[n_layers]) return out->nodes ? TIER_ECAPACITY : TIER_EINVAL;
    int64_t max_edges = 1;
    batch_out o = {};
    o.nodes = out->nodes;
    o.blocks = true;
    for (int l = 0; l < n_layers; ++l) {
        if (!out->row_ptr[l] || !out->col[l] || !out->eid[l]) return TIER_EINVAL;
        if (out->cap_dst[l] < cap_nodes[l] || out->cap_edges[l] < cap_edges[l]) return TIER_ECAPACITY;
        o.row_ptr[l] = out->row_ptr[l];
        o.col[l] = out->col[l];
        o.eid[l] = out->eid[l];
        if (cap_edges[l] > max_edges) max_edges = cap_edges[l];
    }
    rc = ensure_i32(ctx, &ctx->src_tmp, &ctx->cap_src_tmp, max_edges);
    if (rc) return rc;
    rc = enqueue_batch(ctx, seeds, n_seeds, fanouts, n_layers, seed, cap_nodes, cap_edges, o);
    if (rc) return rc;
    rc = tier_sync_meta(ctx);
    for (int l = 0; l <= n_layers; ++l) out->n_nodes[l] = ctx->meta_host[META_NFRONT + l];
    for (int l = 0; l < n_layers; ++l) out->n_edges[l] = ctx->meta_host[META_NEDGES + l];
    return rc;
}

int tier_presample(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                   const int32_t *fanouts, int32_t n_layers, int32_t epochs, uint64_t seed, uint32_t *counts,
                   int64_t *total_rows, int64_t *total_edges)
{
    if (!ctx || !counts || n_train < 0 || (n_train > 0 && !train_ids) || batch_size < 1 || epochs < 0)
        return TIER_EINVAL;
    int rc = check_fanouts(fanouts, n_layers);
    if (rc) return rc;
    const int64_t first = n_train < batch_size ? n_train : batch_size;
    int64_t cap_nodes[TIER_MAX_LAYERS + 1], cap_edges[TIER_MAX_LAYERS];
    rc = tier_blocks_bounds(ctx->n_nodes, first, fanouts, n_layers, cap_nodes, cap_edges);
    if (rc) return rc;
    if (first > ctx->n_nodes) return TIER_EINVAL;
    rc = ensure_i32(ctx, &ctx->ps_nodes, &ctx->cap_ps_nodes, cap_nodes[n_layers] > 0 ? cap_nodes[n_layers] : 1);
    if (rc) return rc;

    k_fill_u32<<<clamp_grid(ctx->n_nodes, kBlock, 4096), kBlock, 0, ctx->stream>>>(counts, ctx->n_nodes, 0u);
    k_clear_totals<<<1, 1, 0, ctx->stream>>>(ctx->meta);
    batch_out o = {};
    o.nodes = ctx->ps_nodes;
    o.blocks = false;
    o.counts = counts;
    const int64_t n_batches = (n_train + batch_size - 1) / batch_size;
    for (int e = 0; e < epochs; ++e) {
        for (int64_t b = 0; b < n_batches; ++b) {
            const int64_t lo = b * batch_size;
            const int32_t n = (int32_t)(n_train - lo < batch_size ? n_train - lo : batch_size);
            rc = enqueue_batch(ctx, train_ids + lo, n, fanouts, n_layers,
                               tier_batch_seed(seed, (uint32_t)e, (uint32_t)b), cap_nodes, cap_edges, o);
            if (rc) return rc;
        }
    }
    if (total_rows || total_edges) {
        rc = tier_sync_meta(ctx);
        if (total_rows) *total_rows = ctx->meta_host[META_TOTAL_ROWS];
        if (total_edges) *total_edges = ctx->meta_host[META_TOTAL_EDGES];
        return rc;
    }
    return TIER_OK;
}

}  // extern "C"
