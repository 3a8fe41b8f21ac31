// Neighbour sampling of mini-batches (Sec. 2.2) and the access counts built on
// it (Sec. 3.1, Sec. 5.2).
//
// A mini-batch of ~1000 seeds is far too small to fill 256 compute units, so the
// sampler works on up to TIER_MAX_BATCHES mini-batches side by side: every
// kernel below is launched on a (blocks, slots) grid, blockIdx.y naming the slot
// (one mini-batch with its own frontier, its own `local_idx` and bitmap scratch
// and its own size bookkeeping).  One hop over the current frontiers is a short
// chain of kernels on the context's stream; all sizes stay on the device
// (tier_internal.h, META_*):
//
//   k_hop_partial   per-block sums of min(fanout, degree) over the frontier
//   k_hop_rowptr    offsets of every dst's edges (scan of the sums above)
//   k_hop_sample    a group of G lanes per dst draws its neighbours: lane i owns
//                   draw i, the Floyd collision rule is resolved with in-group
//                   shuffles; every neighbour not yet in the frontier sets its
//                   bit in a bitmap over all nodes
//   k_bm_partial    popcounts of the nodes reached at this hop
//   k_bm_emit       bitmap -> ascending list of new nodes appended to the
//                   frontier (dedup and sort in one pass), their frontier index
//                   recorded in local_idx[] where it is needed
//   k_relabel       once per mini-batch, all hops: col[e] = frontier index of
//                   the sampled neighbour (col[] held its node id until then)
//   k_finish        takes the mini-batch's nodes out of local_idx[] and the bitmaps
//
// Two layouts of that bookkeeping, by graph size:
//
// Up to 32 M nodes (bitmap of up to 4 MB per slot: walking it whole is cheap and it
// stays in the L2 caches): two bitmaps per slot, `seen` = frontier + nodes reached at
// this hop and `prev` = the frontier before the hop.  The hop kernel asks `prev`
// whether a neighbour is in the frontier - one bit per node instead of a 4-byte
// local_idx[] entry, whose 128-byte line came from HBM or the last-level cache for
// most sampled edges - and sets the bit in `seen` otherwise; `prev` does not change
// during the hop, so the words of the hubs, which most edges lead to, stay in each
// compute unit's own cache.  New nodes = seen ^ prev, then prev = seen.  (Asking
// `seen` itself, to skip the atomic for neighbours already marked at this hop, was
// slower either way: cached reads see stale zeros and the hubs' words drown in
// atomics, device-scope reads pile up on the L2 channels of those same words.)
//
// Above 32 M nodes: membership from local_idx[] (a bitmap of that size is no more
// cache-friendly), the bitmap holds this hop's new nodes only and a summary bitmap
// holds one bit per bitmap word (set by whoever sets the first bit of that word), so
// that the kernels reading the bitmap visit only its non-zero words and their cost
// follows the mini-batch, not the graph.
//
// tier_presample runs the same chain without materialising blocks (no offsets,
// no edge ids, no relabel; on the smaller graphs no local_idx[] either) and gives
// every node of the final frontier one access.  On the smaller graphs the slots'
// `seen` bitmaps hold exactly those frontiers when the chain ends, and one pass adds
// them up column by column (k_count_columns: no atomics, the nodes of the last hop
// are never listed).  On the larger graphs the nodes reached at the last hop take an
// atomic increment straight from the bitmap (k_bm_count, never listed either) and the
// earlier ones from the list (k_finish): within a mini-batch the frontier nodes are
// distinct, so only mini-batches of different slots can meet on one counter, spread
// over all nodes - no hot spot an LDS staging could absorb.
#include "rng.h"
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;

// What every sampler kernel needs to find its slot's data (passed by value).
struct wide_t {
    const int32_t *seeds;        // slot s reads seeds + s * batch_size
    int64_t n_seeds_total;
    int32_t batch_size;
    int32_t n_slots;
    int32_t count_edges;         // != 0: add the sampled edges to META_TOTAL_EDGES (costs an atomic per block)
    int64_t n_nodes;             // graph nodes
    int64_t n_words;             // bitmap words per slot
    int64_t n_sum;               // summary words per slot (one bit per bitmap word)
    int32_t *nodes;              // slot s: nodes + s * nodes_stride
    int64_t nodes_stride;
    int32_t *local_idx;          // [slot][n_nodes]
    uint32_t *bitmap;            // [slot][n_words]  "seen": frontier + reached at this hop
    uint32_t *prev;              // [slot][n_words]  the frontier before this hop
    uint32_t *summary;           // [slot][n_sum]
    int32_t frontier_bits;       // != 0 (graphs of up to 32 M nodes): the bitmaps hold the frontier too, see k_hop_sample
    int32_t index_nodes;         // != 0: local_idx[] records every frontier node's index (blocks; membership on large graphs)
    int32_t clear_bitmaps;       // != 0: k_finish zeroes the slot's two bitmaps (k_count_columns does it in counting mode)
    int64_t *meta;               // [slot][META_WORDS]; totals and the error flag live in slot 0
    int32_t *partial_hop;        // [slot][TIER_SCAN_BLOCKS]
    int32_t *partial_bm;         // [slot][TIER_SCAN_BLOCKS]
    uint32_t key0[TIER_MAX_BATCHES], key1[TIER_MAX_BATCHES];   // halves of each slot's seed
};

struct layer_out_t {             // one hop's outputs, slot-strided
    int32_t *row_ptr;
    int64_t row_ptr_stride;
    int32_t *col;
    int64_t *eid;
    int64_t edge_stride;
};

struct relabel_t {
    int32_t *col[TIER_MAX_LAYERS];
    int64_t stride[TIER_MAX_LAYERS];
    int32_t n_layers;
};

struct slot_view {
    int32_t *nodes;
    int32_t *local_idx;
    uint32_t *bitmap;
    uint32_t *prev;
    uint32_t *summary;
    int64_t *meta;
    int32_t *partial_hop;
    int32_t *partial_bm;
};

__device__ inline slot_view view_of(const wide_t &w)
{
    const int64_t s = blockIdx.y;
    slot_view v;
    v.nodes = w.nodes + s * w.nodes_stride;
    v.local_idx = w.local_idx + s * w.n_nodes;
    v.bitmap = w.bitmap + s * w.n_words;
    v.prev = w.prev + s * w.n_words;
    v.summary = w.summary + s * w.n_sum;
    v.meta = w.meta + s * META_WORDS;
    v.partial_hop = w.partial_hop + s * TIER_SCAN_BLOCKS;
    v.partial_bm = w.partial_bm + s * TIER_SCAN_BLOCKS;
    return v;
}

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

__global__ void k_init_seeds(wide_t w)
{
    const slot_view v = view_of(w);
    const int64_t first = (int64_t)blockIdx.y * w.batch_size;
    int64_t n = w.n_seeds_total - first;
    n = n < 0 ? 0 : (n > w.batch_size ? w.batch_size : n);
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) v.meta[META_NFRONT] = n;
    if (i < n) {
        int32_t u = w.seeds[first + i];
        if ((uint32_t)u >= (uint64_t)w.n_nodes) {
            atomicOr((int *)&w.meta[META_ERROR], 1);
            u = 0;                                   // keep every later index in range
        }
        v.nodes[i] = u;
        if (w.index_nodes) v.local_idx[u] = (int32_t)i;
        if (w.frontier_bits) {
            atomicOr(&v.bitmap[(uint32_t)u >> 5], 1u << (u & 31));
            atomicOr(&v.prev[(uint32_t)u >> 5], 1u << (u & 31));
        }
    }
}

template <typename OffT>
__global__ __launch_bounds__(kBlock) void k_hop_partial(wide_t w, const OffT *__restrict__ indptr, int layer, int k)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int64_t lo, hi;
    block_range(v.meta[META_NFRONT + layer], lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
        int32_t u = v.nodes[i];
        int64_t d = (int64_t)(indptr[u + 1] - indptr[u]);
        sum += d < k ? (int)d : k;
    }
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) v.partial_hop[blockIdx.x] = tot;
}

// Offsets of every dst's edges: row_ptr[i] = sum of min(k, degree) over dst 0..i-1.
// Same grid as k_hop_partial; block b owns the same contiguous share of the frontier.
template <typename OffT>
__global__ __launch_bounds__(kBlock) void k_hop_rowptr(wide_t w, const OffT *__restrict__ indptr, int layer, int k,
                                                       layer_out_t o)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int32_t *row_ptr = o.row_ptr + (int64_t)blockIdx.y * o.row_ptr_stride;
    const int64_t n = v.meta[META_NFRONT + layer];
    int64_t lo, hi;
    block_range(n, lo, hi);
    int carry, all;
    partial_prefix(v.partial_hop, carry, all, s_wave);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        v.meta[META_NEDGES + layer] = all;
        row_ptr[n] = all;
    }
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        int cnt = 0;
        if (i < hi) {
            int32_t u = v.nodes[i];
            int64_t d = (int64_t)(indptr[u + 1] - indptr[u]);
            cnt = d < k ? (int)d : k;
        }
        int tot;
        int rp = carry + block_excl_scan(cnt, tot, s_wave);
        if (i < hi) row_ptr[i] = rp;
        carry += tot;
    }
}

// One dst node, handled by a group of G consecutive lanes (G a power of two, k <= G).
// d <= k: all neighbours in adjacency order.  d > k: Floyd's subset algorithm, draw i
// on lane i: t_i uniform in [0, d-k+i]; position = t_i unless an earlier draw already
// took t_i, then d-k+i.
template <int G, bool BLOCKS, bool TWO_LEVEL, typename OffT>
__device__ inline void sample_one(int lane, int32_t v, OffT beg, int32_t d, int k, int layer, uint32_t key0,
                                  uint32_t key1, const int32_t *__restrict__ indices,
                                  const int32_t *__restrict__ local_idx, uint32_t *__restrict__ seen,
                                  const uint32_t *__restrict__ prev, uint32_t *__restrict__ summary, int64_t *__restrict__ eid,
                                  int32_t *__restrict__ col, int32_t rp)
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
            col[rp + lane] = u;                     // node id for now; k_relabel turns it into an index
        }
        const uint32_t word = (uint32_t)u >> 5, bit = 1u << (u & 31);
        if (TWO_LEVEL) {
            // large graph: membership from local_idx[], `seen` holds this hop's new nodes only
            if (local_idx[u] < 0 && atomicOr(&seen[word], bit) == 0u)       // first bit of this word
                atomicOr(&summary[word >> 5], 1u << (word & 31));
        } else {
            // one bit per node: in the frontier already?  `prev` does not change during the hop, so
            // the words of the hubs, which most edges lead to, stay in the compute unit's own cache
            if (!(prev[word] & bit)) atomicOr(&seen[word], bit);
        }
    }
}

// One group of G lanes per dst node, all dst nodes of the frontier side by side.
template <typename OffT, int G, bool BLOCKS, bool TWO_LEVEL>
__global__ __launch_bounds__(kBlock) void k_hop_sample(wide_t w, const OffT *__restrict__ indptr,
                                                       const int32_t *__restrict__ indices, int layer, int k,
                                                       layer_out_t o)
{
    __shared__ int s_wave[kBlock / 64];
    constexpr int kGroups = kBlock / G;
    const slot_view v = view_of(w);
    const int s = blockIdx.y;
    const int32_t *row_ptr = BLOCKS ? o.row_ptr + (int64_t)s * o.row_ptr_stride : nullptr;
    int32_t *col = BLOCKS ? o.col + (int64_t)s * o.edge_stride : nullptr;
    int64_t *eid = BLOCKS ? o.eid + (int64_t)s * o.edge_stride : nullptr;
    const uint32_t key0 = w.key0[s], key1 = w.key1[s];
    const int lane = threadIdx.x % G;
    const int64_t n = v.meta[META_NFRONT + layer];
    const int64_t stride = (int64_t)gridDim.x * kGroups;
    int edges = 0;
    for (int64_t i = (int64_t)blockIdx.x * kGroups + threadIdx.x / G; i < n; i += stride) {
        const int32_t u = v.nodes[i];
        const OffT beg = indptr[u];
        const int32_t d = (int32_t)(indptr[u + 1] - beg);
        int32_t rp = 0;
        if (BLOCKS) rp = row_ptr[i];
        else if (w.count_edges && lane == 0) edges += d < k ? d : k;
        sample_one<G, BLOCKS, TWO_LEVEL, OffT>(lane, u, beg, d, k, layer, key0, key1, indices, v.local_idx, v.bitmap, v.prev, v.summary,
                                    eid, col, rp);
    }
    if (!BLOCKS && w.count_edges) {
        int tot = block_sum(edges, s_wave);
        if (threadIdx.x == 0 && tot)
            atomicAdd((unsigned long long *)&w.meta[META_TOTAL_EDGES], (unsigned long long)tot);
    }
}

// Each thread owns one summary word = 32 bitmap words = 1024 node ids.
__global__ __launch_bounds__(kBlock) void k_bm_partial(wide_t w)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int64_t lo, hi;
    block_range(w.n_sum, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
        uint32_t live = v.summary[i];
        while (live) {
            int j = __ffs(live) - 1;
            live &= live - 1;
            sum += __popc(v.bitmap[i * 32 + j]);
        }
    }
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) v.partial_bm[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kBlock) void k_bm_emit(wide_t w, int layer)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int64_t lo, hi;
    block_range(w.n_sum, lo, hi);
    int carry, all;
    partial_prefix(v.partial_bm, carry, all, s_wave);
    const int64_t base = v.meta[META_NFRONT + layer];
    if (blockIdx.x == 0 && threadIdx.x == 0) v.meta[META_NFRONT + layer + 1] = base + all;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        const uint32_t live0 = i < hi ? v.summary[i] : 0u;
        int cnt = 0;
        for (uint32_t live = live0; live;) {
            int j = __ffs(live) - 1;
            live &= live - 1;
            cnt += __popc(v.bitmap[i * 32 + j]);
        }
        int tot;
        int64_t pos = base + carry + block_excl_scan(cnt, tot, s_wave);
        carry += tot;
        if (live0) {
            v.summary[i] = 0u;
            for (uint32_t live = live0; live;) {
                int j = __ffs(live) - 1;
                live &= live - 1;
                const int64_t word = i * 32 + j;
                uint32_t bits = v.bitmap[word];
                v.bitmap[word] = 0u;
                while (bits) {
                    int b = __ffs(bits) - 1;
                    bits &= bits - 1;
                    int32_t u = (int32_t)(word * 32 + b);
                    v.nodes[pos] = u;
                    v.local_idx[u] = (int32_t)pos;
                    ++pos;
                }
            }
        }
    }
}

// Flat variant for graphs whose whole bitmap is cheap to walk: every thread owns one
// bitmap word, no summary is kept.
__global__ __launch_bounds__(kBlock) void k_bm_partial_flat(wide_t w)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int64_t lo, hi;
    block_range(w.n_words, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) sum += __popc(v.bitmap[i] ^ v.prev[i]);
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) v.partial_bm[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kBlock) void k_bm_emit_flat(wide_t w, int layer)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int64_t lo, hi;
    block_range(w.n_words, lo, hi);
    int carry, all;
    partial_prefix(v.partial_bm, carry, all, s_wave);
    const int64_t base = v.meta[META_NFRONT + layer];
    if (blockIdx.x == 0 && threadIdx.x == 0) v.meta[META_NFRONT + layer + 1] = base + all;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        const uint32_t cur = i < hi ? v.bitmap[i] : 0u;
        uint32_t bits = i < hi ? cur ^ v.prev[i] : 0u;
        int tot;
        int64_t pos = base + carry + block_excl_scan(__popc(bits), tot, s_wave);
        carry += tot;
        if (bits) {
            v.prev[i] = cur;
            while (bits) {
                int b = __ffs(bits) - 1;
                bits &= bits - 1;
                int32_t u = (int32_t)(i * 32 + b);
                v.nodes[pos] = u;
                if (w.index_nodes) v.local_idx[u] = (int32_t)pos;
                ++pos;
            }
        }
    }
}

// Access counting on the larger graphs, last hop: the nodes reached there are neither listed
// nor indexed (no further hop, no relabelling), each takes its one access straight from the
// bitmap; k_finish counts the listed ones.
__global__ __launch_bounds__(kBlock) void k_bm_count(wide_t w, uint32_t *__restrict__ counts)
{
    __shared__ int s_wave[kBlock / 64];
    const slot_view v = view_of(w);
    int64_t lo, hi;
    block_range(w.n_sum, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
        uint32_t live = v.summary[i];
        if (live) v.summary[i] = 0u;
        while (live) {
            int j = __ffs(live) - 1;
            live &= live - 1;
            const int64_t word = i * 32 + j;
            uint32_t bits = v.bitmap[word];
            v.bitmap[word] = 0u;
            sum += __popc(bits);
            while (bits) {
                int b = __ffs(bits) - 1;
                bits &= bits - 1;
                atomicAdd(&counts[word * 32 + b], 1u);
            }
        }
    }
    const int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0 && tot)
        atomicAdd((unsigned long long *)&w.meta[META_TOTAL_ROWS], (unsigned long long)tot);
}

// Counting mode on graphs of up to 32 M nodes, end of a chain: `seen` of a slot now holds the
// whole final frontier of its mini-batch, so counts[v] grows by the number of slots whose bit
// v is set.  One thread owns one bitmap word position = 32 counters across all slots: it adds
// the slots' words bit-sliced (five planes hold sums up to 31; a flush every 31 slots), updates
// its counters without atomics (no other thread of this kernel touches them, and kernels on
// the stream run one after the other) and clears both bitmaps.
__global__ __launch_bounds__(kBlock) void k_count_columns(wide_t w, uint32_t *__restrict__ counts)
{
    __shared__ int s_wave[kBlock / 64];
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int rows = 0;
    if (i < w.n_words) {
        uint32_t plane[5] = {0u, 0u, 0u, 0u, 0u};
        int held = 0;
        auto flush = [&]() {
            if (plane[0] | plane[1] | plane[2] | plane[3] | plane[4]) {
                uint32_t *c = counts + i * 32;
                const int64_t left = w.n_nodes - i * 32;         // the last word may be ragged
#pragma unroll
                for (int b = 0; b < 32; ++b) {
                    const uint32_t add = ((plane[0] >> b) & 1u) | (((plane[1] >> b) & 1u) << 1) |
                                         (((plane[2] >> b) & 1u) << 2) | (((plane[3] >> b) & 1u) << 3) |
                                         (((plane[4] >> b) & 1u) << 4);
                    if (add && b < left) c[b] += add;
                }
            }
#pragma unroll
            for (int p = 0; p < 5; ++p) plane[p] = 0u;
            held = 0;
        };
        for (int s = 0; s < w.n_slots; ++s) {
            uint32_t *seen = w.bitmap + (int64_t)s * w.n_words + i;
            uint32_t carry = *seen;
            if (carry) {
                *seen = 0u;
                w.prev[(int64_t)s * w.n_words + i] = 0u;
                rows += __popc(carry);
#pragma unroll
                for (int p = 0; p < 5; ++p) {                     // ripple-carry add of one bit per column
                    const uint32_t t = plane[p] & carry;
                    plane[p] ^= carry;
                    carry = t;
                }
                if (++held == 31) flush();
            }
        }
        flush();
    }
    const int tot = block_sum(rows, s_wave);
    if (threadIdx.x == 0 && tot)
        atomicAdd((unsigned long long *)&w.meta[META_TOTAL_ROWS], (unsigned long long)tot);
}

__global__ void k_relabel(wide_t w, relabel_t r)
{
    const slot_view v = view_of(w);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int l = 0; l < r.n_layers; ++l) {
        int32_t *col = r.col[l] + (int64_t)blockIdx.y * r.stride[l];
        const int64_t n = v.meta[META_NEDGES + l];
        for (int64_t e = t; e < n; e += stride) col[e] = v.local_idx[col[e]];
    }
}

// End of a mini-batch: take the nodes of frontier `layer` (the last one that was listed) out
// of local_idx[] and of the bitmaps; with COUNT, one access per node (the rows a gather for
// this mini-batch reads) - k_bm_count has dealt with the nodes of the last hop.
template <bool COUNT>
__global__ void k_finish(wide_t w, int layer, uint32_t *__restrict__ counts)
{
    const slot_view v = view_of(w);
    const int64_t n = v.meta[META_NFRONT + layer];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t; i < n; i += stride) {
        int32_t u = v.nodes[i];
        if (w.index_nodes) v.local_idx[u] = -1;
        if (COUNT) atomicAdd(&counts[u], 1u);
    }
    if (w.clear_bitmaps)                        // small enough to stream through whole: cheaper than two
        for (int64_t i = t; i < w.n_words; i += stride) {     // scattered stores per frontier node
            v.bitmap[i] = 0u;
            v.prev[i] = 0u;
        }
    if (COUNT && t == 0 && n)
        atomicAdd((unsigned long long *)&w.meta[META_TOTAL_ROWS], (unsigned long long)n);
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

struct wide_out {             // where the mini-batches' results go
    layer_out_t layer[TIER_MAX_LAYERS];
    bool blocks;              // false: frontiers only (access counting)
    uint32_t *counts;         // non-null: count the final frontiers
};

// The summary bitmap pays off once walking the whole bitmap costs more than the
// returning atomics it needs: above 2^20 bitmap words (32 M nodes).
bool two_level(const tier_ctx *c) { return c->n_words > (1 << 20); }

template <typename OffT, int G, bool TWO_LEVEL>
void launch_hop_sample2(tier_ctx *c, const wide_t &w, int64_t cap_dst, int layer, int k, const wide_out &o)
{
    const OffT *ip = (const OffT *)c->indptr;
    const dim3 grid(clamp_grid(cap_dst, kBlock / G, 16384), w.n_slots);
    if (o.blocks)
        k_hop_sample<OffT, G, true, TWO_LEVEL><<<grid, kBlock, 0, c->stream>>>(w, ip, c->indices, layer, k,
                                                                               o.layer[layer]);
    else
        k_hop_sample<OffT, G, false, TWO_LEVEL><<<grid, kBlock, 0, c->stream>>>(w, ip, c->indices, layer, k,
                                                                                layer_out_t{});
}

template <typename OffT, int G>
void launch_hop_sample(tier_ctx *c, const wide_t &w, int64_t cap_dst, int layer, int k, const wide_out &o)
{
    if (two_level(c)) launch_hop_sample2<OffT, G, true>(c, w, cap_dst, layer, k, o);
    else launch_hop_sample2<OffT, G, false>(c, w, cap_dst, layer, k, o);
}

template <typename OffT>
void launch_hop(tier_ctx *c, const wide_t &w, int64_t cap_dst, int layer, int k, const wide_out &o)
{
    if (o.blocks) {
        const dim3 grid(clamp_grid(cap_dst, kBlock, TIER_SCAN_BLOCKS), w.n_slots);
        k_hop_partial<OffT><<<grid, kBlock, 0, c->stream>>>(w, (const OffT *)c->indptr, layer, k);
        k_hop_rowptr<OffT><<<grid, kBlock, 0, c->stream>>>(w, (const OffT *)c->indptr, layer, k, o.layer[layer]);
    }
    if (k <= 4) launch_hop_sample<OffT, 4>(c, w, cap_dst, layer, k, o);
    else if (k <= 8) launch_hop_sample<OffT, 8>(c, w, cap_dst, layer, k, o);
    else if (k <= 16) launch_hop_sample<OffT, 16>(c, w, cap_dst, layer, k, o);
    else if (k <= 32) launch_hop_sample<OffT, 32>(c, w, cap_dst, layer, k, o);
    else launch_hop_sample<OffT, 64>(c, w, cap_dst, layer, k, o);
}

// Enqueue w.n_slots mini-batches.  cap_nodes / cap_edges: the bounds of tier_blocks_bounds
// for one mini-batch of w.batch_size seeds.
int enqueue_wide(tier_ctx *c, const wide_t &w, const int32_t *fanouts, int n_layers, const int64_t *cap_nodes,
                 const int64_t *cap_edges, const wide_out &o)
{
    const unsigned slots = (unsigned)w.n_slots;
    k_init_seeds<<<dim3(clamp_grid(w.batch_size, kBlock, 1 << 20), slots), kBlock, 0, c->stream>>>(w);
    const bool tl = two_level(c);
    const dim3 bm_grid(tl ? clamp_grid(c->n_sum, kBlock, TIER_SCAN_BLOCKS)
                          : clamp_grid(c->n_words, 4 * kBlock, TIER_SCAN_BLOCKS), slots);
    for (int l = 0; l < n_layers; ++l) {
        if (c->indptr_i64) launch_hop<int64_t>(c, w, cap_nodes[l], l, fanouts[l], o);
        else launch_hop<int32_t>(c, w, cap_nodes[l], l, fanouts[l], o);
        if (o.counts && l == n_layers - 1) {
            // the last hop's nodes are never listed: counted from the bitmaps (see k_count_columns / k_bm_count)
            if (tl) k_bm_count<<<bm_grid, kBlock, 0, c->stream>>>(w, o.counts);
            else k_count_columns<<<clamp_grid(c->n_words, kBlock, 1 << 22), kBlock, 0, c->stream>>>(w, o.counts);
        } else if (tl) {
            k_bm_partial<<<bm_grid, kBlock, 0, c->stream>>>(w);
            k_bm_emit<<<bm_grid, kBlock, 0, c->stream>>>(w, l);
        } else {
            k_bm_partial_flat<<<bm_grid, kBlock, 0, c->stream>>>(w);
            k_bm_emit_flat<<<bm_grid, kBlock, 0, c->stream>>>(w, l);
        }
    }
    if (o.blocks) {
        relabel_t r = {};
        r.n_layers = n_layers;
        int64_t most = 1;
        for (int l = 0; l < n_layers; ++l) {
            r.col[l] = o.layer[l].col;
            r.stride[l] = o.layer[l].edge_stride;
            if (cap_edges[l] > most) most = cap_edges[l];
        }
        k_relabel<<<dim3(clamp_grid(most, kBlock, 4096), slots), kBlock, 0, c->stream>>>(w, r);
    }
    const int last = o.counts ? n_layers - 1 : n_layers;       // last frontier that was listed
    const dim3 fgrid(clamp_grid(cap_nodes[last], kBlock, 4096), slots);
    if (o.counts && tl) k_finish<true><<<fgrid, kBlock, 0, c->stream>>>(w, last, o.counts);
    else if (!o.counts) k_finish<false><<<fgrid, kBlock, 0, c->stream>>>(w, last, nullptr);
    TIER_HIP(c, hipGetLastError());
    return TIER_OK;
}

wide_t make_wide(tier_ctx *c, const int32_t *seeds, int64_t n_seeds_total, int32_t batch_size, int32_t n_slots,
                 int32_t *nodes, int64_t nodes_stride)
{
    wide_t w = {};
    w.seeds = seeds;
    w.n_seeds_total = n_seeds_total;
    w.batch_size = batch_size;
    w.n_slots = n_slots;
    w.n_nodes = c->n_nodes;
    w.n_words = c->n_words;
    w.nodes = nodes;
    w.nodes_stride = nodes_stride;
    w.local_idx = c->local_idx;
    w.bitmap = c->bitmap;
    w.prev = c->prev;
    w.summary = c->summary;
    w.n_sum = c->n_sum;
    w.meta = c->meta;
    w.partial_hop = c->partial_hop;
    w.partial_bm = c->partial_bm;
    return w;
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

int tier_max_batches(const tier_ctx *ctx) { return ctx ? ctx->n_slots : 0; }

int tier_sample_minibatches(tier_ctx *ctx, const int32_t *seeds, int64_t n_seeds_total, int32_t batch_size,
                            int32_t n_batches, const int32_t *fanouts, int32_t n_layers,
                            const uint64_t *batch_seeds, tier_blocks_batch *out)
{
    if (!ctx || !out || !batch_seeds || n_seeds_total < 0 || (n_seeds_total > 0 && !seeds) || batch_size < 1)
        return TIER_EINVAL;
    if (n_batches < 1 || n_batches > ctx->n_slots) return TIER_EINVAL;
    if (n_seeds_total > (int64_t)batch_size * n_batches) return TIER_EINVAL;
    int rc = check_fanouts(fanouts, n_layers);
    if (rc) return rc;
    const int64_t per_batch = n_seeds_total < batch_size ? n_seeds_total : batch_size;
    int64_t cap_nodes[TIER_MAX_LAYERS + 1], cap_edges[TIER_MAX_LAYERS];
    rc = tier_blocks_bounds(ctx->n_nodes, per_batch, fanouts, n_layers, cap_nodes, cap_edges);
    if (rc) return rc;
    if (per_batch > ctx->n_nodes) return TIER_EINVAL;          // seeds of a mini-batch are distinct
    if (!out->nodes || !out->n_nodes || !out->n_edges) return TIER_EINVAL;
    if (out->nodes_stride < cap_nodes[n_layers]) return TIER_ECAPACITY;
    wide_out o = {};
    o.blocks = true;
    for (int l = 0; l < n_layers; ++l) {
        if (!out->row_ptr[l] || !out->col[l] || !out->eid[l]) return TIER_EINVAL;
        if (out->row_ptr_stride[l] < cap_nodes[l] + 1 || out->edge_stride[l] < cap_edges[l]) return TIER_ECAPACITY;
        o.layer[l] = layer_out_t{out->row_ptr[l], out->row_ptr_stride[l], out->col[l], out->eid[l],
                                 out->edge_stride[l]};
    }
    wide_t w = make_wide(ctx, seeds, n_seeds_total, batch_size, n_batches, out->nodes, out->nodes_stride);
    w.frontier_bits = two_level(ctx) ? 0 : 1;
    w.index_nodes = 1;
    w.clear_bitmaps = w.frontier_bits;
    for (int s = 0; s < n_batches; ++s) {
        w.key0[s] = (uint32_t)batch_seeds[s];
        w.key1[s] = (uint32_t)(batch_seeds[s] >> 32);
    }
    rc = enqueue_wide(ctx, w, fanouts, n_layers, cap_nodes, cap_edges, o);
    if (rc) return rc;
    rc = tier_sync_meta(ctx);
    for (int s = 0; s < n_batches; ++s) {
        const int64_t *m = ctx->meta_host + (int64_t)s * META_WORDS;
        for (int l = 0; l <= n_layers; ++l) out->n_nodes[s * (TIER_MAX_LAYERS + 1) + l] = m[META_NFRONT + l];
        for (int l = 0; l < n_layers; ++l) out->n_edges[s * TIER_MAX_LAYERS + l] = m[META_NEDGES + l];
    }
    return rc;
}

int tier_sample_minibatch(tier_ctx *ctx, const int32_t *seeds, int32_t n_seeds, const int32_t *fanouts,
                          int32_t n_layers, uint64_t seed, tier_blocks *out)
{
    if (!out || n_seeds < 0 || n_layers < 1 || n_layers > TIER_MAX_LAYERS) return TIER_EINVAL;
    // one mini-batch = a batch of one; the caps of tier_blocks serve as strides
    tier_blocks_batch b = {};
    b.nodes = out->nodes;
    b.nodes_stride = out->cap_nodes;
    for (int l = 0; l < n_layers; ++l) {
        b.row_ptr[l] = out->row_ptr[l];
        b.col[l] = out->col[l];
        b.eid[l] = out->eid[l];
        b.row_ptr_stride[l] = out->cap_dst[l] + 1;
        b.edge_stride[l] = out->cap_edges[l];
    }
    b.n_nodes = out->n_nodes;
    b.n_edges = out->n_edges;
    return tier_sample_minibatches(ctx, seeds, n_seeds, n_seeds > 0 ? n_seeds : 1, 1, fanouts, n_layers, &seed, &b);
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
    const int64_t stride = cap_nodes[n_layers] > 0 ? cap_nodes[n_layers] : 1;
    rc = ensure_i32(ctx, &ctx->ps_nodes, &ctx->cap_ps_nodes, stride * ctx->n_slots);
    if (rc) return rc;

    k_fill_u32<<<clamp_grid(ctx->n_nodes, kBlock, 4096), kBlock, 0, ctx->stream>>>(counts, ctx->n_nodes, 0u);
    k_clear_totals<<<1, 1, 0, ctx->stream>>>(ctx->meta);
    wide_out o = {};
    o.blocks = false;
    o.counts = counts;
    const int64_t n_batches = (n_train + batch_size - 1) / batch_size;
    for (int e = 0; e < epochs; ++e) {
        for (int64_t b = 0; b < n_batches; b += ctx->n_slots) {
            const int slots = (int)(n_batches - b < ctx->n_slots ? n_batches - b : ctx->n_slots);
            const int64_t lo = b * batch_size;
            wide_t w = make_wide(ctx, train_ids + lo, n_train - lo, batch_size, slots, ctx->ps_nodes, stride);
            w.frontier_bits = two_level(ctx) ? 0 : 1;
            w.index_nodes = w.frontier_bits ? 0 : 1;       // small graphs: nothing is relabelled, local_idx[] stays untouched
            w.clear_bitmaps = 0;                           // k_count_columns clears the bitmaps
            w.count_edges = total_edges != nullptr;
            for (int s = 0; s < slots; ++s) {
                const uint64_t bs = tier_batch_seed(seed, (uint32_t)e, (uint32_t)(b + s));
                w.key0[s] = (uint32_t)bs;
                w.key1[s] = (uint32_t)(bs >> 32);
            }
            rc = enqueue_wide(ctx, w, fanouts, n_layers, cap_nodes, cap_edges, o);
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
