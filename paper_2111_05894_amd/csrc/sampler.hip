// Neighbour sampling of mini-batches (Sec. 2.2) and the access counts built on
// it (Sec. 3.1, Sec. 5.2).
//
// A mini-batch of ~1000 seeds is far too small to fill 256 compute units, so the
// sampler works on up to TIER_MAX_BATCHES mini-batches side by side, each in a slot
// of its own (its own frontier, its own scratch, its own size bookkeeping).  One hop
// over the current frontiers is a short chain of kernels on the context's stream;
// all sizes stay on the device (tier_internal.h, META_*):
//
//   k_hop_partial   per-block sums of min(fanout, degree) over the frontier
//   k_hop_rowptr    offsets of every dst's edges (scan of the sums above)
//   k_hop_sample    a group of G lanes per dst draws its neighbours: lane i owns
//                   draw i, the Floyd collision rule is resolved with in-group
//                   shuffles; a neighbour already in the frontier gets its frontier
//                   index at once, any other is new at this hop
//   (new nodes)     deduplicated, listed in ascending order behind the frontier, and
//                   every edge that led to one gets its index: one of the two ways below
//   k_settle        the new nodes' adjacency offsets and degrees, listed beside the
//                   frontier (every later hop reads them in order instead of chasing
//                   indptr[] again), and the second half of entering them into the
//                   frontier index
//   k_finish        leaves the slot's scratch clean for the next mini-batch
//
// What the design is built around, measured on MI355X: an atomic of any kind and
// scope runs at ~27 G/s for the whole chip, a random 4-byte read from HBM at ~50 G/s
// (and costs HBM a whole 128-byte line), and a random read or plain store that stays in
// one XCD's 4 MB L2 at ~240 G/s.  So
//   - every kernel maps workgroups to slots by XCD (workgroup i runs on XCD i % 8; a
//     slot is served by one XCD only and the slots of an XCD one after the other), so
//     that a slot's small structures live in that XCD's L2; nothing depends on this
//     mapping for correctness;
//   - the frontier index is an open-addressing table (node -> position in nodes[], 4
//     bytes per cell, key checked against nodes[]) sized for the largest frontier that
//     ever draws (a few MB at most for the usual fanouts), not an array over all nodes:
//     membership test and index are one lookup in L2;
//   - nodes enter the table without atomics: the kernel that lists them stores into an
//     empty home cell with a plain store, k_settle (next kernel) checks who won a
//     contested cell and moves only the losers on, by compare-and-swap;
//   - a dst node's work is a chain of dependent reads (offsets, neighbour id, index cell,
//     key), and with every wave slot taken the chain's latency, not any throughput, set
//     the pace: k_hop_sample therefore works on four dst nodes per lane group at a time,
//     issuing each stage's reads for all four before it uses any;
//   - the nodes reached at the last hop never enter the table (nothing is drawn from
//     them).
//
// The new nodes of a hop, two ways (the layout of a context: tier_set_segment_words):
//   - bitmap, graphs of up to 32 M nodes: k_hop_sample sets the node's bit in `fresh`, a
//     bitmap over all nodes (the one atomic per sampled edge), and a flag byte for the
//     bitmap word; k_bm_partial / k_bm_emit walk the flags (a byte per 32 nodes) and turn
//     the flagged words into the ascending list; k_relabel, once per mini-batch, gives the
//     edges that led to new nodes their index (index lookup, or for the last hop the
//     word's start position + the rank of the bit).  The whole bitmap sits in the
//     last-level cache.
//   - buckets, above: there nearly every new node would sit alone in its 128-byte line
//     of the bitmap (an atomic, then the line read again to count, to list, to relabel,
//     to clear).  Instead the hop's new neighbours are sorted into buckets of consecutive
//     ids (k_part_*, further down): no global atomics, no relabel pass.
//
// tier_presample runs the same chains without materialising blocks (no offsets, no
// edge ids).  On the bitmap layout it keeps the frontier itself in two bitmaps per slot
// (`seen` = frontier + reached at this hop, `prev` = frontier before the hop;
// membership is one bit of `prev`, which stays in cache) and needs no index at all; on
// the other it uses the table for membership, buckets for the hops before the last, and
// a bitmap `all` that collects the whole frontier (the last hop marks it directly).
// Either way a slot ends with the bitmap of its mini-batch's final frontier, and one
// pass adds the slots' bitmaps column by column (k_count_columns: no atomics; the nodes
// of the last hop are never listed).  Within a mini-batch the frontier nodes are
// distinct, so no counter is a hot spot that LDS staging could absorb.
//
// tier_presample_draws counts by the other reading (every seed and every drawn neighbour adds
// one): the same chains, k_hop_sample<.., DRAWS> adding as it draws, through a small table per
// block in LDS; k_count_columns then only clears the bitmaps.
#include "rng.h"
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kXcds = 8;             // XCDs of an MI355X; workgroup i of a launch runs on XCD i % 8
constexpr int kPartBlocks = 16;      // blocks per slot that sort a hop's new neighbours into buckets (best of 8 .. 64, at 16 to 64 slots)

enum { MODE_BLOCKS = 0, MODE_COUNT_SMALL = 1, MODE_COUNT_LARGE = 2 };

// What every sampler kernel needs to find its slot's data (passed by value).
struct wide_t {
    const int32_t *seeds;        // slot s reads seeds + s * batch_size
    int64_t n_seeds_total;
    int32_t batch_size;
    int32_t n_slots;
    int32_t count_edges;         // != 0: add the sampled edges to META_TOTAL_EDGES (costs an atomic per block)
    int32_t seg_log2;            // 0: bitmap layout; 5: bucket layout (large graphs)
    int64_t n_nodes;             // graph nodes
    int64_t n_words;             // bitmap words that cover the graph
    int64_t bm_stride;           // bitmap words per slot (n_words rounded up to whole 128-byte lines; the rest stays zero)
    int64_t n_seg;               // segments per slot
    int64_t flag_stride;         // bytes of flags per slot (n_seg rounded up)
    int32_t *nodes;              // slot s: nodes + s * nodes_stride
    int64_t nodes_stride;
    uint32_t *fresh;             // [slot][bm_stride]  nodes first reached at this hop (MODE_COUNT_SMALL: `seen`)
    uint32_t *aux;               // [slot][bm_stride]  MODE_COUNT_SMALL: `prev`; MODE_COUNT_LARGE: `all`
    uint8_t *flag;               // [slot][flag_stride]  != 0: the segment holds a bit of `fresh`
    int32_t *segbase;            // [slot][n_seg]    last hop of a block call: new nodes listed before the segment's first
    uint32_t *table;             // [slot][1 << table_log2]  frontier index: position in nodes[] + 1, 0 = empty
    int32_t table_log2;
    int32_t pad_;
    int64_t *beg;                // [slot][deg_stride]  indptr[node] of the frontier nodes that draw
    int32_t *deg;                // [slot][deg_stride]  their degrees
    int64_t deg_stride;
    int64_t *meta;               // [slot][META_WORDS]; totals and the error flag live in slot 0
    int32_t *partial_hop;        // [slot][TIER_SCAN_BLOCKS]
    int32_t *partial_bm;         // [slot][TIER_SCAN_BLOCKS]
    uint32_t *draws;             // tier_presample_draws: counts[] that every seed and every drawn neighbour adds to
    // last hop of a block call by buckets (n_buckets != 0): see k_part_hist
    unsigned long long *rec;     // [slot][rec_stride]  node << 32 | edge, grouped by bucket
    int32_t *lrank;              // [slot][rec_stride]  rank of the record's node among its bucket's distinct nodes
    int32_t *stage;              // [slot][rec_stride]  a bucket's distinct nodes, ascending, from the bucket's start
    int64_t rec_stride;
    int32_t *rows;               // [slot][kPartBlocks][n_buckets]
    int32_t *bk;                 // [slot][3][n_buckets + 1]
    int32_t n_buckets;           // 0: the last hop marks `fresh` like the others
    int32_t bucket_log2;         // a bucket is 1 << bucket_log2 consecutive node ids
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
    uint32_t *fresh;
    uint32_t *aux;
    uint8_t *flag;
    int32_t *segbase;
    uint32_t *table;
    int64_t *beg;
    int32_t *deg;
    int64_t *meta;
    int32_t *partial_hop;
    int32_t *partial_bm;
    unsigned long long *rec;
    int32_t *lrank;
    int32_t *stage;
    int32_t *rows;
    int32_t *bk_start;           // [n_buckets + 1] first record of a bucket; the last entry is the number of records
    int32_t *bk_cnt;             // [n_buckets]     distinct nodes of a bucket
    int32_t *bk_before;          // [n_buckets]     distinct nodes of the buckets before it
};

// Which slot and which of the slot's gx blocks this workgroup is.  The launch has
// 8 * gx * ceil(n_slots / 8) workgroups; workgroup f runs on XCD f % 8 and serves slot
// (f % 8) + 8 * ((f / 8) / gx): every slot is served by one XCD, and an XCD takes its
// slots one after the other, so the structures of one or two slots are what its L2 holds
// at any time.  Workgroups that fall on a slot beyond n_slots have nothing to do.
struct spot_t {
    int slot;
    int bx;      // block index within the slot, 0 .. gx - 1
    int gx;
};

__device__ inline bool my_spot(const wide_t &w, int gx, spot_t &p)
{
    const unsigned f = blockIdx.x;
    const unsigned k = f / kXcds;
    p.slot = (int)(f % kXcds) + kXcds * (int)(k / (unsigned)gx);
    p.bx = (int)(k % (unsigned)gx);
    p.gx = gx;
    return p.slot < w.n_slots;
}

__device__ inline slot_view view_of(const wide_t &w, int slot)
{
    const int64_t s = slot;
    slot_view v;
    v.nodes = w.nodes + s * w.nodes_stride;
    v.fresh = w.fresh + s * w.bm_stride;
    v.aux = w.aux + s * w.bm_stride;
    v.flag = w.flag + s * w.flag_stride;
    v.segbase = w.segbase + s * w.n_seg;
    v.table = w.table + (s << w.table_log2);
    v.beg = w.beg + s * w.deg_stride;
    v.deg = w.deg + s * w.deg_stride;
    v.meta = w.meta + s * META_WORDS;
    v.partial_hop = w.partial_hop + s * TIER_SCAN_BLOCKS;
    v.partial_bm = w.partial_bm + s * TIER_SCAN_BLOCKS;
    v.rec = w.rec + s * w.rec_stride;
    v.lrank = w.lrank + s * w.rec_stride;
    v.stage = w.stage + s * w.rec_stride;
    v.rows = w.rows + s * kPartBlocks * (int64_t)w.n_buckets;
    v.bk_start = w.bk + s * 3 * (int64_t)(w.n_buckets + 1);
    v.bk_cnt = v.bk_start + (w.n_buckets + 1);
    v.bk_before = v.bk_cnt + (w.n_buckets + 1);
    return v;
}

// ---- frontier index: open addressing, linear probing, key = nodes[cell - 1] --------------------

__device__ inline uint32_t home_of(uint32_t node, int table_log2) { return (node * 0x9E3779B1u) >> (32 - table_log2); }

// Position of `node` in nodes[], or -1.  The table holds at most half as many nodes as cells.
__device__ inline int32_t index_of(const uint32_t *__restrict__ table, int table_log2,
                                   const int32_t *__restrict__ nodes, int32_t node)
{
    const uint32_t mask = (1u << table_log2) - 1u;
    uint32_t h = home_of((uint32_t)node, table_log2);
    for (;;) {
        const uint32_t cell = table[h];
        if (cell == 0u) return -1;
        if (nodes[cell - 1u] == node) return (int32_t)(cell - 1u);
        h = (h + 1u) & mask;
    }
}

// Enter nodes[pos] with compare-and-swap (the few seeds; the losers of k_settle).
__device__ inline void index_insert_cas(uint32_t *__restrict__ table, int table_log2, uint32_t h, uint32_t pos)
{
    const uint32_t mask = (1u << table_log2) - 1u;
    while (atomicCAS(&table[h], 0u, pos + 1u) != 0u) h = (h + 1u) & mask;
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

// The same for a block of NW waves.
template <int NW>
__device__ inline int block_excl_scan_n(int x, int &total, int *s_wave)
{
    const int incl = wave_incl_scan(x);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 63) s_wave[w] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        int t = s_wave[i];
        base += (i < w) ? t : 0;
        tot += t;
    }
    total = tot;
    return base + incl - x;
}

// Contiguous share of [0, n) for block p.bx of p.gx: a multiple of kBlock items.
__device__ inline void block_range(const spot_t &p, int64_t n, int64_t &lo, int64_t &hi)
{
    int64_t chunk = (n + p.gx - 1) / p.gx;
    chunk = (chunk + kBlock - 1) / kBlock * kBlock;
    lo = (int64_t)p.bx * chunk;
    if (lo > n) lo = n;
    hi = lo + chunk;
    if (hi > n) hi = n;
}

// Sum of partial[0 .. p.bx) and of all p.gx partials (p.gx <= TIER_SCAN_BLOCKS).
__device__ inline void partial_prefix(const spot_t &p, const int32_t *partial, int &before, int &all, int *s_wave)
{
    int b = 0, a = 0;
    for (int i = threadIdx.x; i < p.gx; i += kBlock) {
        int q = partial[i];
        a += q;
        b += (i < p.bx) ? q : 0;
    }
    before = block_sum(b, s_wave);
    all = block_sum(a, s_wave);
}

template <int MODE, typename OffT>
__global__ __launch_bounds__(kBlock) void k_init_seeds(wide_t w, int gx, const OffT *__restrict__ indptr)
{
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int64_t first = (int64_t)p.slot * w.batch_size;
    int64_t n = w.n_seeds_total - first;
    n = n < 0 ? 0 : (n > w.batch_size ? w.batch_size : n);
    const int64_t i = (int64_t)p.bx * kBlock + threadIdx.x;
    if (i == 0) v.meta[META_NFRONT] = n;
    if (i < n) {
        int32_t u = w.seeds[first + i];
        if ((uint32_t)u >= (uint64_t)w.n_nodes) {
            atomicOr((int *)&w.meta[META_ERROR], 1);
            u = 0;                                   // keep every later index in range
        }
        v.nodes[i] = u;
        if (MODE != MODE_BLOCKS && w.draws) atomicAdd(&w.draws[u], 1u);
        const OffT first_edge = indptr[u];
        v.beg[i] = (int64_t)first_edge;
        v.deg[i] = (int32_t)(indptr[u + 1] - first_edge);
        const uint32_t word = (uint32_t)u >> 5, bit = 1u << (u & 31);
        bool twice = false;                          // the seeds of a mini-batch must be distinct
        if (MODE == MODE_COUNT_SMALL) {
            twice = (atomicOr(&v.fresh[word], bit) & bit) != 0u;
            atomicOr(&v.aux[word], bit);
        } else {
            __threadfence();                         // nodes[i] before the cell that points to it
            const uint32_t mask = (1u << w.table_log2) - 1u;
            uint32_t h = home_of((uint32_t)u, w.table_log2);
            for (;;) {
                const uint32_t cell = atomicCAS(&v.table[h], 0u, (uint32_t)i + 1u);
                if (cell == 0u) break;
                if (__hip_atomic_load(&v.nodes[cell - 1u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == u) twice = true;
                h = (h + 1u) & mask;
            }
            if (MODE == MODE_COUNT_LARGE) atomicOr(&v.aux[word], bit);
        }
        if (twice) atomicOr((int *)&w.meta[META_ERROR], 1);
    }
}

__global__ __launch_bounds__(kBlock) void k_hop_partial(wide_t w, int gx, int layer, int k)
{
    __shared__ int s_wave[kBlock / 64];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int64_t lo, hi;
    block_range(p, v.meta[META_NFRONT + layer], lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
        const int d = v.deg[i];
        sum += d < k ? d : k;
    }
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) v.partial_hop[p.bx] = tot;
}

// Offsets of every dst's edges: row_ptr[i] = sum of min(k, degree) over dst 0..i-1.
// Same grid as k_hop_partial; a block owns the same contiguous share of the frontier.
__global__ __launch_bounds__(kBlock) void k_hop_rowptr(wide_t w, int gx, int layer, int k, layer_out_t o)
{
    __shared__ int s_wave[kBlock / 64];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int32_t *row_ptr = o.row_ptr + (int64_t)p.slot * o.row_ptr_stride;
    const int64_t n = v.meta[META_NFRONT + layer];
    int64_t lo, hi;
    block_range(p, n, lo, hi);
    int carry, all;
    partial_prefix(p, v.partial_hop, carry, all, s_wave);
    if (p.bx == 0 && threadIdx.x == 0) {
        v.meta[META_NEDGES + layer] = all;
        row_ptr[n] = all;
    }
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        int cnt = 0;
        if (i < hi) {
            const int d = v.deg[i];
            cnt = d < k ? d : k;
        }
        int tot;
        int rp = carry + block_excl_scan(cnt, tot, s_wave);
        if (i < hi) row_ptr[i] = rp;
        carry += tot;
    }
}

constexpr int kAtOnce = 4;       // dst nodes a lane group works on at a time

// One group of G consecutive lanes per dst node (G a power of two, k <= G), all dst nodes of
// the frontier side by side.  d <= k: all neighbours in adjacency order.  d > k: Floyd's subset
// algorithm, draw i on lane i: t_i uniform in [0, d-k+i]; position = t_i unless an earlier draw
// already took t_i, then d-k+i.  A group takes kAtOnce dst nodes at a time and goes through them
// stage by stage, so that the reads of one stage are in flight together.
//
// DRAWS (tier_presample_draws): every drawn neighbour adds one to w.draws[].  Most draws of a block
// lead to few nodes (the hubs), so a block keeps a small table of (node, count) in LDS, adds there
// when the node's cell is free or its own, and hands the sums over with one global atomic per cell
// when it is through; a draw whose cell is taken by another node goes to the global counter at once.
constexpr int kPrivCells = 1024;

template <int G, int MODE, bool DRAWS>
__global__ __launch_bounds__(kBlock) void k_hop_sample(wide_t w, int gx, const int32_t *__restrict__ indices, int layer,
                                                       int k, int last, int mark, layer_out_t o)
{
    __shared__ int s_wave[kBlock / 64];
    __shared__ uint32_t s_priv_key[DRAWS ? kPrivCells : 1], s_priv_cnt[DRAWS ? kPrivCells : 1];
    constexpr int kGroups = kBlock / G;
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    if (DRAWS) {
        for (int i = threadIdx.x; i < kPrivCells; i += kBlock) {
            s_priv_key[i] = 0xffffffffu;
            s_priv_cnt[i] = 0u;
        }
        __syncthreads();
    }
    const slot_view v = view_of(w, p.slot);
    const int s = p.slot;
    const int32_t *row_ptr = MODE == MODE_BLOCKS ? o.row_ptr + (int64_t)s * o.row_ptr_stride : nullptr;
    int32_t *col = MODE == MODE_BLOCKS ? o.col + (int64_t)s * o.edge_stride : nullptr;
    // access counting on the large-graph layout, not the last hop: k entries per dst node for the k_part_* kernels
    int32_t *dense_col = (MODE == MODE_COUNT_LARGE && o.col) ? o.col + (int64_t)s * o.edge_stride : nullptr;
    int64_t *eid = MODE == MODE_BLOCKS ? o.eid + (int64_t)s * o.edge_stride : nullptr;
    const uint32_t key0 = w.key0[s], key1 = w.key1[s];
    const int lane = threadIdx.x % G;
    const int64_t n = v.meta[META_NFRONT + layer];
    const int64_t sweep = (int64_t)gx * kGroups;                  // dst nodes all the slot's groups cover side by side
    const uint32_t mask = (1u << w.table_log2) - 1u;
    int edges = 0;
    for (int64_t i0 = (int64_t)p.bx * kGroups + threadIdx.x / G; i0 < n; i0 += sweep * kAtOnce) {
        // stage 1: the dst nodes, their offsets and degrees (listed by k_init_seeds / k_settle)
        int32_t node[kAtOnce], d[kAtOnce], rp[kAtOnce];
        int64_t beg[kAtOnce];
#pragma unroll
        for (int j = 0; j < kAtOnce; ++j) {
            const int64_t i = i0 + j * sweep;
            const bool there = i < n;
            node[j] = there ? v.nodes[i] : 0;
            beg[j] = there ? v.beg[i] : 0;
            d[j] = there ? v.deg[i] : 0;
            rp[j] = (MODE == MODE_BLOCKS && there) ? row_ptr[i] : 0;
        }
        // stage 2: positions in the adjacency lists
        int32_t pos[kAtOnce];
#pragma unroll
        for (int j = 0; j < kAtOnce; ++j) {
            const bool draw = d[j] > k;
            pos[j] = lane;
            const int32_t top = d[j] - k + lane;
            int32_t t = -1;
            if (draw && lane < k) {
                uint64_t r = tier::philox_r64(key0, key1, (uint32_t)node[j], (uint32_t)lane, (uint32_t)layer, tier::kTagNeighbour);
                t = (int32_t)__umul64hi(r, (uint64_t)(uint32_t)(top + 1));
                pos[j] = t;
            }
            if (draw) {
                bool taken = false;
                for (int q = 0; q + 1 < k; ++q) {
                    int32_t f = __shfl(pos[j], q, G);          // final position of draw q
                    taken = taken || (lane > q && t == f);
                    if (lane == q + 1) pos[j] = taken ? top : t;
                }
            }
            if (MODE != MODE_BLOCKS && w.count_edges && lane == 0) edges += d[j] < k ? d[j] : k;
        }
        // stage 3: the neighbours
        bool take[kAtOnce];
        int32_t u[kAtOnce];
#pragma unroll
        for (int j = 0; j < kAtOnce; ++j) {
            take[j] = lane < (d[j] < k ? d[j] : k);
            u[j] = take[j] ? indices[beg[j] + pos[j]] : 0;
        }
        if (DRAWS) {
#pragma unroll
            for (int j = 0; j < kAtOnce; ++j)
                if (take[j]) {
                    const uint32_t cell = ((uint32_t)u[j] * 0x9E3779B1u) >> 22;          // kPrivCells = 2^10
                    const uint32_t was = atomicCAS(&s_priv_key[cell], 0xffffffffu, (uint32_t)u[j]);
                    if (was == 0xffffffffu || was == (uint32_t)u[j]) atomicAdd(&s_priv_cnt[cell], 1u);
                    else atomicAdd(&w.draws[u[j]], 1u);
                }
            if (last) continue;                       // nothing is listed after the last hop, and nothing marked
        }
        if (MODE == MODE_COUNT_SMALL) {
            // one bit per node: in the frontier already?  `prev` does not change during the hop, so
            // the words of the hubs, which most edges lead to, stay in the compute unit's own cache
            uint32_t old[kAtOnce];
#pragma unroll
            for (int j = 0; j < kAtOnce; ++j) old[j] = take[j] ? v.aux[(uint32_t)u[j] >> 5] : 0xffffffffu;
#pragma unroll
            for (int j = 0; j < kAtOnce; ++j) {
                const uint32_t bit = 1u << (u[j] & 31);
                if (!(old[j] & bit)) atomicOr(&v.fresh[(uint32_t)u[j] >> 5], bit);
            }
            continue;
        }
        // stage 4: in the frontier already?  home cell of the index, then the key it points to
        uint32_t h[kAtOnce], cell[kAtOnce];
#pragma unroll
        for (int j = 0; j < kAtOnce; ++j) {
            h[j] = home_of((uint32_t)u[j], w.table_log2);
            cell[j] = take[j] ? v.table[h[j]] : 0u;
        }
        int32_t key[kAtOnce];
#pragma unroll
        for (int j = 0; j < kAtOnce; ++j) key[j] = cell[j] ? v.nodes[cell[j] - 1u] : -1;
        // stage 5: results
#pragma unroll
        for (int j = 0; j < kAtOnce; ++j) {
            if (MODE == MODE_COUNT_LARGE && dense_col && !take[j] && lane < k && i0 + j * sweep < n)
                dense_col[(i0 + j * sweep) * k + lane] = 0;      // no draw here
            if (!take[j]) continue;
            int32_t at = -1;
            if (cell[j]) {
                at = (int32_t)(cell[j] - 1u);
                if (key[j] != u[j]) {                            // another node's cell: walk on (rare)
                    uint32_t hh = h[j];
                    for (;;) {
                        hh = (hh + 1u) & mask;
                        const uint32_t c2 = v.table[hh];
                        if (c2 == 0u) { at = -1; break; }
                        if (v.nodes[c2 - 1u] == u[j]) { at = (int32_t)(c2 - 1u); break; }
                    }
                }
            }
            if (MODE == MODE_BLOCKS) {
                eid[rp[j] + lane] = beg[j] + pos[j];
                col[rp[j] + lane] = at >= 0 ? at : ~u[j];        // negative: new at this hop; its place comes later
            }
            if (MODE == MODE_COUNT_LARGE && dense_col) dense_col[(i0 + j * sweep) * k + lane] = at >= 0 ? 0 : ~u[j];
            if (at < 0 && mark) {                                // mark == 0: the k_part_* kernels read ~node from col[]
                const uint32_t word = (uint32_t)u[j] >> 5, bit = 1u << (u[j] & 31);
                if (MODE == MODE_COUNT_LARGE && last) {
                    atomicOr(&v.aux[word], bit);                 // nobody lists the last hop's nodes: straight into `all`
                } else {
                    atomicOr(&v.fresh[word], bit);
                    v.flag[word] = 1;
                }
            }
        }
    }
    if (MODE != MODE_BLOCKS && w.count_edges) {
        int tot = block_sum(edges, s_wave);
        if (threadIdx.x == 0 && tot)
            atomicAdd((unsigned long long *)&w.meta[META_TOTAL_EDGES], (unsigned long long)tot);
    }
    if (DRAWS) {
        __syncthreads();
        for (int i = threadIdx.x; i < kPrivCells; i += kBlock)
            if (s_priv_cnt[i]) atomicAdd(&w.draws[s_priv_key[i]], s_priv_cnt[i]);
    }
}

// ---- walking the flagged words (bitmap layout: graphs of up to 32 M nodes) -----------------------
// A flag byte per bitmap word says whether the hop set a bit in it, so the kernels below read one
// byte per 32 nodes and touch only flagged words: their cost follows the mini-batch, not the graph.

// Popcounts of the flagged words, summed per block (for the scan over blocks).
__global__ __launch_bounds__(kBlock) void k_bm_partial(wide_t w, int gx)
{
    __shared__ int s_wave[kBlock / 64];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int64_t lo, hi;
    block_range(p, w.n_seg, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock)
        if (v.flag[i]) sum += __popc(v.fresh[i]);
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) v.partial_bm[p.bx] = tot;
}

// The new nodes of one bitmap word, ascending, to nodes[pos ..); keep == 0: each also enters the
// frontier index (first half: a plain store into an empty home cell).
__device__ inline int64_t emit_word(const slot_view &v, int table_log2, int64_t cap, int64_t word, uint32_t bits, int64_t pos,
                                    int keep)
{
    while (bits) {
        const int b = __ffs(bits) - 1;
        bits &= bits - 1;
        const int32_t u = (int32_t)(word * 32 + b);
        if (pos >= cap) break;                       // only after repeated seeds (an error the call reports)
        v.nodes[pos] = u;
        if (!keep) {
            const uint32_t h = home_of((uint32_t)u, table_log2);
            if (v.table[h] == 0u) v.table[h] = (uint32_t)pos + 1u;      // may lose to another store: k_settle
        }
        ++pos;
    }
    return pos;
}

// The nodes reached at hop `layer`, ascending, appended to the frontier.  keep == 0: they will
// draw at the next hop, so they enter the frontier index (k_settle settles contested cells)
// and the word's bits and flag are cleared for the next hop.  keep != 0 (last hop): nothing
// draws from them; the word's start position is recorded for k_relabel and the bits stay until
// k_finish.
__global__ __launch_bounds__(kBlock) void k_bm_emit(wide_t w, int gx, int layer, int keep, int64_t cap_next)
{
    __shared__ int s_wave[kBlock / 64];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int64_t lo, hi;
    block_range(p, w.n_seg, lo, hi);
    int carry, all;
    partial_prefix(p, v.partial_bm, carry, all, s_wave);
    const int64_t base = v.meta[META_NFRONT + layer];
    // cap_next = the bound of tier_blocks_bounds on the next frontier; only repeated seeds (an error
    // the call reports) can take the sum beyond it
    if (p.bx == 0 && threadIdx.x == 0) v.meta[META_NFRONT + layer + 1] = base + all < cap_next ? base + all : cap_next;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        const bool live = i < hi && v.flag[i] != 0;
        const uint32_t bits = live ? v.fresh[i] : 0u;
        int tot;
        const int before = carry + block_excl_scan(__popc(bits), tot, s_wave);
        carry += tot;
        if (live) {
            if (keep) {
                v.segbase[i] = before;
            } else {
                v.flag[i] = 0;
                v.fresh[i] = 0u;
            }
            emit_word(v, w.table_log2, cap_next, i, bits, base + before, keep);
        }
    }
}

// The frontier positions [n_layer, n_layer+1) that k_bm_emit (or k_bm_emit_flat) has just listed:
// their adjacency offsets and degrees go beside them, and (MODE with an index) a node whose home
// cell holds another node's position - an older entry, or the winner of this hop's plain stores -
// takes the next empty cell by compare-and-swap.  Cells never empty again within a mini-batch, so
// every node stays reachable from its home cell without a gap.
template <int MODE, typename OffT>
__global__ __launch_bounds__(kBlock) void k_settle(wide_t w, int gx, const OffT *__restrict__ indptr, int layer)
{
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int64_t lo = v.meta[META_NFRONT + layer], hi = v.meta[META_NFRONT + layer + 1];
    const uint32_t mask = (1u << w.table_log2) - 1u;
    for (int64_t pos = lo + (int64_t)p.bx * kBlock + threadIdx.x; pos < hi; pos += (int64_t)gx * kBlock) {
        const int32_t u = v.nodes[pos];
        const OffT first_edge = indptr[u];
        v.beg[pos] = (int64_t)first_edge;
        v.deg[pos] = (int32_t)(indptr[u + 1] - first_edge);
        if (MODE != MODE_COUNT_SMALL) {
            const uint32_t h = home_of((uint32_t)u, w.table_log2);
            if (v.table[h] != (uint32_t)pos + 1u) index_insert_cas(v.table, w.table_log2, (h + 1u) & mask, (uint32_t)pos);
        }
    }
}

// ---- block calls on the large-graph layout: buckets instead of the bitmap ------------------------
// On a graph of 10^8 nodes nearly every node that a hop reaches sits alone in its 128-byte line of
// `fresh`: an atomic to set the bit, then the line read again to count, to list, to relabel and to
// clear, and a walk over every segment's flag on top.  Instead k_hop_sample leaves ~node in col[]
// (as it does anyway) and sets nothing, and the hop's edges whose neighbour is new are sorted by
// node id into buckets of 2^bucket_log2 consecutive ids (at most 8192 buckets, a few dozen records
// each), with LDS atomics only:
//   k_part_hist     each of kPartBlocks blocks per slot counts its share of the edges per bucket
//   k_part_cols     per bucket: records of the blocks before each block, and of all blocks
//   k_part_scan     first record of every bucket
//   k_part_scatter  records (node, edge) to their bucket's range (order inside a bucket: any)
//   k_part_bucket   one wave sorts a window of whole buckets across its lanes -> distinct nodes,
//                   ascending, and the rank of every record's node among its bucket's
//   k_part_scan     distinct nodes before every bucket; size of the next frontier
//   k_part_final    final col[] of the records' edges (no k_relabel), the new nodes appended to
//                   the frontier and, unless it is the last hop, entered into the frontier index
// A slot's records, counts and lists stay in its XCD's L2 like the frontier index.  Measured on
// 111 M nodes, per new node: 32 ns this way, 190 ns through the bitmap.

// dense_k != 0 (access counting, which keeps no edge offsets): col[] holds dense_k entries for every
// dst node of the hop, ~node where a new node was drawn and 0 elsewhere.
__global__ __launch_bounds__(kBlock) void k_part_hist(wide_t w, int layer, int dense_k, layer_out_t o)
{
    extern __shared__ int s_bins[];
    spot_t p;
    if (!my_spot(w, kPartBlocks, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int32_t *col = o.col + (int64_t)p.slot * o.edge_stride;
    for (int i = threadIdx.x; i < w.n_buckets; i += kBlock) s_bins[i] = 0;
    __syncthreads();
    int64_t lo, hi;
    block_range(p, dense_k ? v.meta[META_NFRONT + layer] * dense_k : v.meta[META_NEDGES + layer], lo, hi);
    for (int64_t e0 = lo + threadIdx.x; e0 < hi; e0 += 4 * kBlock) {
        int32_t c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = e0 + j * kBlock < hi ? col[e0 + j * kBlock] : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c[j] < 0) atomicAdd(&s_bins[(uint32_t)~c[j] >> w.bucket_log2], 1);
    }
    __syncthreads();
    int32_t *row = v.rows + (int64_t)p.bx * w.n_buckets;
    for (int i = threadIdx.x; i < w.n_buckets; i += kBlock) row[i] = s_bins[i];
}

// One thread per bucket: rows[b][i] becomes the records of bucket i in the blocks before b, and
// bk_start[i] the records of bucket i in all blocks (k_part_scan turns them into start positions).
__global__ __launch_bounds__(kBlock) void k_part_cols(wide_t w, int gx)
{
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int i = p.bx * kBlock + threadIdx.x;
    if (i >= w.n_buckets) return;
    int32_t t[kPartBlocks];
#pragma unroll
    for (int b = 0; b < kPartBlocks; ++b) t[b] = v.rows[(int64_t)b * w.n_buckets + i];
    int32_t run = 0;
#pragma unroll
    for (int b = 0; b < kPartBlocks; ++b) {
        v.rows[(int64_t)b * w.n_buckets + i] = run;
        run += t[b];
    }
    v.bk_start[i] = run;
}

constexpr int kScanThreads = 1024;

// One block per slot, exclusive prefix sum over the buckets.  which == 0: bk_start[] in place (records
// per bucket -> first record), the total to bk_start[n_buckets].  which == 1: bk_cnt[] -> bk_before[],
// and the size of the final frontier (at most cap_next: the bound of tier_blocks_bounds; only
// repeated seeds, which the call reports, can take the sum beyond it).
__global__ __launch_bounds__(kScanThreads) void k_part_scan(wide_t w, int which, int layer, int64_t cap_next)
{
    __shared__ int s_wave[kScanThreads / 64];
    spot_t p;
    if (!my_spot(w, 1, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int32_t *in = which ? v.bk_cnt : v.bk_start;
    int32_t *out = which ? v.bk_before : v.bk_start;
    const int nb = w.n_buckets;
    int carry = 0;
    for (int tile = 0; tile < nb; tile += 4 * kScanThreads) {
        const int first = tile + 4 * (int)threadIdx.x;
        int x[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[j] = first + j < nb ? in[first + j] : 0;
            sum += x[j];
        }
        int tot;
        int run = carry + block_excl_scan_n<kScanThreads / 64>(sum, tot, s_wave);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (first + j < nb) out[first + j] = run;
            run += x[j];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) {
        if (which == 0) {
            out[nb] = carry;
        } else {
            const int64_t base = v.meta[META_NFRONT + layer];
            v.meta[META_NFRONT + layer + 1] = base + carry < cap_next ? base + carry : cap_next;
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_part_scatter(wide_t w, int layer, int dense_k, layer_out_t o)
{
    extern __shared__ int s_bins[];
    spot_t p;
    if (!my_spot(w, kPartBlocks, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int32_t *col = o.col + (int64_t)p.slot * o.edge_stride;
    const int32_t *row = v.rows + (int64_t)p.bx * w.n_buckets;
    for (int i = threadIdx.x; i < w.n_buckets; i += kBlock) s_bins[i] = v.bk_start[i] + row[i];
    __syncthreads();
    int64_t lo, hi;
    block_range(p, dense_k ? v.meta[META_NFRONT + layer] * dense_k : v.meta[META_NEDGES + layer], lo, hi);   // as in k_part_hist
    for (int64_t e0 = lo + threadIdx.x; e0 < hi; e0 += 4 * kBlock) {
        int32_t c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = e0 + j * kBlock < hi ? col[e0 + j * kBlock] : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c[j] < 0) {
                const uint32_t u = (uint32_t)~c[j];
                const int at = atomicAdd(&s_bins[u >> w.bucket_log2], 1);
                v.rec[at] = ((unsigned long long)u << 32) | (uint32_t)(e0 + j * kBlock);
            }
    }
}

// One bucket with more than 64 records (a node that many edges of the hop lead to): the nodes of its
// records as bits of an LDS bitmap over the bucket's id range; per-word prefix counts give every
// record's node its rank among the bucket's distinct nodes, and the set bits, in order, are those
// nodes.  Called by the whole block (one wave) at once.
__device__ inline void bucket_by_bitmap(const wide_t &w, const slot_view &v, int q, int lo, int hi, uint32_t *bits,
                                        uint32_t *before, int n_words)
{
    const int lane = threadIdx.x;
    const uint32_t id_mask = (1u << w.bucket_log2) - 1u;
    const int per_lane = (n_words + 63) / 64;
    const int first = lane * per_lane;
    for (int i = lane; i < n_words; i += 64) bits[i] = 0u;
    __syncthreads();
    for (int r = lo + lane; r < hi; r += 64) {
        const uint32_t local = (uint32_t)(v.rec[r] >> 32) & id_mask;
        atomicOr(&bits[local >> 5], 1u << (local & 31));
    }
    __syncthreads();
    int mine = 0;
    for (int j = 0; j < per_lane; ++j)
        if (first + j < n_words) mine += __popc(bits[first + j]);
    const int incl = wave_incl_scan(mine);
    const int total = __shfl(incl, 63);
    int run = incl - mine;
    int32_t at = lo + run;                                           // distinct nodes <= records: they fit from lo on
    for (int j = 0; j < per_lane; ++j)
        if (first + j < n_words) {
            uint32_t x = bits[first + j];
            before[first + j] = (uint32_t)run;
            run += __popc(x);
            while (x) {
                const int b = __ffs(x) - 1;
                x &= x - 1;
                v.stage[at++] = (int32_t)(((uint32_t)q << w.bucket_log2) + (uint32_t)(first + j) * 32u + (uint32_t)b);
            }
        }
    if (lane == 0) v.bk_cnt[q] = total;
    __syncthreads();
    for (int r = lo + lane; r < hi; r += 64) {
        const uint32_t local = (uint32_t)(v.rec[r] >> 32) & id_mask;
        v.lrank[r] = (int32_t)(before[local >> 5] + __popc(bits[local >> 5] & ((1u << (local & 31)) - 1u)));
    }
    __syncthreads();                                                 // before another bucket clears the bitmap
}

// Ascending bitonic sort of one key per lane over the 64 lanes of a wave.
__device__ inline uint32_t wave_sort(uint32_t key)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const uint32_t other = (uint32_t)__shfl_xor((int)key, j);
            const bool rising = (lane & k) == 0;                     // k == 64: the whole wave
            const bool lower = (lane & j) == 0;
            const uint32_t mn = key < other ? key : other, mx = key < other ? other : key;
            key = lower == rising ? mn : mx;
        }
    }
    return key;
}

// A block of one wave takes kBucketsPerWave consecutive buckets at a time (their bounds with one
// load) and goes through them in windows of whole buckets with at most 64 records together, the
// usual case being several buckets per window: lane i takes record i of the window, the wave sorts
// (node, lane) pairs, and in sorted order a node is new where it differs from its left neighbour, a
// bucket begins where the bucket number does; the rank of a record's node among its bucket's distinct
// nodes is the number of new nodes between the bucket's first lane and its own.  A bucket with more
// than 64 records of its own goes through the LDS bitmap (2 x n_words words).
constexpr int kBucketsPerWave = 8;

__global__ __launch_bounds__(64) void k_part_bucket(wide_t w, int gx, int n_words)
{
    extern __shared__ uint32_t s_mem[];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int lane = threadIdx.x;
    const int nb = w.n_buckets;
    const int b = w.bucket_log2;
    const int n_groups = (nb + kBucketsPerWave - 1) / kBucketsPerWave;
    const unsigned long long through_me = (2ull << lane) - 1ull;    // lanes 0 .. lane
    for (int g = p.bx; g < n_groups; g += gx) {                      // g and every branch on scalars below: the same for all lanes
        const int q0 = g * kBucketsPerWave;
        int bound = q0 + lane;                                       // lanes 0..8: where the group's buckets begin and end
        bound = bound < nb ? bound : nb;
        const int my_start = lane <= kBucketsPerWave ? v.bk_start[bound] : 0;
        const int next_start = __shfl_down(my_start, 1);
        // empty buckets have no lane of their own below
        if (lane < kBucketsPerWave && q0 + lane < nb && next_start == my_start) v.bk_cnt[q0 + lane] = 0;
        auto lo = [&](int j) { return __builtin_amdgcn_readlane(my_start, j); };   // first record of bucket q0 + j
        int j = 0;
        while (j < kBucketsPerWave && q0 + j < nb) {
            if (lo(j + 1) - lo(j) > 64) {
                bucket_by_bitmap(w, v, q0 + j, lo(j), lo(j + 1), s_mem, s_mem + n_words, n_words);
                ++j;
                continue;
            }
            int end = j + 1;                                         // window = buckets j .. end - 1
            while (end < kBucketsPerWave && lo(end + 1) - lo(j) <= 64) ++end;
            const int first = lo(j), n = lo(end) - first;
            const int q_first = q0 + j;
            j = end;
            if (n == 0) continue;
            // (node - first id of the window's first bucket) << 6 | lane: below 2^(bucket_log2 + 3 + 6) <= 2^27
            uint32_t key = 0xffffffffu;                              // lanes beyond the records sort to the end
            if (lane < n) key = ((((uint32_t)(v.rec[first + lane] >> 32)) - ((uint32_t)q_first << b)) << 6) | (uint32_t)lane;
            key = wave_sort(key);
            const bool there = key != 0xffffffffu;
            const uint32_t local = key >> 6;                         // node, counted from the window's first id
            const int from = (int)(key & 63u);                       // the record is number `from` of the window
            const uint32_t left = (uint32_t)__shfl_up((int)local, 1);
            const bool new_node = there && (lane == 0 || left != local);
            const bool new_bucket = there && (lane == 0 || (left >> b) != (local >> b));
            const unsigned long long nodes_mask = __ballot(new_node), buckets_mask = __ballot(new_bucket);
            if (there) {
                const int begin = 63 - __clzll(buckets_mask & through_me);             // first lane of my bucket
                const unsigned long long mine = nodes_mask & ~((1ull << begin) - 1ull);    // new nodes from there on
                const int rank = __popcll(mine & through_me) - 1;
                v.lrank[first + from] = rank;
                if (new_node) v.stage[first + begin + rank] = (int32_t)(local + ((uint32_t)q_first << b));
                if (new_bucket) {                                    // distinct nodes of the bucket: up to the next bucket's first lane
                    const unsigned long long later = buckets_mask & ~through_me;
                    const int stop = later ? __ffsll((long long)later) - 1 : 64;
                    const unsigned long long upto = stop == 64 ? ~0ull : (1ull << stop) - 1ull;
                    v.bk_cnt[q_first + (int)(local >> b)] = __popcll(mine & upto);
                }
            }
        }
    }
}

// One thread per record: col[] of its edge, and (the first `distinct` records of a bucket) one of the
// bucket's nodes to its place in the frontier.
// insert != 0 (not the last hop): the nodes will draw, so they enter the frontier index as in k_bm_emit
// (a plain store into an empty home cell; k_settle settles contested cells).
// counting != 0 (access counting): col[] is scratch and stays as it is, and the new nodes join `all`.
__global__ __launch_bounds__(kBlock) void k_part_final(wide_t w, int gx, int layer, int64_t cap_next, int insert, int counting,
                                                     layer_out_t o)
{
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int32_t *col = o.col + (int64_t)p.slot * o.edge_stride;
    const int64_t n_rec = v.bk_start[w.n_buckets];
    const int64_t hop_base = v.meta[META_NFRONT + layer];
    for (int64_t r = (int64_t)p.bx * kBlock + threadIdx.x; r < n_rec; r += (int64_t)gx * kBlock) {
        const unsigned long long rec = v.rec[r];
        const uint32_t q = (uint32_t)(rec >> 32) >> w.bucket_log2;
        const int64_t place = hop_base + v.bk_before[q];
        if (!counting) col[(uint32_t)rec] = (int32_t)(place + v.lrank[r]);
        const int64_t i = r - v.bk_start[q];
        if (i < v.bk_cnt[q] && place + i < cap_next) {
            const int32_t u = v.stage[r];
            v.nodes[place + i] = u;
            if (counting) atomicOr(&v.aux[(uint32_t)u >> 5], 1u << (u & 31));
            if (insert) {
                const uint32_t h = home_of((uint32_t)u, w.table_log2);
                if (v.table[h] == 0u) v.table[h] = (uint32_t)(place + i) + 1u;   // may lose to another store: k_settle
            }
        }
    }
}

// Flat variant for access counting on graphs whose whole bitmap is cheap to walk: every thread
// owns one bitmap word; new = seen ^ prev, then prev = seen.
__global__ __launch_bounds__(kBlock) void k_bm_partial_flat(wide_t w, int gx)
{
    __shared__ int s_wave[kBlock / 64];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int64_t lo, hi;
    block_range(p, w.n_words, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) sum += __popc(v.fresh[i] ^ v.aux[i]);
    int tot = block_sum(sum, s_wave);
    if (threadIdx.x == 0) v.partial_bm[p.bx] = tot;
}

__global__ __launch_bounds__(kBlock) void k_bm_emit_flat(wide_t w, int gx, int layer, int64_t cap_next)
{
    __shared__ int s_wave[kBlock / 64];
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    int64_t lo, hi;
    block_range(p, w.n_words, lo, hi);
    int carry, all;
    partial_prefix(p, v.partial_bm, carry, all, s_wave);
    const int64_t base = v.meta[META_NFRONT + layer];
    // cap_next = the bound of tier_blocks_bounds on the next frontier; only repeated seeds (an error
    // the call reports) can take the sum beyond it
    if (p.bx == 0 && threadIdx.x == 0) v.meta[META_NFRONT + layer + 1] = base + all < cap_next ? base + all : cap_next;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        const uint32_t cur = i < hi ? v.fresh[i] : 0u;
        uint32_t bits = i < hi ? cur ^ v.aux[i] : 0u;
        int tot;
        int64_t pos = base + carry + block_excl_scan(__popc(bits), tot, s_wave);
        carry += tot;
        if (bits) {
            v.aux[i] = cur;
            while (bits) {
                int b = __ffs(bits) - 1;
                bits &= bits - 1;
                if (pos < cap_next) v.nodes[pos] = (int32_t)(i * 32 + b);
                ++pos;
            }
        }
    }
}

// Access counting, end of a chain: one bitmap of every slot now holds the whole final frontier
// of its mini-batch (`seen` on the smaller graphs, `all` above), so counts[v] grows by the
// number of slots whose bit v is set.  One thread owns one bitmap word position = 32 counters
// across all slots: it adds the slots' words bit-sliced (five planes hold sums up to 31; a flush
// every 31 slots), updates its counters without atomics (no other thread of this kernel touches
// them, and kernels on the stream run one after the other) and clears the bitmaps.
__global__ __launch_bounds__(kBlock) void k_count_columns(wide_t w, int large, uint32_t *__restrict__ counts)
{
    __shared__ int s_wave[kBlock / 64];
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int rows = 0;
    if (i < w.n_words) {
        uint32_t plane[5] = {0u, 0u, 0u, 0u, 0u};
        int held = 0;
        auto flush = [&]() {
            if (counts && (plane[0] | plane[1] | plane[2] | plane[3] | plane[4])) {    // no counts: the bitmaps are only cleared
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
            for (int q = 0; q < 5; ++q) plane[q] = 0u;
            held = 0;
        };
        uint32_t *column = (large ? w.aux : w.fresh) + i;
        for (int s0 = 0; s0 < w.n_slots; s0 += 8) {                // eight slots' words in flight at a time
            uint32_t x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = s0 + j < w.n_slots ? column[(int64_t)(s0 + j) * w.bm_stride] : 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t carry = x[j];
                if (carry) {
                    column[(int64_t)(s0 + j) * w.bm_stride] = 0u;
                    if (!large) w.aux[(int64_t)(s0 + j) * w.bm_stride + i] = 0u;
                    rows += __popc(carry);
#pragma unroll
                    for (int q = 0; q < 5; ++q) {                 // ripple-carry add of one bit per column
                        const uint32_t t = plane[q] & carry;
                        plane[q] ^= carry;
                        carry = t;
                    }
                    if (++held == 31) flush();
                }
            }
        }
        flush();
    }
    const int tot = block_sum(rows, s_wave);
    if (threadIdx.x == 0 && tot)
        atomicAdd((unsigned long long *)&w.meta[META_TOTAL_ROWS], (unsigned long long)tot);
}

// Block calls by the bitmap (one word per segment): col[e] of the sampled neighbours that were not
// in the frontier when they were drawn (k_hop_sample left ~node there).  New at a hop that is not
// the last: the node has entered the index since.  New at the last hop: its position is the
// frontier size before the hop + the new nodes listed before its word + the bits below its own
// (the bitmap still holds the hop's bits).
__global__ __launch_bounds__(kBlock) void k_relabel(wide_t w, int gx, relabel_t r)
{
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int64_t stride = (int64_t)gx * kBlock;
    const int64_t t = (int64_t)p.bx * kBlock + threadIdx.x;
    for (int l = 0; l < r.n_layers; ++l) {
        int32_t *col = r.col[l] + (int64_t)p.slot * r.stride[l];
        const int64_t n = v.meta[META_NEDGES + l];
        const bool last = l == r.n_layers - 1;
        const int32_t before_hop = (int32_t)v.meta[META_NFRONT + l];
        if (!last) {
            for (int64_t e = t; e < n; e += stride) {
                const int32_t c = col[e];
                if (c < 0) col[e] = index_of(v.table, w.table_log2, v.nodes, ~c);
            }
        } else {
            for (int64_t e = t; e < n; e += stride) {
                const int32_t c = col[e];
                if (c >= 0) continue;
                const int32_t u = ~c;
                const int64_t word = (uint32_t)u >> 5;
                col[e] = before_hop + v.segbase[word] + __popc(v.fresh[word] & ((1u << (u & 31)) - 1u));
            }
        }
    }
}

// End of a mini-batch: the frontier index back to all empty, and (block calls by the bitmap, one
// word per segment) the bits and flags that the last hop left in place for k_relabel.
__global__ __launch_bounds__(kBlock) void k_finish(wide_t w, int gx, int clear_fresh)
{
    spot_t p;
    if (!my_spot(w, gx, p)) return;
    const slot_view v = view_of(w, p.slot);
    const int64_t stride = (int64_t)gx * kBlock;
    const int64_t t = (int64_t)p.bx * kBlock + threadIdx.x;
    uint4 *cells = (uint4 *)v.table;                              // a slot's table is a multiple of 1024 cells
    const int64_t n_cells4 = (1ll << w.table_log2) / 4;
    for (int64_t i = t; i < n_cells4; i += stride) cells[i] = make_uint4(0u, 0u, 0u, 0u);
    if (!clear_fresh) return;
    for (int64_t i = t; i < w.n_seg; i += stride)
        if (v.flag[i]) {
            v.flag[i] = 0;
            v.fresh[i] = 0u;
        }
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

// Blocks per slot of the kernels whose blocks loop over their slot's items.  The bounds the grids are
// sized from are several times the real sizes (degrees below the fanout, repeated neighbours), and a
// slot is served by one XCD, which holds 256 blocks at a time: more blocks than twice that only queue
// up to find nothing to do (measured best of 128 / 256 / 512 / 1024 and no cap).
constexpr int kLoopBlocks = 512;
constexpr int kBucketBlocks = 1024;  // one-wave blocks per slot of k_part_bucket

int clamp_grid(int64_t items, int per_block, int cap)
{
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

// Workgroups of a launch that gives every slot gx blocks (see my_spot).
unsigned grid_of(int gx, int n_slots) { return (unsigned)(kXcds * gx * ((n_slots + kXcds - 1) / kXcds)); }

struct wide_out {             // where the mini-batches' results go
    layer_out_t layer[TIER_MAX_LAYERS];
    uint32_t *counts;         // access counting: where the final frontiers are counted
};

// With 32 words per segment (the layout of graphs above 32 M nodes) access counting uses the index.
bool large_graph(const tier_ctx *c) { return c->seg_log2 != 0; }

template <int G, int MODE>
void launch_hop_sample(tier_ctx *c, const wide_t &w, int64_t cap_dst, int layer, int k, bool last, bool mark,
                       const wide_out &o)
{
    const int gx = clamp_grid(cap_dst, (kBlock / G) * kAtOnce, kLoopBlocks);
    if (MODE != MODE_BLOCKS && w.draws)
        k_hop_sample<G, MODE == MODE_BLOCKS ? MODE_COUNT_SMALL : MODE, true><<<grid_of(gx, w.n_slots), kBlock, 0, c->stream>>>(
            w, gx, c->indices, layer, k, last ? 1 : 0, mark ? 1 : 0, o.layer[layer]);
    else
        k_hop_sample<G, MODE, false><<<grid_of(gx, w.n_slots), kBlock, 0, c->stream>>>(
            w, gx, c->indices, layer, k, last ? 1 : 0, mark ? 1 : 0, o.layer[layer]);
}

template <int MODE>
void launch_hop(tier_ctx *c, const wide_t &w, int64_t cap_dst, int layer, int k, bool last, bool mark, const wide_out &o)
{
    if (MODE == MODE_BLOCKS) {
        const int gx = clamp_grid(cap_dst, kBlock, kLoopBlocks);
        const unsigned grid = grid_of(gx, w.n_slots);
        k_hop_partial<<<grid, kBlock, 0, c->stream>>>(w, gx, layer, k);
        k_hop_rowptr<<<grid, kBlock, 0, c->stream>>>(w, gx, layer, k, o.layer[layer]);
    }
    if (k <= 4) launch_hop_sample<4, MODE>(c, w, cap_dst, layer, k, last, mark, o);
    else if (k <= 8) launch_hop_sample<8, MODE>(c, w, cap_dst, layer, k, last, mark, o);
    else if (k <= 16) launch_hop_sample<16, MODE>(c, w, cap_dst, layer, k, last, mark, o);
    else if (k <= 32) launch_hop_sample<32, MODE>(c, w, cap_dst, layer, k, last, mark, o);
    else launch_hop_sample<64, MODE>(c, w, cap_dst, layer, k, last, mark, o);
}

// Enqueue w.n_slots mini-batches.  cap_nodes / cap_edges: the bounds of tier_blocks_bounds
// for one mini-batch of w.batch_size seeds.
template <int MODE, typename OffT>
int enqueue_wide_t(tier_ctx *c, const wide_t &w, const int32_t *fanouts, int n_layers, const int64_t *cap_nodes,
                   const int64_t *cap_edges, const wide_out &o)
{
    const int slots = w.n_slots;
    hipStream_t st = c->stream;
    const OffT *indptr = (const OffT *)c->indptr;
    {
        const int gx = clamp_grid(w.batch_size, kBlock, 1 << 16);
        k_init_seeds<MODE, OffT><<<grid_of(gx, slots), kBlock, 0, st>>>(w, gx, indptr);
    }
    const int seg_gx = clamp_grid(w.n_seg, kBlock, TIER_SCAN_BLOCKS);
    const int flat_gx = clamp_grid(w.n_words, 4 * kBlock, TIER_SCAN_BLOCKS);
    // on the large-graph layout the new nodes of a hop are listed by buckets (k_part_*), not by the bitmap
    const bool by_buckets = MODE != MODE_COUNT_SMALL && w.n_buckets > 0;
    const bool counting = MODE != MODE_BLOCKS;
    for (int l = 0; l < n_layers; ++l) {
        const bool last = l == n_layers - 1;
        launch_hop<MODE>(c, w, cap_nodes[l], l, fanouts[l], last, !by_buckets || (counting && last), o);
        if (MODE != MODE_BLOCKS && last) break;               // counted from the bitmaps, never listed
        if (by_buckets) {
            const int dense_k = counting ? fanouts[l] : 0;
            const int nb = w.n_buckets;
            const size_t bins = (size_t)nb * sizeof(int);
            const int n_words = w.bucket_log2 > 5 ? 1 << (w.bucket_log2 - 5) : 1;
            const unsigned part_grid = grid_of(kPartBlocks, slots);
            k_part_hist<<<part_grid, kBlock, bins, st>>>(w, l, dense_k, o.layer[l]);
            const int cols_gx = clamp_grid(nb, kBlock, 1 << 16);
            k_part_cols<<<grid_of(cols_gx, slots), kBlock, 0, st>>>(w, cols_gx);
            k_part_scan<<<grid_of(1, slots), kScanThreads, 0, st>>>(w, 0, l, cap_nodes[l + 1]);
            k_part_scatter<<<part_grid, kBlock, bins, st>>>(w, l, dense_k, o.layer[l]);
            const int bucket_gx = clamp_grid(nb, kBucketsPerWave, kBucketBlocks);
            k_part_bucket<<<grid_of(bucket_gx, slots), 64, 2 * (size_t)n_words * sizeof(uint32_t), st>>>(w, bucket_gx, n_words);
            k_part_scan<<<grid_of(1, slots), kScanThreads, 0, st>>>(w, 1, l, cap_nodes[l + 1]);
            const int final_gx = clamp_grid(cap_edges[l], kBlock, kLoopBlocks);
            k_part_final<<<grid_of(final_gx, slots), kBlock, 0, st>>>(w, final_gx, l, cap_nodes[l + 1], last ? 0 : 1,
                                                                      counting ? 1 : 0, o.layer[l]);
        } else if (MODE == MODE_COUNT_SMALL) {
            k_bm_partial_flat<<<grid_of(flat_gx, slots), kBlock, 0, st>>>(w, flat_gx);
            k_bm_emit_flat<<<grid_of(flat_gx, slots), kBlock, 0, st>>>(w, flat_gx, l, cap_nodes[l + 1]);
        } else {
            k_bm_partial<<<grid_of(seg_gx, slots), kBlock, 0, st>>>(w, seg_gx);
            k_bm_emit<<<grid_of(seg_gx, slots), kBlock, 0, st>>>(w, seg_gx, l, last ? 1 : 0, cap_nodes[l + 1]);
        }
        if (!last) {
            const int gx = clamp_grid(cap_nodes[l + 1], kBlock, kLoopBlocks);
            k_settle<MODE, OffT><<<grid_of(gx, slots), kBlock, 0, st>>>(w, gx, indptr, l);
        }
    }
    if (MODE == MODE_BLOCKS) {
        relabel_t r = {};
        r.n_layers = n_layers;
        int64_t most = 1;
        for (int l = 0; l < n_layers; ++l) {
            r.col[l] = o.layer[l].col;
            r.stride[l] = o.layer[l].edge_stride;
            if (cap_edges[l] > most) most = cap_edges[l];
        }
        const int gx = clamp_grid(most, kBlock, kLoopBlocks);
        if (!by_buckets) k_relabel<<<grid_of(gx, slots), kBlock, 0, st>>>(w, gx, r);      // k_part_final writes final col[]
    } else {
        // tier_presample_draws has counted on the way: only the bitmaps are cleared
        k_count_columns<<<clamp_grid(c->n_words, kBlock, 1 << 22), kBlock, 0, st>>>(w, MODE == MODE_COUNT_LARGE ? 1 : 0,
                                                                                 w.draws ? nullptr : o.counts);
    }
    if (MODE != MODE_COUNT_SMALL) {
        const int64_t cells4 = (1ll << w.table_log2) / 4;
        const int gx = clamp_grid(cells4 > w.n_seg ? cells4 : w.n_seg, 4 * kBlock, kLoopBlocks);
        k_finish<<<grid_of(gx, slots), kBlock, 0, st>>>(w, gx, MODE == MODE_BLOCKS && !by_buckets ? 1 : 0);
    }
    TIER_HIP(c, hipGetLastError());
    return TIER_OK;
}

template <int MODE>
int enqueue_wide(tier_ctx *c, const wide_t &w, const int32_t *fanouts, int n_layers, const int64_t *cap_nodes,
                 const int64_t *cap_edges, const wide_out &o)
{
    return c->indptr_i64 ? enqueue_wide_t<MODE, int64_t>(c, w, fanouts, n_layers, cap_nodes, cap_edges, o)
                         : enqueue_wide_t<MODE, int32_t>(c, w, fanouts, n_layers, cap_nodes, cap_edges, o);
}

// Offsets and degrees of the frontier nodes that draw: `per_slot` entries for every slot.
int ensure_degrees(tier_ctx *c, int64_t per_slot)
{
    const size_t n = (size_t)per_slot * (size_t)c->n_slots;
    int rc = tier_ensure(c, (void **)&c->f_beg, &c->f_beg_cap, n * sizeof(int64_t));
    if (rc == TIER_OK) rc = tier_ensure(c, (void **)&c->f_deg, &c->f_deg_cap, n * sizeof(int32_t));
    return rc;
}

// The frontier index of a call: room for twice the largest frontier that draws (cap_nodes of the
// last hop's dst side), a power of two of at least 1024 cells per slot; zero between calls.
int ensure_table(tier_ctx *c, int64_t most_members, int *table_log2)
{
    int lg = 10;
    while ((1ll << lg) < 2 * most_members) ++lg;
    if (lg > 31) return TIER_EINVAL;
    const size_t bytes = ((size_t)c->n_slots << lg) * sizeof(uint32_t);
    if (!c->table || c->table_cap < bytes) {
        int rc = tier_ensure(c, (void **)&c->table, &c->table_cap, bytes);
        if (rc != TIER_OK) return rc;
        k_fill_u32<<<4096, kBlock, 0, c->stream>>>(c->table, (int64_t)(bytes / sizeof(uint32_t)), 0u);
        TIER_HIP(c, hipGetLastError());
    }
    *table_log2 = lg;
    return TIER_OK;
}

wide_t make_wide(tier_ctx *c, const int32_t *seeds, int64_t n_seeds_total, int32_t batch_size, int32_t n_slots,
                 int32_t *nodes, int64_t nodes_stride, int table_log2, int64_t deg_stride)
{
    wide_t w = {};
    w.seeds = seeds;
    w.n_seeds_total = n_seeds_total;
    w.batch_size = batch_size;
    w.n_slots = n_slots;
    w.n_nodes = c->n_nodes;
    w.n_words = c->n_words;
    w.bm_stride = c->bm_stride;
    w.n_seg = c->n_seg;
    w.flag_stride = c->flag_stride;
    w.seg_log2 = c->seg_log2;
    w.nodes = nodes;
    w.nodes_stride = nodes_stride;
    w.fresh = c->fresh;
    w.aux = c->aux;
    w.flag = c->flag;
    w.segbase = c->segbase;
    w.table = c->table;
    w.table_log2 = table_log2;
    w.beg = c->f_beg;
    w.deg = c->f_deg;
    w.deg_stride = deg_stride;
    w.meta = c->meta;
    w.partial_hop = c->partial_hop;
    w.partial_bm = c->partial_bm;
    return w;
}

// Scratch of the last hop by buckets for a call of n_slots mini-batches with at most `edges` edges each
// at that hop.  A bucket is 2^b consecutive ids with b such that there are at most 8192 buckets
// (their counters fit a block's LDS) and b >= 5 (a bucket is at least one bitmap word).
int ensure_buckets(tier_ctx *c, wide_t *w, int64_t edges, int n_slots)
{
    int lg = 0;
    while ((1ll << lg) < c->n_nodes) ++lg;
    const int b = lg - 13 > 5 ? lg - 13 : 5;
    const int64_t nb = (c->n_nodes + (1ll << b) - 1) >> b;
    if (nb < 1) return TIER_OK;                                  // no nodes: nothing to sort
    const size_t per = (size_t)(edges > 0 ? edges : 1) * (size_t)n_slots;
    int rc = tier_ensure(c, (void **)&c->part_rec, &c->part_rec_cap, per * sizeof(unsigned long long));
    if (rc == TIER_OK) rc = tier_ensure(c, (void **)&c->part_rank, &c->part_rank_cap, per * sizeof(int32_t));
    if (rc == TIER_OK) rc = tier_ensure(c, (void **)&c->part_stage, &c->part_stage_cap, per * sizeof(int32_t));
    if (rc == TIER_OK)
        rc = tier_ensure(c, (void **)&c->part_rows, &c->part_rows_cap,
                         (size_t)n_slots * kPartBlocks * (size_t)nb * sizeof(int32_t));
    if (rc == TIER_OK)
        rc = tier_ensure(c, (void **)&c->part_bk, &c->part_bk_cap, (size_t)n_slots * 3 * (size_t)(nb + 1) * sizeof(int32_t));
    if (rc) return rc;
    w->rec = c->part_rec;
    w->lrank = c->part_rank;
    w->stage = c->part_stage;
    w->rec_stride = edges > 0 ? edges : 1;
    w->rows = c->part_rows;
    w->bk = c->part_bk;
    w->n_buckets = (int32_t)nb;
    w->bucket_log2 = b;
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
    for (int l = 0; l < n_layers; ++l) {
        if (!out->row_ptr[l] || !out->col[l] || !out->eid[l]) return TIER_EINVAL;
        if (out->row_ptr_stride[l] < cap_nodes[l] + 1 || out->edge_stride[l] < cap_edges[l]) return TIER_ECAPACITY;
        o.layer[l] = layer_out_t{out->row_ptr[l], out->row_ptr_stride[l], out->col[l], out->eid[l],
                                 out->edge_stride[l]};
    }
    int table_log2 = 0;
    rc = ensure_table(ctx, cap_nodes[n_layers - 1], &table_log2);
    const int64_t drawing = cap_nodes[n_layers - 1] > 0 ? cap_nodes[n_layers - 1] : 1;    // nodes that draw at the last hop
    if (rc == TIER_OK) rc = ensure_degrees(ctx, drawing);
    if (rc) return rc;
    wide_t w = make_wide(ctx, seeds, n_seeds_total, batch_size, n_batches, out->nodes, out->nodes_stride, table_log2,
                         drawing);
    for (int s = 0; s < n_batches; ++s) {
        w.key0[s] = (uint32_t)batch_seeds[s];
        w.key1[s] = (uint32_t)(batch_seeds[s] >> 32);
    }
    if (large_graph(ctx)) {
        int64_t most_edges = 0;                                  // any hop may go by buckets
        for (int l = 0; l < n_layers; ++l) most_edges = cap_edges[l] > most_edges ? cap_edges[l] : most_edges;
        rc = ensure_buckets(ctx, &w, most_edges, n_batches);
        if (rc) return rc;
    }
    rc = enqueue_wide<MODE_BLOCKS>(ctx, w, fanouts, n_layers, cap_nodes, cap_edges, o);
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

// The mini-batches [first_batch, first_batch + n_run) of every epoch; accumulate: counts[] is added to.
static int presample(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                     const int32_t *fanouts, int32_t n_layers, int32_t epochs, uint64_t seed, uint32_t *counts,
                     int64_t *total_rows, int64_t *total_edges, bool draws, int64_t first_batch = 0,
                     int64_t n_run = INT64_MAX, bool accumulate = false)
{
    if (!ctx || !counts || n_train < 0 || (n_train > 0 && !train_ids) || batch_size < 1 || epochs < 0)
        return TIER_EINVAL;
    if (first_batch < 0 || n_run < 0) return TIER_EINVAL;
    int rc = check_fanouts(fanouts, n_layers);
    if (rc) return rc;
    const int64_t first = n_train < batch_size ? n_train : batch_size;
    int64_t cap_nodes[TIER_MAX_LAYERS + 1], cap_edges[TIER_MAX_LAYERS];
    rc = tier_blocks_bounds(ctx->n_nodes, first, fanouts, n_layers, cap_nodes, cap_edges);
    if (rc) return rc;
    if (first > ctx->n_nodes) return TIER_EINVAL;
    // only the nodes that draw are listed: the frontier before the last hop
    const int64_t stride = cap_nodes[n_layers - 1] > 0 ? cap_nodes[n_layers - 1] : 1;
    rc = ensure_i32(ctx, &ctx->ps_nodes, &ctx->cap_ps_nodes, stride * ctx->n_slots);
    if (rc == TIER_OK) rc = ensure_degrees(ctx, stride);
    if (rc) return rc;
    const bool large = large_graph(ctx);
    int table_log2 = 10;
    int64_t dense_edges = 0;        // large-graph layout: the hops before the last list their new nodes by buckets
    if (large) {
        rc = ensure_table(ctx, cap_nodes[n_layers - 1], &table_log2);
        for (int l = 0; l + 1 < n_layers; ++l) dense_edges = cap_edges[l] > dense_edges ? cap_edges[l] : dense_edges;
        if (rc == TIER_OK && dense_edges > 0)
            rc = tier_ensure(ctx, (void **)&ctx->ps_col, &ctx->ps_col_cap, (size_t)dense_edges * ctx->n_slots * sizeof(int32_t));
        if (rc) return rc;
    }

    if (!accumulate)
        k_fill_u32<<<clamp_grid(ctx->n_nodes, kBlock, 4096), kBlock, 0, ctx->stream>>>(counts, ctx->n_nodes, 0u);
    k_clear_totals<<<1, 1, 0, ctx->stream>>>(ctx->meta);
    wide_out o = {};
    o.counts = counts;
    if (dense_edges > 0)
        for (int l = 0; l + 1 < n_layers; ++l) {
            o.layer[l].col = ctx->ps_col;       // fanout entries per dst node: ~node where a new node was drawn
            o.layer[l].edge_stride = dense_edges;
        }
    const int64_t all_batches = (n_train + batch_size - 1) / batch_size;
    const int64_t n_batches = n_run < all_batches - first_batch ? first_batch + n_run : all_batches;   // end of the range
    for (int e = 0; e < epochs; ++e) {
        for (int64_t b = first_batch; b < n_batches; b += ctx->n_slots) {
            const int slots = (int)(n_batches - b < ctx->n_slots ? n_batches - b : ctx->n_slots);
            const int64_t lo = b * batch_size;
            wide_t w = make_wide(ctx, train_ids + lo, n_train - lo, batch_size, slots, ctx->ps_nodes, stride, table_log2,
                                 stride);
            w.count_edges = total_edges != nullptr;
            w.draws = draws ? counts : nullptr;
            if (dense_edges > 0) {
                rc = ensure_buckets(ctx, &w, dense_edges, slots);
                if (rc) return rc;
            }
            for (int s = 0; s < slots; ++s) {
                const uint64_t bs = tier_batch_seed(seed, (uint32_t)e, (uint32_t)(b + s));
                w.key0[s] = (uint32_t)bs;
                w.key1[s] = (uint32_t)(bs >> 32);
            }
            rc = large ? enqueue_wide<MODE_COUNT_LARGE>(ctx, w, fanouts, n_layers, cap_nodes, cap_edges, o)
                       : enqueue_wide<MODE_COUNT_SMALL>(ctx, w, fanouts, n_layers, cap_nodes, cap_edges, o);
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

int tier_presample(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                   const int32_t *fanouts, int32_t n_layers, int32_t epochs, uint64_t seed, uint32_t *counts,
                   int64_t *total_rows, int64_t *total_edges)
{
    return presample(ctx, train_ids, n_train, batch_size, fanouts, n_layers, epochs, seed, counts, total_rows,
                     total_edges, false);
}

int tier_presample_range(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                         const int32_t *fanouts, int32_t n_layers, int32_t epochs, uint64_t seed, int64_t first_batch,
                         int64_t n_batches, int32_t accumulate, uint32_t *counts)
{
    return presample(ctx, train_ids, n_train, batch_size, fanouts, n_layers, epochs, seed, counts, nullptr, nullptr,
                     false, first_batch, n_batches, accumulate != 0);
}

int tier_presample_draws(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                         const int32_t *fanouts, int32_t n_layers, int32_t epochs, uint64_t seed, uint32_t *counts,
                         int64_t *total_draws)
{
    int64_t edges = 0;
    const int rc = presample(ctx, train_ids, n_train, batch_size, fanouts, n_layers, epochs, seed, counts, nullptr,
                             total_draws ? &edges : nullptr, true);
    if (rc == TIER_OK && total_draws) *total_draws = edges + (int64_t)epochs * n_train;
    return rc;
}

}  // extern "C"
