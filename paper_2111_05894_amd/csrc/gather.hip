// Tiered feature gather (Sec. 4.1; Listing 1 without peer GPUs).
//
// For every requested id the row comes from the HBM cache when the node->slot
// map places it there, and from pinned host memory (read in place over the
// host link) otherwise.  A group of LPR lanes copies one row in 16-byte pieces,
// so a row is read and written with full-width coalesced accesses; several rows
// per group are in flight to cover the host link's latency.
//
// Shared misses (tier_set_gather_dedup): the mini-batches gathered by one call overlap
// (on a low-skew 10 M-node graph two thirds of a call's cold rows are requested more
// than once), so the call can first mark its cold ids in a bitmap over all nodes, turn
// the bitmap into an ascending list of distinct cold ids (k_gbm_*), fetch those rows
// over the host link once into an HBM staging area, and then serve every request from
// HBM: cache rows for hits, staged rows for misses.
//
// Split gather (tier_set_gather_split): the host link is saturated by the requests of a
// few dozen blocks.  A full grid that queues megabytes of host reads gains nothing on the
// link, holds every compute unit's slots until the link has served them, and makes
// everything else that crosses the link wait behind its queue (the command processor
// fetching the packets of other streams' kernels included: ~0.3 ms per launch at 16 MB
// in flight).  A call can therefore leave its cold rows to the first few blocks of the
// launch (row 0 of the grid, dispatched first): they look through the requests, copy the
// cold ones and stay until the link has delivered them, while all other blocks copy hot
// rows only and drain at HBM speed, leaving the chip to whoever else has work.
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowsInFlight = 4;        // measured best of 2 / 4 / 8 on MI355X
constexpr int kLinkBlocks = 64;         // blocks of a launch that reads host rows only (best of 32 .. 512, full grid)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The id lists one launch serves (blockIdx.y picks one): a mini-batch each.
struct id_lists_t {
    const int32_t *ids[TIER_MAX_BATCHES];
    int64_t n[TIER_MAX_BATCHES];
    int64_t out_row[TIER_MAX_BATCHES];   // first output row of the list
    const int64_t *n_dev;                // non-null: the length of list 0 is read from the device
};

// An id outside the graph is nobody's cold row: the blocks that copy hot rows write its row of zeros.
template <int MODE>
__device__ inline int is_cold(int32_t id, const int32_t *__restrict__ slot, int64_t n_nodes, int64_t n_hot)
{
    if ((uint32_t)id >= (uint64_t)n_nodes) return 0;
    return MODE == GATHER_SLOT ? slot[id] < 0 : id >= n_hot;
}

// The cold workers of a split launch: the first `workers` blocks of grid row 0.  The
// requests are numbered in units of 64 (list by list); a wave takes the next unit off a
// counter, which makes the waves finish together whatever the mix of hot and cold in
// their units, and appends the unit's cold requests (one ballot) to a small queue of its
// own in LDS.  Whenever the queue holds a full pass - kRowsInFlight rows for each group of
// LPR lanes - the wave copies one, so the bytes it keeps in flight on the host link do not
// depend on how many of the requests are cold.  Three stages run ahead of that: the
// counter is read three units ahead, the ids two, the slot lookups one, so the copies
// never wait for a lookup.  The last wave to run dry leaves both counters at zero for the
// next launch on the stream.
template <int LPR, int MODE>
__device__ inline void scan_cold_rows(const id_lists_t &lists, int n_lists, const int32_t *__restrict__ slot,
                                      int64_t n_nodes, int64_t n_hot, int workers,
                                      const uint4 *__restrict__ host, uint4 *__restrict__ out_base, int cpr,
                                      int64_t *__restrict__ meta)
{
    constexpr int kGroupsPerWave = 64 / LPR;
    constexpr int kPerPass = kGroupsPerWave * kRowsInFlight;
    constexpr int kQueue = 128;                       // ring: at most kPerPass - 1 + 64 entries wait
    __shared__ int32_t s_src[kBlock / 64][kQueue];    // host row of a waiting cold request
    __shared__ int64_t s_dst[kBlock / 64][kQueue];    // its output row
    if ((int)blockIdx.x >= workers) return;
    const int lane64 = threadIdx.x & 63;
    const int g = lane64 / LPR, lane = lane64 % LPR;
    int32_t *q_src = s_src[threadIdx.x >> 6];
    int64_t *q_dst = s_dst[threadIdx.x >> 6];
    const unsigned long long n_waves = (unsigned long long)workers * (kBlock / 64);
    unsigned long long *next = (unsigned long long *)&meta[META_COLD_NEXT];
    unsigned long long *done = (unsigned long long *)&meta[META_COLD_DONE];
    int64_t total = 0;
    for (int b = 0; b < n_lists; ++b) total += (lists.n[b] + 63) / 64;

    // the counter's value arrives in lane 0; it is broadcast only where it is needed, an
    // iteration later, so that the atomic's latency hides behind the work in between
    auto grab = [&]() -> unsigned long long { return lane64 == 0 ? atomicAdd(next, 1ull) : 0ull; };
    auto bcast = [&](unsigned long long raw) -> int64_t { return (int64_t)__shfl(raw, 0); };
    // this lane's request of unit u (-1 beyond the list or the call) and the unit's first output row
    auto load_unit = [&](int64_t u, int64_t &row0) -> int32_t {
        row0 = 0;
        if (u >= total) return -1;
        int b = 0;
        for (;; ++b) {                              // u < total: ends inside the lists
            const int64_t nu = (lists.n[b] + 63) / 64;
            if (u < nu) break;
            u -= nu;
        }
        row0 = lists.out_row[b] + u * 64;
        const int64_t i = u * 64 + lane64;
        return i < lists.n[b] ? lists.ids[b][i] : -1;
    };
    // copy the n (<= kPerPass) requests at the head of the queue
    auto copy_pass = [&](unsigned head, int n) {
        const uint4 *src[kRowsInFlight];
        uint4 *dst[kRowsInFlight];
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) {
            const int k = g * kRowsInFlight + j;
            src[j] = nullptr;
            dst[j] = nullptr;
            if (k < n) {
                const unsigned e = (head + (unsigned)k) % kQueue;
                src[j] = host + (int64_t)q_src[e] * cpr;
                dst[j] = out_base + q_dst[e] * cpr;
            }
        }
        for (int cc = lane; cc < cpr; cc += LPR) {
            uint4 v[kRowsInFlight];
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j) {
                v[j] = make_uint4(0, 0, 0, 0);
                if (src[j]) v[j] = src[j][cc];
            }
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j)
                if (dst[j]) {
                    u32x4 t4 = {v[j].x, v[j].y, v[j].z, v[j].w};
                    __builtin_nontemporal_store(t4, (u32x4 *)&dst[j][cc]);
                }
        }
    };

    unsigned head = 0, waiting = 0;                   // wave-uniform state of the queue
    int64_t q0 = bcast(grab()), q1 = bcast(grab());
    unsigned long long raw2 = grab();
    int64_t row0, row1, row2;
    int32_t id0 = load_unit(q0, row0), id1 = load_unit(q1, row1);
    int cold0 = id0 >= 0 ? is_cold<MODE>(id0, slot, n_nodes, n_hot) : 0;
    while (q0 < total) {
        const unsigned long long raw3 = grab();
        const int64_t q2 = bcast(raw2);
        const int32_t id2 = load_unit(q2, row2);
        const int cold1 = id1 >= 0 ? is_cold<MODE>(id1, slot, n_nodes, n_hot) : 0;
        // the cold requests of unit 0 join the queue in request order
        const unsigned long long mask = __ballot(cold0);
        if (cold0) {
            const unsigned before = __popcll(mask & ((1ull << lane64) - 1ull));
            const unsigned e = (head + waiting + before) % kQueue;
            q_src[e] = id0;
            q_dst[e] = row0 + lane64;
        }
        waiting += (unsigned)__popcll(mask);
        __builtin_amdgcn_wave_barrier();
        while (waiting >= (unsigned)kPerPass) {
            copy_pass(head, kPerPass);
            head = (head + kPerPass) % kQueue;
            waiting -= kPerPass;
        }
        __builtin_amdgcn_wave_barrier();
        q0 = q1;
        q1 = q2;
        raw2 = raw3;
        id0 = id1;
        id1 = id2;
        row0 = row1;
        row1 = row2;
        cold0 = cold1;
    }
    if (waiting) copy_pass(head, (int)waiting);       // fewer than a pass left
    if (lane64 == 0 && atomicAdd(done, 1ull) == n_waves - 1) {    // every other wave has made its last grab
        atomicExch(next, 0ull);
        atomicExch(done, 0ull);
    }
}

// MODE: GATHER_SLOT     hot <=> slot[id] >= 0, cache row = slot[id]      (ids keep their meaning)
//       GATHER_BOUNDARY hot <=> id < n_hot, cache row = id, cold row = id - n_hot of the cold
//                       part (rows in rank order: the two-way branch of Listing 1)
//       GATHER_HOST     every row from host memory: the untiered copy that fills the HBM
//                       cache at placement time
// STAGED: cold rows come from the staging area (row stage_slot[id]) instead of host memory.
// SPLIT:  grid row 0 holds the cold workers (copy_cold_rows), list b is served by grid row b + 1
//         and skips its cold rows.
template <int LPR, int MODE, bool STAGED, bool SPLIT>
__global__ __launch_bounds__(kBlock) void k_gather(id_lists_t lists, const int32_t *__restrict__ slot,
                                                   const uint4 *__restrict__ cache,
                                                   const uint4 *__restrict__ host,
                                                   const uint4 *__restrict__ stage,
                                                   const int32_t *__restrict__ stage_slot,
                                                   uint4 *__restrict__ out_base, int cpr, int64_t n_nodes,
                                                   int64_t n_hot, int64_t *__restrict__ meta, int count_hits,
                                                   int cold_workers)
{
    constexpr int kGroups = kBlock / LPR;
    if (SPLIT && blockIdx.y == 0) {
        scan_cold_rows<LPR, MODE>(lists, (int)gridDim.y - 1, slot, n_nodes, n_hot, cold_workers, host, out_base, cpr,
                                  meta);
        return;
    }
    const int list = SPLIT ? blockIdx.y - 1 : blockIdx.y;
    const int32_t *__restrict__ ids = lists.ids[list];
    const int64_t n = lists.n_dev ? *lists.n_dev : lists.n[list];
    uint4 *__restrict__ out = out_base + lists.out_row[list] * cpr;
    const int lane = threadIdx.x % LPR;
    const int64_t group = (int64_t)blockIdx.x * kGroups + threadIdx.x / LPR;
    const int64_t n_groups = (int64_t)gridDim.x * kGroups;
    int hits = 0;
    int bad = 0;

    for (int64_t r0 = group * kRowsInFlight; r0 < n; r0 += n_groups * kRowsInFlight) {
        const uint4 *src[kRowsInFlight];
        bool put[kRowsInFlight];
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) {
            int64_t r = r0 + j;
            src[j] = nullptr;
            put[j] = r < n;
            if (r < n) {
                int32_t id = ids[r];
                if ((uint32_t)id >= (uint64_t)n_nodes) {
                    bad = 1;                       // row of zeros, error reported by the host
                } else {
                    int32_t s = -1;
                    if (MODE == GATHER_SLOT) s = slot[id];
                    if (MODE == GATHER_BOUNDARY) s = id < n_hot ? id : -1;
                    if (s >= 0) {
                        src[j] = cache + (int64_t)s * cpr;
                        hits += (lane == 0);
                    } else if (SPLIT) {
                        put[j] = false;
                    } else if (STAGED) {
                        src[j] = stage + (int64_t)stage_slot[id] * cpr;
                    } else if (MODE == GATHER_BOUNDARY) {
                        const uint4 *cold = host + n_hot * cpr;          // first row of the cold part
                        src[j] = cold + ((int64_t)id - n_hot) * cpr;
                    } else {
                        src[j] = host + (int64_t)id * cpr;
                    }
                }
            }
        }
        for (int c = lane; c < cpr; c += LPR) {
            uint4 v[kRowsInFlight];
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j) {
                v[j] = make_uint4(0, 0, 0, 0);
                if (src[j]) v[j] = src[j][c];      // cached load: hot rows recur across mini-batches
            }
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j)
                if (put[j]) {                      // streaming store: the output is not read back here
                    u32x4 t = {v[j].x, v[j].y, v[j].z, v[j].w};
                    __builtin_nontemporal_store(t, (u32x4 *)&out[(r0 + j) * cpr + c]);
                }
        }
    }
    if (bad) atomicOr((int *)&meta[META_ERROR], 1);
    if (count_hits) {
        // one atomic per block, on one of META_HIT_STRIPES counters
        __shared__ int s_hits[kBlock / 64];
        for (int off = 32; off > 0; off >>= 1) hits += __shfl_down(hits, off);
        if ((threadIdx.x & 63) == 0) s_hits[threadIdx.x >> 6] = hits;
        __syncthreads();
        if (threadIdx.x == 0) {
            int t = 0;
            for (int i = 0; i < kBlock / 64; ++i) t += s_hits[i];
            if (t)
                atomicAdd((unsigned long long *)&meta[META_HIT_ROWS + ((blockIdx.x + blockIdx.y) & (META_HIT_STRIPES - 1))],
                          (unsigned long long)t);
        }
    }
}

// ---- shared misses: distinct cold ids of a call ---------------------------------------

__device__ inline int gblock_sum(int x, int *s_wave)
{
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = x;
    __syncthreads();
    int t = 0;
    for (int i = 0; i < kBlock / 64; ++i) t += s_wave[i];
    return t;
}

__device__ inline void gblock_range(int64_t n, int64_t &lo, int64_t &hi)
{
    int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    chunk = (chunk + kBlock - 1) / kBlock * kBlock;
    lo = (int64_t)blockIdx.x * chunk;
    if (lo > n) lo = n;
    hi = lo + chunk;
    if (hi > n) hi = n;
}

template <int MODE>
__global__ void k_mark_misses(id_lists_t lists, const int32_t *__restrict__ slot, int64_t n_nodes, int64_t n_hot,
                              uint32_t *__restrict__ bitmap)
{
    const int32_t *__restrict__ ids = lists.ids[blockIdx.y];
    const int64_t n = lists.n[blockIdx.y];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += stride) {
        const int32_t id = ids[r];
        if ((uint32_t)id >= (uint64_t)n_nodes) continue;            // reported by the gather itself
        const bool hit = MODE == GATHER_SLOT ? slot[id] >= 0 : id < n_hot;
        if (!hit) {
            const uint32_t bit = 1u << (id & 31);
            if (!(bitmap[id >> 5] & bit)) atomicOr(&bitmap[id >> 5], bit);   // most repeats stop at the read
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_gbm_partial(const uint32_t *__restrict__ bitmap, int64_t n_words,
                                                        int32_t *__restrict__ partial)
{
    __shared__ int s_wave[kBlock / 64];
    int64_t lo, hi;
    gblock_range(n_words, lo, hi);
    int sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) sum += __popc(bitmap[i]);
    int tot = gblock_sum(sum, s_wave);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

// bitmap -> ascending list of distinct cold ids; stage_slot[id] = its row in the staging area
__global__ __launch_bounds__(kBlock) void k_gbm_emit(uint32_t *__restrict__ bitmap, int64_t n_words,
                                                     const int32_t *__restrict__ partial,
                                                     int32_t *__restrict__ uniq, int32_t *__restrict__ stage_slot,
                                                     int64_t *__restrict__ meta)
{
    __shared__ int s_wave[kBlock / 64];
    int64_t lo, hi;
    gblock_range(n_words, lo, hi);
    int b4 = 0, all = 0;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += kBlock) {
        int p = partial[i];
        all += p;
        b4 += (i < (int)blockIdx.x) ? p : 0;
    }
    int carry = gblock_sum(b4, s_wave);
    all = gblock_sum(all, s_wave);
    if (blockIdx.x == 0 && threadIdx.x == 0) meta[META_NFRONT] = all;      // distinct cold rows of this call
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int64_t tile = lo; tile < hi; tile += kBlock) {
        const int64_t i = tile + threadIdx.x;
        uint32_t bits = i < hi ? bitmap[i] : 0u;
        int incl = __popc(bits);
        const int mine = incl;
        for (int d = 1; d < 64; d <<= 1) {
            int y = __shfl_up(incl, d);
            if (l >= d) incl += y;
        }
        __syncthreads();
        if (l == 63) s_wave[w] = incl;
        __syncthreads();
        int base = 0, tot = 0;
        for (int q = 0; q < kBlock / 64; ++q) {
            int t = s_wave[q];
            base += q < w ? t : 0;
            tot += t;
        }
        int pos = carry + base + incl - mine;
        carry += tot;
        if (bits) {
            bitmap[i] = 0u;
            while (bits) {
                int b = __ffs(bits) - 1;
                bits &= bits - 1;
                int32_t u = (int32_t)(i * 32 + b);
                uniq[pos] = u;
                stage_slot[u] = pos;
                ++pos;
            }
        }
    }
}

__global__ void k_clear_hits(int64_t *meta)
{
    if (threadIdx.x < META_HIT_STRIPES) meta[META_HIT_ROWS + threadIdx.x] = 0;
}
__global__ void k_clear_gather_error(int64_t *meta) { meta[META_ERROR] = 0; }

}  // namespace

// One k_gather launch on stream st, bookkeeping words in meta.
static int launch_lists(tier_ctx *ctx, const id_lists_t &lists, int n_lists, int64_t n_max, int mode, bool staged,
                        void *out, bool count_hits, hipStream_t st, int64_t *meta, bool split = false)
{
    if (count_hits) k_clear_hits<<<1, META_HIT_STRIPES, 0, st>>>(meta);
    if (n_max <= 0) return TIER_OK;
    const int cpr = (int)(ctx->row_bytes / 16);
    int lpr = 8;
    while (lpr < cpr && lpr < 64) lpr *= 2;
    const int groups = kBlock / lpr;
    int64_t blocks = (n_max + (int64_t)groups * kRowsInFlight - 1) / ((int64_t)groups * kRowsInFlight);
    const int64_t max_blocks = 1 << 18;     // beyond that groups loop; fewer blocks cost ~5 % of the all-hit rate
    if (blocks > max_blocks) blocks = max_blocks;
    if (mode == GATHER_HOST && ctx->rows_on_host) {
        // every row over the host link: a few dozen blocks fill it, more only queue up
        if (blocks > kLinkBlocks) blocks = kLinkBlocks;
    }
    const int cold_workers = split ? (int)(ctx->link_blocks < blocks ? ctx->link_blocks : blocks) : 0;
    const dim3 grid((unsigned)blocks, (unsigned)(n_lists + (split ? 1 : 0)));
#define GATHER_LAUNCH(L, M, S, P)                                                                    \
    k_gather<L, M, S, P><<<grid, kBlock, 0, st>>>(lists, ctx->slot, (const uint4 *)ctx->cache,       \
                                                  (const uint4 *)ctx->host_rows, (const uint4 *)ctx->stage, \
                                                  ctx->stage_slot, (uint4 *)out, cpr, ctx->n_nodes,  \
                                                  ctx->n_hot, meta, count_hits ? 1 : 0, cold_workers)
#define GATHER_CASE(L)                                                                               \
    case L:                                                                                          \
        if (mode == GATHER_SLOT && split) GATHER_LAUNCH(L, GATHER_SLOT, false, true);                \
        else if (mode == GATHER_BOUNDARY && split) GATHER_LAUNCH(L, GATHER_BOUNDARY, false, true);   \
        else if (mode == GATHER_SLOT && staged) GATHER_LAUNCH(L, GATHER_SLOT, true, false);          \
        else if (mode == GATHER_SLOT) GATHER_LAUNCH(L, GATHER_SLOT, false, false);                   \
        else if (mode == GATHER_BOUNDARY && staged) GATHER_LAUNCH(L, GATHER_BOUNDARY, true, false);  \
        else if (mode == GATHER_BOUNDARY) GATHER_LAUNCH(L, GATHER_BOUNDARY, false, false);           \
        else GATHER_LAUNCH(L, GATHER_HOST, false, false);                                            \
        break;
    switch (lpr) {
        GATHER_CASE(8)
        GATHER_CASE(16)
        GATHER_CASE(32)
        GATHER_CASE(64)
    }
#undef GATHER_CASE
#undef GATHER_LAUNCH
    TIER_HIP(ctx, hipGetLastError());
    return TIER_OK;
}

int tier_launch_gather(tier_ctx *ctx, const int32_t *ids, int64_t n, int mode, void *out, bool count_hits)
{
    id_lists_t lists = {};
    lists.ids[0] = ids;
    lists.n[0] = n;
    return launch_lists(ctx, lists, 1, n, mode, false, out, count_hits, ctx->gather_stream, ctx->gmeta);
}

static int grow(tier_ctx *ctx, void **buf, int64_t *cap, int64_t want, size_t elem)
{
    if (want <= *cap) return TIER_OK;
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    if (*buf) TIER_HIP(ctx, hipFree(*buf));
    *buf = nullptr;
    *cap = 0;
    TIER_HIP(ctx, hipMalloc(buf, (size_t)want * elem));
    *cap = want;
    return TIER_OK;
}

// The tiered gather of one call: one uniform launch, one launch with cold workers apart, or
// every distinct cold row fetched once.
static int gather_call(tier_ctx *ctx, const id_lists_t &lists, int n_lists, int64_t n_max, int64_t n_total, void *out,
                       bool count_hits)
{
    const int mode = ctx->boundary ? GATHER_BOUNDARY : GATHER_SLOT;
    hipStream_t st = ctx->gather_stream;
    // nothing to split off when every row is in the cache
    if (!ctx->dedup && ctx->link_blocks > 0 && n_total > 0 && n_total >= ctx->split_min_rows &&
        ctx->n_hot < ctx->n_nodes)
        return launch_lists(ctx, lists, n_lists, n_max, mode, false, out, count_hits, st, ctx->gmeta, true);
    if (!ctx->dedup || n_total == 0)
        return launch_lists(ctx, lists, n_lists, n_max, mode, false, out, count_hits, st, ctx->gmeta);

    // at most min(requests, nodes) distinct cold rows
    const int64_t cap = n_total < ctx->n_nodes ? n_total : ctx->n_nodes;
    int rc = grow(ctx, (void **)&ctx->stage, &ctx->stage_cap, cap, (size_t)ctx->row_bytes);
    if (rc == TIER_OK) rc = grow(ctx, (void **)&ctx->uniq_ids, &ctx->uniq_cap, cap, sizeof(int32_t));
    if (rc != TIER_OK) return rc;
    const dim3 mgrid((unsigned)((n_max + kBlock - 1) / kBlock < 4096 ? (n_max + kBlock - 1) / kBlock : 4096),
                     (unsigned)n_lists);
    if (mode == GATHER_SLOT)
        k_mark_misses<GATHER_SLOT><<<mgrid, kBlock, 0, st>>>(lists, ctx->slot, ctx->n_nodes, ctx->n_hot, ctx->gbitmap);
    else
        k_mark_misses<GATHER_BOUNDARY><<<mgrid, kBlock, 0, st>>>(lists, ctx->slot, ctx->n_nodes, ctx->n_hot,
                                                                 ctx->gbitmap);
    int64_t g = (ctx->n_words + 4 * kBlock - 1) / (4 * kBlock);
    const int bgrid = (int)(g < 1 ? 1 : (g > TIER_SCAN_BLOCKS ? TIER_SCAN_BLOCKS : g));
    k_gbm_partial<<<bgrid, kBlock, 0, st>>>(ctx->gbitmap, ctx->n_words, ctx->gpartial);
    k_gbm_emit<<<bgrid, kBlock, 0, st>>>(ctx->gbitmap, ctx->n_words, ctx->gpartial, ctx->uniq_ids, ctx->stage_slot,
                                         ctx->gmeta);
    TIER_HIP(ctx, hipGetLastError());
    id_lists_t fetch = {};
    fetch.ids[0] = ctx->uniq_ids;
    fetch.n[0] = cap;
    fetch.n_dev = &ctx->gmeta[META_NFRONT];
    rc = launch_lists(ctx, fetch, 1, cap, GATHER_HOST, false, ctx->stage, false, st, ctx->gmeta);
    if (rc != TIER_OK) return rc;
    return launch_lists(ctx, lists, n_lists, n_max, mode, true, out, count_hits, st, ctx->gmeta);
}

// hit / miss rows of the launch(es) since the last k_clear_hits on the gather stream
static int read_stats(tier_ctx *ctx, int64_t n_total, tier_gather_stats *stats)
{
    TIER_HIP(ctx, hipMemcpyAsync(ctx->gmeta_host, ctx->gmeta, GMETA_WORDS * sizeof(int64_t), hipMemcpyDeviceToHost,
                                 ctx->gather_stream));
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    if (ctx->gmeta_host[META_ERROR] != 0) {
        k_clear_gather_error<<<1, 1, 0, ctx->gather_stream>>>(ctx->gmeta);
        return TIER_EINVAL;
    }
    stats->hit_rows = 0;
    for (int i = 0; i < META_HIT_STRIPES; ++i) stats->hit_rows += ctx->gmeta_host[META_HIT_ROWS + i];
    stats->miss_rows = n_total - stats->hit_rows;
    stats->link_rows = ctx->dedup && n_total > 0 ? ctx->gmeta_host[META_NFRONT] : stats->miss_rows;
    return TIER_OK;
}

extern "C" int tier_gather_minibatches(tier_ctx *ctx, const int32_t *nodes, int64_t nodes_stride,
                                       const int64_t *n_rows, const int64_t *out_row_offset, int32_t n_batches,
                                       void *out, tier_gather_stats *stats)
{
    if (!ctx || !n_rows || !out_row_offset || n_batches < 1 || n_batches > TIER_MAX_BATCHES || nodes_stride < 0)
        return TIER_EINVAL;
    if (((uintptr_t)out & 15u) != 0) return TIER_EINVAL;
    if (!ctx->placed) return TIER_ESTATE;
    id_lists_t lists = {};
    int64_t n_max = 0, n_total = 0;
    for (int b = 0; b < n_batches; ++b) {
        if (n_rows[b] < 0 || out_row_offset[b] < 0 || n_rows[b] > nodes_stride) return TIER_EINVAL;
        lists.ids[b] = nodes + (int64_t)b * nodes_stride;
        lists.n[b] = n_rows[b];
        lists.out_row[b] = out_row_offset[b];
        n_max = n_rows[b] > n_max ? n_rows[b] : n_max;
        n_total += n_rows[b];
    }
    if (n_total > 0 && (!nodes || !out)) return TIER_EINVAL;
    int rc = gather_call(ctx, lists, n_batches, n_max, n_total, out, stats != nullptr);
    if (rc != TIER_OK) return rc;
    if (stats) return read_stats(ctx, n_total, stats);
    return TIER_OK;
}

extern "C" int tier_gather_features(tier_ctx *ctx, const int32_t *ids, int64_t n, void *out,
                                    tier_gather_stats *stats)
{
    if (!ctx || n < 0 || (n > 0 && (!ids || !out))) return TIER_EINVAL;
    if (((uintptr_t)out & 15u) != 0) return TIER_EINVAL;
    if (!ctx->placed) return TIER_ESTATE;
    id_lists_t lists = {};
    lists.ids[0] = ids;
    lists.n[0] = n;
    int rc = gather_call(ctx, lists, 1, n, n, out, stats != nullptr);
    if (rc != TIER_OK) return rc;
    if (stats) return read_stats(ctx, n, stats);
    return TIER_OK;
}

extern "C" int tier_set_gather_split(tier_ctx *ctx, int32_t link_blocks, int64_t min_rows)
{
    if (!ctx || link_blocks < 0 || link_blocks > 65536 || min_rows < 0) return TIER_EINVAL;
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    ctx->link_blocks = link_blocks;
    ctx->split_min_rows = min_rows;
    return TIER_OK;
}

extern "C" int tier_set_gather_dedup(tier_ctx *ctx, int on)
{
    if (!ctx) return TIER_EINVAL;
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    if (on && !ctx->gbitmap) {
        const size_t words = (size_t)(ctx->n_words > 0 ? ctx->n_words : 1);
        TIER_HIP(ctx, hipMalloc(&ctx->gbitmap, words * sizeof(uint32_t)));
        TIER_HIP(ctx, hipMemsetAsync(ctx->gbitmap, 0, words * sizeof(uint32_t), ctx->gather_stream));
        TIER_HIP(ctx, hipMalloc(&ctx->stage_slot, (size_t)(ctx->n_nodes > 0 ? ctx->n_nodes : 1) * sizeof(int32_t)));
        TIER_HIP(ctx, hipMalloc(&ctx->gpartial, TIER_SCAN_BLOCKS * sizeof(int32_t)));
        TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    }
    ctx->dedup = on != 0;
    return TIER_OK;
}
