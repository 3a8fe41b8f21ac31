// Hot/cold placement (Sec. 3.2: order by descending score, old-id -> rank map;
// Sec. 4.1: the top rows live in GPU memory, the rest in host memory).
//
// Ordering by (score descending, id ascending) is a stable sort of the ids 0..N-1
// by a key that grows as the score falls: ~count for integer scores (access
// counts, degrees), the complemented order-preserving bit pattern for real ones.
// The sort is a least-significant-digit radix sort with 8-bit digits that runs
// only the digits in which the keys differ at all (small counts: one or two
// passes).  Each wavefront owns one contiguous share of the input, so stability
// needs no cross-wavefront ordering: per-(digit, wavefront) counts are scanned
// digit-major into start offsets, and inside a wavefront the rank among equal
// digits comes from ballots.
#include "tier_internal.h"

namespace {

constexpr int kWave = 64;
constexpr int kDigits = 256;
constexpr int kMaxShares = 4096;
constexpr int kScanBlock = 256;

__global__ void k_keys_from_counts(const uint32_t *__restrict__ counts, int64_t n, uint32_t *__restrict__ keys)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) keys[i] = ~counts[i];
}

// ascending unsigned order of the key = descending order of the value (-0.0 counts as 0.0)
__global__ void k_keys_from_scores(const double *__restrict__ scores, int64_t n, uint64_t *__restrict__ keys)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t b = (uint64_t)__double_as_longlong(scores[i] + 0.0);
        b ^= (b >> 63) ? ~0ull : (1ull << 63);          // now ascending with the value
        keys[i] = ~b;
    }
}

// bits in which any key differs from the first one
template <typename K>
__global__ void k_varying_bits(const K *__restrict__ keys, int64_t n, unsigned long long *__restrict__ out)
{
    const K first = keys[0];
    K m = 0;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) m |= keys[i] ^ first;
    unsigned long long mm = (unsigned long long)m;
    for (int off = 32; off > 0; off >>= 1) mm |= (unsigned long long)__shfl_xor((long long)mm, off);
    if ((threadIdx.x & 63) == 0 && mm) atomicOr(out, mm);
}

// launched with one wavefront per block; block b owns items [b*share, (b+1)*share)
template <typename K>
__global__ __launch_bounds__(kWave) void k_radix_hist(const K *__restrict__ keys_in, int64_t n, int64_t share,
                                                      int shift, uint32_t *__restrict__ hist, int n_shares)
{
    __shared__ uint32_t s_hist[kDigits];
    for (int d = threadIdx.x; d < kDigits; d += kWave) s_hist[d] = 0;
    __syncthreads();
    int64_t lo = (int64_t)blockIdx.x * share, hi = lo + share;
    if (hi > n) hi = n;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kWave)
        atomicAdd(&s_hist[(uint32_t)(keys_in[i] >> shift) & 255u], 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < kDigits; d += kWave) hist[(int64_t)d * n_shares + blockIdx.x] = s_hist[d];
}

// Exclusive scan of x[0..n) in place, two launches with the same grid (<= 1024 blocks).
__device__ inline uint32_t block_sum_u32(uint32_t x, uint32_t *s_wave)
{
    for (int off = 32; off > 0; off >>= 1) x += (uint32_t)__shfl_xor((int)x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = x;
    __syncthreads();
    uint32_t t = 0;
    for (int i = 0; i < kScanBlock / 64; ++i) t += s_wave[i];
    return t;
}

__device__ inline void scan_range(int64_t n, int64_t &lo, int64_t &hi)
{
    int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    chunk = (chunk + kScanBlock - 1) / kScanBlock * kScanBlock;
    lo = (int64_t)blockIdx.x * chunk;
    if (lo > n) lo = n;
    hi = lo + chunk;
    if (hi > n) hi = n;
}

__global__ __launch_bounds__(kScanBlock) void k_scan_partial(const uint32_t *__restrict__ x, int64_t n,
                                                             uint32_t *__restrict__ partial)
{
    __shared__ uint32_t s_wave[kScanBlock / 64];
    int64_t lo, hi;
    scan_range(n, lo, hi);
    uint32_t sum = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kScanBlock) sum += x[i];
    uint32_t tot = block_sum_u32(sum, s_wave);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kScanBlock) void k_scan_apply(uint32_t *__restrict__ x, int64_t n,
                                                           const uint32_t *__restrict__ partial)
{
    __shared__ uint32_t s_wave[kScanBlock / 64];
    int64_t lo, hi;
    scan_range(n, lo, hi);
    uint32_t before = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kScanBlock) before += partial[i];
    uint32_t carry = block_sum_u32(before, s_wave);
    for (int64_t tile = lo; tile < hi; tile += kScanBlock) {
        int64_t i = tile + threadIdx.x;
        uint32_t v = i < hi ? x[i] : 0u;
        uint32_t incl = v;
        const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
        for (int d = 1; d < 64; d <<= 1) {
            uint32_t y = (uint32_t)__shfl_up((int)incl, d);
            if (l >= d) incl += y;
        }
        __syncthreads();
        if (l == 63) s_wave[w] = incl;
        __syncthreads();
        uint32_t base = 0, tot = 0;
        for (int q = 0; q < kScanBlock / 64; ++q) {
            uint32_t t = s_wave[q];
            base += q < w ? t : 0u;
            tot += t;
        }
        if (i < hi) x[i] = carry + base + incl - v;
        carry += tot;
    }
}

template <typename K>
__global__ __launch_bounds__(kWave) void k_radix_scatter(const K *__restrict__ keys_in,
                                                         const int32_t *__restrict__ vals_in, int64_t n,
                                                         int64_t share, int shift,
                                                         const uint32_t *__restrict__ offsets, int n_shares,
                                                         K *__restrict__ keys_out, int32_t *__restrict__ vals_out)
{
    __shared__ uint32_t s_off[kDigits];
    for (int d = threadIdx.x; d < kDigits; d += kWave) s_off[d] = offsets[(int64_t)d * n_shares + blockIdx.x];
    __syncthreads();
    int64_t lo = (int64_t)blockIdx.x * share, hi = lo + share;
    if (hi > n) hi = n;
    const uint64_t below = (1ull << threadIdx.x) - 1ull;
    for (int64_t base = lo; base < hi; base += kWave) {
        const int64_t i = base + threadIdx.x;
        const bool valid = i < hi;
        K key = 0;
        int32_t val = 0;
        if (valid) {
            key = keys_in[i];
            val = vals_in ? vals_in[i] : (int32_t)i;
        }
        const uint32_t digit = (uint32_t)(key >> shift) & 255u;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1u;
            const uint64_t bal = __ballot(valid && bit);
            peers &= bit ? bal : ~bal;
        }
        const int rank = __popcll(peers & below);
        const int same = __popcll(peers);
        uint32_t start = 0;
        if (valid) start = s_off[digit];
        __syncthreads();
        if (valid) {
            const int64_t dst = (int64_t)start + rank;
            if (keys_out) keys_out[dst] = key;
            vals_out[dst] = val;
            if (rank == same - 1) s_off[digit] = start + (uint32_t)same;
        }
        __syncthreads();
    }
}

__global__ void k_iota(int32_t *__restrict__ p, int64_t n)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = (int32_t)i;
}

// order[r] = node of rank r  ->  slot[node] = r for the first n_hot ranks, else -1
__global__ void k_slot_map(const int32_t *__restrict__ order, int64_t n, int64_t n_hot, int32_t *__restrict__ slot)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += stride)
        slot[order[r]] = r < n_hot ? (int32_t)r : -1;
}

// hot_bits: bit v set <=> slot[v] >= 0.  One thread per word reads its 32 slots in order.
__global__ void k_hot_bits(const int32_t *__restrict__ slot, int64_t n, uint32_t *__restrict__ hot_bits)
{
    const int64_t n_words = (n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < n_words; w += stride) {
        uint32_t bits = 0u;
        const int64_t first = w * 32;
        const int lim = n - first < 32 ? (int)(n - first) : 32;
        for (int b = 0; b < lim; ++b) bits |= (slot[first + b] >= 0 ? 1u : 0u) << b;
        hot_bits[w] = bits;
    }
}

__global__ void k_zero_u64(unsigned long long *p) { *p = 0; }

int grid_for(int64_t n, int block, int cap)
{
    int64_t g = (n + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

typedef tier_sort_bufs sort_bufs;     // owned by the context, reused by every placement

// The previous placement's cache fill reads the old order on the gather stream.
int release_sort_bufs(tier_ctx *ctx)
{
    if (ctx->fill_pending) {
        TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
        ctx->fill_pending = false;
    }
    return TIER_OK;
}

// Stable ascending sort of 0..n-1 by keys (b.keys[0], already filled) on the context's
// stream.  *order_out points into b (position -> id) and is valid until the next sort.
// Waits once (for the set of digits in which the keys differ).
template <typename K>
int sort_ids_by_keys(tier_ctx *ctx, sort_bufs &b, int32_t **order_out)
{
    const int64_t n = ctx->n_nodes;
    hipStream_t st = ctx->stream;
    K *keys[2] = {(K *)b.keys[0], nullptr};
    if (!b.mask) TIER_HIP(ctx, hipMalloc(&b.mask, sizeof(unsigned long long)));
    k_zero_u64<<<1, 1, 0, st>>>(b.mask);
    if (n > 0) k_varying_bits<K><<<grid_for(n, 256, 2048), 256, 0, st>>>(keys[0], n, b.mask);
    TIER_HIP(ctx, hipMemcpyAsync(ctx->meta_host, b.mask, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    TIER_HIP(ctx, hipStreamSynchronize(st));
    const unsigned long long mask = *(unsigned long long *)ctx->meta_host;
    int shifts[8], passes = 0;
    for (int d = 0; d < (int)sizeof(K); ++d)
        if ((mask >> (8 * d)) & 0xffull) shifts[passes++] = 8 * d;

    int rc = tier_ensure(ctx, (void **)&b.vals[0], &b.vals_cap[0], (size_t)n * sizeof(int32_t));
    if (rc != TIER_OK) return rc;
    if (passes == 0) {
        k_iota<<<grid_for(n, 256, 4096), 256, 0, st>>>(b.vals[0], n);
        TIER_HIP(ctx, hipGetLastError());
        *order_out = b.vals[0];
        return TIER_OK;
    }
    int64_t share = (n + kMaxShares - 1) / kMaxShares;
    if (share < 16 * kWave) share = 16 * kWave;
    share = (share + kWave - 1) / kWave * kWave;
    const int n_shares = (int)((n + share - 1) / share);
    const int64_t n_hist = (int64_t)kDigits * n_shares;
    const int scan_grid = grid_for(n_hist, 4 * kScanBlock, 1024);
    rc = tier_ensure(ctx, (void **)&b.hist, &b.hist_cap, (size_t)n_hist * sizeof(uint32_t));
    if (rc != TIER_OK) return rc;
    if (!b.partial) TIER_HIP(ctx, hipMalloc(&b.partial, 1024 * sizeof(uint32_t)));
    if (passes > 1) {
        rc = tier_ensure(ctx, (void **)&b.vals[1], &b.vals_cap[1], (size_t)n * sizeof(int32_t));
        if (rc == TIER_OK) rc = tier_ensure(ctx, &b.keys[1], &b.keys_cap[1], (size_t)n * sizeof(K));
        if (rc != TIER_OK) return rc;
        keys[1] = (K *)b.keys[1];
    }
    // pass j reads buffers j % 2 and writes buffers (j + 1) % 2; with one pass only ids move
    for (int j = 0; j < passes; ++j) {
        const int src = j % 2, dst = (j + 1) % 2;
        const bool last = j == passes - 1;
        int32_t *vals_out = passes == 1 ? b.vals[0] : b.vals[dst];
        k_radix_hist<K><<<n_shares, kWave, 0, st>>>(keys[src], n, share, shifts[j], b.hist, n_shares);
        k_scan_partial<<<scan_grid, kScanBlock, 0, st>>>(b.hist, n_hist, b.partial);
        k_scan_apply<<<scan_grid, kScanBlock, 0, st>>>(b.hist, n_hist, b.partial);
        k_radix_scatter<K><<<n_shares, kWave, 0, st>>>(keys[src], j == 0 ? nullptr : b.vals[src], n, share, shifts[j],
                                                       b.hist, n_shares, last ? nullptr : keys[dst], vals_out);
    }
    TIER_HIP(ctx, hipGetLastError());
    *order_out = passes == 1 ? b.vals[0] : b.vals[passes % 2];
    return TIER_OK;
}

}  // namespace

// Order the node ids by (count descending, id ascending).
static int sort_by_count(tier_ctx *ctx, const uint32_t *counts, sort_bufs &b, int32_t **order_out)
{
    const int64_t n = ctx->n_nodes;
    int rc = release_sort_bufs(ctx);
    if (rc == TIER_OK) rc = tier_ensure(ctx, &b.keys[0], &b.keys_cap[0], (size_t)n * sizeof(uint32_t));
    if (rc != TIER_OK) return rc;
    if (n > 0)
        k_keys_from_counts<<<grid_for(n, 256, 4096), 256, 0, ctx->stream>>>(counts, n, (uint32_t *)b.keys[0]);
    return sort_ids_by_keys<uint32_t>(ctx, b, order_out);
}

// Order the node ids by (score descending, id ascending); scores must not be NaN.
static int sort_by_score(tier_ctx *ctx, const double *scores, sort_bufs &b, int32_t **order_out)
{
    const int64_t n = ctx->n_nodes;
    int rc = release_sort_bufs(ctx);
    if (rc == TIER_OK) rc = tier_ensure(ctx, &b.keys[0], &b.keys_cap[0], (size_t)n * sizeof(uint64_t));
    if (rc != TIER_OK) return rc;
    if (n > 0)
        k_keys_from_scores<<<grid_for(n, 256, 4096), 256, 0, ctx->stream>>>(scores, n, (uint64_t *)b.keys[0]);
    return sort_ids_by_keys<uint64_t>(ctx, b, order_out);
}

// rank / order outputs shared by tier_rank and tier_rank_scores
static int emit_rank(tier_ctx *ctx, const int32_t *ord, int32_t *rank, int32_t *order)
{
    const int64_t n = ctx->n_nodes;
    if (rank && n > 0) k_slot_map<<<grid_for(n, 256, 4096), 256, 0, ctx->stream>>>(ord, n, n, rank);
    if (order && n > 0)
        TIER_HIP(ctx, hipMemcpyAsync(order, ord, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, ctx->stream));
    TIER_HIP(ctx, hipGetLastError());
    return TIER_OK;
}

static int64_t rows_within(const tier_ctx *ctx, uint64_t budget_bytes)
{
    const int64_t n_hot = (int64_t)(budget_bytes / (uint64_t)ctx->row_bytes);
    return n_hot > ctx->n_nodes ? ctx->n_nodes : n_hot;
}

// Before a placement writes the slot map: no gather may still read the old map or cache.  (A copy
// of rows fetched ahead that is still running reads neither: the placement queues up behind it.)
static int begin_place(tier_ctx *ctx)
{
    if (ctx->gather_stream != ctx->stream && ctx->maps_in_use) TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    ctx->maps_in_use = false;
    ctx->placed = false;
    ctx->boundary = false;
    ctx->n_hot = 0;
    return TIER_OK;
}

// The HBM cache for a slot map that is already on its way on the context's stream: order =
// rank -> node for the first n_hot ranks (in the context's sort scratch).  The cache is filled
// on the gather stream behind the map; the call does not wait for either.
static int finish_place(tier_ctx *ctx, const int32_t *order, int64_t n_hot, int32_t *slot_map, int64_t *n_hot_out)
{
    const int64_t n = ctx->n_nodes;
    hipStream_t st = ctx->stream, gs = ctx->gather_stream;
    TIER_HIP(ctx, hipGetLastError());

    // (re)build the HBM cache: cache row r = feature row of the node of rank r
    if (n_hot > 0) {
        int rc = tier_ensure(ctx, (void **)&ctx->cache, &ctx->cache_cap, (size_t)n_hot * (size_t)ctx->row_bytes);
        if (rc != TIER_OK) return rc;
    }
    if (gs != st) {
        // everything later on the gather stream (the fill below, every gather) comes after the map,
        // also when nothing is placed: a gather must never meet a half-written map
        TIER_HIP(ctx, hipEventRecord(ctx->ev_place, st));
        TIER_HIP(ctx, hipStreamWaitEvent(gs, ctx->ev_place, 0));
    }
    if (n_hot > 0) {
        if (gs != st) ctx->fill_pending = true;
        // rows that tier_prefetch has staged come from HBM, the others over the host link
        int rc = ctx->staged_rows > 0 ? tier_launch_fill_staged(ctx, order, n_hot, ctx->cache)
                                      : tier_launch_gather(ctx, order, n_hot, GATHER_HOST, ctx->cache, false);
        if (rc != TIER_OK) return rc;
    }
    ctx->staged_rows = 0;        // staged for one placement: the table may change before the next
    ctx->n_hot = n_hot;
    if (slot_map && n > 0)
        TIER_HIP(ctx, hipMemcpyAsync(slot_map, ctx->slot, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    ctx->placed = true;
    if (n_hot_out) *n_hot_out = n_hot;
    return TIER_OK;
}

// slot map + HBM cache from a complete order (rank -> node, in the context's sort scratch).
static int place_from_order(tier_ctx *ctx, const int32_t *order, uint64_t budget_bytes, int32_t *slot_map,
                            int64_t *n_hot_out)
{
    const int64_t n = ctx->n_nodes, n_hot = rows_within(ctx, budget_bytes);
    int rc = begin_place(ctx);
    if (rc != TIER_OK) return rc;
    if (n > 0) {
        k_slot_map<<<grid_for(n, 256, 4096), 256, 0, ctx->stream>>>(order, n, n_hot, ctx->slot);
        k_hot_bits<<<grid_for((n + 31) / 32, 256, 4096), 256, 0, ctx->stream>>>(ctx->slot, n, ctx->hot_bits);
    }
    return finish_place(ctx, order, n_hot, slot_map, n_hot_out);
}

extern "C" int tier_rank(tier_ctx *ctx, const uint32_t *counts, int32_t *rank, int32_t *order)
{
    if (!ctx || (!counts && ctx->n_nodes > 0)) return TIER_EINVAL;
    sort_bufs &b = ctx->sort;
    int32_t *ord = nullptr;
    int rc = sort_by_count(ctx, counts, b, &ord);
    if (rc != TIER_OK) return rc;
    return emit_rank(ctx, ord, rank, order);
}

extern "C" int tier_rank_scores(tier_ctx *ctx, const double *scores, int32_t *rank, int32_t *order)
{
    if (!ctx || (!scores && ctx->n_nodes > 0)) return TIER_EINVAL;
    sort_bufs &b = ctx->sort;
    int32_t *ord = nullptr;
    int rc = sort_by_score(ctx, scores, b, &ord);
    if (rc != TIER_OK) return rc;
    return emit_rank(ctx, ord, rank, order);
}

extern "C" int tier_place_scores(tier_ctx *ctx, const double *scores, uint64_t budget_bytes, int32_t *slot_map,
                                 int64_t *n_hot_out)
{
    if (!ctx || (!scores && ctx->n_nodes > 0)) return TIER_EINVAL;
    sort_bufs &b = ctx->sort;
    int32_t *order = nullptr;
    int rc = sort_by_score(ctx, scores, b, &order);
    if (rc != TIER_OK) return rc;
    return place_from_order(ctx, order, budget_bytes, slot_map, n_hot_out);
}

constexpr int kPrefetchBlocks = 32;

// ---- which rows to fetch ahead: the max_rows largest counts, without sorting ---------------------
// Four passes find the max_rows-th largest count t, one byte of it per pass from the top (a
// histogram of that byte over the counts that agree with t in the bytes above, then a walk down the
// histogram); a last pass takes every node with a larger count and as many of those with count t
// as are still missing, both by ascending id (two more passes: per-block counts, their prefix sums,
// then the places).  All on the device; nothing here waits.
constexpr int kSelectBlocks = 8192;  // most blocks of the last two passes; each owns a contiguous share of the nodes

struct select_t {
    uint32_t prefix;                 // the bytes of t found so far
    uint32_t pad_;
    unsigned long long remaining;    // rows still to find among the counts that agree with prefix
    uint32_t hist[256];
    uint32_t above[kSelectBlocks];   // per block: nodes of its share with count > t (then: of the shares before it)
    uint32_t equal[kSelectBlocks];   // likewise with count == t
};

__global__ void k_select_init(select_t *sel, unsigned long long max_rows)
{
    if (threadIdx.x == 0) {
        sel->prefix = 0u;
        sel->remaining = max_rows;
    }
    sel->hist[threadIdx.x] = 0u;     // 256 threads
}

__global__ __launch_bounds__(256) void k_select_hist(const uint32_t *__restrict__ counts, int64_t n, int shift, select_t *sel)
{
    __shared__ uint32_t s_h[256];
    s_h[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t prefix = sel->prefix;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    constexpr int kAhead = 4;                        // loads in flight per lane
    // (the whole wave takes every step: the first index is the same for all its lanes' steps)
    for (int64_t v0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v0 - threadIdx.x < n; v0 += kAhead * stride) {
        uint32_t keys[kAhead];
#pragma unroll
        for (int j = 0; j < kAhead; ++j) {
            const int64_t v = v0 + j * stride;
            keys[j] = v < n ? counts[v] : 0u;
        }
#pragma unroll
        for (int j = 0; j < kAhead; ++j) {
            const uint32_t key = keys[j];
            const bool in = v0 + j * stride < n && (shift == 24 || (key >> (shift + 8)) == (prefix >> (shift + 8)));
            const uint32_t digit = (key >> shift) & 255u;
            // counts are small numbers: most lanes of a wave hold the same digit, so one lane adds for all of them
            unsigned long long todo = __ballot(in);
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const uint32_t d = (uint32_t)__shfl((int)digit, leader);
                const unsigned long long same = __ballot(in && digit == d);
                if ((threadIdx.x & 63) == leader) atomicAdd(&s_h[d], (uint32_t)__popcll(same));
                todo &= ~same;
            }
        }
    }
    __syncthreads();
    if (s_h[threadIdx.x]) atomicAdd(&sel->hist[threadIdx.x], s_h[threadIdx.x]);
}

// The byte of t at `shift`: the largest digit d such that the counts with a digit >= d (and the bytes
// above as in prefix) number at least `remaining`.
__global__ void k_select_digit(select_t *sel, int shift)
{
    __shared__ uint32_t s_h[256];
    s_h[threadIdx.x] = sel->hist[threadIdx.x];
    sel->hist[threadIdx.x] = 0u;     // for the next pass
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long rem = sel->remaining;
        int d = 255;
        for (; d > 0; --d) {
            if (s_h[d] >= rem) break;
            rem -= s_h[d];
        }
        sel->prefix |= (uint32_t)d << shift;
        sel->remaining = rem;
    }
}

// Block b owns the nodes [b * share, (b + 1) * share), share a multiple of 256: how many of them
// lie above t, how many on it.
__global__ __launch_bounds__(256) void k_select_count(const uint32_t *__restrict__ counts, int64_t n, int64_t share, select_t *sel)
{
    __shared__ int s_a[4], s_e[4];
    const uint32_t t = sel->prefix;
    const int64_t lo = (int64_t)blockIdx.x * share;
    int64_t hi = lo + share;
    if (hi > n) hi = n;
    int a = 0, e = 0;
    for (int64_t v = lo + threadIdx.x; v < hi; v += 256) {
        const uint32_t key = counts[v];
        a += key > t;
        e += key == t;
    }
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off);
        e += __shfl_xor(e, off);
    }
    if ((threadIdx.x & 63) == 0) {
        s_a[threadIdx.x >> 6] = a;
        s_e[threadIdx.x >> 6] = e;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        sel->above[blockIdx.x] = (uint32_t)(s_a[0] + s_a[1] + s_a[2] + s_a[3]);
        sel->equal[blockIdx.x] = (uint32_t)(s_e[0] + s_e[1] + s_e[2] + s_e[3]);
    }
}

// Exclusive prefix sums over the blocks' two counts, in place (one block of 1024 threads).
__global__ __launch_bounds__(1024) void k_select_scan(select_t *sel, int n_blocks)
{
    __shared__ uint32_t s_w[2][16];
    constexpr int kPer = kSelectBlocks / 1024;
    const int first = threadIdx.x * kPer, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int which = 0; which < 2; ++which) {
        uint32_t *x = which ? sel->equal : sel->above;
        uint32_t mine[kPer], sum = 0u;
        for (int j = 0; j < kPer; ++j) {
            mine[j] = first + j < n_blocks ? x[first + j] : 0u;
            sum += mine[j];
        }
        uint32_t incl = sum;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t y = (uint32_t)__shfl_up((int)incl, d);
            if (lane >= d) incl += y;
        }
        if (lane == 63) s_w[which][wave] = incl;
        __syncthreads();
        uint32_t run = incl - sum;
        for (int w = 0; w < wave; ++w) run += s_w[which][w];
        for (int j = 0; j < kPer; ++j) {
            if (first + j < n_blocks) x[first + j] = run;
            run += mine[j];
        }
    }
}

// staged_of[v] = place of v's row in the staging area, or -1; staged_ids[place] = v; staged_bits as
// k_hot_bits would make them.  Places go by node id: first the nodes above t, then, as long as rows
// are missing, those on it.  A wave takes 64 consecutive nodes at a time.  keys_out (may be null):
// keys_out[place] = ~count, the sort key of the placement.
__global__ __launch_bounds__(256) void k_select_take(const uint32_t *__restrict__ counts, int64_t n, int64_t share,
                                                      int64_t max_rows, const select_t *sel, int32_t *__restrict__ staged_ids,
                                                      int32_t *__restrict__ staged_of, uint32_t *__restrict__ staged_bits,
                                                      uint32_t *__restrict__ keys_out)
{
    __shared__ int s_a[4], s_e[4];
    const uint32_t t = sel->prefix;
    const int64_t want_equal = (int64_t)sel->remaining;              // of the counts == t
    const int64_t n_above = max_rows - want_equal;                   // counts > t: all of them
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long below_me = (1ull << lane) - 1ull;
    const int64_t lo = (int64_t)blockIdx.x * share;
    int64_t hi = lo + share;
    if (hi > n) hi = n;
    int64_t base_a = sel->above[blockIdx.x], base_e = sel->equal[blockIdx.x];
    for (int64_t v0 = lo; v0 < hi; v0 += 256) {                      // the whole block takes every step
        const int64_t v = v0 + threadIdx.x;
        const uint32_t key = v < hi ? counts[v] : 0u;
        const bool above = v < hi && key > t, equal = v < hi && key == t;
        const unsigned long long m_above = __ballot(above), m_equal = __ballot(equal);
        __syncthreads();
        if (lane == 0) {
            s_a[wave] = __popcll(m_above);
            s_e[wave] = __popcll(m_equal);
        }
        __syncthreads();
        int64_t wa = base_a, we = base_e;
        for (int w = 0; w < wave; ++w) {
            wa += s_a[w];
            we += s_e[w];
        }
        int64_t place = -1;
        if (above) place = wa + __popcll(m_above & below_me);
        if (equal) {
            const int64_t j = we + __popcll(m_equal & below_me);
            if (j < want_equal) place = n_above + j;
        }
        if (v < hi) {
            staged_of[v] = (int32_t)place;
            if (place >= 0) {
                staged_ids[place] = (int32_t)v;
                if (keys_out) keys_out[place] = ~key;
            }
        }
        const unsigned long long m_in = __ballot(place >= 0);
        const int64_t w0 = v0 + 64 * wave;                           // this wave's first node
        if (lane == 0 && w0 < hi) {
            staged_bits[w0 >> 5] = (uint32_t)m_in;
            if (w0 + 32 < n) staged_bits[(w0 >> 5) + 1] = (uint32_t)(m_in >> 32);
        }
        base_a += s_a[0] + s_a[1] + s_a[2] + s_a[3];
        base_e += s_e[0] + s_e[1] + s_e[2] + s_e[3];
    }
}

// The passes that find t and the per-block places (everything but k_select_take), on the context's stream.
struct select_shape {
    int64_t share;     // nodes per block of the last passes
    int n_blocks;
};

static int select_threshold(tier_ctx *ctx, const uint32_t *counts, int64_t max_rows, select_shape *shape)
{
    const int64_t n = ctx->n_nodes;
    hipStream_t st = ctx->stream;
    int rc = tier_ensure(ctx, (void **)&ctx->select, &ctx->select_cap, sizeof(select_t));
    if (rc != TIER_OK) return rc;
    select_t *sel = (select_t *)ctx->select;
    const int grid = grid_for(n, 256, kSelectBlocks);
    shape->share = ((n + grid - 1) / grid + 255) / 256 * 256;
    shape->n_blocks = (int)((n + shape->share - 1) / shape->share);      // <= grid
    k_select_init<<<1, 256, 0, st>>>(sel, (unsigned long long)max_rows);
    for (int shift = 24; shift >= 0; shift -= 8) {
        k_select_hist<<<grid, 256, 0, st>>>(counts, n, shift, sel);
        k_select_digit<<<1, 256, 0, st>>>(sel, shift);
    }
    k_select_count<<<shape->n_blocks, 256, 0, st>>>(counts, n, shape->share, sel);
    k_select_scan<<<1, 1024, 0, st>>>(sel, shape->n_blocks);
    TIER_HIP(ctx, hipGetLastError());
    return TIER_OK;
}

// Fetch ahead of a placement: max_rows rows with the largest counts go to a staging area in HBM on
// the gather stream, and the next placement's cache fill takes every row it finds there from HBM.
extern "C" int tier_prefetch(tier_ctx *ctx, const uint32_t *counts, int64_t max_rows)
{
    if (!ctx || (!counts && ctx->n_nodes > 0) || max_rows < 0) return TIER_EINVAL;
    const int64_t n = ctx->n_nodes;
    hipStream_t st = ctx->stream, gs = ctx->gather_stream;
    if (max_rows > n) max_rows = n;
    // an earlier fill may still read the staging area and its maps
    if (gs != st) TIER_HIP(ctx, hipStreamSynchronize(gs));
    ctx->maps_in_use = false;
    ctx->fill_pending = false;
    ctx->staged_rows = 0;
    if (max_rows == 0) return TIER_OK;
    int rc = tier_ensure(ctx, (void **)&ctx->staged_ids, &ctx->staged_ids_cap, (size_t)max_rows * sizeof(int32_t));
    if (rc == TIER_OK) rc = tier_ensure(ctx, (void **)&ctx->staged_of, &ctx->staged_of_cap, (size_t)n * sizeof(int32_t));
    if (rc == TIER_OK)
        rc = tier_ensure(ctx, (void **)&ctx->staged_bits, &ctx->staged_bits_cap, (size_t)((n + 31) / 32) * sizeof(uint32_t));
    if (rc == TIER_OK)
        rc = tier_ensure(ctx, (void **)&ctx->staging, &ctx->staging_cap, (size_t)max_rows * (size_t)ctx->row_bytes);
    select_shape sh;
    if (rc == TIER_OK) rc = select_threshold(ctx, counts, max_rows, &sh);
    if (rc != TIER_OK) return rc;
    k_select_take<<<sh.n_blocks, 256, 0, st>>>(counts, n, sh.share, max_rows, (const select_t *)ctx->select, ctx->staged_ids,
                                               ctx->staged_of, ctx->staged_bits, nullptr);
    TIER_HIP(ctx, hipGetLastError());
    if (gs != st) {
        TIER_HIP(ctx, hipEventRecord(ctx->ev_place, st));
        TIER_HIP(ctx, hipStreamWaitEvent(gs, ctx->ev_place, 0));
    }
    // Half the blocks that a fill takes: this copy runs beside other work, whose kernel launches themselves
    // cross the host link and slow down the more requests are queued there (cfg3, 260 presampling launches
    // beside it: +4 ms with 32 blocks, +12 ms with 64; with 16 the copy loses more than the launches gain).
    rc = tier_launch_gather(ctx, ctx->staged_ids, max_rows, GATHER_HOST, ctx->staging, false, kPrefetchBlocks);
    if (rc != TIER_OK) return rc;
    ctx->staged_rows = max_rows;
    return TIER_OK;
}

// Placement by access count (Sec. 3.2, Sec. 4.1).  Only the n_hot first ranks matter, so on a large
// graph, when they are at most half the nodes, the order is not made for all of them: the n_hot nodes
// are selected as in tier_prefetch (above the n_hot-th largest count, then on it, by ascending id),
// which also writes slot = -1 for everyone else and the hot bits, and only those n_hot (key ~count,
// node) pairs are sorted, all four digits, stable from their id order: the same ranks as the full
// sort gives (111 M nodes, 10 % hot: 3 ms instead of 5.5), and nothing here waits for the set of
// varying digits.  It takes ~30 launches where the full sort of small counts takes ~10: below
// 16 M nodes the full sort is faster (2.4 M nodes: 0.2 ms against 0.65).
constexpr int64_t kSelectMinNodes = 1 << 24;
extern "C" int tier_place(tier_ctx *ctx, const uint32_t *counts, uint64_t budget_bytes, int32_t *slot_map,
                          int64_t *n_hot_out)
{
    if (!ctx || (!counts && ctx->n_nodes > 0)) return TIER_EINVAL;
    sort_bufs &b = ctx->sort;
    const int64_t n = ctx->n_nodes, n_hot = rows_within(ctx, budget_bytes);
    if (n < kSelectMinNodes || n_hot <= 0 || 2 * n_hot > n) {
        int32_t *order = nullptr;
        int rc = sort_by_count(ctx, counts, b, &order);
        if (rc != TIER_OK) return rc;
        return place_from_order(ctx, order, budget_bytes, slot_map, n_hot_out);
    }
    hipStream_t st = ctx->stream;
    int64_t share = (n_hot + kMaxShares - 1) / kMaxShares;
    if (share < 16 * kWave) share = 16 * kWave;
    share = (share + kWave - 1) / kWave * kWave;
    const int n_shares = (int)((n_hot + share - 1) / share);
    const int64_t n_hist = (int64_t)kDigits * n_shares;
    const int scan_grid = grid_for(n_hist, 4 * kScanBlock, 1024);
    int rc = release_sort_bufs(ctx);
    for (int i = 0; i < 2 && rc == TIER_OK; ++i) {
        rc = tier_ensure(ctx, &b.keys[i], &b.keys_cap[i], (size_t)n_hot * sizeof(uint32_t));
        if (rc == TIER_OK) rc = tier_ensure(ctx, (void **)&b.vals[i], &b.vals_cap[i], (size_t)n_hot * sizeof(int32_t));
    }
    if (rc == TIER_OK) rc = tier_ensure(ctx, (void **)&b.hist, &b.hist_cap, (size_t)n_hist * sizeof(uint32_t));
    if (rc != TIER_OK) return rc;
    if (!b.partial) TIER_HIP(ctx, hipMalloc(&b.partial, 1024 * sizeof(uint32_t)));
    select_shape sh;
    rc = select_threshold(ctx, counts, n_hot, &sh);
    if (rc == TIER_OK) rc = begin_place(ctx);
    if (rc != TIER_OK) return rc;
    uint32_t *keys[2] = {(uint32_t *)b.keys[0], (uint32_t *)b.keys[1]};
    k_select_take<<<sh.n_blocks, 256, 0, st>>>(counts, n, sh.share, n_hot, (const select_t *)ctx->select, b.vals[0], ctx->slot,
                                               ctx->hot_bits, keys[0]);
    for (int j = 0; j < 4; ++j) {                  // an even number of passes: the order ends up in vals[0]
        const int src = j % 2, dst = (j + 1) % 2;
        k_radix_hist<uint32_t><<<n_shares, kWave, 0, st>>>(keys[src], n_hot, share, 8 * j, b.hist, n_shares);
        k_scan_partial<<<scan_grid, kScanBlock, 0, st>>>(b.hist, n_hist, b.partial);
        k_scan_apply<<<scan_grid, kScanBlock, 0, st>>>(b.hist, n_hist, b.partial);
        k_radix_scatter<uint32_t><<<n_shares, kWave, 0, st>>>(keys[src], b.vals[src], n_hot, share, 8 * j, b.hist, n_shares,
                                                              j == 3 ? nullptr : keys[dst], b.vals[dst]);
    }
    k_slot_map<<<grid_for(n_hot, 256, 4096), 256, 0, st>>>(b.vals[0], n_hot, n_hot, ctx->slot);     // ranks of the chosen
    return finish_place(ctx, b.vals[0], n_hot, slot_map, n_hot_out);
}

// Placement for a graph and table already ordered by rank (Sec. 3.2 second method,
// Sec. 4.1): the first n_hot rows are the hot part, copied to HBM in one piece.
extern "C" int tier_place_boundary(tier_ctx *ctx, uint64_t budget_bytes, int64_t *n_hot_out)
{
    if (!ctx) return TIER_EINVAL;
    hipStream_t st = ctx->stream;
    int64_t n_hot = (int64_t)(budget_bytes / (uint64_t)ctx->row_bytes);
    if (n_hot > ctx->n_nodes) n_hot = ctx->n_nodes;
    TIER_HIP(ctx, hipStreamSynchronize(st));
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    ctx->placed = false;
    ctx->fill_pending = false;
    ctx->staged_rows = 0;
    ctx->n_hot = 0;
    if (n_hot > 0) {
        int rc = tier_ensure(ctx, (void **)&ctx->cache, &ctx->cache_cap, (size_t)n_hot * (size_t)ctx->row_bytes);
        if (rc != TIER_OK) return rc;
        TIER_HIP(ctx, hipMemcpyAsync(ctx->cache, ctx->host_rows, (size_t)n_hot * (size_t)ctx->row_bytes,
                                     hipMemcpyDefault, st));
        TIER_HIP(ctx, hipStreamSynchronize(st));
    }
    ctx->n_hot = n_hot;
    ctx->boundary = true;
    ctx->placed = true;
    if (n_hot_out) *n_hot_out = n_hot;
    return TIER_OK;
}

// ---- ranking for callers that cannot allocate ---------------------------------------------------
// Same ordering as tier_rank, with the sort's scratch (two key buffers, two id buffers, the digit
// histograms and the block sums of their scan) in one file-scope device array instead of memory
// the context allocates.  Nothing here calls hipMalloc, hipFree or any routine that allocates; all
// four 8-bit digits are sorted, so the call does not have to wait for the set of varying digits
// either and only enqueues kernels.  Every GPU holds its own copy of the array, at its own address,
// which hipGetSymbolAddress reports once per device; host code uses that address only, never the
// array's name.  Every kernel below overwrites what it reads of the scratch before it reads it
// (histograms and block sums are written in full each pass), so nothing has to be cleared between
// calls; two calls that overlap on one GPU would race on it.
namespace {

constexpr int64_t kStaticMaxNodes = TIER_RANK_STATIC_MAX_NODES;
constexpr int64_t kStaticShares = 1024;                        // shares of at least 1024 keys: at most 1024 of them
constexpr size_t kStaticKeys = (size_t)kStaticMaxNodes * sizeof(uint32_t);
constexpr size_t kStaticHist = (size_t)kDigits * kStaticShares * sizeof(uint32_t);
constexpr size_t kStaticPartial = 1024 * sizeof(uint32_t);
constexpr size_t kStaticBytes = 4 * kStaticKeys + kStaticHist + kStaticPartial;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once known

// Address of this device's copy of `scratch` (looked up on the first call on the device).
int static_scratch(unsigned char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return TIER_EHIP;
    }
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return TIER_EHIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = (unsigned char *)g_scratch_ptr[dev];
    return TIER_OK;
}

}  // namespace

extern "C" int tier_rank_static(const uint32_t *counts, int64_t n_nodes, int32_t *rank, int32_t *order, void *stream)
{
    if (n_nodes < 0 || (n_nodes > 0 && !counts) || (!rank && !order)) return TIER_EINVAL;
    if (n_nodes > kStaticMaxNodes) return TIER_ECAPACITY;      // more nodes than the static scratch holds
    if (n_nodes == 0) return TIER_OK;
    unsigned char *base = nullptr;
    int rc = static_scratch(&base);
    if (rc != TIER_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int64_t n = n_nodes;
    uint32_t *keys[2] = {(uint32_t *)base, (uint32_t *)(base + kStaticKeys)};
    int32_t *vals[2] = {(int32_t *)(base + 2 * kStaticKeys), (int32_t *)(base + 3 * kStaticKeys)};
    uint32_t *hist = (uint32_t *)(base + 4 * kStaticKeys);
    uint32_t *partial = (uint32_t *)(base + 4 * kStaticKeys + kStaticHist);

    int64_t share = (n + kStaticShares - 1) / kStaticShares;
    if (share < 16 * kWave) share = 16 * kWave;
    share = (share + kWave - 1) / kWave * kWave;
    const int n_shares = (int)((n + share - 1) / share);      // <= kStaticShares
    const int64_t n_hist = (int64_t)kDigits * n_shares;
    const int scan_grid = grid_for(n_hist, 4 * kScanBlock, 1024);
    k_keys_from_counts<<<grid_for(n, 256, 4096), 256, 0, st>>>(counts, n, keys[0]);
    // pass j reads buffers j % 2 and writes buffers (j + 1) % 2; the last pass writes the order where it is wanted
    for (int j = 0; j < 4; ++j) {
        const int src = j % 2, dst = (j + 1) % 2;
        const bool last = j == 3;
        int32_t *vals_out = last && order ? order : vals[dst];
        k_radix_hist<uint32_t><<<n_shares, kWave, 0, st>>>(keys[src], n, share, 8 * j, hist, n_shares);
        k_scan_partial<<<scan_grid, kScanBlock, 0, st>>>(hist, n_hist, partial);
        k_scan_apply<<<scan_grid, kScanBlock, 0, st>>>(hist, n_hist, partial);
        k_radix_scatter<uint32_t><<<n_shares, kWave, 0, st>>>(keys[src], j == 0 ? nullptr : vals[src], n, share, 8 * j, hist,
                                                              n_shares, last ? nullptr : keys[dst], vals_out);
    }
    if (rank) k_slot_map<<<grid_for(n, 256, 4096), 256, 0, st>>>(order ? order : vals[0], n, n, rank);
    if (hipGetLastError() != hipSuccess) return TIER_EHIP;
    return TIER_OK;
}
