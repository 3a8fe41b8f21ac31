// Hot/cold placement (Sec. 3.2: order by descending score, old-id -> rank map;
// Sec. 4.1: the top rows live in GPU memory, the rest in host memory).
//
// The score is the access count.  Ordering by (count descending, id ascending)
// is a stable sort of the ids 0..N-1 by the key (max_count - count): a
// least-significant-digit radix sort with 8-bit digits over only as many digits
// as max_count has.  Each wavefront owns one contiguous share of the input, so
// stability needs no cross-wavefront ordering: per-(digit, wavefront) counts are
// scanned digit-major into start offsets, and inside a wavefront the rank among
// equal digits comes from ballots.
#include "tier_internal.h"

namespace {

constexpr int kWave = 64;
constexpr int kDigits = 256;
constexpr int kMaxShares = 4096;
constexpr int kScanBlock = 256;

__global__ void k_max_u32(const uint32_t *__restrict__ x, int64_t n, uint32_t *__restrict__ out)
{
    uint32_t m = 0;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) m = x[i] > m ? x[i] : m;
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)m, off);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0 && m) atomicMax(out, m);
}

// keys of the first pass come from the counts; later passes read the previous pass
__device__ inline uint32_t load_key(const uint32_t *__restrict__ counts, const uint32_t *__restrict__ keys_in,
                                    uint32_t max_count, int64_t i)
{
    return counts ? max_count - counts[i] : keys_in[i];
}

// launched with one wavefront per block; block b owns items [b*share, (b+1)*share)
__global__ __launch_bounds__(kWave) void k_radix_hist(const uint32_t *__restrict__ counts,
                                                      const uint32_t *__restrict__ keys_in, uint32_t max_count,
                                                      int64_t n, int64_t share, int shift,
                                                      uint32_t *__restrict__ hist, int n_shares)
{
    __shared__ uint32_t s_hist[kDigits];
    for (int d = threadIdx.x; d < kDigits; d += kWave) s_hist[d] = 0;
    __syncthreads();
    int64_t lo = (int64_t)blockIdx.x * share, hi = lo + share;
    if (hi > n) hi = n;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kWave) {
        uint32_t key = load_key(counts, keys_in, max_count, i);
        atomicAdd(&s_hist[(key >> shift) & 255u], 1u);
    }
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

__global__ __launch_bounds__(kWave) void k_radix_scatter(const uint32_t *__restrict__ counts,
                                                         const uint32_t *__restrict__ keys_in,
                                                         const int32_t *__restrict__ vals_in, uint32_t max_count,
                                                         int64_t n, int64_t share, int shift,
                                                         const uint32_t *__restrict__ offsets, int n_shares,
                                                         uint32_t *__restrict__ keys_out,
                                                         int32_t *__restrict__ vals_out)
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
        uint32_t key = 0;
        int32_t val = 0;
        if (valid) {
            key = load_key(counts, keys_in, max_count, i);
            val = vals_in ? vals_in[i] : (int32_t)i;
        }
        const uint32_t digit = (key >> shift) & 255u;
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

__global__ void k_zero_u32(uint32_t *p) { *p = 0; }

int grid_for(int64_t n, int block, int cap)
{
    int64_t g = (n + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

struct sort_bufs {
    uint32_t *keys[2] = {nullptr, nullptr};
    int32_t *vals[2] = {nullptr, nullptr};
    uint32_t *hist = nullptr;
    uint32_t *partial = nullptr;
    uint32_t *max_dev = nullptr;
    ~sort_bufs()
    {
        for (int i = 0; i < 2; ++i) {
            (void)hipFree(keys[i]);
            (void)hipFree(vals[i]);
        }
        (void)hipFree(hist);
        (void)hipFree(partial);
        (void)hipFree(max_dev);
    }
};

}  // namespace

// Order the node ids by (count descending, id ascending) on the context's stream.
// *order points into b (rank -> node id) and is valid until b dies.  Waits once
// (for the largest count, which fixes the number of radix passes).
static int sort_by_count(tier_ctx *ctx, const uint32_t *counts, sort_bufs &b, int32_t **order_out)
{
    const int64_t n = ctx->n_nodes;
    hipStream_t st = ctx->stream;
    TIER_HIP(ctx, hipMalloc(&b.max_dev, sizeof(uint32_t)));
    k_zero_u32<<<1, 1, 0, st>>>(b.max_dev);
    if (n > 0) k_max_u32<<<grid_for(n, 256, 2048), 256, 0, st>>>(counts, n, b.max_dev);
    uint32_t max_count = 0;
    TIER_HIP(ctx, hipMemcpyAsync(ctx->meta_host, b.max_dev, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    TIER_HIP(ctx, hipStreamSynchronize(st));
    max_count = *(uint32_t *)ctx->meta_host;
    int passes = 0;
    while (passes < 4 && (max_count >> (8 * passes)) != 0) ++passes;

    TIER_HIP(ctx, hipMalloc(&b.vals[0], (size_t)(n > 0 ? n : 1) * sizeof(int32_t)));
    int32_t *order = b.vals[0];
    if (passes == 0) {
        k_iota<<<grid_for(n, 256, 4096), 256, 0, st>>>(order, n);
    } else {
        int64_t share = (n + kMaxShares - 1) / kMaxShares;
        if (share < 16 * kWave) share = 16 * kWave;
        share = (share + kWave - 1) / kWave * kWave;
        const int n_shares = (int)((n + share - 1) / share);
        const int64_t n_hist = (int64_t)kDigits * n_shares;
        const int scan_grid = grid_for(n_hist, 4 * kScanBlock, 1024);
        TIER_HIP(ctx, hipMalloc(&b.hist, (size_t)n_hist * sizeof(uint32_t)));
        TIER_HIP(ctx, hipMalloc(&b.partial, 1024 * sizeof(uint32_t)));
        if (passes > 1) {
            TIER_HIP(ctx, hipMalloc(&b.vals[1], (size_t)n * sizeof(int32_t)));
            TIER_HIP(ctx, hipMalloc(&b.keys[0], (size_t)n * sizeof(uint32_t)));
            if (passes > 2) TIER_HIP(ctx, hipMalloc(&b.keys[1], (size_t)n * sizeof(uint32_t)));
        }
        // ping-pong so that the last pass writes vals[0]
        int dst = (passes % 2 == 1) ? 0 : 1;
        const uint32_t *keys_in = nullptr;
        const int32_t *vals_in = nullptr;
        for (int p = 0; p < passes; ++p) {
            const uint32_t *cnt = p == 0 ? counts : nullptr;
            const bool last = p == passes - 1;
            uint32_t *keys_out = last ? nullptr : b.keys[passes > 2 ? dst : 0];
            k_radix_hist<<<n_shares, kWave, 0, st>>>(cnt, keys_in, max_count, n, share, 8 * p, b.hist, n_shares);
            k_scan_partial<<<scan_grid, kScanBlock, 0, st>>>(b.hist, n_hist, b.partial);
            k_scan_apply<<<scan_grid, kScanBlock, 0, st>>>(b.hist, n_hist, b.partial);
            k_radix_scatter<<<n_shares, kWave, 0, st>>>(cnt, keys_in, vals_in, max_count, n, share, 8 * p, b.hist,
                                                        n_shares, keys_out, b.vals[dst]);
            keys_in = keys_out;
            vals_in = b.vals[dst];
            dst ^= 1;
        }
    }
    TIER_HIP(ctx, hipGetLastError());
    *order_out = order;
    return TIER_OK;
}

extern "C" int tier_rank(tier_ctx *ctx, const uint32_t *counts, int32_t *rank, int32_t *order)
{
    if (!ctx || (!counts && ctx->n_nodes > 0)) return TIER_EINVAL;
    const int64_t n = ctx->n_nodes;
    sort_bufs b;
    int32_t *ord = nullptr;
    int rc = sort_by_count(ctx, counts, b, &ord);
    if (rc != TIER_OK) return rc;
    if (rank && n > 0) k_slot_map<<<grid_for(n, 256, 4096), 256, 0, ctx->stream>>>(ord, n, n, rank);
    if (order && n > 0)
        TIER_HIP(ctx, hipMemcpyAsync(order, ord, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, ctx->stream));
    TIER_HIP(ctx, hipGetLastError());
    TIER_HIP(ctx, hipStreamSynchronize(ctx->stream));   // the sort buffers are freed on return
    return TIER_OK;
}

extern "C" int tier_place(tier_ctx *ctx, const uint32_t *counts, uint64_t budget_bytes, int32_t *slot_map,
                          int64_t *n_hot_out)
{
    if (!ctx || (!counts && ctx->n_nodes > 0)) return TIER_EINVAL;
    const int64_t n = ctx->n_nodes;
    hipStream_t st = ctx->stream;
    int64_t n_hot = (int64_t)(budget_bytes / (uint64_t)ctx->row_bytes);
    if (n_hot > n) n_hot = n;

    sort_bufs b;
    int32_t *order = nullptr;
    int rc = sort_by_count(ctx, counts, b, &order);
    if (rc != TIER_OK) return rc;
    if (n > 0) k_slot_map<<<grid_for(n, 256, 4096), 256, 0, st>>>(order, n, n_hot, ctx->slot);

    // (re)build the HBM cache: cache row r = feature row of the node of rank r
    TIER_HIP(ctx, hipStreamSynchronize(st));
    ctx->placed = false;
    ctx->boundary = false;
    if (ctx->cache) TIER_HIP(ctx, hipFree(ctx->cache));
    ctx->cache = nullptr;
    ctx->n_hot = 0;
    if (n_hot > 0) {
        TIER_HIP(ctx, hipMalloc(&ctx->cache, (size_t)n_hot * (size_t)ctx->row_bytes));
        rc = tier_launch_gather(ctx, order, n_hot, GATHER_HOST, ctx->cache, false);
        if (rc != TIER_OK) return rc;
    }
    ctx->n_hot = n_hot;
    if (slot_map && n > 0)
        TIER_HIP(ctx, hipMemcpyAsync(slot_map, ctx->slot, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    TIER_HIP(ctx, hipStreamSynchronize(st));   // `order` is freed on return
    ctx->placed = true;
    if (n_hot_out) *n_hot_out = n_hot;
    return TIER_OK;
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
    ctx->placed = false;
    if (ctx->cache) TIER_HIP(ctx, hipFree(ctx->cache));
    ctx->cache = nullptr;
    ctx->n_hot = 0;
    if (n_hot > 0) {
        TIER_HIP(ctx, hipMalloc(&ctx->cache, (size_t)n_hot * (size_t)ctx->row_bytes));
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
