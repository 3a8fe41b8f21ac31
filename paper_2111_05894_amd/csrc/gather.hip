// Tiered feature gather (Sec. 4.1; Listing 1 without peer GPUs).
//
// For every requested id the row comes from the HBM cache when the node->slot
// map places it there, and from pinned host memory (read in place over the
// host link) otherwise.  A group of LPR lanes copies one row in 16-byte pieces,
// so a row is read and written with full-width coalesced accesses; several rows
// per group are in flight to cover the host link's latency.
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowsInFlight = 4;        // measured best of 2 / 4 / 8 on MI355X
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The id lists one launch serves (blockIdx.y picks one): a mini-batch each.
struct id_lists_t {
    const int32_t *ids[TIER_MAX_BATCHES];
    int64_t n[TIER_MAX_BATCHES];
    int64_t out_row[TIER_MAX_BATCHES];   // first output row of the list
};

// MODE: GATHER_SLOT     hot <=> slot[id] >= 0, cache row = slot[id]      (ids keep their meaning)
//       GATHER_BOUNDARY hot <=> id < n_hot, cache row = id, cold row = id - n_hot of the cold
//                       part (rows in rank order: the two-way branch of Listing 1)
//       GATHER_HOST     every row from host memory: the untiered copy that fills the HBM
//                       cache at placement time
template <int LPR, int MODE>
__global__ __launch_bounds__(kBlock) void k_gather(id_lists_t lists, const int32_t *__restrict__ slot,
                                                   const uint4 *__restrict__ cache,
                                                   const uint4 *__restrict__ host,
                                                   uint4 *__restrict__ out_base, int cpr, int64_t n_nodes,
                                                   int64_t n_hot, int64_t *__restrict__ meta, int count_hits)
{
    constexpr int kGroups = kBlock / LPR;
    const int32_t *__restrict__ ids = lists.ids[blockIdx.y];
    const int64_t n = lists.n[blockIdx.y];
    uint4 *__restrict__ out = out_base + lists.out_row[blockIdx.y] * cpr;
    const int lane = threadIdx.x % LPR;
    const int64_t group = (int64_t)blockIdx.x * kGroups + threadIdx.x / LPR;
    const int64_t n_groups = (int64_t)gridDim.x * kGroups;
    int hits = 0;
    int bad = 0;

    for (int64_t r0 = group * kRowsInFlight; r0 < n; r0 += n_groups * kRowsInFlight) {
        const uint4 *src[kRowsInFlight];
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) {
            int64_t r = r0 + j;
            src[j] = nullptr;
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
                if (r0 + j < n) {                  // streaming store: the output is not read back here
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

__global__ void k_clear_hits(int64_t *meta)
{
    if (threadIdx.x < META_HIT_STRIPES) meta[META_HIT_ROWS + threadIdx.x] = 0;
}
__global__ void k_clear_gather_error(int64_t *meta) { meta[META_ERROR] = 0; }

}  // namespace

// Cache fills (GATHER_HOST) run on the context's main stream, gathers on the gather stream
// with bookkeeping words of their own.
static int launch_lists(tier_ctx *ctx, const id_lists_t &lists, int n_lists, int64_t n_max, int mode, void *out,
                        bool count_hits)
{
    hipStream_t st = mode == GATHER_HOST ? ctx->stream : ctx->gather_stream;
    int64_t *meta = mode == GATHER_HOST ? ctx->meta : ctx->gmeta;
    if (count_hits) k_clear_hits<<<1, META_HIT_STRIPES, 0, st>>>(meta);
    if (n_max <= 0) return TIER_OK;
    const int cpr = (int)(ctx->row_bytes / 16);
    int lpr = 8;
    while (lpr < cpr && lpr < 64) lpr *= 2;
    const int groups = kBlock / lpr;
    int64_t blocks = (n_max + (int64_t)groups * kRowsInFlight - 1) / ((int64_t)groups * kRowsInFlight);
    const int64_t max_blocks = 1 << 18;     // beyond that groups loop; fewer blocks cost ~5 % of the all-hit rate
    if (blocks > max_blocks) blocks = max_blocks;
    const dim3 grid((unsigned)blocks, (unsigned)n_lists);
#define GATHER_LAUNCH(L, M)                                                                          \
    k_gather<L, M><<<grid, kBlock, 0, st>>>(lists, ctx->slot, (const uint4 *)ctx->cache,             \
                                            (const uint4 *)ctx->host_rows, (uint4 *)out, cpr,        \
                                            ctx->n_nodes, ctx->n_hot, meta, count_hits ? 1 : 0)
#define GATHER_CASE(L)                                                                               \
    case L:                                                                                          \
        if (mode == GATHER_SLOT) GATHER_LAUNCH(L, GATHER_SLOT);                                      \
        else if (mode == GATHER_BOUNDARY) GATHER_LAUNCH(L, GATHER_BOUNDARY);                         \
        else GATHER_LAUNCH(L, GATHER_HOST);                                                          \
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
    return launch_lists(ctx, lists, 1, n, mode, out, count_hits);
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
    int rc = launch_lists(ctx, lists, n_batches, n_max, ctx->boundary ? GATHER_BOUNDARY : GATHER_SLOT, out,
                          stats != nullptr);
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
    int rc = tier_launch_gather(ctx, ids, n, ctx->boundary ? GATHER_BOUNDARY : GATHER_SLOT, out, stats != nullptr);
    if (rc != TIER_OK) return rc;
    if (stats) return read_stats(ctx, n, stats);
    return TIER_OK;
}
