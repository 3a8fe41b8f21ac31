// Context life cycle, pinned host memory, size bounds and error strings.
#include <new>
#include "rng.h"
#include "tier_internal.h"

namespace {

// One pass over the graph at context creation: offsets non-decreasing and inside
// [0, n_edges], neighbour ids inside [0, n_nodes).  The sampler indexes with
// these values unchecked afterwards.
template <typename OffT>
__global__ void k_validate_csr(const OffT *__restrict__ indptr, const int32_t *__restrict__ indices,
                               int64_t n_nodes, int64_t n_edges, int *__restrict__ bad)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int flag = 0;
    for (int64_t v = t; v < n_nodes; v += stride) {
        int64_t a = (int64_t)indptr[v], b = (int64_t)indptr[v + 1];
        if (a < 0 || b < a || b > n_edges || b - a > 0x7fffffffLL) flag = 1;
    }
    if (t == 0 && (int64_t)indptr[0] != 0) flag = 1;
    if (t == 0 && (int64_t)indptr[n_nodes] != n_edges) flag = 1;
    for (int64_t e = t; e < n_edges; e += stride) {
        uint32_t u = (uint32_t)indices[e];
        if (u >= (uint64_t)n_nodes) flag = 1;
    }
    if (flag) atomicOr(bad, 1);
}

__global__ void k_fill_i32(int32_t *__restrict__ p, int64_t n, int32_t value)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = value;
}

__global__ void k_clear_error(int64_t *meta) { meta[META_ERROR] = 0; }

int grid_for(int64_t n, int block, int cap)
{
    int64_t g = (n + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

// Copy the bookkeeping array to the host and wait; a pending id error is
// reported once and cleared.
int tier_sync_meta(tier_ctx *c)
{
    TIER_HIP(c, hipMemcpyAsync(c->meta_host, c->meta, (size_t)c->n_slots * META_WORDS * sizeof(int64_t),
                               hipMemcpyDeviceToHost, c->stream));
    TIER_HIP(c, hipStreamSynchronize(c->stream));
    if (c->meta_host[META_ERROR] != 0) {
        k_clear_error<<<1, 1, 0, c->stream>>>(c->meta);
        return TIER_EINVAL;
    }
    return TIER_OK;
}

extern "C" {

int tier_host_alloc(void **ptr, size_t bytes)
{
    if (!ptr) return TIER_EINVAL;
    *ptr = nullptr;
    if (bytes == 0) return TIER_OK;
    hipError_t e = hipHostMalloc(ptr, bytes, hipHostMallocMapped | hipHostMallocPortable);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *ptr = nullptr;
        return e == hipErrorOutOfMemory ? TIER_ENOMEM : TIER_EHIP;
    }
    return TIER_OK;
}

int tier_host_free(void *ptr)
{
    if (!ptr) return TIER_OK;
    hipError_t e = hipHostFree(ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return TIER_EHIP;
    }
    return TIER_OK;
}

int tier_blocks_bounds(int64_t n_graph_nodes, int64_t n_seeds, const int32_t *fanouts, int32_t n_layers,
                       int64_t *cap_nodes, int64_t *cap_edges)
{
    if (!fanouts || !cap_nodes || !cap_edges || n_graph_nodes < 0 || n_seeds < 0) return TIER_EINVAL;
    if (n_layers < 1 || n_layers > TIER_MAX_LAYERS) return TIER_EINVAL;
    int64_t n = n_seeds < n_graph_nodes ? n_seeds : n_graph_nodes;
    cap_nodes[0] = n;
    for (int l = 0; l < n_layers; ++l) {
        int64_t k = fanouts[l];
        if (k < 1 || k > TIER_MAX_FANOUT) return TIER_EINVAL;
        cap_edges[l] = n * k;
        if (cap_edges[l] > 0x7fffffffLL) return TIER_EINVAL;   // block offsets are int32
        n = n * (1 + k);
        if (n > n_graph_nodes) n = n_graph_nodes;
        cap_nodes[l + 1] = n;
    }
    return TIER_OK;
}

uint64_t tier_batch_seed(uint64_t seed, uint32_t epoch, uint32_t batch)
{
    return tier::philox_r64((uint32_t)seed, (uint32_t)(seed >> 32), epoch, batch, 0u, tier::kTagBatch);
}

void tier_destroy(tier_ctx *ctx)
{
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);
    (void)hipFree(ctx->fresh);
    (void)hipFree(ctx->aux);
    (void)hipFree(ctx->flag);
    (void)hipFree(ctx->segbase);
    (void)hipFree(ctx->table);
    (void)hipFree(ctx->part_rec);
    (void)hipFree(ctx->part_rank);
    (void)hipFree(ctx->part_stage);
    (void)hipFree(ctx->part_rows);
    (void)hipFree(ctx->part_bk);
    (void)hipFree(ctx->f_beg);
    (void)hipFree(ctx->f_deg);
    (void)hipFree(ctx->slot);
    (void)hipFree(ctx->hot_bits);
    (void)hipFree(ctx->cache);
    (void)hipFree(ctx->staged_ids);
    (void)hipFree(ctx->staging);
    (void)hipFree(ctx->staged_of);
    (void)hipFree(ctx->staged_bits);
    (void)hipFree(ctx->select);
    (void)hipStreamSynchronize(ctx->gather_stream);
    (void)hipFree(ctx->claim);
    (void)hipFree(ctx->deferred);
    for (int i = 0; i < 2; ++i) {
        (void)hipFree(ctx->sort.keys[i]);
        (void)hipFree(ctx->sort.vals[i]);
    }
    (void)hipFree(ctx->sort.hist);
    (void)hipFree(ctx->sort.partial);
    (void)hipFree(ctx->sort.mask);
    if (ctx->ev_place) (void)hipEventDestroy(ctx->ev_place);
    (void)hipFree(ctx->gmeta);
    (void)hipHostFree(ctx->gmeta_host);
    (void)hipFree(ctx->meta);
    (void)hipHostFree(ctx->meta_host);
    (void)hipFree(ctx->partial_hop);
    (void)hipFree(ctx->partial_bm);
    (void)hipFree(ctx->ps_nodes);
    (void)hipFree(ctx->ps_col);
    (void)hipFree(ctx->pulled);
    (void)hipFree(ctx->scan_partial);
    (void)hipGetLastError();
    delete ctx;
}

static int create_impl(tier_ctx *c, const tier_csr *csr, const tier_feat *feat)
{
    TIER_HIP(c, hipGetDevice(&c->device));
    // the feature table must be memory the GPU can read in place
    hipPointerAttribute_t attr;
    TIER_HIP(c, hipPointerGetAttributes(&attr, feat->host_rows));
    if (attr.type != hipMemoryTypeHost && attr.type != hipMemoryTypeDevice &&
        attr.type != hipMemoryTypeManaged)
        return TIER_EINVAL;
    void *dev_view = nullptr;
    c->rows_on_host = attr.type == hipMemoryTypeHost;
    if (attr.type == hipMemoryTypeHost) {
        TIER_HIP(c, hipHostGetDevicePointer(&dev_view, const_cast<void *>(feat->host_rows), 0));
    } else {
        dev_view = const_cast<void *>(feat->host_rows);
    }
    c->host_rows = (const uint8_t *)dev_view;
    if (((uintptr_t)c->host_rows & 15u) != 0) return TIER_EINVAL;

    const int64_t n = c->n_nodes;
    c->n_words = (n + 31) / 32;
    c->bm_stride = (c->n_words + 31) / 32 * 32;
    if (c->bm_stride == 0) c->bm_stride = 32;
    c->seg_log2 = c->n_words > (1 << 20) ? 5 : 0;      // as sampler.hip's large_graph()
    c->n_seg = (c->n_words + (1ll << c->seg_log2) - 1) >> c->seg_log2;
    c->flag_stride = (c->n_seg + 15) / 16 * 16;
    // as many mini-batch slots as fit in 8 GiB of per-node scratch (two bitmaps, a flag byte and a
    // start position per segment: 0.26 - 0.41 bytes per node and slot)
    const int64_t per_slot = c->bm_stride * 8 + c->flag_stride + c->n_seg * 4 + 64;
    int64_t slots = (8LL << 30) / per_slot;
    c->n_slots = (int)(slots < 1 ? 1 : (slots > TIER_MAX_BATCHES ? TIER_MAX_BATCHES : slots));
    const size_t S = (size_t)c->n_slots;
    const int64_t words = c->bm_stride * (int64_t)S;
    const int64_t flags4 = (c->flag_stride > 0 ? c->flag_stride : 16) * (int64_t)S / 4;
    const int64_t segs = (c->n_seg > 0 ? c->n_seg : 1) * (int64_t)S;
    TIER_HIP(c, hipMalloc(&c->fresh, (size_t)words * sizeof(uint32_t)));
    TIER_HIP(c, hipMalloc(&c->aux, (size_t)words * sizeof(uint32_t)));
    TIER_HIP(c, hipMalloc(&c->flag, (size_t)flags4 * 4));
    TIER_HIP(c, hipMalloc(&c->segbase, (size_t)segs * sizeof(int32_t)));
    TIER_HIP(c, hipMalloc(&c->slot, (size_t)(n > 0 ? n : 1) * sizeof(int32_t)));
    TIER_HIP(c, hipMalloc(&c->hot_bits, (size_t)(c->n_words > 0 ? c->n_words : 1) * sizeof(uint32_t)));
    TIER_HIP(c, hipMalloc(&c->meta, S * META_WORDS * sizeof(int64_t)));
    TIER_HIP(c, hipHostMalloc((void **)&c->meta_host, S * META_WORDS * sizeof(int64_t), hipHostMallocDefault));
    TIER_HIP(c, hipMalloc(&c->gmeta, GMETA_WORDS * sizeof(int64_t)));
    TIER_HIP(c, hipHostMalloc((void **)&c->gmeta_host, GMETA_WORDS * sizeof(int64_t), hipHostMallocDefault));
    TIER_HIP(c, hipEventCreateWithFlags(&c->ev_place, hipEventDisableTiming));
    TIER_HIP(c, hipMalloc(&c->partial_hop, S * TIER_SCAN_BLOCKS * sizeof(int32_t)));
    TIER_HIP(c, hipMalloc(&c->partial_bm, S * TIER_SCAN_BLOCKS * sizeof(int32_t)));
    k_fill_i32<<<grid_for(words, 256, 8192), 256, 0, c->stream>>>((int32_t *)c->fresh, words, 0);
    k_fill_i32<<<grid_for(words, 256, 8192), 256, 0, c->stream>>>((int32_t *)c->aux, words, 0);
    k_fill_i32<<<grid_for(flags4, 256, 8192), 256, 0, c->stream>>>((int32_t *)c->flag, flags4, 0);
    k_fill_i32<<<grid_for(n, 256, 8192), 256, 0, c->stream>>>(c->slot, n, -1);          // nothing placed yet
    k_fill_i32<<<grid_for(c->n_words, 256, 8192), 256, 0, c->stream>>>((int32_t *)c->hot_bits, c->n_words, 0);
    k_fill_i32<<<1, 64, 0, c->stream>>>((int32_t *)c->gmeta, GMETA_WORDS * 2, 0);
    k_fill_i32<<<4, 256, 0, c->stream>>>((int32_t *)c->meta, (int64_t)S * META_WORDS * 2, 0);
    TIER_HIP(c, hipGetLastError());

    // validate the graph once
    int *bad = (int *)&c->meta[META_ERROR];
    int g = grid_for(c->n_edges > n ? c->n_edges : n, 256, 8192);
    if (c->indptr_i64)
        k_validate_csr<int64_t><<<g, 256, 0, c->stream>>>((const int64_t *)c->indptr, c->indices, n, c->n_edges, bad);
    else
        k_validate_csr<int32_t><<<g, 256, 0, c->stream>>>((const int32_t *)c->indptr, c->indices, n, c->n_edges, bad);
    TIER_HIP(c, hipGetLastError());
    TIER_HIP(c, hipMemcpyAsync(c->meta_host, c->meta, META_WORDS * sizeof(int64_t), hipMemcpyDeviceToHost, c->stream));
    TIER_HIP(c, hipStreamSynchronize(c->stream));
    if (c->meta_host[META_ERROR] != 0) return TIER_EINVAL;
    return TIER_OK;
}

int tier_create(tier_ctx **out, const tier_csr *csr, const tier_feat *feat, void *stream)
{
    if (!out) return TIER_EINVAL;
    *out = nullptr;
    if (!csr || !feat || !csr->indptr || (!csr->indices && csr->n_edges > 0) || !feat->host_rows) return TIER_EINVAL;
    if (csr->n_nodes < 0 || csr->n_nodes > 0x7fffffffLL || csr->n_edges < 0) return TIER_EINVAL;
    if (!csr->indptr_is_i64 && csr->n_edges > 0x7fffffffLL) return TIER_EINVAL;
    if (feat->row_bytes <= 0 || (feat->row_bytes & 15) != 0) return TIER_EINVAL;
    tier_ctx *c = new (std::nothrow) tier_ctx();
    if (!c) return TIER_ENOMEM;
    c->stream = (hipStream_t)stream;
    c->gather_stream = c->stream;
    c->n_nodes = csr->n_nodes;
    c->n_edges = csr->n_edges;
    c->indptr = csr->indptr;
    c->indptr_i64 = csr->indptr_is_i64 != 0;
    c->indices = csr->indices;
    c->row_bytes = feat->row_bytes;
    int rc = create_impl(c, csr, feat);
    if (rc != TIER_OK) {
        tier_destroy(c);
        return rc;
    }
    *out = c;
    return TIER_OK;
}

}  // extern "C"

int tier_ensure(tier_ctx *ctx, void **buf, size_t *cap, size_t bytes)
{
    if (bytes == 0) bytes = 1;
    if (*buf && *cap >= bytes) return TIER_OK;
    TIER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    if (*buf) TIER_HIP(ctx, hipFree(*buf));
    *buf = nullptr;
    *cap = 0;
    TIER_HIP(ctx, hipMalloc(buf, bytes));
    *cap = bytes;
    return TIER_OK;
}

extern "C" {

const char *tier_strerror(int status)
{
    switch (status) {
    case TIER_OK: return "ok";
    case TIER_EINVAL: return "invalid argument";
    case TIER_ENOMEM: return "out of memory";
    case TIER_EHIP: return "HIP call failed";
    case TIER_ECAPACITY: return "output buffer smaller than the upper bound";
    case TIER_ESTATE: return "call out of order";
    default: return "unknown status";
    }
}

int tier_last_hip_error(const tier_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

int tier_set_segment_words(tier_ctx *ctx, int32_t words)
{
    if (!ctx || (words != 1 && words != 32)) return TIER_EINVAL;
    TIER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const int seg_log2 = words == 32 ? 5 : 0;
    if (seg_log2 == ctx->seg_log2) return TIER_OK;
    const int64_t n_seg = (ctx->n_words + words - 1) / words;
    const int64_t flag_stride = (n_seg + 15) / 16 * 16;
    const int64_t flags4 = (flag_stride > 0 ? flag_stride : 16) * (int64_t)ctx->n_slots / 4;
    const int64_t segs = (n_seg > 0 ? n_seg : 1) * (int64_t)ctx->n_slots;
    uint8_t *flag = nullptr;
    int32_t *segbase = nullptr;
    TIER_HIP(ctx, hipMalloc(&flag, (size_t)flags4 * 4));
    hipError_t e = hipMalloc(&segbase, (size_t)segs * sizeof(int32_t));
    if (e != hipSuccess) {
        (void)hipFree(flag);
        TIER_HIP(ctx, e);
    }
    (void)hipFree(ctx->flag);
    (void)hipFree(ctx->segbase);
    ctx->flag = flag;
    ctx->segbase = segbase;
    ctx->seg_log2 = seg_log2;
    ctx->n_seg = n_seg;
    ctx->flag_stride = flag_stride;
    k_fill_i32<<<grid_for(flags4, 256, 8192), 256, 0, ctx->stream>>>((int32_t *)ctx->flag, flags4, 0);
    TIER_HIP(ctx, hipGetLastError());
    return TIER_OK;
}

int tier_set_gather_stream(tier_ctx *ctx, void *stream)
{
    if (!ctx) return TIER_EINVAL;
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    ctx->gather_stream = stream ? (hipStream_t)stream : ctx->stream;
    return TIER_OK;
}

}  // extern "C"
