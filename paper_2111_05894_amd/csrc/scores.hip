// The paper's predictive score functions (Sec. 3.1), alternatives to the measured access
// count as input of the placement: out degree, and (weighted) reverse PageRank (Alg. 1).
//
// Row v of the context's CSR lists the sources of the edges into v, so in_degree(v) is
// the length of row v, and both scores are one pass over the edge list per round:
//   degree:  every entry u of the edge list adds 1 to degree[u]
//   Alg. 1:  after score[v] /= in_degree[v], every entry u of row v adds score[v] to
//            pulled[u] (u targets v, so u pulls v's score); then the damping step.
// Edges are spread evenly over threads (the row of an edge is found by bisection inside
// the block's span of rows), so hub rows need no special case.  The sums use hardware
// fp64 atomics: their order varies from run to run, the result to ~1e-16 relative.
#include "tier_internal.h"

#pragma clang fp contract(off)   // keep a + d * b as written (a product, then a sum)

namespace {

constexpr int kBlock = 256;
constexpr int kSpan = 2048;

__global__ void k_fill_u32(uint32_t *__restrict__ p, int64_t n, uint32_t v)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

__global__ void k_fill_f64(double *__restrict__ p, int64_t n, double v)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

__global__ void k_out_degree(const int32_t *__restrict__ indices, int64_t n_edges, uint32_t *__restrict__ degree)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride)
        atomicAdd(&degree[indices[e]], 1u);
}

__global__ void k_weight_train(const int32_t *__restrict__ tid, int64_t n_train, int64_t n_nodes, double weight,
                               double *__restrict__ score, int64_t *__restrict__ meta)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_train; i += stride) {
        int32_t v = tid[i];
        if ((uint32_t)v >= (uint64_t)n_nodes) atomicOr((int *)&meta[META_ERROR], 1);
        else score[v] = score[v] * weight;
    }
}

template <typename OffT>
__global__ void k_divide(const OffT *__restrict__ indptr, int64_t n, double *__restrict__ score,
                         double *__restrict__ pulled)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += stride) {
        const int64_t in_degree = (int64_t)(indptr[j + 1] - indptr[j]);
        if (in_degree > 0) score[j] = score[j] / (double)in_degree;
        pulled[j] = 0.0;
    }
}

template <typename OffT>
__device__ inline int64_t row_of(const OffT *__restrict__ nd, int64_t lo, int64_t hi, int64_t e)
{
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if ((int64_t)nd[mid] <= e) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <typename OffT>
__global__ __launch_bounds__(kBlock) void k_pull(const OffT *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                 int64_t n, int64_t n_edges, const double *__restrict__ score,
                                                 double *__restrict__ pulled)
{
    __shared__ int64_t s_span[2];
    for (int64_t first = (int64_t)blockIdx.x * kSpan; first < n_edges; first += (int64_t)gridDim.x * kSpan) {
        const int64_t last = (first + kSpan < n_edges ? first + kSpan : n_edges) - 1;
        __syncthreads();
        if (threadIdx.x < 2) s_span[threadIdx.x] = row_of<OffT>(indptr, 0, n - 1, threadIdx.x == 0 ? first : last);
        __syncthreads();
        const int64_t r_lo = s_span[0], r_hi = s_span[1];
        for (int64_t e = first + threadIdx.x; e <= last; e += kBlock) {
            const int64_t v = row_of<OffT>(indptr, r_lo, r_hi, e);
            unsafeAtomicAdd(&pulled[indices[e]], score[v]);
        }
    }
}

__global__ void k_damp(const double *__restrict__ pulled, int64_t n, double base, double d, double *__restrict__ score)
{
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += stride) {
        const double b = d * pulled[j];
        score[j] = base + b;
    }
}

int grid_for(int64_t n, int per_block, int cap)
{
    int64_t g = (n + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

extern "C" {

int tier_score_degree(tier_ctx *ctx, uint32_t *degree)
{
    if (!ctx || (!degree && ctx->n_nodes > 0)) return TIER_EINVAL;
    k_fill_u32<<<grid_for(ctx->n_nodes, kBlock, 4096), kBlock, 0, ctx->stream>>>(degree, ctx->n_nodes, 0u);
    if (ctx->n_edges > 0)
        k_out_degree<<<grid_for(ctx->n_edges, kBlock, 16384), kBlock, 0, ctx->stream>>>(ctx->indices, ctx->n_edges,
                                                                                       degree);
    TIER_HIP(ctx, hipGetLastError());
    return TIER_OK;
}

int tier_score_wrpr(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t iterations, double damp,
                    double *score)
{
    if (!ctx || (!score && ctx->n_nodes > 0) || n_train < 0 || (n_train > 0 && !train_ids) || iterations < 0)
        return TIER_EINVAL;
    if (!(damp >= 0.0 && damp <= 1.0)) return TIER_EINVAL;
    const int64_t n = ctx->n_nodes, ne = ctx->n_edges;
    if (n == 0) return TIER_OK;
    hipStream_t st = ctx->stream;
    int rc = tier_ensure(ctx, (void **)&ctx->pulled, &ctx->pulled_cap, (size_t)n * sizeof(double));
    if (rc != TIER_OK) return rc;
    double *pulled = ctx->pulled;        // kept by the context: no allocation after the first call
    const int g = grid_for(n, kBlock, 4096);
    k_fill_f64<<<g, kBlock, 0, st>>>(score, n, 1.0 / (double)n);
    if (n_train > 0)
        k_weight_train<<<grid_for(n_train, kBlock, 4096), kBlock, 0, st>>>(train_ids, n_train, n,
                                                                          (double)n / (double)n_train, score, ctx->meta);
    const double base = (1.0 - damp) / (double)n;
    for (int it = 0; it < iterations; ++it) {
        if (ctx->indptr_i64) {
            k_divide<int64_t><<<g, kBlock, 0, st>>>((const int64_t *)ctx->indptr, n, score, pulled);
            if (ne > 0)
                k_pull<int64_t><<<grid_for(ne, kSpan, 65536), kBlock, 0, st>>>((const int64_t *)ctx->indptr,
                                                                               ctx->indices, n, ne, score, pulled);
        } else {
            k_divide<int32_t><<<g, kBlock, 0, st>>>((const int32_t *)ctx->indptr, n, score, pulled);
            if (ne > 0)
                k_pull<int32_t><<<grid_for(ne, kSpan, 65536), kBlock, 0, st>>>((const int32_t *)ctx->indptr,
                                                                               ctx->indices, n, ne, score, pulled);
        }
        k_damp<<<g, kBlock, 0, st>>>(pulled, n, base, damp, score);
    }
    TIER_HIP(ctx, hipGetLastError());
    return tier_sync_meta(ctx);          // waits: reports a training id outside the graph
}

}  // extern "C"
