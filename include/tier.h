/*
 * tier.h -- C ABI of the data-tiering hot path for mini-batch GNN training
 *           on one MI355X (gfx950).
 *
 * The library keeps frequently read node-feature rows in GPU memory (HBM) and
 * the rest in pinned host memory that GPU threads read directly ("zero-copy"),
 * after the method of "Graph Neural Network Training with Data Tiering"
 * (Min et al., MLSys 2022).  Its four steps:
 *
 *   tier_presample          access count of every node over sampled mini-batches
 *                           (the measured access frequency of Sec. 3.1 / Sec. 5.2)
 *   tier_place              order nodes by count, keep the top rows in HBM
 *                           (Sec. 3.2 ordering and old-id -> rank map, Sec. 4.1 placement)
 *   tier_sample_minibatch   uniform fixed-fanout neighbour sampling and the
 *                           sub-graph of the sampled nodes (Sec. 2.2)
 *   tier_gather_features    dense rows for a list of node ids, each row read
 *                           from HBM when placed there and from host memory
 *                           otherwise (Sec. 4.1; Listing 1 without peer GPUs)
 *
 * Conventions
 *   - Every pointer is marked (device) or (host).  "device" means memory the GPU
 *     can address: hipMalloc memory, or pinned host memory for the feature table.
 *   - The caller owns every buffer it passes in; the library owns the context,
 *     the HBM cache, the node->slot map and its scratch memory.
 *   - All work is enqueued on the HIP stream given to tier_create.  A call that
 *     returns host-side results (sizes, counters) waits for that stream; the
 *     others return once the work is enqueued.
 *   - Return value: TIER_OK (0) or a negative tier_status.  Nothing is thrown and
 *     nothing is printed.  tier_strerror names a status; tier_last_hip_error gives
 *     the HIP error behind a TIER_EHIP.
 *   - A context must not be used from two threads at once.
 *   - Node ids are int32 in [0, n_nodes); every degree is below 2^31.  Adjacency lists
 *     need not be sorted.  Positions of a list are what is sampled: a list that holds a
 *     neighbour twice can have it drawn twice (two edges of the block, one frontier node).
 */
#ifndef TIER_H
#define TIER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIER_MAX_LAYERS 8    /* hops per mini-batch                              */
#define TIER_MAX_FANOUT 64   /* neighbours drawn per node per hop (one wavefront) */
#define TIER_MAX_BATCHES 64  /* mini-batches one tier_sample_minibatches call can take  */

typedef enum {
    TIER_OK = 0,
    TIER_EINVAL = -1,     /* bad argument: null pointer, size < 0, row_bytes not a multiple of 16,
                             fanout outside [1, TIER_MAX_FANOUT], layers outside [1, TIER_MAX_LAYERS] */
    TIER_ENOMEM = -2,     /* host or device allocation failed                                      */
    TIER_EHIP = -3,       /* a HIP call failed; see tier_last_hip_error                            */
    TIER_ECAPACITY = -4,  /* a caller-provided output buffer is smaller than the upper bound       */
    TIER_ESTATE = -5      /* call out of order (gather before place)                               */
} tier_status;

typedef struct tier_ctx tier_ctx;

/* Graph in compressed sparse rows (Sec. 3.2: node list + edge list).  Row v lists
 * the nodes that are sampled for v, i.e. the sources of the edges into v. */
typedef struct {
    int64_t n_nodes;
    int64_t n_edges;
    const void *indptr;       /* (device) n_nodes + 1 offsets, int32 or int64       */
    int32_t indptr_is_i64;    /* 0: int32 offsets, 1: int64 offsets                 */
    const int32_t *indices;   /* (device) n_edges neighbour ids                      */
} tier_csr;

/* Node feature table, one row per node (Sec. 2.1: N x D matrix; rows of 512 B - 4 KB). */
typedef struct {
    const void *host_rows;    /* (device-visible pinned host) n_nodes * row_bytes bytes,
                                 e.g. from tier_host_alloc or hipHostMalloc            */
    int64_t row_bytes;        /* bytes per row, a multiple of 16                       */
} tier_feat;

/* Sub-graph of one mini-batch: one block per hop (Sec. 2.2).
 * frontier_0 = the seeds; frontier_{l+1} = frontier_l followed by the nodes first
 * reached at hop l in ascending id order.  nodes[] holds frontier_L, and frontier_l
 * is its first n_nodes[l] entries.  Block l: dst = frontier_l, src = frontier_{l+1};
 * the sampled neighbours of dst i are entries row_ptr[l][i] .. row_ptr[l][i+1]-1 of
 * col[l] (index into nodes[]) and eid[l] (position in the graph's indices[]).
 * The caller allocates the device buffers to the sizes tier_blocks_bounds reports
 * and fills the cap_* fields; the library fills n_nodes / n_edges. */
typedef struct {
    int32_t *nodes;                       /* (device) cap_nodes entries                  */
    int64_t cap_nodes;
    int32_t *row_ptr[TIER_MAX_LAYERS];    /* (device) cap_dst[l] + 1 entries             */
    int32_t *col[TIER_MAX_LAYERS];        /* (device) cap_edges[l] entries               */
    int64_t *eid[TIER_MAX_LAYERS];        /* (device) cap_edges[l] entries               */
    int64_t cap_dst[TIER_MAX_LAYERS];
    int64_t cap_edges[TIER_MAX_LAYERS];
    int64_t n_nodes[TIER_MAX_LAYERS + 1]; /* (host, out) |frontier_l|, l = 0..n_layers   */
    int64_t n_edges[TIER_MAX_LAYERS];     /* (host, out) edges of block l                */
} tier_blocks;

/* Blocks of several mini-batches sampled by one call, each array strided by
 * mini-batch: mini-batch s has its frontier at nodes + s * nodes_stride, its block l
 * at row_ptr[l] + s * row_ptr_stride[l], col[l] + s * edge_stride[l] and
 * eid[l] + s * edge_stride[l], laid out as in tier_blocks.  Strides must reach the
 * bounds of tier_blocks_bounds for one mini-batch (row_ptr: bound + 1). */
typedef struct {
    int32_t *nodes;                           /* (device) n_batches * nodes_stride entries          */
    int64_t nodes_stride;
    int32_t *row_ptr[TIER_MAX_LAYERS];        /* (device) n_batches * row_ptr_stride[l] entries     */
    int32_t *col[TIER_MAX_LAYERS];            /* (device) n_batches * edge_stride[l] entries        */
    int64_t *eid[TIER_MAX_LAYERS];            /* (device) n_batches * edge_stride[l] entries        */
    int64_t row_ptr_stride[TIER_MAX_LAYERS];
    int64_t edge_stride[TIER_MAX_LAYERS];
    int64_t *n_nodes;   /* (host, out) n_batches x (TIER_MAX_LAYERS + 1): |frontier_l| of batch s at [s*(TIER_MAX_LAYERS+1) + l] */
    int64_t *n_edges;   /* (host, out) n_batches x TIER_MAX_LAYERS: edges of block l of batch s at [s*TIER_MAX_LAYERS + l]      */
} tier_blocks_batch;

typedef struct {
    int64_t hit_rows;    /* rows read from the HBM cache   */
    int64_t miss_rows;   /* rows not in the HBM cache      */
    int64_t link_rows;   /* rows read over the host link: miss_rows, or the distinct ones among them
                            when tier_set_gather_dedup is on */
} tier_gather_stats;

/* Pinned, GPU-mapped host memory for a feature table (the zero-copy space of
 * Sec. 4.1).  *ptr is valid on the host and on the GPU.  Free with tier_host_free. */
int tier_host_alloc(void **ptr, size_t bytes);
int tier_host_free(void *ptr);

/* Upper bounds of the sizes of one mini-batch's blocks: frontier sizes
 * cap_nodes[0..n_layers] and per-hop edge counts cap_edges[0..n_layers-1], both
 * (host, out).  Block l needs cap_dst = cap_nodes[l]; nodes[] needs cap_nodes[n_layers]. */
int tier_blocks_bounds(int64_t n_graph_nodes, int64_t n_seeds, const int32_t *fanouts /* host */,
                       int32_t n_layers, int64_t *cap_nodes, int64_t *cap_edges);

/* Create a context for one graph and one feature table on the current device.
 * The graph arrays and the feature table are referenced, not copied, and must
 * outlive the context.  stream is a hipStream_t (NULL = the default stream).
 * Allocates scratch proportional to n_nodes: 4 bytes per node for the slot map and
 * 0.26 - 0.41 bytes per node for each mini-batch that can be sampled at once (as many,
 * up to TIER_MAX_BATCHES, as fit in 8 GiB).  The first sampling call adds the sampler's
 * index (8 bytes per node of the largest frontier that can draw, per mini-batch slot) and,
 * above 32 M nodes, 16 bytes per edge of the bound on the largest hop's edges for every
 * mini-batch of the call (new nodes are sorted there, not marked in a bitmap). */
int tier_create(tier_ctx **out, const tier_csr *csr, const tier_feat *feat, void *stream);
void tier_destroy(tier_ctx *ctx);

/* Access counts (Sec. 3.1, Sec. 5.2).  train_ids (device, n_train ids, distinct) is
 * cut into consecutive mini-batches of batch_size seeds in the given order; batch b
 * of epoch e is sampled exactly as tier_sample_minibatch would with the seed
 * tier_batch_seed(seed, e, b); counts[v] (device, n_nodes entries, overwritten) is
 * the number of (epoch, batch) pairs whose sampled sub-graph contains v, i.e. the
 * number of feature rows of v a gather per mini-batch would read.  Asynchronous.
 * total_rows / total_edges (host, optional): sums over all batches of the frontier
 * size and of the sampled edges; asking for either makes the call wait. */
int tier_presample(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                   const int32_t *fanouts /* host */, int32_t n_layers, int32_t epochs, uint64_t seed,
                   uint32_t *counts, int64_t *total_rows, int64_t *total_edges);

/* A part of tier_presample (Sec. 3.1): the mini-batches [first_batch, first_batch + n_batches)
 * of every epoch, cut from train_ids and seeded exactly as there, so that the ranges of several
 * calls add up to tier_presample's counts.  accumulate != 0: counts[] is added to, not
 * overwritten.  What it is for: counts of the first mini-batches already tell which rows will
 * be hottest (see tier_prefetch).  Asynchronous. */
int tier_presample_range(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                         const int32_t *fanouts /* host */, int32_t n_layers, int32_t epochs, uint64_t seed,
                         int64_t first_batch, int64_t n_batches, int32_t accumulate, uint32_t *counts);

/* Access counts by the other reading of Sec. 3.1's "number of samples": the same
 * mini-batches as tier_presample, but counts[v] (device, n_nodes entries, overwritten) is
 * the number of times v is a seed plus the number of sampled edges whose source it is,
 * so a node that a mini-batch reaches over many edges counts that many times and the sum
 * of counts is the number of seeds plus the number of sampled edges.  A score for
 * tier_place like the counts of tier_presample.  Asynchronous; total_draws (host,
 * optional) receives that sum and makes the call wait. */
int tier_presample_draws(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t batch_size,
                         const int32_t *fanouts /* host */, int32_t n_layers, int32_t epochs, uint64_t seed,
                         uint32_t *counts, int64_t *total_draws);

/* Seed of mini-batch `batch` of epoch `epoch` derived from a run seed (host only). */
uint64_t tier_batch_seed(uint64_t seed, uint32_t epoch, uint32_t batch);

/* Placement (Sec. 3.2, Sec. 4.1).  Nodes are ordered by descending count, equal
 * counts by ascending id; rank = position in that order (the old-id -> rank map of
 * Sec. 3.2).  The first n_hot = min(n_nodes, budget_bytes / row_bytes) rows are
 * copied into an HBM cache owned by the context (cache row = rank) and the
 * node->slot map becomes slot[v] = rank[v] if rank[v] < n_hot, else -1.  Replaces
 * any earlier placement.  counts: (device) n_nodes entries.  slot_map (device,
 * optional): receives a copy of the map.  n_hot (host, optional).  Waits for gathers
 * still running on the gather stream and, on graphs below 2^24 nodes or with more than
 * half the nodes hot (where all nodes are sorted), once inside the sort; then returns with
 * the map enqueued on the context's stream and the cache fill enqueued on the gather
 * stream (tier_set_gather_stream), ahead of every later gather: the caller may go on
 * sampling while the hot rows cross the host link.  The host table must not change
 * before that fill is done (synchronize the gather stream first). */
int tier_place(tier_ctx *ctx, const uint32_t *counts, uint64_t budget_bytes,
               int32_t *slot_map, int64_t *n_hot);

/* The paper's predictive scores (Sec. 3.1), alternatives to the measured access count.
 * Edges run source -> target and row v of the graph lists the sources of the edges into v.
 *
 * tier_score_degree: degree[u] = out degree of u = number of adjacency lists that hold u
 * (the simplest of the scores of Sec. 3.1).  degree: (device) n_nodes entries, overwritten; feed it
 * to tier_place / tier_rank as the counts.  Asynchronous.
 *
 * tier_score_wrpr: weighted reverse PageRank (Alg. 1): score = 1/N, times N/n_train on the
 * training nodes; `iterations` rounds of { score[j] /= in_degree[j] (skipped when 0);
 * every node sums the scores of the nodes it targets; score[j] = (1-damp)/N + damp*sum }.
 * n_train = 0 gives plain reverse PageRank cut after `iterations` rounds (Sec. 3.1).
 * The paper runs 5 rounds and leaves damp open (0.85 is PageRank's usual value).
 * train_ids: (device) distinct ids.  score: (device) n_nodes doubles, overwritten.
 * fp64 throughout; the order of each node's sum varies from run to run, so results
 * agree to ~1e-15 relative, not bit for bit.  Waits. */
int tier_score_degree(tier_ctx *ctx, uint32_t *degree);
int tier_score_wrpr(tier_ctx *ctx, const int32_t *train_ids, int64_t n_train, int32_t iterations, double damp,
                    double *score);

/* Ranking and placement by a real-valued score (descending, equal scores by ascending
 * id; no NaN): as tier_rank and tier_place.  scores: (device) n_nodes doubles. */
int tier_rank_scores(tier_ctx *ctx, const double *scores, int32_t *rank, int32_t *order);
int tier_place_scores(tier_ctx *ctx, const double *scores, uint64_t budget_bytes, int32_t *slot_map,
                      int64_t *n_hot);

/* The ranking alone (Sec. 3.2: "srt_idx", the indices that sort the scores in
 * descending order, and the old-id -> new-id map built from them).  counts: (device)
 * n_nodes scores.  rank (device, optional): rank[v] = position of v in the order (count
 * descending, id ascending) = the new id of v.  order (device, optional): order[r] = the
 * node of rank r.  Waits once inside the sort; the outputs are complete in the order of
 * the context's stream. */
int tier_rank(tier_ctx *ctx, const uint32_t *counts, int32_t *rank, int32_t *order);

/* tier_rank for callers that cannot allocate memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same rank / order as tier_rank for the same
 * counts, needs no context, calls no allocating routine and does not wait: it only enqueues
 * kernels on `stream` (a hipStream_t, NULL = the default stream).  The sort's scratch lives in a
 * device array inside the library, TIER_RANK_STATIC_MAX_NODES keys long (about 17 MB on every
 * GPU the library is used on, held until the process ends); more nodes give TIER_ECAPACITY.
 * All calls on one GPU share that scratch: calls that overlap in time on one GPU (different
 * streams or threads) race on it; calls on one stream are safe one after the other.
 * counts: (device) n_nodes entries; rank, order: (device, either may be NULL, not both) n_nodes
 * entries each, complete in the order of `stream`. */
#define TIER_RANK_STATIC_MAX_NODES (1 << 20)
int tier_rank_static(const uint32_t *counts, int64_t n_nodes, int32_t *rank, int32_t *order, void *stream);

/* Graph reordering (Sec. 3.2, Alg. 2): the context's graph with every node renamed to
 * rank[node]: new node r has the neighbour list of order[r], in its old order, values
 * renamed.  indptr_new: (device) n_nodes + 1 offsets of the context graph's offset type;
 * indices_new: (device) n_edges ids.  rank/order as from tier_rank; TIER_EINVAL (and
 * nothing written) unless rank is a permutation of 0..n_nodes-1 and order its inverse.  Waits. */
int tier_reorder_graph(tier_ctx *ctx, const int32_t *rank, const int32_t *order, void *indptr_new,
                       int32_t *indices_new);

/* Feature rows follow their nodes (Sec. 3.2): rows_new[rank[v]] = row v of the context's
 * table.  rows_new: (device-visible: pinned host or device) n_nodes * row_bytes bytes,
 * 16-byte aligned, not overlapping the table.  Waits for a check of rank (TIER_EINVAL
 * unless it is a permutation), then the copy itself is asynchronous. */
int tier_reorder_rows(tier_ctx *ctx, const int32_t *rank, void *rows_new);

/* out[i] = rank[ids[i]] (e.g. the training ids of the reordered graph).  ids, out:
 * (device) n entries.  Waits; TIER_EINVAL if an id is outside [0, n_nodes). */
int tier_relabel_ids(tier_ctx *ctx, const int32_t *rank, const int32_t *ids, int64_t n, int32_t *out);

/* Fetch ahead of a placement (Sec. 4.1's hot part, moved early).  The max_rows first rows by
 * `counts` (device, n_nodes entries; count descending, id ascending: the order of tier_place)
 * are copied from the feature table to a staging area in HBM, on the gather stream behind
 * whatever is queued there.  The next tier_place / tier_place_scores takes every row of its
 * cache that it finds staged from HBM instead of the table; the placement itself (slot map,
 * cache contents) is the same with or without this call, whatever counts were given here.
 * For callers whose host link is idle while counts are still being collected: counts of the
 * first mini-batches (tier_presample_range) already name the hottest rows.  The staged rows
 * serve one placement and must not change in the table before it.  Scratch owned by the
 * context: max_rows * row_bytes + 4.2 bytes per node.  Asynchronous once that scratch is
 * there (it waits for the gather stream first when that is a stream of its own). */
int tier_prefetch(tier_ctx *ctx, const uint32_t *counts, int64_t max_rows);

/* Placement for a context whose graph and table are already in rank order (created on
 * the outputs of tier_reorder_graph / tier_reorder_rows): the hot part is the first
 * n_hot = min(n_nodes, budget_bytes / row_bytes) rows (Sec. 4.1), copied to HBM in one
 * piece; tier_gather_features then branches on id < n_hot (Listing 1: the cold part is
 * indexed by id - n_hot) and reads no map.  Replaces any earlier placement.  Waits. */
int tier_place_boundary(tier_ctx *ctx, uint64_t budget_bytes, int64_t *n_hot);

/* One mini-batch (Sec. 2.2).  seeds: (device) n_seeds distinct node ids (an id outside the
 * graph or a repeated seed makes the call return TIER_EINVAL, its outputs undefined).  At hop l
 * every node of frontier_l draws min(fanouts[l], degree) distinct neighbours
 * uniformly at random (all of them, in adjacency order, when degree <= fanouts[l]);
 * draws are a pure function of (seed, node, hop, draw index), so a mini-batch is
 * reproducible.  Buffers in *out must reach the bounds of tier_blocks_bounds, else
 * TIER_ECAPACITY.  Waits (it returns the block sizes). */
int tier_sample_minibatch(tier_ctx *ctx, const int32_t *seeds, int32_t n_seeds,
                          const int32_t *fanouts /* host */, int32_t n_layers, uint64_t seed,
                          tier_blocks *out);

/* Several mini-batches at once (Sec. 2.2; one mini-batch alone cannot fill the GPU,
 * so a training loop that prefetches samples them together).  seeds: (device)
 * n_seeds_total ids; mini-batch s takes seeds[s*batch_size .. (s+1)*batch_size) (the
 * last one what is left, possibly nothing) and samples with batch_seeds[s] (host,
 * n_batches entries), giving exactly what tier_sample_minibatch gives for those seeds
 * and that seed.  1 <= n_batches <= tier_max_batches(ctx);
 * n_seeds_total <= n_batches * batch_size.  Waits. */
int tier_sample_minibatches(tier_ctx *ctx, const int32_t *seeds, int64_t n_seeds_total, int32_t batch_size,
                            int32_t n_batches, const int32_t *fanouts /* host */, int32_t n_layers,
                            const uint64_t *batch_seeds /* host */, tier_blocks_batch *out);

/* Mini-batches one call can take with this context's scratch memory (1..TIER_MAX_BATCHES). */
int tier_max_batches(const tier_ctx *ctx);

/* Layout of the sampler's scratch (tuning and testing; results never depend on it).
 * words = 1, the default up to 32 M nodes: the nodes first reached at a hop are marked in a
 * bitmap over all nodes, one flag byte per 32-bit word of it tells the kernels that list
 * them where to look, and tier_presample keeps its frontiers in bitmaps (0.4 bytes of
 * scratch per node and mini-batch slot).  words = 32, the default above: the new nodes of
 * a hop are sorted into buckets of consecutive ids instead, and tier_presample keeps its
 * frontiers in the sampler's index (0.26 bytes per node and slot).  Waits for the
 * context's stream; TIER_EINVAL for any other value. */
int tier_set_segment_words(tier_ctx *ctx, int32_t words);

/* Tiered gather (Sec. 4.1, Listing 1).  out[i, :] = feature row of ids[i], read from
 * the HBM cache when slot[ids[i]] >= 0 and from host memory otherwise; the result
 * does not depend on the placement.  ids: (device) n ids, repeats allowed.
 * out: (device) n * row_bytes bytes, 16-byte aligned.  stats (host, optional): row
 * counts per tier; asking for them makes the call wait, otherwise asynchronous.
 * Ids inside [0, n_nodes) are a precondition that only a call with stats checks: such
 * a call returns TIER_EINVAL when one of its own ids is outside (stats then unset); a
 * call without stats returns TIER_OK.  Either way the row of such an id is all zero
 * bytes and no memory outside the tables is touched. */
int tier_gather_features(tier_ctx *ctx, const int32_t *ids, int64_t n, void *out,
                         tier_gather_stats *stats);

/* The gathers of several mini-batches in one launch (one mini-batch's rows are too few
 * to keep the host link and the GPU busy across a launch boundary).  Mini-batch b reads the
 * ids nodes[b * nodes_stride .. + n_rows[b]) (the layout of tier_blocks_batch) and writes
 * its rows from row out_row_offset[b] of out on, n_rows[b] dense rows (the caller packs
 * the mini-batches, e.g. at the running sum of n_rows).  nodes: (device); n_rows,
 * out_row_offset: (host) n_batches entries; 1 <= n_batches <= TIER_MAX_BATCHES; out:
 * (device) 16-byte aligned.  stats as in tier_gather_features, summed over the launch. */
int tier_gather_minibatches(tier_ctx *ctx, const int32_t *nodes, int64_t nodes_stride, const int64_t *n_rows,
                            const int64_t *out_row_offset, int32_t n_batches, void *out,
                            tier_gather_stats *stats);

/* Split gather (Sec. 4.1: the cold tier is read in place over the host link, whose
 * bandwidth the requests of a few dozen blocks already fill).  With link_blocks > 0, in a
 * gather call of at least min_rows rows in total the first link_blocks blocks of the
 * launch look through the requests and copy the cold rows, staying until the link has
 * delivered them; every other block copies hot rows only and leaves at HBM speed.  Same
 * results as the uniform launch (link_blocks = 0, the default), in which every block waits
 * on host reads and the kernels of other streams wait for the whole launch: use it when
 * something else (sampling, training) should run beside the gather.  0 <= link_blocks <=
 * 65536, min_rows >= 0.  Waits for the gather stream. */
int tier_set_gather_split(tier_ctx *ctx, int32_t link_blocks, int64_t min_rows);

/* Shared misses.  With on != 0 every gather call reads each distinct cold row among all
 * its requests over the host link once: the cold workers of the split launch (which this
 * option implies for every call with cold rows; link_blocks as set by
 * tier_set_gather_split, else 64) claim a cold id in a table over all nodes before they
 * fetch it, the requests that find it claimed are served by a second, short kernel that
 * copies the row inside HBM from the output row of the request that fetched it.  (A call
 * that asks for at least twice as many rows as the graph has nodes, of at most 4096 bytes
 * each, is served another way: a first kernel threads the cold requests of every id into
 * a list, and the worker that fetches a row writes it to every request on its list; no
 * second kernel.)  Results are the same; it pays when the mini-batches of one
 * tier_gather_minibatches call overlap in their cold rows and costs one atomic per cold
 * request and that second kernel otherwise.  Scratch owned by the context: 8 n_nodes
 * bytes for the claims (allocated here) and 16 bytes per request of the largest call.
 * Off by default.  Waits for the gather stream. */
int tier_set_gather_dedup(tier_ctx *ctx, int on);

/* Put the gathers of this context on a stream of their own (NULL = back to the stream of
 * tier_create), so that a caller can sample the next mini-batches while the current ones
 * are gathered (sampling is bound by launch and memory latency, the gather by the host
 * link; they overlap well).  The gather reads only ids, the slot map and the two tiers,
 * all of which sampling leaves alone; ordering between the two streams (ids complete
 * before the gather, gather complete before the ids are overwritten) is the caller's,
 * and tier_place / tier_place_boundary must not run while gathers are in flight. */
int tier_set_gather_stream(tier_ctx *ctx, void *stream);

const char *tier_strerror(int status);
/* hipError_t value of the last failing HIP call seen by this context (0 if none). */
int tier_last_hip_error(const tier_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* TIER_H */
