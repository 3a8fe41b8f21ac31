// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "tier.h"

// Slots of the device-side bookkeeping array (int64 each).  Kernels read the
// sizes of the current mini-batch from here, so a chain of launches needs no
// host round trip.
enum {
    META_NFRONT = 0,                          // [0 .. TIER_MAX_LAYERS]   |frontier_l|
    META_NEDGES = TIER_MAX_LAYERS + 1,        // [.. + TIER_MAX_LAYERS)   edges of block l
    META_TOTAL_ROWS = META_NEDGES + TIER_MAX_LAYERS,
    META_TOTAL_EDGES,
    META_ERROR,                               // != 0: a kernel saw an id outside [0, n_nodes)
    META_COLD_NEXT,                           // split gather: next chunk of requests for the cold workers,
    META_COLD_DONE,                           //   workers' waves that ran dry; both zero between launches
    META_DEFER_N,                             // shared misses: deferred entries reserved by the cold workers,
    META_DEFER_DONE,                          //   blocks of the copy kernel that are through; both zero between calls
    META_LINK_ROWS,                           //   rows they read over the host link (counted on request)
    META_HIT_ROWS,                            // first of META_HIT_STRIPES counters (gather bookkeeping only)
    META_WORDS
};
#define META_HIT_STRIPES 64                   // hit counters are striped over blocks to keep the atomics apart
#define GMETA_WORDS (META_WORDS + META_HIT_STRIPES)

#define TIER_SCAN_BLOCKS 1024                 // upper limit of blocks in a two-phase scan

// Scratch of the placement sort, kept by the context between calls.  `vals` of the last
// sort holds the order (rank -> node) that the cache fill reads on the gather stream.
struct tier_sort_bufs {
    void *keys[2];
    size_t keys_cap[2];          // bytes
    int32_t *vals[2];
    size_t vals_cap[2];
    uint32_t *hist;
    size_t hist_cap;
    uint32_t *partial;           // 1024 words
    unsigned long long *mask;    // one word
};

struct tier_ctx {
    hipStream_t stream;
    hipStream_t gather_stream;   // stream of tier_gather_features (= stream unless set apart)
    int64_t *gmeta;              // device: error flag and hit counter of the gather stream
    int64_t *gmeta_host;         // pinned mirror
    // shared misses (tier_set_gather_dedup): state of the gather stream
    bool dedup;
    bool maps_in_use;            // a gather enqueued since the library last waited for the gather stream may still read
                                 //   the slot map, the hot bits or the cache
    bool last_deduped;           // the last gather call ran with claims (its link rows are in META_LINK_ROWS)
    unsigned long long *claim;   // n_nodes; stamp << 40 | output row of the request that fetches the id in that call
    uint32_t claim_stamp;        // stamp of the last call that claimed (24 bits, then the table is cleared)
    int64_t *deferred;           // pairs (output row, output row to copy from) left by the cold workers
    size_t deferred_cap;         // bytes
    // split gather (tier_set_gather_split): the cold rows of a call go to a few blocks of the launch
    int link_blocks;             // how many; 0 = every block copies hot and cold rows alike
    int64_t split_min_rows;      // calls with fewer rows keep the uniform launch
    int device;
    int last_hip;
    // graph and features (referenced, caller-owned)
    int64_t n_nodes, n_edges;
    const void *indptr;
    bool indptr_i64;
    const int32_t *indices;
    const uint8_t *host_rows;
    bool rows_on_host;       // the table is host memory read over the link (not a device allocation)
    int64_t row_bytes;
    // sampler scratch over all nodes, one copy per slot (mini-batch sampled side by side); all of it
    // is zero between mini-batches
    int n_slots;
    uint32_t *fresh;         // [n_slots][bm_stride]; bits of the nodes first reached at the current hop
    uint32_t *aux;           // [n_slots][bm_stride]; access counting only: the frontier so far
    uint8_t *flag;           // [n_slots][flag_stride]; bitmap layout: != 0: the bitmap word holds a bit of `fresh`
    int32_t *segbase;        // [n_slots][n_seg]; bitmap layout: start position of a word's new nodes (last hop of a block call)
    int64_t n_words;         // ceil(n_nodes / 32)
    int64_t bm_stride;       // bitmap words per slot: n_words rounded up to whole 128-byte lines
    int seg_log2;            // 0: bitmap layout (up to 32 M nodes), a flag and a start position per bitmap word; 5: bucket
                             // layout (above), where the sampler lists new nodes by sorting and leaves `fresh`, `flag`
                             // and `segbase` alone (flags and positions are then sized per 32 words)
    int64_t n_seg;           // flags per slot: n_words >> seg_log2, rounded up
    int64_t flag_stride;     // n_seg rounded up to a multiple of 16
    int64_t *f_beg;          // [n_slots][nodes that draw in the current call]: indptr[node] beside the frontier
    size_t f_beg_cap;        // bytes
    int32_t *f_deg;          // likewise: degrees
    size_t f_deg_cap;
    uint32_t *table;         // frontier index of the sampler, [n_slots][cells of the current call]; grown on demand
    size_t table_cap;        // bytes
    // last hop of a block call on the large-graph layout: its new neighbours are sorted into buckets of
    // consecutive node ids instead of marked in `fresh` (sampler.hip); all grown on demand
    unsigned long long *part_rec;   // [slots of the call][edges of the last hop]: node << 32 | edge
    size_t part_rec_cap;            // bytes
    int32_t *part_rank;             // likewise: rank of the record's node among its bucket's distinct nodes
    size_t part_rank_cap;
    int32_t *part_stage;            // likewise: every bucket's distinct nodes, ascending, at the bucket's start
    size_t part_stage_cap;
    int32_t *part_rows;             // [slots][blocks that scatter][buckets]: records of a block per bucket
    size_t part_rows_cap;
    int32_t *part_bk;               // [slots][3][buckets + 1]: start, distinct nodes, distinct nodes before, per bucket
    size_t part_bk_cap;
    // placement
    int32_t *slot;           // n_nodes
    uint32_t *hot_bits;      // ceil(n_nodes / 32): bit v set <=> slot[v] >= 0 (what the split gather's cold workers ask)
    uint8_t *cache;          // n_hot * row_bytes
    size_t cache_cap;        // bytes allocated (kept across placements, grown on demand)
    tier_sort_bufs sort;
    hipEvent_t ev_place;     // orders the cache fill (gather stream) after the slot map (main stream)
    bool fill_pending;       // a cache fill may still be reading sort.vals on the gather stream
    int64_t n_hot;
    // rows fetched ahead of a placement (tier_prefetch): the next cache fill takes them from `staging`
    int64_t staged_rows;     // 0: nothing staged
    int32_t *staged_ids;     // staged_rows node ids, in the order of the ranking they were chosen by
    size_t staged_ids_cap;   // bytes
    uint8_t *staging;        // staged_rows x row_bytes: row i = feature row of staged_ids[i]
    size_t staging_cap;
    int32_t *staged_of;      // n_nodes: position in `staging`, or -1
    size_t staged_of_cap;
    uint32_t *staged_bits;   // ceil(n_nodes / 32): bit v set <=> staged_of[v] >= 0
    size_t staged_bits_cap;
    void *select;            // device scratch of tier_prefetch's search for the rows to stage
    size_t select_cap;
    bool placed;
    bool boundary;           // true: rows are in rank order, hot <=> id < n_hot (no slot map)
    // sampler scratch
    int64_t *meta;           // device, [n_slots][META_WORDS]; slot 0 also holds totals, error flag, hit counter
    int64_t *meta_host;      // pinned mirror
    int32_t *partial_hop;    // [n_slots][TIER_SCAN_BLOCKS]
    int32_t *partial_bm;     // [n_slots][TIER_SCAN_BLOCKS]
    int32_t *ps_nodes;       // frontier buffers used by tier_presample
    int64_t cap_ps_nodes;
    int32_t *ps_col;         // tier_presample on the large-graph layout: per dst node and draw, ~node of a new node or 0
    size_t ps_col_cap;       // bytes
    // scratch of the score functions and of the graph reordering, kept between calls
    double *pulled;          // n_nodes sums of one round of tier_score_wrpr
    size_t pulled_cap;       // bytes
    int64_t *scan_partial;   // TIER_SCAN_BLOCKS block sums of the offsets' prefix sum (tier_reorder_graph)
    size_t scan_partial_cap;
};

#define TIER_HIP(ctx, call)                                              \
    do {                                                                 \
        hipError_t e_ = (call);                                          \
        if (e_ != hipSuccess) {                                          \
            if (ctx) (ctx)->last_hip = (int)e_;                          \
            (void)hipGetLastError();                                     \
            return e_ == hipErrorOutOfMemory ? TIER_ENOMEM : TIER_EHIP;  \
        }                                                                \
    } while (0)

// gather.hip: row copy used by tier_gather_features and by the cache fill of tier_place.
// mode 0: every row from host_rows; 1: through the slot map; 2: by the boundary n_hot.
// link_blocks_cap > 0 (mode 0, table in host memory): fewer blocks than the launch would take by itself.
enum { GATHER_HOST = 0, GATHER_SLOT = 1, GATHER_BOUNDARY = 2 };
int tier_launch_gather(tier_ctx *ctx, const int32_t *ids, int64_t n, int mode, void *out, bool count_hits,
                       int link_blocks_cap = 0);
// gather.hip: the cache fill when rows are staged: out row i = feature row of ids[i], from `staging`
// where staged_of[ids[i]] >= 0 and from host_rows otherwise (a split launch on the gather stream).
int tier_launch_fill_staged(tier_ctx *ctx, const int32_t *ids, int64_t n, void *out);

// context.hip: make *buf at least `bytes` long (contents are not kept).  Growing waits for both streams.
int tier_ensure(tier_ctx *ctx, void **buf, size_t *cap, size_t bytes);

// context.hip: copy the bookkeeping array into ctx->meta_host and wait for the
// stream.  Returns TIER_EINVAL once (and clears the flag) when a kernel met an id
// outside [0, n_nodes).
int tier_sync_meta(tier_ctx *ctx);
