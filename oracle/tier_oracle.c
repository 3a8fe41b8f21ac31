/*
 * tier_oracle.c -- CPU oracle for the data-tiering hot path (test infrastructure).
 *
 * This file is TEST INFRASTRUCTURE, not the product: it is a plain, slow,
 * single-threaded C implementation of what the GPU library computes, written
 * from the paper's statement of the method so that the two can be compared
 * bit for bit.  It shares no code, header, table or helper with the HIP path
 * and must never be called from it.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.
 *
 * What the paper fixes, and where:
 *   - neighbour sampling: a fixed number of neighbours per target node per
 *     layer, chosen uniformly at random, resampled every iteration, followed by
 *     a sub-graph of the sampled nodes (Sec. 2.2 "Neighbor Sampling");
 *   - only labelled (training) nodes start a sample (Sec. 3.1);
 *   - the access frequency of a node is how often its feature row is read
 *     during mini-batch training (Sec. 3.1, Sec. 5.2);
 *   - nodes are ordered by descending score, the map runs old id -> rank
 *     (worked example in Sec. 3.2), the top part goes to GPU memory and the
 *     rest stays in host memory (Sec. 4.1);
 *   - a row read picks the GPU pointer when the row is inside the hot part
 *     and the host pointer otherwise, and copies the row (Sec. 4.1, Listing 1
 *     with zero peer GPUs).
 * What the paper leaves open (random generator, with/without replacement,
 * ordering of the sub-graph, tie-break, byte->row rounding) is fixed here by
 * the readings listed at each function.
 *
 * Pins (tests, CPU only): Philox known-answer vectors; Floyd subsets checked
 * by chi-square against the uniform law and by brute-force enumeration;
 * full-fanout sampling equals a separately written BFS; counts sum to the
 * frontier sizes and match a closed-form expectation; placement equals a
 * stable library sort and the paper's worked example; gather equals library
 * fancy indexing.  No function here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Random numbers.  The paper names no generator.  Reading: Philox4x32 with   */
/* 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11), the published counter-based */
/* generator; any draw is addressed directly by (seed, node, draw, layer).    */
/* ------------------------------------------------------------------------ */

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 64 random bits for one addressed draw: words 0 and 1 of the Philox block
 * with counter (a, b, c, tag) and key = the two halves of the 64-bit seed. */
static uint64_t random64(uint64_t seed, uint32_t a, uint32_t b, uint32_t c, uint32_t tag)
{
    uint32_t ctr[4] = { a, b, c, tag };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    return ((uint64_t)w[1] << 32) | (uint64_t)w[0];
}

enum { TAG_NEIGHBOUR = 1, TAG_BATCH = 2 };

/* Uniform integer in [0, m): high half of the 128-bit product r * m.
 * No rejection step; the bias is at most m / 2^64. */
uint64_t orc_bounded(uint64_t r, uint64_t m)
{
    return (uint64_t)(((unsigned __int128)r * (unsigned __int128)m) >> 64);
}

/* Seed of mini-batch b of epoch e, derived from the run's seed. */
uint64_t orc_batch_seed(uint64_t seed, uint32_t epoch, uint32_t batch)
{
    return random64(seed, epoch, batch, 0u, TAG_BATCH);
}

/* ------------------------------------------------------------------------ */
/* One node's draw (Sec. 2.2: a fixed number of neighbours, uniformly).       */
/* Reading: without replacement; a node of degree d <= k keeps all d          */
/* neighbours in adjacency order and uses no random numbers; otherwise a      */
/* uniformly random k-subset of the d positions by Floyd's subset algorithm   */
/* (Bentley & Floyd, CACM 1987), emitted in draw order.                       */
/* Returns the number of positions written to pos[] (min(k, d)).              */
/* ------------------------------------------------------------------------ */
int orc_draw_positions(uint64_t seed, uint32_t layer, uint32_t node,
                       int64_t d, int k, int64_t *pos)
{
    if (d <= (int64_t)k) {
        for (int64_t i = 0; i < d; ++i) pos[i] = i;
        return (int)d;
    }
    for (int i = 0; i < k; ++i) {
        int64_t j = d - k + i;
        int64_t t = (int64_t)orc_bounded(random64(seed, node, (uint32_t)i, layer, TAG_NEIGHBOUR),
                                         (uint64_t)j + 1u);
        int seen = 0;
        for (int q = 0; q < i; ++q)
            if (pos[q] == t) seen = 1;
        pos[i] = seen ? j : t;
    }
    return k;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* ------------------------------------------------------------------------ */
/* One mini-batch (Sec. 2.2): L hops outward from the seeds, then the         */
/* sub-graph of the sampled nodes as one block per hop.                       */
/*                                                                            */
/* frontier_0 = seeds in the given order.  At hop l every node of frontier_l  */
/* (seeds and nodes reached earlier alike) draws with fanouts[l] and layer    */
/* index l from its adjacency list indices[indptr[v] .. indptr[v+1]).         */
/* frontier_{l+1} = frontier_l followed by the newly reached nodes in         */
/* ascending id order.  Block l has dst = frontier_l, src = frontier_{l+1};   */
/* row_ptr is the running sum of per-dst edge counts in dst order, col the    */
/* position of each sampled neighbour in frontier_{l+1}, eid its position in  */
/* indices[].                                                                 */
/*                                                                            */
/* Storage: nodes[] receives frontier_L (frontier_l is its first n_nodes[l]   */
/* entries).  row_ptr_all, col_all and eid_all hold the layers back to back:  */
/* layer l's row_ptr starts at sum_{m<l} (n_nodes[m] + 1), its col/eid at     */
/* sum_{m<l} n_edges[m].  Any of the three may be NULL (not wanted).          */
/* local_idx: N entries, all -1 on entry; all -1 again on return.             */
/* Returns 0, or -1 when a capacity is too small (outputs then undefined,     */
/* local_idx still restored).                                                 */
/* ------------------------------------------------------------------------ */
int orc_sample_minibatch(int64_t n_nodes_graph, const int64_t *indptr, const int32_t *indices,
                         const int32_t *seeds, int64_t n_seeds,
                         const int32_t *fanouts, int n_layers, uint64_t seed,
                         int32_t *local_idx,
                         int32_t *nodes, int64_t cap_nodes,
                         int32_t *row_ptr_all, int64_t cap_row_ptr,
                         int32_t *col_all, int64_t *eid_all, int64_t cap_edges,
                         int64_t *n_nodes /* n_layers+1 */, int64_t *n_edges /* n_layers */)
{
    (void)n_nodes_graph;
    int rc = 0;
    int64_t n_front = 0;
    int64_t rp_base = 0, e_base = 0;
    int64_t pos[64];

    if (n_seeds > cap_nodes) return -1;
    for (int64_t i = 0; i < n_seeds; ++i) {
        nodes[i] = seeds[i];
        local_idx[seeds[i]] = (int32_t)i;
    }
    n_front = n_seeds;
    n_nodes[0] = n_front;

    for (int l = 0; l < n_layers && rc == 0; ++l) {
        int k = fanouts[l];
        int64_t n_dst = n_front;
        int64_t n_e = 0;
        int64_t n_new = 0;           /* candidates appended after nodes[n_front) */
        if (row_ptr_all && rp_base + n_dst + 1 > cap_row_ptr) { rc = -1; break; }

        for (int64_t i = 0; i < n_dst && rc == 0; ++i) {
            int32_t v = nodes[i];
            int64_t beg = indptr[v], d = indptr[v + 1] - beg;
            if (row_ptr_all) row_ptr_all[rp_base + i] = (int32_t)n_e;
            int cnt = orc_draw_positions(seed, (uint32_t)l, (uint32_t)v, d, k, pos);
            if (e_base + n_e + cnt > cap_edges) { rc = -1; break; }
            for (int q = 0; q < cnt; ++q) {
                int64_t e = beg + pos[q];
                int32_t u = indices[e];
                if (eid_all) eid_all[e_base + n_e] = e;
                /* col is filled after the new nodes are ordered; keep u for now */
                if (col_all) col_all[e_base + n_e] = u;
                if (local_idx[u] == -1) {            /* first time reached */
                    if (n_front + n_new >= cap_nodes) { rc = -1; break; }
                    local_idx[u] = -2;               /* reached at this hop */
                    nodes[n_front + n_new] = u;
                    ++n_new;
                }
                ++n_e;
            }
        }
        if (rc == 0) {
            if (row_ptr_all) row_ptr_all[rp_base + n_dst] = (int32_t)n_e;
            qsort(nodes + n_front, (size_t)n_new, sizeof(int32_t), cmp_i32);
        }
        /* give the new nodes their places (also on failure, so that the
         * clean-up below finds every touched entry through nodes[]) */
        for (int64_t j = 0; j < n_new; ++j)
            local_idx[nodes[n_front + j]] = (int32_t)(n_front + j);
        if (rc == 0 && col_all)
            for (int64_t e = 0; e < n_e; ++e)
                col_all[e_base + e] = local_idx[col_all[e_base + e]];
        n_front += n_new;
        if (rc == 0) {
            n_nodes[l + 1] = n_front;
            n_edges[l] = n_e;
            rp_base += n_dst + 1;
            e_base += n_e;
        }
    }
    for (int64_t i = 0; i < n_front; ++i) local_idx[nodes[i]] = -1;
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Access counts (Sec. 3.1, Sec. 5.2: measured access frequency of each node  */
/* during mini-batch training).  Reading: one access per node per mini-batch  */
/* whose sampled sub-graph contains it -- exactly the rows a feature gather   */
/* for that mini-batch reads.  Mini-batches are consecutive chunks of         */
/* train_ids in the caller's order; batch b of epoch e samples with           */
/* orc_batch_seed(seed, e, b).  counts[] is overwritten.  Batches             */
/* [batch_begin, batch_end) of every epoch are processed, so that a caller    */
/* may split the work; the full job is batch_begin = 0, batch_end = number    */
/* of batches.  nodes_scratch: room for the largest frontier.                 */
/* total_out (optional): sum over processed batches of the frontier size.     */
/* ------------------------------------------------------------------------ */
int orc_presample(int64_t n_nodes_graph, const int64_t *indptr, const int32_t *indices,
                  const int32_t *train_ids, int64_t n_train, int64_t batch_size,
                  const int32_t *fanouts, int n_layers, int epochs, uint64_t seed,
                  int64_t batch_begin, int64_t batch_end,
                  int32_t *local_idx, int32_t *nodes_scratch, int64_t cap_nodes,
                  uint32_t *counts, int64_t *total_out, int64_t *edges_out)
{
    int64_t n_batches = (n_train + batch_size - 1) / batch_size;
    int64_t nn[16], ne[16];
    int64_t total = 0, edges = 0;
    if (batch_end > n_batches) batch_end = n_batches;
    memset(counts, 0, (size_t)n_nodes_graph * sizeof(uint32_t));
    for (int e = 0; e < epochs; ++e) {
        for (int64_t b = batch_begin; b < batch_end; ++b) {
            int64_t lo = b * batch_size;
            int64_t n = n_train - lo < batch_size ? n_train - lo : batch_size;
            int rc = orc_sample_minibatch(n_nodes_graph, indptr, indices, train_ids + lo, n,
                                          fanouts, n_layers,
                                          orc_batch_seed(seed, (uint32_t)e, (uint32_t)b),
                                          local_idx, nodes_scratch, cap_nodes,
                                          NULL, 0, NULL, NULL, INT64_MAX, nn, ne);
            if (rc) return rc;
            for (int64_t i = 0; i < nn[n_layers]; ++i) counts[nodes_scratch[i]] += 1u;
            total += nn[n_layers];
            for (int l = 0; l < n_layers; ++l) edges += ne[l];
        }
    }
    if (total_out) *total_out = total;
    if (edges_out) *edges_out = edges;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Access counts, the other reading of "number of samples" (Sec. 3.1): every  */
/* time a node is drawn as a neighbour counts, and so does every seed, i.e.   */
/* counts[v] = occurrences of v among the seeds and among the source ends of  */
/* all sampled edges, over the same mini-batches as orc_presample.  The sum   */
/* of counts is the number of seeds plus the number of sampled edges.         */
/* eid_scratch: room for the edges of one mini-batch.                         */
/* ------------------------------------------------------------------------ */
int orc_presample_draws(int64_t n_nodes_graph, const int64_t *indptr, const int32_t *indices,
                        const int32_t *train_ids, int64_t n_train, int64_t batch_size,
                        const int32_t *fanouts, int n_layers, int epochs, uint64_t seed,
                        int64_t batch_begin, int64_t batch_end,
                        int32_t *local_idx, int32_t *nodes_scratch, int64_t cap_nodes,
                        int64_t *eid_scratch, int64_t cap_edges,
                        uint32_t *counts, int64_t *draws_out)
{
    int64_t n_batches = (n_train + batch_size - 1) / batch_size;
    int64_t nn[16], ne[16];
    int64_t draws = 0;
    if (batch_end > n_batches) batch_end = n_batches;
    memset(counts, 0, (size_t)n_nodes_graph * sizeof(uint32_t));
    for (int e = 0; e < epochs; ++e) {
        for (int64_t b = batch_begin; b < batch_end; ++b) {
            int64_t lo = b * batch_size;
            int64_t n = n_train - lo < batch_size ? n_train - lo : batch_size;
            int rc = orc_sample_minibatch(n_nodes_graph, indptr, indices, train_ids + lo, n,
                                          fanouts, n_layers,
                                          orc_batch_seed(seed, (uint32_t)e, (uint32_t)b),
                                          local_idx, nodes_scratch, cap_nodes,
                                          NULL, 0, NULL, eid_scratch, cap_edges, nn, ne);
            if (rc) return rc;
            int64_t n_e = 0;
            for (int l = 0; l < n_layers; ++l) n_e += ne[l];
            for (int64_t i = 0; i < n; ++i) counts[train_ids[lo + i]] += 1u;
            for (int64_t i = 0; i < n_e; ++i) counts[indices[eid_scratch[i]]] += 1u;
            draws += n + n_e;
        }
    }
    if (draws_out) *draws_out = draws;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Placement (Sec. 3.2, Sec. 4.1): order the nodes by descending score, map   */
/* old id -> rank, keep the top part in GPU memory.  The score is the access  */
/* count.  Readings: equal counts are ordered by ascending id; the budget in  */
/* bytes admits floor(budget / row_bytes) rows, at most N; rows with count 0  */
/* may be placed.  rank[] and slot[] are both old id -> position; slot is -1  */
/* for rows left in host memory.                                              */
/* ------------------------------------------------------------------------ */
typedef struct { uint32_t count; int32_t id; } scored;

static int cmp_scored(const void *a, const void *b)
{
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->count != y->count) return x->count > y->count ? -1 : 1;   /* descending */
    return (x->id > y->id) - (x->id < y->id);                        /* ascending  */
}

int orc_place(const uint32_t *counts, int64_t n, int64_t row_bytes, uint64_t budget_bytes,
              int32_t *rank, int32_t *slot, int64_t *n_hot_out)
{
    scored *s = (scored *)malloc((size_t)(n > 0 ? n : 1) * sizeof(scored));
    if (!s) return -1;
    for (int64_t v = 0; v < n; ++v) { s[v].count = counts[v]; s[v].id = (int32_t)v; }
    qsort(s, (size_t)n, sizeof(scored), cmp_scored);
    int64_t n_hot = (int64_t)(budget_bytes / (uint64_t)row_bytes);
    if (n_hot > n) n_hot = n;
    for (int64_t r = 0; r < n; ++r) {
        int32_t v = s[r].id;
        if (rank) rank[v] = (int32_t)r;
        slot[v] = r < n_hot ? (int32_t)r : -1;
    }
    free(s);
    *n_hot_out = n_hot;
    return 0;
}

/* cache[slot[v]] = feat[v] for every placed row. */
void orc_fill_cache(const uint8_t *feat, int64_t n, int64_t row_bytes,
                    const int32_t *slot, uint8_t *cache)
{
    for (int64_t v = 0; v < n; ++v)
        if (slot[v] >= 0)
            memcpy(cache + (size_t)slot[v] * (size_t)row_bytes,
                   feat + (size_t)v * (size_t)row_bytes, (size_t)row_bytes);
}

/* ------------------------------------------------------------------------ */
/* Tiered gather (Sec. 4.1; Listing 1 with no peer GPUs): a row inside the    */
/* hot part is read from the GPU-resident copy, any other from host memory.   */
/* ------------------------------------------------------------------------ */
void orc_gather(const uint8_t *feat, const uint8_t *cache, const int32_t *slot,
                int64_t row_bytes, const int32_t *ids, int64_t n, uint8_t *out,
                int64_t *hit_rows, int64_t *miss_rows)
{
    int64_t hit = 0;
    for (int64_t i = 0; i < n; ++i) {
        int32_t v = ids[i];
        const uint8_t *row;
        if (slot[v] >= 0) { row = cache + (size_t)slot[v] * (size_t)row_bytes; ++hit; }
        else              { row = feat  + (size_t)v       * (size_t)row_bytes; }
        memcpy(out + (size_t)i * (size_t)row_bytes, row, (size_t)row_bytes);
    }
    if (hit_rows)  *hit_rows = hit;
    if (miss_rows) *miss_rows = n - hit;
}

/* ------------------------------------------------------------------------ */
/* Graph and feature reordering (Sec. 3.2, Alg. 2): every node takes its     */
/* rank as its new id.  The result has a plain definition, written out here:  */
/* new node r owns the neighbour list of the node whose rank is r, entries in */
/* their old order, every entry replaced by its own rank; offsets_new is the  */
/* running sum of those list lengths.  (Alg. 2 reaches the same arrays by a   */
/* scatter of lengths, a prefix sum and a relocation, so that every step is   */
/* parallel; the GPU path does it that way.)                                  */
/* Reading: Alg. 2's last loop, as printed, addresses the new offsets with    */
/* the old id; its accompanying text places a list at the offset of the       */
/* node's new id, which is also the only reading consistent with the first    */
/* loop, and is what the definition above says.                               */
/* ------------------------------------------------------------------------ */
void orc_reorder_graph(int64_t n, const int64_t *indptr, const int32_t *indices, const int32_t *rank,
                       int64_t *indptr_new, int32_t *indices_new)
{
    int32_t *who = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));   /* who[r] = node of rank r */
    for (int64_t i = 0; i < n; ++i) who[rank[i]] = (int32_t)i;
    indptr_new[0] = 0;
    for (int64_t r = 0; r < n; ++r) {
        const int64_t i = who[r];
        const int64_t len = indptr[i + 1] - indptr[i];
        indptr_new[r + 1] = indptr_new[r] + len;
        for (int64_t j = 0; j < len; ++j)
            indices_new[indptr_new[r] + j] = rank[indices[indptr[i] + j]];
    }
    free(who);
}

/* Feature rows follow their nodes (Sec. 3.2: the table is reordered by score). */
void orc_reorder_rows(const uint8_t *feat, int64_t n, int64_t row_bytes, const int32_t *rank,
                      uint8_t *feat_new)
{
    for (int64_t i = 0; i < n; ++i)
        memcpy(feat_new + (size_t)rank[i] * (size_t)row_bytes, feat + (size_t)i * (size_t)row_bytes,
               (size_t)row_bytes);
}

/* Tiered gather on reordered data (Sec. 4.1; Listing 1 with no peer GPUs): ids below */
/* the boundary index the hot tensor, the others index the cold tensor by their       */
/* offset from the boundary.                                                          */
void orc_gather_boundary(const uint8_t *hot, const uint8_t *cold, int64_t boundary, int64_t row_bytes,
                         const int32_t *ids, int64_t n, uint8_t *out, int64_t *hit_rows)
{
    int64_t hit = 0;
    for (int64_t i = 0; i < n; ++i) {
        const uint8_t *row;
        if (ids[i] < boundary) { row = hot + (size_t)ids[i] * (size_t)row_bytes; ++hit; }
        else                   { row = cold + (size_t)(ids[i] - boundary) * (size_t)row_bytes; }
        memcpy(out + (size_t)i * (size_t)row_bytes, row, (size_t)row_bytes);
    }
    if (hit_rows) *hit_rows = hit;
}

/* ------------------------------------------------------------------------ */
/* The paper's own score functions (Sec. 3.1), alternatives to the measured  */
/* access count.  Edges run source -> target; row v of the CSR lists the     */
/* sources of the edges into v, so in_degree(v) is the length of row v and   */
/* out_degree(u) the number of rows that contain u.                          */
/* ------------------------------------------------------------------------ */

/* Score 1: the out degree of each node. */
void orc_score_degree(int64_t n, const int64_t *indptr, const int32_t *indices, uint32_t *degree)
{
    memset(degree, 0, (size_t)n * sizeof(uint32_t));
    for (int64_t e = 0; e < indptr[n]; ++e) degree[indices[e]] += 1u;
}

/* Score 3: weighted reverse PageRank (Sec. 3.1, Alg. 1), an iteration, so its rounds  */
/* are taken as the paper orders them.  Start: every node 1/N, a training node N/n_train */
/* times that.  One round: each node v splits its score evenly over its incoming edges   */
/* (share[v] = score[v] / in_degree(v)); each node u collects the shares of the nodes it */
/* points to; score[u] = (1 - damp)/N + damp * collected[u].  Without training ids the   */
/* start is uniform and this is plain reverse PageRank (score 2) cut after `iterations`  */
/* rounds.  Readings: a node nobody points to keeps its score undivided (no node         */
/* collects from it); what a node collects replaces its score (a node that points        */
/* nowhere collects 0); sums run over the rows in order and over each row in list order. */
void orc_score_wrpr(int64_t n, const int64_t *indptr, const int32_t *indices,
                    const int32_t *train_ids, int64_t n_train, int iterations, double damp, double *score)
{
    double *share = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    double *collected = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    for (int64_t v = 0; v < n; ++v) score[v] = 1.0 / (double)n;
    if (n_train > 0) {
        const double boost = (double)n / (double)n_train;
        for (int64_t t = 0; t < n_train; ++t) score[train_ids[t]] = score[train_ids[t]] * boost;
    }
    for (int round = 0; round < iterations; ++round) {
        for (int64_t v = 0; v < n; ++v) {
            const int64_t in_degree = indptr[v + 1] - indptr[v];     /* row v lists the sources of the edges into v */
            share[v] = in_degree > 0 ? score[v] / (double)in_degree : score[v];
            collected[v] = 0.0;
        }
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) collected[indices[e]] += share[v];   /* indices[e] points to v */
        for (int64_t u = 0; u < n; ++u) {
            const double floor_part = (1.0 - damp) / (double)n;
            const double pulled_part = damp * collected[u];
            score[u] = floor_part + pulled_part;
        }
    }
    free(share);
    free(collected);
}

/* Ranking by a real-valued score: descending score, equal scores by ascending id. */
typedef struct { double score; int32_t id; } rscored;

static int cmp_rscored(const void *a, const void *b)
{
    const rscored *x = (const rscored *)a, *y = (const rscored *)b;
    if (x->score != y->score) return x->score > y->score ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

int orc_rank_scores(const double *score, int64_t n, int32_t *rank)
{
    rscored *s = (rscored *)malloc((size_t)(n > 0 ? n : 1) * sizeof(rscored));
    if (!s) return -1;
    for (int64_t v = 0; v < n; ++v) { s[v].score = score[v]; s[v].id = (int32_t)v; }
    qsort(s, (size_t)n, sizeof(rscored), cmp_rscored);
    for (int64_t r = 0; r < n; ++r) rank[s[r].id] = (int32_t)r;
    free(s);
    return 0;
}
