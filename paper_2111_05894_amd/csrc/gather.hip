// Tiered feature gather (Sec. 4.1; Listing 1 without peer GPUs).
//
// For every requested id the row comes from the HBM cache when the node->slot
// map places it there, and from pinned host memory (read in place over the
// host link) otherwise.  A group of LPR lanes copies one row in 16-byte pieces,
// so a row is read and written with full-width coalesced accesses; several rows
// per group are in flight to cover the host link's latency.
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
//
// Shared misses (tier_set_gather_dedup): the mini-batches gathered by one call overlap
// (on a low-skew 10 M-node graph two thirds of a call's cold rows are requested more
// than once).  The cold workers then claim every cold id in a table over all nodes
// before they fetch it: the first request of an id in the call wins and reads the row
// over the host link, every later one only notes "my row = that request's row", and a
// short second kernel copies those rows inside HBM (k_copy_deferred).  A claim is the
// call's stamp and the winner's output row in one 64-bit word, so the table needs no
// clearing between calls.
//
// Shared misses with most requests repeating an id (a call that asks for at least twice as
// many rows as the graph has nodes): the copies afterwards would move most of the call's
// bytes through HBM a second time, behind the host link's back.  Instead a first kernel
// (k_link) threads the cold requests of every id into a list (claim = the last request to
// arrive, every request remembers the one before it and its own output row), and the cold
// workers fetch a row where they meet the head of its list and write it to every request on
// the list straight from their registers: no second kernel, no row read back from HBM.
#include "tier_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowsInFlight = 4;        // measured best of 2 / 4 / 8 on MI355X
constexpr int kLinkBlocks = 64;         // blocks of a launch that reads host rows only (best of 32 .. 512, full grid)
constexpr int kClaimRowBits = 40;       // claim = stamp << 40 | output row of the winning request
constexpr int kDeferBlock = 512;        // deferred copies are reserved up to 512 entries at a time
constexpr int kFanPieces = 4;           // lists of requests: a lane holds up to 4 pieces of 16 bytes of each row in flight
constexpr int kUnitsPerGrab = 8;        // a cold worker's wave takes up to 8 units of 64 requests off the counter at a time
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The id lists one launch serves (blockIdx.y picks one): a mini-batch each.
struct id_lists_t {
    const int32_t *ids[TIER_MAX_BATCHES];
    int64_t n[TIER_MAX_BATCHES];
    int64_t out_row[TIER_MAX_BATCHES];   // first output row of the list
    int64_t first_req[TIER_MAX_BATCHES]; // requests of the lists before it (number of a request = this + its place in the list)
};

// What the cold workers of a split launch need beyond the lists.
struct cold_t {
    int workers;                         // blocks of grid row 0 that copy cold rows
    unsigned long long stamp;            // shared misses: this call's stamp, already shifted; 0 = off
    unsigned long long *claim;           // [n_nodes]
    int64_t *deferred;                   // pairs (output row, output row to copy from); first < 0: unused
                                         // (lists of requests: pairs (request before this one or -1, output row), by request)
};

// An id outside the graph is nobody's cold row: the blocks that copy hot rows write its row of zeros.
// The cold workers only need to know whether a row is placed, not where: one bit per node
// (tier_place builds it beside the slot map) instead of the 4-byte slot, whose 128-byte line
// the hot blocks fetch anyway.  The bitmap is 1/32 of the map and mostly stays in cache.
template <int MODE>
__device__ inline int is_cold(int32_t id, const uint32_t *__restrict__ hot_bits, int64_t n_nodes, int64_t n_hot)
{
    if ((uint32_t)id >= (uint64_t)n_nodes) return 0;
    return MODE == GATHER_SLOT ? !((hot_bits[(uint32_t)id >> 5] >> (id & 31)) & 1u) : id >= n_hot;
}

// The cold workers of a split launch: the first `workers` blocks of grid row 0.  The
// requests are numbered in units of 64 (list by list); a wave takes the next unit off a
// counter, or in a large call the next few (atomics on one address run at ~26 M/s for the
// whole chip: one per unit would cost a 100 M-request call 60 ms; in a small call a wave that
// is left with several units at the end would keep the others waiting), which makes the waves
// finish together whatever the mix of hot and cold in their units, and appends each unit's
// cold requests (one ballot) to a small queue of its own in LDS.  Whenever the queue holds a full pass - kRowsInFlight rows for each group of
// LPR lanes - the wave copies one, so the bytes it keeps in flight on the host link do not
// depend on how many of the requests are cold.  Four stages run ahead of that, a unit
// each: the counter, the ids, the slot lookups and (shared misses) the claims, so the
// copies never wait for any of them.  The last wave to run dry leaves both counters at
// zero for the next launch on the stream.
// SHARE: 0 every cold request reads its row; 1 claims and deferred copies; 2 lists of requests.
template <int LPR, int MODE, int SHARE>
__device__ inline void scan_cold_rows(const id_lists_t &lists, int n_lists, const uint32_t *__restrict__ hot_bits,
                                      int64_t n_nodes, int64_t n_hot, const cold_t &cold,
                                      const uint4 *__restrict__ host, uint4 *__restrict__ out_base, int cpr,
                                      int64_t *__restrict__ meta, int count_rows)
{
    constexpr int kGroupsPerWave = 64 / LPR;
    constexpr int kPerPass = kGroupsPerWave * kRowsInFlight;
    constexpr int kQueue = 128;                       // ring: at most kPerPass - 1 + 64 entries wait
    __shared__ int32_t s_src[kBlock / 64][kQueue];    // host row of a waiting cold request
    __shared__ int64_t s_dst[kBlock / 64][kQueue];    // its output row
    if ((int)blockIdx.x >= cold.workers) return;
    const int lane64 = threadIdx.x & 63;
    const int g = lane64 / LPR, lane = lane64 % LPR;
    int32_t *q_src = s_src[threadIdx.x >> 6];
    int64_t *q_dst = s_dst[threadIdx.x >> 6];
    const unsigned long long n_waves = (unsigned long long)cold.workers * (kBlock / 64);
    unsigned long long *next = (unsigned long long *)&meta[META_COLD_NEXT];
    unsigned long long *done = (unsigned long long *)&meta[META_COLD_DONE];
    int64_t total = 0;
    for (int b = 0; b < n_lists; ++b) total += (lists.n[b] + 63) / 64;

    struct unit_t {
        int64_t q;        // number of the unit (wave-uniform)
        int64_t row0;     // output row of its first request (wave-uniform); SHARE == 2: number of its first request
        int32_t id;       // this lane's request, -1 beyond the list or the call
        int fetch;        // this lane's request is cold (after the claim stage: and is the one that reads the row)
    };
    // the counter's value arrives in lane 0; it is broadcast only where it is needed, an iteration
    // or more later, so that the atomic's latency hides behind the work in between
    auto grab = [&]() -> unsigned long long { return lane64 == 0 ? atomicAdd(next, 1ull) : 0ull; };
    auto bcast = [&](unsigned long long raw) -> int64_t { return (int64_t)__shfl(raw, 0); };
    int64_t run = bcast(grab());                      // the run of units this wave is in
    unsigned long long raw = grab();                  // the run after it, on its way
    // units per run: 1 until every wave has 128 runs to take, then more, up to kUnitsPerGrab
    const int64_t fit = total / ((int64_t)n_waves * 128);
    const int per = fit < 1 ? 1 : fit > kUnitsPerGrab ? kUnitsPerGrab : (int)fit;
    int sub = 0;
    auto next_unit = [&]() -> int64_t {
        if (sub == per) {
            run = bcast(raw);
            raw = grab();
            sub = 0;
        }
        return run * per + sub++;
    };
    auto load_ids = [&](unit_t &u) {
        u.row0 = 0;
        u.id = -1;
        u.fetch = 0;
        int64_t c = u.q;
        if (c >= total) return;
        int b = 0;
        for (;; ++b) {                              // c < total: ends inside the lists
            const int64_t nu = (lists.n[b] + 63) / 64;
            if (c < nu) break;
            c -= nu;
        }
        u.row0 = (SHARE == 2 ? lists.first_req[b] : lists.out_row[b]) + c * 64;
        const int64_t i = c * 64 + lane64;
        if (i < lists.n[b]) u.id = lists.ids[b][i];
    };
    auto classify = [&](unit_t &u) { u.fetch = u.id >= 0 ? is_cold<MODE>(u.id, hot_bits, n_nodes, n_hot) : 0; };

    // shared misses: the first request of an id in this call fetches the row, the others
    // get a deferred copy from that request's output row
    int64_t def_base = -1;                            // wave-uniform: current block of deferred entries
    // entries are reserved in blocks: large ones in a large call (fewer atomics on the one counter), small ones
    // otherwise (what a wave leaves unused of its last block, the copy kernel still has to look through)
    const int defer_block = per > 1 ? kDeferBlock : 64;
    int def_used = defer_block;
    int fetched = 0;                                  // rows this lane sent over the link
    auto pad_deferred = [&]() {                       // unused entries of the current block
        if (def_base < 0) return;
        for (int e = def_used + lane64; e < defer_block; e += 64) cold.deferred[2 * (def_base + e)] = -1;
    };
    auto claim = [&](unit_t &u) {
        if (SHARE == 0) return;
        if (SHARE == 2) {                             // the head of an id's list fetches for the whole list
            if (u.fetch) {
                const unsigned long long cur = cold.claim[u.id];
                u.fetch = (int64_t)(cur & ((1ull << kClaimRowBits) - 1ull)) == u.row0 + lane64;
            }
            return;
        }
        int lose = 0;
        int64_t from = 0;
        if (u.fetch) {
            const unsigned long long mine = cold.stamp | (unsigned long long)(u.row0 + lane64);
            unsigned long long *c = &cold.claim[u.id];
            unsigned long long cur = __hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (;;) {
                if ((cur >> kClaimRowBits) == (cold.stamp >> kClaimRowBits)) {     // claimed in this call: final
                    lose = 1;
                    from = (int64_t)(cur & ((1ull << kClaimRowBits) - 1ull));
                    break;
                }
                const unsigned long long seen = atomicCAS(c, cur, mine);
                if (seen == cur) break;                                           // the claim is ours
                cur = seen;
            }
        }
        const unsigned long long losers = __ballot(lose);
        if (losers) {
            const int n = __popcll(losers);
            const int64_t old_base = def_base;
            if (def_used + n > defer_block) {         // wave-uniform: the entries run over into a fresh block
                unsigned long long base = 0;
                if (lane64 == 0) base = atomicAdd((unsigned long long *)&meta[META_DEFER_N], (unsigned long long)defer_block);
                def_base = (int64_t)__shfl(base, 0);
                def_used -= defer_block;              // < 0: that many entries still go to the old block
            }
            if (lose) {
                const int at = def_used + __popcll(losers & ((1ull << lane64) - 1ull));
                const int64_t e = at < 0 ? old_base + defer_block + at : def_base + at;
                cold.deferred[2 * e] = u.row0 + lane64;
                cold.deferred[2 * e + 1] = from;
                u.fetch = 0;
            }
            def_used += n;
        }
    };
    // copy the n (<= kPerPass) requests at the head of the queue
    // lists of requests: the n (<= kPerPass) rows at the head of the queue, each read once from the host
    // and written to every request on its id's list (q_dst holds the number of the list's head).  A
    // list ends at -1 and every entry points to a request that arrived before it: the walk ends.
    auto fan_out_pass = [&](unsigned head, int n) {
        const uint4 *src[kRowsInFlight];
        int64_t at[kRowsInFlight];
        uint4 v[kRowsInFlight][kFanPieces];
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) {
            const int k = g * kRowsInFlight + j;
            src[j] = nullptr;
            at[j] = -1;
            if (k < n) {
                const unsigned e = (head + (unsigned)k) % kQueue;
                src[j] = host + (int64_t)q_src[e] * cpr;
                at[j] = q_dst[e];
            }
        }
#pragma unroll
        for (int p = 0; p < kFanPieces; ++p) {
            const int cc = lane + p * LPR;
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j) {
                v[j][p] = make_uint4(0, 0, 0, 0);
                if (src[j] && cc < cpr) v[j][p] = src[j][cc];
            }
        }
        bool more = true;
        while (more) {                                // the lanes of a group walk together
            more = false;
            int64_t next[kRowsInFlight], row[kRowsInFlight];
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j) {
                next[j] = -1;
                row[j] = -1;
                if (at[j] >= 0) {
                    next[j] = cold.deferred[2 * at[j]];
                    row[j] = cold.deferred[2 * at[j] + 1];
                }
            }
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j) {
                if (row[j] >= 0) {
                    uint4 *dst = out_base + row[j] * cpr;
#pragma unroll
                    for (int p = 0; p < kFanPieces; ++p) {
                        const int cc = lane + p * LPR;
                        if (cc < cpr) {
                            u32x4 t4 = {v[j][p].x, v[j][p].y, v[j][p].z, v[j][p].w};
                            __builtin_nontemporal_store(t4, (u32x4 *)&dst[cc]);
                        }
                    }
                }
                at[j] = next[j];
                more = more || next[j] >= 0;
            }
        }
    };
    auto copy_pass = [&](unsigned head, int n) {
        if (SHARE == 2) {
            fan_out_pass(head, n);
            return;
        }
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
    unit_t u0, u1, u2, u3;
    u0.q = next_unit();
    u1.q = next_unit();
    u2.q = next_unit();
    u3.q = next_unit();
    load_ids(u0);
    load_ids(u1);
    load_ids(u2);
    classify(u0);
    classify(u1);
    claim(u0);
    while (u0.q < total) {
        load_ids(u3);
        classify(u2);
        claim(u1);
        // the requests of unit 0 that read their row from the host join the queue in request order
        const unsigned long long mask = __ballot(u0.fetch);
        if (u0.fetch) {
            const unsigned before = __popcll(mask & ((1ull << lane64) - 1ull));
            const unsigned e = (head + waiting + before) % kQueue;
            q_src[e] = u0.id;
            q_dst[e] = u0.row0 + lane64;
            ++fetched;
        }
        waiting += (unsigned)__popcll(mask);
        __builtin_amdgcn_wave_barrier();
        while (waiting >= (unsigned)kPerPass) {
            copy_pass(head, kPerPass);
            head = (head + kPerPass) % kQueue;
            waiting -= kPerPass;
        }
        __builtin_amdgcn_wave_barrier();
        u0 = u1;
        u1 = u2;
        u2 = u3;
        u3.q = next_unit();
    }
    if (waiting) copy_pass(head, (int)waiting);       // fewer than a pass left
    if (SHARE) {
        if (SHARE == 1) pad_deferred();
        if (count_rows) {
            for (int off = 32; off > 0; off >>= 1) fetched += __shfl_down(fetched, off);
            if (lane64 == 0 && fetched)
                atomicAdd((unsigned long long *)&meta[META_LINK_ROWS], (unsigned long long)fetched);
        }
    }
    // The wave's last grab (its value is never looked at) must have reached the counter before the wave
    // counts as done: the increment of `done` releases everything this lane issued before it, so the
    // wave that sees n_waves - 1 resets a counter nobody will touch again in this launch.
    if (lane64 == 0 &&
        __hip_atomic_fetch_add(done, 1ull, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == n_waves - 1) {
        atomicExch(next, 0ull);
        atomicExch(done, 0ull);
    }
}

// MODE: GATHER_SLOT     hot <=> slot[id] >= 0, cache row = slot[id]      (ids keep their meaning)
//       GATHER_BOUNDARY hot <=> id < n_hot, cache row = id, cold row = id - n_hot of the cold
//                       part (rows in rank order: the two-way branch of Listing 1)
//       GATHER_HOST     every row from host memory: the untiered copy that fills the HBM
//                       cache at placement time
// SPLIT:  grid row 0 holds the cold workers (scan_cold_rows), list b is served by grid row b + 1
//         and skips its cold rows.  SHARE != 0: the workers fetch every distinct cold row once.
template <int LPR, int MODE, bool SPLIT, int SHARE>
__global__ __launch_bounds__(kBlock) void k_gather(id_lists_t lists, const int32_t *__restrict__ slot,
                                                   const uint32_t *__restrict__ hot_bits,
                                                   const uint4 *__restrict__ cache,
                                                   const uint4 *__restrict__ host,
                                                   uint4 *__restrict__ out_base, int cpr, int64_t n_nodes,
                                                   int64_t n_hot, int64_t *__restrict__ meta, int count_hits,
                                                   cold_t cold)
{
    constexpr int kGroups = kBlock / LPR;
    if (SPLIT && blockIdx.y == 0) {
        scan_cold_rows<LPR, MODE, SHARE>(lists, (int)gridDim.y - 1, hot_bits, n_nodes, n_hot, cold, host, out_base, cpr,
                                         meta, count_hits);
        return;
    }
    const int list = SPLIT ? blockIdx.y - 1 : blockIdx.y;
    const int32_t *__restrict__ ids = lists.ids[list];
    const int64_t n = lists.n[list];
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
                    } else if (MODE == GATHER_BOUNDARY) {
                        const uint4 *cold_part = host + n_hot * cpr;     // first row of the cold part
                        src[j] = cold_part + ((int64_t)id - n_hot) * cpr;
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

// Lists of requests, first step: every cold request of the call enters the list of its id.  claim[id] =
// stamp | number of the last request that arrived; the pair of a request = (the one that was last before
// it, or -1 if the claim was not of this call; its output row).  Grid row b serves list b.
template <int MODE>
__global__ __launch_bounds__(kBlock) void k_link(id_lists_t lists, const uint32_t *__restrict__ hot_bits, int64_t n_nodes,
                                                 int64_t n_hot, unsigned long long *__restrict__ claim,
                                                 unsigned long long stamp, int64_t *__restrict__ pairs)
{
    const int b = blockIdx.y;
    const int32_t *__restrict__ ids = lists.ids[b];
    const int64_t n = lists.n[b], stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const int32_t id = ids[i];
        if (!is_cold<MODE>(id, hot_bits, n_nodes, n_hot)) continue;
        const int64_t req = lists.first_req[b] + i;
        const unsigned long long old = atomicExch(&claim[id], stamp | (unsigned long long)req);
        const bool mine = (old >> kClaimRowBits) == (stamp >> kClaimRowBits);
        pairs[2 * req] = mine ? (int64_t)(old & ((1ull << kClaimRowBits) - 1ull)) : -1;
        pairs[2 * req + 1] = lists.out_row[b] + i;
    }
}

// Shared misses, second step: out[first] = out[second] for every deferred pair the cold
// workers of the launch before left behind (rows that another request of the same call
// has already brought over the host link).  A copy inside HBM.
template <int LPR>
__global__ __launch_bounds__(kBlock) void k_copy_deferred(const int64_t *__restrict__ deferred,
                                                          int64_t *__restrict__ meta,
                                                          uint4 *__restrict__ out, int cpr)
{
    constexpr int kGroups = kBlock / LPR;
    const int64_t n = meta[META_DEFER_N];             // entries reserved, unused ones marked
    const int lane = threadIdx.x % LPR;
    const int64_t group = (int64_t)blockIdx.x * kGroups + threadIdx.x / LPR;
    const int64_t n_groups = (int64_t)gridDim.x * kGroups;
    for (int64_t e0 = group * kRowsInFlight; e0 < n; e0 += n_groups * kRowsInFlight) {
        const uint4 *src[kRowsInFlight];
        uint4 *dst[kRowsInFlight];
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) {
            src[j] = nullptr;
            dst[j] = nullptr;
            if (e0 + j < n) {
                const int64_t to = deferred[2 * (e0 + j)];
                if (to >= 0) {
                    dst[j] = out + to * cpr;
                    src[j] = out + deferred[2 * (e0 + j) + 1] * cpr;
                }
            }
        }
        for (int c = lane; c < cpr; c += LPR) {
            uint4 v[kRowsInFlight];
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j) {
                v[j] = make_uint4(0, 0, 0, 0);
                if (src[j]) v[j] = src[j][c];
            }
#pragma unroll
            for (int j = 0; j < kRowsInFlight; ++j)
                if (dst[j]) dst[j][c] = v[j];
        }
    }
    // the last block to finish leaves the list empty for the next call (every block has read n by then)
    __syncthreads();
    if (threadIdx.x == 0 &&
        atomicAdd((unsigned long long *)&meta[META_DEFER_DONE], 1ull) == (unsigned long long)gridDim.x - 1) {
        meta[META_DEFER_N] = 0;
        meta[META_DEFER_DONE] = 0;
    }
}

// Before a launch that counts: hit counters, link rows and the id-error flag back to zero, so that the
// statistics (and the error) a call reports are its own.
__global__ void k_gather_prepare(int64_t *meta)
{
    if (threadIdx.x < META_HIT_STRIPES) meta[META_HIT_ROWS + threadIdx.x] = 0;
    if (threadIdx.x == 0) {
        meta[META_LINK_ROWS] = 0;
        meta[META_ERROR] = 0;
    }
}

__global__ void k_zero_claims(unsigned long long *claim, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) claim[i] = 0ull;
}

int lanes_per_row(int cpr)
{
    int lpr = 8;
    while (lpr < cpr && lpr < 64) lpr *= 2;
    return lpr;
}

}  // namespace

// One k_gather launch on stream st, bookkeeping words in meta.  split: with cold workers;
// share (with split only): they fetch every distinct cold row of the launch once, by claims and
// deferred copies (1) or by lists of requests (2: k_link first, no copies afterwards).
// The hot tier a launch reads: the context's placement, or the rows staged ahead of one.
struct hot_tier_t {
    const int32_t *slot;
    const uint32_t *hot_bits;
    const void *rows;
    int64_t n_hot;
};

static int launch_lists(tier_ctx *ctx, const id_lists_t &lists, int n_lists, int64_t n_max, int mode, void *out,
                        bool count_hits, hipStream_t st, int64_t *meta, bool split = false, int share = 0,
                        const hot_tier_t *other_tier = nullptr, int link_blocks_cap = 0)
{
    const hot_tier_t hot = other_tier ? *other_tier : hot_tier_t{ctx->slot, ctx->hot_bits, ctx->cache, ctx->n_hot};
    if (count_hits) k_gather_prepare<<<1, META_HIT_STRIPES, 0, st>>>(meta);
    if (n_max <= 0) return TIER_OK;
    const int cpr = (int)(ctx->row_bytes / 16);
    const int lpr = lanes_per_row(cpr);
    const int groups = kBlock / lpr;
    int64_t blocks = (n_max + (int64_t)groups * kRowsInFlight - 1) / ((int64_t)groups * kRowsInFlight);
    const int64_t max_blocks = 1 << 18;     // beyond that groups loop; fewer blocks cost ~5 % of the all-hit rate
    if (blocks > max_blocks) blocks = max_blocks;
    if (mode == GATHER_HOST && ctx->rows_on_host) {
        // every row over the host link: a few dozen blocks fill it, more only queue up
        if (blocks > kLinkBlocks) blocks = kLinkBlocks;
        if (link_blocks_cap > 0 && blocks > link_blocks_cap) blocks = link_blocks_cap;
    }
    cold_t cold = {};
    if (split) {
        const int want = ctx->link_blocks > 0 ? ctx->link_blocks : kLinkBlocks;
        cold.workers = (int)(want < blocks ? want : blocks);
        if (share) {
            cold.stamp = (unsigned long long)ctx->claim_stamp << kClaimRowBits;
            cold.claim = ctx->claim;
            cold.deferred = ctx->deferred;
        }
    }
    if (split && share == 2) {
        int64_t lb = (n_max + kBlock - 1) / kBlock;
        if (lb > 4096) lb = 4096;
        const dim3 lgrid((unsigned)lb, (unsigned)n_lists);
        if (mode == GATHER_BOUNDARY)
            k_link<GATHER_BOUNDARY><<<lgrid, kBlock, 0, st>>>(lists, hot.hot_bits, ctx->n_nodes, hot.n_hot, ctx->claim, cold.stamp,
                                                              ctx->deferred);
        else
            k_link<GATHER_SLOT><<<lgrid, kBlock, 0, st>>>(lists, hot.hot_bits, ctx->n_nodes, hot.n_hot, ctx->claim, cold.stamp,
                                                          ctx->deferred);
    }
    const dim3 grid((unsigned)blocks, (unsigned)(n_lists + (split ? 1 : 0)));
#define GATHER_LAUNCH(L, M, P, D)                                                                    \
    k_gather<L, M, P, D><<<grid, kBlock, 0, st>>>(lists, hot.slot, hot.hot_bits, (const uint4 *)hot.rows, \
                                                  (const uint4 *)ctx->host_rows, (uint4 *)out, cpr,  \
                                                  ctx->n_nodes, hot.n_hot, meta, count_hits ? 1 : 0, cold)
#define GATHER_CASE(L)                                                                               \
    case L:                                                                                          \
        if (mode == GATHER_SLOT && split && share == 2) GATHER_LAUNCH(L, GATHER_SLOT, true, 2);      \
        else if (mode == GATHER_BOUNDARY && split && share == 2) GATHER_LAUNCH(L, GATHER_BOUNDARY, true, 2); \
        else if (mode == GATHER_SLOT && split && share) GATHER_LAUNCH(L, GATHER_SLOT, true, 1);      \
        else if (mode == GATHER_BOUNDARY && split && share) GATHER_LAUNCH(L, GATHER_BOUNDARY, true, 1); \
        else if (mode == GATHER_SLOT && split) GATHER_LAUNCH(L, GATHER_SLOT, true, 0);               \
        else if (mode == GATHER_BOUNDARY && split) GATHER_LAUNCH(L, GATHER_BOUNDARY, true, 0);       \
        else if (mode == GATHER_SLOT) GATHER_LAUNCH(L, GATHER_SLOT, false, 0);                       \
        else if (mode == GATHER_BOUNDARY) GATHER_LAUNCH(L, GATHER_BOUNDARY, false, 0);               \
        else GATHER_LAUNCH(L, GATHER_HOST, false, 0);                                                \
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
    if (split && share == 1) {
        const dim3 dgrid(1024);
        switch (lpr) {
        case 8: k_copy_deferred<8><<<dgrid, kBlock, 0, st>>>(ctx->deferred, meta, (uint4 *)out, cpr); break;
        case 16: k_copy_deferred<16><<<dgrid, kBlock, 0, st>>>(ctx->deferred, meta, (uint4 *)out, cpr); break;
        case 32: k_copy_deferred<32><<<dgrid, kBlock, 0, st>>>(ctx->deferred, meta, (uint4 *)out, cpr); break;
        default: k_copy_deferred<64><<<dgrid, kBlock, 0, st>>>(ctx->deferred, meta, (uint4 *)out, cpr); break;
        }
        TIER_HIP(ctx, hipGetLastError());
    }
    return TIER_OK;
}

int tier_launch_gather(tier_ctx *ctx, const int32_t *ids, int64_t n, int mode, void *out, bool count_hits,
                       int link_blocks_cap)
{
    id_lists_t lists = {};
    lists.ids[0] = ids;
    lists.n[0] = n;
    return launch_lists(ctx, lists, 1, n, mode, out, count_hits, ctx->gather_stream, ctx->gmeta, false, false, nullptr,
                        link_blocks_cap);
}

int tier_launch_fill_staged(tier_ctx *ctx, const int32_t *ids, int64_t n, void *out)
{
    id_lists_t lists = {};
    lists.ids[0] = ids;
    lists.n[0] = n;
    const hot_tier_t staged = {ctx->staged_of, ctx->staged_bits, ctx->staging, ctx->staged_rows};
    return launch_lists(ctx, lists, 1, n, GATHER_SLOT, out, false, ctx->gather_stream, ctx->gmeta, true, false, &staged);
}

// Claims hold an output row in kClaimRowBits bits.
static bool dedup_applies(const tier_ctx *ctx, const id_lists_t &lists, int n_lists, int64_t n_total)
{
    if (!ctx->dedup || n_total <= 0 || ctx->n_hot >= ctx->n_nodes) return false;
    for (int b = 0; b < n_lists; ++b)
        if (lists.out_row[b] + lists.n[b] >= (1LL << kClaimRowBits)) return false;
    return true;
}

// The tiered gather of one call: one uniform launch, or one launch with cold workers
// apart, which with shared misses fetch every distinct cold row once.
static int gather_call(tier_ctx *ctx, const id_lists_t &lists, int n_lists, int64_t n_max, int64_t n_total, void *out,
                       bool count_hits)
{
    const int mode = ctx->boundary ? GATHER_BOUNDARY : GATHER_SLOT;
    hipStream_t st = ctx->gather_stream;
    ctx->maps_in_use = true;
    const bool any_cold = n_total > 0 && ctx->n_hot < ctx->n_nodes;     // nothing to split off otherwise
    ctx->last_deduped = dedup_applies(ctx, lists, n_lists, n_total);
    if (ctx->last_deduped) {
        // deferred entries: one per request at most, plus the block that each worker wave leaves part empty
        const int64_t workers = ctx->link_blocks > 0 ? ctx->link_blocks : kLinkBlocks;
        const int64_t entries = n_total + (int64_t)kDeferBlock * (workers * (kBlock / 64) + 1);
        int rc = tier_ensure(ctx, (void **)&ctx->deferred, &ctx->deferred_cap, (size_t)entries * 2 * sizeof(int64_t));
        if (rc != TIER_OK) return rc;
        if (++ctx->claim_stamp >= (1u << (64 - kClaimRowBits))) {     // stamps used up: start over on a clean table
            k_zero_claims<<<4096, kBlock, 0, st>>>(ctx->claim, ctx->n_nodes);
            ctx->claim_stamp = 1;
        }
        // a call that asks for at least twice as many rows as there are nodes repeats most of its ids: lists of
        // requests instead of copies afterwards (rows of up to kFanPieces x 64 x 16 bytes: a lane holds the pieces)
        const bool by_lists = n_total >= 2 * ctx->n_nodes && ctx->row_bytes <= kFanPieces * 64 * 16;
        id_lists_t numbered = lists;
        int64_t before = 0;
        for (int b = 0; b < n_lists; ++b) {
            numbered.first_req[b] = before;
            before += lists.n[b];
        }
        return launch_lists(ctx, numbered, n_lists, n_max, mode, out, count_hits, st, ctx->gmeta, true, by_lists ? 2 : 1);
    }
    const bool split = ctx->link_blocks > 0 && any_cold && n_total >= ctx->split_min_rows;
    return launch_lists(ctx, lists, n_lists, n_max, mode, out, count_hits, st, ctx->gmeta, split);
}

// hit / miss rows of the launch since the last k_gather_prepare on the gather stream
static int read_stats(tier_ctx *ctx, int64_t n_total, tier_gather_stats *stats)
{
    TIER_HIP(ctx, hipMemcpyAsync(ctx->gmeta_host, ctx->gmeta, GMETA_WORDS * sizeof(int64_t), hipMemcpyDeviceToHost,
                                 ctx->gather_stream));
    TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
    if (ctx->gmeta_host[META_ERROR] != 0) return TIER_EINVAL;     // an id of this call outside [0, n_nodes)
    stats->hit_rows = 0;
    for (int i = 0; i < META_HIT_STRIPES; ++i) stats->hit_rows += ctx->gmeta_host[META_HIT_ROWS + i];
    stats->miss_rows = n_total - stats->hit_rows;
    stats->link_rows = ctx->last_deduped ? ctx->gmeta_host[META_LINK_ROWS] : stats->miss_rows;
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
    if (on && !ctx->claim) {
        const int64_t n = ctx->n_nodes > 0 ? ctx->n_nodes : 1;
        TIER_HIP(ctx, hipMalloc(&ctx->claim, (size_t)n * sizeof(unsigned long long)));
        k_zero_claims<<<4096, kBlock, 0, ctx->gather_stream>>>(ctx->claim, n);
        TIER_HIP(ctx, hipGetLastError());
        TIER_HIP(ctx, hipStreamSynchronize(ctx->gather_stream));
        ctx->claim_stamp = 0;
    }
    ctx->dedup = on != 0;
    return TIER_OK;
}
