#!/usr/bin/env python3
"""Benchmark of the data-tiering hot path on one MI355X.

One *step* is one pass of the whole path over one synthetic workload: a
presampling epoch (access counts), placement under the HBM budget, then one
measured epoch of mini-batches, each sampled (tier_sample_minibatch) and then
gathered (tier_gather_features).  The measured epoch uses another seed and
another order of the training nodes than the presampling epoch.

Prints ONE JSON line.  ``value`` is gathered feature bytes per second of step
wall time (everything above included); the per-kernel figures, the roofline of
the dominant kernel (the tiered gather, timed per launch with events on its
stream) and a CPU baseline (the tests' oracle on the host cores, on a bounded
sample of the same workload) ride along.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
LINK_PEAK_GBPS = 64.0           # PCIe Gen5 x16, one direction, nominal
SPLIT_MIN_ROWS = 1 << 17        # gather calls below this many rows keep the uniform launch


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg3",
                    help="cfg1..cfg5; the default is the largest configuration that fits one GPU and this host's pinned "
                         "memory (cfg3: 111 M nodes, 56.8 GB of features)")
    ap.add_argument("--budget", type=float, default=None, help="override: fraction of feature bytes kept in HBM")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-streams", action="store_true", help="skip the all-hit / all-miss gather runs")
    ap.add_argument("--no-reorder", action="store_true",
                    help="skip the reordered variant (graph and table renamed by rank, gather by boundary)")
    ap.add_argument("--no-scores", action="store_true",
                    help="skip the comparison of score functions (presampled counts vs the paper's scores)")
    ap.add_argument("--sweeps", action="store_true",
                    help="also sweep the HBM budget and the sampling depth (analogues of the paper's Fig. 5 and 6)")
    ap.add_argument("--link-blocks", type=int, default=-1,
                    help="blocks of the cold-row launch of the split gather (0: one uniform launch per call; default: 48, "
                         "which leaves the sampling calls beside the gathers a third more room than 64 at the same gather "
                         "time, and 192 on cfg5: nine of ten cold requests there are repeats within the call, and it takes "
                         "that many blocks to look through them, and to write every fetched row to all its requests, "
                         "as fast as the link delivers)")
    ap.add_argument("--group", type=int, default=0,
                    help="mini-batches per sampling / gather call (at most what the context takes, up to 64); a larger "
                         "group shares more cold rows per call and holds that many mini-batches' rows in HBM at once.  "
                         "0: 16, or 64 on the miss-dominated cfg5, where the rows held are small next to the cache")
    ap.add_argument("--sample-group", type=int, default=0,
                    help="mini-batches per sampling call (a multiple of --group; the blocks of one sampling call are "
                         "gathered --group at a time).  0: as many as the context takes, up to 64: blocks are small "
                         "(7 MB per mini-batch on cfg3) and the sampler's many short kernels fill the chip better "
                         "with more mini-batches side by side")
    ap.add_argument("--no-groups", action="store_true", help="skip the comparison of group sizes 16 / 32 / 64")
    ap.add_argument("--no-budget-sweep", action="store_true",
                    help="skip the placement + epoch at the other HBM budgets of the workload (cfg3: 5 % and 20 %)")
    ap.add_argument("--no-prefetch", action="store_true",
                    help="presample in one piece; default: the counts of the first quarter of the mini-batches pick rows "
                         "that are fetched into HBM while the rest is presampled (tier_prefetch)")
    ap.add_argument("--prefetch-share", type=float, default=0.3, help="share of the cache's rows fetched ahead")
    ap.add_argument("--prefetch-first", type=int, default=0,
                    help="mini-batches presampled before the rows to fetch ahead are chosen (default: a quarter, whole chains of 64)")
    ap.add_argument("--no-shared-misses", action="store_true",
                    help="read every requested cold row over the host link, also those a call requests more than once")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink nodes, edges and budget alike")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB streaming kernel (reference for profiler byte counters)")
    ap.add_argument("--cpu-batches", type=int, default=192, help="mini-batches in the CPU baseline's sample")
    ap.add_argument("--sampler-part", choices=("both", "counts", "blocks"), default="both",
                    help="with --sampler-only: presampling only, the epoch's blocks only, or both (for kernel profiles by part)")
    ap.add_argument("--sampler-only", action="store_true",
                    help="run only the sampler (presampling epoch, then the measured epoch's blocks, no gathers) and print "
                         "its own JSON line: a clean subject for rocprofv3 runs on the sampling kernels")
    args = ap.parse_args()
    if args.link_blocks < 0:
        args.link_blocks = 192 if args.workload == "cfg5" else 48
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2111_05894_amd import synth, tier

    tier._load()                                   # fail loudly when the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = synth.WORKLOADS[args.workload]
    t0 = time.time()
    dtype = torch.float32 if wl.dtype == "float32" else torch.float16
    scale = args.scale
    try:
        table = tier.tier_host_alloc(max(64, int(wl.n_nodes * scale)), wl.dim, dtype)
    except tier.TierError as e:
        # the host refuses to pin that much memory: same recipe at 2/3 of the size
        scale = scale * 0.66
        log(f"[bench] {wl.feature_bytes * args.scale / 2**30:.1f} GiB of pinned host memory refused ({e}); "
            f"running at scale {scale}")
        table = tier.tier_host_alloc(max(64, int(wl.n_nodes * scale)), wl.dim, dtype)
    indptr, indices, train = synth.make_graph(wl, dev, scale)
    torch.cuda.synchronize()
    n = indptr.numel() - 1
    log(f"[bench] {wl.name}: {n} nodes, {indices.numel()} edges, {train.numel()} train nodes "
        f"({time.time() - t0:.1f}s to generate)")
    synth.fill_features(table.tensor, wl.dist, synth.GRAPH_SEED + 2, dev)
    torch.cuda.synchronize()
    log(f"[bench] features: {table.nbytes / 1e9:.2f} GB pinned ({time.time() - t0:.1f}s)")

    ctx = tier.tier_create(indptr, indices, table)
    R = ctx.row_bytes
    budget = int(wl.budget_bytes(args.budget) * scale)
    n_train = train.numel()
    bs = wl.batch_size
    n_batches = -(-n_train // bs)
    order = synth.random_order(n_train, synth.EPOCH_SEED, 1, dev)
    epoch_ids = train[order].contiguous()
    B_max = tier.tier_max_batches(ctx)             # mini-batches sampled side by side per call
    group = args.group if args.group > 0 else (64 if wl.name == "cfg5" else 16)
    B = min(B_max, group)
    group_sizes = sorted({min(B_max, g) for g in (16, 32, 64)} | {B}) if not args.no_groups else [B]

    def grouping(size):
        return [list(range(g, min(g + size, n_batches))) for g in range(0, n_batches, size)]

    groups = grouping(B)
    S = args.sample_group if args.sample_group > 0 else 64
    per_sample = max(1, min(B_max, S) // B)        # gather groups per sampling call
    bseed = [tier.tier_batch_seed(synth.EPOCH_SEED, 0, b) for b in range(n_batches)]
    # three sets of block buffers: while up to two groups of mini-batches wait for or run their
    # gather (gather stream, host-link bound) the next group is sampled (main stream, latency bound)
    blocks2 = [tier.BlocksBatch(n, bs, wl.fanouts, max(max(group_sizes), B * per_sample), dev) for _ in range(3)]
    blocks = blocks2[0]
    out_buf = [torch.empty((blocks.cap_nodes[-1], wl.dim), dtype=dtype, device=dev)]
    counts = torch.empty(n, dtype=torch.int32, device=dev)
    L = len(wl.fanouts)
    gs = torch.cuda.Stream()
    tier.tier_set_gather_stream(ctx, gs)
    tier.tier_set_gather_split(ctx, args.link_blocks, SPLIT_MIN_ROWS)
    shared_on = not args.no_shared_misses
    tier.tier_set_gather_dedup(ctx, shared_on)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def sample_group(g, into=None):
        lo = g[0] * bs
        hi = min(n_train, (g[-1] + 1) * bs)
        return tier.tier_sample_minibatches(ctx, epoch_ids[lo:hi], bs, [bseed[b] for b in g], wl.fanouts,
                                            into if into is not None else blocks)

    def sample_span(span, into=None):
        """One sampling call for the mini-batches of consecutive groups."""
        return sample_group([b for g in span for b in g], into)

    def timed_gather(blk, nb, first=0):
        """One gather launch (nb mini-batches of the blocks, from mini-batch `first` on) bracketed by events on its stream."""
        rows = sum(blk.n_nodes[first + i][L] for i in range(nb))
        if rows > out_buf[0].shape[0]:             # grows during warm-up only
            torch.cuda.synchronize()
            out_buf[0] = torch.empty((int(rows * 1.1), wl.dim), dtype=dtype, device=dev)
        with torch.cuda.stream(gs):
            a, b_ = ev(), ev()
            a.record()
            tier.tier_gather_minibatches(ctx, blk, nb, out_buf[0], first_batch=first)
            b_.record()
        return a, b_, rows

    def epoch(record, begin=None, groups=groups, per=per_sample):
        """The measured epoch: the mini-batches sampled `per` groups per call (main stream) and gathered
        a group per call (gather stream).  begin: event on the gather stream from which the epoch's wall
        time counts (the end of the cache fill, which the first sampling calls overlap); default: now."""
        if begin is None:
            torch.cuda.synchronize()
            with torch.cuda.stream(gs):
                begin = ev(); begin.record()
        rows = edges = most = 0
        s_pairs, g_pairs = [], []
        NB = len(blocks2)
        reads_done = [None] * NB                   # last gather that reads blocks2[i]
        for si in range(0, len(groups), per):
            # the gathers of a sampling call's groups are launched as soon as it returns; the host then
            # sits in the next (synchronous) sampling call while they run, so the gather stream always
            # has a launch waiting, and the third buffer keeps the host from waiting for a gather to end
            span, buf = groups[si:si + per], (si // per) % NB
            if reads_done[buf] is not None:
                reads_done[buf].synchronize()      # its ids are about to be overwritten
            s0, s1 = ev(), ev()
            s0.record(); blk = sample_span(span, blocks2[buf]); s1.record()
            s_pairs.append((s0, s1))
            first = 0
            for g in span:
                a, b_, r = timed_gather(blk, len(g), first)
                g_pairs.append((a, b_))
                rows += r; edges += sum(sum(blk.n_edges[first + i]) for i in range(len(g)))
                most = max(most, r)
                first += len(g)
            reads_done[buf] = b_
        torch.cuda.synchronize()
        if record is not None:
            record["epoch_wall_ms"].append(begin.elapsed_time(g_pairs[-1][1]) if g_pairs else 0.0)
            record["sample_ms"].append(sum(a.elapsed_time(b_) for a, b_ in s_pairs))
            record["gather_ms"].append(sum(a.elapsed_time(b_) for a, b_ in g_pairs))
            record["rows"] = rows; record["edges"] = edges
            record["gather_launches"] = len(g_pairs)
            record["most_rows_per_call"] = most
        return rows, edges

    # Fetching ahead: the host link has nothing to do while the access counts are collected, and the
    # counts of the first mini-batches already name the hottest rows.  So the first quarter of the
    # mini-batches (whole chains of 64) is presampled, the rows that rank first by those counts start
    # moving into HBM on the gather stream, and the rest is presampled meanwhile; the placement then
    # fills the cache from HBM where it can.  Same counts, same slot map, same cache.
    # (below 256 mini-batches the presampling is too short for this to pay: cfg2, cfg5 measured 1 % slower)
    first_batches = (n_batches // 4) // 64 * 64
    if args.prefetch_first > 0:
        first_batches = min(args.prefetch_first, n_batches)
    prefetch_rows = int(args.prefetch_share * min(n, budget // R)) if (first_batches and not args.no_prefetch) else 0

    def step(record, prefetch=True):
        e_begin, e_pre, e_sorted, e_fill = ev(), ev(), ev(), ev()
        e_begin.record()
        if prefetch and prefetch_rows > 0:
            tier.tier_presample_range(ctx, train, bs, wl.fanouts, 1, synth.PRESAMPLE_SEED, 0, first_batches, counts)
            tier.tier_prefetch(ctx, counts, prefetch_rows)
            tier.tier_presample_range(ctx, train, bs, wl.fanouts, 1, synth.PRESAMPLE_SEED, first_batches, 1 << 40, counts,
                                      accumulate=True)
        else:
            tier.tier_presample(ctx, train, bs, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts)
        e_pre.record()
        _, n_hot = tier.tier_place(ctx, counts, budget, want_slot_map=False)
        e_sorted.record()                          # order and slot map; the cache fill runs on the gather stream
        with torch.cuda.stream(gs):
            e_fill.record()
        rows, edges = epoch(record, e_fill)
        if record is not None:
            record["presample_ms"].append(e_begin.elapsed_time(e_pre))
            record["place_ms"].append(e_pre.elapsed_time(e_fill))
            record["place_sort_ms"].append(e_pre.elapsed_time(e_sorted))
            record["n_hot"] = n_hot
        return rows, edges

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)       # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        torch.bitwise_not(src, out=dst)                                # a plain streaming kernel, by name in the trace
        torch.cuda.synchronize()
        del src, dst

    if args.sampler_only:
        def timed_ms(f):
            a, b_ = ev(), ev()
            torch.cuda.synchronize()
            a.record(); r = f(); b_.record(); torch.cuda.synchronize()
            return r, a.elapsed_time(b_)
        def sample_epoch():
            e = 0
            for si in range(0, len(groups), per_sample):
                span = groups[si:si + per_sample]
                blk = sample_span(span)
                e += sum(sum(blk.n_edges[i]) for i in range(sum(len(g) for g in span)))
            return e
        pre, smp = [], []
        edges_e = 0
        for it in range(args.warmup + max(args.steps, 1)):
            t_pre = t_smp = float("inf")
            if args.sampler_part != "blocks":
                _, t_pre = timed_ms(lambda: tier.tier_presample(ctx, train, bs, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts))
            if args.sampler_part != "counts":
                edges_e, t_smp = timed_ms(sample_epoch)
            if it >= args.warmup:
                pre.append(t_pre); smp.append(t_smp)
        rows_p = edges_p = 0
        if args.sampler_part != "blocks":
            _, rows_p, edges_p = tier.tier_presample(ctx, train, bs, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts, want_totals=True)
        print(json.dumps({"workload": wl.name, "mini_batches": n_batches, "mini_batches_per_call": B * per_sample,
                          "sampler_part": args.sampler_part,
                          "presample_ms": round(min(pre), 3) if edges_p else None, "presample_rows": rows_p, "presample_edges": edges_p,
                          "presample_edges_per_s": round(edges_p / (min(pre) * 1e-3)) if edges_p else None,
                          "sample_epoch_ms": round(min(smp), 3) if edges_e else None, "sample_epoch_edges": edges_e,
                          "sampled_edges_per_s": round(edges_e / (min(smp) * 1e-3)) if edges_e else None,
                          "note": "presampling = one epoch in counting mode (up to 64 mini-batches per chain, no blocks); "
                                  "sample_epoch = the measured epoch's blocks, mini_batches_per_call per call; best of steps"}), flush=True)
        ctx.close()
        return

    mean = lambda xs: sum(xs) / len(xs) if xs else 0.0
    for _ in range(args.warmup):
        step(None)
    rec = {"presample_ms": [], "place_ms": [], "place_sort_ms": [], "sample_ms": [], "gather_ms": [], "epoch_wall_ms": []}
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    ms_per_step = wall * 1e3 / max(args.steps, 1)

    # the same step without fetching ahead (one presampling call, the whole cache filled after the ranking)
    prefetch = None
    if prefetch_rows > 0:
        prec = {"presample_ms": [], "place_ms": [], "place_sort_ms": [], "sample_ms": [], "gather_ms": [], "epoch_wall_ms": []}
        step(None, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = min(max(args.steps, 1), 2)
        for _ in range(reps):
            step(prec, False)
        torch.cuda.synchronize()
        prefetch = {"first_mini_batches": first_batches, "rows_fetched_ahead": prefetch_rows,
                    "share_of_the_cache": args.prefetch_share,
                    "step_ms_without": round((time.perf_counter() - t0) * 1e3 / reps, 3),
                    "presample_ms_without": round(mean(prec["presample_ms"]), 3),
                    "place_ms_without": round(mean(prec["place_ms"]), 3),
                    "note": "timed step: the first mini-batches' counts rank the rows, the first of them move into HBM "
                            "on the gather stream while the rest is presampled (phase presample then includes that "
                            "ranking), the placement fills the cache from HBM where it can; without: one presampling "
                            "call, then the whole cache over the host link.  Counts, slot map and cache are the same"}

    # the same epoch with the uniform gather launch (every block copies hot and cold rows)
    uniform = None
    if args.link_blocks > 0:
        tier.tier_set_gather_dedup(ctx, False)
        tier.tier_set_gather_split(ctx, 0, 0)
        urec = {"sample_ms": [], "gather_ms": [], "epoch_wall_ms": []}
        epoch(None)
        for _ in range(min(max(args.steps, 1), 3)):
            epoch(urec)
        tier.tier_set_gather_split(ctx, args.link_blocks, SPLIT_MIN_ROWS)
        tier.tier_set_gather_dedup(ctx, shared_on)
        uniform = {"epoch_wall_ms": round(sum(urec["epoch_wall_ms"]) / len(urec["epoch_wall_ms"]), 3),
                   "gather_ms": round(sum(urec["gather_ms"]) / len(urec["gather_ms"]), 3),
                   "sample_ms": round(sum(urec["sample_ms"]) / len(urec["sample_ms"]), 3)}

    def epoch_stats(groups):
        """hit rows and rows over the host link of the measured epoch (asking for them waits per call)."""
        hits = links = 0
        for g in groups:
            blk = sample_group(g)
            _, _, h, m = tier.tier_gather_minibatches(ctx, blk, len(g), out_buf[0], want_stats=True)
            hits += h
            links += ctx.last_link_rows          # the misses, or with shared misses the distinct ones per call
        return hits, links

    # the same epoch (same placement) with other numbers of mini-batches per call
    group_table = None
    if len(group_sizes) > 1:
        group_table = {}
        for size in group_sizes:
            gg = grouping(size)
            grec = {"sample_ms": [], "gather_ms": [], "epoch_wall_ms": []}
            epoch(None, groups=gg, per=1)          # grows the output buffer
            for _ in range(2):
                epoch(grec, groups=gg, per=1)
            hits, links = epoch_stats(gg)
            cold = grec["rows"] - hits
            alone = []
            for _ in range(2):                     # the same calls with no gather beside them
                torch.cuda.synchronize()
                a, b_ = ev(), ev()
                a.record()
                for g in gg:
                    sample_group(g)
                b_.record(); torch.cuda.synchronize()
                alone.append(a.elapsed_time(b_))
            group_table[str(size)] = {
                "sample_alone_ms": round(min(alone), 3),
                "sampled_edges_per_s": round(grec["edges"] / (min(alone) * 1e-3)),
                "epoch_wall_ms": round(min(grec["epoch_wall_ms"]), 3), "gather_ms": round(min(grec["gather_ms"]), 3),
                "sample_ms": round(min(grec["sample_ms"]), 3),
                "cold_requests_crossing_the_link": round(links / cold, 4) if cold else 1.0,
                "output_rows_held": grec["most_rows_per_call"], "output_bytes_held": grec["most_rows_per_call"] * R,
                "gather_launches": grec["gather_launches"]}
        group_table["note"] = ("same placement, whole epoch sampled and gathered `size` mini-batches per call each (best of 2); "
                               "a larger call shares more cold rows and holds that many mini-batches' output rows at once; "
                               "sample_alone_ms / sampled_edges_per_s: the epoch's sampling calls with the GPU to themselves")

    # hit / miss rows of the measured epoch (outside the timed region: asking for them waits per batch)
    hit_rows, link_rows = epoch_stats(groups)
    # the sampler on its own (in the timed region it shares the GPU with the gathers)
    torch.cuda.synchronize()
    a, b_ = ev(), ev()
    a.record()
    for si in range(0, len(groups), per_sample):
        sample_span(groups[si:si + per_sample])
    b_.record(); torch.cuda.synchronize()
    sample_alone_ms = a.elapsed_time(b_)
    rows, edges = rec["rows"], rec["edges"]
    h = hit_rows / rows if rows else 0.0
    gather_ms, sample_ms = mean(rec["gather_ms"]), mean(rec["sample_ms"])
    gathered_bytes = rows * R
    value = gathered_bytes / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the gather.  Algorithmic bytes per row: the row read once (HBM or
    # host link) and written once (HBM), plus the 4-byte id and the 4-byte slot lookup.
    alg_bytes_row = 2 * R + 8
    launches = rec["gather_launches"]
    avg_launch_ms = gather_ms / launches if launches else 0.0
    alg_per_launch = alg_bytes_row * rows / launches if launches else 0.0
    achieved = alg_per_launch / (avg_launch_ms * 1e-3) / 1e9 if avg_launch_ms else 0.0
    # d = share of the cold requests that have to cross the link: all of them, or with shared misses
    # the distinct ones of each call (the repeats are copies inside HBM)
    d = link_rows / (rows - hit_rows) if rows > hit_rows else 1.0
    hbm_b = (1 + h + (1 - h) * (1 - d)) * R + 8     # per row through HBM
    link_b = (1 - h) * d * R                        # per row over the host link
    peak_time_additive = alg_bytes_row / (hbm_b / HBM_PEAK_GBPS + link_b / LINK_PEAK_GBPS)
    peak_overlap = alg_bytes_row / max(hbm_b / HBM_PEAK_GBPS, link_b / LINK_PEAK_GBPS)   # both streams fully overlapped
    peak_arithmetic = h * HBM_PEAK_GBPS + (1 - h) * LINK_PEAK_GBPS
    link_share = (link_b / LINK_PEAK_GBPS) / (hbm_b / HBM_PEAK_GBPS + link_b / LINK_PEAK_GBPS)
    roofline = {
        "bound": "host-link+hbm", "binding_term": f"host link: {100 * link_share:.0f} % of the blend's time per row is the cold rows' "
                                                  f"crossing of the PCIe link, the rest HBM traffic",
        "kernel": "k_gather", "achieved": round(achieved, 2),
        "peak": round(peak_time_additive, 2), "unit": "GB/s",
        "frac": round(achieved / peak_time_additive, 4) if peak_time_additive else None,
        "traffic": measured_traffic(wl.name) if scale == 1.0 and args.budget is None else None,
        "peak_model": "time-additive blend: (2R+8) / (hbm_bytes/HBM + link_bytes/link) per row, link_bytes = (1-h) d R, "
                      "hbm_bytes = (1 + h + (1-h)(1-d)) R + 8, d = share of the cold requests that must cross the link "
                      "(1, or with shared misses the distinct cold rows of each call); HBM 8000 GB/s, host link 64 GB/s",
        "overlap_bound_peak": round(peak_overlap, 2),
        "frac_vs_overlap_bound": round(achieved / peak_overlap, 4) if peak_overlap else None,
        "overlap_bound_model": "(2R+8) / max(hbm_bytes/HBM, link_bytes/link): the strict ceiling when HBM and link "
                               "transfers overlap perfectly; the time-additive peak above adds the two times and "
                               "can be exceeded by a kernel that overlaps them",
        "hit_fraction": round(h, 4), "cold_requests_crossing_the_link": round(d, 4),
        "avg_launch_ms": round(avg_launch_ms, 4), "launches_per_step": launches,
        "alg_bytes_per_launch": round(alg_per_launch),
        "feature_read_GBps": round(gathered_bytes / (gather_ms * 1e-3) / 1e9, 2) if gather_ms else None,
        "host_link_GBps": round(link_rows * R / (gather_ms * 1e-3) / 1e9, 2) if gather_ms else None,
        "arithmetic_blend_peak": round(peak_arithmetic, 1),
        "arithmetic_blend_frac": round(gathered_bytes / (gather_ms * 1e-3) / 1e9 / peak_arithmetic, 4) if gather_ms else None,
    }

    # the workload's other HBM budgets: placement (cache fill included) and the measured epoch at each
    budget_sweep = None
    other = {"cfg3": (0.05, 0.20)}.get(wl.name, ())
    if other and not args.no_budget_sweep and args.budget is None:
        budget_sweep = {}
        for frac in other:
            bud = int(wl.budget_bytes(frac) * scale)
            brec = {"sample_ms": [], "gather_ms": [], "epoch_wall_ms": []}
            place_ms = []
            for timed in (False, True):
                torch.cuda.synchronize()
                e0, e1 = ev(), ev()
                e0.record()
                _, bhot = tier.tier_place(ctx, counts, bud, want_slot_map=False)
                with torch.cuda.stream(gs):
                    e1.record()
                epoch(brec if timed else None, e1)
                if timed:
                    place_ms.append(e0.elapsed_time(e1))
            bhits, blinks = epoch_stats(groups)
            brows = brec["rows"]
            bh = bhits / brows
            bd = blinks / (brows - bhits) if brows > bhits else 1.0
            bpeak = alg_bytes_row / (((1 + bh + (1 - bh) * (1 - bd)) * R + 8) / HBM_PEAK_GBPS + (1 - bh) * bd * R / LINK_PEAK_GBPS)
            bms = brec["gather_ms"][0]
            budget_sweep[f"{frac:.2f}"] = {
                "budget_bytes": bud, "n_hot": bhot, "hit_fraction": round(bh, 4),
                "place_ms": round(place_ms[0], 3), "epoch_wall_ms": round(brec["epoch_wall_ms"][0], 3),
                "gather_ms": round(bms, 3), "gather_GBps": round(brows * R / (bms * 1e-3) / 1e9, 2),
                "host_link_bytes_tiered": blinks * R, "host_link_reduction": round(1 - blinks / brows, 4),
                "roofline_frac": round(alg_bytes_row * brows / (bms * 1e-3) / 1e9 / bpeak, 4),
                "step_ms_with_this_budget": round((prefetch["presample_ms_without"] if prefetch else mean(rec["presample_ms"]))
                                                  + place_ms[0] + brec["epoch_wall_ms"][0], 3)}
            log(f"[bench] budget {frac}: {budget_sweep[f'{frac:.2f}']}")
        budget_sweep["note"] = ("same counts, other budgets: placement (order, slot map, cache fill over the host link, no rows "
                                "fetched ahead) and the measured epoch, timed as in the step; step_ms_with_this_budget = "
                                "presampling in one piece + these two; roofline_frac as roofline.frac")
        tier.tier_place(ctx, counts, budget, want_slot_map=False)
        torch.cuda.synchronize()

    # the two streams on their own: every row from HBM, then every row over the host link
    streams = None
    if not args.no_streams:
        streams = {}
        tier.tier_set_gather_dedup(ctx, False)         # every requested row really crosses the link here
        for name, bud in (("all_hit", n * R), ("all_miss", 0)):
            tier.tier_place(ctx, counts, bud, want_slot_map=False)
            ms = 0.0; nrows = 0; nl = 0
            for g in groups[:4]:
                blk = sample_group(g)
                a, b_, r = timed_gather(blk, len(g))
                torch.cuda.synchronize()
                ms += a.elapsed_time(b_); nrows += r; nl += 1
            if name == "all_hit":
                streams[name] = {"hbm_GBps": round(nrows * alg_bytes_row / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak":
                                 round(nrows * alg_bytes_row / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                 "avg_launch_ms": round(ms / nl, 4), "launches": nl}
            else:
                streams[name] = {"host_link_GBps": round(nrows * R / (ms * 1e-3) / 1e9, 2), "frac_of_link_peak":
                                 round(nrows * R / (ms * 1e-3) / 1e9 / LINK_PEAK_GBPS, 4),
                                 "avg_launch_ms": round(ms / nl, 4), "launches": nl}
        tier.tier_set_gather_dedup(ctx, shared_on)
        roofline["streams"] = streams
        # the same blend with the rates the two streams reach on their own instead of the published peaks
        t_row = ((h + (1 - h) * (1 - d)) * alg_bytes_row / (streams["all_hit"]["hbm_GBps"] * 1e9)
                 + (1 - h) * d * R / (streams["all_miss"]["host_link_GBps"] * 1e9))
        roofline["frac_of_measured_streams"] = round(t_row * rows / (gather_ms * 1e-3), 4) if gather_ms else None
        roofline["measured_streams_model"] = ("time per row = (h + (1-h)(1-d)) (2R+8) / all-hit rate + (1-h) d R / all-miss rate, over the "
                                              "measured time per row: above 1 when the hits hide under the misses")
        untiered_ms = rows * R / (streams["all_miss"]["host_link_GBps"] * 1e9) * 1e3
        roofline["untiered_epoch_gather_ms"] = round(untiered_ms, 2)
        roofline["gather_speedup_vs_untiered"] = round(untiered_ms / gather_ms, 2) if gather_ms else None

    scores = None
    # the same epoch gathered alone (no sampling beside it), plain and with shared misses
    shared = None
    if not args.no_streams:
        shared = {}
        tier.tier_presample(ctx, train, bs, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts)
        tier.tier_place(ctx, counts, budget, want_slot_map=False)
        for name, on in (("plain", False), ("shared_misses", True)):
            tier.tier_set_gather_dedup(ctx, on)
            for timed in (False, True):                 # first pass grows the staging area and counts, second times
                ms = 0.0; call_links = 0
                for g in groups:
                    blk = sample_group(g)
                    if timed:
                        a, b_, r = timed_gather(blk, len(g))
                        torch.cuda.synchronize()
                        ms += a.elapsed_time(b_)
                    else:
                        tier.tier_gather_minibatches(ctx, blk, len(g), out_buf[0], want_stats=True)
                        call_links += ctx.last_link_rows
                if not timed:
                    links = call_links
            shared[name] = {"gather_ms": round(ms, 3), "host_link_bytes": links * R,
                            "gathered_GBps": round(rows * R / (ms * 1e-3) / 1e9, 2) if ms else None}
        tier.tier_set_gather_dedup(ctx, shared_on)
        shared["note"] = ("one pass over the measured epoch, gathers only; shared_misses reads every distinct cold row "
                          "of a call over the host link once")

    out = out_buf[0]
    if not args.no_scores:
        scores = score_comparison(tier, synth, torch, ctx, wl, counts, train, budget, groups, sample_group, L)

    sweeps = None
    if args.sweeps:
        sweeps = run_sweeps(tier, synth, torch, ctx, wl, counts, train, n, R, groups, sample_group, L, log, timed_gather, gs)

    reorder = None
    if not args.no_reorder:
        reorder = reordered_variant(tier, synth, torch, ctx, wl, table, counts, train, budget, n, dtype, dev, log, args.link_blocks, shared_on, B)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(args, wl, indptr, indices, train, epoch_ids, table, budget, bseed)

    result = {
        "metric": "gathered feature GB/s (whole pass: presample + place + sampled and gathered epoch)",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"{wl.name}{'' if scale == 1.0 else f' at scale {scale:g}'}: {wl.graph} graph, {n} nodes, {indices.numel()} edges, "
                               f"{wl.dim} x {wl.dtype} features, fanout {list(wl.fanouts)}, batch {bs}, "
                               f"{n_batches} mini-batches per epoch sampled {B * per_sample} and gathered {B} per call, HBM budget {budget} B ({rec['n_hot']} rows)"},
        "sampled_edges_per_s": round(edges / (sample_alone_ms * 1e-3)) if sample_alone_ms else None,
        "sample_alone_ms": round(sample_alone_ms, 3),
        "gather_GBps": round(gathered_bytes / (gather_ms * 1e-3) / 1e9, 2) if gather_ms else None,
        "rows_per_epoch": rows, "edges_per_epoch": edges, "hit_fraction": round(h, 4),
        "host_link_bytes_tiered": link_rows * R, "host_link_bytes_untiered": rows * R,
        "host_link_reduction": round(1 - link_rows / rows, 4) if rows else None,
        "phase_note": "presample + place + epoch_wall = the step.  place = ordering, slot map (place_sort) and the cache "
                      "fill, which runs on the gather stream while the main stream already samples; epoch_wall counts from "
                      "the end of that fill to the end of the last gather.  sample and gather are per-stream busy times "
                      "inside the epoch (two streams, overlapping); sample_alone_ms is the same epoch's sampling with the "
                      "GPU to itself (basis of sampled_edges_per_s)",
        "phase_ms": {"presample": round(mean(rec["presample_ms"]), 3), "place": round(mean(rec["place_ms"]), 3),
                     "place_sort": round(mean(rec["place_sort_ms"]), 3),
                     "sample": round(sample_ms, 3), "gather": round(gather_ms, 3),
                     "epoch_wall": round(mean(rec["epoch_wall_ms"]), 3)},
        "budget_sweep": budget_sweep,
        "prefetch": prefetch,
        "gather_launch": {"link_blocks": args.link_blocks, "min_rows": SPLIT_MIN_ROWS, "shared_misses": shared_on,
                          "mini_batches_per_call": B, "mini_batches_per_sampling_call": B * per_sample,
                          "output_rows_held": rec["most_rows_per_call"],
                          "groups": group_table,
                          "note": "split launch: the first link_blocks blocks copy the cold rows (host link), all others the "
                                  "hot rows (HBM); uniform_launch_epoch is the same epoch with every block copying both",
                          "uniform_launch_epoch": uniform},
        "paper_context": "paper (2x Xeon 6230 + V100 32 GB, OGB datasets, DGL): 87-95 % less PCIe traffic with 10 % of the "
                         "features on the GPU and 1.6-2.1x faster training than zero-copy only; context, not a target",
        "roofline": roofline, "shared_misses": shared, "score_functions": scores, "sweeps": sweeps, "reordered": reorder, "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)
    ctx.close()


def score_comparison(tier, synth, torch, ctx, wl, counts, train, budget, groups, sample_group, L):
    """Hit fraction of the measured epoch when the same budget is filled by each score
    (the paper's Sec. 5.2 question: how well does a score predict the measured accesses),
    and the time each score takes.  Hits are counted from the slot map of each placement."""
    def timed(f):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()                    # e.g. a cache fill still running on the gather stream
        a.record(); r = f(); b.record(); torch.cuda.synchronize()
        return r, round(a.elapsed_time(b), 3)

    frontiers = []
    for g in groups:
        blk = sample_group(g)
        frontiers += [blk.frontier(i).clone() for i in range(len(g))]
    rows = sum(f.numel() for f in frontiers)
    none = train[:0]
    res = {}
    _, t = timed(lambda: tier.tier_presample(ctx, train, wl.batch_size, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts))
    makers = {
        "presampled_counts": (lambda: counts, t, "int"),
        # the other reading of the access count: every draw of a node and every seed counts
        "presampled_draw_counts": (lambda: tier.tier_presample_draws(ctx, train, wl.batch_size, wl.fanouts, 1,
                                                                      synth.PRESAMPLE_SEED), None, "int"),
        "out_degree": (lambda: tier.tier_score_degree(ctx), None, "int"),
        "reverse_pagerank_5": (lambda: tier.tier_score_wrpr(ctx, none, 5, 0.85), None, "real"),
        "weighted_reverse_pagerank_5": (lambda: tier.tier_score_wrpr(ctx, train, 5, 0.85), None, "real"),
    }
    for name, (make, t_known, kind) in makers.items():
        sc, t = timed(make)
        place = tier.tier_place if kind == "int" else tier.tier_place_scores
        slot, n_hot = place(ctx, sc, budget)
        hits = sum(int((slot[f.long()] >= 0).sum()) for f in frontiers)
        res[name] = {"score_ms": t_known if t_known is not None else t, "hit_fraction": round(hits / rows, 4)}
    tier.tier_presample(ctx, train, wl.batch_size, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts)
    tier.tier_place(ctx, counts, budget, want_slot_map=False)          # leave the context as the main run had it
    return res


def run_sweeps(tier, synth, torch, ctx, wl, counts, train, n, R, groups, sample_group, L, log, timed_gather, gs):
    """Harness-only analysis on the library's outputs.
    budget: hit fraction of the measured epoch against the share of rows kept in HBM, for placement by
    presampled counts and by weighted reverse PageRank, and for the placement by counts the measured
    time of the placement (cache fill included) and of the epoch's gathers (the paper's Fig. 6 sweeps
    the loaded share and plots PCIe traffic and time).
    depth: share of all measured accesses that falls on the top 10 % of nodes by score, for fanouts
    (10,10) .. (10,10,10,10,10) (the paper's Fig. 5), accesses measured by tier_presample with the
    measured epoch's seed over at most 64 mini-batches."""
    frontiers = []
    for g in groups:
        blk = sample_group(g)
        frontiers += [blk.frontier(i).clone() for i in range(len(g))]
    allf = torch.cat(frontiers).long()
    rows = allf.numel()
    tier.tier_presample(ctx, train, wl.batch_size, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts)
    rank_c, _ = tier.tier_rank(ctx, counts)
    wr = tier.tier_score_wrpr(ctx, train, 5, 0.85)
    rank_w, _ = tier.tier_rank_scores(ctx, wr)
    deg = tier.tier_score_degree(ctx)
    rank_d, _ = tier.tier_rank(ctx, deg)
    shares = [0.0, 0.01, 0.02, 0.05, 0.10, 0.15, 0.20, 0.25, 0.50, 1.0]
    budget = []
    for p in shares:
        n_hot = int(p * n)
        row = {"share_in_hbm": p}
        for name, rk in (("counts", rank_c), ("wrpr", rank_w), ("degree", rank_d)):
            h = float((rk[allf] < n_hot).sum()) / rows
            row[f"hit_{name}"] = round(h, 4)
        row["host_link_bytes_counts"] = int(round((1 - row["hit_counts"]) * rows)) * R
        # measured: placement by counts at this share, then the epoch's gathers (alone on the GPU)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        tier.tier_place(ctx, counts, n_hot * R, want_slot_map=False)
        with torch.cuda.stream(gs):
            e1.record()
        torch.cuda.synchronize()
        row["place_ms"] = round(e0.elapsed_time(e1), 3)
        ms = 0.0
        for g in groups:
            blk = sample_group(g)
            a, b_, _ = timed_gather(blk, len(g))
            torch.cuda.synchronize()
            ms += a.elapsed_time(b_)
        row["epoch_gather_ms"] = round(ms, 3)
        budget.append(row)
        log(f"[bench] budget sweep {p}: {row}")
    depth = []
    sub = train[: min(train.numel(), 64 * wl.batch_size)].contiguous()
    acc = torch.empty_like(counts)
    for d in range(2, 6):
        fan = (10,) * d
        _, tot_rows, _ = tier.tier_presample(ctx, sub, wl.batch_size, fan, 1, synth.EPOCH_SEED, acc, want_totals=True)
        a = acc.long()
        top = int(0.10 * n)
        row = {"fanouts": list(fan), "rows": tot_rows}
        for name, rk in (("wrpr", rank_w), ("degree", rank_d)):
            row[f"top10pct_share_{name}"] = round(float(a[rk < top].sum()) / max(tot_rows, 1), 4)
        depth.append(row)
        log(f"[bench] depth sweep {fan}: {row}")
    tier.tier_presample(ctx, train, wl.batch_size, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts)
    return {"budget": budget, "depth": depth}


def reordered_variant(tier, synth, torch, ctx, wl, table, counts, train, budget, n, dtype, dev, log, link_blocks, shared_on, group):
    """The paper's own layout (Sec. 3.2, Alg. 2): graph and table renamed by rank, hot part =
    ids below the boundary, gather without a map.  Times the reordering and one sampled and
    gathered epoch on the reordered data (its draws differ: they are keyed by node id)."""
    def timed(f):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()                    # e.g. a cache fill still running on the gather stream
        a.record(); r = f(); b.record(); torch.cuda.synchronize()
        return r, a.elapsed_time(b)

    res = {}
    tier.tier_presample(ctx, train, wl.batch_size, wl.fanouts, 1, synth.PRESAMPLE_SEED, counts)
    (rank, order), res["rank_ms"] = timed(lambda: tier.tier_rank(ctx, counts))
    (ip2, ix2), res["graph_ms"] = timed(lambda: tier.tier_reorder_graph(ctx, rank, order))
    try:
        table2 = tier.tier_host_alloc(n, wl.dim, dtype)
    except tier.TierError as e:
        res["note"] = f"no second pinned table of {table.nbytes / 2**30:.1f} GiB on this host ({e}): rows not reordered"
        log("[bench] " + res["note"])
        return {k: (round(v, 3) if isinstance(v, float) else v) for k, v in res.items()}
    try:
        _, res["rows_ms"] = timed(lambda: tier.tier_reorder_rows(ctx, rank, table2))
        train2 = tier.tier_relabel_ids(ctx, rank, train)
        ctx2 = tier.tier_create(ip2, ix2, table2)
        tier.tier_set_gather_split(ctx2, link_blocks, SPLIT_MIN_ROWS)
        tier.tier_set_gather_dedup(ctx2, shared_on)
        n_hot, res["place_boundary_ms"] = timed(lambda: tier.tier_place_boundary(ctx2, budget))
        bs = wl.batch_size; L = len(wl.fanouts)
        n_train = train2.numel(); n_batches = -(-n_train // bs)
        order_e = synth.random_order(n_train, synth.EPOCH_SEED, 1, dev)
        ep = train2[order_e].contiguous()
        B = min(group, tier.tier_max_batches(ctx2))
        blocks = tier.BlocksBatch(n, bs, wl.fanouts, B, dev)
        out = None
        rows = hits = links = 0; ms = 0.0; launches = 0
        for g0 in range(0, n_batches, B):
            g = list(range(g0, min(g0 + B, n_batches)))
            blk = tier.tier_sample_minibatches(ctx2, ep[g[0] * bs: min(n_train, (g[-1] + 1) * bs)], bs,
                                               [tier.tier_batch_seed(synth.EPOCH_SEED, 0, b) for b in g], wl.fanouts,
                                               blocks)
            r = sum(blk.n_nodes[i][L] for i in range(len(g)))
            if out is None or out.shape[0] < r:
                out = torch.empty((int(r * 1.2), wl.dim), dtype=dtype, device=dev)
            a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); tier.tier_gather_minibatches(ctx2, blk, len(g), out); b_.record()
            torch.cuda.synchronize()
            ms += a.elapsed_time(b_); launches += 1; rows += r
            hits += sum(int((blk.frontier(i) < n_hot).sum()) for i in range(len(g)))
            if shared_on:                           # cold rows that have to cross the link: the distinct ones of the call
                ids = torch.cat([blk.frontier(i) for i in range(len(g))])
                links += int(torch.unique(ids[ids >= n_hot]).numel())
        if not shared_on:
            links = rows - hits
        R = ctx2.row_bytes
        h = hits / rows if rows else 0.0
        d = links / (rows - hits) if rows > hits else 1.0
        res.update({"n_hot": n_hot, "rows_per_epoch": rows, "hit_fraction": round(h, 4),
                    "gather_ms": round(ms, 3), "gather_GBps": round(rows * R / (ms * 1e-3) / 1e9, 2) if ms else None,
                    "avg_launch_ms": round(ms / launches, 4) if launches else None})
        peak = (2 * R + 4) / (((1 + h + (1 - h) * (1 - d)) * R + 4) / HBM_PEAK_GBPS + (1 - h) * d * R / LINK_PEAK_GBPS)
        res["roofline_frac"] = round((2 * R + 4) * rows / (ms * 1e-3) / 1e9 / peak, 4) if ms else None
        ctx2.close()
    finally:
        table2.free()
    return {k: (round(v, 3) if isinstance(v, float) else v) for k, v in res.items()}


def cpu_baseline(args, wl, indptr, indices, train, epoch_ids, table, budget, bseed):
    """The oracle as it stands, on the host cores, on the first few mini-batches of
    the same workload: their presampling share, the placement (all nodes), then
    sampling and gathering them.  Threads run whole mini-batches side by side."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle import oracle as orc

    cores = len(os.sched_getaffinity(0))
    nb = max(1, args.cpu_batches)
    bs = wl.batch_size
    ip = indptr.cpu().numpy().astype(np.int64); ix = indices.cpu().numpy()
    tr = train.cpu().numpy(); ep = epoch_ids.cpu().numpy()
    n = ip.shape[0] - 1
    feat = table.tensor.view(-1).view(torch.uint8).numpy().reshape(n, -1)
    R = feat.shape[1]
    nb = min(nb, -(-len(tr) // bs))
    threads = min(cores, nb)
    t0 = time.perf_counter()
    counts, _, _ = orc.presample(ip, ix, tr[: nb * bs], bs, wl.fanouts, 1, synth_seed("pre"), threads=threads)
    _, slot, n_hot = orc.place(counts, R, budget)
    cache = orc.fill_cache(feat, slot, n_hot)

    def one(b):
        blk = orc.sample_minibatch(ip, ix, ep[b * bs:(b + 1) * bs], wl.fanouts, bseed[b])
        rows, _, _ = orc.gather(feat, cache, slot, blk["nodes"])
        return rows.shape[0]

    with ThreadPoolExecutor(threads) as ex:
        rows = sum(ex.map(one, range(nb)))
    dt = time.perf_counter() - t0
    # one thread: sample + gather of a sixteenth of those mini-batches (placement as above)
    nb1 = max(1, nb // 16)
    t1 = time.perf_counter()
    rows1 = sum(one(b) for b in range(nb1))
    dt1 = time.perf_counter() - t1
    t2 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        rows_sg = sum(ex.map(one, range(nb)))
    dt_sg = time.perf_counter() - t2
    return {"value": round(rows * R / dt / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nb} of the mini-batches: presample of {nb} batches, placement of all {n} nodes, "
                      f"then sample + gather of {nb} batches; {dt:.1f} s wall on {threads} threads",
            "seconds": round(dt, 2),
            "sample_gather_only": {"value": round(rows_sg * R / dt_sg / 1e9, 4), "cores": threads,
                                   "sample": f"sample + gather of the same {nb} mini-batches, {dt_sg:.1f} s"},
            "single_thread": {"value": round(rows1 * R / dt1 / 1e9, 4), "cores": 1,
                              "sample": f"sample + gather of the first {nb1} mini-batches, {dt1:.1f} s"}}


def measured_traffic(workload):
    """HBM bytes per gather launch measured with rocprofv3 counters (FETCH_SIZE and
    WRITE_SIZE runs of this script, scaled by a plain copy of known size); read from
    the committed summary of those runs, None when there is none for the workload."""
    path = os.path.join(ROOT, "profiles", f"gather_{workload}_hbm_traffic.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def synth_seed(which):
    from paper_2111_05894_amd import synth
    return synth.PRESAMPLE_SEED if which == "pre" else synth.EPOCH_SEED


if __name__ == "__main__":
    main()
