#!/usr/bin/env python3
"""Benchmark of the TAGC hot path on one MI355X.

One "step" is one pass of the whole hot path (sparsify + index, Index OR, sketch
encode, sketch sum, peeling decode) over one full synthetic gradient of the
workload: every bucket, every simulated rank.  Inputs are resident in HBM before
the timed region starts.  Prints ONE JSON line (the fields are described in README.md).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# Kernels of the library grouped into the stages of the path.
STAGES = {
    "S1+S2 sparsify+index": ["fill_zero", "accumulate", "prepare", "scan_spill", "hist1",
                             "hist2c", "hist2", "select2", "count", "place", "widen4"],
    "S3a index OR": ["index_or", "header", "bounds", "salt", "ranges"],
    "S2' encode": ["encode"],
    "S3b sketch sum": ["sketch_sum"],
    "S4 decode": ["enumerate", "peel", "dense"],
}
FUSED_STAGE = "S3b+S4 sketch sum inside decode"


def stages_of(fused):
    """Kernels per stage; with the fused call the last two stages are one."""
    if not fused:
        return STAGES
    st = {k: v for k, v in STAGES.items() if k not in ("S3b sketch sum", "S4 decode")}
    st[FUSED_STAGE] = ["enumerate", "sum_peel", "dense"]
    return st


def stage_phases(fused):
    """The calls (--only-phases names) that make up each stage."""
    st = {"S1+S2 sparsify+index": ["index"], "S3a index OR": ["agg_index"],
          "S2' encode": ["sketch"]}
    if fused:
        st[FUSED_STAGE] = ["decode"]
    else:
        st["S3b sketch sum"] = ["agg_sketch"]
        st["S4 decode"] = ["decode"]
    return st


def profile_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` as the tracked rocprofv3 counter summary of this
    workload has them (profiles/<workload>_all_kernels.txt, the table written from the
    --pmc FETCH_SIZE / WRITE_SIZE runs; its column scaled_total_MB is already calibrated).
    None when there is no such summary or it does not list the kernel."""
    path = os.path.join(ROOT, "profiles", "%s_all_kernels.txt" % workload)
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    in_table = False
    for line in lines:
        if line.startswith("kernel") and "scaled_total_MB" in line:
            in_table = True
            continue
        f = line.split()
        if in_table and len(f) == 5 and f[0] == kernel:
            return int(float(f[4]) * 1e6)
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="config5",
                    choices=["config1", "config2", "config3", "config4", "config5"])
    ap.add_argument("--pool", type=int, default=8,
                    help="distinct bucket data sets resident in HBM (buckets cycle through them)")
    ap.add_argument("--lf", type=int, default=0, help="load factor x1000 (0 = workload default)")
    ap.add_argument("--dense", type=int, default=1, help="also write the dense summed gradient")
    ap.add_argument("--buckets", type=int, default=0,
                    help="only the first B buckets of the workload (0 = all; for experiments)")
    ap.add_argument("--lanes", type=int, default=12,
                    help="buckets in flight at once: bucket i runs on HIP stream i %% lanes with "
                         "that lane's own buffers (buckets are independent of each other)")
    ap.add_argument("--decode-workgroups", type=int, default=-1,
                    help="with more than one bucket in flight: most workgroups of the peeling "
                         "kernel at once (it needs a compute unit's whole local memory, so "
                         "this leaves the other compute units to the other buckets' "
                         "bandwidth-bound kernels); 0 = one per compute unit; default: 96 "
                         "with the fused decoder, 64 without (what measured best)")
    ap.add_argument("--part-unknowns", type=int, default=0,
                    help="non-zeros per sketch partition (0 = library default)")
    ap.add_argument("--part-cells", type=int, default=0,
                    help="sketch cells per partition (0 = library default)")
    ap.add_argument("--error-feedback", action="store_true",
                    help="give every rank a gradient accumulator (Algorithm 1, lines 1-2): "
                         "adds one read and one write of the gradient's size per rank")
    ap.add_argument("--index-mode", type=int, default=0, choices=[0, 1, 2],
                    help="0 Index merged by OR (the headline), 1 by addition of the 1-bit "
                         "Index, 2 by addition of 4-bit counters (section 2.2)")
    ap.add_argument("--ranks", type=int, default=0,
                    help="simulated ranks (0 = the workload's)")
    ap.add_argument("--ratio", type=int, default=0,
                    help="fixed-ratio sketch, c x1000 (Table 1: cells = n / c); 0 = sized by "
                         "load factor")
    ap.add_argument("--keep-ppm", type=int, default=0,
                    help="survivors per million for every compressed segment (Table 1: "
                         "(1 - theta) * 10^6); 0 = the workload's dynamic ratios")
    ap.add_argument("--cell-bits", type=int, default=32, choices=[32, 16],
                    help="a rank's sketch cells on the wire: float32, or rounded to bfloat16 "
                         "(section 5: quantised communication)")
    ap.add_argument("--decode-mode", type=int, default=0, choices=[0, 1, 2],
                    help="0 peeling only (the headline), 1 peeling + estimation of what it "
                         "leaves, 2 estimation only (section 2.2's two decompression algorithms)")
    ap.add_argument("--fused-decode", type=int, default=1, choices=[0, 1],
                    help="1 (default): tagc_reduce_decompress, the decoder adds up the ranks' "
                         "sketches itself and the summed sketch is never written (float32 "
                         "cells, default partition size, up to 32 ranks: otherwise the two "
                         "calls are made); 0: tagc_aggregate(PHASE_SKETCH) then "
                         "tagc_decompress")
    ap.add_argument("--only-phases", default="",
                    help="measurement aid: comma list out of index,agg_index,sketch,agg_sketch,"
                         "decode; the timed steps make only these calls for every bucket, on the "
                         "buffers the warm-up steps (always the whole path) left; ms_per_step "
                         "then describes that subset, the byte-based fractions are null and no "
                         "per-kernel pass is made")
    ap.add_argument("--graph", type=int, default=1, choices=[0, 1],
                    help="1 (default): capture each bucket's call sequence in a HIP graph after "
                         "the warm-up and replay it in the timed steps (the library only enqueues "
                         "kernels, so a caller may do that), which keeps the result independent "
                         "of how fast the host issues launches; 0: issue every launch eagerly.  "
                         "Off with --error-feedback, whose steps take a different gradient each")
    ap.add_argument("--grad-sets", type=int, default=0,
                    help="distinct gradients per bucket data set, one per step in turn (0 = 3 "
                         "with --error-feedback, where feeding the same gradient every step "
                         "would double the accumulator's scale from step to step, else 1)")
    ap.add_argument("--arena-gb", type=int, default=-1,
                    help="allocate and release one block of this many GiB before anything else, "
                         "so that torch's caching allocator serves every buffer from one "
                         "device allocation (measured: the first process on a box is 2 %% faster "
                         "that way, later ones the same); -1 = three quarters of the free "
                         "memory, 0 = off")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibration-copy", type=int, default=0,
                    help="before the timed region, copy this many MiB device to device three "
                         "times (a kernel of known traffic to scale rocprof byte counters by)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    return ap.parse_args()


def make_buckets(args):
    from synth import gradients as G
    w = args.workload
    if w == "config1":
        bs = [G.config1(args.seed)]
    elif w == "config2":
        bs = G.config2(args.seed)
    elif w == "config3":
        bs = [G.config3(args.seed)]
    elif w == "config4":
        bs = G.config4(args.seed)
    else:
        bs = G.config5(args.seed)
    if args.buckets:
        bs = bs[:args.buckets]
    for b in bs:
        if args.lf:
            b.sizing_milli = args.lf
        if args.ratio:
            b.sizing_milli = args.ratio
        if args.ranks:
            b.n_ranks = args.ranks
        if args.keep_ppm:
            b.segments = [s._replace(keep_ppm=args.keep_ppm) if s.flags & 1 else s
                          for s in b.segments]
    return bs


def alg_bytes(b, z, hdr, k_total, dense, ef=False, wire=1, cell=4, fused=False):
    """Algorithmic bytes per stage for one bucket: one read of the gradient (with error
    feedback also one read and one write of the accumulator), every message
    materialised once; work-lists, histograms and degree tables are not credited.
    `fused`: the decoder sums the ranks' sketches itself, so the summed sketch is neither
    written nor read back and is not credited either."""
    N, e = b.n_ranks, b.elem_bytes
    n_c, U, m = z.n_c, hdr["U"], hdr["m"]
    passes = 3 if ef else 1
    out = {
        "S1+S2 sparsify+index": passes * N * z.n_real * e + 8 * k_total + wire * N * n_c // 8,
        "S3a index OR": wire * N * n_c // 8 + n_c // 8,
        "S2' encode": 8 * k_total + N * cell * m,
    }
    if fused:
        out[FUSED_STAGE] = N * cell * m + n_c // 8 + 8 * U + (4 * n_c if dense else 0)
    else:
        out["S3b sketch sum"] = (N * cell + 4) * m
        out["S4 decode"] = n_c // 8 + 4 * m + 8 * U + (4 * n_c if dense else 0)
    return out


def kernel_alg_bytes(b, z, hdr, k_total, dense, ef=False, wire=1, cell=4):
    """Bytes each bandwidth-relevant kernel must itself move per bucket (all its
    launches together).  hist1 and compact each read the gradient once, so their sum
    exceeds the stage's algorithmic bytes: the stage figure shows the cost of the
    second read, this one prices each kernel against what it has to touch."""
    N, e = b.n_ranks, b.elem_bytes
    n_c, U, m = z.n_c, hdr["U"], hdr["m"]
    return {
        "scan_spill": (3 if ef else 1) * N * z.n_real * e,
        "hist1": N * z.n_real * e,
        "hist2": N * z.n_real * e,
        # place = the candidate route's last pass + the dense route's (which reads the gradient
        # again); priced as the former, which is all it is for a bucket without dense-route
        # segments; count reads the candidate slots (about 1.3 x 4 bytes per pair)
        "place": 8 * k_total + N * n_c // 8,
        "count": int(1.3 * 4 * k_total),
        "index_or": (wire * N + 1) * n_c // 8,
        "widen4": (1 + 4) * N * n_c // 8,
        "encode": 8 * k_total + N * cell * m,
        "sketch_sum": (N * cell + 4) * m,
        "enumerate": n_c // 8 + 4 * U,
        "peel": 4 * m + 8 * U,
        "sum_peel": N * cell * m + 8 * U,
        "dense": n_c // 8 + 4 * U + 4 * n_c,
    }


def cpu_baseline(args):
    """The oracle, as it stands, timed on this machine's host cores on a bounded sample of the
    same workload: the first bucket whole (config5: all seven segments of block 0) for all
    its ranks, the per-rank steps spread over the host's threads."""
    from concurrent.futures import ThreadPoolExecutor
    import torch
    from oracle import tagc_oracle as O
    from synth import gradients as G
    b = make_buckets(args)[0]
    n_ranks = min(b.n_ranks, 16)
    gen = G.config3_rank_gradient if args.workload == "config3" else G.rank_gradient
    # generated on the device and copied over (faster than the host's generator; the
    # oracle's input is host memory either way)
    grads = [G.to_numpy_raw(gen(b, r, "cuda" if torch.cuda.is_available() else "cpu"))
             for r in range(n_ranks)]
    cfg = O.Config(dtype=b.dtype, sizing_milli=b.sizing_milli, seed=args.seed)
    segs = [O.Segment(s.offset, s.length, s.keep_ppm, s.flags) for s in b.segments]
    offs, n_c = O.c_offsets(segs)
    n_real = b.compressed_elems()
    threads = min(n_ranks, os.cpu_count() or 1, 16)
    O.lib()
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:   # ranks are independent until the OR
        ranks = list(ex.map(lambda g: O.sparsify(g, cfg, segs), grads))
    bitmap, U = O.index_or([r.bitmap for r in ranks])
    A, m_sub, m = O.layout(U, cfg, n_real)
    bnd = O.bounds(bitmap, n_c, U, A)
    salt = O.salts(bitmap, n_c, U, A, m_sub, cfg.seed)
    with ThreadPoolExecutor(threads) as ex:
        sks = list(ex.map(lambda r: O.encode(r.idx, r.val, bnd, A, m_sub, cfg.seed, salt=salt),
                          ranks))
    total = O.sketch_sum(sks)
    dec = O.peel(bitmap, n_c, U, A, m_sub, cfg.seed, total, salt=salt)
    dt = time.perf_counter() - t0
    nbytes = n_ranks * n_real * b.elem_bytes
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "%s whole (%d compressed segments, %d elements) x %d ranks, whole path, "
                      "%.1f s" % (b.name, sum(1 for s in segs if s.flags & 1), n_real,
                                  n_ranks, dt),
            "n_unresolved": dec.n_unresolved}


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (N simulated ranks are "
                         "summed locally); --gpus %d is not supported\n" % args.gpus)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible; libtagc has no CPU path\n")
        sys.exit(2)
    torch.cuda.set_device(0)
    from synth import gradients as G
    from paper_2504_05638_amd import binding as B
    from paper_2504_05638_amd.bucket import TagcBucket

    if args.error_feedback and args.workload == "config5" and not args.buckets:
        # every bucket's ranks keep an accumulator of the gradient's size: all 32 blocks x 16
        # ranks (207 GB) plus three gradient sets do not fit the device
        args.buckets, args.pool = 12, min(args.pool, 2)
        sys.stderr.write("bench.py: --error-feedback on config5 runs the first 12 buckets "
                         "(accumulators of all 32 do not fit beside the inputs)\n")
    if args.arena_gb < 0:
        args.arena_gb = int(torch.cuda.mem_get_info()[0] * 3 // 4) >> 30
    if args.arena_gb:
        try:
            arena = torch.empty(args.arena_gb << 30, dtype=torch.uint8, device="cuda")
            del arena
        except RuntimeError:   # no block of that size to be had: allocate piecemeal
            sys.stderr.write("bench.py: no single block of %d GiB, going on without it\n"
                             % args.arena_gb)
            args.arena_gb = 0
    buckets = make_buckets(args)
    n_b = len(buckets)
    pool = max(1, min(args.pool, n_b))
    N = buckets[0].n_ranks
    gen = G.config3_rank_gradient if args.workload == "config3" else G.rank_gradient

    # ---- inputs resident in HBM (pool of distinct bucket data sets)
    t0 = time.perf_counter()
    import dataclasses
    n_sets = args.grad_sets or (3 if args.error_feedback else 1)
    if n_sets > 1:
        args.graph = 0  # a captured graph reads the buffers it was captured with
    data_sets = [[[gen(dataclasses.replace(buckets[d], seed=buckets[d].seed + 7919 * v), r, "cuda")
                   for r in range(N)] for d in range(pool)] for v in range(n_sets)]
    data = data_sets[0]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t0

    # ---- one plan per bucket, device buffers shared (buckets run one after another)
    # (the first bucket allocates every buffer at the largest size any bucket needs)
    fields = {"sh_bitmap": "shared_bitmap_bytes", "sh_sketch": "shared_sketch_bytes",
              "sh_bounds": "shared_bounds_bytes", "sh_ws": "shared_workspace_bytes",
              "rank_ws": "rank_workspace_bytes", "idx": "rank_idx_bytes",
              "val": "rank_val_bytes", "cnt": "rank_cnt_bytes", "bitmap": "rank_bitmap_bytes",
              "sketch": "rank_sketch_bytes", "out_idx": "out_idx_bytes",
              "out_val": "out_val_bytes", "out_dense": "out_dense_bytes"}
    need = {k: 0 for k in fields}
    sizing = B.TAGC_SIZE_FIXED_RATIO if args.ratio else B.TAGC_SIZE_LOAD_FACTOR
    for b in buckets:
        cfg = B.tagc_config(dtype=b.dtype, n_ranks=N, n_hash=3, sizing=sizing,
                            sizing_milli=b.sizing_milli, index_mode=args.index_mode,
                            part_unknowns=args.part_unknowns, part_cells=args.part_cells,
                            seed=args.seed, decode_mode=args.decode_mode,
                            cell_type=int(args.cell_bits == 16))
        plan = B.tagc_plan(cfg, [tuple(s[:4]) for s in b.segments])
        z = B.tagc_plan_sizes(plan)
        for k, f in fields.items():
            need[k] = max(need[k], getattr(z, f))
        B.tagc_plan_destroy(plan)
    lanes = max(1, min(args.lanes, n_b))
    fused = bool(args.fused_decode) and args.cell_bits == 32 and N <= 32 and \
        args.part_unknowns <= 8192 and args.part_cells <= 12288
    if args.decode_workgroups < 0:
        args.decode_workgroups = 96 if fused else 64
    peel_wgs = args.decode_workgroups if lanes > 1 else 0
    tbs = []
    for i, b in enumerate(buckets):
        first = i < lanes  # a lane's first bucket owns the buffers the lane's others reuse
        tbs.append(TagcBucket(b.segments, b.dtype, N, sizing_milli=b.sizing_milli,
                              seed=args.seed, dense=bool(args.dense),
                              part_unknowns=args.part_unknowns, part_cells=args.part_cells,
                              error_feedback=args.error_feedback,
                              decode_mode=args.decode_mode, index_mode=args.index_mode,
                              sizing=sizing, cell_type=int(args.cell_bits == 16),
                              decode_workgroups=peel_wgs,
                              share=None if first else tbs[i % lanes],
                              min_bytes=need if first else None))
    stream = torch.cuda.current_stream()
    streams = [stream] + [torch.cuda.Stream() for _ in range(lanes - 1)]
    phases = [p for p in args.only_phases.split(",") if p]
    unknown = set(phases) - {"index", "agg_index", "sketch", "agg_sketch", "decode"}
    if unknown:
        sys.stderr.write("bench.py: unknown phase(s) %s\n" % ", ".join(sorted(unknown)))
        sys.exit(2)
    if phases:
        args.no_profile_pass = True

    def run_subset(tb, grads, s=None, phases=phases):
        """The calls of one bucket that --only-phases (or `phases`) names."""
        if "index" in phases:
            for r in range(N):
                tb.compress_index(r, grads[r], s)
        if "agg_index" in phases:
            tb.aggregate_index(N, s)
        if "sketch" in phases:
            for r in range(N):
                tb.compress_sketch(r, s)
        if fused and "decode" in phases:
            tb.reduce_decompress(N, s)
        else:
            if "agg_sketch" in phases:
                tb.aggregate_sketch(N, s)
            if "decode" in phases:
                tb.decompress(s)

    step_no = [0]

    def step(one_stream=False):
        cur = data_sets[step_no[0] % n_sets]  # every step a different gradient, in turn
        step_no[0] += 1
        for i in range(n_b):
            tbs[i].run(cur[i % pool], stream if one_stream else streams[i % lanes],
                       whole_device_decode=one_stream, fused=fused)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.ones(args.calibration_copy << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- per-bucket facts (U, m, pairs) for the byte accounting, from one more pass
    input_bytes = 0
    balg = {k: 0 for k in stages_of(fused)}
    kalg = {}
    unresolved = estimated = rounds = 0
    wire = 4 if args.index_mode == B.TAGC_INDEX_ADD4 else 1
    cell = args.cell_bits // 8
    U_tot = m_tot = k_tot = 0
    flags = 0
    facts = []
    for i in range(n_b):
        tbs[i].run(data[i % pool], stream, fused=fused)
        torch.cuda.synchronize()
        hdr, st = tbs[i].header(), tbs[i].status()
        facts.append((hdr, st))
        kt = sum(tbs[i].rank_counts(r)["total"] for r in range(N))
        flags |= st["flags"]
        for r in range(N):
            flags |= tbs[i].rank_counts(r)["flags"]
        for k, v in alg_bytes(buckets[i], tbs[i].sizes, hdr, kt, args.dense, args.error_feedback, wire, cell, fused).items():
            balg[k] += v
        for k, v in kernel_alg_bytes(buckets[i], tbs[i].sizes, hdr, kt, args.dense, args.error_feedback, wire, cell).items():
            kalg[k] = kalg.get(k, 0) + v
        input_bytes += N * tbs[i].sizes.n_real * buckets[i].elem_bytes
        unresolved += st["n_unresolved"]
        estimated += st["n_estimated"]
        rounds = max(rounds, st["rounds"])
        U_tot += hdr["U"]
        m_tot += hdr["m"]
        k_tot += kt
    if flags:
        sys.stderr.write("bench.py: library reported error flags %d\n" % flags)
        sys.exit(1)

    if args.graph:
        graphs = []
        capture_stream = torch.cuda.Stream()   # capture needs a non-default stream
        for i in range(n_b):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=capture_stream):
                if phases:
                    run_subset(tbs[i], data[i % pool])
                else:
                    tbs[i].run(data[i % pool], fused=fused)
            graphs.append(g)
        torch.cuda.synchronize()

        def step(one_stream=False):  # noqa: F811 -- the timed steps replay the graphs
            if one_stream:
                for i in range(n_b):
                    tbs[i].run(data[i % pool], stream, whole_device_decode=True, fused=fused)
                return
            for i in range(n_b):
                with torch.cuda.stream(streams[i % lanes]):
                    graphs[i].replay()
        step()
        torch.cuda.synchronize()

    if phases and not args.graph:
        def step(one_stream=False):  # noqa: F811 -- the timed steps make the named calls only
            for i in range(n_b):
                run_subset(tbs[i], data[i % pool], streams[i % lanes])

    # ---- timed region: exactly K steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    t_steps = []
    for _ in range(args.steps):
        t1 = time.perf_counter()
        step()
        t_steps.append(time.perf_counter() - t1)
    t_issue = time.perf_counter() - t0   # the host has enqueued everything
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    # What enqueueing one step costs the host: the median over the steps.  Once the device's
    # queues are full (some twenty steps of graph launches ahead) a launch call blocks until
    # the device has caught up, so the total over many steps measures the device again.
    t_issue_step = sorted(t_steps)[len(t_steps) // 2]
    ms_per_step = 1e3 * t_total / args.steps
    # the buffers now hold each lane's last bucket: it must have come out as it did alone
    for i in range(n_b - lanes, n_b):
        hdr, st = tbs[i].header(), tbs[i].status()
        bad = st["flags"]
        for r in range(N):
            bad |= tbs[i].rank_counts(r)["flags"]
        # (with error feedback every pass starts from different accumulators, so U and the
        # residue legitimately change from pass to pass: only the flags are checked then)
        if phases:
            continue  # a subset of the calls leaves the buffers in between
        if bad or (not args.error_feedback and n_sets == 1 and (hdr, st) != facts[i]):
            sys.stderr.write("bench.py: bucket %d differs when run with %d buckets in flight "
                             "(flags %d)\n" % (i, lanes, bad))
            sys.exit(1)
    value = input_bytes / (ms_per_step * 1e-3) / 1e9
    balg_total = sum(balg.values())

    # ---- same K steps again with the library's per-kernel HIP events switched on, one
    # bucket at a time on one stream: a kernel's duration is then its own, not that of
    # whatever shared the device with it
    stages, roofline = {}, None
    if not args.no_profile_pass:
        B.tagc_profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(one_stream=True)
        torch.cuda.synchronize()
        t_prof = time.perf_counter() - t0
        prof = B.tagc_profile_read(64)
        B.tagc_profile_enable(False)
        for sname, kernels in stages_of(fused).items():
            ms = sum(prof[k][0] for k in kernels if k in prof) / args.steps
            stages[sname] = {
                "ms_per_step": round(ms, 4),
                "gradient_GBps": round(input_bytes / (ms * 1e-3) / 1e9, 1) if ms else None,
                "alg_bytes": balg[sname],
                "hbm_frac": round(balg[sname] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if ms else None,
            }
        dom = max(prof, key=lambda k: prof[k][0])
        d_ms, d_n = prof[dom]
        avg_ms = d_ms / d_n
        # algorithmic bytes per launch of the dominant kernel (one launch = one rank of
        # one bucket for per-rank kernels, one bucket for aggregation / decode),
        # averaged over the launches of the timed steps
        per_launch = kalg.get(dom, 0) * args.steps / d_n
        achieved = per_launch / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4),
                    # HBM bytes per launch, from the tracked counter runs of this workload
                    "traffic": profile_traffic(args.workload, dom),
                    "traffic_source": "profiles/%s_all_kernels.txt" % args.workload,
                    "avg_launch_ms": round(avg_ms, 5), "launches": d_n,
                    "alg_bytes_per_launch": int(per_launch),
                    "events_pass": "same steps, one bucket in flight (so decode on the whole "
                                   "device), HIP events around every kernel on its stream",
                    "events_pass_ms_per_step": round(1e3 * t_prof / args.steps, 3),
                    "kernels_ms_per_step": {k: round(v[0] / args.steps, 4)
                                            for k, v in sorted(prof.items(),
                                                               key=lambda kv: -kv[1][0])}}

    # ---- every stage on its own in the launch configuration of the timed region (graphs
    # replayed, `lanes` buckets in flight): the calls of that stage only, for every bucket, on
    # the buffers the complete steps left.  The events pass above times kernels one bucket at
    # a time, which leaves every launch's ramp-up and tail exposed; this is what a stage costs
    # when other buckets' launches of the same kind fill them.
    stages_in_flight = {}
    if stages and args.graph and not phases:
        k_steps = min(args.steps, 10)
        for sname, which in stage_phases(fused).items():
            gs = []
            for i in range(n_b):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=capture_stream):
                    run_subset(tbs[i], data[i % pool], phases=which)
                gs.append(g)
            torch.cuda.synchronize()
            for timed in (False, True):   # one untimed pass first
                t0 = time.perf_counter()
                for _ in range(k_steps if timed else 1):
                    for i in range(n_b):
                        with torch.cuda.stream(streams[i % lanes]):
                            gs[i].replay()
                torch.cuda.synchronize()
                ms = 1e3 * (time.perf_counter() - t0) / k_steps
            stages_in_flight[sname] = {
                "ms_per_step": round(ms, 4),
                "hbm_frac": round(balg[sname] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            del gs
    # `stages`: per stage, the time in the timed region's launch configuration where that was
    # measured (it is what adds up to ms_per_step), with the one-bucket-at-a-time figures of
    # the events pass beside it; otherwise the events pass alone
    for sname, st in stages.items():
        if sname in stages_in_flight:
            fl = stages_in_flight[sname]
            st["one_bucket_at_a_time"] = {"ms_per_step": st["ms_per_step"],
                                          "hbm_frac": st["hbm_frac"]}
            st["ms_per_step"], st["hbm_frac"] = fl["ms_per_step"], fl["hbm_frac"]
            st["gradient_GBps"] = round(input_bytes / (fl["ms_per_step"] * 1e-3) / 1e9, 1)
            st["measured"] = "%d buckets in flight, this stage's calls only" % lanes
        else:
            st["measured"] = "one bucket at a time, HIP events around every kernel"

    out = {
        "metric": "gradient GB/s compressed+aggregated+decoded on 1 MI355X; % of HBM peak",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d buckets x %d simulated ranks, %s grads, %s %.1f, %s"
                               % (args.workload + (" + error feedback" if args.error_feedback
                                                   else ""), n_b, N,
                                  "bf16" if buckets[0].dtype == G.BF16 else "fp32",
                                  "fixed ratio" if args.ratio else "lf",
                                  buckets[0].sizing_milli / 1000.0,
                                  "sparse+dense output" if args.dense else "sparse output"),
                   "input_bytes_per_step": input_bytes, "distinct_bucket_data_sets": pool,
                   "buckets_in_flight": lanes, "decode_workgroups": peel_wgs,
                   "host_issue_ms_per_step": round(1e3 * t_issue_step, 3),
                   "host_issue_total_ms_per_step": round(1e3 * t_issue / args.steps, 3),
                   "pairs_per_step": k_tot, "union_nonzeros_per_step": U_tot,
                   "sketch_cells_per_step": m_tot, "n_unresolved": unresolved,
                   "n_estimated": estimated, "decode_mode": args.decode_mode,
                   "fused_decode": fused,
                   "only_phases": phases or None,
                   "index_mode": args.index_mode, "cell_bits": args.cell_bits,
                   "graph_replay": bool(args.graph), "gradient_sets": n_sets,
                   "peel_rounds_max": rounds, "input_generation_s": round(t_gen, 2)},
        "hbm_frac_end_to_end": None if phases else round(
            balg_total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "alg_bytes_per_step": balg_total,
        "stages": stages,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
