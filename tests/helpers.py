"""Shared test plumbing: feeds the same seeded inputs to the oracle and to the
HIP library and compares them stage by stage.  Holds no method arithmetic."""
from __future__ import annotations

import numpy as np

from oracle import tagc_oracle as O
from synth import gradients as G


def oracle_segments(bucket):
    return [O.Segment(s.offset, s.length, s.keep_ppm, s.flags) for s in bucket.segments]


def oracle_config(bucket, sizing=O.SIZE_LOAD_FACTOR, seed=0, P=8192, T=12288, index_mode=0,
                  cell_type=0):
    return O.Config(dtype=bucket.dtype, sizing=sizing, sizing_milli=bucket.sizing_milli,
                    seed=seed, part_unknowns=P, part_cells=T, index_mode=index_mode,
                    cell_type=cell_type)


def segment_of(c_index, bucket):
    """compressed-segment ordinal of each c-index."""
    offs, _ = O.c_offsets(oracle_segments(bucket))
    starts = np.array([o for o in offs if o is not None], np.int64)
    return np.searchsorted(starts, np.asarray(c_index, np.int64), side="right") - 1


def value_tolerance(ores, rel=1e-5):
    """|delta| allowed per decoded entry: rel * max(|ref_i|, V_i), V_i being the
    largest decoded magnitude inside entry i's sketch partition.  A decoded value is
    a float32 cell minus the other values sharing that cell, along a peeling chain
    that stays inside one partition; with a different summation order each step may
    differ by one float32 rounding (6e-8) of the largest value involved, so the
    difference is bounded relative to the partition's scale, not to the entry itself
    (an entry that cancels across ranks may be far smaller than its terms)."""
    idx = ores.decoded.idx
    ref = np.abs(ores.decoded.val.astype(np.float64))
    if idx.size == 0:
        return ref
    part = np.searchsorted(ores.bnd[1:ores.A], idx, side="right")
    vmax = np.zeros(ores.A)
    np.maximum.at(vmax, part, ref)
    return rel * np.maximum(ref, vmax[part])


def segment_floor(bucket, ores):
    """tau_l per compressed segment: the smallest magnitude any rank selected in it.  Every
    contribution to a decoded entry of the segment is at least that large, so it is the
    natural floor of a relative tolerance for entries that cancel across ranks."""
    n_seg = sum(1 for s in bucket.segments if s.flags & 1)
    tau = np.full(n_seg, np.inf)
    for r in ores.ranks:
        if r.idx.size:
            np.minimum.at(tau, segment_of(r.idx, bucket), np.abs(r.val.astype(np.float64)))
    return tau


# Decoded float32 values are held to the stated bound first: |delta| <= 1e-5 * max(|ref|,
# tau_l).  An entry may exceed it only by having been mixed, in its cells and along its
# peeling chain, with entries far larger than itself (each float32 subtraction there rounds
# by 6e-8 of the larger operand): it must then be small against its partition's largest
# value, stay within 1e-5 of that scale, and such entries must be few.
MIXED_SMALL = 0.1          # an excepted entry is below this fraction of its partition's scale
MIXED_CEILING = 5e-3       # and at most this fraction of a bucket's decoded entries is excepted
excepted_log = []          # (what, excepted, total) of every comparison, for the record


def check_decoded_values(what, val, ref, strict, loose, ceiling=MIXED_CEILING):
    """`strict`, `loose`: per-entry absolute bounds (stated / partition-scale)."""
    err = np.abs(np.asarray(val, np.float64) - np.asarray(ref, np.float64))
    over = err > strict
    n_over = int(np.count_nonzero(over))
    excepted_log.append((what, n_over, int(err.size)))
    if n_over:
        print("[tolerance] %s: %d of %d decoded entries beyond 1e-5*max(|ref|, tau)"
              % (what, n_over, err.size), flush=True)
        assert np.all(err[over] <= loose[over]), "worst excess %g" % (err - loose)[over].max()
        # loose = rel * max(|ref|, partition scale): the entry is small against that scale
        assert np.all(np.abs(np.asarray(ref, np.float64))[over] * 1e-5 <= MIXED_SMALL * loose[over])
        assert n_over <= max(2, ceiling * err.size), (n_over, err.size)
    return n_over


def estimate_tolerance(ores, seed, rel=1e-5):
    """Tolerance for estimated entries: an estimate is a cell reading, and a cell is the
    outcome of float32 adds (encode, aggregation) and subtracts (peeling) of everything
    that was ever in it; in another order each of them rounds differently by at most
    6e-8 of a partial sum, which the cell's total magnitude bounds.  An entry's tolerance
    is `rel` times the largest such total among its three cells."""
    mag = np.zeros(max(ores.m, 1), np.float64)
    for r in ores.ranks:
        mag[:ores.m] += O.encode(r.idx, np.abs(r.val), ores.bnd, ores.A, ores.m_sub, seed,
                                 plus_only=True, salt=ores.salt).astype(np.float64)
    U = ores.U
    tol = np.zeros(U)
    part = (np.arange(U, dtype=np.int64) * 0)
    if ores.A:
        starts = np.array([a * U // ores.A for a in range(ores.A)], np.int64)
        part = np.searchsorted(starts, np.arange(U), side="right") - 1
    for t in np.flatnonzero(ores.decoded.round == 0):
        i = int(ores.decoded.idx[t])
        tol[t] = rel * max(
            mag[(int(part[t]) * 3 + j) * ores.m_sub
                + O.hash_slot(i, seed, j, ores.m_sub, int(ores.salt[part[t]]))[0]]
            for j in range(3))
    return tol


def run_both(bucket, grads_torch_cpu, seed=0, P=0, T=0, sizing=O.SIZE_LOAD_FACTOR, dense=True,
             decode_mode=0, index_mode=0, cell_type=0, decode_workgroups=0, fused=False):
    """Runs oracle and library on the same inputs; returns (oracle result, TagcBucket).
    `fused`: the library sums the sketches inside the decoder (tagc_reduce_decompress)."""
    import torch
    from paper_2504_05638_amd.bucket import TagcBucket

    ocfg = oracle_config(bucket, sizing, seed, P or 8192, T or 12288, index_mode, cell_type)
    ores = O.run_bucket([G.to_numpy_raw(g) for g in grads_torch_cpu], ocfg,
                        oracle_segments(bucket), decode_mode=decode_mode)
    tb = TagcBucket(bucket.segments, bucket.dtype, len(grads_torch_cpu),
                    sizing_milli=bucket.sizing_milli, sizing=sizing, seed=seed,
                    part_unknowns=P, part_cells=T, dense=dense, decode_mode=decode_mode,
                    index_mode=index_mode, cell_type=cell_type,
                    decode_workgroups=decode_workgroups)
    dev = [g.cuda() for g in grads_torch_cpu]
    tb.run(dev, fused=fused)
    torch.cuda.synchronize()
    return ores, tb


def compare_all(bucket, ores, tb, exact_values=False, rel=1e-5, mixed_ceiling=MIXED_CEILING):
    """Stage-by-stage comparison; integer work bit-exact, floats within tolerance
    (bit-exact too when `exact_values`).  `mixed_ceiling`: largest fraction of the decoded
    entries that may exceed the stated bound for having been mixed with far larger ones
    (inputs that plant values hundreds of times above the rest raise it)."""
    n_ranks = len(ores.ranks)
    z = tb.sizes
    assert z.n_c == ores.n_c
    # --- stage 1: survivors and local Index
    for r in range(n_ranks):
        cnt = tb.rank_counts(r)
        assert cnt["flags"] == 0 and cnt["nonfinite"] == 0
        assert cnt["total"] == ores.ranks[r].cnt
        comp_cnt = [c for c, s in zip(ores.ranks[r].seg_cnt, bucket.segments) if s.flags & 1]
        assert cnt["seg"] == comp_cnt
        idx, val = tb.rank_pairs(r)
        assert np.array_equal(idx, ores.ranks[r].idx)
        assert np.array_equal(val.view(np.uint32), ores.ranks[r].val.view(np.uint32))
        local = ores.ranks[r].bitmap[:z.bitmap_words]
        assert np.array_equal(tb.rank_bitmap(r), O.index_widen4(local)
                              if tb.cfg.index_mode == O.INDEX_ADD4 else local)
    # --- stage 3a: merged Index, layout, bounds
    hdr = tb.header()
    assert hdr == dict(U=ores.U, A=ores.A, m_sub=ores.m_sub, m=ores.m)
    assert np.array_equal(tb.shared_bitmap(), ores.bitmap[:z.bitmap_words])
    if ores.A:
        assert np.array_equal(tb.bounds(), ores.bnd)
        assert np.array_equal(tb.salts(), ores.salt)
    # --- stage 2': sketches.  A cell is a float32 sum of signed values; with a different
    # order each add may round differently, by at most 6e-8 of the largest partial sum,
    # which the sum of the magnitudes in the cell bounds.
    for r in range(n_ranks):
        got, want = tb.rank_sketch(r), ores.ranks[r].sketch
        if exact_values:
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        elif tb.cfg.cell_type:
            # 16-bit wire cells: the float32 cell behind it may differ in its last bits with
            # the order of the adds, which now and then tips the rounding to the neighbouring
            # bfloat16 (one unit in the 8th significant bit)
            d = np.abs(got.astype(np.float64) - want)
            assert np.all(d <= 2.0 ** -7 * np.abs(want) + 1e-37)
            assert got.size == 0 or np.mean(got.view(np.uint32) == want.view(np.uint32)) > 0.995
        else:
            mag = O.encode(ores.ranks[r].idx, np.abs(ores.ranks[r].val), ores.bnd, ores.A,
                           ores.m_sub, tb.cfg.seed, plus_only=True,
                           mask=ores.bitmap if tb.cfg.index_mode else None, salt=ores.salt)
            assert np.all(np.abs(got.astype(np.float64) - want) <= rel * mag.astype(np.float64))
            # cells with at most two contributions do not depend on the order
            assert got.size == 0 or np.mean(got.view(np.uint32) == want.view(np.uint32)) > 0.8
    # --- stage 4: decoded gradient
    st = tb.status()
    assert st["flags"] == 0
    assert st["n_unresolved"] == ores.decoded.n_unresolved
    assert st["rounds"] == ores.decoded.rounds
    idx, val = tb.outputs()
    assert np.array_equal(idx, ores.decoded.idx)
    unresolved = ores.decoded.round == 0
    mode = tb.cfg.decode_mode
    assert st["n_estimated"] == (ores.decoded.n_unresolved if mode else 0)
    if mode == 0:
        assert np.all(val[unresolved] == 0)
    if exact_values:
        # equal as numbers: an entry that cancels to zero across ranks may come out as +0
        # or -0 depending on which of its clean cells (and so which hash sign) supplied it
        assert np.array_equal(val, ores.decoded.val)
    elif mode == 0 and not tb.cfg.cell_type:
        ref = ores.decoded.val.astype(np.float64)
        tau = segment_floor(bucket, ores)
        strict = rel * np.maximum(np.abs(ref), tau[segment_of(idx, bucket)]) if idx.size else ref
        check_decoded_values(bucket.name, val, ref, strict, value_tolerance(ores, rel),
                             mixed_ceiling)
    else:
        tol = value_tolerance(ores, rel)
        if tb.cfg.cell_type:
            # a wire cell that rounded the other way moves what was decoded through it by one
            # bfloat16 unit of the cell; rare (checked above), but it has to be allowed for
            loose = value_tolerance(ores, 2.0 ** -6)
            err_q = np.abs(val.astype(np.float64) - ores.decoded.val.astype(np.float64))
            assert np.all(err_q <= loose) and np.mean(err_q <= tol) > 0.97
            tol = loose
        if mode and unresolved.any():
            tol[unresolved] = estimate_tolerance(ores, tb.cfg.seed, rel)[unresolved]
        err = np.abs(val.astype(np.float64) - ores.decoded.val.astype(np.float64))
        assert np.all(err <= tol), "worst excess %g at %d" % (
            (err - tol).max(), int(np.argmax(err - tol)))
    if tb.out_dense is not None:
        dense = tb.dense()
        want = np.zeros(z.n_c, np.float32)
        want[idx] = val
        assert np.array_equal(dense.view(np.uint32), want.view(np.uint32))
    return hdr, st
