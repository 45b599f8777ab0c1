"""GPU parity at the workloads' full sizes: one 7B-shaped bucket of the benchmark (config5,
block 0: 202 M bf16 entries x 16 ranks, load factor 1.5, default partitions, dense output),
run exactly as bench.py runs it; one bucket of the sharded 7B workload (config4); the 64 M
heavy-tailed bucket with half-shared supports (config3) at two of its (keep, load factor)
points, one of which takes the two-read route.  The oracle cannot redo all of it in test
time, so: sampled (rank, segment)
pairs go through the oracle's sparsifier bit for bit; one rank's whole sketch and a slice of
the summed one go through the oracle's encode and sum; the cheap stages (Index merge, layout,
bounds) are redone in full; everything else is checked through what must hold at any size --
counts, order, Index <-> pairs, the magnitude rule, and the decoded values against the
definition of the result, the per-index sum of what the ranks sent."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import oracle_segments

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[fullsize] " + msg, flush=True)


def _check_full_size(b, data, seed=0, oracle_ranks=(0,), max_unresolved=20,
                     decode_workgroups=0):
    from paper_2504_05638_amd.bucket import TagcBucket
    N = b.n_ranks
    bf16 = b.dtype == G.BF16
    segs = [s for s in b.segments if s.flags & 1]
    offs, n_c = O.c_offsets(oracle_segments(b))
    c_off = [o for o, s in zip(offs, b.segments) if s.flags & 1]
    k = [O.keep_count(s.length, s.keep_ppm) for s in segs]
    tb = TagcBucket(b.segments, b.dtype, N, sizing_milli=b.sizing_milli, seed=seed, dense=True,
                    decode_workgroups=decode_workgroups)
    tb.run(data)
    torch.cuda.synchronize()
    z = tb.sizes
    assert z.n_c == n_c
    _say("library done")

    # ---- stage 1, every rank: counts, order, flags
    pairs = []
    for r in range(N):
        cnt = tb.rank_counts(r)
        assert cnt["flags"] == 0 and cnt["nonfinite"] == 0
        assert cnt["seg"] == k and cnt["total"] == sum(k)       # enough non-zeros everywhere
        idx, val = tb.rank_pairs(r)
        assert idx.size == sum(k) and np.all(np.diff(idx.astype(np.int64)) > 0)
        pairs.append((idx, val))
    _say("counts and order of all ranks")

    # ---- stage 1, sampled ranks: Index <-> pairs, values, and the selection rule, which
    # with the count fixes the kept set: nothing left out is larger than anything kept, of
    # the entries that tie with the smallest kept one the lowest positions are kept, zeros
    # never.  Sampled segments (largest, smallest, one in between) also through the oracle.
    by_len = sorted(range(len(segs)), key=lambda l: segs[l].length)
    sampled_segs = {by_len[0], by_len[len(by_len) // 2], by_len[-1]}
    for r in sorted({0, N // 2 + 1} | set(oracle_ranks)):
        idx, val = pairs[r]
        bits = np.zeros(n_c, bool)
        bits[idx] = True
        assert np.array_equal(np.packbits(bits, bitorder="little").view(np.uint32),
                              tb.rank_bitmap(r))
        del bits
        raw = G.to_numpy_raw(data[r])          # bf16 bit patterns, or float32
        pos = 0
        for l, s in enumerate(segs):
            i_l = idx[pos:pos + k[l]].astype(np.int64) - c_off[l]
            v_l = val[pos:pos + k[l]]
            pos += k[l]
            assert i_l.min() >= 0 and i_l.max() < s.length
            seg_raw = raw[s.offset:s.offset + s.length]
            wide = (seg_raw.astype(np.uint32) << 16) if bf16 else seg_raw.view(np.uint32)
            assert np.array_equal(v_l.view(np.uint32), wide[i_l])        # the entries themselves
            key = wide & 0x7FFFFFFF
            T = key[i_l].min()
            assert T > 0
            tie_pos = np.flatnonzero(key == T)
            kept_ties = np.isin(tie_pos, i_l, assume_unique=True)
            assert kept_ties[0] and not np.any(np.diff(kept_ties.astype(np.int8)) > 0)
            key[i_l] = 0
            assert key.max() <= T
            del key
            if l in sampled_segs and r in oracle_ranks:
                one = [O.Segment(0, s.length, s.keep_ppm, 1)]
                st = O.sparsify(np.ascontiguousarray(seg_raw), O.Config(dtype=b.dtype), one)
                assert np.array_equal(st.idx.astype(np.int64), i_l)
                assert np.array_equal(st.val.view(np.uint32), v_l.view(np.uint32))
        del raw
        _say("rank %d against its gradient%s" % (r, " and the oracle" if r in oracle_ranks else ""))

    # ---- stage 3a in full: merged Index, U, layout, bounds
    maps = [tb.rank_bitmap(r) for r in range(N)]
    merged, U = O.index_or(maps)
    assert np.array_equal(tb.shared_bitmap(), merged)
    hdr = tb.header()
    cfg = O.Config(dtype=b.dtype, sizing_milli=b.sizing_milli, seed=seed)
    A, m_sub, m = O.layout(U, cfg, z.n_real)
    assert hdr == dict(U=U, A=A, m_sub=m_sub, m=m)
    bnd = O.bounds(merged, n_c, U, A)
    assert np.array_equal(tb.bounds(), bnd)
    _say("Index merge, layout, bounds: U=%d A=%d m=%d" % (U, A, m))

    # ---- stage 2': one rank's whole sketch through the oracle's encode
    r = N // 3
    want = O.encode(pairs[r][0], pairs[r][1], bnd, A, m_sub, seed)
    mag = O.encode(pairs[r][0], np.abs(pairs[r][1]), bnd, A, m_sub, seed, plus_only=True)
    got = tb.rank_sketch(r)
    assert np.all(np.abs(got.astype(np.float64) - want) <= 1e-5 * mag.astype(np.float64))
    assert np.mean(got.view(np.uint32) == want.view(np.uint32)) > 0.99
    del want, mag, got
    _say("rank %d sketch" % r)

    # ---- stage 3b: a slice of the summed sketch (the ranks' sketches are still on the device)
    c0 = m // 3
    c1 = min(m, c0 + (1 << 20))
    parts = [tb.rank_sketch(q)[c0:c1].copy() for q in range(N)]
    want = O.sketch_sum(parts)
    got = tb.shared_sketch()[c0:c1]
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))     # same order, same bits
    _say("summed sketch slice")

    # ---- stage 4 against the definition: per index, the sum of what the ranks sent
    ref = np.zeros(n_c, np.float64)
    big = np.zeros(n_c, np.float64)
    for idx, val in pairs:
        ref[idx] += val                  # a rank's indices are distinct: plain fancy add is exact
        big[idx] = np.maximum(big[idx], np.abs(val))
    st = tb.status()
    out_idx, out_val = tb.outputs()
    assert st["flags"] == 0 and out_idx.size == U
    assert np.array_equal(out_idx, np.flatnonzero(
        np.unpackbits(merged.view(np.uint8), bitorder="little")[:n_c]).astype(np.uint32))
    part = np.searchsorted(bnd[1:A], out_idx, side="right")
    scale = np.zeros(A)
    np.maximum.at(scale, part, np.maximum(np.abs(ref[out_idx]), big[out_idx]))
    err = np.abs(out_val.astype(np.float64) - ref[out_idx])
    bad = err > 1e-5 * scale[part]
    # what peeling could not recover is reported as 0 and counted, nothing else is off
    assert bad.sum() <= st["n_unresolved"] <= max_unresolved
    assert np.all(out_val[bad] == 0)
    dense = tb.dense()
    want = np.zeros(n_c, np.float32)
    want[out_idx] = out_val
    assert np.array_equal(dense.view(np.uint32), want.view(np.uint32))
    _say("decode against the definition: %d unresolved of %d, %d rounds"
         % (st["n_unresolved"], U, st["rounds"]))
    return tb


def test_config5_bucket_as_the_benchmark_runs_it():
    print("\n[case] config5 block 0 at full size", flush=True)
    b = G.config5(0)[0]
    assert b.n_ranks == 16 and b.n_elems > 200_000_000
    data = [G.rank_gradient(b, r, "cuda") for r in range(b.n_ranks)]
    tb = _check_full_size(b, data, oracle_ranks=(0, 9), decode_workgroups=64)  # as bench.py
    assert all(tb.rank_counts(r)["dense_segments"] == 0 for r in range(1, b.n_ranks))


def test_config5_buckets_in_flight_as_the_benchmark_keeps_them():
    """Three 7B-shaped buckets (blocks 0, 1, 2; 8 ranks to fit the test's time) issued
    round-robin on three streams, each with its own buffers and the peeling kernel limited
    to 64 workgroups, twice over: every bucket must come out as it does alone on an idle
    device -- same counts, pairs, Index, layout and decoded indices bit for bit; decoded
    values within the float tolerance (the order of peeling's float subtractions inside a
    round is free)."""
    from paper_2504_05638_amd.bucket import TagcBucket
    print("\n[case] three config5 buckets in flight", flush=True)
    buckets = G.config5(0, n_ranks=8)[:3]
    data = [[G.rank_gradient(b, r, "cuda") for r in range(b.n_ranks)] for b in buckets]
    tbs = [TagcBucket(b.segments, b.dtype, b.n_ranks, sizing_milli=b.sizing_milli, seed=3,
                      dense=False, decode_workgroups=64) for b in buckets]

    def snapshot(tb):
        hdr, st = tb.header(), tb.status()
        U = hdr["U"]
        ranks = [(tb.rank_counts(r), tb._rk_tensors[r]["idx"].clone(),
                  tb._rk_tensors[r]["val"].clone()) for r in (0, tb.n_ranks - 1)]
        return (hdr, st, ranks, tb.sh_bitmap.clone(), tb.out_idx[:4 * U].clone(),
                tb.out_val[:4 * U].view(torch.float32).clone())

    alone = []
    for tb, d in zip(tbs, data):
        tb.run(d)
        torch.cuda.synchronize()
        alone.append(snapshot(tb))
        assert alone[-1][1]["flags"] == 0 and alone[-1][1]["n_unresolved"] <= 20
    _say("alone done")
    streams = [torch.cuda.Stream() for _ in tbs]
    torch.cuda.synchronize()
    for _ in range(2):
        for tb, d, s in zip(tbs, data, streams):
            tb.run(d, s)
    torch.cuda.synchronize()
    for i, (tb, ref) in enumerate(zip(tbs, alone)):
        hdr, st, ranks, bitmap, oidx, oval = snapshot(tb)
        assert hdr == ref[0] and st["flags"] == 0
        assert st["n_unresolved"] == ref[1]["n_unresolved"] and st["rounds"] == ref[1]["rounds"]
        for (c, ix, vl), (rc, rix, rvl) in zip(ranks, ref[2]):
            k = 4 * c["total"]
            same = ("total", "nonfinite", "flags", "seg")   # the rest is diagnostic
            assert all(c[f] == rc[f] for f in same)
            assert torch.equal(ix[:k], rix[:k]) and torch.equal(vl[:k], rvl[:k])
        assert torch.equal(bitmap, ref[3]) and torch.equal(oidx, ref[4])
        scale = float(ref[5].abs().max())
        assert float((oval - ref[5]).abs().max()) <= 1e-5 * scale
        _say("bucket %d in flight == alone (U = %d)" % (i, hdr["U"]))


def test_config4_sharded_7b_bucket():
    print("\n[case] config4 block 0 at full size", flush=True)
    b = G.config4(0)[0]
    assert b.n_ranks == 8 and b.n_elems > 25_000_000
    data = [G.rank_gradient(b, r, "cuda") for r in range(b.n_ranks)]
    _check_full_size(b, data, oracle_ranks=(0, 5))


@pytest.mark.parametrize("keep_ppm,lf,dense_route", [(10_000, 1500, False), (100_000, 3000, True)])
def test_config3_heavy_tails_shared_supports(keep_ppm, lf, dense_route):
    """64 M Student-t entries per rank, half of every rank's support shared with all others;
    at 10 % kept the plan takes the two-read route."""
    print("\n[case] config3 at full size keep=%d lf=%d" % (keep_ppm, lf), flush=True)
    b = G.config3(0, keep_ppm=keep_ppm, sizing_milli=lf)
    assert b.n_elems == 1 << 26 and b.n_ranks == 8
    data = [G.config3_rank_gradient(b, r, "cuda") for r in range(b.n_ranks)]
    tb = _check_full_size(b, data, oracle_ranks=(3,))
    assert (tb.rank_counts(0)["dense_segments"] == 1) == dense_route
    k = (b.n_elems * keep_ppm) // 10 ** 6
    # 8 ranks, half of each support shared: k/2 + 8 * k/2 positions, less what the private
    # halves happen to share at 10 %
    assert 3.5 * k < tb.header()["U"] < 4.6 * k


def test_one_segment_of_almost_two_to_the_31_entries():
    """The largest segment the format allows (just under 2^31 entries, 4.3 GB of bf16), one
    rank, through the whole path.  Too large for the oracle or for host-side checks: the
    selection rule, the Index and the decoded values are verified with torch's own device
    primitives (count, gather, compare), which is all the rule needs."""
    from paper_2504_05638_amd.bucket import TagcBucket
    print("\n[case] one segment of 2^31 - 4096 entries", flush=True)
    n = (1 << 31) - 4096
    b = G.Bucket("max", G.BF16, 1, [G.Seg(0, n, 10_000, 1, "w")], n, 1500, {"w": 1e-3})
    g = G.rank_gradient(b, 0, "cuda")
    k = (n * 10_000) // 10 ** 6
    tb = TagcBucket(b.segments, b.dtype, 1, sizing_milli=b.sizing_milli, seed=0, dense=False)
    tb.run([g])
    torch.cuda.synchronize()
    cnt = tb.rank_counts(0)
    assert cnt["flags"] == 0 and cnt["nonfinite"] == 0 and cnt["total"] == k and cnt["seg"] == [k]
    t = tb._rk_tensors[0]
    idx = t["idx"].view(torch.int32)[:k].to(torch.int64)
    val = t["val"].view(torch.float32)[:k]
    assert bool((idx >= 0).all()) and int(idx[-1]) < n
    assert bool((idx[1:] > idx[:-1]).all())
    assert torch.equal(val, g[idx].to(torch.float32))                  # the entries themselves
    mag = g.abs()
    T = val.abs().min().to(torch.bfloat16)
    assert float(T) > 0
    assert int((mag > T).sum()) <= k <= int((mag >= T).sum())         # the k largest
    ties = torch.nonzero(mag == T).flatten()
    kept = torch.isin(ties, idx, assume_unique=True)
    n_kept = int(kept.sum())
    assert n_kept >= 1 and bool(kept[:n_kept].all())                   # the lowest positions
    del mag
    _say("selection rule: %d ties at the threshold, %d kept" % (ties.numel(), n_kept))
    lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device="cuda")
    words = tb.sizes.bitmap_words
    bm = t["bitmap"][:4 * words]
    assert int(lut[bm.to(torch.int64)].sum()) == k
    assert bool(((bm[idx >> 3].to(torch.int64) >> (idx & 7)) & 1).all())  # Index <-> pairs
    hdr, st = tb.header(), tb.status()
    assert hdr["U"] == k and st["flags"] == 0 and st["n_unresolved"] <= 20
    out_idx = tb.out_idx.view(torch.int32)[:k].to(torch.int64)
    out_val = tb.out_val.view(torch.float32)[:k]
    assert torch.equal(out_idx, idx)
    off = out_val != val                   # one rank: the decoded sum is what it sent
    rel = (out_val - val).abs() / val.abs()
    assert int((off & (rel > 1e-5)).sum()) <= st["n_unresolved"]
    _say("decode: %d unresolved of %d, %d rounds" % (st["n_unresolved"], k, st["rounds"]))


def test_7b_shaped_bucket_in_fp32():
    """The same block shapes with float32 gradients (4 ranks): the path that needs the low 16
    key bits as well (a second histogram over the candidates of the threshold bin)."""
    import dataclasses
    print("\n[case] config5 block 0 shapes, fp32, 4 ranks", flush=True)
    b = dataclasses.replace(G.config5(0)[0], dtype=G.F32, n_ranks=4)
    data = [G.rank_gradient(b, r, "cuda") for r in range(b.n_ranks)]
    assert data[0].dtype == torch.float32
    _check_full_size(b, data, oracle_ranks=(1,))
