"""GPU parity at the workloads' full sizes: one 7B-shaped bucket of the benchmark (config5,
block 0: 202 M bf16 entries x 16 ranks, load factor 1.5, default partitions, dense output),
run exactly as bench.py runs it; one bucket of the sharded 7B workload (config4); the 64 M
heavy-tailed bucket with half-shared supports (config3) at two of its (keep, load factor)
points (a hundredth kept: dozens of candidates per chunk; a tenth: hundreds) and once from an
unaligned offset, which takes the dense route.  The oracle cannot redo all of it in test
time, so: sampled (rank, segment) pairs go through the oracle's sparsifier bit for bit; one rank's whole sketch and a slice of
the summed one go through the oracle's encode and sum; the cheap stages (Index merge, layout,
bounds, salts) are redone in full; everything else is checked, for every rank, through what
must hold at any size -- counts, order, Index <-> pairs, values against the gradient, the
magnitude rule (verified on the device) -- and the decoded values against the definition of
the result: per index the float64 sum, over the ranks, of the gradient entries the rule
selects."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import oracle_segments

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[fullsize] " + msg, flush=True)


def _bits(t):
    """magnitude keys of a gradient tensor as int32 (bf16 keys are 15 bits)"""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).to(torch.int32) & 0x7FFF
    return t.view(torch.int32) & 0x7FFFFFFF


def _check_full_size(b, data, seed=0, oracle_ranks=(0,), decode_workgroups=0):
    from paper_2504_05638_amd.bucket import TagcBucket
    from tests.helpers import check_decoded_values
    N = b.n_ranks
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

    # ---- stage 1, EVERY rank, on the device: counts, order, Index <-> pairs, the values
    # against the gradient, and the selection rule, which with the count fixes the kept set:
    # everything above the threshold is kept, of the entries that tie with the smallest kept
    # one exactly the lowest positions are, zeros never.  The reference of the decoded result
    # is built here too, from the gradients at the positions the rule has just confirmed:
    # per index the float64 sum over the ranks, and per segment tau_l, the smallest magnitude
    # any rank kept.
    lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device="cuda")
    ref = torch.zeros(n_c, dtype=torch.float64, device="cuda")
    tau = [float("inf")] * len(segs)
    n_ties = 0
    for r in range(N):
        cnt = tb.rank_counts(r)
        assert cnt["flags"] == 0 and cnt["nonfinite"] == 0
        assert cnt["seg"] == k and cnt["total"] == sum(k)       # enough non-zeros everywhere
        t = tb._rk_tensors[r]
        idx = t["idx"].view(torch.int32)[:sum(k)].to(torch.int64)
        val = t["val"].view(torch.float32)[:sum(k)]
        assert bool((idx[1:] > idx[:-1]).all())
        bm = t["bitmap"][:4 * z.bitmap_words]
        assert int(lut[bm.to(torch.int64)].sum()) == sum(k)
        assert bool(((bm[idx >> 3].to(torch.int64) >> (idx & 7)) & 1).all())
        g = data[r]
        pos = 0
        for l, s in enumerate(segs):
            i_l = idx[pos:pos + k[l]] - c_off[l]
            v_l = val[pos:pos + k[l]]
            pos += k[l]
            assert int(i_l[0]) >= 0 and int(i_l[-1]) < s.length
            seg = g[s.offset:s.offset + s.length]
            sent = seg[i_l].to(torch.float32)
            assert torch.equal(v_l.view(torch.int32), sent.view(torch.int32))   # the entries themselves
            key = _bits(seg)
            kept = key[i_l]
            T = int(kept.min())
            assert T > 0                                                    # zeros never
            above = int((key > T).sum())
            assert above == int((kept > T).sum()) and above < k[l]          # all of them kept
            ties = torch.nonzero(key == T).flatten()
            need = k[l] - above
            assert ties.numel() >= need
            assert torch.equal(i_l[kept == T], ties[:need])                 # the lowest positions
            n_ties += int(ties.numel())
            ref.index_add_(0, idx[pos - k[l]:pos], sent.to(torch.float64))
            tau[l] = min(tau[l], float(sent.abs().min()))
            del key, kept, ties, seg, sent
    _say("all %d ranks against their gradients (%d entries tie at a threshold)" % (N, n_ties))

    # ---- sampled (rank, segment) pairs also through the oracle's sparsifier
    by_len = sorted(range(len(segs)), key=lambda l: segs[l].length)
    sampled_segs = {by_len[0], by_len[len(by_len) // 2], by_len[-1]}
    for r in oracle_ranks:
        idx, val = tb.rank_pairs(r)
        raw = G.to_numpy_raw(data[r])
        pos = 0
        for l, s in enumerate(segs):
            if l in sampled_segs:
                one = [O.Segment(0, s.length, s.keep_ppm, 1)]
                st = O.sparsify(np.ascontiguousarray(raw[s.offset:s.offset + s.length]),
                                O.Config(dtype=b.dtype), one)
                assert np.array_equal(st.idx.astype(np.int64),
                                      idx[pos:pos + k[l]].astype(np.int64) - c_off[l])
                assert np.array_equal(st.val.view(np.uint32), val[pos:pos + k[l]].view(np.uint32))
            pos += k[l]
        del raw
        _say("rank %d, three segments through the oracle's sparsifier" % r)

    # ---- stage 3a in full: merged Index, U, layout, bounds, salts
    maps = [tb.rank_bitmap(r) for r in range(N)]
    merged, U = O.index_or(maps)
    del maps
    assert np.array_equal(tb.shared_bitmap(), merged)
    hdr = tb.header()
    cfg = O.Config(dtype=b.dtype, sizing_milli=b.sizing_milli, seed=seed)
    A, m_sub, m = O.layout(U, cfg, z.n_real)
    assert hdr == dict(U=U, A=A, m_sub=m_sub, m=m)
    bnd = O.bounds(merged, n_c, U, A)
    assert np.array_equal(tb.bounds(), bnd)
    salt = O.salts(merged, n_c, U, A, m_sub, seed)
    assert np.array_equal(tb.salts(), salt)
    _say("Index merge, layout, bounds, salts: U=%d A=%d m=%d, %d partitions salted"
         % (U, A, m, int(np.count_nonzero(salt))))

    # ---- stage 2': one rank's whole sketch through the oracle's encode
    r = N // 3
    pr = tb.rank_pairs(r)
    want = O.encode(pr[0], pr[1], bnd, A, m_sub, seed, salt=salt)
    mag = O.encode(pr[0], np.abs(pr[1]), bnd, A, m_sub, seed, plus_only=True, salt=salt)
    got = tb.rank_sketch(r)
    assert np.all(np.abs(got.astype(np.float64) - want) <= 1e-5 * mag.astype(np.float64))
    assert np.mean(got.view(np.uint32) == want.view(np.uint32)) > 0.99
    del want, mag, got, pr
    _say("rank %d sketch" % r)

    # ---- stage 3b: a slice of the summed sketch (the ranks' sketches are still on the device)
    c0 = m // 3
    c1 = min(m, c0 + (1 << 20))
    parts = [tb.rank_sketch(q)[c0:c1].copy() for q in range(N)]
    want = O.sketch_sum(parts)
    got = tb.shared_sketch()[c0:c1]
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))     # same order, same bits
    _say("summed sketch slice")

    # ---- stage 4 against the definition of the result.  Lossless: nothing unresolved.
    # Values: |delta| <= 1e-5 * max(|ref|, tau_l) first; what exceeds that must be an entry
    # mixed with far larger ones (see tests/helpers.py), within 1e-5 of its partition's scale.
    # Checked twice: as tagc_aggregate(PHASE_SKETCH) + tagc_decompress left it, and after
    # tagc_reduce_decompress (the decoder summing the ranks' sketches itself) on the same
    # buffers, which is how bench.py decodes by default.
    want_idx = np.flatnonzero(
        np.unpackbits(merged.view(np.uint8), bitorder="little")[:n_c]).astype(np.uint32)
    ref_u = ref[torch.from_numpy(want_idx.astype(np.int64)).cuda()].cpu().numpy()
    del ref
    starts = np.array(c_off, np.int64)
    seg_of = np.searchsorted(starts, want_idx.astype(np.int64), side="right") - 1
    strict = 1e-5 * np.maximum(np.abs(ref_u), np.array(tau)[seg_of])
    part = np.searchsorted(bnd[1:A], want_idx, side="right")
    scale = np.zeros(A)
    np.maximum.at(scale, part, np.abs(ref_u))
    loose = 1e-5 * np.maximum(np.abs(ref_u), scale[part])

    def check_decode(label):
        st = tb.status()
        out_idx, out_val = tb.outputs()
        assert st["flags"] == 0 and out_idx.size == U and st["n_unresolved"] == 0
        assert np.array_equal(out_idx, want_idx)
        n_over = check_decoded_values(b.name, out_val, ref_u, strict, loose)
        dense = tb.dense()
        want = np.zeros(n_c, np.float32)
        want[out_idx] = out_val
        assert np.array_equal(dense.view(np.uint32), want.view(np.uint32))
        _say("%s against the definition: %d of %d beyond the stated bound, %d rounds"
             % (label, n_over, U, st["rounds"]))
        return st

    st2 = check_decode("decode")
    tb.sh_status.zero_()
    tb.out_val.zero_()
    tb.out_dense.zero_()
    tb.reduce_decompress(N)
    torch.cuda.synchronize()
    st1 = check_decode("sum inside decode")
    assert st1 == st2
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
        assert alone[-1][1]["flags"] == 0 and alone[-1][1]["n_unresolved"] == 0
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


@pytest.mark.parametrize("keep_ppm,lf,offset,dense_route",
                         [(10_000, 1500, 0, False), (100_000, 3000, 0, False),
                          (100_000, 3000, 3, True)])
def test_config3_heavy_tails_shared_supports(keep_ppm, lf, offset, dense_route):
    """64 M Student-t entries per rank, half of every rank's support shared with all others.
    At 10 % kept a chunk holds hundreds of candidates (count and place with a wave per
    super-chunk); the same from an offset that is no multiple of a 16-byte vector, which
    the plan sends down the route that reads the gradient three times."""
    print("\n[case] config3 at full size keep=%d lf=%d offset=%d" % (keep_ppm, lf, offset),
          flush=True)
    b = G.config3(0, keep_ppm=keep_ppm, sizing_milli=lf)
    assert b.n_elems == 1 << 26 and b.n_ranks == 8
    if offset:
        b.segments = [G.Seg(offset, b.n_elems - offset, keep_ppm, 1, "w")]
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
    assert hdr["U"] == k and st["flags"] == 0 and st["n_unresolved"] == 0
    out_idx = tb.out_idx.view(torch.int32)[:k].to(torch.int64)
    out_val = tb.out_val.view(torch.float32)[:k]
    assert torch.equal(out_idx, idx)
    # one rank: the decoded sum is what it sent, to 1e-5 relative, entry by entry
    rel = (out_val - val).abs() / val.abs()
    assert int((rel > 1e-5).sum()) == 0
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
