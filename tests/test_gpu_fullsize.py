"""GPU parity at the benchmark's full size: one 7B-shaped bucket (config5, block 0: 202 M
bf16 entries x 16 ranks, load factor 1.5, default partitions, dense output), run exactly as
bench.py runs it.  The oracle cannot redo all of it in test time, so: sampled (rank, segment)
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


def test_config5_bucket_as_the_benchmark_runs_it():
    from paper_2504_05638_amd.bucket import TagcBucket
    print("\n[case] config5 block 0 at full size", flush=True)
    b = G.config5(0)[0]
    N = b.n_ranks
    assert N == 16 and b.n_elems > 200_000_000
    segs = [s for s in b.segments if s.flags & 1]
    offs, n_c = O.c_offsets(oracle_segments(b))
    c_off = [o for o, s in zip(offs, b.segments) if s.flags & 1]
    k = [O.keep_count(s.length, s.keep_ppm) for s in segs]
    data = [G.rank_gradient(b, r, "cuda") for r in range(N)]
    tb = TagcBucket(b.segments, b.dtype, N, sizing_milli=b.sizing_milli, seed=0, dense=True)
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

    # ---- stage 1, sampled ranks: Index <-> pairs, values, magnitude rule; oracle on sampled
    # segments (the largest, the smallest, one in between)
    by_len = sorted(range(len(segs)), key=lambda l: segs[l].length)
    sampled_segs = {by_len[0], by_len[len(by_len) // 2], by_len[-1]}
    for r in (0, 9):
        idx, val = pairs[r]
        bits = np.zeros(n_c, bool)
        bits[idx] = True
        assert np.array_equal(np.packbits(bits, bitorder="little").view(np.uint32),
                              tb.rank_bitmap(r))
        del bits
        raw = G.to_numpy_raw(data[r])                            # bf16 bit patterns
        pos = 0
        for l, s in enumerate(segs):
            i_l = idx[pos:pos + k[l]].astype(np.int64) - c_off[l]
            v_l = val[pos:pos + k[l]]
            pos += k[l]
            assert i_l.min() >= 0 and i_l.max() < s.length
            seg_raw = raw[s.offset:s.offset + s.length]
            wide = (seg_raw.astype(np.uint32) << 16)
            assert np.array_equal(v_l.view(np.uint32), wide[i_l])        # the entries themselves
            key = wide & 0x7FFFFFFF
            kept_min = key[i_l].min()
            key[i_l] = 0
            assert key.max() <= kept_min                                  # the k largest magnitudes
            if l in sampled_segs:
                one = [O.Segment(0, s.length, s.keep_ppm, 1)]
                st = O.sparsify(np.ascontiguousarray(seg_raw), O.Config(dtype=O.BF16), one)
                assert np.array_equal(st.idx.astype(np.int64), i_l)      # ties included
                assert np.array_equal(st.val.view(np.uint32), v_l.view(np.uint32))
        del raw
        _say("rank %d against its gradient and the oracle" % r)

    # ---- stage 3a in full: merged Index, U, layout, bounds
    maps = [tb.rank_bitmap(r) for r in range(N)]
    merged, U = O.index_or(maps)
    assert np.array_equal(tb.shared_bitmap(), merged)
    hdr = tb.header()
    cfg = O.Config(dtype=O.BF16, sizing_milli=b.sizing_milli, seed=0)
    A, m_sub, m = O.layout(U, cfg, z.n_real)
    assert hdr == dict(U=U, A=A, m_sub=m_sub, m=m)
    bnd = O.bounds(merged, n_c, U, A)
    assert np.array_equal(tb.bounds(), bnd)
    _say("Index merge, layout, bounds: U=%d A=%d m=%d" % (U, A, m))

    # ---- stage 2': one rank's whole sketch through the oracle's encode
    r = 5
    want = O.encode(pairs[r][0], pairs[r][1], bnd, A, m_sub, 0)
    mag = O.encode(pairs[r][0], np.abs(pairs[r][1]), bnd, A, m_sub, 0, plus_only=True)
    got = tb.rank_sketch(r)
    assert np.all(np.abs(got.astype(np.float64) - want) <= 1e-5 * mag.astype(np.float64))
    assert np.mean(got.view(np.uint32) == want.view(np.uint32)) > 0.99
    del want, mag, got
    _say("rank %d sketch" % r)

    # ---- stage 3b: a slice of the summed sketch (the ranks' sketches are still on the device)
    c0, c1 = m // 3, m // 3 + (1 << 20)
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
        np.maximum.at(big, idx, np.abs(val).astype(np.float64))
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
    assert bad.sum() <= st["n_unresolved"] <= 20
    assert np.all(out_val[bad] == 0)
    dense = tb.dense()
    want = np.zeros(n_c, np.float32)
    want[out_idx] = out_val
    assert np.array_equal(dense.view(np.uint32), want.view(np.uint32))
    _say("decode against the definition: %d unresolved of %d, %d rounds"
         % (st["n_unresolved"], U, st["rounds"]))
