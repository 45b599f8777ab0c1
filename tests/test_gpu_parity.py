"""GPU parity: the HIP library against the CPU oracle, element by element, on the
same seeded inputs, through the C ABI.  Integer work (selected indices, Index
bits, layout, bounds, resolved set, rounds) must be bit-exact; float values within
1e-5 relative (only atomic summation order may differ); exact for inputs whose
float32 arithmetic is exact."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import run_both, compare_all

pytestmark = pytest.mark.gpu


def _grads(bucket, gen=G.rank_gradient):
    return [gen(bucket, r, "cpu") for r in range(bucket.n_ranks)]


def _announce(name):
    print("\n[case] %s" % name, flush=True)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("lf", [1500, 3000])
def test_small_mixed_bucket(dtype, lf):
    """Ragged lengths, unaligned offsets, skipped segments, a k = 0 segment, several
    sketch partitions."""
    _announce("small_mixed dtype=%d lf=%d" % (dtype, lf))
    b = G.small_mixed_bucket(seed=3, dtype=dtype, n_ranks=3, sizing_milli=lf)
    ores, tb = run_both(b, _grads(b), seed=5, P=256, T=768)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["A"] > 1


def test_config1_full_size():
    """Benchmark configuration 1: 4 ranks x 1,048,576 fp32 ~ N(0, 1e-3), top 1 %, lf 3."""
    _announce("config1")
    b = G.config1(seed=0)
    ores, tb = run_both(b, _grads(b), seed=0)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["U"] > 40_000 and st["n_unresolved"] == 0
    for r in range(4):
        assert tb.rank_counts(r)["total"] == 10_485
        assert tb.rank_counts(r)["dense_segments"] == 0   # single-read route


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_integer_values_are_bit_exact_end_to_end(dtype):
    """Small-integer inputs: every float32 add is exact, so sketch cells and decoded
    values must match the oracle bit for bit whatever the atomic order."""
    _announce("integer exact dtype=%d" % dtype)
    rng = np.random.default_rng(12)
    n, N = 300_000, 5
    segs = [G.Seg(0, 100_000, 30_000, 1, "a"), G.Seg(100_000, 200_000, 20_000, 1, "b")]
    b = G.Bucket("ints", dtype, N, segs, n, 1500)
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = [torch.from_numpy(rng.integers(-100, 101, n).astype(np.float32)).to(td)
             for _ in range(N)]
    ores, tb = run_both(b, grads, seed=1, P=2048, T=3072)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    assert hdr["A"] > 4


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("kind", ["all_equal", "two_valued", "mostly_zero", "all_zero"])
def test_heavy_ties_and_zeros(dtype, kind):
    """The threshold sits inside a huge tie class (or there are fewer non-zeros than
    k): the lowest positions must win, zeros must never be kept."""
    _announce("ties %s dtype=%d" % (kind, dtype))
    rng = np.random.default_rng(4)
    n, N = 70_001, 2
    segs = [G.Seg(0, 40_001, 100_000, 1, "a"), G.Seg(40_008, 29_993, 250_000, 1, "b")]
    b = G.Bucket("ties", dtype, N, segs, n, 3000)
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = []
    for r in range(N):
        if kind == "all_equal":
            v = np.full(n, 0.5, np.float32) * (1 if r == 0 else -1)
        elif kind == "two_valued":
            v = rng.choice([-1.0, 2.0], n).astype(np.float32)
        elif kind == "mostly_zero":
            v = (rng.integers(1, 9, n) * (rng.random(n) < 0.01)).astype(np.float32)
        else:
            v = np.zeros(n, np.float32)
        grads.append(torch.from_numpy(v).to(td))
    ores, tb = run_both(b, grads, seed=2, P=1024, T=3072)
    compare_all(b, ores, tb, exact_values=True)


def test_gpt2_block_shapes_fp32():
    """One GPT-2-small block of benchmark configuration 2 (4 compressed linear layers, biases
    and LayerNorms skipped, per-layer keep ratio), 3 ranks."""
    _announce("config2 block0")
    b = G.config2(seed=0, n_ranks=3)[0]
    ores, tb = run_both(b, _grads(b), seed=0)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_unresolved"] <= 2


def test_repeated_calls_on_short_fp32_segments_select_the_same_every_time():
    """A selection must not depend on when workgroups finish.  The last workgroup of a
    segment to arrive selects the threshold from counts that the others added with atomics;
    each workgroup has to wait for its own adds before it counts as arrived.  Short fp32
    segments, whose few workgroups end almost together, are where an early arrival would
    show: every one of many calls on the same plan must give the oracle's survivors."""
    _announce("config2 block6, repeated calls")
    b = G.config2(seed=0, n_ranks=4)[6]
    grads = _grads(b)
    ores, tb = run_both(b, grads, seed=0)
    compare_all(b, ores, tb)
    dev = [g.cuda() for g in grads]
    for it in range(12):
        tb.run(dev)
        torch.cuda.synchronize()
        for r in range(b.n_ranks):
            cnt = tb.rank_counts(r)
            assert cnt["flags"] == 0 and cnt["total"] == ores.ranks[r].cnt, (it, r, cnt)
            idx, val = tb.rank_pairs(r)
            assert np.array_equal(idx, ores.ranks[r].idx), (it, r)
            assert np.array_equal(val.view(np.uint32), ores.ranks[r].val.view(np.uint32))
        assert tb.header()["U"] == ores.U and tb.status()["n_unresolved"] == 0


def test_bf16_many_tiles_ragged_tail_student_t():
    """bf16, heavy-tailed values, length not a multiple of the tile or the vector,
    load factor 1.5 (benchmark configuration 3 at reduced length, with its overlap recipe)."""
    _announce("config3 reduced")
    b = G.config3(seed=0, n=(1 << 21) + 4321, n_ranks=4, keep_ppm=10_000, sizing_milli=1500)
    grads = [G.config3_rank_gradient(b, r, "cpu") for r in range(4)]
    ores, tb = run_both(b, grads, seed=0)
    hdr, st = compare_all(b, ores, tb)
    k = (b.n_elems * 10_000) // 10 ** 6
    assert 2.0 * k < hdr["U"] < 3.5 * k        # supports overlap by about half


@pytest.mark.parametrize("ratio_milli,theta_ppm", [(2000, 200_000), (10_000, 12_500)])
def test_fixed_ratio_mode_table1(ratio_milli, theta_ppm):
    """Table 1 regimes: c-x compression at the stated sparsity, two ranks."""
    _announce("fixed ratio %d" % ratio_milli)
    n = 400_000
    b = G.Bucket("t1", G.F32, 2, [G.Seg(0, n, theta_ppm, 1, "w")], n, ratio_milli)
    ores, tb = run_both(b, _grads(b), seed=3, sizing=O.SIZE_FIXED_RATIO)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["m"] <= n * 1000 // ratio_milli
    assert st["n_unresolved"] <= 2


def test_undersized_sketch_reports_residue():
    """Below the peeling threshold the decoder must say so, not invent values."""
    _announce("undersized")
    b = G.config1(seed=1, n=200_000, n_ranks=2)
    b.sizing_milli = 1100
    ores, tb = run_both(b, _grads(b), seed=0, P=1024, T=3072)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_unresolved"] > 0.3 * hdr["U"]


def test_empty_and_degenerate_buckets():
    _announce("degenerate")
    # no compressed segment at all
    b = G.Bucket("none", G.F32, 2, [G.Seg(0, 100, 500_000, 0, "x")], 100, 3000)
    ores, tb = run_both(b, _grads(b))
    assert tb.header() == dict(U=0, A=0, m_sub=0, m=0) and ores.U == 0
    # keep count rounds to zero everywhere
    b = G.Bucket("k0", G.BF16, 2, [G.Seg(0, 999, 1_000, 1, "x")], 999, 3000)
    ores, tb = run_both(b, _grads(b))
    compare_all(b, ores, tb)
    assert tb.header()["U"] == 0
    assert not tb.dense().any()
    # a single element
    b = G.Bucket("one", G.F32, 1, [G.Seg(0, 1, 1_000_000, 1, "x")], 1, 3000)
    ores, tb = run_both(b, _grads(b))
    compare_all(b, ores, tb, exact_values=True)
    assert tb.header()["U"] == 1


def test_integer_outputs_are_reproducible_run_to_run():
    """Atomics may only perturb float low bits: two runs give identical indices,
    bit maps, bounds and resolved sets."""
    _announce("determinism")
    b = G.small_mixed_bucket(seed=8, dtype=G.BF16, n_ranks=4, sizing_milli=1500)
    grads = _grads(b)
    _, t1 = run_both(b, grads, seed=9, P=256, T=768)
    _, t2 = run_both(b, grads, seed=9, P=256, T=768)
    assert np.array_equal(t1.shared_bitmap(), t2.shared_bitmap())
    assert np.array_equal(t1.bounds(), t2.bounds())
    for r in range(4):
        assert np.array_equal(t1.rank_pairs(r)[0], t2.rank_pairs(r)[0])
    i1, v1 = t1.outputs()
    i2, v2 = t2.outputs()
    assert np.array_equal(i1, i2) and np.array_equal(v1 == 0, v2 == 0)
    assert t1.status() == t2.status()


def test_nonfinite_inputs_are_counted():
    _announce("nonfinite")
    b = G.config1(seed=2, n=50_000, n_ranks=1)
    g = G.rank_gradient(b, 0, "cpu")
    g[[7, 4097, 49_999]] = torch.tensor([float("inf"), float("nan"), float("-inf")])
    from paper_2504_05638_amd.bucket import TagcBucket
    tb = TagcBucket(b.segments, b.dtype, 1, sizing_milli=3000)
    tb.compress_index(0, g.cuda())
    torch.cuda.synchronize()
    assert tb.rank_counts(0)["nonfinite"] == 3


def test_hash_on_device_matches_host_helper_and_oracle():
    """Slots are observable through the sketch: one unit pair per rank lands in
    exactly the three cells the host helper and the oracle name."""
    _announce("hash slots")
    n = 4096
    b = G.Bucket("h", G.F32, 1, [G.Seg(0, n, 1_000_000, 1, "w")], n, 3000)
    from paper_2504_05638_amd import binding as B
    for pos in (0, 1, 31, 32, 1000, 4095):
        g = torch.zeros(n)
        g[pos] = 1.0
        ores, tb = run_both(b, [g], seed=77)
        sk = tb.rank_sketch(0)
        hdr = tb.header()
        assert hdr["U"] == 1 and hdr["A"] == 1
        want = np.zeros(hdr["m"], np.float32)
        for j in range(3):
            slot, sign = B.tagc_hash_host(pos, 77, j, hdr["m_sub"])
            assert (slot, sign) == O.hash_slot(pos, 77, j, hdr["m_sub"])
            want[j * hdr["m_sub"] + slot] = sign
        assert np.array_equal(sk, want)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_partition_salts(dtype):
    """Tiny partitions, so that many of them hold two non-zeros with the same three cells:
    the Index aggregation must pick the oracle's salts, and encode and decode must hash
    under them (cells, rounds and decoded values are compared as everywhere)."""
    _announce("partition salts dtype=%d" % dtype)
    n, N = 200_000, 3
    b = G.Bucket("salts", dtype, N, [G.Seg(0, n, 30_000, 1, "w")], n, 1500, {"w": 1e-3})
    ores, tb = run_both(b, _grads(b), seed=11, P=64, T=48)
    hdr, st = compare_all(b, ores, tb)
    salted = int(np.count_nonzero(ores.salt))
    assert hdr["A"] > 200 and salted > 20 and ores.salt.max() >= 2
    assert np.array_equal(tb.salts(), ores.salt)
    # without them the format loses at least the colliding pairs
    plain = O.run_bucket([G.to_numpy_raw(g) for g in _grads(b)],
                         O.Config(dtype=dtype, sizing_milli=1500, seed=11, part_unknowns=64,
                                  part_cells=48),
                         [O.Segment(0, n, 30_000)], salted=False)
    assert plain.decoded.n_unresolved >= st["n_unresolved"] + 2 * salted


def test_a_planted_pair_with_the_same_three_cells_is_decoded():
    """Two positions whose cells coincide under salt 0 (found by search on the host helper):
    the partition gets another salt and both values come out exactly."""
    _announce("planted colliding pair")
    from paper_2504_05638_amd import binding as B
    seed, n, m_sub = 17, 200_000, 32
    seen, pair = {}, None
    for i in range(n):
        key = tuple(B.tagc_hash_host(i, seed, j, m_sub)[0] for j in range(3))
        if key in seen:
            pair = (seen[key], i)
            break
        seen[key] = i
    assert pair is not None
    rng = np.random.default_rng(0)
    others = rng.choice(np.setdiff1d(np.arange(n), pair), 62, replace=False)
    g = torch.zeros(n)
    g[torch.from_numpy(others)] = torch.from_numpy(rng.integers(1, 100, 62).astype(np.float32))
    g[pair[0]], g[pair[1]] = 1234.0, -77.0
    b = G.Bucket("pair", G.F32, 1, [G.Seg(0, n, 1_000_000, 1, "w")], n, 1500)
    ores, tb = run_both(b, [g], seed=seed, P=64, T=96)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    assert (hdr["A"], hdr["m_sub"]) == (1, m_sub) and tb.salts().tolist() != [0]
    idx, val = tb.outputs()
    assert val[idx == pair[0]] == 1234.0 and val[idx == pair[1]] == -77.0


# ---------------------------------------------------------------------------
# Routes of the sparsifier: long aligned segments stream the gradient once and keep only
# "candidates" above a sampled pre-threshold; everything else, and every case where that
# shortcut does not hold k entries, falls back to the two-read dense route.  Both must
# give the oracle's answer.


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_candidate_and_dense_routes_in_one_bucket(dtype):
    _announce("routes mixed dtype=%d" % dtype)
    segs = [G.Seg(0, (1 << 18) + 13, 10_000, 1, "long_ragged"),
            G.Seg(262_168, 5000, 20_000, 1, "short"),
            G.Seg(267_176, (1 << 17), 25_000, 1, "long_dense_keep"),
            G.Seg(398_251, (1 << 17) + 64, 10_000, 1, "long_unaligned"),
            G.Seg(529_392, 300_000, 100, 1, "long_tiny_k")]
    n = 829_392
    b = G.Bucket("routes", dtype, 3, segs, n, 1500,
                 {"long_ragged": 1e-3, "short": 1e-2, "long_dense_keep": 1e-4,
                  "long_unaligned": 3e-3, "long_tiny_k": 1e-3})
    ores, tb = run_both(b, _grads(b), seed=6, P=4096, T=6144)
    compare_all(b, ores, tb)
    # short, unaligned and tiny-k segments read the gradient twice, the other two once
    assert [tb.rank_counts(r)["dense_segments"] for r in range(3)] == [3, 3, 3]


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("kind", ["all_equal", "two_valued", "ints", "sample_high",
                                  "sample_low", "dense_cluster"])
def test_candidate_route_fallbacks(dtype, kind):
    """Inputs that defeat the sampled pre-threshold: huge tie classes (every entry is a
    candidate, the slots overflow), samples that are all larger / all smaller than the
    rest, and a cluster denser than the slots of its chunk."""
    _announce("fallback %s dtype=%d" % (kind, dtype))
    rng = np.random.default_rng(21)
    n = 400_000 + 24
    vec = 4 if dtype == G.F32 else 8
    if kind == "all_equal":
        v = np.full(n, -0.25, np.float32)
    elif kind == "two_valued":
        v = rng.choice([-1.0, 2.0], n).astype(np.float32)
    elif kind == "ints":
        v = rng.integers(-50, 51, n).astype(np.float32)
    else:
        v = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        nvec = n // vec
        stride = nvec // 4096
        sampled = (np.arange(4096) * stride + stride // 2)[:, None] * vec + np.arange(vec)
        if kind == "sample_high":       # the sample sees only the largest values
            v[sampled.ravel()] = rng.choice([-1.0, 1.0], sampled.size) * 0.5
        elif kind == "sample_low":      # the sample sees only tiny values (10 octaves down;
            v[sampled.ravel()] *= 1e-3  # the candidate histogram spans 12)
        else:                           # 3000 large values inside one 2048-entry chunk
            v[100_000:103_000] = rng.choice([-1.0, 1.0], 3000) * (0.1 + rng.random(3000))
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    # the sample covers 4 % of the entries: it only misleads when more than that is kept
    keep = 100_000 if kind == "sample_high" else 10_000
    b = G.Bucket("fb", dtype, 2, [G.Seg(0, n, keep, 1, "w")], n, 3000)
    grads = [torch.from_numpy(v).to(td), torch.from_numpy(np.roll(v, 7777)).to(td)]
    ores, tb = run_both(b, grads, seed=2)
    # (the planted values are 50 to 500 times the rest: entries that share cells with them
    # carry float32 rounding of that scale, see tests/helpers.py)
    compare_all(b, ores, tb, exact_values=kind in ("all_equal", "two_valued", "ints"),
                mixed_ceiling=0.1)
    # Whether the shortcut was abandoned.  A pre-threshold that is merely far too low is
    # not a reason any more: the scan raises it as it goes.  Tie classes larger than the
    # slots, and a cluster that drives one wave's pre-threshold above the true threshold,
    # still are.  (With "ints" the 2 % tie class at the threshold fits the slots.)
    if kind != "ints":
        assert tb.rank_counts(0)["dense_segments"] == (0 if kind == "sample_low" else 1)


def test_buckets_in_flight_on_separate_streams():
    """Three different buckets issued round-robin on three HIP streams, three rounds
    each, with both sparsifier routes and several super-chunks in play: every bucket
    must come out as it does alone (no state shared between plans, no kernel that
    needs the device to itself)."""
    from paper_2504_05638_amd.bucket import TagcBucket
    from tests.helpers import oracle_config, oracle_segments
    _announce("three buckets in flight")
    routes = G.Bucket("routes", G.BF16, 3,
                      [G.Seg(0, (1 << 18) + 13, 10_000, 1, "long_ragged"),
                       G.Seg(262_168, 5000, 20_000, 1, "short"),
                       G.Seg(267_176, (1 << 17), 25_000, 1, "long_dense_keep"),
                       G.Seg(398_251, (1 << 17) + 64, 10_000, 1, "long_unaligned"),
                       G.Seg(529_392, 300_000, 100, 1, "long_tiny_k")], 829_392, 1500,
                      {"long_ragged": 1e-3, "short": 1e-2, "long_dense_keep": 1e-4,
                       "long_unaligned": 3e-3, "long_tiny_k": 1e-3})
    buckets = [routes, G.config1(seed=4, n=(1 << 22) + 777, n_ranks=3),
               G.small_mixed_bucket(seed=8, dtype=G.BF16, n_ranks=3, sizing_milli=2000)]
    grads = [_grads(b) for b in buckets]
    dev = [[g.cuda() for g in gs] for gs in grads]
    tbs = [TagcBucket(b.segments, b.dtype, b.n_ranks, sizing_milli=b.sizing_milli, seed=11 + i,
                      dense=True) for i, b in enumerate(buckets)]
    streams = [torch.cuda.Stream() for _ in buckets]
    torch.cuda.synchronize()
    for _ in range(3):
        for tb, d, s in zip(tbs, dev, streams):
            tb.run(d, s)
    torch.cuda.synchronize()
    for i, (b, gs, tb) in enumerate(zip(buckets, grads, tbs)):
        ores = O.run_bucket([G.to_numpy_raw(g) for g in gs], oracle_config(b, seed=11 + i),
                            oracle_segments(b))
        compare_all(b, ores, tb)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_ordered_output_over_many_items_per_segment(dtype):
    """The sparsifier's last two kernels order their output through per-item counts (count,
    then place): same pairs, same Index as the oracle on the candidate route (many
    super-chunks per segment, ties at the threshold) and on the dense route (many tiles per
    segment, ragged and unaligned ones, one that keeps two entries in five), twice in a row
    on the same buffers (the counters the kernels keep in the plan's table must be back at
    zero)."""
    _announce("ordered output dtype=%d" % dtype)
    segs = [G.Seg(0, (1 << 21) + 13, 10_000, 1, "long_ragged"),
            G.Seg(2_097_176, 5000, 20_000, 1, "short"),
            G.Seg(2_102_184, (1 << 20), 400_000, 1, "keeps_two_fifths"),
            G.Seg(3_150_763, (1 << 19) + 64, 10_000, 1, "long_unaligned"),
            G.Seg(3_675_120, 3 << 20, 12_500, 1, "long")]
    n = 3_675_120 + (3 << 20)
    b = G.Bucket("ordered", dtype, 2, segs, n, 1500,
                 {"long_ragged": 1e-3, "short": 1e-2, "keeps_two_fifths": 1e-4,
                  "long_unaligned": 3e-3, "long": 1e-3})
    grads = _grads(b)
    ores, tb = run_both(b, grads, seed=6)
    compare_all(b, ores, tb)
    assert tb.rank_counts(0)["dense_segments"] == 3
    tb.run([g.cuda() for g in grads])          # again, now from carried pre-thresholds
    torch.cuda.synchronize()
    compare_all(b, ores, tb)
    assert tb.rank_counts(1)["dense_segments"] == 3
    # integers: heavy ties at every threshold, bit for bit
    rng = np.random.default_rng(5)
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = [torch.from_numpy(rng.integers(-40, 41, n).astype(np.float32)).to(td)
             for _ in range(2)]
    ores, tb = run_both(b, grads, seed=7)
    compare_all(b, ores, tb, exact_values=True)


@pytest.mark.parametrize("wgs", [1, 4, 64])
def test_decode_on_a_limited_number_of_workgroups(wgs):
    """A caller with other buckets in flight limits the peeling kernel's grid; a workgroup
    then takes several partitions in turn (18 here, so 1 -> all of them, 4 -> a ragged
    deal, 64 -> some workgroups idle).  Integer inputs: bit for bit, sparse and dense;
    then the same buffers decoded by the sibling plan without the limit."""
    _announce("decode_workgroups=%d" % wgs)
    rng = np.random.default_rng(21)
    n, N = 400_000, 4
    segs = [G.Seg(0, 150_000, 30_000, 1, "a"), G.Seg(150_000, 250_000, 20_000, 1, "b")]
    b = G.Bucket("ints", G.BF16, N, segs, n, 1500)
    grads = [torch.from_numpy(rng.integers(-100, 101, n).astype(np.float32)).to(torch.bfloat16)
             for _ in range(N)]
    ores, tb = run_both(b, grads, seed=2, P=2048, T=3072, decode_workgroups=wgs)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    assert hdr["A"] > 16 and hdr["A"] % 4 and st["n_unresolved"] == 0
    nv, nd = 4 * hdr["U"], 4 * tb.sizes.n_c      # bytes the decoder writes
    f32 = lambda t, nb: t[:nb].view(torch.float32)   # as numbers: a sum that cancels may
    val, dense = f32(tb.out_val, nv).clone(), f32(tb.out_dense, nd).clone()  # be +0 or -0
    tb.out_val.zero_()
    tb.out_dense.zero_()
    tb.decompress(whole_device=True)
    torch.cuda.synchronize()
    assert torch.equal(f32(tb.out_val, nv), val) and torch.equal(f32(tb.out_dense, nd), dense)
    # random floats too, against the oracle within the usual tolerance
    b2 = G.small_mixed_bucket(seed=5, dtype=G.F32, n_ranks=3, sizing_milli=1500)
    ores, tb = run_both(b2, _grads(b2), seed=6, P=256, T=768, decode_workgroups=wgs)
    compare_all(b2, ores, tb)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_pre_threshold_carried_between_calls_never_changes_results(dtype):
    """A plan keeps each segment's pre-threshold from one PHASE_INDEX call to the next.
    Here consecutive calls see the same distribution (the hint holds), then gradients 100x
    larger (far too many candidates for the slots), then 10000x smaller (no
    candidate at all), then the first scale again with one rank that is mostly zeros.
    Whatever the hint is worth, every rank's survivors must be exactly the oracle's."""
    _announce("pre-threshold hints dtype=%d" % dtype)
    n = (1 << 19) + 40
    rng = np.random.default_rng(77)
    scales = [1e-3, 1e-3, 1e-1, 1e-5, 1e-3, 1e-3, 1e-3]
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = []
    for r, sc in enumerate(scales):
        v = (rng.standard_normal(n) * sc).astype(np.float32)
        if r == 4:
            v[rng.random(n) < 0.97] = 0.0   # fewer non-zeros than the sample can judge
        grads.append(torch.from_numpy(v).to(td))
    b = G.Bucket("hints", dtype, len(scales), [G.Seg(0, n, 10_000, 1, "w")], n, 3000)
    ores, tb = run_both(b, grads, seed=9)
    # (ranks whose scales differ by 100 and 10^4 share cells: more entries than usual carry
    # the float32 rounding of far larger ones)
    compare_all(b, ores, tb, mixed_ceiling=0.05)
    dense = [tb.rank_counts(r)["dense_segments"] for r in range(len(scales))]
    assert dense[0] == 0 and dense[1] == 0      # sampled, then the carried hint
    assert dense[2] == 0      # hint far too low: the scan raises it as it goes
    assert dense[3] == 1      # hint far too high, no candidates: exact two-read fallback
    assert dense[6] == 0                        # and recovered (rank 5 still pays for rank 4)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_falling_scale_costs_one_fallback_not_one_per_call(dtype):
    """Every call sees gradients 12 % smaller than the one before: the carried pre-threshold
    is too high each time.  The first such call falls back to the two-read route; after it
    the plan lowers the carried value by what it fell since the call before, for a few
    calls, so the following calls do not.  Results exact throughout."""
    _announce("falling scale dtype=%d" % dtype)
    n = (1 << 19) + 40
    rng = np.random.default_rng(5)
    scales = [1e-3 * 0.88 ** r for r in range(7)]
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = [torch.from_numpy((rng.standard_normal(n) * sc).astype(np.float32)).to(td)
             for sc in scales]
    b = G.Bucket("falling", dtype, len(scales), [G.Seg(0, n, 10_000, 1, "w")], n, 3000)
    ores, tb = run_both(b, grads, seed=4)
    compare_all(b, ores, tb)
    dense = [tb.rank_counts(r)["dense_segments"] for r in range(len(scales))]
    assert dense == [0, 1, 0, 0, 0, 0, 0]


@pytest.mark.parametrize("keep_lo,keep_hi", [(5_000, 30_000), (60_000, 220_000)])
def test_more_than_64_candidate_route_segments(keep_lo, keep_hi):
    """70 segments that all take the candidate route (the final kernel reads the segment
    tables lane-parallel for up to 64 segments and falls back to a search beyond), with
    ragged lengths so that super-chunks end inside chunks, and varying keep ratios: a few
    per cent (dozens of candidates per chunk) and Table 1's dense regimes (hundreds: the
    last two kernels then give a wave to every super-chunk)."""
    _announce("70 fast segments, keep %d-%d ppm" % (keep_lo, keep_hi))
    rng = np.random.default_rng(5)
    segs, sigma, off = [], {}, 0
    for i in range(70):
        n = (1 << 17) + int(rng.integers(0, 5000))
        name = "s%d" % i
        keep = int(rng.integers(keep_lo, keep_hi))
        if keep_lo >= 50_000 and i % 5 == 4:
            keep = 10_000   # (one read per chunk among segments that need several)
        segs.append(G.Seg(off, n, keep, 1, name))
        sigma[name] = float(10 ** rng.uniform(-4, -2))
        off = (off + n + 7) // 8 * 8
    b = G.Bucket("many", G.BF16, 2, segs, off, 1500, sigma)
    ores, tb = run_both(b, _grads(b), seed=13)
    compare_all(b, ores, tb)
    assert [tb.rank_counts(r)["dense_segments"] for r in range(2)] == [0, 0]


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("keep_ppm", [50_000, 100_000, 200_000])
def test_hundreds_of_candidates_per_chunk(dtype, keep_ppm):
    """Table 1's dense regimes on the candidate route: a twentieth, a tenth and a fifth of
    the entries kept, so that a 4 KiB chunk holds hundreds of candidates (slots staged per
    wave at the lower two ratios, written in place at the highest; count and place with a
    wave per super-chunk).  Several super-chunks per segment, a ragged tail, one segment
    of small integers (a tie class at the threshold that spans chunks and super-chunks, so
    the quota of ties runs out in the middle of a read), two segments that keep one entry
    in a hundred among them (a few dozen candidates per chunk, one read per chunk; one of
    them small integers again), one short segment on the dense route; twice on the same
    buffers, the second time from carried pre-thresholds."""
    _announce("wide emit dtype=%d keep=%d" % (dtype, keep_ppm))
    a = (1 << 19) + 4099
    o1 = (a + 7) // 8 * 8
    o2 = o1 + (3 << 17)
    o3 = o2 + 40_000
    o4 = o3 + (1 << 18) + 8
    n = o4 + (1 << 18) + 24
    segs = [G.Seg(0, a, keep_ppm, 1, "ragged"),
            G.Seg(o1, 3 << 17, keep_ppm, 1, "ints"),
            G.Seg(o2, 40_000, keep_ppm, 1, "short"),
            G.Seg(o3, (1 << 18) + 8, 10_000, 1, "sparse"),
            G.Seg(o4, (1 << 18) + 24, 10_000, 1, "sparse_ints")]
    b = G.Bucket("wide", dtype, 2, segs, n, 1500,
                 {"ragged": 1e-3, "ints": 1.0, "short": 1e-3, "sparse": 2e-3,
                  "sparse_ints": 1.0})
    rng = np.random.default_rng(keep_ppm + dtype)
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = []
    for g in _grads(b):
        v = g.to(torch.float32).numpy().copy()
        v[o1:o2] = rng.integers(-40, 41, o2 - o1).astype(np.float32)
        # (one entry in a hundred kept of 81 equally likely values: the threshold class is
        # two and a half times the quota, a few dozen candidates per chunk)
        v[o4:n] = rng.integers(-40, 41, n - o4).astype(np.float32)
        grads.append(torch.from_numpy(v).to(td))
    ores, tb = run_both(b, grads, seed=17)
    compare_all(b, ores, tb, mixed_ceiling=0.02)   # (unit-scale integers beside 1e-3 values)
    assert [tb.rank_counts(r)["dense_segments"] for r in range(2)] == [1, 1]
    tb.run([g.cuda() for g in grads])
    torch.cuda.synchronize()
    compare_all(b, ores, tb, mixed_ceiling=0.02)
    assert [tb.rank_counts(r)["dense_segments"] for r in range(2)] == [1, 1]
