"""GPU parity for tagc_reduce_decompress: the Reduce of the sketches (Algorithm 1) done by
the decoder itself, against the oracle's sum followed by its peel, and against the library's
own two-call path, through the C ABI."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from paper_2504_05638_amd import binding as B
from tests.helpers import run_both, compare_all

pytestmark = pytest.mark.gpu


def _grads(bucket, gen=G.rank_gradient):
    return [gen(bucket, r, "cpu") for r in range(bucket.n_ranks)]


def _announce(name):
    print("\n[case] %s" % name, flush=True)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("lf", [1500, 3000])
def test_small_mixed_bucket_fused(dtype, lf):
    """Several small partitions (a workgroup takes many in turn, so every partition but its
    first is summed while the one before is peeled), ragged segments, 3 ranks."""
    _announce("fused small_mixed dtype=%d lf=%d" % (dtype, lf))
    b = G.small_mixed_bucket(seed=3, dtype=dtype, n_ranks=3, sizing_milli=lf)
    ores, tb = run_both(b, _grads(b), seed=5, P=256, T=768, fused=True)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["A"] > 1 and st["n_unresolved"] == 0


@pytest.mark.parametrize("n_ranks", [1, 2, 5, 16, 32])
def test_integer_values_bit_exact_for_any_number_of_ranks(n_ranks):
    """Small integers: every float32 add is exact, so the fused path must agree bit for bit
    with the oracle and with the two-call path, for one rank (nothing to add), odd and even
    numbers, and the most the call takes."""
    _announce("fused integer exact ranks=%d" % n_ranks)
    rng = np.random.default_rng(40 + n_ranks)
    n = 200_000
    segs = [G.Seg(0, 120_000, 20_000, 1, "a"), G.Seg(120_000, 80_000, 30_000, 1, "b")]
    b = G.Bucket("ints", G.BF16, n_ranks, segs, n, 1500)
    grads = [torch.from_numpy(rng.integers(-60, 61, n).astype(np.float32)).to(torch.bfloat16)
             for _ in range(n_ranks)]
    ores, tb = run_both(b, grads, seed=2, P=1024, T=3072, fused=True)
    compare_all(b, ores, tb, exact_values=True)
    idx_f, val_f = tb.outputs()
    dense_f = tb.dense()
    st_f = tb.status()
    # the same buffers through tagc_aggregate(PHASE_SKETCH) + tagc_decompress
    tb.sh_status.zero_()
    tb.aggregate_sketch(n_ranks)
    tb.decompress()
    torch.cuda.synchronize()
    idx_u, val_u = tb.outputs()
    assert np.array_equal(idx_f, idx_u) and np.array_equal(val_f, val_u)
    assert np.array_equal(dense_f, tb.dense())
    assert st_f == tb.status()
    assert np.array_equal(tb.shared_sketch(), ores.sketch[:tb.header()["m"]])


def test_config1_on_three_workgroups():
    """Benchmark configuration 1 (fp32, 4 ranks), the decoder on 3 workgroups: each sums and
    peels several full-size partitions in a row."""
    _announce("fused config1")
    b = G.config1(seed=0)
    ores, tb = run_both(b, _grads(b), seed=0, fused=True, decode_workgroups=3)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["A"] >= 6 and st["n_unresolved"] == 0


@pytest.mark.parametrize("mode", [O.DECODE_PEEL_ESTIMATE, O.DECODE_ESTIMATE])
def test_estimation_modes_fused(mode):
    """Estimation of what peeling leaves, and estimation alone, on an undersized sketch."""
    _announce("fused estimate mode=%d" % mode)
    b = G.small_mixed_bucket(seed=3, dtype=G.BF16, n_ranks=3, sizing_milli=1150)
    ores, tb = run_both(b, _grads(b), seed=5, P=256, T=768, decode_mode=mode, fused=True)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_estimated"] == st["n_unresolved"] > 0


def test_heavy_tailed_many_partitions_fused():
    """bf16 Student-t values with half-shared supports (configuration 3 at reduced length):
    full-size partitions whose cell count is not a multiple of anything convenient, 4 ranks."""
    _announce("fused config3 reduced")
    b = G.config3(seed=0, n=(1 << 21) + 4321, n_ranks=4, keep_ppm=10_000, sizing_milli=1500)
    grads = [G.config3_rank_gradient(b, r, "cpu") for r in range(4)]
    ores, tb = run_both(b, grads, seed=0, fused=True)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_unresolved"] == 0


@pytest.mark.parametrize("ratio_milli,theta_ppm", [(4000, 100_000), (10_000, 12_500)])
def test_fixed_ratio_sketch_two_ranks_fused(ratio_milli, theta_ppm):
    """Table 1's regimes (sketch of n / c cells, 2 ranks): the 4x one peels close to the
    threshold over some twenty rounds, each with the peelers' own barrier."""
    _announce("fused fixed ratio %d" % ratio_milli)
    n = 600_000
    b = G.Bucket("t1", G.F32, 2, [G.Seg(0, n, theta_ppm, 1, "w")], n, ratio_milli)
    grads = [torch.from_numpy((np.random.default_rng(70 + r).standard_normal(n) * 1e-3)
                              .astype(np.float32)) for r in range(2)]
    ores, tb = run_both(b, grads, seed=3, sizing=O.SIZE_FIXED_RATIO, fused=True)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_unresolved"] == 0 and hdr["m"] <= n * 1000 // ratio_milli


def test_repeated_calls_give_the_same_result():
    """The loaders and the peelers of a workgroup meet at barriers of two kinds; nothing may
    depend on who gets there first: twenty calls on the same buffers, the same integers out."""
    _announce("fused repeated")
    b = G.config3(seed=1, n=(1 << 20) + 77, n_ranks=6, keep_ppm=20_000, sizing_milli=1500)
    grads = [G.config3_rank_gradient(b, r, "cpu") for r in range(6)]
    ores, tb = run_both(b, grads, seed=3, fused=True)
    compare_all(b, ores, tb)
    idx0, val0 = tb.outputs()
    st0 = tb.status()
    for _ in range(20):
        tb.sh_status.zero_()
        tb.reduce_decompress(6)
        torch.cuda.synchronize()
        idx, val = tb.outputs()
        assert np.array_equal(idx, idx0) and tb.status() == st0
        assert np.array_equal(val == 0, val0 == 0)
        assert np.allclose(val, val0, rtol=1e-4, atol=1e-9)


def test_empty_bucket_fused():
    """Nothing kept anywhere: U = 0, no partition, nothing to sum."""
    _announce("fused empty")
    n = 4096
    b = G.Bucket("empty", G.F32, 2, [G.Seg(0, n, 0, 1, "w")], n, 1500)
    grads = [torch.zeros(n) for _ in range(2)]
    ores, tb = run_both(b, grads, fused=True)
    compare_all(b, ores, tb, exact_values=True)
    assert tb.header()["U"] == 0


def test_16_bit_cells_are_refused():
    """The fused call reads float32 cells only."""
    _announce("fused refuses bf16 cells")
    b = G.small_mixed_bucket(seed=3, dtype=G.BF16, n_ranks=2, sizing_milli=1500)
    ores, tb = run_both(b, _grads(b), seed=5, P=256, T=768, cell_type=1)
    with pytest.raises(B.TagcError) as e:
        tb.reduce_decompress(2)
    assert e.value.code == -3
