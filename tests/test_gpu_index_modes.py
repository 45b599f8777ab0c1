"""GPU parity for the addition-simulated Index All-Reduce (section 2.2): 1-bit wire Index
with its carries, 4-bit counters (wire Index four times bigger, exact up to 15 ranks,
overflowing beyond), and the encode restricted to the merged Index, against the oracle
through the C ABI; every stage bit-exact or within tolerance as for the OR."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import run_both, compare_all

pytestmark = pytest.mark.gpu


def _grads(bucket):
    return [G.rank_gradient(bucket, r, "cpu") for r in range(bucket.n_ranks)]


def _announce(name):
    print("\n[case] %s" % name, flush=True)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("mode", [O.INDEX_ADD1, O.INDEX_ADD4])
def test_small_mixed_bucket(dtype, mode):
    _announce("index mode %d dtype=%d mixed" % (mode, dtype))
    b = G.small_mixed_bucket(seed=3, dtype=dtype, n_ranks=3, sizing_milli=1500)
    ores, tb = run_both(b, _grads(b), seed=5, P=256, T=768, index_mode=mode)
    hdr, st = compare_all(b, ores, tb)
    true_or, U_or = O.index_or([r.bitmap for r in ores.ranks])
    if mode == O.INDEX_ADD4:
        assert np.array_equal(ores.bitmap, true_or)          # 3 ranks: counters cannot overflow
        assert tb.sizes.rank_bitmap_bytes >= 4 * 4 * tb.sizes.bitmap_words
    else:
        assert not np.array_equal(ores.bitmap, true_or)      # overlapping supports collide


@pytest.mark.parametrize("mode", [O.INDEX_ADD1, O.INDEX_ADD4])
def test_config1_overlapping_supports(mode):
    """Half of each rank's support shared with the others (config1's recipe): the 1-bit
    sum loses those positions and flips their neighbours; several partitions, ragged tail."""
    _announce("index mode %d config1" % mode)
    b = G.config1(seed=4, n=(1 << 20) + 777, n_ranks=4)
    ores, tb = run_both(b, _grads(b), seed=1, P=2048, T=3072, index_mode=mode)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["A"] > 4


@pytest.mark.parametrize("mode", [O.INDEX_ADD1, O.INDEX_ADD4])
def test_twenty_ranks_integer_values_bit_exact(mode):
    """20 ranks: 4-bit counters overflow where exactly 16 ranks keep a position (planted),
    and invent the position after it.  Integer values: everything exact."""
    _announce("index mode %d 20 ranks" % mode)
    rng = np.random.default_rng(7)
    n, N = 200_000, 20
    segs = [G.Seg(0, n, 50_000, 1, "w")]
    b = G.Bucket("ranks20", G.F32, N, segs, n, 3000)
    hot = rng.choice(n, 500, replace=False)
    grads = []
    for r in range(N):
        g = rng.integers(-50, 51, n).astype(np.float32)
        g[hot] = 1000 + r if r < 16 else 0
        grads.append(torch.from_numpy(g))
    ores, tb = run_both(b, grads, seed=3, P=1024, T=3072, index_mode=mode)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    true_or, _ = O.index_or([r.bitmap for r in ores.ranks])
    assert not np.array_equal(ores.bitmap, true_or)
    assert st["n_unresolved"] == 0


def test_four_bit_counters_more_ranks_than_one_pass():
    """40 ranks: the counters are summed in two launches with the running sum kept in the
    shared workspace."""
    _announce("index mode 4-bit 40 ranks")
    rng = np.random.default_rng(9)
    n, N = 70_000, 40
    b = G.Bucket("ranks40", G.F32, N, [G.Seg(0, n, 100_000, 1, "w")], n, 3000)
    grads = [torch.from_numpy(rng.integers(-50, 51, n).astype(np.float32)) for _ in range(N)]
    ores, tb = run_both(b, grads, seed=3, P=1024, T=3072, index_mode=O.INDEX_ADD4)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    assert st["n_unresolved"] == 0
