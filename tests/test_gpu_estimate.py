"""GPU parity for the estimation decode (section 2.2: the second decompression algorithm):
the residue of a stalled peeling estimated from the cells as peeling left them, and
estimation alone on the summed sketch, against the oracle, through the C ABI."""
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
@pytest.mark.parametrize("mode", [O.DECODE_PEEL_ESTIMATE, O.DECODE_ESTIMATE])
def test_undersized_sketch_mixed_bucket(dtype, mode):
    """Load factor 1.15, several partitions, ragged segments: part of every partition
    peels, the rest is estimated (mode 1), or everything is (mode 2)."""
    _announce("estimate mixed dtype=%d mode=%d" % (dtype, mode))
    b = G.small_mixed_bucket(seed=3, dtype=dtype, n_ranks=3, sizing_milli=1150)
    ores, tb = run_both(b, _grads(b), seed=5, P=256, T=768, decode_mode=mode)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["A"] > 1 and st["n_estimated"] == st["n_unresolved"] > 0
    if mode == O.DECODE_ESTIMATE:
        assert st["n_estimated"] == hdr["U"] and st["rounds"] == 0


@pytest.mark.parametrize("mode", [O.DECODE_PEEL_ESTIMATE, O.DECODE_ESTIMATE])
def test_integer_values_estimates_are_bit_exact(mode):
    """Small integers: every cell, residual cell and reading is exact in float32, so the
    estimates must agree exactly whatever order the adds and subtracts took."""
    _announce("estimate ints mode=%d" % mode)
    N, n = 4, 300_000
    segs = [G.Seg(0, 100_000, 30_000, 1, "a"), G.Seg(100_000, 200_000, 20_000, 1, "b")]
    b = G.Bucket("ints", G.F32, N, segs, n, 1100)
    rng = np.random.default_rng(21)
    grads = [torch.from_numpy(rng.integers(-100, 101, n).astype(np.float32)) for _ in range(N)]
    ores, tb = run_both(b, grads, seed=2, P=1024, T=3072, decode_mode=mode)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    assert st["n_estimated"] > 0.2 * hdr["U"]


def test_fixed_ratio_dense_regime_estimation_only():
    """The regime the paper says peeling cannot serve (section 2.2): 2x compression of a
    gradient that is only 50 % sparse -- one cell per non-zero.  Estimation alone decodes
    it, noisily; the library's estimates are the oracle's."""
    _announce("estimate dense regime")
    n = 400_000
    b = G.Bucket("dense2x", G.F32, 2, [G.Seg(0, n, 300_000, 1, "w")], n, 2000)
    ores, tb = run_both(b, _grads(b), seed=3, sizing=O.SIZE_FIXED_RATIO,
                        decode_mode=O.DECODE_ESTIMATE)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_estimated"] == hdr["U"] > 0.4 * n


def test_estimation_is_idle_when_peeling_succeeds():
    _announce("estimate idle")
    b = G.config1(seed=1, n=200_000, n_ranks=2)
    ores, tb = run_both(b, _grads(b), seed=0, P=1024, T=3072,
                        decode_mode=O.DECODE_PEEL_ESTIMATE)
    hdr, st = compare_all(b, ores, tb)
    assert st["n_unresolved"] == 0 and st["n_estimated"] == 0
