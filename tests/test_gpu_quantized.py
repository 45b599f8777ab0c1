"""GPU parity for 16-bit sketch cells on the wire (section 5: quantised communication):
encode's rounding to bfloat16, the float32 sum of the widened cells, and the unchanged
decode, against the oracle through the C ABI."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import run_both, compare_all

pytestmark = pytest.mark.gpu


def _announce(name):
    print("\n[case] %s" % name, flush=True)


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_small_integers_are_lossless_and_bit_exact(dtype):
    """|v| <= 16 and a handful of entries per cell: every wire cell is a bfloat16 number, so
    rank sketches, summed sketch and decoded values equal the oracle's bit for bit."""
    _announce("bf16 cells ints dtype=%d" % dtype)
    rng = np.random.default_rng(5)
    n, N = 300_000, 5
    segs = [G.Seg(0, 100_000, 30_000, 1, "a"), G.Seg(100_000, 200_000, 20_000, 1, "b")]
    b = G.Bucket("ints16", dtype, N, segs, n, 3000)
    td = torch.float32 if dtype == G.F32 else torch.bfloat16
    grads = [torch.from_numpy(rng.integers(-16, 17, n).astype(np.float32)).to(td)
             for _ in range(N)]
    ores, tb = run_both(b, grads, seed=1, P=2048, T=3 * 2047, cell_type=O.CELL_BF16)
    hdr, st = compare_all(b, ores, tb, exact_values=True)
    assert hdr["A"] > 4 and st["n_unresolved"] == 0
    assert tb.sizes.rank_sketch_bytes * 2 <= tb.sizes.shared_sketch_bytes + 32


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_mixed_bucket_random_values(dtype):
    """Ragged segments and sub-tables whose start is not a multiple of eight cells (the
    unaligned head and tail of the 16-byte stores), random values."""
    _announce("bf16 cells mixed dtype=%d" % dtype)
    b = G.small_mixed_bucket(seed=3, dtype=dtype, n_ranks=3, sizing_milli=1610)
    grads = [G.rank_gradient(b, r, "cpu") for r in range(b.n_ranks)]
    ores, tb = run_both(b, grads, seed=5, P=256, T=768, cell_type=O.CELL_BF16)
    hdr, st = compare_all(b, ores, tb)
    assert hdr["A"] > 1 and hdr["m_sub"] % 8 != 0


def test_config1_many_partitions_forty_ranks():
    """More ranks than one launch of the sum takes, several hundred partitions."""
    _announce("bf16 cells config1 40 ranks")
    b = G.config1(seed=4, n=(1 << 19) + 777, n_ranks=40)
    grads = [G.rank_gradient(b, r, "cpu") for r in range(b.n_ranks)]
    ores, tb = run_both(b, grads, seed=1, P=1024, T=3072, cell_type=O.CELL_BF16)
    compare_all(b, ores, tb)
