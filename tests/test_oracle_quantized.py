"""CPU pins for the oracle's 16-bit sketch cells (section 5 names quantising what is
communicated, e.g. to bfloat16, as the next step beyond the float32-only implementation):
the rounding against torch's own bfloat16 conversion, losslessness whenever every rank's
cells are bfloat16 numbers anyway (checked against the definition of the summed gradient),
and the size of the error otherwise."""
import numpy as np
import pytest
import torch

from oracle import tagc_oracle as O
from oracle import definition as D


def test_cell_rounding_is_torchs_bfloat16_conversion():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200_000) * np.exp(rng.uniform(-20, 20, 200_000))).astype(np.float32)
    # exact ties between two bfloat16 neighbours, both parities, both signs; zeros; tiny values
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 256.0 + 1.0,
                     256.0 + 3.0, 0.0, -0.0, 1e-40, -3e-39], np.float32)
    x[:ties.size] = ties
    got = O.quantize_cells_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert got[0] == 1.0 and got[1] == 1.015625 and got[3] == 256.0 and got[4] == 260.0


def _ranks(rng, n, N, lo, hi, density):
    out = []
    for _ in range(N):
        v = rng.integers(lo, hi + 1, n).astype(np.float32)
        v *= rng.random(n) < density
        out.append(v)
    return out


def test_lossless_when_every_cell_is_a_bfloat16_number():
    """Integers of magnitude <= 16, at most a handful per cell: every rank's cell is an
    integer below 256 and survives the rounding, so the decoded sum is the definition's."""
    rng = np.random.default_rng(1)
    n, N = 40_000, 6
    segs = [O.Segment(0, n, 1_000_000)]
    grads = _ranks(rng, n, N, -16, 16, 0.02)
    cfg = O.Config(dtype=O.F32, sizing_milli=3000, seed=5, part_unknowns=512, part_cells=1536,
                   cell_type=O.CELL_BF16)
    res = O.run_bucket(grads, cfg, segs)
    for r in res.ranks:
        assert np.all(np.abs(r.sketch) <= 256) and not np.any(r.sketch.view(np.uint32) & 0xFFFF)
    idx, val = D.sparse_sum(grads, O.F32, segs)
    assert res.decoded.n_unresolved == 0
    assert np.array_equal(res.decoded.idx, idx)
    assert np.array_equal(res.decoded.val.astype(np.float64), val)
    ref = O.run_bucket(grads, O.Config(dtype=O.F32, sizing_milli=3000, seed=5, part_unknowns=512,
                                       part_cells=1536), segs)
    assert np.array_equal(ref.sketch, res.sketch)        # identical to the float32 cells here


@pytest.mark.parametrize("seed", [2, 3])
def test_error_is_of_the_size_of_the_rounding(seed):
    """Random float gradients: the structure of the decode (who is resolved, in which round)
    does not depend on cell values; the values come back with the rounding noise of the
    cells they passed through, 2^-9 relative per cell on average."""
    rng = np.random.default_rng(seed)
    n, N = 60_000, 4
    segs = [O.Segment(0, n, 20_000)]
    grads = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(N)]
    base = dict(dtype=O.F32, sizing_milli=1500, seed=seed, part_unknowns=512, part_cells=1536)
    exact = O.run_bucket(grads, O.Config(**base), segs)
    quant = O.run_bucket(grads, O.Config(cell_type=O.CELL_BF16, **base), segs)
    assert np.array_equal(exact.decoded.idx, quant.decoded.idx)
    assert np.array_equal(exact.decoded.round, quant.decoded.round)
    assert exact.decoded.rounds == quant.decoded.rounds > 3
    ok = exact.decoded.round > 0
    err = np.abs(quant.decoded.val.astype(np.float64) - exact.decoded.val)[ok]
    scale = np.abs(exact.decoded.val[ok]).max()
    assert 2.0 ** -12 < np.median(err) / np.median(np.abs(exact.decoded.val[ok])) < 2.0 ** -6
    assert err.max() < 0.05 * scale                       # no blow-up along peeling chains
    # the wire cells are bfloat16 numbers; the summed sketch is float32 again
    assert not np.any(quant.ranks[0].sketch.view(np.uint32) & 0xFFFF)
    assert np.any(quant.sketch.view(np.uint32) & 0xFFFF)
