"""CPU pins for the oracle's error-feedback step (Algorithm 1, lines 1-2; section 3.2,
local gradient accumulation): the add in the gradient's own type against torch's bf16 /
fp32 add, the conservation law summed = sent + acc_next, and the property that makes
accumulation worth having: nothing is lost over time."""
import numpy as np
import pytest
import torch

from oracle import tagc_oracle as O
from synth import gradients as G


def _raw(t):
    return G.to_numpy_raw(t)


def _seg(n, ppm=10_000):
    return [O.Segment(0, n, ppm, 1)]


@pytest.mark.parametrize("dtype,td", [(O.F32, torch.float32), (O.BF16, torch.bfloat16)])
def test_accumulate_is_the_add_of_the_gradient_type(dtype, td):
    """g + acc in the gradient's type: torch's own add on tensors of that type is the
    library routine the step reduces to (bf16: float32 add, round to nearest even).
    The values include exact ties of the bf16 rounding and sums that cancel."""
    rng = np.random.default_rng(3)
    n = 20_000
    g = torch.from_numpy((rng.standard_normal(n) * 1e-2).astype(np.float32)).to(td)
    a = torch.from_numpy((rng.standard_normal(n) * 1e-3).astype(np.float32)).to(td)
    if dtype == O.BF16:
        # 1 + 2^-8 and 1 + 3*2^-8 are ties between two bf16 neighbours: even mantissa wins
        g[:4] = torch.tensor([1.0, 1.0, -1.0, 256.0]).to(td)
        a[:4] = torch.tensor([2.0 ** -8, 3 * 2.0 ** -8, -2.0 ** -8, 1.0]).to(td)
    g[4], a[4] = 0.375, -0.375
    cfg = O.Config(dtype=dtype, sizing_milli=3000, seed=0)
    st, acc_next = O.error_feedback_step(_raw(g), _raw(a), cfg, _seg(n, 1_000_000))
    want = _raw(g + a)          # keep everything: the pairs are the sums themselves
    got = np.zeros(n, np.float32)
    got[st.idx] = st.val
    ref = (g + a).to(torch.float32).numpy()
    nz = ref != 0
    assert np.array_equal(got[nz].view(np.uint32), ref[nz].view(np.uint32))
    if dtype == O.BF16:
        assert ref[0] == 1.0 and ref[1] == 1.015625 and ref[2] == -1.0 and ref[3] == 256.0
    # everything non-zero was sent, so nothing is left behind
    assert not np.any(acc_next.view(np.uint16 if dtype == O.BF16 else np.uint32)[:n][nz])
    assert want.shape == acc_next.shape


@pytest.mark.parametrize("dtype,td", [(O.F32, torch.float32), (O.BF16, torch.bfloat16)])
def test_sent_plus_residual_is_the_sum(dtype, td):
    """summed = sent + acc_next element by element, acc_next is zero exactly at the
    selected positions, and the selected ones are the k largest of |g + acc|."""
    rng = np.random.default_rng(8)
    n = 30_000
    g = torch.from_numpy((rng.standard_normal(n) * 1e-2).astype(np.float32)).to(td)
    a = torch.from_numpy((rng.standard_normal(n) * 1e-2).astype(np.float32)).to(td)
    cfg = O.Config(dtype=dtype, sizing_milli=3000, seed=0)
    st, acc_next = O.error_feedback_step(_raw(g), _raw(a), cfg, _seg(n, 50_000))
    summed = (g + a).to(torch.float32).numpy()
    resid = torch.from_numpy(acc_next.view(np.int16 if dtype == O.BF16 else np.float32).copy())
    resid = (resid.view(torch.bfloat16) if dtype == O.BF16 else resid).to(torch.float32).numpy()
    sent = np.zeros(n, np.float32)
    sent[st.idx] = st.val
    assert st.cnt == 1500
    assert np.array_equal(sent + resid, summed)
    assert not np.any(resid[st.idx]) and np.array_equal(resid[sent == 0], summed[sent == 0])
    order = np.lexsort((np.arange(n), -np.abs(summed)))[:1500]
    assert np.array_equal(np.sort(order), st.idx)


def test_nothing_is_lost_over_steps():
    """With a constant integer-valued gradient every add is exact: after T steps the sum of
    everything sent plus the accumulator equals T times the gradient, and every entry has
    been sent at least once when T is a few times mean|g| / (keep * min|g|) (section 3.2: accumulation avoids losing
    the gradients that were set to zero)."""
    rng = np.random.default_rng(4)
    n, T = 4000, 100
    g = rng.integers(1, 5, n).astype(np.float32) * rng.choice([-1.0, 1.0], n).astype(np.float32)
    cfg = O.Config(dtype=O.F32, sizing_milli=3000, seed=0)
    acc = np.zeros(n, np.float32)
    total = np.zeros(n, np.float64)
    touched = np.zeros(n, bool)
    for _ in range(T):
        st, acc = O.error_feedback_step(g, acc, cfg, _seg(n, 100_000))
        assert st.cnt == 400
        total[st.idx] += st.val
        touched[st.idx] = True
    assert np.array_equal(total + acc, T * g.astype(np.float64))
    assert touched.all()


def test_segments_outside_the_compressed_set_are_left_alone():
    n = 3000
    rng = np.random.default_rng(5)
    g = rng.standard_normal(n).astype(np.float32)
    a = rng.standard_normal(n).astype(np.float32)
    segs = [O.Segment(0, 1000, 100_000, 1), O.Segment(1000, 1000, 0, 0),
            O.Segment(2000, 1000, 0, 1)]   # compressed / skipped / compressed with k = 0
    cfg = O.Config(dtype=O.F32, sizing_milli=3000, seed=0)
    st, nxt = O.error_feedback_step(g, a, cfg, segs)
    assert st.seg_cnt == [100, 0, 0]
    assert np.array_equal(nxt[1000:2000], a[1000:2000])           # untouched
    assert np.array_equal(nxt[2000:], (g + a)[2000:])             # nothing sent: all kept
