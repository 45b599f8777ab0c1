"""GPU parity for the error-feedback step (Algorithm 1, lines 1-2; section 3.2): over
several chained steps the survivors, the local Index and the accumulator left behind must
equal the oracle's bit for bit, on both sparsifier routes, through re-routed segments, and
end to end through the sketch."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import oracle_config, oracle_segments, compare_all

pytestmark = pytest.mark.gpu


def _mixed_bucket(dtype, n_ranks):
    """Candidate-route and dense-route segments, an unaligned one, one keeping nothing, a
    skipped one in between."""
    segs = [G.Seg(0, (1 << 18) + 13, 10_000, 1, "long_ragged"),
            G.Seg(262_168, 5000, 20_000, 1, "short"),
            G.Seg(267_176, 4096, 0, 0, "skipped"),
            G.Seg(271_272, (1 << 17), 25_000, 1, "long_dense_keep"),
            G.Seg(402_347, (1 << 17) + 64, 10_000, 1, "long_unaligned"),
            G.Seg(533_488, 300_000, 100, 1, "long_tiny_k"),
            G.Seg(833_488, 1000, 0, 1, "keeps_nothing")]
    sigma = {"long_ragged": 1e-3, "short": 1e-2, "skipped": 1.0, "long_dense_keep": 1e-4,
             "long_unaligned": 3e-3, "long_tiny_k": 1e-3, "keeps_nothing": 1e-2}
    return G.Bucket("ef", dtype, n_ranks, segs, 834_488, 1500, sigma)


def _step_grads(b, step, scale=1.0):
    out = []
    for r in range(b.n_ranks):
        bb = G.Bucket(b.name, b.dtype, b.n_ranks, b.segments, b.n_elems, b.sizing_milli,
                      b.sigma, b.kind, b.seed + 97 * step, b.bucket_id)
        g = G.rank_gradient(bb, r, "cpu")
        out.append((g.to(torch.float32) * scale).to(g.dtype))
    return out


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
@pytest.mark.parametrize("apply_every_step", [False, True])
@pytest.mark.parametrize("index_mode", [O.INDEX_OR1, O.INDEX_ADD4])
def test_error_feedback_chain_matches_oracle(dtype, apply_every_step, index_mode):
    """The library leaves acc_next as (sums everywhere, the rank's Index naming what reads as
    zero); tagc_feedback_apply turns it into the plain array, compared here with the oracle's
    bit for bit -- after every step, or only after the last one, with the same pairs at every
    step either way (the next step does not depend on it).  With 4-bit counters on the wire
    the sent entries are read from the counters."""
    from paper_2504_05638_amd.bucket import TagcBucket
    print("\n[case] error feedback chain dtype=%d apply=%d index_mode=%d"
          % (dtype, apply_every_step, index_mode), flush=True)
    b = _mixed_bucket(dtype, 2)
    cfg = oracle_config(b, seed=3, index_mode=index_mode)
    segs = oracle_segments(b)
    tb = TagcBucket(b.segments, b.dtype, b.n_ranks, sizing_milli=b.sizing_milli, seed=3,
                    dense=True, error_feedback=True, index_mode=index_mode)
    n_steps = 5
    raw0 = np.zeros(b.n_elems, np.uint16 if dtype == G.BF16 else np.float32)
    acc = [raw0.copy() for _ in range(b.n_ranks)]
    # steps 2 and 3 change scale by 100x and 1e-4x: carried pre-thresholds fail, segments are
    # re-routed after the accumulator has already been updated by the streaming pass
    for step, scale in enumerate([1.0, 1.0, 100.0, 1e-4, 1.0]):
        grads = _step_grads(b, step, scale)
        states = []
        for r in range(b.n_ranks):
            st, acc[r] = O.error_feedback_step(G.to_numpy_raw(grads[r]), acc[r], cfg, segs)
            states.append(st)
        tb.run([g.cuda() for g in grads])
        torch.cuda.synchronize()
        for r in range(b.n_ranks):
            cnt = tb.rank_counts(r)
            assert cnt["flags"] == 0
            assert cnt["total"] == states[r].cnt, (step, r)
            idx, val = tb.rank_pairs(r)
            assert np.array_equal(idx, states[r].idx), (step, r)
            assert np.array_equal(val.view(np.uint32), states[r].val.view(np.uint32)), (step, r)
            local = states[r].bitmap[:tb.sizes.bitmap_words]
            assert np.array_equal(tb.rank_bitmap(r), O.index_widen4(local)
                                  if index_mode == O.INDEX_ADD4 else local)
            if apply_every_step or step == n_steps - 1:
                tb.feedback_apply(r)
                tb.feedback_apply(r)            # idempotent
                torch.cuda.synchronize()
                got = tb.rank_acc(r)[:b.n_elems]
                want = acc[r].view(got.dtype)
                assert np.array_equal(got, want), (step, r, int(np.argmax(got != want)))
        # the rest of the path on the same survivors: merged Index, sketch, decode
        bitmap, U = O.merge_index([s.bitmap for s in states], index_mode)
        assert tb.header()["U"] == U


def test_error_feedback_end_to_end_against_oracle_bucket():
    """One step with a non-zero accumulator through the whole path: the decoded sum equals
    the oracle's run on the pre-summed gradients (the accumulate step changes the input of
    the path and nothing else)."""
    from paper_2504_05638_amd.bucket import TagcBucket
    print("\n[case] error feedback end to end", flush=True)
    b = G.config1(seed=2, n=(1 << 19) + 100, n_ranks=3)
    b.sizing_milli = 2000
    cfg = oracle_config(b, seed=4)
    segs = oracle_segments(b)
    tb = TagcBucket(b.segments, b.dtype, b.n_ranks, sizing_milli=b.sizing_milli, seed=4,
                    dense=True, error_feedback=True)
    g1 = [G.rank_gradient(b, r, "cpu") for r in range(b.n_ranks)]
    tb.run([g.cuda() for g in g1])              # step 1 leaves a residual in every accumulator
    torch.cuda.synchronize()
    acc = [O.error_feedback_step(G.to_numpy_raw(g), np.zeros(b.n_elems, np.float32), cfg, segs)[1]
           for g in g1]
    b2 = G.config1(seed=9, n=(1 << 19) + 100, n_ranks=3)
    g2 = [G.rank_gradient(b2, r, "cpu") for r in range(b.n_ranks)]
    summed = [(g.numpy() + a).astype(np.float32) for g, a in zip(g2, acc)]
    ores = O.run_bucket(summed, cfg, segs)
    tb.run([g.cuda() for g in g2])
    torch.cuda.synchronize()
    compare_all(b, ores, tb)
