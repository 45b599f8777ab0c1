"""tagc_compress_static: tagc_compress on the library's own device array instead of a
caller's workspace, for callers that cannot allocate.  Its outputs must equal those of
tagc_compress bit for bit (pairs, counts, Index), on two calls in a row, the second with a
smaller input, and the rest of the path must run on from them unchanged (float32 sums
within the 1e-5 tolerance: their order of adds is free in both entry points)."""
import numpy as np
import pytest
import torch

from synth import gradients as G

pytestmark = pytest.mark.gpu


def _run(tb, grads, static):
    """The whole path; PHASE_INDEX and PHASE_SKETCH through either entry point."""
    from paper_2504_05638_amd import binding as B
    s = int(torch.cuda.current_stream().cuda_stream)
    n = len(grads)
    for r in range(n):
        if static:
            rk = B.tagc_rank_buffers.from_buffer_copy(tb.rk[r])
            rk.workspace = None   # ignored by the static variant
            B.tagc_compress_static(tb.plan, B.TAGC_PHASE_INDEX, grads[r].data_ptr(), rk,
                                   tb.shared, s)
        else:
            tb.compress_index(r, grads[r])
    tb.aggregate_index(n)
    for r in range(n):
        if static:
            rk = B.tagc_rank_buffers.from_buffer_copy(tb.rk[r])
            rk.workspace = None
            B.tagc_compress_static(tb.plan, B.TAGC_PHASE_SKETCH, None, rk, tb.shared, s)
        else:
            tb.compress_sketch(r)
    tb.aggregate_sketch(n)
    tb.decompress()
    torch.cuda.synchronize()


def _snapshot(tb, n):
    out = {"hdr": tb.header(), "st": tb.status(), "sh_bitmap": tb.shared_bitmap(),
           "out": tb.outputs()}
    for r in range(n):
        out[r] = (tb.rank_counts(r), tb.rank_pairs(r), tb.rank_bitmap(r), tb.rank_sketch(r))
    return out


def test_static_workspace_variant_equals_tagc_compress():
    from paper_2504_05638_amd import binding as B
    from paper_2504_05638_amd.bucket import TagcBucket
    big = G.config1(seed=5, n=(1 << 20) + 4321, n_ranks=3)           # fp32, one long segment
    small = G.small_mixed_bucket(seed=3, dtype=G.BF16, n_ranks=3, sizing_milli=1500)
    for case, b in enumerate((big, small)):                           # the second is smaller
        print("\n[case] static workspace: bucket %s (%d elements)" % (b.name, b.n_elems),
              flush=True)
        grads = [G.rank_gradient(b, r, "cuda") for r in range(b.n_ranks)]
        kw = dict(sizing_milli=b.sizing_milli, seed=9, part_unknowns=512, part_cells=1536)
        ref = TagcBucket(b.segments, b.dtype, b.n_ranks, **kw)
        got = TagcBucket(b.segments, b.dtype, b.n_ranks, **kw)
        assert got.sizes.rank_workspace_bytes <= B.TAGC_STATIC_WORKSPACE_BYTES
        for rep in range(2):    # the second repetition starts from the pre-thresholds of the first
            _run(ref, grads, static=False)
            want = _snapshot(ref, b.n_ranks)
            _run(got, grads, static=True)
            have = _snapshot(got, b.n_ranks)
            assert have["hdr"] == want["hdr"] and have["st"] == want["st"]
            assert want["st"]["flags"] == 0
            assert np.array_equal(have["sh_bitmap"], want["sh_bitmap"])
            for r in range(b.n_ranks):
                (c0, (i0, v0), m0, s0), (c1, (i1, v1), m1, s1) = want[r], have[r]
                assert c0 == c1 and c0["total"] > 0
                assert np.array_equal(i0, i1)
                assert np.array_equal(v0.view(np.uint32), v1.view(np.uint32))
                assert np.array_equal(m0, m1)
                # a sketch cell is a float32 sum whose order of adds is free (LDS atomics):
                # two runs of the same entry point differ in the same way
                scale = float(np.abs(v0).max())
                assert np.all(np.abs(s0.astype(np.float64) - s1) <= 1e-5 * scale)
            assert np.array_equal(have["out"][0], want["out"][0])
            scale = float(np.abs(want["out"][1]).max())
            assert np.all(np.abs(want["out"][1].astype(np.float64) - have["out"][1])
                          <= 1e-5 * scale)
        ref.close()
        got.close()


def test_static_workspace_variant_rejects_what_does_not_fit():
    from paper_2504_05638_amd import binding as B
    b = G.config5()[0]     # 202 M entries: the candidate slots alone exceed the array
    cfg = B.tagc_config(dtype=b.dtype, n_ranks=1, n_hash=3, sizing=B.TAGC_SIZE_LOAD_FACTOR,
                        sizing_milli=1500)
    plan = B.tagc_plan(cfg, [tuple(s[:4]) for s in b.segments])
    assert B.tagc_plan_sizes(plan).rank_workspace_bytes > B.TAGC_STATIC_WORKSPACE_BYTES
    g = torch.zeros(64, dtype=torch.bfloat16, device="cuda")   # never read: rejected first
    with pytest.raises(B.TagcError) as e:
        B.tagc_compress_static(plan, B.TAGC_PHASE_INDEX, g.data_ptr(), B.tagc_rank_buffers(),
                               B.tagc_shared_buffers(),
                               int(torch.cuda.current_stream().cuda_stream))
    assert e.value.code == -2   # TAGC_ESIZE
    B.tagc_plan_destroy(plan)
