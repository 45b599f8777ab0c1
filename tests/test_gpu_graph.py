"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no
synchronisation in any per-call entry point), so a caller may capture a bucket's whole call
sequence in a HIP graph.  Replays -- with fresh gradients copied into the captured input
buffers, eager work and synchronisations in between -- must give what the oracle gives for
those gradients, every time."""
import numpy as np
import pytest
import torch

from synth import gradients as G
from oracle import tagc_oracle as O
from tests.helpers import oracle_config, oracle_segments, compare_all

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [G.F32, G.BF16])
def test_bucket_call_sequence_replayed_from_a_graph(dtype):
    from paper_2504_05638_amd.bucket import TagcBucket
    print("\n[case] graph replay dtype=%d" % dtype, flush=True)
    b = G.small_mixed_bucket(seed=6, dtype=dtype, n_ranks=3, sizing_milli=1500)
    big = G.config1(seed=2, n=(1 << 19) + 333, n_ranks=3)
    for bucket in (b, big) if dtype == G.F32 else (b,):
        tb = TagcBucket(bucket.segments, bucket.dtype, bucket.n_ranks,
                        sizing_milli=bucket.sizing_milli, seed=7, part_unknowns=256,
                        part_cells=768, dense=True)
        inputs = [torch.zeros(bucket.n_elems, dtype=bucket.torch_dtype, device="cuda")
                  for _ in range(bucket.n_ranks)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            tb.run(inputs)                      # warm-up outside the capture (one-time set-up)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            tb.run(inputs)
        ocfg = oracle_config(bucket, seed=7, P=256, T=768)
        for rep, scale in enumerate([1.0, 30.0, 1.0, 1e-2]):
            bb = G.Bucket(bucket.name, bucket.dtype, bucket.n_ranks, bucket.segments,
                          bucket.n_elems, bucket.sizing_milli, bucket.sigma, bucket.kind,
                          bucket.seed + 13 * rep, bucket.bucket_id)
            grads = [(G.rank_gradient(bb, r, "cpu").float() * scale).to(bucket.torch_dtype)
                     for r in range(bucket.n_ranks)]
            for dst, g in zip(inputs, grads):
                dst.copy_(g.cuda())             # eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ores = O.run_bucket([G.to_numpy_raw(g) for g in grads], ocfg,
                                oracle_segments(bucket))
            compare_all(bucket, ores, tb)
        tb.close()
