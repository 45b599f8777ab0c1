"""Host-side checks of libtagc that need no GPU: the library loads, exports every
symbol include/tagc.h declares, and its plan arithmetic agrees with the oracle's
and with the numbers the paper prints."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import tagc_oracle as O
from paper_2504_05638_amd import binding as B
from synth import gradients as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    d = dict(dtype=B.TAGC_F32, n_ranks=4, n_hash=3, sizing=B.TAGC_SIZE_LOAD_FACTOR,
             sizing_milli=3000, index_mode=B.TAGC_INDEX_OR1, part_unknowns=0,
             part_cells=0, seed=0)
    d.update(kw)
    return B.tagc_config(**d)


def test_library_exports_every_declared_symbol():
    text = "".join(open(os.path.join(ROOT, "include", h)).read()
                   for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(tagc_[a-z_0-9]+)\s*\(", text))
    assert set(B.EXPORTS) == declared
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_plan_matches_oracle_bookkeeping():
    for b in [G.small_mixed_bucket(dtype=G.F32), G.small_mixed_bucket(dtype=G.BF16),
              G.config2()[3], G.config5()[0]]:
        plan = B.tagc_plan(_cfg(dtype=b.dtype, n_ranks=b.n_ranks,
                                sizing_milli=b.sizing_milli), b.segments)
        z = B.tagc_plan_sizes(plan)
        osegs = [O.Segment(s.offset, s.length, s.keep_ppm, s.flags) for s in b.segments]
        offs, n_c = O.c_offsets(osegs)
        assert z.n_c == n_c and z.bitmap_words == n_c // 32
        assert z.n_real == b.compressed_elems()
        K = sum(O.keep_count(s.length, s.keep_ppm) for s in osegs if s.flags & 1)
        assert z.pair_capacity == K
        assert z.union_capacity == min(z.n_real, b.n_ranks * K)
        assert z.grad_elems <= b.n_elems
        # capacities dominate every layout the oracle can produce
        ocfg = O.Config(sizing_milli=b.sizing_milli)
        for U in {0, 1, z.union_capacity // 3, z.union_capacity}:
            A, ms, m = O.layout(U, ocfg, z.n_real)
            assert A <= z.partition_capacity and m <= z.sketch_cells_capacity
        B.tagc_plan_destroy(plan)


def test_wire_accounting_reproduces_the_papers_numbers():
    n = 32 * 100_000
    seg = [(0, n, 12_500, 1)]
    z = B.tagc_plan_sizes(B.tagc_plan(_cfg(sizing=B.TAGC_SIZE_FIXED_RATIO,
                                           sizing_milli=10_000), seg))
    assert abs(z.wire_total_bits - 5.2) < 1e-9           # 2*1 + 32/10
    assert round(32.0 / z.wire_total_bits, 2) == 6.15      # section 3.1
    z = B.tagc_plan_sizes(B.tagc_plan(_cfg(sizing=B.TAGC_SIZE_FIXED_RATIO,
                                           sizing_milli=2000), seg))
    assert abs(z.wire_sketch_bits - 16.0) < 1e-9           # Figure 1 caption
    assert abs(z.wire_total_bits - O.wire_bits_per_param(1, 2)) < 1e-9


def test_four_bit_index_sizes_and_wire_volume():
    """The 4-bit Index is four times the 1-bit one, on the wire and in the rank's buffer
    (section 2.2); the merged Index stays 1 bit per parameter."""
    seg = [(0, 1_024_000, 12_500, 1)]
    z1 = B.tagc_plan_sizes(B.tagc_plan(_cfg(sizing=B.TAGC_SIZE_FIXED_RATIO, sizing_milli=10_000),
                                       seg))
    z4 = B.tagc_plan_sizes(B.tagc_plan(_cfg(sizing=B.TAGC_SIZE_FIXED_RATIO, sizing_milli=10_000,
                                            index_mode=B.TAGC_INDEX_ADD4), seg))
    za = B.tagc_plan_sizes(B.tagc_plan(_cfg(sizing=B.TAGC_SIZE_FIXED_RATIO, sizing_milli=10_000,
                                            index_mode=B.TAGC_INDEX_ADD1), seg))
    assert z4.rank_bitmap_bytes == 4 * z1.rank_bitmap_bytes == 4 * za.rank_bitmap_bytes
    assert z4.shared_bitmap_bytes == z1.shared_bitmap_bytes
    assert abs(z4.wire_index_bits - 4 * z1.wire_index_bits) < 1e-12
    assert abs(z1.wire_total_bits - O.wire_bits_per_param(1, 10)) < 1e-9   # 5.2 bit
    assert abs(z4.wire_total_bits - O.wire_bits_per_param(4, 10)) < 1e-9   # 11.2 bit
    assert z4.rank_workspace_bytes >= z1.rank_workspace_bytes + 1_024_000 // 8


def test_argument_errors():
    seg = [(0, 1000, 10_000, 1)]
    for bad in (dict(dtype=7), dict(n_hash=2), dict(n_ranks=0), dict(sizing=9),
                dict(sizing_milli=0), dict(part_cells=100), dict(part_cells=3 * 6000),
                dict(part_unknowns=1 << 20), dict(reserved=1)):
        with pytest.raises(B.TagcError) as e:
            B.tagc_plan(_cfg(**bad), seg)
        assert e.value.code == -1
    with pytest.raises(B.TagcError) as e:
        B.tagc_plan(_cfg(index_mode=3), seg)
    assert e.value.code == -3
    with pytest.raises(B.TagcError):
        B.tagc_plan(_cfg(decode_mode=3), seg)
    with pytest.raises(B.TagcError) as e:
        B.tagc_plan(_cfg(), [(0, 1 << 31, 10_000, 1)])
    assert e.value.code == -2
    with pytest.raises(B.TagcError):
        B.tagc_plan(_cfg(), [(0, 1000, 2_000_000, 1)])
    assert B.strerror(-2).startswith("size")
    # any limit on the peeling grid is a valid plan, with the same sizes
    z0 = B.tagc_plan_sizes(B.tagc_plan(_cfg(), seg))
    z1 = B.tagc_plan_sizes(B.tagc_plan(_cfg(decode_workgroups=1 << 30), seg))
    assert bytes(z0) == bytes(z1)
    # null / misaligned device pointers are rejected before anything is launched
    plan = B.tagc_plan(_cfg(), seg)
    rk, sh = B.tagc_rank_buffers(), B.tagc_shared_buffers()
    with pytest.raises(B.TagcError):
        B.tagc_compress(plan, B.TAGC_PHASE_INDEX, 256, rk, sh)
    with pytest.raises(B.TagcError):
        B.tagc_decompress(plan, sh, 256, 256)


def test_static_workspace_variant_rejects_a_plan_that_does_not_fit_before_touching_anything():
    """tagc_compress_static checks the plan's workspace size first: no device is needed to
    be told that a 7B-shaped bucket does not fit the library's own array."""
    b = G.config5()[0]
    plan = B.tagc_plan(_cfg(dtype=b.dtype, n_ranks=1, sizing_milli=1500), b.segments)
    assert B.tagc_plan_sizes(plan).rank_workspace_bytes > B.TAGC_STATIC_WORKSPACE_BYTES
    rk, sh = B.tagc_rank_buffers(), B.tagc_shared_buffers()
    with pytest.raises(B.TagcError) as e:
        B.tagc_compress_static(plan, B.TAGC_PHASE_INDEX, 4096, rk, sh, 0)
    assert e.value.code == -2
    with pytest.raises(B.TagcError) as e:
        B.tagc_compress_static(None, B.TAGC_PHASE_INDEX, 4096, rk, sh, 0)
    assert e.value.code == -1
    B.tagc_plan_destroy(plan)


def test_fused_decode_refuses_what_its_kernel_cannot_hold_before_touching_anything():
    """tagc_reduce_decompress takes float32 cells, partitions of the default size at most and
    up to 32 ranks; anything else is TAGC_EUNSUPPORTED before a pointer is looked at."""
    seg = [(0, 1 << 20, 10_000, B.TAGC_SEG_COMPRESS)]
    rk, sh = B.tagc_rank_buffers(), B.tagc_shared_buffers()
    for kw in (dict(cell_type=B.TAGC_CELL_BF16), dict(part_unknowns=8192, part_cells=12291),
               dict(n_ranks=40)):
        cfg = dict(n_ranks=2)
        cfg.update(kw)
        plan = B.tagc_plan(_cfg(**cfg), seg)
        with pytest.raises(B.TagcError) as e:
            B.tagc_reduce_decompress(plan, [rk] * cfg["n_ranks"], sh, 256, 256)
        assert e.value.code == -3, kw
        B.tagc_plan_destroy(plan)
    plan = B.tagc_plan(_cfg(n_ranks=2), seg)
    with pytest.raises(B.TagcError) as e:   # supported, but null buffers
        B.tagc_reduce_decompress(plan, [rk, rk], sh, 256, 256)
    assert e.value.code == -1
    B.tagc_plan_destroy(plan)


def test_bench_refuses_more_than_one_gpu_and_fails_loudly_without_one():
    """bench.py measures one GPU: asked for more it says so and exits; without a GPU it
    must not fall back to anything (there is no CPU path)."""
    import subprocess
    import sys
    bench = os.path.join(ROOT, "bench.py")
    r = subprocess.run([sys.executable, bench, "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, bench, "--steps", "1", "--warmup", "0",
                            "--workload", "config1", "--no-cpu-baseline"],
                           capture_output=True, text=True, timeout=300)
        assert r.returncode != 0 and not r.stdout.strip().startswith("{")


def test_host_hash_helper_agrees_with_known_answers():
    path = os.path.join(ROOT, "tests", "golden", "hash_kat.txt")
    for line in open(path):
        if line.startswith("#"):
            continue
        seed, i, j, ms, salt, slot, sign = (int(x) for x in line.split())
        assert B.tagc_hash_host(i, seed, j, ms, salt) == (slot, sign)


def test_product_package_does_not_reach_into_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_05638_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, os.path.join(dirpath, f)
