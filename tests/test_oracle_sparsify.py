"""Pins for the oracle's sparsifier and Index (section 3.2 threshold rule,
Algorithm 1 sparsify/create_index): brute force, library top-k, invariants."""
import numpy as np
import pytest
import torch

from oracle import tagc_oracle as O
from oracle import definition as D


def _bf16_bits(x_f32):
    t = torch.from_numpy(np.asarray(x_f32, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def _brute_select(values, k):
    """Pure-Python restatement: stable sort of positions by |v| descending."""
    order = sorted(range(len(values)), key=lambda p: (-abs(float(values[p])), p))
    return sorted(p for p in order[:k] if float(values[p]) != 0.0)


def _run_one(values_raw, dtype, k_ppm, offset=0, c_off=0):
    n = len(values_raw) - offset
    seg = [O.Segment(offset, n, k_ppm)]
    st = O.sparsify(values_raw, O.Config(dtype=dtype), seg)
    return st


VECTORS = {
    "gauss": lambda rng, n: rng.standard_normal(n).astype(np.float32),
    "all_equal": lambda rng, n: np.full(n, 0.5, np.float32),
    "two_valued": lambda rng, n: rng.choice([-1.0, 2.0], n).astype(np.float32),
    "many_zero": lambda rng, n: (rng.standard_normal(n)
                                 * (rng.random(n) < 0.01)).astype(np.float32),
    "signed_zero": lambda rng, n: np.where(rng.random(n) < 0.5, -0.0, 0.0
                                           ).astype(np.float32),
    "ties_int": lambda rng, n: rng.integers(-3, 4, n).astype(np.float32),
}


@pytest.mark.parametrize("name", sorted(VECTORS))
@pytest.mark.parametrize("n,ppm", [(1, 1_000_000), (33, 100_000), (1000, 10_000),
                                   (4096, 12_500), (4095, 200_000), (777, 0)])
@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_matches_brute_force(name, n, ppm, dtype):
    rng = np.random.default_rng(hash((name, n, ppm)) % 2 ** 32)
    v = VECTORS[name](rng, n)
    raw = v if dtype == O.F32 else _bf16_bits(v)
    vw = D.widen(raw, dtype)
    k = (n * ppm) // 1_000_000
    assert O.keep_count(n, ppm) == k
    st = _run_one(raw, dtype, ppm)
    want = _brute_select(vw, k)
    assert st.idx.tolist() == want
    assert st.val.tolist() == [float(vw[p]) for p in want]
    # Index: exactly the selected bits
    bits = np.unpackbits(st.bitmap.view(np.uint8), bitorder="little")
    assert np.flatnonzero(bits).tolist() == want
    # exact count unless there are fewer non-zeros than k (section 3.2:
    # at least theta% become zero)
    assert st.cnt == min(k, int(np.count_nonzero(vw)))
    assert n - st.cnt >= n - k


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_kept_dominate_dropped_and_agree_with_library_topk(dtype):
    rng = np.random.default_rng(5)
    n, ppm = 200_000, 10_000
    v = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    raw = v if dtype == O.F32 else _bf16_bits(v)
    vw = D.widen(raw, dtype)
    st = _run_one(raw, dtype, ppm)
    k = (n * ppm) // 1_000_000
    assert st.cnt == k
    mag = np.abs(vw)
    kept = np.zeros(n, bool)
    kept[st.idx] = True
    assert mag[kept].min() >= mag[~kept].max()
    # a library top-k agrees as a set on everything strictly above the
    # threshold magnitude; at the threshold only the lowest positions are kept
    thr = mag[kept].min()
    lib_top = torch.topk(torch.from_numpy(mag), k).indices.numpy()
    strictly = set(np.flatnonzero(mag > thr).tolist())
    assert strictly <= set(lib_top.tolist())
    assert strictly <= set(st.idx.tolist())
    ties = np.flatnonzero(mag == thr)
    need = k - len(strictly)
    assert sorted(set(st.idx.tolist()) - strictly) == ties[:need].tolist()
    # numpy's partition gives the same threshold value
    assert np.partition(mag, n - k)[n - k] == thr


def test_offsets_c_offsets_and_skipped_segments():
    rng = np.random.default_rng(11)
    segs = [O.Segment(3, 100, 100_000), O.Segment(103, 50, 500_000, flags=0),
            O.Segment(160, 70, 100_000), O.Segment(230, 5, 100_000)]
    g = rng.standard_normal(240).astype(np.float32)
    offs, n_c = O.c_offsets(segs)
    assert offs == [0, None, 128, 224] and n_c == 256
    st = O.sparsify(g, O.Config(), segs)
    want = []
    for s, co in zip(segs, offs):
        if co is None:
            continue
        sel = _brute_select(g[s.offset:s.offset + s.length],
                            (s.length * s.keep_ppm) // 10 ** 6)
        want += [co + p for p in sel]
    assert st.idx.tolist() == want
    assert st.seg_cnt == [10, 0, 7, 0]
    # definition module agrees (independent selection routine)
    i1, v1 = D.sparse_sum([g], O.F32, segs)
    assert i1.tolist() == want
    assert np.array_equal(v1.astype(np.float32), st.val)


def test_nonfinite_is_an_error():
    g = np.ones(64, np.float32)
    g[5] = np.inf
    with pytest.raises(ValueError):
        O.sparsify(g, O.Config(), [O.Segment(0, 64, 500_000)])
    g[5] = np.nan
    with pytest.raises(ValueError):
        O.sparsify(g, O.Config(), [O.Segment(0, 64, 500_000)])


def test_index_or_is_union():
    rng = np.random.default_rng(3)
    maps = [rng.integers(0, 2 ** 32, 100, dtype=np.uint32) for _ in range(5)]
    out, U = O.index_or(maps)
    want = maps[0].copy()
    for m in maps[1:]:
        want |= m
    assert np.array_equal(out, want)
    assert U == int(np.unpackbits(want.view(np.uint8)).sum())
