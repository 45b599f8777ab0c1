"""Pins for the hash family and the sketch layout.

The numpy hash below is a third, independent implementation (neither the C
oracle nor the HIP code); the known-answer file freezes the vectors."""
import os

import numpy as np
import pytest

from oracle import tagc_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hash_kat.txt")
M32 = np.uint64(0xFFFFFFFF)


def np_mix32(x):
    x = np.asarray(x, np.uint64) & M32
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x6A09E667)) & M32
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0xBB67AE85)) & M32
    x ^= x >> np.uint64(16)
    return x


def np_seed_word(seed, j):
    lo = np.uint64(seed & 0xFFFFFFFF)
    hi = np.uint64(seed >> 32)
    inner = np_mix32((hi + np.uint64(0x9E3779B9) * np.uint64(j + 1)) & M32)
    return np_mix32(lo ^ inner)


def np_hash(i, seed, j, m_sub, salt=0):
    h = np_mix32(np.asarray(i, np.uint64) ^ np_seed_word(seed, j + 3 * salt))
    slot = (h * np.uint64(m_sub)) >> np.uint64(32)
    sign = np.where(h & np.uint64(1), -1, 1)
    return slot.astype(np.int64), sign.astype(np.int64)


def _kat():
    rows = []
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#"):
                continue
            rows.append(tuple(int(x) for x in line.split()))
    return rows


def test_known_answers_three_way():
    rows = _kat()
    assert len(rows) > 900
    assert any(r[4] for r in rows)          # salted vectors too
    for seed, i, j, ms, salt, slot, sign in rows:
        assert O.hash_slot(i, seed, j, ms, salt) == (slot, sign)
        s2, g2 = np_hash(i, seed, j, ms, salt)
        assert (int(s2), int(g2)) == (slot, sign)
        assert 0 <= slot < ms


def test_mix32_is_a_bijection_on_a_sample_and_avalanches():
    L = O.lib()
    xs = np.arange(1 << 16, dtype=np.uint64)
    hs = np_mix32(xs)
    assert len(set(hs.tolist())) == len(xs)
    assert all(int(L.tagco_mix32(int(x))) == int(h)
               for x, h in zip(xs[:500], hs[:500]))
    # flipping one input bit flips about half the output bits
    base = np_mix32(xs)
    for b in (0, 7, 16, 31):
        flipped = np_mix32(xs ^ np.uint64(1 << b))
        diff = base ^ flipped
        bits = np.unpackbits(diff.astype(np.uint32).view(np.uint8)).mean() * 32
        assert 14.0 < bits < 18.0


@pytest.mark.parametrize("m_sub", [97, 8192])
def test_uniform_slots_and_balanced_signs(m_sub):
    n = 200 * m_sub
    i = np.arange(n, dtype=np.uint64) * np.uint64(3) + np.uint64(12345)
    for j in range(3):
        slot, sign = np_hash(i, 42, j, m_sub)
        counts = np.bincount(slot, minlength=m_sub)
        chi2 = ((counts - 200.0) ** 2 / 200.0).sum()
        # chi-square with m_sub-1 dof: mean m_sub, sd sqrt(2 m_sub)
        assert abs(chi2 - m_sub) < 6 * np.sqrt(2 * m_sub)
        assert abs(sign.mean()) < 6 / np.sqrt(n)


def test_hash_functions_are_pairwise_independent_enough():
    m_sub = 64
    i = np.arange(400_000, dtype=np.uint64)
    s0, g0 = np_hash(i, 7, 0, m_sub)
    s1, g1 = np_hash(i, 7, 1, m_sub)
    s2, _ = np_hash(i, 7, 2, m_sub)
    for a, b in ((s0, s1), (s0, s2), (s1, s2)):
        joint = np.bincount(a * m_sub + b, minlength=m_sub * m_sub)
        e = len(i) / (m_sub * m_sub)
        chi2 = ((joint - e) ** 2 / e).sum()
        dof = m_sub * m_sub - 1
        assert abs(chi2 - dof) < 6 * np.sqrt(2 * dof)
    assert abs((g0 * g1).mean()) < 6 / np.sqrt(len(i))
    # sign of hash j is not determined by its slot
    assert abs((g0 * np.where(s0 & 1, 1, -1)).mean()) < 6 / np.sqrt(len(i))


# ------------------------------------------------------------------ layout


@pytest.mark.parametrize("mode,milli", [(O.SIZE_LOAD_FACTOR, 1500),
                                        (O.SIZE_LOAD_FACTOR, 3000),
                                        (O.SIZE_LOAD_FACTOR, 1100),
                                        (O.SIZE_FIXED_RATIO, 2000),
                                        (O.SIZE_FIXED_RATIO, 10_000)])
def test_layout_invariants(mode, milli):
    rng = np.random.default_rng(1)
    for P_cap, T_cap in ((16384, 24576), (256, 768), (1000, 999)):
        for U in [0, 1, 2, 255, 256, 257, 5000, 16384, 16385, 10 ** 6,
                  int(rng.integers(1, 10 ** 8))]:
            n_real = max(U, 1) * 7
            cfg = O.Config(sizing=mode, sizing_milli=milli,
                           part_unknowns=P_cap, part_cells=T_cap)
            A, ms, m = O.layout(U, cfg, n_real)
            if U == 0:
                assert (A, ms, m) == (0, 0, 0)
                continue
            assert m == 3 * A * ms and ms >= 1 and A >= 1
            assert 3 * ms <= T_cap // 3 * 3          # a partition fits its tile
            ps = O.lib().tagco_part_start
            for rng_a in ((range(A),) if A < 2000 else
                          (range(1000), range(A - 1000, A))):
                sizes = [ps(a + 1, U, A) - ps(a, U, A) for a in rng_a]
                assert max(sizes) <= P_cap            # and its unknown budget
                assert min(sizes) >= U // A
            assert ps(0, U, A) == 0 and ps(A, U, A) == U
            if mode == O.SIZE_LOAD_FACTOR:
                assert m * 1000 >= milli * U          # at least lf x U cells
                assert m <= milli * U / 1000 + 3 * A + 3
            else:
                assert m <= max(3 * A, -(-n_real * 1000 // milli))


def test_bounds_are_the_ranked_set_bits():
    rng = np.random.default_rng(2)
    n_c = 32 * 500
    bits = rng.random(n_c) < 0.07
    bitmap = np.packbits(bits, bitorder="little").view(np.uint32)
    pos = np.flatnonzero(bits)
    U = len(pos)
    for A in (1, 2, 7, 50, U, U + 5):
        bnd = O.bounds(bitmap, n_c, U, A)
        for a in range(A):
            st = (a * U) // A
            assert bnd[a] == (pos[st] if st < U else n_c)
        assert bnd[A] == n_c
        assert np.all(np.diff(bnd.astype(np.int64)) >= 0)


def test_paper_table1_compression_levels_give_the_fixed_ratio_size():
    # n/c cells for c-x compression (Figure 1 caption, Table 1)
    n = 3 * 24576 * 10
    for ratio_milli, c in ((2000, 2), (4000, 4), (10_000, 10)):
        cfg = O.Config(sizing=O.SIZE_FIXED_RATIO, sizing_milli=ratio_milli)
        A, ms, m = O.layout(n // 50, cfg, n)
        assert m <= n // c and m >= n // c - 3 * A
