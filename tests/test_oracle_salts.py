"""Pins for the per-partition hash salts (oracle/tagc_oracle.c: tagco_salts).

The compression is called lossless (section 2.2, Table 1).  Two non-zeros of a sketch
partition that fall into the same three cells can never be peeled apart; the salts, a
function of the merged Index and the seed alone, rule that out.  Pinned here without
retyping the oracle's routine: a brute-force search over the third (numpy) implementation
of the hash; a planted pair that is lost without its partition's salt and recovered with
it; the expected number of salted partitions from the birthday bound (the closed form
13.5 U / (lf^3 P^2) of colliding pairs); and losslessness itself."""
import numpy as np
import pytest

from oracle import definition as D
from oracle import tagc_oracle as O
from tests.test_oracle_hash import np_hash


def _bits(pos, n_c):
    b = np.zeros(n_c, np.uint8)
    b[pos] = 1
    return np.packbits(b, bitorder="little").view(np.uint32)


def _triples(idx, seed, m_sub, salt):
    s = [np_hash(idx, seed, j, m_sub, salt)[0] for j in range(3)]
    return list(zip(s[0].tolist(), s[1].tolist(), s[2].tolist()))


@pytest.mark.parametrize("P,T,lf", [(64, 48, 1500), (40, 60, 1500), (100, 75, 1500)])
def test_salt_is_the_smallest_one_without_a_shared_triple(P, T, lf):
    rng = np.random.default_rng(P)
    n_c = 32 * 2000
    pos = np.sort(rng.choice(n_c, 6000, replace=False)).astype(np.uint32)
    bm = _bits(pos, n_c)
    cfg = O.Config(sizing_milli=lf, part_unknowns=P, part_cells=T, seed=21)
    A, m_sub, m = O.layout(pos.size, cfg, n_c)
    got = O.salts(bm, n_c, pos.size, A, m_sub, cfg.seed)
    assert got.shape == (A,)
    want = []
    for a in range(A):
        mine = pos[a * pos.size // A:(a + 1) * pos.size // A]
        s_a = O.SALT_LIMIT - 1
        for s in range(O.SALT_LIMIT):
            tr = _triples(mine, cfg.seed, m_sub, s)
            if len(set(tr)) == len(tr):
                s_a = s
                break
        want.append(s_a)
    assert got.tolist() == want
    assert 0 < np.count_nonzero(got) < A      # the case has both kinds of partition


def test_salts_of_nothing_and_of_a_partition_no_salt_can_help():
    assert O.salts(np.zeros(4, np.uint32), 128, 0, 0, 0, 3).size == 0
    # two non-zeros, one cell per hash function: every salt maps both to (0, 0, 0)
    bm = _bits([5, 77], 128)
    assert O.salts(bm, 128, 2, 1, 1, 3).tolist() == [O.SALT_LIMIT - 1]


def _colliding_pair(seed, m_sub, limit=200_000):
    """two c-indices below `limit` with the same three slots under salt 0"""
    i = np.arange(limit, dtype=np.uint64)
    key = sum(np_hash(i, seed, j, m_sub)[0] * (m_sub ** j) for j in range(3))
    order = np.argsort(key, kind="stable")
    same = np.flatnonzero(np.diff(key[order]) == 0)
    assert same.size, "no collision below the limit"
    return int(order[same[0]]), int(order[same[0] + 1])


def test_a_pair_sharing_all_three_cells_is_lost_without_the_salt_and_recovered_with_it():
    seed, n = 17, 200_000
    cfg = O.Config(sizing_milli=1500, seed=seed, part_unknowns=64, part_cells=96)
    # one partition of 64 non-zeros: m_sub = ceil(1.5 * 64 / 3) = 32
    i, k = _colliding_pair(seed, 32, n)
    rng = np.random.default_rng(0)
    others = rng.choice(np.setdiff1d(np.arange(n), [i, k]), 62, replace=False)
    g = np.zeros(n, np.float32)
    g[others] = rng.integers(1, 100, 62).astype(np.float32)
    g[i], g[k] = 1234.0, -77.0
    segs = [O.Segment(0, n, 1_000_000)]
    plain = O.run_bucket([g], cfg, segs, salted=False)
    assert (plain.A, plain.m_sub) == (1, 32)
    lost = plain.decoded.idx[plain.decoded.round == 0].tolist()
    assert i in lost and k in lost                      # peeling cannot separate them
    assert plain.decoded.val[plain.decoded.idx == i] == 0
    salted = O.run_bucket([g], cfg, segs)
    assert salted.salt.tolist() != [0]
    idx, val = D.sparse_sum([g], O.F32, segs)
    # (a 64-entry partition may still stall elsewhere; the planted pair must come out)
    ok = salted.decoded.round > 0
    assert ok[salted.decoded.idx == i] and ok[salted.decoded.idx == k]
    assert np.array_equal(salted.decoded.val[ok].astype(np.float64), val[ok])


def test_salted_partitions_follow_the_birthday_bound():
    """Expected pairs of a partition's n non-zeros sharing all three of m_sub^3 triples:
    n^2 / (2 m_sub^3); over a bucket, with m_sub = lf P / 3: 13.5 U / (lf^3 P^2).  The
    number of partitions that need a salt follows it (Poisson), and so does, without the
    salts, the number of entries lost."""
    rng = np.random.default_rng(5)
    U, n = 1_000_000, 12_000_000
    pos = np.sort(rng.choice(n, U, replace=False))
    g = np.zeros(n, np.float32)
    g[pos] = rng.integers(1, 1000, U).astype(np.float32)
    cfg = O.Config(sizing_milli=1500, seed=2, part_unknowns=512, part_cells=1536)
    segs = [O.Segment(0, n, 1_000_000)]
    r = O.run_bucket([g], cfg, segs)
    expect = 13.5 * U / (1.5 ** 3 * 512 ** 2)            # ~15.3 pairs
    salted = int(np.count_nonzero(r.salt))
    assert abs(salted - expect) < 5 * np.sqrt(expect)
    assert r.salt.max() <= 2
    plain = O.run_bucket([g], cfg, segs, salted=False)
    assert plain.decoded.n_unresolved >= 2 * salted       # two entries per pair at least
    assert plain.decoded.n_unresolved < 2 * salted + 40
    # what the salts leave: stopping sets of four and more non-zeros, 1.125 n^4 / m_sub^6
    # per partition to leading order (about 0.5 such sets in this bucket)
    assert r.decoded.n_unresolved <= 12


@pytest.mark.parametrize("lf", [1500, 3000])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_default_partitions_peel_completely_at_both_load_factors(lf, seed):
    """lf in {1.5, 3} at U >= 10^5: nothing is left, whatever the seed."""
    rng = np.random.default_rng(100 + seed)
    n = 1_500_000
    g = (rng.integers(1, 1000, n) * (rng.random(n) < 0.08)).astype(np.float32)
    r = O.run_bucket([g], O.Config(sizing_milli=lf, seed=seed), [O.Segment(0, n, 1_000_000)])
    assert r.U > 100_000 and r.A > 10
    assert r.decoded.n_unresolved == 0
    idx, val = D.sparse_sum([g], O.F32, [O.Segment(0, n, 1_000_000)])
    assert np.array_equal(r.decoded.val.astype(np.float64), val)
