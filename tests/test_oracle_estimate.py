"""CPU pins for the oracle's estimation decode (section 2.2: the second decompression
algorithm, usable at any density but noisy).  The oracle's function is a Count Sketch
point query, so it is pinned by what such a query must satisfy whatever the code looks
like: exactness whenever two of an unknown's three cells are private, the deterministic
error bound by the middle of the three cells' foreign mass, the closed form for two
unknowns that share all their cells, and -- for the residue of a stalled peeling -- that
only unresolved neighbours may show up in the error."""
import itertools

import numpy as np
import pytest

from oracle import tagc_oracle as O


def _setup(rng, n, U, lf_milli, seed, P=256, T=768, lo=-1000, hi=1001):
    """One rank, U integer-valued non-zeros at random positions of [0, n)."""
    pos = np.sort(rng.choice(n, U, replace=False)).astype(np.uint32)
    val = rng.integers(lo, hi, U).astype(np.float32)
    val[val == 0] = 7
    n_c = (n + 31) // 32 * 32
    bm = np.zeros(n_c // 32, np.uint32)
    np.bitwise_or.at(bm, pos >> 5, np.uint32(1) << (pos & 31))
    cfg = O.Config(dtype=O.F32, sizing=O.SIZE_LOAD_FACTOR, sizing_milli=lf_milli, seed=seed,
                   part_unknowns=P, part_cells=T)
    A, m_sub, m = O.layout(U, cfg, n)
    bnd = O.bounds(bm, n_c, U, A)
    sk = O.encode(pos, val, bnd, A, m_sub, seed)
    return pos, val, bm, n_c, A, m_sub, sk


def _cells(pos, A, m_sub, seed):
    """(global cell, sign) of every unknown, from the partition rule and the hash
    (both pinned on their own elsewhere)."""
    U = pos.size
    cell = np.zeros((U, 3), np.int64)
    sign = np.zeros((U, 3), np.int64)
    for t, i in enumerate(pos):
        a = max(a for a in range(A) if a * U // A <= t)
        for j in range(3):
            s, sg = O.hash_slot(int(i), seed, j, m_sub)
            cell[t, j] = (a * 3 + j) * m_sub + s
            sign[t, j] = sg
    return cell, sign


def _foreign_mass(cell, val, members):
    """For each unknown and each of its cells: sum of |value| of the *other* members."""
    mass = {}
    for t in members:
        for j in range(3):
            mass[cell[t, j]] = mass.get(cell[t, j], 0.0) + abs(float(val[t]))
    out = np.zeros(cell.shape)
    for t in range(cell.shape[0]):
        for j in range(3):
            own = abs(float(val[t])) if t in members else 0.0
            out[t, j] = mass.get(cell[t, j], 0.0) - own
    return out


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_estimate_only_is_exact_with_two_private_cells_and_bounded_otherwise(seed):
    rng = np.random.default_rng(seed)
    # two cells per unknown: 1.5 unknowns per cell and hash function on average
    pos, val, bm, n_c, A, m_sub, sk = _setup(rng, 60_000, 1500, 2000, seed)
    dec = O.decompress(bm, n_c, pos.size, A, m_sub, seed, sk, O.DECODE_ESTIMATE)
    assert np.array_equal(dec.idx, pos) and dec.n_unresolved == pos.size
    cell, _ = _cells(pos, A, m_sub, seed)
    noise = _foreign_mass(cell, val, set(range(pos.size)))
    private = (noise == 0).sum(axis=1)
    two = private >= 2
    assert two.sum() > 20 and (~two).sum() > 200          # both kinds present
    assert np.array_equal(dec.val[two], val[two])           # the median is a clean reading
    # each reading is off by at most its cell's foreign mass, so the median of three is
    # off by at most the middle one of the three masses
    bound = np.sort(noise, axis=1)[:, 1]
    assert np.all(np.abs(dec.val.astype(np.float64) - val) <= bound)
    # and it is really a median: min or max of the readings would break the bound
    # somewhere (one polluted cell next to two private ones)
    one_bad = two & (private == 2)
    assert one_bad.sum() > 10
    assert np.count_nonzero(dec.val != val) > 100


def test_two_unknowns_sharing_all_cells_closed_form():
    """x and y alone in the same three cells: the readings of x are x + s_j(x) s_j(y) y,
    so the estimate is x + y or x - y by the majority of the sign products."""
    seed, m_sub = 5, 2
    # brute force over small indices: a pair with identical slots under all three hashes
    found = None
    for i, k in itertools.combinations(range(200), 2):
        if all(O.hash_slot(i, seed, j, m_sub)[0] == O.hash_slot(k, seed, j, m_sub)[0]
               for j in range(3)):
            prods = [O.hash_slot(i, seed, j, m_sub)[1] * O.hash_slot(k, seed, j, m_sub)[1]
                     for j in range(3)]
            if found is None or (sum(prods) < 0) != (sum(found[2]) < 0):
                if found is None:
                    found = (i, k, prods)
                else:
                    other = (i, k, prods)
                    break
    for i, k, prods in (found, other):      # one pair with majority +, one with majority -
        n_c = 224
        bm = np.zeros(n_c // 32, np.uint32)
        for q in (i, k):
            bm[q >> 5] |= np.uint32(1 << (q & 31))
        x, y = 40.0, 3.0
        bnd = O.bounds(bm, n_c, 2, 1)
        sk = O.encode(np.array([i, k], np.uint32), np.array([x, y], np.float32), bnd, 1,
                      m_sub, seed)
        dec = O.decompress(bm, n_c, 2, 1, m_sub, seed, sk, O.DECODE_PEEL_ESTIMATE)
        assert dec.n_unresolved == 2 and dec.rounds == 0   # a 2-core: nothing to peel
        maj = 1.0 if sum(prods) > 0 else -1.0
        assert dec.val[0] == x + maj * y
        assert dec.val[1] == y + maj * x
    assert (sum(found[2]) > 0) != (sum(other[2]) > 0)


@pytest.mark.parametrize("seed", [11, 12])
def test_residue_is_estimated_from_what_peeling_left(seed):
    """Below the peeling threshold (load factor 1.15 < 1.22) peeling stalls on a core.
    What it resolved stays exact and untouched; an unknown of the core is estimated from
    cells that now hold core members only, so its error is bounded by the foreign mass of
    the *unresolved* neighbours -- a bound the raw sketch would violate."""
    rng = np.random.default_rng(seed)
    pos, val, bm, n_c, A, m_sub, sk = _setup(rng, 200_000, 4000, 1150, seed, P=4096,
                                             T=3 * 4800)
    plain = O.decompress(bm, n_c, pos.size, A, m_sub, seed, sk, O.DECODE_PEEL)
    dec = O.decompress(bm, n_c, pos.size, A, m_sub, seed, sk, O.DECODE_PEEL_ESTIMATE)
    core = plain.round == 0
    assert plain.n_unresolved == core.sum() and 100 < core.sum() < pos.size
    assert np.array_equal(dec.round, plain.round) and dec.n_unresolved == plain.n_unresolved
    assert np.array_equal(dec.val[~core], val[~core])      # integers: peeled values exact
    assert np.all(plain.val[core] == 0)
    cell, _ = _cells(pos, A, m_sub, seed)
    members = set(np.flatnonzero(core).tolist())
    noise_core = _foreign_mass(cell, val, members)
    bound = np.sort(noise_core, axis=1)[:, 1]
    err = np.abs(dec.val.astype(np.float64) - val)
    assert np.all(err[core] <= bound[core])
    # the same bound does not hold for estimates taken from the raw sketch
    raw = O.decompress(bm, n_c, pos.size, A, m_sub, seed, sk, O.DECODE_ESTIMATE)
    err_raw = np.abs(raw.val.astype(np.float64) - val)
    assert np.any(err_raw[core] > bound[core])
    # estimating the residue beats reporting zeros for it
    assert err[core].sum() < np.abs(val[core]).sum()


def test_estimation_changes_nothing_when_peeling_succeeds():
    rng = np.random.default_rng(4)
    pos, val, bm, n_c, A, m_sub, sk = _setup(rng, 50_000, 2000, 1500, 4)
    a = O.decompress(bm, n_c, pos.size, A, m_sub, 4, sk, O.DECODE_PEEL)
    b = O.decompress(bm, n_c, pos.size, A, m_sub, 4, sk, O.DECODE_PEEL_ESTIMATE)
    assert a.n_unresolved == 0
    assert np.array_equal(a.val, b.val) and np.array_equal(a.val, val)


def test_unbiased_over_seeds():
    """The sign hash makes a polluted reading err in either direction: over many hash
    seeds the mean error of a fixed unknown among positive values tends to 0, while
    without signs it would be the (positive) foreign mass."""
    rng = np.random.default_rng(0)
    errs = []
    for seed in range(200):
        pos, val, bm, n_c, A, m_sub, sk = _setup(rng, 4000, 300, 500, seed, lo=1, hi=50)
        dec = O.decompress(bm, n_c, pos.size, A, m_sub, seed, sk, O.DECODE_ESTIMATE)
        errs.append(float(np.mean(dec.val.astype(np.float64) - val)))
    errs = np.array(errs)
    # typical |error| per entry is tens; the mean over entries and seeds is near 0
    assert abs(errs.mean()) < 3.0 * errs.std() / np.sqrt(errs.size) + 0.5
