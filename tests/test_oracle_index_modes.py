"""CPU pins for the oracle's addition-simulated Index All-Reduce (section 2.2: NCCL has no
bitwise OR, so the OR is simulated by addition on a 1-bit Index, which collides, or on a
4-bit one, which is stable and four times bigger) and for the masked encode that goes with
it.  Pinned by numpy's own OR where the modes must agree with it, by hand-worked carries,
by integer value preservation computed from per-position counts, and end to end by the
definition of what the decoder must then return."""
import numpy as np
import pytest

from oracle import tagc_oracle as O
from oracle import definition as D


def _maps(rng, n_ranks, words, density):
    bits = rng.random((n_ranks, words * 32)) < density
    return [np.packbits(b, bitorder="little").view(np.uint32).copy() for b in bits], bits


def _single(words, positions):
    m = np.zeros(words, np.uint32)
    for c in positions:
        m[c >> 5] |= np.uint32(1 << (c & 31))
    return m


def _set(m):
    return set(np.flatnonzero(np.unpackbits(m.view(np.uint8), bitorder="little")).tolist())


@pytest.mark.parametrize("n_ranks", [1, 2, 7, 15])
def test_four_bit_add_is_the_or_up_to_fifteen_ranks(n_ranks):
    rng = np.random.default_rng(n_ranks)
    maps, _ = _maps(rng, n_ranks, 300, 0.4)     # dense: most positions kept by several ranks
    want = np.bitwise_or.reduce(np.stack(maps), axis=0)
    got, U = O.index_add(maps, 4)
    assert np.array_equal(got, want) and U == len(_set(want))
    got_or, U_or = O.index_or(maps)
    assert np.array_equal(got_or, want) and U_or == U


def test_one_bit_add_is_the_or_on_disjoint_supports():
    rng = np.random.default_rng(0)
    owner = rng.integers(0, 5, 200 * 32)          # every position kept by at most one rank
    keep = rng.random(200 * 32) < 0.5
    maps = [np.packbits((owner == r) & keep, bitorder="little").view(np.uint32).copy()
            for r in range(4)]
    want = np.bitwise_or.reduce(np.stack(maps), axis=0)
    got, U = O.index_add(maps, 1)
    assert np.array_equal(got, want) and U == int(keep[owner < 4].sum())


def test_hand_worked_carries():
    W = 4
    # 1 bit: 1 + 1 = binary 10: the position vanishes, the next one appears
    assert _set(O.index_add([_single(W, [5]), _single(W, [5])], 1)[0]) == {6}
    # three ranks: binary 11
    assert _set(O.index_add([_single(W, [5])] * 3, 1)[0]) == {5, 6}
    # the carry out of a word's last bit is lost
    assert _set(O.index_add([_single(W, [31]), _single(W, [31])], 1)[0]) == set()
    # a carry runs on: {5,6} + {5} -> 5: 0 carry, 6: 1 + carry = 0 carry, 7: 1
    assert _set(O.index_add([_single(W, [5, 6]), _single(W, [5])], 1)[0]) == {7}
    # a carry lands on a position another rank really kept and erases it: {5}+{5}+{6}
    assert _set(O.index_add([_single(W, [5]), _single(W, [5]), _single(W, [6])], 1)[0]) == {7}
    # 4 bit: 15 ranks fill the counter, the 16th wraps it into the next parameter's field
    assert _set(O.index_add([_single(W, [9])] * 15, 4)[0]) == {9}
    assert _set(O.index_add([_single(W, [9])] * 16, 4)[0]) == {10}
    assert _set(O.index_add([_single(W, [9])] * 17, 4)[0]) == {9, 10}
    # parameter 15 is the last field of its wire word (8 parameters per word): carry lost
    assert _set(O.index_add([_single(W, [15])] * 16, 4)[0]) == set()
    # a carry into a full counter runs on: fields 8, 9, 10 = 15, 16, 15 -> 15, 0 carry,
    # 15 + 1 = 0 carry, field 11 = 1
    assert _set(O.index_add([_single(W, [8, 9, 10])] * 15 + [_single(W, [9])], 4)[0]) == {8, 11}
    # below 16 the neighbours of a full counter are untouched
    assert _set(O.index_add([_single(W, [8, 9, 10])] * 14 + [_single(W, [9])], 4)[0]) == {8, 9, 10}


@pytest.mark.parametrize("bits,n_ranks", [(1, 2), (1, 5), (1, 16), (4, 16), (4, 40)])
def test_sum_preserves_the_integer_value_of_every_wire_word(bits, n_ranks):
    """Per position, count how many ranks kept it; a wire word of the sum is
    sum_p count_p * (2^bits)^p modulo 2^32, computed here in Python integers."""
    rng = np.random.default_rng(bits * 100 + n_ranks)
    words = 64
    maps, b = _maps(rng, n_ranks, words, 0.6)
    count = b.sum(axis=0)
    per_word = 32 // bits
    want = np.zeros(words * 32, bool)
    for w in range(words * bits):
        total = sum(int(count[w * per_word + p]) << (bits * p) for p in range(per_word))
        total %= 1 << 32
        for p in range(per_word):
            want[w * per_word + p] = (total >> (bits * p)) & ((1 << bits) - 1) != 0
    got, U = O.index_add(maps, bits)
    assert _set(got) == set(np.flatnonzero(want).tolist()) and U == int(want.sum())
    if bits == 1:
        assert U < b.any(axis=0).sum()          # collisions lose positions at this density


def test_widen4_layout():
    rng = np.random.default_rng(3)
    (m,), b = _maps(rng, 1, 50, 0.3)
    wire = O.index_widen4(m)
    assert wire.size == 4 * m.size
    nib = (wire[:, None] >> (4 * np.arange(8, dtype=np.uint32))) & 0xF
    assert np.array_equal(nib.reshape(-1), b[0].astype(np.uint32))


@pytest.mark.parametrize("mode", [O.INDEX_ADD1, O.INDEX_ADD4])
def test_end_to_end_against_the_definition(mode):
    """What the decoder returns under an addition-simulated Index: for every position of
    the merged Index the sum of the entries of the ranks that kept it -- 0 for a position a
    carry invented -- and nothing for positions a carry erased.  20 ranks, so that the
    4-bit counters overflow too."""
    rng = np.random.default_rng(7)
    n, N = 6000, 20
    segs = [O.Segment(0, n, 50_000)]
    cfg = O.Config(dtype=O.F32, sizing_milli=3000, seed=3, part_unknowns=256, part_cells=768,
                   index_mode=mode)
    grads = []
    hot = rng.choice(n, 40, replace=False)      # positions exactly 16 ranks keep
    for r in range(N):
        g = rng.integers(-50, 51, n).astype(np.float32)
        g[hot] = 1000 + r if r < 16 else 0      # zeros are never kept
        grads.append(g)
    res = O.run_bucket(grads, cfg, segs)
    u_idx, u_val = D.sparse_sum(grads, O.F32, segs)     # true union and its sums
    union = dict(zip(u_idx.tolist(), u_val.tolist()))
    merged = _set(res.bitmap)
    assert merged != set(union)                         # the Index did collide
    if mode == O.INDEX_ADD4:                            # only full counters overflow
        assert set(hot.tolist()) - merged and set(union) - merged <= set(hot.tolist())
    assert res.decoded.n_unresolved == 0
    assert set(res.decoded.idx.tolist()) == merged
    want = np.array([union.get(int(i), 0.0) for i in res.decoded.idx])
    assert np.array_equal(res.decoded.val.astype(np.float64), want)
