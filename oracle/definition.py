"""End result of the method, written out as its definition -- TEST
INFRASTRUCTURE, NOT PRODUCT CODE.

The scheme is lossless (paper section 2.2; section 5 "inherits the potential
of lossless compression"), so when peeling completes, what the master device
holds is exactly  R = sum_r S(g_r),  where S zeroes everything but the
entries the sparsifier keeps (section 3.2).  This module computes R directly
with numpy, in float64, with no hashing, sketch or bit map involved, and with
its own selection routine (a lexicographic sort), independent of the C
oracle's.
"""
from __future__ import annotations

import numpy as np

F32, BF16 = 0, 1
FLAG_COMPRESS = 1


def widen(grad, dtype):
    """float32 view of a gradient given as float32 or as bf16 bit patterns."""
    if dtype == F32:
        return np.asarray(grad, np.float32)
    return (np.asarray(grad, np.uint16).astype(np.uint32) << 16).view(np.float32)


def select_positions(values_f32, k):
    """Positions kept by the sparsifier: the k largest magnitudes, ties to the
    lower position, exact zeros never kept (section 3.2)."""
    n = values_f32.size
    k = min(k, n)
    if k == 0:
        return np.zeros(0, np.int64)
    mag = np.abs(values_f32.astype(np.float64))
    order = np.lexsort((np.arange(n), -mag))  # magnitude desc, position asc
    top = order[:k]
    top = top[mag[top] > 0]
    return np.sort(top)


def sparse_sum(grads, dtype, segments):
    """(c-indices ascending, float64 sums) of R over the union of supports."""
    acc = {}
    c = 0
    for s in segments:
        if not (s.flags & FLAG_COMPRESS):
            continue
        k = (s.length * s.keep_ppm) // 1_000_000
        for g in grads:
            v = widen(g, dtype)[s.offset:s.offset + s.length]
            for p in select_positions(v, k):
                acc[c + int(p)] = acc.get(c + int(p), 0.0) + float(v[p])
        c = (c + s.length + 31) // 32 * 32
    idx = np.array(sorted(acc), np.int64)
    val = np.array([acc[i] for i in idx], np.float64)
    return idx, val
