"""ctypes front end of the TAGC oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Builds ``tagc_oracle.c`` with gcc on first use and exposes its functions, plus
``run_bucket`` which strings them together in the order of the paper's
Algorithm 1 (sparsify, create_index, All-Reduce(index) as OR, compress,
Reduce as sum, peeling_decompress) for N simulated ranks.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
module; it imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tagc_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libtagc_oracle.so")

F32, BF16 = 0, 1
SIZE_LOAD_FACTOR, SIZE_FIXED_RATIO = 0, 1
FLAG_COMPRESS = 1


def build(force: bool = False) -> str:
    """Compile the oracle (gcc -O2); returns the library path."""
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u32p, f32p, u64p = (C.POINTER(C.c_uint32), C.POINTER(C.c_float),
                            C.POINTER(C.c_uint64))
        L.tagco_key.restype = C.c_uint32
        L.tagco_key.argtypes = [C.c_uint32]
        L.tagco_keep_count.restype = C.c_uint64
        L.tagco_keep_count.argtypes = [C.c_uint64, C.c_uint32]
        L.tagco_sparsify_segment.restype = C.c_int64
        L.tagco_sparsify_segment.argtypes = [
            C.c_void_p, C.c_int, C.c_uint64, C.c_uint64, C.c_uint64,
            C.c_uint32, u32p, f32p, u32p, u64p]
        L.tagco_index_or.restype = C.c_uint64
        L.tagco_accumulate.restype = None
        L.tagco_accumulate.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_uint64,
                                       C.c_uint64, C.c_void_p]
        L.tagco_residual.restype = None
        L.tagco_residual.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint64, u32p,
                                     C.c_uint64, C.c_void_p]
        L.tagco_index_or.argtypes = [C.POINTER(u32p), C.c_uint32, C.c_uint64,
                                     u32p]
        L.tagco_layout.restype = None
        L.tagco_layout.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32,
                                   C.c_uint64, C.c_uint32, C.c_uint32, u64p,
                                   u64p, u64p]
        L.tagco_part_start.restype = C.c_uint64
        L.tagco_part_start.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        L.tagco_bounds.restype = None
        L.tagco_bounds.argtypes = [u32p, C.c_uint64, C.c_uint64, C.c_uint64,
                                   u32p]
        L.tagco_mix32.restype = C.c_uint32
        L.tagco_mix32.argtypes = [C.c_uint32]
        L.tagco_seed_word.restype = C.c_uint32
        L.tagco_seed_word.argtypes = [C.c_uint64, C.c_uint32]
        L.tagco_hash.restype = None
        L.tagco_hash.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32,
                                 C.c_uint32, u32p, C.POINTER(C.c_int32)]
        L.tagco_salts.restype = C.c_int
        L.tagco_salts.argtypes = [u32p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64,
                                  C.c_uint64, u32p]
        L.tagco_encode.restype = None
        L.tagco_encode.argtypes = [u32p, f32p, C.c_uint64, u32p, C.c_uint64,
                                   C.c_uint64, C.c_uint64, u32p, C.c_int, u32p, f32p]
        L.tagco_quantize_cells_bf16.restype = None
        L.tagco_quantize_cells_bf16.argtypes = [f32p, C.c_uint64]
        L.tagco_index_add.restype = C.c_uint64
        L.tagco_index_add.argtypes = [C.POINTER(u32p), C.c_uint32, C.c_uint64, C.c_uint32,
                                      u32p]
        L.tagco_index_widen4.restype = None
        L.tagco_index_widen4.argtypes = [u32p, C.c_uint64, u32p]
        L.tagco_sum.restype = None
        L.tagco_sum.argtypes = [C.POINTER(f32p), C.c_uint32, C.c_uint64, f32p]
        L.tagco_peel.restype = C.c_int
        L.tagco_peel.argtypes = [u32p, C.c_uint64, C.c_uint64, C.c_uint64,
                                 C.c_uint64, C.c_uint64, u32p, C.c_int, f32p, u32p,
                                 f32p, u32p, u32p, u64p]
        L.tagco_estimate.restype = C.c_uint64
        L.tagco_estimate.argtypes = [u32p, u32p, C.c_uint64, C.c_uint64, C.c_uint64,
                                     C.c_uint64, u32p, f32p, f32p]
        L.tagco_wire_bits_per_param.restype = C.c_double
        L.tagco_wire_bits_per_param.argtypes = [C.c_double, C.c_double,
                                                C.c_int]
        _lib = L
    return _lib


def _u32p(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


def _f32p(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


# --------------------------------------------------------------------------
# bucket description


@dataclass
class Segment:
    offset: int          # element offset in the rank's gradient buffer
    length: int          # n_l
    keep_ppm: int        # survivors per million (1 - theta)
    flags: int = FLAG_COMPRESS


@dataclass
class Config:
    dtype: int = F32
    sizing: int = SIZE_LOAD_FACTOR
    sizing_milli: int = 3000
    seed: int = 0
    part_unknowns: int = 8192    # P_cap
    part_cells: int = 12288      # T_cap (multiple of 3)
    index_mode: int = 0          # INDEX_OR1 | INDEX_ADD1 | INDEX_ADD4
    cell_type: int = 0           # CELL_F32 | CELL_BF16: what a sketch cell is on the wire


def c_offsets(segments):
    """c-index offset of every compressed segment (None for skipped ones) and
    the padded total n_c.  Layer-selective compression (section 3.2,
    "Selective Compressing"): segments without the COMPRESS flag get no index
    bits and no sketch cells.  Offsets are rounded up to a multiple of 32 so a
    bit-map word never belongs to two segments."""
    offs, c = [], 0
    for s in segments:
        if s.flags & FLAG_COMPRESS:
            offs.append(c)
            c = (c + s.length + 31) // 32 * 32
        else:
            offs.append(None)
    return offs, c


def keep_count(n, ppm):
    return int(lib().tagco_keep_count(n, ppm))


def _as_raw(grad, dtype):
    """grad: numpy float32 array (F32) or uint16 array of bf16 bit patterns."""
    want = np.float32 if dtype == F32 else np.uint16
    a = np.ascontiguousarray(grad)
    if a.dtype != want:
        raise TypeError("oracle expects %s for dtype %d, got %s"
                        % (want, dtype, a.dtype))
    return a


@dataclass
class RankState:
    idx: np.ndarray
    val: np.ndarray
    cnt: int
    seg_cnt: list
    bitmap: np.ndarray
    sketch: np.ndarray | None = None


def sparsify(grad, cfg: Config, segments) -> RankState:
    """sparsify + create_index over all compressed segments of one rank."""
    L = lib()
    g = _as_raw(grad, cfg.dtype)
    offs, n_c = c_offsets(segments)
    cap = sum(keep_count(s.length, s.keep_ppm) for s in segments
              if s.flags & FLAG_COMPRESS)
    idx = np.zeros(max(cap, 1), np.uint32)
    val = np.zeros(max(cap, 1), np.float32)
    bitmap = np.zeros(max(n_c // 32, 1), np.uint32)
    pos, seg_cnt = 0, []
    for s, co in zip(segments, offs):
        if co is None:
            seg_cnt.append(0)
            continue
        if s.offset + s.length > g.size:
            raise ValueError("segment exceeds gradient buffer")
        k = keep_count(s.length, s.keep_ppm)
        c = C.c_uint64(0)
        nf = L.tagco_sparsify_segment(
            g.ctypes.data_as(C.c_void_p), cfg.dtype, s.offset, s.length, k, co,
            _u32p(idx[pos:]), _f32p(val[pos:]), _u32p(bitmap), C.byref(c))
        if nf < 0:
            raise MemoryError("oracle allocation failed")
        if nf > 0:
            raise ValueError("non-finite gradient values: %d" % nf)
        seg_cnt.append(int(c.value))
        pos += int(c.value)
    return RankState(idx[:pos].copy(), val[:pos].copy(), pos, seg_cnt, bitmap)


def error_feedback_step(grad, acc, cfg: Config, segments):
    """Algorithm 1 lines 1-2 for one rank: g' = g + acc over the compressed segments,
    sparsify(g'), and acc_next = g' minus what was selected.  `grad`, `acc`: raw arrays
    as for `sparsify`.  Returns (RankState of g', acc_next raw array).  Elements outside
    the compressed segments are passed through unchanged in acc_next."""
    L = lib()
    g, a = _as_raw(grad, cfg.dtype), _as_raw(acc, cfg.dtype)
    if a.size < g.size:
        raise ValueError("accumulator shorter than the gradient")
    summed = a.copy()
    offs, _ = c_offsets(segments)
    for s, co in zip(segments, offs):
        if co is None:
            continue
        L.tagco_accumulate(g.ctypes.data_as(C.c_void_p), a.ctypes.data_as(C.c_void_p),
                           cfg.dtype, s.offset, s.length, summed.ctypes.data_as(C.c_void_p))
    st = sparsify(summed[:g.size] if summed.size != g.size else summed, cfg, segments)
    acc_next = summed.copy()
    pos = 0
    for s, co, c in zip(segments, offs, st.seg_cnt):
        if co is None:
            continue
        sel = np.ascontiguousarray(st.idx[pos:pos + c] - np.uint32(co))
        L.tagco_residual(summed.ctypes.data_as(C.c_void_p), cfg.dtype, s.offset, s.length,
                         _u32p(sel) if c else None, c, acc_next.ctypes.data_as(C.c_void_p))
        pos += c
    return st, acc_next


def index_or(bitmaps):
    L = lib()
    n = len(bitmaps)
    words = bitmaps[0].size
    arr = (C.POINTER(C.c_uint32) * n)(*[_u32p(b) for b in bitmaps])
    out = np.zeros(words, np.uint32)
    U = L.tagco_index_or(arr, n, words, _u32p(out))
    return out, int(U)


INDEX_OR1, INDEX_ADD1, INDEX_ADD4 = 0, 1, 2


def index_add(bitmaps, bits):
    """All-Reduce of the Index simulated by addition (section 2.2), 1-bit or 4-bit
    fields; returns the merged 1-bit Index and its number of set bits."""
    n, words = len(bitmaps), bitmaps[0].size
    arr = (C.POINTER(C.c_uint32) * n)(*[_u32p(b) for b in bitmaps])
    out = np.zeros(words, np.uint32)
    U = lib().tagco_index_add(arr, n, words, bits, _u32p(out))
    return out, int(U)


def index_widen4(bitmap):
    """A rank's 4-bit wire Index (four words per word of the local 1-bit Index)."""
    bitmap = np.ascontiguousarray(bitmap, np.uint32)
    out = np.zeros(4 * bitmap.size, np.uint32)
    lib().tagco_index_widen4(_u32p(bitmap), bitmap.size, _u32p(out))
    return out


def merge_index(bitmaps, mode):
    if mode == INDEX_OR1:
        return index_or(bitmaps)
    return index_add(bitmaps, 1 if mode == INDEX_ADD1 else 4)


def layout(U, cfg: Config, n_real):
    A, ms, m = C.c_uint64(), C.c_uint64(), C.c_uint64()
    lib().tagco_layout(U, cfg.sizing, cfg.sizing_milli, n_real,
                       cfg.part_unknowns, cfg.part_cells, C.byref(A),
                       C.byref(ms), C.byref(m))
    return int(A.value), int(ms.value), int(m.value)


def bounds(bitmap, n_c, U, A):
    bnd = np.zeros(A + 1, np.uint32)
    lib().tagco_bounds(_u32p(bitmap), n_c, U, A, _u32p(bnd))
    return bnd


def hash_slot(i, seed, j, m_sub, salt=0):
    slot, sign = C.c_uint32(), C.c_int32()
    lib().tagco_hash(i, seed, j, salt, m_sub, C.byref(slot), C.byref(sign))
    return int(slot.value), int(sign.value)


SALT_LIMIT = 16


def salts(bitmap, n_c, U, A, m_sub, seed):
    """Per-partition hash salts, a function of the merged Index and the seed alone: the
    smallest salt under which no two non-zeros of the partition share all three cells."""
    out = np.zeros(max(A, 1), np.uint32)
    if lib().tagco_salts(_u32p(bitmap), n_c, U, A, m_sub, seed, _u32p(out)) != 0:
        raise MemoryError("oracle allocation failed")
    return out[:A]


def _salt_arg(salt, A):
    """`salt=None` stands for the all-zero salts (every partition hashed as it is)."""
    if salt is None:
        return np.zeros(max(A, 1), np.uint32)
    s = np.ascontiguousarray(salt, np.uint32)
    if s.size < A:
        raise ValueError("one salt per partition expected")
    return s if s.size else np.zeros(1, np.uint32)


def encode(idx, val, bnd, A, m_sub, seed, plus_only=False, mask=None, salt=None):
    m = 3 * A * m_sub
    sk = np.zeros(max(m, 1), np.float32)
    idx = np.ascontiguousarray(idx, np.uint32)
    val = np.ascontiguousarray(val, np.float32)
    lib().tagco_encode(_u32p(idx), _f32p(val), idx.size, _u32p(bnd), A, m_sub,
                       seed, _u32p(_salt_arg(salt, A)), int(plus_only),
                       None if mask is None else _u32p(mask), _f32p(sk))
    return sk[:m]


CELL_F32, CELL_BF16 = 0, 1


def quantize_cells_bf16(sketch):
    """A rank's sketch as it goes on the wire with 16-bit cells: every cell rounded to the
    nearest bfloat16, ties to even (returned as float32 values)."""
    out = np.array(sketch, np.float32, copy=True)
    if out.size:
        lib().tagco_quantize_cells_bf16(_f32p(out), out.size)
    return out


def sketch_sum(sketches):
    n = len(sketches)
    m = sketches[0].size
    keep = [np.ascontiguousarray(s, np.float32) for s in sketches]
    arr = (C.POINTER(C.c_float) * n)(*[_f32p(s) for s in keep])
    out = np.zeros(max(m, 1), np.float32)
    if m:
        lib().tagco_sum(arr, n, m, _f32p(out))
    return out[:m]


@dataclass
class Decoded:
    idx: np.ndarray
    val: np.ndarray
    round: np.ndarray
    rounds: int
    n_unresolved: int
    residual: np.ndarray = field(default=None, repr=False)


def peel(bitmap, n_c, U, A, m_sub, seed, sketch, plus_only=False, salt=None) -> Decoded:
    idx = np.zeros(max(U, 1), np.uint32)
    val = np.zeros(max(U, 1), np.float32)
    rnd = np.zeros(max(U, 1), np.uint32)
    work = np.array(sketch, np.float32, copy=True)
    if work.size == 0:
        work = np.zeros(1, np.float32)
    rounds, unres = C.c_uint32(), C.c_uint64()
    rc = lib().tagco_peel(_u32p(bitmap), n_c, U, A, m_sub, seed,
                          _u32p(_salt_arg(salt, A)),
                          int(plus_only), _f32p(work), _u32p(idx), _f32p(val),
                          _u32p(rnd), C.byref(rounds), C.byref(unres))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return Decoded(idx[:U], val[:U], rnd[:U], int(rounds.value),
                   int(unres.value), work)


DECODE_PEEL, DECODE_PEEL_ESTIMATE, DECODE_ESTIMATE = 0, 1, 2


def estimate(dec: Decoded, A, m_sub, seed, sketch, only_unresolved=True, salt=None) -> int:
    """Count Sketch point queries (median of the three signed readings) for the unknowns
    of `dec` that peeling left (or for all of them), on `sketch`; fills dec.val in place
    and returns how many were estimated (section 2.2, the estimation algorithm)."""
    U = dec.idx.size
    if U == 0:
        return 0
    sk = np.ascontiguousarray(sketch, np.float32)
    rnd = np.ascontiguousarray(dec.round, np.uint32)
    return int(lib().tagco_estimate(
        _u32p(dec.idx), _u32p(rnd) if only_unresolved else None, U, A, m_sub, seed,
        _u32p(_salt_arg(salt, A)), _f32p(sk), _f32p(dec.val)))


def decompress(bitmap, n_c, U, A, m_sub, seed, sketch, mode=DECODE_PEEL,
               salt=None) -> Decoded:
    """peeling_decompress of Algorithm 1, optionally followed by estimation of what it
    could not recover (mode 1), or estimation alone on the raw sketch (mode 2)."""
    if mode == DECODE_ESTIMATE:
        bits = np.unpackbits(np.ascontiguousarray(bitmap, np.uint32).view(np.uint8),
                             bitorder="little")[:n_c]
        idx = np.flatnonzero(bits).astype(np.uint32)  # the unknowns, ascending
        assert idx.size == U
        dec = Decoded(idx, np.zeros(U, np.float32), np.zeros(U, np.uint32), 0, U,
                      np.array(sketch, np.float32, copy=True))
        estimate(dec, A, m_sub, seed, dec.residual, only_unresolved=False, salt=salt)
        return dec
    dec = peel(bitmap, n_c, U, A, m_sub, seed, sketch, salt=salt)
    if mode == DECODE_PEEL_ESTIMATE and dec.n_unresolved:
        estimate(dec, A, m_sub, seed, dec.residual, salt=salt)
    return dec


@dataclass
class BucketResult:
    ranks: list
    bitmap: np.ndarray
    U: int
    A: int
    m_sub: int
    m: int
    bnd: np.ndarray
    sketch: np.ndarray
    decoded: Decoded
    n_c: int
    salt: np.ndarray = None


def run_bucket(grads, cfg: Config, segments, plus_only=False,
               decode_mode=DECODE_PEEL, salted=True) -> BucketResult:
    """Algorithm 1 for one bucket and len(grads) simulated ranks.  `salted=False` leaves
    every partition's salt at 0 (for tests that show what the salts are for)."""
    offs, n_c = c_offsets(segments)
    n_real = sum(s.length for s in segments if s.flags & FLAG_COMPRESS)
    ranks = [sparsify(g, cfg, segments) for g in grads]
    bitmap, U = merge_index([r.bitmap for r in ranks], cfg.index_mode)
    A, m_sub, m = layout(U, cfg, n_real)
    bnd = bounds(bitmap, n_c, U, A)
    salt = (salts(bitmap, n_c, U, A, m_sub, cfg.seed) if salted
            else np.zeros(A, np.uint32))
    mask = None if cfg.index_mode == INDEX_OR1 else bitmap
    for r in ranks:
        r.sketch = encode(r.idx, r.val, bnd, A, m_sub, cfg.seed, plus_only, mask, salt)
        if cfg.cell_type == CELL_BF16:
            r.sketch = quantize_cells_bf16(r.sketch)
    total = sketch_sum([r.sketch for r in ranks])
    if decode_mode == DECODE_PEEL:
        dec = peel(bitmap, n_c, U, A, m_sub, cfg.seed, total, plus_only, salt)
    else:
        assert not plus_only
        dec = decompress(bitmap, n_c, U, A, m_sub, cfg.seed, total, decode_mode, salt)
    return BucketResult(ranks, bitmap, U, A, m_sub, m, bnd, total, dec, n_c, salt)


def wire_bits_per_param(index_bits, ratio, lhc=False):
    return float(lib().tagco_wire_bits_per_param(index_bits, ratio, int(lhc)))
