"""ctypes binding of libtagc: the same entry points as include/tagc.h, argument
marshalling only.  Every step of the hot path runs inside the library's HIP
kernels; torch is used for device memory and streams, nothing else.

The library must have been built (python -m paper_2504_05638_amd.build); a
missing library is an error, there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtagc.so")

TAGC_F32, TAGC_BF16 = 0, 1
TAGC_SIZE_LOAD_FACTOR, TAGC_SIZE_FIXED_RATIO = 0, 1
TAGC_INDEX_OR1, TAGC_INDEX_ADD1, TAGC_INDEX_ADD4 = 0, 1, 2
TAGC_PHASE_INDEX, TAGC_PHASE_SKETCH = 1, 2
TAGC_SEG_COMPRESS = 1
TAGC_CNT_TOTAL, TAGC_CNT_NONFINITE, TAGC_CNT_FLAGS, TAGC_CNT_DENSE = 0, 1, 2, 3
TAGC_CNT_RESERVED, TAGC_CNT_SEG0 = 4, 5
TAGC_HDR_U, TAGC_HDR_A, TAGC_HDR_MSUB, TAGC_HDR_M, TAGC_HDR_WORDS = 0, 1, 2, 3, 8
TAGC_ST_UNRESOLVED, TAGC_ST_ROUNDS, TAGC_ST_FLAGS, TAGC_ST_WORDS = 0, 1, 2, 8
TAGC_ST_ESTIMATED = 3
TAGC_DECODE_PEEL, TAGC_DECODE_PEEL_ESTIMATE, TAGC_DECODE_ESTIMATE = 0, 1, 2
TAGC_CELL_F32, TAGC_CELL_BF16 = 0, 1
TAGC_FLAG_OVERFLOW = 2
TAGC_STATIC_WORKSPACE_BYTES = 16 << 20

EXPORTS = ["tagc_plan", "tagc_plan_destroy", "tagc_plan_sizes",
           "tagc_plan_upload", "tagc_compress", "tagc_compress_static", "tagc_feedback_apply", "tagc_aggregate",
           "tagc_decompress", "tagc_reduce_decompress", "tagc_profile_enable", "tagc_profile_read",
           "tagc_hash_host", "tagc_strerror"]


class tagc_segment(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("length", C.c_uint64),
                ("keep_ppm", C.c_uint32), ("flags", C.c_uint32)]


class tagc_config(C.Structure):
    _fields_ = [("dtype", C.c_uint32), ("n_ranks", C.c_uint32),
                ("n_hash", C.c_uint32), ("sizing", C.c_uint32),
                ("sizing_milli", C.c_uint32), ("index_mode", C.c_uint32),
                ("part_unknowns", C.c_uint32), ("part_cells", C.c_uint32),
                ("seed", C.c_uint64), ("decode_mode", C.c_uint32),
                ("cell_type", C.c_uint32), ("decode_workgroups", C.c_uint32),
                ("reserved", C.c_uint32)]


_SIZE_FIELDS = [
    "n_seg_compressed", "n_real", "n_c", "bitmap_words", "pair_capacity",
    "union_capacity", "partition_capacity", "sketch_cells_capacity",
    "part_unknowns", "part_cells", "grad_elems", "table_bytes",
    "rank_idx_bytes", "rank_val_bytes", "rank_cnt_bytes", "rank_bitmap_bytes",
    "rank_sketch_bytes", "rank_workspace_bytes", "shared_bitmap_bytes",
    "shared_sketch_bytes", "shared_header_bytes", "shared_bounds_bytes",
    "shared_workspace_bytes", "shared_status_bytes", "out_idx_bytes",
    "out_val_bytes", "out_dense_bytes"]


class tagc_sizes(C.Structure):
    _fields_ = ([(n, C.c_uint64) for n in _SIZE_FIELDS]
                + [("wire_index_bits", C.c_double),
                   ("wire_sketch_bits", C.c_double),
                   ("wire_total_bits", C.c_double)])

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class tagc_rank_buffers(C.Structure):
    _fields_ = [("idx", C.c_void_p), ("val", C.c_void_p), ("cnt", C.c_void_p),
                ("bitmap", C.c_void_p), ("sketch", C.c_void_p),
                ("workspace", C.c_void_p), ("acc", C.c_void_p)]


class tagc_shared_buffers(C.Structure):
    _fields_ = [("table", C.c_void_p), ("bitmap", C.c_void_p),
                ("sketch", C.c_void_p), ("header", C.c_void_p),
                ("bounds", C.c_void_p), ("workspace", C.c_void_p),
                ("status", C.c_void_p)]


class TagcError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s: %s (%d)" % (what, strerror(code), code))
        self.code = code


_lib = None


def lib():
    """Loads libtagc.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libtagc.so is missing: build it with "
                "`python -m paper_2504_05638_amd.build` (there is no fallback)")
        # libtagc uses whatever HIP runtime the process has loaded.  A caller that hands it
        # torch's device memory and streams needs that to be torch's own copy, so torch (when
        # there is one) is loaded first: the other order ends in HIP errors at the first
        # call that takes a stream.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.tagc_plan.restype = C.c_int
        L.tagc_plan.argtypes = [C.POINTER(tagc_config), C.POINTER(tagc_segment),
                                C.c_uint32, C.POINTER(vp)]
        L.tagc_plan_destroy.restype = None
        L.tagc_plan_destroy.argtypes = [vp]
        L.tagc_plan_sizes.restype = C.c_int
        L.tagc_plan_sizes.argtypes = [vp, C.POINTER(tagc_sizes)]
        L.tagc_plan_upload.restype = C.c_int
        L.tagc_plan_upload.argtypes = [vp, vp, vp]
        L.tagc_compress.restype = C.c_int
        L.tagc_compress.argtypes = [vp, C.c_uint32, vp,
                                    C.POINTER(tagc_rank_buffers),
                                    C.POINTER(tagc_shared_buffers), vp]
        L.tagc_compress_static.restype = C.c_int
        L.tagc_compress_static.argtypes = L.tagc_compress.argtypes
        L.tagc_aggregate.restype = C.c_int
        L.tagc_feedback_apply.restype = C.c_int
        L.tagc_feedback_apply.argtypes = [vp, C.POINTER(tagc_rank_buffers),
                                          C.POINTER(tagc_shared_buffers), vp]
        L.tagc_aggregate.argtypes = [vp, C.c_uint32,
                                     C.POINTER(tagc_rank_buffers), C.c_uint32,
                                     C.POINTER(tagc_shared_buffers), vp]
        L.tagc_decompress.restype = C.c_int
        L.tagc_decompress.argtypes = [vp, C.POINTER(tagc_shared_buffers), vp,
                                      vp, vp, vp]
        L.tagc_reduce_decompress.restype = C.c_int
        L.tagc_reduce_decompress.argtypes = [vp, C.POINTER(tagc_rank_buffers), C.c_uint32,
                                             C.POINTER(tagc_shared_buffers), vp, vp, vp, vp]
        L.tagc_profile_enable.restype = C.c_int
        L.tagc_profile_enable.argtypes = [C.c_int]
        L.tagc_profile_read.restype = C.c_int
        L.tagc_profile_read.argtypes = [C.POINTER(C.c_char_p),
                                        C.POINTER(C.c_double),
                                        C.POINTER(C.c_uint64), C.c_uint32]
        L.tagc_hash_host.restype = None
        L.tagc_hash_host.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32,
                                     C.c_uint32, C.POINTER(C.c_uint32),
                                     C.POINTER(C.c_int32)]
        L.tagc_strerror.restype = C.c_char_p
        L.tagc_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def strerror(code):
    return lib().tagc_strerror(code).decode()


def _check(rc, what):
    if rc != 0:
        raise TagcError(rc, what)


# ---------------------------------------------------------------- entry points


def tagc_plan(config: tagc_config, segments) -> C.c_void_p:
    """segments: iterable of (offset, length, keep_ppm, flags[, ...])."""
    segs = list(segments)
    arr = (tagc_segment * max(len(segs), 1))()
    for i, s in enumerate(segs):
        arr[i] = tagc_segment(int(s[0]), int(s[1]), int(s[2]), int(s[3]))
    out = C.c_void_p()
    _check(lib().tagc_plan(C.byref(config), arr, len(segs), C.byref(out)),
           "tagc_plan")
    return out


def tagc_plan_destroy(plan):
    lib().tagc_plan_destroy(plan)


def tagc_plan_sizes(plan) -> tagc_sizes:
    z = tagc_sizes()
    _check(lib().tagc_plan_sizes(plan, C.byref(z)), "tagc_plan_sizes")
    return z


def tagc_plan_upload(plan, table_dev: int, stream: int = 0):
    _check(lib().tagc_plan_upload(plan, table_dev, stream), "tagc_plan_upload")


def tagc_compress(plan, phase, grad_dev, rank: tagc_rank_buffers,
                  shared: tagc_shared_buffers, stream: int = 0):
    _check(lib().tagc_compress(plan, phase, grad_dev, C.byref(rank),
                               C.byref(shared), stream), "tagc_compress")


def tagc_compress_static(plan, phase, grad_dev, rank: tagc_rank_buffers,
                         shared: tagc_shared_buffers, stream: int = 0):
    """tagc_compress on the library's own workspace (rank.workspace is ignored)."""
    _check(lib().tagc_compress_static(plan, phase, grad_dev, C.byref(rank),
                                      C.byref(shared), stream), "tagc_compress_static")


def tagc_feedback_apply(plan, rank: tagc_rank_buffers, shared: tagc_shared_buffers,
                        stream: int = 0):
    _check(lib().tagc_feedback_apply(plan, C.byref(rank), C.byref(shared), stream),
           "tagc_feedback_apply")


def tagc_aggregate(plan, phase, ranks, shared: tagc_shared_buffers,
                   stream: int = 0):
    arr = (tagc_rank_buffers * len(ranks))(*ranks)
    _check(lib().tagc_aggregate(plan, phase, arr, len(ranks), C.byref(shared),
                                stream), "tagc_aggregate")


def tagc_decompress(plan, shared: tagc_shared_buffers, idx_out, val_out,
                    dense_out=None, stream: int = 0):
    _check(lib().tagc_decompress(plan, C.byref(shared), idx_out, val_out,
                                 dense_out, stream), "tagc_decompress")


def tagc_reduce_decompress(plan, ranks, shared: tagc_shared_buffers, idx_out, val_out,
                           dense_out=None, stream: int = 0):
    arr = (tagc_rank_buffers * len(ranks))(*ranks)
    _check(lib().tagc_reduce_decompress(plan, arr, len(ranks), C.byref(shared), idx_out,
                                        val_out, dense_out, stream), "tagc_reduce_decompress")


def tagc_profile_enable(on: bool):
    _check(lib().tagc_profile_enable(int(on)), "tagc_profile_enable")


def tagc_profile_read(cap: int = 64):
    """{kernel name: (total ms, launches)} since the last read."""
    names = (C.c_char_p * cap)()
    ms = (C.c_double * cap)()
    cnt = (C.c_uint64 * cap)()
    n = lib().tagc_profile_read(names, ms, cnt, cap)
    if n < 0:
        raise TagcError(n, "tagc_profile_read")
    return {names[i].decode(): (ms[i], int(cnt[i])) for i in range(n)}


def tagc_hash_host(i, seed, j, m_sub, salt=0):
    slot, sign = C.c_uint32(), C.c_int32()
    lib().tagc_hash_host(i, seed, j, salt, m_sub, C.byref(slot), C.byref(sign))
    return int(slot.value), int(sign.value)
