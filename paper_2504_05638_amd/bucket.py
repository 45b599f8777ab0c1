"""Device-memory plumbing around the libtagc entry points.

`TagcBucket` owns the torch tensors a bucket needs (sized by tagc_plan_sizes),
hands their addresses to the library, and offers read-backs for tests and
tools.  It performs no arithmetic of the method itself.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _stream_ptr(stream=None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _bytes(n, device):
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(int(n), 16), dtype=torch.uint8, device=device)


class TagcBucket:
    """One gradient bucket: plan + device buffers for `n_ranks` simulated ranks."""

    def __init__(self, segments, dtype, n_ranks, sizing_milli=3000,
                 sizing=B.TAGC_SIZE_LOAD_FACTOR, seed=0, part_unknowns=0,
                 part_cells=0, device="cuda", dense=False, share=None, min_bytes=None,
                 error_feedback=False, decode_mode=B.TAGC_DECODE_PEEL,
                 index_mode=B.TAGC_INDEX_OR1, cell_type=B.TAGC_CELL_F32,
                 decode_workgroups=0):
        if not torch.cuda.is_available():
            raise RuntimeError("libtagc needs a GPU: no CPU path exists")
        self.device = torch.device(device)
        self.cfg = B.tagc_config(dtype=dtype, n_ranks=n_ranks, n_hash=3,
                                 sizing=sizing, sizing_milli=sizing_milli,
                                 index_mode=index_mode,
                                 part_unknowns=part_unknowns,
                                 part_cells=part_cells, seed=seed,
                                 decode_mode=decode_mode, cell_type=cell_type,
                                 decode_workgroups=decode_workgroups)
        self.segments = [tuple(s[:4]) for s in segments]
        self.plan = B.tagc_plan(self.cfg, self.segments)
        # decode_workgroups only shapes tagc_decompress's launch: a plan that differs in
        # nothing else works on the same buffers (for a caller that sometimes decodes with
        # the device to itself)
        self.plan_whole = None
        if decode_workgroups:
            cfg0 = B.tagc_config.from_buffer_copy(self.cfg)
            cfg0.decode_workgroups = 0
            self.plan_whole = B.tagc_plan(cfg0, self.segments)
        self.sizes = B.tagc_plan_sizes(self.plan)
        self.n_ranks = n_ranks
        z, dev = self.sizes, self.device
        self._share = share
        self._min_bytes = min_bytes or {}
        self._t = {}
        al = self._alloc
        self.table = _bytes(z.table_bytes, dev)           # per bucket, never shared
        self.sh_bitmap = al("sh_bitmap", z.shared_bitmap_bytes)
        self.sh_sketch = al("sh_sketch", z.shared_sketch_bytes)
        self.sh_header = al("sh_header", 4 * B.TAGC_HDR_WORDS)
        self.sh_bounds = al("sh_bounds", z.shared_bounds_bytes)
        self.sh_ws = al("sh_ws", z.shared_workspace_bytes)
        self.sh_status = al("sh_status", 4 * B.TAGC_ST_WORDS)
        self.shared = B.tagc_shared_buffers(
            self.table.data_ptr(), self.sh_bitmap.data_ptr(),
            self.sh_sketch.data_ptr(), self.sh_header.data_ptr(),
            self.sh_bounds.data_ptr(), self.sh_ws.data_ptr(),
            self.sh_status.data_ptr())
        self.rank_ws = al("rank_ws", z.rank_workspace_bytes)  # ranks run in turn
        self.rk = []
        self._rk_tensors = []
        for r in range(n_ranks):
            t = dict(idx=al("idx%d" % r, z.rank_idx_bytes),
                     val=al("val%d" % r, z.rank_val_bytes),
                     cnt=al("cnt%d" % r, z.rank_cnt_bytes),
                     bitmap=al("bitmap%d" % r, z.rank_bitmap_bytes),
                     sketch=al("sketch%d" % r, z.rank_sketch_bytes))
            if error_feedback:
                # the rank's error-feedback state: its accumulator and its own Index, both
                # zero before the first step and never shared with another bucket
                t["bitmap"] = torch.zeros(max(int(z.rank_bitmap_bytes), 16), dtype=torch.uint8,
                                          device=dev)
                t["acc"] = torch.zeros(max(int(z.grad_elems), 8), device=dev,
                                       dtype=torch.float32 if dtype == B.TAGC_F32
                                       else torch.bfloat16)
            self._rk_tensors.append(t)
            self.rk.append(B.tagc_rank_buffers(
                t["idx"].data_ptr(), t["val"].data_ptr(), t["cnt"].data_ptr(),
                t["bitmap"].data_ptr(), t["sketch"].data_ptr(),
                self.rank_ws.data_ptr(), t["acc"].data_ptr() if error_feedback else None))
        self.out_idx = al("out_idx", z.out_idx_bytes)
        self.out_val = al("out_val", z.out_val_bytes)
        self.out_dense = al("out_dense", z.out_dense_bytes) if dense else None
        B.tagc_plan_upload(self.plan, self.table.data_ptr(), _stream_ptr())
        torch.cuda.current_stream().synchronize()

    def _alloc(self, name, nbytes):
        """A device buffer of at least nbytes; taken from `share` (another bucket that
        is never in flight at the same time) when that one is large enough."""
        nbytes = max(int(nbytes), int(self._min_bytes.get(name.rstrip("0123456789"), 0)))
        t = None
        if self._share is not None:
            t = self._share._t.get(name)
            if t is not None and t.numel() < nbytes:
                t = None
        if t is None:
            t = _bytes(nbytes, self.device)
        self._t[name] = t
        return t

    def close(self):
        if self.plan is not None:
            B.tagc_plan_destroy(self.plan)
            self.plan = None
        if getattr(self, "plan_whole", None) is not None:
            B.tagc_plan_destroy(self.plan_whole)
            self.plan_whole = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------ the path

    def _check_grad(self, grad):
        want = torch.float32 if self.cfg.dtype == B.TAGC_F32 else torch.bfloat16
        if grad.dtype != want or not grad.is_cuda or not grad.is_contiguous():
            raise ValueError("gradient must be a contiguous %s CUDA tensor" % want)
        if grad.numel() < self.sizes.grad_elems:
            raise ValueError("gradient buffer shorter than the segment table needs")

    def feedback_apply(self, r, stream=None):
        """Clears in rank r's accumulator what the rank sent (optional, see tagc.h)."""
        B.tagc_feedback_apply(self.plan, self.rk[r], self.shared, _stream_ptr(stream))

    def compress_index(self, r, grad, stream=None):
        self._check_grad(grad)
        B.tagc_compress(self.plan, B.TAGC_PHASE_INDEX, grad.data_ptr(), self.rk[r],
                        self.shared, _stream_ptr(stream))

    def aggregate_index(self, n_ranks=None, stream=None):
        B.tagc_aggregate(self.plan, B.TAGC_PHASE_INDEX,
                         self.rk[:n_ranks or self.n_ranks], self.shared,
                         _stream_ptr(stream))

    def compress_sketch(self, r, stream=None):
        B.tagc_compress(self.plan, B.TAGC_PHASE_SKETCH, None, self.rk[r], self.shared,
                        _stream_ptr(stream))

    def aggregate_sketch(self, n_ranks=None, stream=None):
        B.tagc_aggregate(self.plan, B.TAGC_PHASE_SKETCH,
                         self.rk[:n_ranks or self.n_ranks], self.shared,
                         _stream_ptr(stream))

    def decompress(self, stream=None, whole_device=False):
        plan = self.plan_whole if whole_device and self.plan_whole is not None else self.plan
        B.tagc_decompress(plan, self.shared, self.out_idx.data_ptr(),
                          self.out_val.data_ptr(),
                          self.out_dense.data_ptr() if self.out_dense is not None else None,
                          _stream_ptr(stream))

    def reduce_decompress(self, n_ranks=None, stream=None, whole_device=False):
        """Sketch sum and decode in one call (the summed sketch is never written)."""
        plan = self.plan_whole if whole_device and self.plan_whole is not None else self.plan
        B.tagc_reduce_decompress(plan, self.rk[:n_ranks or self.n_ranks], self.shared,
                                 self.out_idx.data_ptr(), self.out_val.data_ptr(),
                                 self.out_dense.data_ptr() if self.out_dense is not None else None,
                                 _stream_ptr(stream))

    def run(self, grads, stream=None, whole_device_decode=False, fused=False):
        """The whole hot path for one bucket; grads[r] is rank r's buffer.  `fused`: the
        sketches are summed by the decoder (tagc_reduce_decompress)."""
        n = len(grads)
        for r in range(n):
            self.compress_index(r, grads[r], stream)
        self.aggregate_index(n, stream)
        for r in range(n):
            self.compress_sketch(r, stream)
        if fused:
            self.reduce_decompress(n, stream, whole_device_decode)
        else:
            self.aggregate_sketch(n, stream)
            self.decompress(stream, whole_device_decode)

    # ---------------------------------------------------------- read-backs

    @staticmethod
    def _np(t, dtype, n=None):
        a = t.cpu().numpy().view(dtype)
        return a[:n].copy() if n is not None else a.copy()

    def header(self):
        h = self._np(self.sh_header, np.uint32, B.TAGC_HDR_WORDS)
        return dict(U=int(h[B.TAGC_HDR_U]), A=int(h[B.TAGC_HDR_A]),
                    m_sub=int(h[B.TAGC_HDR_MSUB]), m=int(h[B.TAGC_HDR_M]))

    def status(self):
        s = self._np(self.sh_status, np.uint32, B.TAGC_ST_WORDS)
        return dict(n_unresolved=int(s[B.TAGC_ST_UNRESOLVED]),
                    rounds=int(s[B.TAGC_ST_ROUNDS]), flags=int(s[B.TAGC_ST_FLAGS]),
                    n_estimated=int(s[B.TAGC_ST_ESTIMATED]))

    def rank_counts(self, r):
        c = self._np(self._rk_tensors[r]["cnt"], np.uint32)
        L = self.sizes.n_seg_compressed
        return dict(total=int(c[B.TAGC_CNT_TOTAL]), nonfinite=int(c[B.TAGC_CNT_NONFINITE]),
                    flags=int(c[B.TAGC_CNT_FLAGS]), dense_segments=int(c[B.TAGC_CNT_DENSE]),
                    seg=c[B.TAGC_CNT_SEG0:B.TAGC_CNT_SEG0 + L].tolist())

    def rank_pairs(self, r):
        n = self.rank_counts(r)["total"]
        return (self._np(self._rk_tensors[r]["idx"], np.uint32, n),
                self._np(self._rk_tensors[r]["val"], np.float32, n))

    def rank_acc(self, r):
        """The rank's accumulator as raw bit patterns (uint16 for bf16, uint32 for fp32)."""
        t = self._rk_tensors[r]["acc"]
        raw = t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
        return raw.cpu().numpy().view(np.uint16 if t.dtype == torch.bfloat16 else np.uint32).copy()

    def rank_bitmap(self, r):
        """The rank's Index as it goes on the wire (4 words per 32 parameters with 4-bit
        counters, 1 otherwise)."""
        wire = 4 if self.cfg.index_mode == B.TAGC_INDEX_ADD4 else 1
        return self._np(self._rk_tensors[r]["bitmap"], np.uint32,
                        wire * self.sizes.bitmap_words)

    def rank_sketch(self, r):
        """The rank's sketch as float32 values (16-bit wire cells widened)."""
        m = self.header()["m"]
        if self.cfg.cell_type == B.TAGC_CELL_BF16:
            half = self._np(self._rk_tensors[r]["sketch"], np.uint16, m)
            return (half.astype(np.uint32) << 16).view(np.float32)
        return self._np(self._rk_tensors[r]["sketch"], np.float32, m)

    def shared_bitmap(self):
        return self._np(self.sh_bitmap, np.uint32, self.sizes.bitmap_words)

    def shared_sketch(self):
        return self._np(self.sh_sketch, np.float32, self.header()["m"])

    def bounds(self):
        return self._np(self.sh_bounds, np.uint32, self.header()["A"] + 1)

    def salts(self):
        """The partitions' hash salts (behind the bounds in the same buffer)."""
        A, cap = self.header()["A"], self.sizes.partition_capacity
        return self._np(self.sh_bounds, np.uint32)[cap + 1:cap + 1 + A].copy()

    def outputs(self):
        U = self.header()["U"]
        return self._np(self.out_idx, np.uint32, U), self._np(self.out_val, np.float32, U)

    def dense(self):
        return self._np(self.out_dense, np.float32, self.sizes.n_c)
