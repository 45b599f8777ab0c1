"""Seeded synthetic gradient buckets shaped like the paper's workloads.

This module only *produces inputs*: bucket descriptions (segment tables) and
random gradient tensors with the shapes, dtypes and value distributions of the
five benchmark configurations.  It contains none of the method's arithmetic
and imports neither the oracle nor the HIP package; both sides are fed from
here so that they see identical data.

The paper trains GPT-2 small on OpenWebText (section 4.1); neither the data
set nor trained weights are used here.  Only layer shapes are borrowed, and
gradient values are drawn from the distributions stated per configuration.

All tensors are torch tensors on the requested device; ``to_numpy_raw`` gives
the oracle's view (float32 array, or uint16 array of bf16 bit patterns).
"""
from __future__ import annotations

import math
from collections import namedtuple
from dataclasses import dataclass, field

import numpy as np
import torch

Seg = namedtuple("Seg", "offset length keep_ppm flags name")

F32, BF16 = 0, 1
COMPRESS = 1


@dataclass
class Bucket:
    name: str
    dtype: int                   # F32 | BF16
    n_ranks: int
    segments: list               # of Seg
    n_elems: int                 # length of each rank's buffer
    sizing_milli: int = 3000     # load factor x 1000
    sigma: dict = field(default_factory=dict)   # per segment name
    kind: str = "normal"         # "normal" | "student_t3"
    seed: int = 0
    bucket_id: int = 0

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == F32 else torch.bfloat16

    @property
    def elem_bytes(self):
        return 4 if self.dtype == F32 else 2

    def compressed_elems(self):
        return sum(s.length for s in self.segments if s.flags & COMPRESS)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def rank_gradient(b: Bucket, rank: int, device="cpu") -> torch.Tensor:
    """Rank `rank`'s flat gradient buffer for bucket `b` (seed = base + rank)."""
    dev = torch.device(device)
    g = _gen(dev, b.seed + rank + 1000003 * b.bucket_id)
    out = torch.zeros(b.n_elems, dtype=b.torch_dtype, device=dev)   # (gaps between segments: 0)
    for s in b.segments:
        sig = b.sigma.get(s.name, 1e-3)
        chunk = 1 << 24
        for lo in range(0, s.length, chunk):
            n = min(chunk, s.length - lo)
            z = torch.randn(n, generator=g, device=dev, dtype=torch.float32)
            if b.kind == "student_t3":
                # t_3 = z / sqrt(chi2_3 / 3)
                c = torch.randn(3, n, generator=g, device=dev,
                                dtype=torch.float32)
                z = z / torch.sqrt((c * c).sum(0) / 3.0)
            out[s.offset + lo:s.offset + lo + n] = (z * sig).to(b.torch_dtype)
    return out


def to_numpy_raw(t: torch.Tensor) -> np.ndarray:
    """float32 array, or uint16 bit patterns for bf16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def _log_uniform(rng, lo, hi):
    return float(math.exp(rng.uniform(math.log(lo), math.log(hi))))


# ---------------------------------------------------------------- config 1


def config1(seed=0, n=1 << 20, n_ranks=4, keep_ppm=10_000):
    """Single bucket, one fp32 layer of n elements ~ N(0, sigma=1e-3), top 1 %
    kept per rank, load factor 3."""
    segs = [Seg(0, n, keep_ppm, COMPRESS, "w")]
    return Bucket("config1", F32, n_ranks, segs, n, 3000, {"w": 1e-3},
                  "normal", seed, 0)


# ---------------------------------------------------------------- config 2


def _gpt2_block_segments(rng, d=768, ffn=3072, keep_lo=5_000, keep_hi=50_000):
    """One GPT-2 block in parameter order.  Weights of the four linear layers
    are compressed; LayerNorm weights/biases and linear biases are present in
    the buffer but flagged off (layer-selective compression)."""
    layout = [
        ("ln1.w", d, False), ("ln1.b", d, False),
        ("attn.qkv.w", d * 3 * d, True), ("attn.qkv.b", 3 * d, False),
        ("attn.proj.w", d * d, True), ("attn.proj.b", d, False),
        ("ln2.w", d, False), ("ln2.b", d, False),
        ("mlp.fc.w", d * ffn, True), ("mlp.fc.b", ffn, False),
        ("mlp.fc2.w", ffn * d, True), ("mlp.fc2.b", d, False),
    ]
    segs, sigma, off = [], {}, 0
    for name, n, comp in layout:
        ppm = int(round(_log_uniform(rng, keep_lo, keep_hi))) if comp else 0
        segs.append(Seg(off, n, ppm, COMPRESS if comp else 0, name))
        sigma[name] = 1e-3 * _log_uniform(rng, 0.1, 10.0)
        off += n
    return segs, sigma, off


def config2(seed=0, n_ranks=8, blocks=12, sizing_milli=3000):
    """GPT-2-small-shaped fp32 gradients: one bucket per transformer block."""
    out = []
    for blk in range(blocks):
        rng = np.random.default_rng([seed, 2, blk])
        segs, sigma, n = _gpt2_block_segments(rng)
        out.append(Bucket("config2.block%d" % blk, F32, n_ranks, segs, n,
                          sizing_milli, sigma, "normal", seed, blk))
    return out


def config2_embeddings(seed=0, n_ranks=8):
    """The 13th bucket: token and position embeddings, present but excluded."""
    segs = [Seg(0, 50257 * 768, 0, 0, "wte"),
            Seg(50257 * 768, 1024 * 768, 0, 0, "wpe")]
    return Bucket("config2.embed", F32, n_ranks, segs, (50257 + 1024) * 768,
                  3000, {}, "normal", seed, 12)


# ---------------------------------------------------------------- config 3


def config3(seed=0, n=1 << 26, n_ranks=8, keep_ppm=10_000, sizing_milli=1500):
    """Heavy-tailed bf16 bucket (Student-t, nu=3, x 1e-3)."""
    segs = [Seg(0, n, keep_ppm, COMPRESS, "w")]
    return Bucket("config3", BF16, n_ranks, segs, n, sizing_milli, {"w": 1e-3},
                  "student_t3", seed, 0)


def config3_rank_gradient(b: Bucket, rank: int, device="cpu") -> torch.Tensor:
    """Config-3 gradients with 50 % support overlap between ranks: a shared
    position set H of size ceil(k/2) (seed = base) is pushed into every rank's
    top-k by overwriting those positions with +-tau_r*(1+|t|), tau_r being the
    rank's floor(k/2)-th largest private magnitude; the other half of each
    support stays private."""
    dev = torch.device(device)
    g = rank_gradient(b, rank, device)
    s = b.segments[0]
    k = (s.length * s.keep_ppm) // 1_000_000
    if k < 2:
        return g
    gh = _gen(dev, b.seed + 7777)
    H = torch.randperm(s.length, generator=gh, device=dev)[: (k + 1) // 2]
    mag = g.float().abs()
    tau = torch.topk(mag, k // 2).values[-1]
    gr = _gen(dev, b.seed + rank + 4242)
    t = torch.randn(H.numel(), generator=gr, device=dev)
    sign = torch.where(torch.rand(H.numel(), generator=gr, device=dev) < 0.5,
                       -1.0, 1.0)
    g[H] = (sign * tau * (1.0 + t.abs())).to(g.dtype)
    return g


# ------------------------------------------------------------ configs 4, 5


def _llama_block_segments(rng, d, ffn, shard, sigma_lo, sigma_hi, keep_fn):
    layout = [("attn.q", d * d), ("attn.k", d * d), ("attn.v", d * d),
              ("attn.o", d * d), ("mlp.gate", d * ffn), ("mlp.up", d * ffn),
              ("mlp.down", ffn * d)]
    segs, sigma, off = [], {}, 0
    for name, n in layout:
        n //= shard
        segs.append(Seg(off, n, 0, COMPRESS, name))
        sigma[name] = _log_uniform(rng, sigma_lo, sigma_hi)
        off += n
    ppm = keep_fn(rng, segs)
    segs = [s._replace(keep_ppm=p) for s, p in zip(segs, ppm)]
    return segs, sigma, off


def config4(seed=0, n_ranks=8, blocks=32, sizing_milli=1500, d=4096,
            ffn=11008):
    """One rank's 1/8 FSDP shard of a Llama-7B-shaped model: bf16, per-layer
    sigma = 1e-3 * log-uniform[0.1, 10], keep 1 %.  RMSNorm weights and
    embeddings are excluded and not allocated."""
    out = []
    for blk in range(blocks):
        rng = np.random.default_rng([seed, 4, blk])
        segs, sigma, n = _llama_block_segments(
            rng, d, ffn, 8, 1e-4, 1e-2, lambda r, s: [10_000] * len(s))
        out.append(Bucket("config4.block%d" % blk, BF16, n_ranks, segs, n,
                          sizing_milli, sigma, "normal", seed, blk))
    return out


def _dynamic_keep(rng, segs, mean_ppm=10_000):
    """keep_ppm_l = mean * 2^u, u ~ U(-1, 1), rescaled so that the
    element-weighted mean is `mean_ppm`."""
    raw = np.array([mean_ppm * 2.0 ** rng.uniform(-1, 1) for _ in segs])
    w = np.array([s.length for s in segs], float)
    raw *= mean_ppm / float((raw * w).sum() / w.sum())
    return [max(1, int(round(x))) for x in raw]


def config5(seed=0, n_ranks=16, blocks=32, sizing_milli=1500, d=4096,
            ffn=11008):
    """Full Llama-7B-shaped gradient, one bucket per block: bf16, per-layer
    sigma log-uniform in [1e-5, 1e-2], dynamic keep ratio with mean 1 %."""
    out = []
    for blk in range(blocks):
        rng = np.random.default_rng([seed, 5, blk])
        segs, sigma, n = _llama_block_segments(rng, d, ffn, 1, 1e-5, 1e-2,
                                               _dynamic_keep)
        out.append(Bucket("config5.block%d" % blk, BF16, n_ranks, segs, n,
                          sizing_milli, sigma, "normal", seed, blk))
    return out


# ------------------------------------------------------------ test helpers


def small_mixed_bucket(seed=0, dtype=F32, n_ranks=3, sizing_milli=3000):
    """A small ragged bucket for tests: several compressed segments with odd
    lengths and offsets, skipped segments in between, one tiny segment whose
    keep count is zero, one segment with many exact zeros."""
    rng = np.random.default_rng([seed, 99])
    lens = [5000, 37, 12345, 64, 8192 + 5, 100, 3001, 7]
    comp = [True, False, True, False, True, True, True, True]
    ppm = [20_000, 0, 50_000, 0, 10_000, 5_000, 100_000, 400_000]
    align = 8 if dtype == BF16 else 4
    segs, off = [], 0
    for i, (n, c, p) in enumerate(zip(lens, comp, ppm)):
        segs.append(Seg(off, n, p, COMPRESS if c else 0, "s%d" % i))
        off += n
        if i % 2 == 0:  # keep some offsets aligned, some not
            off = (off + align - 1) // align * align
    sigma = {s.name: 1e-3 * _log_uniform(rng, 0.1, 10.0) for s in segs}
    return Bucket("small_mixed", dtype, n_ranks, segs, off, sizing_milli,
                  sigma, "normal", seed, 0)
