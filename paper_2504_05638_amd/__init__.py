"""libtagc for MI355X: the per-GPU hot path of TAGC (arXiv 2504.05638).

`binding` mirrors include/tagc.h one to one; `bucket.TagcBucket` is the
device-memory plumbing around it; `build.build()` compiles the library.
Nothing here computes any step of the method on the CPU.
"""
from . import binding  # noqa: F401

__all__ = ["binding", "bucket", "build"]
