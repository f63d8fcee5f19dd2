"""libwkv: the WeightedKV (arXiv 2503.01330) per-token decode step, native on MI355X.

`paper_2503_01330_amd.binding` is a thin ctypes face of the C ABI declared in
include/wkv.h; `paper_2503_01330_amd.synth` draws the seeded synthetic streams.
Nothing is imported eagerly so that the stream generator can be used on a
machine where the HIP library has not been built.
"""
__all__ = ["binding", "synth"]
