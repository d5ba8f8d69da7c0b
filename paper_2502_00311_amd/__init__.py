"""MI355X-native hot path of Sparse Gradient Compression (SGC).

`paper_2502_00311_amd.sgc` is the thin binding over the C-ABI HIP library
(`csrc/`), `paper_2502_00311_amd.synth` the seeded input generators. Nothing is
imported eagerly so that the generators can be used without the GPU library.
"""
__all__ = ["sgc", "synth"]
