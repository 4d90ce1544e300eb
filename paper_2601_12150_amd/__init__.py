"""Neighbourhood-sparse ViT attention and CLS-score token filtering on MI355X (gfx950).

`paper_2601_12150_amd.binding` wraps the C-ABI library `libnsattn.so` (hand-written HIP
kernels); `paper_2601_12150_amd.synth` generates the seeded synthetic inputs.  Importing
the package loads nothing; the binding raises if the HIP library has not been built.
"""
__all__ = ["binding", "synth"]
