"""FlashOmni's unified sparse attention kernel, written for AMD MI355X (gfx950).

The product is the C-ABI library built from ``csrc/`` (declared in ``include/sparse_attn.h``);
this package is the thin Python binding over it plus the seeded synthetic workloads.
"""
from . import synth  # noqa: F401
