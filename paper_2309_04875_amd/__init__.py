"""Reduced-ring secret-shared DReLU / ReLU on MI355X (gfx950).

`hb` is the Python binding of the C-ABI library (include/hb.h); `workloads` makes seeded
synthetic inputs.  Importing the package does not load the GPU library; calling into `hb`
does, and fails loudly when it has not been built.
"""
from . import workloads  # noqa: F401
