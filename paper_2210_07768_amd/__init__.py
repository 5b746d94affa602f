"""FeatureBox-style batched feature extraction for AMD MI355X (gfx950).

The product is the C-ABI library ``libfbx.so`` (hand-written HIP kernels plus a
small C++ host side) and the thin ctypes binding in :mod:`.binding`.  The
``workloads`` sub-package only generates seeded synthetic inputs.
"""

__all__ = ["binding", "workloads", "build"]
