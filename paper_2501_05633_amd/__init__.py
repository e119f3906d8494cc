"""RegTop-k per-round hot path for MI355X (gfx950).

``paper_2501_05633_amd.binding`` is the thin ctypes layer over the C-ABI
library built from ``csrc/``; ``paper_2501_05633_amd.workloads`` draws the
synthetic gradients.  Nothing is loaded at import time.
"""
__all__ = ["binding", "workloads", "build"]
