"""Pruned fully-connected inference in permutation-block-permutation form,
hand-written for AMD MI355X (gfx950).

``paper_1712_01084_amd.binding`` is the thin ctypes layer over the C-ABI
library built from ``csrc/``; ``paper_1712_01084_amd.workloads`` draws the
seeded synthetic inputs.  Nothing here falls back to a CPU implementation:
without the built library the binding raises.
"""

__all__ = ["binding", "workloads"]
