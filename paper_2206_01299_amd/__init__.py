"""MI355X-native stage-boundary codec of AQ-SGD (activation-change quantisation).

``paper_2206_01299_amd.binding`` is the thin ctypes layer over the C-ABI
library built from ``csrc/``; ``paper_2206_01299_amd.workloads`` draws the
seeded synthetic inputs.  Importing the package loads nothing native.
"""
__all__ = ["binding", "workloads", "build"]
