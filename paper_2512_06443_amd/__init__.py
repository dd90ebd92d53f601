"""Vector-LUT ternary x INT8 mpGeMM for MI355X: Python side of the C-ABI library libvlut.so.

`binding` needs torch with a ROCm device; `workloads` (seeded synthetic inputs) needs numpy only.
"""
__all__ = ["binding", "workloads", "build"]
