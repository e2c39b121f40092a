"""Neuron-aware sparse FFN decode path for MI355X (gfx950).

`paper_2312_12456_amd.pf` is the thin ctypes binding of the C-ABI library libpf.so
(hand-written HIP kernels); `paper_2312_12456_amd.workload` draws the seeded synthetic
layers and inputs.  Nothing here computes on the CPU: without the built library the
binding raises.
"""
__all__ = ["pf", "workload"]
