"""MI355X-native Data Coordinator reshard path (DistFlow, Sec. 6).

``workloads`` draws seeded synthetic rollout batches; ``binding`` is the thin
ctypes layer over the C-ABI library ``libdc.so`` (HIP kernels for gfx950).
Nothing here computes on the CPU: without the built library the binding raises.
"""
__all__ = ["workloads", "binding"]
