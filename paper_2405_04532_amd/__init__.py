"""MI355X-native W4A8 GEMM with progressive group quantization (QoQ, arXiv 2405.04532).

The product is the C-ABI library built from csrc/ (hand-written HIP for gfx950); `api`
is its thin ctypes binding and `workloads` the seeded synthetic inputs.  Nothing here
falls back to a CPU implementation: without the built library the binding raises.
"""
__all__ = ["api", "workloads"]
