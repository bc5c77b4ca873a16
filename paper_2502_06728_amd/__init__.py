"""MI355X-native optimizer hot path of FlexDeMo / DeMo-SGD (arXiv 2502.06728, Algorithm 1).

``binding`` is the thin ctypes layer over the C-ABI library built from ``csrc/``;
``synth`` makes the seeded synthetic shards.  Nothing here computes on the CPU: every
step of the path runs in the HIP kernels, and the binding raises if the library has
not been built.
"""
__all__ = ["binding", "synth", "build"]
