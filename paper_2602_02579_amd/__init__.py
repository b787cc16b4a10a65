"""ProphetKV selective-recomputation hot path for AMD MI355X (gfx950).

``api`` holds the Python binding of the C-ABI library (argument marshalling
only; every step runs in the HIP kernels of ``csrc/``), ``synth`` the seeded
synthetic input generator.  The binding raises if the compiled library is
missing: there is no CPU fallback.
"""

__all__ = ["api", "synth"]
