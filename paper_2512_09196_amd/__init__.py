"""MI355X (gfx950) tile-kernel family  Y = GELU_erf(A.B + bias)  with a
profiling-guided variant loop, behind a C-ABI library.

``paper_2512_09196_amd.tf`` is the thin binding over the C-ABI; it raises if
the HIP library has not been built.  ``paper_2512_09196_amd.workloads`` holds
the seeded input generators only.
"""
__all__ = ["tf", "workloads"]
