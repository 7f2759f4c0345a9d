"""MI355X-native arithmetic reduction encoded as chains of matrix-multiply-accumulate
operations against an all-ones operand (the tensor-core reduction of Section IV-A).

``redux``      thin ctypes binding of the C-ABI library (HIP kernels for gfx950).
``workloads``  seeded synthetic input generators (host side, no reduction arithmetic).

Nothing is imported eagerly: ``import paper_1903_03640_amd.workloads`` must work on a
machine where the HIP library has not been built.
"""
__all__ = ["redux", "workloads"]
