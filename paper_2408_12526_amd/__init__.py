"""Student Parallelism K-student forward for MI355X (gfx950).

``paper_2408_12526_amd.sp`` is the thin binding over the C-ABI library (HIP
kernels); ``paper_2408_12526_amd.synth`` draws the seeded synthetic workloads.
Nothing is imported eagerly so that the input generator can be used on machines
without the built library.
"""
__all__ = ["sp", "synth"]
