"""sp24: 2:4 structured-sparse matrix multiply for AMD MI355X (gfx950).

``paper_2104_08378_amd.sp24`` is the binding over the C-ABI library
(``libsp24.so``, hand-written HIP); ``paper_2104_08378_amd.synth`` makes the
seeded synthetic workloads.  Importing the package loads nothing native.
"""
