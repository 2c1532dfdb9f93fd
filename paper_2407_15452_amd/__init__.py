"""Random-walk sampling + SGNS embedding updates on AMD gfx950 (one GPU).

``inputs`` makes seeded synthetic workloads; ``binding`` is the thin ctypes
layer over ``libgs.so`` (hand-written HIP kernels behind a C boundary declared
in ``include/gs.h``).  Importing the package loads nothing; the shared library
is opened on the first call and a missing library is an error, never a
fallback.
"""
