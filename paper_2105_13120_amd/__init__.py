"""Ring Self-Attention (RSA) forward and backward for MI355X (gfx950).

The compute lives in a C-ABI HIP library (csrc/, declared in include/rsa.h);
`rsa` is its thin ctypes binding and `inputs` the seeded synthetic workloads.
"""
