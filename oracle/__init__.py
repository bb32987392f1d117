"""fp64 CPU oracle for Ring Self-Attention.  Test infrastructure only.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package.  It shares nothing with the HIP library.
"""
from .rsa_oracle import (  # noqa: F401
    build,
    forward,
    backward,
    threads,
)
from . import proj_oracle as proj  # noqa: F401  (the linear maps of Table 2 around RSA)
from . import linformer_oracle as linformer  # noqa: F401  (Table 3: projected keys and values)
