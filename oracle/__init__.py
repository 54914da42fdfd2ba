"""CPU oracle for N:M transposable masks -- TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.  It is a
ctypes front-end to ``tmask_oracle.c`` (plain C, fp64 where floating point is involved) and never
touches the HIP library.
"""
from .oracle import (approx, exact, score, apply_pack, unpack, network_sizes, build, lib_path,  # noqa: F401
                     F32, BF16)
