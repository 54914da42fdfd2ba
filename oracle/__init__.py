"""CPU oracle for N:M transposable masks -- TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.  It is a
ctypes front-end to ``tmask_oracle.c`` (plain C, fp64 where floating point is involved) and never
touches the HIP library.
"""
from .oracle import (approx, exact, score, apply_pack, unpack, spmm, prune_1d, apply_dense, flip_count, pattern_violations, mask_diversity_log10, nm_sparse_probability, bf16_to_f64, network_sizes,  # noqa: F401
                     build, lib_path, F32, BF16)
