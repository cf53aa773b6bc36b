"""Seeded synthetic workloads for sparse graph attention.

This package holds *data only*: the mask parameter records, the five benchmark
workload shapes and the seeded tensor generators.  It contains none of the
method's arithmetic (no mask predicate, no neighbour enumeration, no softmax),
so that the CPU oracle and the HIP path can both draw their inputs from it
without sharing any computation.
"""
from .masks import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL,
                    KIND_BIGBIRD, KIND_NONLOCAL, KIND_DILATED_2D, KIND_NAMES, RandomMaskSpec)
from .configs import (Workload, WORKLOADS, TABLE3_WORKLOADS, E2_RANDOM_WORKLOADS, BASE_SEED,
                      small_variants)
from .tensors import (numpy_qkv, torch_qkv, torch_random_csr, DTYPE_F32, DTYPE_F16)

__all__ = [
    "MaskSpec", "KIND_SLIDING", "KIND_DILATED", "KIND_GLOBAL_LOCAL",
    "KIND_BIGBIRD", "KIND_NONLOCAL", "KIND_DILATED_2D", "KIND_NAMES", "Workload", "WORKLOADS", "TABLE3_WORKLOADS", "E2_RANDOM_WORKLOADS", "RandomMaskSpec", "torch_random_csr",
    "BASE_SEED",
    "small_variants", "numpy_qkv", "torch_qkv", "DTYPE_F32", "DTYPE_F16",
]
