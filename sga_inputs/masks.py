"""Mask parameter record (the attention-specific parameters P_a of Algorithm 1).

Only the numbers that name a mask live here.  What the numbers *mean* (which
(i, j) pairs are edges) is implemented twice, independently: once in
``oracle/`` and once in the HIP library.
"""
from dataclasses import dataclass

KIND_SLIDING = 0        # local window, Section II-C "Local/Windowed Attention"
KIND_DILATED = 1        # 1-D dilated window, Section II-C
KIND_GLOBAL_LOCAL = 2   # local window plus leading global tokens
KIND_BIGBIRD = 3        # block mask: window + global + random key blocks
KIND_NONLOCAL = 4       # global tokens minus the local window (Section IV-B "Global (non-local)")
KIND_DILATED_2D = 5     # 2-D dilated blocks on the diagonal, Section II-C

KIND_NAMES = {
    KIND_SLIDING: "sliding",
    KIND_DILATED: "dilated",
    KIND_GLOBAL_LOCAL: "global_local",
    KIND_BIGBIRD: "bigbird",
    KIND_NONLOCAL: "nonlocal",
    KIND_DILATED_2D: "dilated_2d",
}


@dataclass(frozen=True)
class MaskSpec:
    """Plain record of mask parameters.

    kind             one of the KIND_* codes
    L                context length (rows = queries, columns = keys)
    window           half-width in steps: sliding/global_local/nonlocal use |i-j| <= window,
                     dilated uses |i-j| <= window*stride
    stride           distance between attended keys (1 = contiguous, 2 = every other);
                     dilated_2d keeps every stride-th row and column of a block
    n_global         global tokens occupy positions 0..n_global-1 (global_local, nonlocal)
    block            block edge in tokens (bigbird, dilated_2d)
    window_blocks    neighbouring key blocks on each side (bigbird)
    n_global_blocks  global blocks occupy block indices 0..n_global_blocks-1 (bigbird)
    n_random_blocks  random key blocks per non-global query block (bigbird)
    seed             seed of the counter-based block selection (bigbird)
    """
    kind: int
    L: int
    window: int = 0
    stride: int = 1
    n_global: int = 0
    block: int = 0
    window_blocks: int = 0
    n_global_blocks: int = 0
    n_random_blocks: int = 0
    seed: int = 0

    @property
    def name(self) -> str:
        return KIND_NAMES[self.kind]


@dataclass(frozen=True)
class RandomMaskSpec:
    """A uniformly random mask (the "uniform random" pattern of Section II-C and the random CSR
    runs of the microbenchmark, Section V-C): every (i, j) pair is an edge with probability
    `density`, drawn on the device from `seed` (sga_inputs.tensors.torch_random_csr).  It has no
    closed form: both sides consume the drawn CSR arrays."""
    L: int
    density: float
    seed: int = 0

    @property
    def name(self) -> str:
        return "random"
