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

KIND_NAMES = {
    KIND_SLIDING: "sliding",
    KIND_DILATED: "dilated",
    KIND_GLOBAL_LOCAL: "global_local",
    KIND_BIGBIRD: "bigbird",
}


@dataclass(frozen=True)
class MaskSpec:
    """Plain record of mask parameters.

    kind             one of the KIND_* codes
    L                context length (rows = queries, columns = keys)
    window           half-width in steps: sliding/global_local use |i-j| <= window,
                     dilated uses |i-j| <= window*stride
    stride           distance between attended keys (1 = contiguous, 2 = every other)
    n_global         global tokens occupy positions 0..n_global-1 (global_local)
    block            block edge in tokens (bigbird)
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
