"""The five benchmark workloads and reduced-size variants of each for parity tests."""
from dataclasses import dataclass, replace
from typing import Dict, List

from .masks import (MaskSpec, RandomMaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL,
                    KIND_BIGBIRD)

BASE_SEED = 20250201


@dataclass(frozen=True)
class Workload:
    """One benchmark shape: tensors [H][L][d], a mask, and how it is fed.

    dtype     "f32" or "f16" (storage type; arithmetic accumulates in fp32)
    sigma     Q/K/V are sigma * N(0,1) drawn from `seed`+{0,1,2}, cast to storage
    explicit  True: CSR built by the mask builder and passed to the forward;
              False: neighbours generated inside the kernel, no stored CSR
    """
    name: str
    H: int
    L: int
    d: int
    dtype: str
    sigma: float
    mask: MaskSpec
    explicit: bool
    seed: int = BASE_SEED

    @property
    def scale(self) -> float:
        return 1.0 / float(self.d) ** 0.5


WORKLOADS: Dict[str, Workload] = {
    # Sliding window, |i-j| <= 32, explicit CSR.
    "cfg1_sliding_4k": Workload(
        "cfg1_sliding_4k", H=1, L=4096, d=64, dtype="f32", sigma=1.0,
        mask=MaskSpec(KIND_SLIDING, 4096, window=32), explicit=True),
    # Longformer-style: window 128 plus 16 leading global tokens, explicit CSR.
    "cfg2_longformer_64k": Workload(
        "cfg2_longformer_64k", H=8, L=65536, d=64, dtype="f32", sigma=1.0,
        mask=MaskSpec(KIND_GLOBAL_LOCAL, 65536, window=128, n_global=16),
        explicit=True),
    # Dilated window: j = i + 2k, |k| <= 64, implicit neighbours.
    "cfg3_dilated_1m": Workload(
        "cfg3_dilated_1m", H=4, L=1 << 20, d=64, dtype="f16", sigma=0.5,
        mask=MaskSpec(KIND_DILATED, 1 << 20, window=64, stride=2),
        explicit=False),
    # BigBird-style block mask, explicit CSR.
    "cfg4_bigbird_1m": Workload(
        "cfg4_bigbird_1m", H=4, L=1 << 20, d=64, dtype="f16", sigma=0.5,
        mask=MaskSpec(KIND_BIGBIRD, 1 << 20, block=64, window_blocks=1,
                      n_global_blocks=2, n_random_blocks=3, seed=BASE_SEED + 3),
        explicit=True),
    # 160M-token sliding window, |i-j| <= 16, implicit neighbours.
    "cfg5_sliding_160m": Workload(
        "cfg5_sliding_160m", H=1, L=160_000_000, d=64, dtype="f16", sigma=0.5,
        mask=MaskSpec(KIND_SLIDING, 160_000_000, window=16), explicit=False),
}


def _table3(name, L, s_f):
    """Local attention of the long-context runs (Table III, Section V-E): fp16, one head, the
    window sized so that the mask's sparsity factor is s_f (2w + 1 = round(s_f * L) keys per row)."""
    w = max(0, (int(round(s_f * L)) - 1) // 2)
    return Workload(name, H=1, L=L, d=64, dtype="f16", sigma=0.5,
                    mask=MaskSpec(KIND_SLIDING, L, window=w), explicit=False)


# The four sequence lengths of Table III with the sparsity factors printed there.
TABLE3_WORKLOADS: Dict[str, Workload] = {
    "table3_1p6m": _table3("table3_1p6m", 1_600_000, 0.0017),
    "table3_8m": _table3("table3_8m", 8_000_000, 0.00034),
    "table3_16m": _table3("table3_16m", 16_000_000, 0.00017),
    "table3_160m": _table3("table3_160m", 160_000_000, 0.00001),
}


def _e2_random(L, density, dtype="f32", d=64):
    tag = f"e2_random_{L // 1024}k_sf{int(round(density * 1000)):04d}_{dtype}"
    return tag, Workload(tag, H=1, L=L, d=d, dtype=dtype, sigma=1.0 if dtype == "f32" else 0.5,
                         mask=RandomMaskSpec(L, density, BASE_SEED + 7), explicit=True)


# Random CSR masks of the microbenchmark grid (Section V-C): one head, d = 64, the longest of its
# three sequence lengths, sparsity factors 0.01 and 0.1, both storage types.  These run on the
# per-row (general CSR) kernels: scattered columns fill no 32 x 32 tile.
E2_RANDOM_WORKLOADS: Dict[str, Workload] = dict(
    _e2_random(24576, sf, dt) for sf in (0.01, 0.1) for dt in ("f32", "f16"))


def small_variants() -> List[Workload]:
    """Reduced-L versions of the five workloads that a dense CPU oracle finishes
    in seconds while still spanning several 32/64-row tiles and a ragged tail."""
    out = []
    w1 = WORKLOADS["cfg1_sliding_4k"]
    out.append(replace(w1, name="cfg1_small", L=1000 + 37,
                       mask=replace(w1.mask, L=1037)))
    w2 = WORKLOADS["cfg2_longformer_64k"]
    out.append(replace(w2, name="cfg2_small", H=2, L=1500 + 11,
                       mask=replace(w2.mask, L=1511)))
    w3 = WORKLOADS["cfg3_dilated_1m"]
    out.append(replace(w3, name="cfg3_small", H=2, L=1203,
                       mask=replace(w3.mask, L=1203)))
    w4 = WORKLOADS["cfg4_bigbird_1m"]
    out.append(replace(w4, name="cfg4_small", H=2, L=64 * 23,
                       mask=replace(w4.mask, L=64 * 23)))
    w5 = WORKLOADS["cfg5_sliding_160m"]
    out.append(replace(w5, name="cfg5_small", L=2049,
                       mask=replace(w5.mask, L=2049)))
    return out
