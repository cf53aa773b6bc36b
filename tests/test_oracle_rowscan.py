"""The row-sampled C oracle must equal the dense NumPy oracle (CPU only).

The C code is a second, separately written evaluator (it scans keys row by row
and never forms a matrix); agreement with the dense definition to ~1e-12 on
every mask family pins both against slips that are specific to one of them.
It is also pinned directly: full mask vs scipy softmax attention, and a
single-neighbour row returning that V row exactly.
"""
import math

import numpy as np
import pytest
import scipy.special

from sga_inputs import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL,
                        KIND_BIGBIRD, KIND_NONLOCAL, KIND_DILATED_2D, numpy_qkv, small_variants)
from oracle import reference as R
from oracle import rowscan as C

SPECS = [
    MaskSpec(KIND_SLIDING, 333, window=9),
    MaskSpec(KIND_SLIDING, 20, window=40),
    MaskSpec(KIND_DILATED, 333, window=7, stride=2),
    MaskSpec(KIND_DILATED, 100, window=4, stride=3),
    MaskSpec(KIND_GLOBAL_LOCAL, 333, window=10, n_global=5),
    MaskSpec(KIND_BIGBIRD, 320, block=16, window_blocks=1, n_global_blocks=2,
             n_random_blocks=3, seed=77),
    MaskSpec(KIND_BIGBIRD, 240, block=8, window_blocks=2, n_global_blocks=1,
             n_random_blocks=2, seed=3),
    MaskSpec(KIND_NONLOCAL, 333, window=10, n_global=5),
    MaskSpec(KIND_DILATED_2D, 333, block=40, stride=3),
]


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: f"{s.name}-{s.L}")
def test_neighbours_equal_dense_predicate(spec):
    m = R.dense_mask(spec)
    for i in range(spec.L):
        assert (C.row_neighbors(spec, i) == np.nonzero(m[i])[0]).all()
    assert C.count_edges(spec) == int(m.sum())
    assert (C.degrees(spec, np.arange(spec.L)) == m.sum(axis=1)).all()


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: f"{s.name}-{s.L}")
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_rows_equal_dense_oracle(spec, dtype):
    d = 16
    Q, K, V = numpy_qkv(1, spec.L, d, dtype, 0.7, 100)
    rows = np.arange(spec.L)
    O_c, lse_c, edges = C.attend_rows(spec, Q[0], K[0], V[0], 0.25, rows)
    O_d, lse_d = R.attention_masked(Q, K, V, spec, 0.25)
    assert edges == int(R.dense_mask(spec).sum())
    assert np.abs(O_c - O_d[0]).max() < 1e-12
    empty = np.isneginf(lse_d[0])                 # rows without neighbours: lse = -inf on both sides
    assert (np.isneginf(lse_c) == empty).all()
    assert np.abs(lse_c[~empty] - lse_d[0][~empty]).max() < 1e-12


def test_small_workload_variants_agree():
    for wl in small_variants():
        Q, K, V = numpy_qkv(1, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed)
        rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(wl.L - 40, wl.L),
                                         np.arange(0, wl.L, 37)]))
        O_c, lse_c, _ = C.attend_rows(wl.mask, Q[0], K[0], V[0], wl.scale, rows)
        O_d, lse_d = R.attention_masked(Q, K, V, wl.mask, wl.scale, rows=rows)
        assert np.abs(O_c - O_d[0]).max() < 1e-12, wl.name
        assert np.abs(lse_c - lse_d[0]).max() < 1e-12, wl.name


def test_gathered_full_row_vs_scipy():
    n, d = 500, 64
    rng = np.random.default_rng(0)
    q = rng.standard_normal(d).astype(np.float32)
    Kg = rng.standard_normal((n, d)).astype(np.float32)
    Vg = rng.standard_normal((n, d)).astype(np.float32)
    O, lse = C.attend_gathered(q, Kg, Vg, 0.125)
    s = 0.125 * (Kg.astype(np.float64) @ q.astype(np.float64))
    want = scipy.special.softmax(s) @ Vg.astype(np.float64)
    assert np.abs(O - want).max() < 1e-13
    assert abs(lse - scipy.special.logsumexp(s)) < 1e-12


def test_gathered_single_and_empty():
    d = 8
    rng = np.random.default_rng(1)
    q = rng.standard_normal(d).astype(np.float32)
    Kg = rng.standard_normal((1, d)).astype(np.float32)
    Vg = rng.standard_normal((1, d)).astype(np.float32)
    O, lse = C.attend_gathered(q, Kg, Vg, 2.0)
    assert (O == Vg[0].astype(np.float64)).all()
    assert abs(lse - 2.0 * float(Kg[0].astype(np.float64) @ q.astype(np.float64))) < 1e-13
    O, lse = C.attend_gathered(q, np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 2.0)
    assert (O == 0).all() and lse == -math.inf
