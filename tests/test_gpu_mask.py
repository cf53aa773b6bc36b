"""Mask builder parity: the CSR written by sga_build_mask is bit-identical to the CSR the
oracle enumerates from the dense predicate."""
import numpy as np
import pytest

import paper_2502_01659_amd as sga
from sga_inputs import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL, KIND_BIGBIRD,
                        KIND_NONLOCAL, KIND_DILATED_2D,
                        WORKLOADS, small_variants)
from oracle import reference as R
from oracle import rowscan as C

pytestmark = pytest.mark.gpu

SPECS = [
    MaskSpec(KIND_SLIDING, 1, window=0),
    MaskSpec(KIND_SLIDING, 1, window=5),
    MaskSpec(KIND_SLIDING, 2, window=1),
    MaskSpec(KIND_SLIDING, 777, window=0),
    MaskSpec(KIND_SLIDING, 777, window=32),
    MaskSpec(KIND_SLIDING, 50, window=100),
    MaskSpec(KIND_SLIDING, 1025, window=300),
    MaskSpec(KIND_DILATED, 999, window=64, stride=2),
    MaskSpec(KIND_DILATED, 100, window=64, stride=2),
    MaskSpec(KIND_DILATED, 500, window=7, stride=5),
    MaskSpec(KIND_DILATED, 500, window=9, stride=1),
    MaskSpec(KIND_GLOBAL_LOCAL, 900, window=128, n_global=16),
    MaskSpec(KIND_GLOBAL_LOCAL, 300, window=4, n_global=0),
    MaskSpec(KIND_GLOBAL_LOCAL, 300, window=4, n_global=40),
    MaskSpec(KIND_GLOBAL_LOCAL, 40, window=3, n_global=40),
    MaskSpec(KIND_GLOBAL_LOCAL, 40, window=3, n_global=99),
    MaskSpec(KIND_GLOBAL_LOCAL, 40, window=60, n_global=2),
    MaskSpec(KIND_BIGBIRD, 64 * 23, block=64, window_blocks=1, n_global_blocks=2,
             n_random_blocks=3, seed=20250204),
    MaskSpec(KIND_BIGBIRD, 8 * 40, block=8, window_blocks=2, n_global_blocks=1,
             n_random_blocks=5, seed=1),
    MaskSpec(KIND_BIGBIRD, 3 * 50, block=3, window_blocks=0, n_global_blocks=0,
             n_random_blocks=16, seed=2),
    MaskSpec(KIND_BIGBIRD, 16 * 9, block=16, window_blocks=1, n_global_blocks=3,
             n_random_blocks=3, seed=3),
    MaskSpec(KIND_BIGBIRD, 5 * 12, block=5, window_blocks=3, n_global_blocks=2,
             n_random_blocks=0, seed=4),
    MaskSpec(KIND_NONLOCAL, 900, window=128, n_global=16),
    MaskSpec(KIND_NONLOCAL, 300, window=4, n_global=0),
    MaskSpec(KIND_NONLOCAL, 300, window=4, n_global=40),
    MaskSpec(KIND_NONLOCAL, 40, window=3, n_global=99),
    MaskSpec(KIND_NONLOCAL, 40, window=60, n_global=2),
    MaskSpec(KIND_NONLOCAL, 777, window=0, n_global=3),
    MaskSpec(KIND_DILATED_2D, 64, block=16, stride=2),
    MaskSpec(KIND_DILATED_2D, 1000, block=64, stride=3),
    MaskSpec(KIND_DILATED_2D, 333, block=40, stride=1),
    MaskSpec(KIND_DILATED_2D, 50, block=64, stride=4),
    MaskSpec(KIND_DILATED_2D, 129, block=1, stride=1),
    MaskSpec(KIND_DILATED_2D, 500, block=7, stride=9),
]


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: f"{s.name}-L{s.L}-w{s.window}{s.window_blocks}")
def test_csr_bit_exact_small(spec):
    print("case", spec, flush=True)
    rp, ci = sga.build_mask(spec)
    rp_o, ci_o = R.csr_from_dense(R.dense_mask(spec))
    assert sga.mask_nnz(spec) == int(rp_o[-1])
    assert np.array_equal(rp.cpu().numpy(), rp_o)
    assert np.array_equal(ci.cpu().numpy(), ci_o)


def test_csr_bit_exact_small_workload_variants():
    for wl in small_variants():
        print("case", wl.name, flush=True)
        rp, ci = sga.build_mask(wl.mask)
        rp_o, ci_o = R.csr_from_dense(R.dense_mask(wl.mask))
        assert np.array_equal(rp.cpu().numpy(), rp_o), wl.name
        assert np.array_equal(ci.cpu().numpy(), ci_o), wl.name


def test_csr_cfg1_full_size_bit_exact():
    spec = WORKLOADS["cfg1_sliding_4k"].mask
    rp, ci = sga.build_mask(spec)
    rp_o, ci_o = R.csr_from_dense(R.dense_mask(spec))
    assert np.array_equal(rp.cpu().numpy(), rp_o)
    assert np.array_equal(ci.cpu().numpy(), ci_o)


def _check_large(spec, rows):
    """Full-size masks: every row offset against the oracle's degrees by scanning all keys
    (all rows where affordable, else the sampled rows), sampled rows' column lists bit-exact,
    and full-array structure (sorted, in range) checked on the device."""
    import torch
    rp, ci = sga.build_mask(spec)
    nnz = sga.mask_nnz(spec)
    assert int(rp[-1]) == nnz and int(rp[0]) == 0
    rp_h = rp.cpu().numpy()
    deg = C.degrees(spec, rows)
    assert np.array_equal(rp_h[rows + 1] - rp_h[rows], deg)
    for i in rows[:: max(1, len(rows) // 200)]:
        want = C.row_neighbors(spec, int(i)).astype(np.int32)
        got = ci[rp_h[i]:rp_h[i + 1]].cpu().numpy()
        assert np.array_equal(got, want), int(i)
    # structure of the whole array: strictly increasing inside rows, in [0, L)
    assert int(ci.min()) >= 0 and int(ci.max()) < spec.L
    dif = ci[1:] - ci[:-1]
    row_starts = rp[1:-1]
    row_starts = row_starts[row_starts < nnz]
    ok = dif > 0
    ok[row_starts - 1] = True
    assert bool(ok.all())
    return rp, ci


def test_csr_cfg2_full_size():
    spec = WORKLOADS["cfg2_longformer_64k"].mask
    _check_large(spec, np.arange(spec.L, dtype=np.int64))      # every row's degree: 65536^2 scan


def test_csr_cfg4_full_size_sampled():
    spec = WORKLOADS["cfg4_bigbird_1m"].mask
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([np.arange(0, 260), np.arange(spec.L - 130, spec.L),
                                     rng.integers(0, spec.L, size=1500)])).astype(np.int64)
    _check_large(spec, rows)


def test_build_mask_capacity_error():
    import torch
    spec = MaskSpec(KIND_SLIDING, 100, window=3)
    rp = torch.empty(101, dtype=torch.int64, device="cuda")
    ci = torch.empty(10, dtype=torch.int32, device="cuda")
    st = sga.sga_build_mask(spec, rp.data_ptr(), ci.data_ptr(), 10, None)
    assert st == -3


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: f"{s.name}-L{s.L}-w{s.window}{s.window_blocks}")
def test_validate_csr_accepts_every_built_mask(spec):
    rp, ci = sga.build_mask(spec)
    assert sga.validate_csr(rp, ci) == -1


def test_validate_csr_names_the_first_bad_row():
    """Each way of breaking the contract of an explicit mask (Section IV-B "CSR": row offsets,
    sorted column indices), planted into a copy of a valid mask with empty rows in it; the
    oracle's CSR of the same dense mask is the valid starting point."""
    import torch
    L = 700
    dense = np.random.default_rng(3).random((L, L)) < 0.05
    dense[100:110] = False                      # empty rows: their offsets repeat
    dense[300] = True
    rp_h, ci_h = R.csr_from_dense(dense)
    rp = torch.from_numpy(rp_h).cuda()
    ci = torch.from_numpy(ci_h).cuda()
    assert sga.validate_csr(rp, ci) == -1

    def planted(edit_rp=None, edit_ci=None):
        r, c = rp.clone(), ci.clone()
        if edit_rp:
            edit_rp(r)
        if edit_ci:
            edit_ci(c)
        return sga.validate_csr(r, c)

    e300 = int(rp_h[300])
    assert planted(edit_ci=lambda c: c.__setitem__(e300 + 5, int(ci_h[e300 + 4]))) == 300          # duplicate
    assert planted(edit_ci=lambda c: c.__setitem__(e300 + 5, int(ci_h[e300 + 3]))) == 300          # descending
    assert planted(edit_ci=lambda c: c.__setitem__(int(rp_h[650]), L)) == 650                      # column = L
    assert planted(edit_ci=lambda c: c.__setitem__(int(rp_h[12]), -1)) == 12                       # negative column
    assert planted(edit_ci=lambda c: c.__setitem__(len(ci_h) - 1, 2 ** 31 - 1)) == L - 1           # last edge
    # two violations: the smaller row is named
    def two(c):
        c[int(rp_h[500])] = L + 7
        c[int(rp_h[40])] = -5
    assert planted(edit_ci=two) == 40
    # the first column of a row may lie left of the last column of the row before it, also
    # across empty rows (rows 99 | 100..109 empty | 110), which is no violation: covered by the
    # valid mask above; a row offset that steps back is one
    assert planted(edit_rp=lambda r: r.__setitem__(200, int(rp_h[199]) - 1)) == 199
    assert planted(edit_rp=lambda r: r.__setitem__(0, 1)) == L                                     # row_ptr[0] != 0
    assert planted(edit_rp=lambda r: r.__setitem__(L, len(ci_h) + 1)) == L                         # beyond the columns
    assert planted(edit_rp=lambda r: r.__setitem__(5, -3)) == 4                                    # (row 4 ends before it starts)
    # raw C ABI: status and argument errors
    scratch = torch.empty(2, dtype=torch.int64, device="cuda")
    st, bad = sga.sga_validate_csr(rp.data_ptr(), ci.data_ptr(), L, ci.numel(), scratch.data_ptr(), None)
    assert (st, bad) == (0, -1)
    bad_ci = ci.clone()
    bad_ci[e300 + 5] = int(ci_h[e300 + 4])
    st, bad = sga.sga_validate_csr(rp.data_ptr(), bad_ci.data_ptr(), L, ci.numel(), scratch.data_ptr(), None)
    assert (st, bad) == (-1, 300)
    assert sga.sga_validate_csr(0, ci.data_ptr(), L, ci.numel(), scratch.data_ptr(), None)[0] == -1
    assert sga.sga_validate_csr(rp.data_ptr(), ci.data_ptr(), 0, ci.numel(), scratch.data_ptr(), None)[0] == -1
    assert sga.sga_validate_csr(rp.data_ptr(), ci.data_ptr(), L, ci.numel(), scratch.data_ptr() + 4, None)[0] == -1


def test_validate_csr_at_size():
    """Workload 4's mask (671,014,912 edges, rows of a million columns) passes, and one duplicate
    column planted deep inside it is found."""
    spec = WORKLOADS["cfg4_bigbird_1m"].mask
    rp, ci = sga.build_mask(spec)
    assert sga.validate_csr(rp, ci) == -1
    row = 777_777
    e = int(rp[row]) + 100
    ci[e] = ci[e - 1]
    assert sga.validate_csr(rp, ci) == row
