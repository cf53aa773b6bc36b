"""Pins for the oracle's mask predicates and CSR enumeration (CPU only).

What fixes these independently of the oracle's own code:
  * closed-form edge counts (NNZ of Section II-D) for each mask family, and the
    per-workload counts stored in tests/golden/edge_counts.txt;
  * structure every such mask must have: the diagonal is present, the element
    masks are symmetric, columns are strictly increasing within a row;
  * the printed 1-D dilated predicate of Section II-C (strict bound, r = s-1)
    evaluated literally in a loop: the inclusive reading with half-width w is
    the printed predicate with window w*s+1;
  * per-row structure of the block mask: exactly 3 window + 2 global + 3 random
    distinct key blocks for interior query blocks.
"""
import os

import numpy as np
import pytest

from sga_inputs import (MaskSpec, KIND_NONLOCAL, KIND_DILATED_2D, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL,
                        KIND_BIGBIRD, WORKLOADS)
from oracle import reference as R
from oracle import rowscan as C

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "edge_counts.txt")


def _golden_counts():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, nnz = line.split()
            out[name] = int(nnz)
    return out


@pytest.mark.parametrize("L,w", [(1, 0), (5, 1), (64, 3), (65, 32), (200, 16), (97, 40)])
def test_sliding_count_and_structure(L, w):
    spec = MaskSpec(KIND_SLIDING, L, window=w)
    m = R.dense_mask(spec)
    if L >= 2 * w + 1:
        assert m.sum() == R.nnz_sliding(L, w)
    assert m.diagonal().all()
    assert (m == m.T).all()
    # interior rows have 2w+1 neighbours, the first row w+1 (clipped)
    assert m[0].sum() == min(L, w + 1)
    if L >= 2 * w + 1:
        assert m[L // 2].sum() == 2 * w + 1 or L < 2 * w + 2


@pytest.mark.parametrize("L,W,s", [(50, 3, 2), (131, 8, 2), (257, 5, 3), (300, 64, 2), (40, 4, 1)])
def test_dilated_count_and_printed_predicate(L, W, s):
    spec = MaskSpec(KIND_DILATED, L, window=W, stride=s)
    m = R.dense_mask(spec)
    if L >= 2 * W * s + 1:
        assert m.sum() == R.nnz_dilated(L, W, s)
    assert m.diagonal().all()
    assert (m == m.T).all()
    # Section II-C, 1-D dilated predicate, literally: abs(i-j) < w and abs(i-j) % (r+1) == 0
    w_paper, r = W * s + 1, s - 1
    lit = np.zeros((L, L), dtype=bool)
    for i in range(L):
        for j in range(L):
            lit[i, j] = (abs(i - j) < w_paper) and (abs(i - j) % (r + 1) == 0)
    assert (lit == m).all()


def test_dilated_stride1_is_sliding():
    a = R.dense_mask(MaskSpec(KIND_DILATED, 120, window=9, stride=1))
    b = R.dense_mask(MaskSpec(KIND_SLIDING, 120, window=9))
    assert (a == b).all()


@pytest.mark.parametrize("L,w,g", [(100, 8, 3), (300, 20, 16), (64, 5, 6), (41, 3, 0)])
def test_global_local_count_and_structure(L, w, g):
    spec = MaskSpec(KIND_GLOBAL_LOCAL, L, window=w, n_global=g)
    m = R.dense_mask(spec)
    assert g <= w + 1 and L >= 2 * w + 1 + g
    assert m.sum() == R.nnz_global_local(L, w, g)
    assert (m == m.T).all()
    assert m[:g].all() and m[:, :g].all()
    loc = R.dense_mask(MaskSpec(KIND_SLIDING, L, window=w))
    assert (m[g:, g:] == loc[g:, g:]).all()


@pytest.mark.parametrize("nb,B,R_", [(10, 4, 3), (23, 8, 3), (16, 2, 1), (40, 4, 5)])
def test_bigbird_structure(nb, B, R_):
    L = nb * B
    spec = MaskSpec(KIND_BIGBIRD, L, block=B, window_blocks=1, n_global_blocks=2,
                    n_random_blocks=R_, seed=1234 + nb)
    m = R.dense_mask(spec)
    assert m.sum() == R.nnz_bigbird_g2_w1(L, B, R_)
    assert m.diagonal().all()
    assert m[:2 * B].all() and m[:, :2 * B].all()
    # block-constant: every B x B block is all-0 or all-1
    blk = m.reshape(nb, B, nb, B)
    assert ((blk.sum(axis=(1, 3)) == 0) | (blk.sum(axis=(1, 3)) == B * B)).all()
    bm = blk[:, 0, :, 0]
    for b in range(2, nb):
        s = R.bigbird_block_set(spec, b)
        assert s == sorted(set(s))
        assert list(np.nonzero(bm[b])[0]) == s
        win = {kb for kb in (b - 1, b, b + 1) if 0 <= kb < nb}
        fixed = win | {0, 1}
        assert fixed <= set(s)
        assert len(s) == len(fixed) + R_


def test_bigbird_random_blocks_depend_on_seed_and_spread():
    nb, B = 64, 2
    mk = lambda seed: MaskSpec(KIND_BIGBIRD, nb * B, block=B, window_blocks=1,
                               n_global_blocks=2, n_random_blocks=3, seed=seed)
    a = [R.bigbird_block_set(mk(1), b) for b in range(nb)]
    b_ = [R.bigbird_block_set(mk(2), b) for b in range(nb)]
    assert a != b_
    # the random picks of all query blocks together cover most key blocks
    picks = set()
    for b in range(2, nb):
        fixed = {0, 1, b - 1, b, b + 1}
        picks |= set(a[b]) - fixed
    assert len(picks) > nb // 2


def test_mix64_known_values():
    # splitmix64 with state increments of the golden gamma, first outputs for seed 0
    # (published test vector of the generator: 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4)
    g = 0x9E3779B97F4A7C15
    assert R.mix64(g) == 0xE220A8397B1DCDAF
    assert R.mix64((2 * g) & ((1 << 64) - 1)) == 0x6E789E6AA1B965F4


def test_csr_from_dense_matches_loops():
    spec = MaskSpec(KIND_GLOBAL_LOCAL, 57, window=4, n_global=2)
    m = R.dense_mask(spec)
    rp, ci = R.csr_from_dense(m)
    cols = []
    ptr = [0]
    for i in range(57):
        for j in range(57):
            if m[i, j]:
                cols.append(j)
        ptr.append(len(cols))
    assert list(rp) == ptr and list(ci) == cols
    assert rp.dtype == np.int64 and ci.dtype == np.int32
    for i in range(57):
        row = ci[rp[i]:rp[i + 1]]
        assert (np.diff(row) > 0).all()
    assert R.sparsity_factor(m) == pytest.approx(len(cols) / 57 ** 2)


def test_symmetric_mask_csr_of_transpose_is_same():
    for spec in [MaskSpec(KIND_SLIDING, 90, window=7),
                 MaskSpec(KIND_DILATED, 90, window=5, stride=2),
                 MaskSpec(KIND_GLOBAL_LOCAL, 90, window=6, n_global=4)]:
        m = R.dense_mask(spec)
        a = R.csr_from_dense(m)
        b = R.csr_from_dense(m.T.copy())
        assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


def test_golden_edge_counts_closed_forms():
    g = _golden_counts()
    w = WORKLOADS
    assert R.nnz_sliding(4096, 32) == g["cfg1_sliding_4k"]
    assert R.nnz_global_local(65536, 128, 16) == g["cfg2_longformer_64k"]
    assert R.nnz_dilated(1 << 20, 64, 2) == g["cfg3_dilated_1m"]
    assert R.nnz_bigbird_g2_w1(1 << 20, 64, 3) == g["cfg4_bigbird_1m"]
    assert R.nnz_sliding(160_000_000, 16) == g["cfg5_sliding_160m"]
    assert set(g) == set(w)


def test_golden_edge_counts_by_scanning():
    """Brute-force scan of every (i, j) pair for the two workloads where L^2 is
    affordable on the CPU (4096^2 and 65536^2)."""
    g = _golden_counts()
    for name in ("cfg1_sliding_4k", "cfg2_longformer_64k"):
        assert C.count_edges(WORKLOADS[name].mask) == g[name]


def test_rowscan_degrees_on_large_masks():
    """Sampled rows of the large workloads: degree by scanning all keys equals
    the per-row closed form (interior 2W+1, clipped at the ends; block mask 8
    key blocks of 64 for interior rows, all keys for global rows)."""
    m3 = WORKLOADS["cfg3_dilated_1m"].mask
    rows = np.array([0, 1, 2, 127, 128, 129, 500_000, (1 << 20) - 1, (1 << 20) - 2])
    deg = C.degrees(m3, rows)
    want = [65, 65, 66, 128, 129, 129, 129, 65, 65]
    assert list(deg) == want
    m4 = WORKLOADS["cfg4_bigbird_1m"].mask
    rows = np.array([0, 127, 128, 191, 192, 70_000, (1 << 20) - 1])
    deg = C.degrees(m4, rows)
    # block 2's window {1,2,3} overlaps global block 1: 2 global + {2,3} + 3 random = 7
    assert list(deg) == [1 << 20, 1 << 20, 7 * 64, 7 * 64, 8 * 64, 8 * 64, 7 * 64]


@pytest.mark.parametrize("L,w,g", [(100, 8, 3), (300, 20, 16), (64, 5, 6), (41, 3, 0), (50, 60, 4)])
def test_nonlocal_is_global_minus_local(L, w, g):
    """Section IV-B, "Global (non-local)": the global mask with the local mask subtracted, so
    that local and non-local passes partition the global+local mask."""
    nl = R.dense_mask(MaskSpec(KIND_NONLOCAL, L, window=w, n_global=g))
    loc = R.dense_mask(MaskSpec(KIND_SLIDING, L, window=w))
    gl = R.dense_mask(MaskSpec(KIND_GLOBAL_LOCAL, L, window=w, n_global=g))
    assert not (nl & loc).any()
    assert ((nl | loc) == gl).all()
    # written out pair by pair
    for i in (0, g - 1 if g else 0, g, L // 2, L - 1):
        for j in range(L):
            assert nl[i, j] == ((i < g or j < g) and abs(i - j) > w)
    if g <= w + 1 and L >= 2 * w + 1 + g:
        assert int(nl.sum()) == R.nnz_nonlocal(L, w, g)
    assert (nl == nl.T).all()


@pytest.mark.parametrize("b,r", [(4, 0), (6, 1), (8, 2), (9, 3)])
def test_dilated_2d_printed_predicate_where_it_is_unambiguous(b, r):
    """The printed 2-D predicate (Section II-C) takes the segment id from i / (L / b) and the
    in-block index from i % b; with L = b*b both describe blocks of b tokens, and the printed
    text evaluated literally must equal the oracle's reading."""
    L = b * b
    m = R.dense_mask(MaskSpec(KIND_DILATED_2D, L, block=b, stride=r + 1))
    for i in range(L):
        for j in range(L):
            printed = 0
            if i // (L // b) == j // (L // b):
                i_b, j_b = i % b, j % b
                if i_b % (r + 1) == 0 and j_b % (r + 1) == 0:
                    printed = 1
            assert int(m[i, j]) == printed


@pytest.mark.parametrize("L,b,s", [(64, 16, 2), (100, 16, 3), (333, 40, 3), (50, 64, 4), (96, 32, 1)])
def test_dilated_2d_count_and_structure(L, b, s):
    m = R.dense_mask(MaskSpec(KIND_DILATED_2D, L, block=b, stride=s))
    assert int(m.sum()) == R.nnz_dilated_2d(L, b, s)
    assert (m == m.T).all()
    deg = m.sum(axis=1)
    for i in range(L):
        blk_len = min(b, L - (i // b) * b)
        expect = -(-blk_len // s) if (i % b) % s == 0 else 0
        assert deg[i] == expect
        if expect:
            cols = np.nonzero(m[i])[0]
            assert cols[0] == (i // b) * b and (np.diff(cols) == s).all()
    if s == 1:      # no dilation: dense blocks on the diagonal
        assert int(m.sum()) == sum(min(b, L - k) ** 2 for k in range(0, L, b))
