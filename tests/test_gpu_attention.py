"""Attention parity on the GPU: the HIP path, called through the C ABI, against the CPU
oracle on the same seeded, stored input values.

Tolerances (max-abs-error): 1e-5 for fp32, 2e-3 for fp16 storage with fp32 accumulation.
The small cases span several 32/64-row tiles with a ragged tail; every case runs through
each kernel path the entry point offers.
"""
import math

import numpy as np
import pytest

import paper_2502_01659_amd as sga
from sga_inputs import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL, KIND_BIGBIRD,
                        KIND_NONLOCAL, KIND_DILATED_2D,
                        numpy_qkv, small_variants, Workload)
from oracle import reference as R
from gpu_util import TOL, LSE_TOL, to_device, small_inputs, oracle_full, max_err, sample_rows

pytestmark = pytest.mark.gpu

PATHS = [sga.PATH_GATHER, sga.PATH_TILE, sga.PATH_AUTO]
PATH_IDS = ["gather", "tile", "auto"]


def _run_explicit(wl, Q, K, V, path, with_ws=True):
    dQ, dK, dV = to_device(Q, K, V)
    rp, ci = sga.build_mask(wl.mask)
    ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, int(rp[-1])) if with_ws else None
    O, lse = sga.attention_forward(dQ, dK, dV, rp, ci, wl.scale, workspace=ws, path=path,
                                   want_lse=True)
    return O.cpu().numpy(), lse.cpu().numpy()


def _run_implicit(wl, Q, K, V, path):
    dQ, dK, dV = to_device(Q, K, V)
    ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, -1)
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, wl.mask, wl.scale, workspace=ws,
                                            path=path, want_lse=True)
    return O.cpu().numpy(), lse.cpu().numpy()


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("wl", small_variants(), ids=lambda w: w.name)
def test_small_workloads_explicit(wl, path):
    print("case", wl.name, path, flush=True)
    Q, K, V = small_inputs(wl)
    O, lse = _run_explicit(wl, Q, K, V, path)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    assert max_err(O, O_ref) <= TOL[wl.dtype]
    assert max_err(lse, lse_ref) <= LSE_TOL[wl.dtype]


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("wl", [w for w in small_variants() if w.mask.kind in (KIND_SLIDING, KIND_DILATED)],
                         ids=lambda w: w.name)
def test_small_workloads_implicit(wl, path):
    print("case", wl.name, path, flush=True)
    Q, K, V = small_inputs(wl)
    O, lse = _run_implicit(wl, Q, K, V, path)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    assert max_err(O, O_ref) <= TOL[wl.dtype]
    assert max_err(lse, lse_ref) <= LSE_TOL[wl.dtype]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("spec", [
    MaskSpec(KIND_SLIDING, 1, window=3),
    MaskSpec(KIND_SLIDING, 31, window=2),
    MaskSpec(KIND_SLIDING, 33, window=40),
    MaskSpec(KIND_SLIDING, 700, window=0),
    MaskSpec(KIND_DILATED, 515, window=6, stride=3),
    MaskSpec(KIND_DILATED, 200, window=64, stride=2),
    MaskSpec(KIND_GLOBAL_LOCAL, 257, window=3, n_global=1),
    MaskSpec(KIND_BIGBIRD, 16 * 20, block=16, window_blocks=1, n_global_blocks=1,
             n_random_blocks=2, seed=9),
], ids=lambda s: f"{s.name}-L{s.L}")
@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_ragged_and_degenerate_shapes(spec, dtype, path):
    print("case", spec, dtype, path, flush=True)
    wl = Workload("t", H=3, L=spec.L, d=64, dtype=dtype, sigma=0.8, mask=spec, explicit=True, seed=77)
    Q, K, V = small_inputs(wl)
    O, lse = _run_explicit(wl, Q, K, V, path)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    assert max_err(O, O_ref) <= TOL[dtype]
    assert max_err(lse, lse_ref) <= LSE_TOL[dtype]
    if spec.kind in (KIND_SLIDING, KIND_DILATED):
        O2, _ = _run_implicit(wl, Q, K, V, path)
        assert max_err(O2, O_ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("spec", [
    MaskSpec(KIND_SLIDING, 320, window=64),      # last workgroup: a full 256-key window that ends at L
    MaskSpec(KIND_SLIDING, 319, window=64),
    MaskSpec(KIND_SLIDING, 321, window=64),
    MaskSpec(KIND_SLIDING, 640, window=64),      # interior workgroups with full windows, first and last ragged
    MaskSpec(KIND_SLIDING, 513, window=63),
    MaskSpec(KIND_SLIDING, 513, window=65),      # one key past the workgroup kernel's window
    MaskSpec(KIND_SLIDING, 131, window=16),
    MaskSpec(KIND_SLIDING, 700, window=32),      # 6 key blocks per workgroup: the widest with K and V side by side
    MaskSpec(KIND_SLIDING, 700, window=33),      # 7: the narrowest with K, then V, in one set of blocks
    MaskSpec(KIND_SLIDING, 900, window=32),      # 6 whole blocks per interior workgroup
    MaskSpec(KIND_SLIDING, 901, window=48),      # 7
    MaskSpec(KIND_DILATED, 1801, window=40, stride=2),
    MaskSpec(KIND_DILATED, 1931, window=64, stride=3),   # classes of 644, 644 and 643 tokens
    MaskSpec(KIND_DILATED, 769, window=48, stride=2),
], ids=lambda s: f"{s.name}-L{s.L}-w{s.window}")
def test_window_staging_boundaries(spec, dtype):
    """Implicit windows on the tile path at the sizes where the fp16 workgroup kernels change
    shape: windows of 6 key blocks (K and V side by side in LDS) against 7 and 8 (K, then V over
    it), full 8-block windows next to ragged ones, the widest window the workgroup kernels take
    and the first one they do not, short sequences."""
    print("case", spec, dtype, flush=True)
    wl = Workload("t", H=2, L=spec.L, d=64, dtype=dtype, sigma=0.8, mask=spec, explicit=False, seed=123)
    Q, K, V = small_inputs(wl)
    O, lse = _run_implicit(wl, Q, K, V, sga.PATH_TILE)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    assert max_err(O, O_ref) <= TOL[dtype]
    assert max_err(lse, lse_ref) <= LSE_TOL[dtype]


@pytest.mark.parametrize("spec", [
    MaskSpec(KIND_SLIDING, 3000, window=700),
    MaskSpec(KIND_SLIDING, 1537, window=1536),             # every row attends every key
    MaskSpec(KIND_DILATED, 3001, window=300, stride=3),
    MaskSpec(KIND_DILATED_2D, 2500, block=1100, stride=1),
], ids=lambda s: f"{s.name}-L{s.L}")
@pytest.mark.parametrize("H", [1, 3])
@pytest.mark.parametrize("d,dtype", [(64, "f32"), (128, "f32"), (128, "f16"), (256, "f32")])
def test_short_sequences_with_wide_windows_are_cut_into_key_ranges(spec, H, d, dtype):
    """Window tiles of a call with few tiles and many key blocks per tile (fp32 at d = 64, both
    types at d = 128 and 256) are cut into ranges of key blocks whose partial states are merged
    afterwards (only with a workspace): results with and without a workspace against the oracle,
    and a continuing call on top."""
    print("case", spec, H, d, dtype, flush=True)
    wl = Workload("t", H=H, L=spec.L, d=d, dtype=dtype, sigma=0.9, mask=spec, explicit=False, seed=31)
    Q, K, V = small_inputs(wl)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    dQ, dK, dV = to_device(Q, K, V)
    ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, -1)
    for workspace in (ws, None):
        O, lse = sga.attention_forward_implicit(dQ, dK, dV, spec, wl.scale, workspace=workspace,
                                                path=sga.PATH_TILE, want_lse=True)
        assert max_err(O.cpu().numpy(), O_ref) <= TOL[dtype]
        assert max_err(lse.cpu().numpy(), lse_ref) <= LSE_TOL[dtype]
    # the same mask applied twice in a row: the second call continues the first one's state,
    # which leaves O unchanged and adds ln 2 to lse
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, spec, wl.scale, workspace=ws, path=sga.PATH_TILE,
                                            want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, spec, wl.scale, O, lse, workspace=ws, path=sga.PATH_TILE)
    nonempty = np.isfinite(lse_ref)
    assert max_err(O.cpu().numpy(), O_ref) <= TOL[dtype]
    assert max_err(lse.cpu().numpy()[nonempty], lse_ref[nonempty] + math.log(2.0)) <= LSE_TOL[dtype]


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("sf", [1.0, 0.5, 0.1, 0.01])
def test_verification_protocol_bernoulli_masks(sf, path):
    """Section V-A protocol (L=256, U[0,1) inputs, Bernoulli masks of several sparsity factors,
    allclose atol 1e-8 / rtol 1e-5 against a dense masked reference, empty rows equal), with
    d=64 (the supported head size) and the fp64 oracle as the dense reference; the fp32 kernel
    is held to its own bar of 1e-5 max-abs."""
    import torch
    L, d = 256, 64
    Q, K, V = numpy_qkv(2, L, d, "f32", 1.0, 500, dist="uniform")
    mask = np.random.default_rng(17).random((L, L)) < sf
    rp, ci = R.csr_from_dense(mask)
    dQ, dK, dV = to_device(Q, K, V)
    drp, dci = to_device(rp, ci if len(ci) else np.zeros(1, np.int32))
    ws = sga.alloc_workspace(L, 2, d, "f32", int(rp[-1]))
    O, lse = sga.attention_forward(dQ, dK, dV, drp, dci, 1 / math.sqrt(d), workspace=ws, path=path,
                                   want_lse=True)
    O = O.cpu().numpy()
    lse = lse.cpu().numpy()
    for h in range(2):
        O_ref, lse_ref = R.attention_dense(Q[h], K[h], V[h], mask, 1 / math.sqrt(d))
        assert max_err(O[h], O_ref) <= 1e-5
        empty = ~mask.any(axis=1)
        assert (O[h][empty] == 0).all() and np.isneginf(lse[h][empty]).all()
        assert max_err(lse[h][~empty], lse_ref[~empty]) <= LSE_TOL["f32"]


def _scattered_masks(L):
    """Dense masks with scattered columns at block fills that keep them on the tile path, long
    enough that a tile's key-block list spans several windows of the CSR -> tile pass's bitmap
    walk (32 key blocks each): even fill, fill that falls off along the row (so the late windows
    are sparse), wide empty stretches between scattered ones, scattered columns next to rows that
    are one run (a dense row, a band) or empty, and a scattered start followed by whole runs."""
    rng = np.random.default_rng(23)
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    u = rng.random((L, L))
    out = {}
    out["even_0.3"] = u < 0.3
    out["even_0.7"] = u < 0.7
    out["falling"] = u < 0.9 * (1.0 - j / L) ** 2
    out["gaps"] = (u < 0.5) & ((j // 700) % 2 == 0)
    mixed = u < 0.4
    mixed[5] = True
    mixed[40:50] = False
    mixed[64:96] = (np.abs(i - j) <= 40)[64:96]
    mixed[96:128, :] = (u < 0.4)[96:128, :] | (j >= L - 200)
    out["mixed_rows"] = mixed
    out["scattered_then_runs"] = ((u < 0.5) & (j < 900)) | ((j >= 1500) & (j < 1500 + 64 + i % 200))
    return out


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("name", ["even_0.3", "even_0.7", "falling", "gaps", "mixed_rows", "scattered_then_runs"])
def test_scattered_masks_every_path(name, dtype):
    import torch
    L, d, H = 3301, 64, 2
    mask = _scattered_masks(L)[name]
    Q, K, V = numpy_qkv(H, L, d, dtype, 0.7, 910)
    rp, ci = R.csr_from_dense(mask)
    dQ, dK, dV = to_device(Q, K, V)
    drp, dci = to_device(rp, ci)
    refs = [R.attention_dense(Q[h], K[h], V[h], mask, 0.125) for h in range(H)]
    empty = ~mask.any(axis=1)
    ws = sga.alloc_workspace(L, H, d, dtype, int(rp[-1]))
    for path in PATHS:
        O, lse = sga.attention_forward(dQ, dK, dV, drp, dci, 0.125, workspace=ws, path=path, want_lse=True)
        O, lse = O.cpu().numpy(), lse.cpu().numpy()
        for h in range(H):
            assert max_err(O[h], refs[h][0]) <= TOL[dtype], (path, h)
            assert (O[h][empty] == 0).all() and np.isneginf(lse[h][empty]).all()
            assert max_err(lse[h][~empty], refs[h][1][~empty]) <= LSE_TOL[dtype], (path, h)
    # the graph made once reproduces the call that makes it every time
    O1, l1 = sga.attention_forward(dQ, dK, dV, drp, dci, 0.125, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    ws2 = sga.alloc_workspace(L, H, d, dtype, int(rp[-1]))
    ws2.fill_(0x5A)
    plan = sga.graph_prepare(drp, dci, H, d, dtype, ws2)
    O2, l2 = sga.attention_forward_prepared(dQ, dK, dV, drp, dci, 0.125, plan, ws2, want_lse=True)
    torch.cuda.synchronize()
    assert plan.tiles_left < (L + 31) // 32          # (the tile path took part in it)
    assert torch.equal(O1, O2) and torch.equal(l1, l2)


def _run_masks(L):
    """Dense masks whose rows are made of runs of consecutive columns, one shape per branch of the
    CSR -> tile conversion: every row one run with touching block ranges (the loop without
    reductions), one run per row at far-apart places (block ranges with gaps), two and three
    runs per row, runs that end exactly at block borders, empty rows in between, and dense
    leading rows next to short ones (a tile that is cut into segments)."""
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    out = {}
    out["band"] = np.abs(i - j) <= 70
    start = (i * 37) % (L - 60)
    out["staircase"] = (j >= start) & (j < start + 1 + (i % 50))
    out["two_runs"] = (j < 24) | ((j >= i // 2) & (j < i // 2 + 90))
    out["three_runs"] = (j < 32) | ((j >= 64 + (i % 7)) & (j < 160)) | (j >= L - 32 - (i % 3))
    out["block_borders"] = (j >= 32 * (i // 64)) & (j < 32 * (i // 64) + 96)
    sparse_rows = out["band"].copy()
    sparse_rows[(np.arange(L) % 5) == 2] = False
    out["empty_rows"] = sparse_rows
    dense_head = out["band"].copy()
    dense_head[:20, :] = True
    out["dense_leading_rows"] = dense_head
    return out


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("name", ["band", "staircase", "two_runs", "three_runs", "block_borders",
                                  "empty_rows", "dense_leading_rows"])
def test_run_structured_masks_every_path(name, dtype):
    L, d, H = 4133, 64, 2
    mask = _run_masks(L)[name]
    Q, K, V = numpy_qkv(H, L, d, dtype, 0.7, 900)
    rp, ci = R.csr_from_dense(mask)
    dQ, dK, dV = to_device(Q, K, V)
    drp, dci = to_device(rp, ci)
    ws = sga.alloc_workspace(L, H, d, dtype, int(rp[-1]))
    rows = sample_rows(L, 5, 100)
    refs = [R.attention_dense(Q[h][rows].astype(np.float64), K[h].astype(np.float64),
                              V[h].astype(np.float64), mask[rows], 0.125) for h in range(H)]
    for path in PATHS:
        print("case", name, dtype, path, flush=True)
        O, lse = sga.attention_forward(dQ, dK, dV, drp, dci, 0.125, workspace=ws, path=path, want_lse=True)
        O = O.cpu().numpy()
        lse = lse.cpu().numpy()
        for h in range(H):
            O_ref, lse_ref = refs[h]
            empty = ~mask[rows].any(axis=1)
            assert max_err(O[h][rows], O_ref) <= TOL[dtype]
            assert (O[h][rows][empty] == 0).all() and np.isneginf(lse[h][rows][empty]).all()
            assert max_err(lse[h][rows][~empty], lse_ref[~empty]) <= LSE_TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_single_neighbour_rows_return_v_exactly(dtype, path):
    L, d = 200, 64
    Q, K, V = numpy_qkv(1, L, d, dtype, 1.0, 41)
    perm = np.random.default_rng(2).permutation(L)
    rp = np.arange(L + 1, dtype=np.int64)
    ci = perm.astype(np.int32)
    dQ, dK, dV, drp, dci = to_device(Q, K, V, rp, ci)
    ws = sga.alloc_workspace(L, 1, d, dtype, L)
    O = sga.attention_forward(dQ, dK, dV, drp, dci, 0.125, workspace=ws, path=path).cpu().numpy()
    assert np.array_equal(O[0], V[0][perm])


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_ones_v_gives_ones_everywhere(dtype, path):
    wl = [w for w in small_variants() if w.name == "cfg2_small"][0]
    Q, K, V = numpy_qkv(wl.H, wl.L, wl.d, dtype, 1.0, 3)
    V = np.ones_like(V)
    O, _ = _run_explicit(Workload("t", wl.H, wl.L, wl.d, dtype, 1.0, wl.mask, True), Q, K, V, path)
    assert np.abs(O.astype(np.float64) - 1.0).max() <= (1e-5 if dtype == "f32" else 1e-3)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_large_scores_are_stable_and_shift_invariant(path):
    spec = MaskSpec(KIND_GLOBAL_LOCAL, 400, window=20, n_global=2)
    wl = Workload("t", H=1, L=400, d=64, dtype="f32", sigma=1.0, mask=spec, explicit=True, seed=5)
    Q, K, V = small_inputs(wl)
    Qb = (Q * 12.0).astype(np.float32)           # scores of magnitude ~100
    O, lse = _run_explicit(wl, Qb, K, V, path)
    assert np.isfinite(O).all() and np.isfinite(lse).all()
    O_ref, _ = oracle_full(wl, Qb, K, V)
    assert max_err(O, O_ref) <= 1e-4             # |s| ~ 100: fp32 score rounding ~1e-5 relative
    t = np.random.default_rng(1).standard_normal(64).astype(np.float32)
    O1, _ = _run_explicit(wl, Q, K, V, path)
    O2, _ = _run_explicit(wl, Q, (K + t).astype(np.float32), V, path)
    assert max_err(O1, O2) <= 2e-5


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_split_rows_high_degree(dtype, path):
    """Global tokens over L=20,000: rows of degree 20,000 go through the split-row path."""
    L = 20000
    spec = MaskSpec(KIND_GLOBAL_LOCAL, L, window=5, n_global=3)
    wl = Workload("t", H=2, L=L, d=64, dtype=dtype, sigma=0.7, mask=spec, explicit=True, seed=9)
    Q, K, V = small_inputs(wl)
    O, lse = _run_explicit(wl, Q, K, V, path)
    rows = np.concatenate([np.arange(0, 40), np.arange(9990, 10010), np.arange(L - 20, L)])
    O_ref, lse_ref = R.attention_masked(Q, K, V, spec, wl.scale, rows=rows)
    assert max_err(O[:, rows], O_ref) <= TOL[dtype]
    assert max_err(lse[:, rows], lse_ref) <= LSE_TOL[dtype]
    # without a workspace the long rows run unsplit: same values within tolerance
    O_ns, _ = _run_explicit(wl, Q, K, V, sga.PATH_GATHER, with_ws=False)
    assert max_err(O_ns[:, rows], O_ref) <= TOL[dtype]
    # deterministic: a second run is bit-identical
    O_b, _ = _run_explicit(wl, Q, K, V, path)
    assert np.array_equal(O, O_b)


@pytest.mark.parametrize("dtype,L,p", [("f32", 7000, 0.2), ("f16", 13000, 0.11)])
def test_rows_split_by_l2_share(dtype, L, p):
    """Keys whose K and V do not fit one L2: rows of a uniformly random mask with 1,000 to 2,000
    neighbours (below the ordinary split threshold) are cut into 8 chunks that run on the 8
    XCDs, beside shorter rows that stay whole and two dense rows.  Sampled rows against the dense
    oracle on every path, and a rerun is bit-identical."""
    print("case l2 split", dtype, L, flush=True)
    H, d = 2, 64
    rng = np.random.default_rng(77)
    mask = rng.random((L, L)) < p                    # about 1,400 neighbours per row
    mask[1::3] &= rng.random((L // 3 + 1, L))[: len(mask[1::3])] < 0.3      # every third row: about 420
    mask[5] = True
    mask[L - 2] = True
    mask[40] = False                                 # an empty row
    rp, ci = R.csr_from_dense(mask)
    deg = np.diff(rp)
    assert (deg[0::3][3:] >= 8 * 128).all() and (deg[0::3] <= 2048).all() and (deg[1::3].max() < 8 * 128)
    Q, K, V = numpy_qkv(H, L, d, dtype, 0.6, 31)
    dQ, dK, dV = to_device(Q, K, V)
    drp, dci = to_device(rp, ci)
    ws = sga.alloc_workspace(L, H, d, dtype, int(rp[-1]))
    rows = np.unique(np.concatenate([np.arange(0, 60), [L - 2, L - 1], rng.integers(0, L, 80)]))
    refs = [R.attention_dense(Q[h][rows].astype(np.float64), K[h].astype(np.float64),
                              V[h].astype(np.float64), mask[rows], 0.125) for h in range(H)]
    for path in (sga.PATH_GATHER, sga.PATH_AUTO):
        O, lse = sga.attention_forward(dQ, dK, dV, drp, dci, 0.125, workspace=ws, path=path, want_lse=True)
        O2 = sga.attention_forward(dQ, dK, dV, drp, dci, 0.125, workspace=ws, path=path)
        import torch
        torch.cuda.synchronize()
        assert torch.equal(O, O2)
        for h in range(H):
            _close(O[h].cpu().numpy()[rows], lse[h].cpu().numpy()[rows], refs[h][0], refs[h][1], dtype)


def test_explicit_and_implicit_paths_agree():
    """The same mask through the CSR entry point and the implicit entry point (the paper's
    own cross-check between its CSR and ordered-sparsity kernels, Section V-F)."""
    wl = [w for w in small_variants() if w.name == "cfg3_small"][0]
    Q, K, V = small_inputs(wl)
    for path in PATHS:
        O1, _ = _run_explicit(wl, Q, K, V, path)
        O2, _ = _run_implicit(wl, Q, K, V, path)
        assert max_err(O1, O2) <= 2 * TOL[wl.dtype]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("scale", [-0.125, 0.0, 0.37])
def test_scale_sign_zero_and_non_power_of_two(scale, dtype, path):
    """The scale multiplies the dot product (Eq. 1): a negative one reverses the ranking of the
    neighbours, zero gives uniform weights, and a value that is no power of two is not exact in
    fp16 (the scale must not be folded into the stored inputs)."""
    print("case scale", scale, dtype, path, flush=True)
    # (the three windows run on the three fp16 window kernels of the tile path)
    for spec, implicit in [(MaskSpec(KIND_GLOBAL_LOCAL, 333, window=20, n_global=3), False),
                           (MaskSpec(KIND_DILATED, 333, window=9, stride=2), True),
                           (MaskSpec(KIND_DILATED, 700, window=60, stride=2), True),
                           (MaskSpec(KIND_SLIDING, 500, window=100), True)]:
        wl = Workload("t", H=2, L=spec.L, d=64, dtype=dtype, sigma=1.0, mask=spec, explicit=True, seed=5)
        Q, K, V = small_inputs(wl)
        dQ, dK, dV = to_device(Q, K, V)
        O_ref, lse_ref = R.attention_masked(Q, K, V, spec, scale)
        rp, ci = sga.build_mask(spec)
        ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, int(rp[-1]))
        O, lse = sga.attention_forward(dQ, dK, dV, rp, ci, scale, workspace=ws, path=path, want_lse=True)
        assert max_err(O.cpu().numpy(), O_ref) <= TOL[dtype]
        assert max_err(lse.cpu().numpy(), lse_ref) <= LSE_TOL[dtype]
        if implicit:
            O, lse = sga.attention_forward_implicit(dQ, dK, dV, spec, scale, workspace=ws, path=path,
                                                    want_lse=True)
            assert max_err(O.cpu().numpy(), O_ref) <= TOL[dtype]
            assert max_err(lse.cpu().numpy(), lse_ref) <= LSE_TOL[dtype]


def _carry_factor(dtype, calls):
    """Tolerance factor of a state continued over `calls` calls: fp16 storage rounds O to fp16
    after every call, so the bar scales with the number of calls; fp32 keeps the single-call bar."""
    return calls if dtype == "f16" else 1.0


def _close(O, lse, O_ref, lse_ref, dtype, factor=1.0):
    assert max_err(O, O_ref) <= factor * TOL[dtype]
    empty = np.isneginf(lse_ref)
    assert (np.isneginf(lse) == empty).all()
    if (~empty).any():
        assert max_err(lse[~empty], lse_ref[~empty]) <= LSE_TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("spec", [
    MaskSpec(KIND_NONLOCAL, 700, window=20, n_global=5),
    MaskSpec(KIND_NONLOCAL, 9000, window=128, n_global=16),       # global rows pass the split threshold
    MaskSpec(KIND_NONLOCAL, 100, window=200, n_global=3),          # window covers everything: no edge at all
    MaskSpec(KIND_NONLOCAL, 300, window=2, n_global=64),
    MaskSpec(KIND_DILATED_2D, 640, block=64, stride=2),
    MaskSpec(KIND_DILATED_2D, 1000, block=96, stride=3),
    MaskSpec(KIND_DILATED_2D, 333, block=40, stride=1),
    # classes of 60 and of 64 tokens per block: every key of the class is within 7 or 8 key
    # blocks of 128 queries (fp16: K and V take turns in the workgroup's LDS blocks)
    MaskSpec(KIND_DILATED_2D, 1300, block=120, stride=2),
    MaskSpec(KIND_DILATED_2D, 900, block=64, stride=1),
], ids=lambda s: f"{s.name}-L{s.L}-b{s.block}")
def test_nonlocal_and_dilated_2d_masks(spec, dtype):
    """Explicit CSR (every path) and the implicit generators of the global (non-local) and
    2-D dilated masks against the dense oracle; rows without neighbours are the initial state."""
    print("case", spec, dtype, flush=True)
    wl = Workload("t", H=2, L=spec.L, d=64, dtype=dtype, sigma=0.9, mask=spec, explicit=True, seed=31)
    Q, K, V = small_inputs(wl)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    for path in PATHS:
        O, lse = _run_explicit(wl, Q, K, V, path)
        _close(O, lse, O_ref, lse_ref, dtype)
    for path in PATHS:
        O, lse = _run_implicit(wl, Q, K, V, path)
        _close(O, lse, O_ref, lse_ref, dtype)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("block,stride", [(1000, 3), (700, 2), (4000, 1), (200, 5)])
def test_dilated_2d_implicit_tiles(block, stride, d, dtype):
    """2-D dilated blocks through the implicit tile kernels: blocks of several tiles with a
    ragged last block, blocks longer than the sequence, stride 1 (no empty row), and a continuing
    call, which must leave the rows without neighbours as they are."""
    print("case 2d", block, stride, d, dtype, flush=True)
    L = 2500
    spec = MaskSpec(KIND_DILATED_2D, L, block=block, stride=stride)
    wl = Workload("t", H=2, L=L, d=d, dtype=dtype, sigma=0.9, mask=spec, explicit=True, seed=33)
    Q, K, V = small_inputs(wl)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    for path in (sga.PATH_TILE, sga.PATH_AUTO):
        O, lse = _run_implicit(wl, Q, K, V, path)
        _close(O, lse, O_ref, lse_ref, dtype)
    # local window first, then the 2-D dilated edges that the window does not already hold (as
    # an explicit CSR), then the whole 2-D mask again on top of a copy: rows off the stride keep
    # the earlier state
    dQ, dK, dV = to_device(Q, K, V)
    loc = MaskSpec(KIND_SLIDING, L, window=6)
    wsi = sga.alloc_workspace(L, wl.H, d, dtype, -1)
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=wsi, want_lse=True)
    O0, lse0 = O.clone(), lse.clone()
    sga.attention_accumulate_implicit(dQ, dK, dV, spec, wl.scale, O, lse, workspace=wsi, path=sga.PATH_TILE)
    off = (np.arange(L) % block) % stride != 0
    assert (O.cpu().numpy()[:, off] == O0.cpu().numpy()[:, off]).all()
    assert (lse.cpu().numpy()[:, off] == lse0.cpu().numpy()[:, off]).all()
    # on the stride: the state of window + block edges, counted twice where both masks hold
    # them; compare against the oracle's two-pass composition of the same two masks
    m1 = R.dense_mask(loc)
    m2 = R.dense_mask(spec)
    for h in range(wl.H):
        O1, l1 = R.attention_dense(Q[h], K[h], V[h], m1, wl.scale)
        O2, l2 = R.attention_dense(Q[h], K[h], V[h], m2, wl.scale)
        lse_c = np.logaddexp(l1, l2)
        w1 = np.exp(l1 - lse_c)[:, None]
        w2 = np.where(np.isneginf(l2), 0.0, np.exp(l2 - lse_c))[:, None]
        _close(O[h].cpu().numpy(), lse[h].cpu().numpy(), w1 * O1 + w2 * O2, lse_c, dtype, factor=_carry_factor(dtype, 2.0))


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_sequential_composition_equals_single_mask(dtype, path):
    """Section V-F: local kernel, then the global (non-local) kernel, on one shared state,
    against one call on the combined mask -- with explicit CSR masks, with implicit masks,
    and mixed; and a three-part BigBird-like composition local -> non-local -> CSR(random)."""
    L, w, g = 2500, 24, 7
    wl = Workload("t", H=3, L=L, d=64, dtype=dtype, sigma=1.0,
                  mask=MaskSpec(KIND_GLOBAL_LOCAL, L, window=w, n_global=g), explicit=True, seed=41)
    Q, K, V = small_inputs(wl)
    dQ, dK, dV = to_device(Q, K, V)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    loc = MaskSpec(KIND_SLIDING, L, window=w)
    nl = MaskSpec(KIND_NONLOCAL, L, window=w, n_global=g)
    ws_i = sga.alloc_workspace(L, wl.H, 64, dtype, -1)
    # implicit local -> implicit non-local
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=ws_i, path=path,
                                            want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, nl, wl.scale, O, lse, workspace=ws_i, path=path)
    _close(O.cpu().numpy(), lse.cpu().numpy(), O_ref, lse_ref, dtype, factor=_carry_factor(dtype, 2.0))
    # explicit local -> explicit non-local
    rp1, ci1 = sga.build_mask(loc)
    rp2, ci2 = sga.build_mask(nl)
    ws1 = sga.alloc_workspace(L, wl.H, 64, dtype, int(rp1[-1]))
    ws2 = sga.alloc_workspace(L, wl.H, 64, dtype, int(rp2[-1]))
    O, lse = sga.attention_forward(dQ, dK, dV, rp1, ci1, wl.scale, workspace=ws1, path=path,
                                   want_lse=True)
    sga.attention_accumulate(dQ, dK, dV, rp2, ci2, wl.scale, O, lse, workspace=ws2, path=path)
    _close(O.cpu().numpy(), lse.cpu().numpy(), O_ref, lse_ref, dtype, factor=_carry_factor(dtype, 2.0))
    # non-local first (rows >= g with no global column in reach start empty), then local
    O, lse = sga.attention_forward(dQ, dK, dV, rp2, ci2, wl.scale, workspace=ws2, path=path,
                                   want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, loc, wl.scale, O, lse, workspace=ws_i, path=path)
    _close(O.cpu().numpy(), lse.cpu().numpy(), O_ref, lse_ref, dtype, factor=_carry_factor(dtype, 2.0))
    # three parts: local, non-local, then a random CSR with the first two removed
    rng = np.random.default_rng(5)
    extra = rng.random((L, L)) < 0.002
    covered = R.dense_mask(wl.mask)
    extra &= ~covered
    rp3, ci3 = R.csr_from_dense(extra)
    import torch
    rp3 = torch.from_numpy(rp3).cuda()
    ci3 = torch.from_numpy(ci3).cuda()
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=ws_i, path=path,
                                            want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, nl, wl.scale, O, lse, workspace=ws_i, path=path)
    ws3 = sga.alloc_workspace(L, wl.H, 64, dtype, int(rp3[-1]))
    sga.attention_accumulate(dQ, dK, dV, rp3, ci3, wl.scale, O, lse, workspace=ws3, path=path)
    O3_ref, lse3_ref = R.attention_dense(Q[0], K[0], V[0], covered | extra, wl.scale)
    _close(O[0].cpu().numpy(), lse[0].cpu().numpy(), O3_ref, lse3_ref, dtype, factor=_carry_factor(dtype, 3.0))


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("d", [32, 128, 256])
def test_other_head_dimensions(d, dtype):
    """Head dimensions of the paper's verification (d_k = 32, Section V-A) and microbenchmark
    runs (128, 256, Section V-C): explicit CSR incl. split rows and empty rows, implicit window,
    dilated, 2-D dilated and non-local masks, and a composed local + non-local pass."""
    print("case d", d, dtype, flush=True)
    for spec, implicit in [(MaskSpec(KIND_GLOBAL_LOCAL, 2600, window=9, n_global=3), False),
                           (MaskSpec(KIND_SLIDING, 700, window=20), True),
                           (MaskSpec(KIND_DILATED, 700, window=11, stride=3), True),
                           (MaskSpec(KIND_DILATED_2D, 700, block=50, stride=2), True),
                           (MaskSpec(KIND_NONLOCAL, 2600, window=9, n_global=3), True)]:
        wl = Workload("t", H=2, L=spec.L, d=d, dtype=dtype, sigma=0.8, mask=spec, explicit=True, seed=61)
        Q, K, V = small_inputs(wl)
        O_ref, lse_ref = oracle_full(wl, Q, K, V)
        O, lse = _run_explicit(wl, Q, K, V, sga.PATH_AUTO)
        _close(O, lse, O_ref, lse_ref, dtype)
        O, lse = _run_explicit(wl, Q, K, V, sga.PATH_GATHER, with_ws=False)
        _close(O, lse, O_ref, lse_ref, dtype)
        if d >= 128:      # matrix-core kernels on 64-channel slices
            O, lse = _run_explicit(wl, Q, K, V, sga.PATH_TILE)
            _close(O, lse, O_ref, lse_ref, dtype)
        if implicit:
            for path in [sga.PATH_AUTO, sga.PATH_GATHER] + ([sga.PATH_TILE] if d >= 128 else []):
                O, lse = _run_implicit(wl, Q, K, V, path)
                _close(O, lse, O_ref, lse_ref, dtype)
    # Bernoulli mask with empty rows (the verification protocol's kind of mask)
    L = 300
    rng = np.random.default_rng(8)
    dense = rng.random((L, L)) < 0.02
    wl = Workload("t", H=1, L=L, d=d, dtype=dtype, sigma=1.0, mask=MaskSpec(KIND_SLIDING, L), explicit=True,
                  seed=62)
    Q, K, V = small_inputs(wl)
    dQ, dK, dV = to_device(Q, K, V)
    rp, ci = R.csr_from_dense(dense)
    import torch
    rp = torch.from_numpy(rp).cuda()
    ci_t = torch.from_numpy(ci).cuda() if len(ci) else torch.empty(0, dtype=torch.int32, device="cuda")
    ws = sga.alloc_workspace(L, 1, d, dtype, int(rp[-1]))
    O, lse = sga.attention_forward(dQ, dK, dV, rp, ci_t, wl.scale, workspace=ws, want_lse=True)
    O_ref, lse_ref = R.attention_dense(Q[0], K[0], V[0], dense, wl.scale)
    _close(O[0].cpu().numpy(), lse[0].cpu().numpy(), O_ref, lse_ref, dtype)
    # composition on one state
    loc, nl = MaskSpec(KIND_SLIDING, L, window=5), MaskSpec(KIND_NONLOCAL, L, window=5, n_global=2)
    wsi = sga.alloc_workspace(L, 1, d, dtype, -1)
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=wsi, want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, nl, wl.scale, O, lse, workspace=wsi)
    O_ref, lse_ref = R.attention_masked(Q, K, V, MaskSpec(KIND_GLOBAL_LOCAL, L, window=5, n_global=2), wl.scale)
    _close(O.cpu().numpy(), lse.cpu().numpy(), O_ref, lse_ref, dtype, factor=_carry_factor(dtype, 2.0))
    # the tile kernels work on 64-channel slices
    if d < 64:
        with pytest.raises(sga.SgaError):
            sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=wsi, path=sga.PATH_TILE)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("d", [128, 256])
def test_wide_tiles_segments_and_composition(d, dtype):
    """Head dimensions 128 and 256 on the tile path: dense global rows long enough for
    multi-segment tiles (partial states per 64-channel slice and their merge), a ragged tail, a
    negative scale, and the composed local -> non-local pass through the merge's carry."""
    print("case wide", d, dtype, flush=True)
    L = 3001 if dtype == "f32" else 17001       # 40 global rows: 2 segments or more in either type
    spec = MaskSpec(KIND_GLOBAL_LOCAL, L, window=40, n_global=40)
    wl = Workload("t", H=2, L=L, d=d, dtype=dtype, sigma=0.7, mask=spec, explicit=True, seed=81)
    Q, K, V = small_inputs(wl)
    rows = np.arange(L) if L < 4000 else sample_rows(L, 9, 150, edge=120)
    O_ref, lse_ref = R.attention_masked(Q, K, V, spec, wl.scale, rows=rows)
    O_neg, lse_neg = R.attention_masked(-Q, K, V, spec, wl.scale, rows=rows)

    def close(O, lse, ref, lref, factor=1.0):
        _close(O.cpu().numpy()[:, rows], lse.cpu().numpy()[:, rows], ref, lref, dtype, factor)

    dQ, dK, dV = to_device(Q, K, V)
    rp, ci = sga.build_mask(spec)
    ws = sga.alloc_workspace(L, wl.H, d, dtype, int(rp[-1]))
    O, lse = sga.attention_forward(dQ, dK, dV, rp, ci, wl.scale, workspace=ws, path=sga.PATH_TILE,
                                   want_lse=True)
    close(O, lse, O_ref, lse_ref)
    # negative scale: the oracle on -Q
    O, lse = sga.attention_forward(dQ, dK, dV, rp, ci, -wl.scale, workspace=ws, path=sga.PATH_TILE,
                                   want_lse=True)
    close(O, lse, O_neg, lse_neg)
    # local (implicit) then non-local (CSR, multi-segment tiles) on one state
    loc = MaskSpec(KIND_SLIDING, L, window=40)
    nl = MaskSpec(KIND_NONLOCAL, L, window=40, n_global=40)
    rp2, ci2 = sga.build_mask(nl)
    ws2 = sga.alloc_workspace(L, wl.H, d, dtype, int(rp2[-1]))
    wsi = sga.alloc_workspace(L, wl.H, d, dtype, -1)
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=wsi, path=sga.PATH_TILE,
                                            want_lse=True)
    sga.attention_accumulate(dQ, dK, dV, rp2, ci2, wl.scale, O, lse, workspace=ws2, path=sga.PATH_TILE)
    close(O, lse, O_ref, lse_ref, factor=_carry_factor(dtype, 2.0))
    # and in the other order, the window pass continuing the state
    O, lse = sga.attention_forward(dQ, dK, dV, rp2, ci2, wl.scale, workspace=ws2, path=sga.PATH_TILE,
                                   want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, loc, wl.scale, O, lse, workspace=wsi, path=sga.PATH_TILE)
    close(O, lse, O_ref, lse_ref, factor=_carry_factor(dtype, 2.0))


@pytest.mark.parametrize("wl", [w for w in small_variants() if w.dtype == "f32"], ids=lambda w: w.name)
def test_split_precision_path_small_workloads(wl):
    """fp32 storage with the products on the fp16 matrix cores (three-term split): same
    tolerance as the true-fp32 kernels, explicit and implicit."""
    print("case split", wl.name, flush=True)
    Q, K, V = small_inputs(wl)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    O, lse = _run_explicit(wl, Q, K, V, sga.PATH_TILE_SPLIT)
    assert max_err(O, O_ref) <= TOL["f32"]
    assert max_err(lse, lse_ref) <= 1e-4
    if wl.mask.kind in (KIND_SLIDING, KIND_DILATED):
        O, lse = _run_implicit(wl, Q, K, V, sga.PATH_TILE_SPLIT)
        assert max_err(O, O_ref) <= TOL["f32"]
        assert max_err(lse, lse_ref) <= 1e-4


@pytest.mark.parametrize("sigma", [0.02, 1.0, 6.0])
def test_split_precision_path_value_ranges(sigma):
    """Small, unit and large input magnitudes (the remainders of small values are subnormal in
    fp16 unless scaled; large scores stress the exponent), a mask with global rows (multi-
    segment tiles), ragged tail, negative scale, and the composition call."""
    print("case split sigma", sigma, flush=True)
    spec = MaskSpec(KIND_GLOBAL_LOCAL, 1500, window=40, n_global=5)
    wl = Workload("t", H=2, L=spec.L, d=64, dtype="f32", sigma=sigma, mask=spec, explicit=True, seed=71)
    Q, K, V = small_inputs(wl)
    dQ, dK, dV = to_device(Q, K, V)
    rp, ci = sga.build_mask(spec)
    ws = sga.alloc_workspace(wl.L, wl.H, 64, "f32", int(rp[-1]))
    for scale in (wl.scale, -wl.scale):
        O_ref, lse_ref = R.attention_masked(Q, K, V, spec, scale)
        O, lse = sga.attention_forward(dQ, dK, dV, rp, ci, scale, workspace=ws, path=sga.PATH_TILE_SPLIT,
                                       want_lse=True)
        O32 = sga.attention_forward(dQ, dK, dV, rp, ci, scale, workspace=ws, path=sga.PATH_TILE)
        # O scales with |V|; with scores of +-150 (sigma = 6) the fp32 rounding of the scores
        # themselves dominates, so the true-fp32 kernel's own error is the yardstick there
        tol = max(TOL["f32"] * max(1.0, sigma), 2.0 * max_err(O32.cpu().numpy(), O_ref))
        assert max_err(O.cpu().numpy(), O_ref) <= tol
        assert max_err(lse.cpu().numpy(), lse_ref) <= 1e-4 * max(1.0, sigma * sigma)
    loc, nl = MaskSpec(KIND_SLIDING, spec.L, window=40), MaskSpec(KIND_NONLOCAL, spec.L, window=40, n_global=5)
    wsi = sga.alloc_workspace(wl.L, wl.H, 64, "f32", -1)
    O, lse = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=wsi,
                                            path=sga.PATH_TILE_SPLIT, want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, nl, wl.scale, O, lse, workspace=wsi)
    O32, lse32 = sga.attention_forward_implicit(dQ, dK, dV, loc, wl.scale, workspace=wsi,
                                                path=sga.PATH_TILE, want_lse=True)
    sga.attention_accumulate_implicit(dQ, dK, dV, nl, wl.scale, O32, lse32, workspace=wsi)
    O_ref, lse_ref = R.attention_masked(Q, K, V, spec, wl.scale)
    tol = max(2 * TOL["f32"] * max(1.0, sigma), 2.0 * max_err(O32.cpu().numpy(), O_ref))
    assert max_err(O.cpu().numpy(), O_ref) <= tol
    # fp16 storage has no split path
    with pytest.raises(sga.SgaError):
        h = dQ.half()
        sga.attention_forward_implicit(h, h, h, loc, wl.scale, path=sga.PATH_TILE_SPLIT)


def _random_case(seed):
    """A seeded random (mask, shape) draw over every mask family, ragged lengths and both
    storage types; parameters stay inside the ranges the descriptors document."""
    rng = np.random.default_rng(1000 + seed)
    kind = [KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL, KIND_BIGBIRD, KIND_NONLOCAL,
            KIND_DILATED_2D][seed % 6]
    L = int(rng.integers(1, 900))
    d = int(rng.choice([64, 64, 128, 256, 32]))
    dtype = "f32" if rng.random() < 0.5 else "f16"
    H = int(rng.integers(1, 4))
    if kind == KIND_SLIDING:
        spec = MaskSpec(kind, L, window=int(rng.integers(0, 2 * L + 2)) if rng.random() < 0.3
                        else int(rng.integers(0, 70)))
    elif kind == KIND_DILATED:
        spec = MaskSpec(kind, L, window=int(rng.integers(0, 40)), stride=int(rng.integers(1, 9)))
    elif kind in (KIND_GLOBAL_LOCAL, KIND_NONLOCAL):
        spec = MaskSpec(kind, L, window=int(rng.integers(0, 50)), n_global=int(rng.integers(0, 40)))
    elif kind == KIND_DILATED_2D:
        spec = MaskSpec(kind, L, block=int(rng.integers(1, 2 * L + 2)), stride=int(rng.integers(1, 6)))
    else:
        block = int(rng.choice([8, 16, 32, 64]))
        nb = int(rng.integers(8, 24))
        L = block * nb
        wb, g, r = int(rng.integers(0, 2)), int(rng.integers(0, 3)), int(rng.integers(0, 3))
        spec = MaskSpec(kind, L, block=block, window_blocks=wb, n_global_blocks=g, n_random_blocks=r,
                        seed=int(rng.integers(0, 1 << 30)))
    sigma = float(rng.choice([0.3, 0.6, 1.0]))   # (the absolute tolerances are stated for |O| of order 1)
    return Workload(f"r{seed}", H=H, L=L, d=d, dtype=dtype, sigma=sigma, mask=spec, explicit=True,
                    seed=500 + seed)


@pytest.mark.parametrize("seed", range(36))
def test_random_shapes_every_path(seed):
    """Seeded random draws over mask family, length, head dimension, heads and storage type:
    the explicit call on every path the shape allows, and the implicit call where the family has
    a generator, against the dense oracle."""
    wl = _random_case(seed)
    print("case", wl.name, wl.mask, wl.d, wl.dtype, wl.H, flush=True)
    Q, K, V = small_inputs(wl)
    O_ref, lse_ref = oracle_full(wl, Q, K, V)
    paths = [sga.PATH_AUTO, sga.PATH_GATHER] + ([sga.PATH_TILE] if wl.d >= 64 else [])
    for path in paths:
        O, lse = _run_explicit(wl, Q, K, V, path)
        _close(O, lse, O_ref, lse_ref, wl.dtype)
    kind = wl.mask.kind
    implicit_ok = kind in (KIND_SLIDING, KIND_DILATED, KIND_DILATED_2D) or \
        (kind == KIND_NONLOCAL and wl.mask.n_global <= 64)
    if implicit_ok:
        for path in paths:
            O, lse = _run_implicit(wl, Q, K, V, path)
            _close(O, lse, O_ref, lse_ref, wl.dtype)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_forward_calls_replay_from_a_hip_graph(dtype):
    """The entry points only queue kernels on the caller's stream (no allocation, no
    synchronisation, no memset), so a caller may capture them into a HIP graph: mask build,
    explicit forward and implicit forward are captured once and replayed three times with new
    inputs and eager work in between; every replay must equal the eager result bit for bit."""
    import torch
    spec = MaskSpec(KIND_GLOBAL_LOCAL, 3000, window=70, n_global=20)
    loc = MaskSpec(KIND_SLIDING, 3000, window=48)
    H, L, d = 2, spec.L, 64
    nnz = sga.mask_nnz(spec)
    tdt = torch.float32 if dtype == "f32" else torch.float16
    dev = "cuda:0"
    Q = torch.empty((H, L, d), dtype=tdt, device=dev)
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)
    O = torch.empty_like(Q)
    O2 = torch.empty_like(Q)
    lse = torch.empty((H, L), dtype=torch.float32, device=dev)
    rp = torch.empty(L + 1, dtype=torch.int64, device=dev)
    ci = torch.empty(nnz, dtype=torch.int32, device=dev)
    ws = sga.alloc_workspace(L, H, d, dtype, nnz)
    ws2 = sga.alloc_workspace(L, H, d, dtype, -1)

    def fill(seed):
        q, k, v = numpy_qkv(H, L, d, dtype, 0.9, seed)
        Q.copy_(torch.from_numpy(q).to(dev))
        K.copy_(torch.from_numpy(k).to(dev))
        V.copy_(torch.from_numpy(v).to(dev))

    def step():
        st = sga.sga_build_mask(spec, rp.data_ptr(), ci.data_ptr(), ci.numel(),
                                torch.cuda.current_stream().cuda_stream)
        assert st == 0
        sga.attention_forward(Q, K, V, rp, ci, 0.125, O=O, lse=lse, workspace=ws)
        sga.attention_forward_implicit(Q, K, V, loc, 0.125, O=O2, workspace=ws2)

    fill(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                      # warm-up outside the capture (library load, first launches)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for seed in (2, 3, 4):
        fill(seed)
        step()
        torch.cuda.synchronize()
        want = (O.clone(), O2.clone(), lse.clone())
        O.zero_()
        O2.zero_()
        lse.zero_()
        (Q.float().sum() + 1).item()        # eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want[0]) and torch.equal(O2, want[1]) and torch.equal(lse, want[2])
