"""Parity at the full benchmark sizes, in the launch configuration bench.py times
(same entry points, path = auto, workspace from sga_workspace_bytes).

The oracle cannot enumerate these problems densely, so each test compares
  * a seeded row sample (both sequence ends, rows around 32/64/128/256-row tile boundaries,
    every global row class, random rows) against the row-scan oracle, which evaluates the mask
    predicate over every key of each sampled row; and
  * properties that hold for every row at any size: V = ones gives O = ones everywhere, and
    Q = 0 turns a window mask into a moving average that fp64 prefix sums compute for all rows.
"""
import numpy as np
import pytest

import paper_2502_01659_amd as sga
from sga_inputs import WORKLOADS, TABLE3_WORKLOADS, torch_qkv
from oracle import rowscan as C
from gpu_util import TOL, max_err, neighbor_lists, sample_rows

pytestmark = pytest.mark.gpu


def _forward(wl, Q, K, V):
    import torch
    nnz = sga.mask_nnz(wl.mask)
    if wl.explicit:
        rp, ci = sga.build_mask(wl.mask)
        ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, nnz)
        O, lse = sga.attention_forward(Q, K, V, rp, ci, wl.scale, workspace=ws, want_lse=True)
    else:
        ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, -1)
        O, lse = sga.attention_forward_implicit(Q, K, V, wl.mask, wl.scale, workspace=ws, want_lse=True)
    torch.cuda.synchronize()
    return O, lse


def _check_sampled(wl, Q, K, V, O, lse, rows, heads):
    """Row-scan oracle on `rows` of `heads`; K/V rows are fetched from the device by index."""
    import torch
    worst = 0.0
    lists = neighbor_lists(wl.mask, rows)
    for h in heads:
        for i, nb in zip(rows, lists):
            idx = torch.from_numpy(nb).cuda()
            Kg = K[h].index_select(0, idx).float().cpu().numpy()
            Vg = V[h].index_select(0, idx).float().cpu().numpy()
            q = Q[h, int(i)].float().cpu().numpy()
            o_ref, lse_ref = C.attend_gathered(q, Kg, Vg, wl.scale)
            err = max_err(O[h, int(i)].float().cpu().numpy(), o_ref)
            worst = max(worst, err)
            assert err <= TOL[wl.dtype], (wl.name, h, int(i), err)
            assert abs(float(lse[h, int(i)]) - lse_ref) <= 1e-3, (wl.name, h, int(i))
    return worst


def _check_ones(wl, Q, K):
    import torch
    V1 = torch.ones_like(Q)
    O, _ = _forward(wl, Q, K, V1)
    tol = 1e-5 if wl.dtype == "f32" else 1e-3
    assert float((O.float() - 1.0).abs().max()) <= tol
    del O, V1


def _check_moving_average(wl, K, V, chunk=1 << 22):
    """Q = 0: every row's output is the mean of its neighbours' V rows (window masks).
    The means come from fp64 prefix sums, chunk by chunk with a halo of W rows."""
    import torch
    Q0 = torch.zeros_like(K)
    O, _ = _forward(wl, Q0, K, V)
    del Q0
    s, W, L = wl.mask.stride, wl.mask.window, wl.L
    for h in range(wl.H):
        worst = 0.0
        for p in range(s):
            n = (L - p + s - 1) // s                      # tokens of this residue class
            for a in range(0, n, chunk):
                b = min(n, a + chunk)
                lo_h, hi_h = max(0, a - W), min(n, b + W)  # halo
                v = V[h, p + lo_h * s: p + (hi_h - 1) * s + 1: s].double()
                cs = torch.zeros((v.shape[0] + 1, wl.d), dtype=torch.float64, device=v.device)
                torch.cumsum(v, dim=0, out=cs[1:])
                u = torch.arange(a, b, device=v.device)
                lo = torch.clamp(u - W, min=0) - lo_h
                hi = torch.clamp(u + W, max=n - 1) - lo_h
                want = (cs[hi + 1] - cs[lo]) / (hi - lo + 1).unsqueeze(1).double()
                got = O[h, p + a * s: p + (b - 1) * s + 1: s].double()
                worst = max(worst, float((got - want).abs().max()))
                del v, cs, want, got
        assert worst <= TOL[wl.dtype], (wl.name, h, worst)


def test_cfg1_full_every_row():
    import torch
    wl = WORKLOADS["cfg1_sliding_4k"]
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda")
    O, lse = _forward(wl, Q, K, V)
    O_ref, lse_ref, edges = C.attend_rows(wl.mask, Q[0].cpu().numpy(), K[0].cpu().numpy(),
                                          V[0].cpu().numpy(), wl.scale, np.arange(wl.L))
    assert edges == sga.mask_nnz(wl.mask)
    assert max_err(O[0].cpu().numpy(), O_ref) <= TOL["f32"]
    assert max_err(lse[0].cpu().numpy(), lse_ref) <= 1e-4


def test_cfg2_full_size():
    wl = WORKLOADS["cfg2_longformer_64k"]
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda")
    O, lse = _forward(wl, Q, K, V)
    rows = sample_rows(wl.L, wl.seed + 4, n_random=300, edge=160)
    print("cfg2 sampled rows", len(rows), flush=True)
    # whole K/V of a head fit on the host: scan oracle over the sample for every head
    for h in range(wl.H):
        O_ref, lse_ref, _ = C.attend_rows(wl.mask, Q[h].cpu().numpy(), K[h].cpu().numpy(),
                                          V[h].cpu().numpy(), wl.scale, rows)
        assert max_err(O[h][rows].cpu().numpy(), O_ref) <= TOL["f32"], h
        assert max_err(lse[h][rows].cpu().numpy(), lse_ref) <= 1e-4, h
    _check_ones(wl, Q, K)
    # the split-precision path (fp16 matrix-core products) on the same problem: two heads against
    # the oracle sample, all heads against the true-fp32 result
    rp, ci = sga.build_mask(wl.mask)
    ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, int(rp[-1]))
    Os, lses = sga.attention_forward(Q, K, V, rp, ci, wl.scale, workspace=ws, path=sga.PATH_TILE_SPLIT,
                                     want_lse=True)
    for h in (0, wl.H - 1):
        O_ref, lse_ref, _ = C.attend_rows(wl.mask, Q[h].cpu().numpy(), K[h].cpu().numpy(),
                                          V[h].cpu().numpy(), wl.scale, rows)
        assert max_err(Os[h][rows].cpu().numpy(), O_ref) <= TOL["f32"], h
        assert max_err(lses[h][rows].cpu().numpy(), lse_ref) <= 1e-4, h
    assert float((Os - O).abs().max()) <= 2 * TOL["f32"]


def test_cfg3_full_size():
    wl = WORKLOADS["cfg3_dilated_1m"]
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda")
    O, lse = _forward(wl, Q, K, V)
    rows = sample_rows(wl.L, wl.seed + 4, n_random=120, edge=140, n_tile_idx=6)
    print("cfg3 sampled rows", len(rows), flush=True)
    _check_sampled(wl, Q, K, V, O, lse, rows, heads=[0, wl.H - 1])
    _check_ones(wl, Q, K)
    _check_moving_average(wl, K, V)


def test_cfg4_full_size():
    wl = WORKLOADS["cfg4_bigbird_1m"]
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda")
    O, lse = _forward(wl, Q, K, V)
    rng = np.random.default_rng(wl.seed + 4)
    rows = np.unique(np.concatenate([
        [0, 31, 32, 127],                         # global query blocks (degree L)
        [128, 129, 191, 192, 255, 256],           # first non-global blocks
        [wl.L - 1, wl.L - 64, wl.L - 65],
        rng.integers(128, wl.L, size=40)]))
    print("cfg4 sampled rows", len(rows), flush=True)
    _check_sampled(wl, Q, K, V, O, lse, rows, heads=[0, wl.H - 1])
    _check_ones(wl, Q, K)


def test_cfg5_full_size():
    import torch
    wl = WORKLOADS["cfg5_sliding_160m"]
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda")
    O, lse = _forward(wl, Q, K, V)
    # every sampled row takes its neighbour list from the oracle's scan of the predicate over
    # all 160M keys (both sequence ends, rows around tile boundaries, random rows)
    rows = sample_rows(wl.L, wl.seed + 4, n_random=24, edge=12, n_tile_idx=2)
    print("cfg5 sampled rows", len(rows), flush=True)
    _check_sampled(wl, Q, K, V, O, lse, rows, heads=[0])
    del O, lse
    torch.cuda.empty_cache()
    _check_moving_average(wl, K, V)


def _table3_case(wl, n_random, edge):
    """A long-context shape of Table III (Section V-E) through sga_attention_forward_implicit:
    sampled rows against the row-scan oracle, V = ones on every row, Q = 0 (moving average by
    fp64 prefix sums) on every row."""
    import torch
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda")
    O, lse = _forward(wl, Q, K, V)
    rows = sample_rows(wl.L, wl.seed + 4, n_random=n_random, edge=edge, n_tile_idx=2)
    print(wl.name, "window", wl.mask.window, "sampled rows", len(rows), flush=True)
    worst = _check_sampled(wl, Q, K, V, O, lse, rows, heads=[0])
    print(wl.name, "worst sampled error", worst, flush=True)
    del O, lse
    torch.cuda.empty_cache()
    _check_ones(wl, Q, K)
    del Q
    torch.cuda.empty_cache()
    _check_moving_average(wl, K, V)


def test_table3_1p6m_wide_band():
    # +-1359 keys: 87 key blocks per 64-query pair of tiles
    _table3_case(TABLE3_WORKLOADS["table3_1p6m"], n_random=60, edge=24)


def test_table3_160m_wide_band():
    # +-799 keys at 160M tokens: element offsets pass 2^31 and 2^33
    _table3_case(TABLE3_WORKLOADS["table3_160m"], n_random=16, edge=8)


@pytest.mark.parametrize("L,H,W,s", [(40013, 4, 700, 1), (70001, 3, 200, 3), (33000, 8, 65, 1),
                                     (50_000_017, 1, 300, 1)])      # (byte offsets past 2^33)
def test_d128_wide_band(L, H, W, s):
    """Wide fp16 bands at d = 128 (the head size of the models of Table IV) on calls large enough
    for the kernel that keeps all 128 channels of a sub-tile in one wavefront: ragged lengths,
    a dilated window, and the narrowest window that takes it; sampled rows against the row-scan
    oracle, V = ones and the Q = 0 moving average on every row."""
    from sga_inputs import MaskSpec, Workload, KIND_SLIDING, KIND_DILATED
    spec = MaskSpec(KIND_SLIDING if s == 1 else KIND_DILATED, L, window=W, stride=s)
    wl = Workload(f"d128_L{L}_w{W}_s{s}", H=H, L=L, d=128, dtype="f16", sigma=0.5, mask=spec, explicit=False,
                  seed=77)
    _table3_case(wl, n_random=40, edge=40)
