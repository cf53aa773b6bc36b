"""Prepared graphs (sga_graph_prepare + *_prepared calls) against the unprepared calls.

A prepared call launches fewer kernels on the same tile graph, so its output must equal the
unprepared call's bit for bit (same workspace size, hence the same work decomposition), for new
Q/K/V on the same plan, call after call (the schedule counters put themselves back), and for
the continuing (accumulate) form.  The unprepared calls are themselves checked against the
oracle in test_gpu_attention.py; one case here also goes to the oracle directly.
"""
import numpy as np
import pytest

import paper_2502_01659_amd as sga
from sga_inputs import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL, KIND_BIGBIRD, KIND_NONLOCAL,
                        numpy_qkv, Workload)
from oracle import reference as R
from gpu_util import TOL, to_device, max_err

pytestmark = pytest.mark.gpu


def _bernoulli_csr(L, p, seed, dense_rows=()):
    rng = np.random.default_rng(seed)
    dense = rng.random((L, L)) < p
    for r in dense_rows:
        dense[r, :] = True
    return dense


def _cases():
    out = []
    # (name, L, H, d, dtype, dense mask or spec)
    out.append(("window_small_f32", 1037, 1, 64, "f32", MaskSpec(KIND_SLIDING, 1037, window=32)))
    out.append(("longformer_segments_f32", 3001, 2, 64, "f32",
                MaskSpec(KIND_GLOBAL_LOCAL, 3001, window=40, n_global=40)))      # multi-segment tiles
    out.append(("longformer_segments_f16", 17001, 2, 64, "f16",
                MaskSpec(KIND_GLOBAL_LOCAL, 17001, window=40, n_global=40)))
    out.append(("bigbird_f16", 64 * 23, 2, 64, "f16",
                MaskSpec(KIND_BIGBIRD, 64 * 23, block=64, window_blocks=1, n_global_blocks=2,
                         n_random_blocks=3, seed=5)))
    out.append(("nonlocal_f32", 2500, 3, 64, "f32", MaskSpec(KIND_NONLOCAL, 2500, window=24, n_global=7)))
    # scattered columns: no tile qualifies, every row runs on the per-row kernels
    out.append(("bernoulli_sparse_f32", 700, 2, 64, "f32", _bernoulli_csr(700, 0.02, 1)))
    # three dense rows that do not fill a tile: split rows on the per-row kernels beside tiles
    out.append(("dense_rows_f16", 9000, 2, 64, "f16", _bernoulli_csr(9000, 0.0005, 2, dense_rows=(5, 4000, 8999))))
    # a window mask with one aligned tile of scattered rows: tiles and leftover rows in one call
    mixed = np.abs(np.subtract.outer(np.arange(1300), np.arange(1300))) <= 40
    mixed[128:160] = _bernoulli_csr(1300, 0.01, 3)[128:160]
    out.append(("mixed_tiles_and_rows_f32", 1300, 2, 64, "f32", mixed))
    out.append(("longformer_d128_f32", 3001, 2, 128, "f32",
                MaskSpec(KIND_GLOBAL_LOCAL, 3001, window=40, n_global=40)))
    out.append(("window_d256_f16", 900, 1, 256, "f16", MaskSpec(KIND_SLIDING, 900, window=50)))
    return out


def _csr(mask):
    import torch
    if isinstance(mask, MaskSpec):
        return sga.build_mask(mask)
    rp, ci = R.csr_from_dense(mask)
    rp = torch.from_numpy(rp).cuda()
    ci = torch.from_numpy(ci).cuda() if len(ci) else torch.empty(0, dtype=torch.int32, device="cuda")
    return rp, ci


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c[0])
def test_prepared_forward_is_bit_identical(case):
    import torch
    name, L, H, d, dtype, mask = case
    print("case", name, flush=True)
    rp, ci = _csr(mask)
    nnz = int(rp[-1])
    ws_a = sga.alloc_workspace(L, H, d, dtype, nnz)      # unprepared calls
    ws_b = sga.alloc_workspace(L, H, d, dtype, nnz)      # the prepared graph lives here
    ws_b.fill_(0xA5)                                     # nothing may rely on a clean workspace
    plan = sga.graph_prepare(rp, ci, H, d, dtype, ws_b)
    assert plan.L == L and plan.nnz == nnz and plan.H == H and plan.d == d
    print("  plan: tiles_left", plan.tiles_left, "multi_tiles", plan.multi_tiles, "tile_parts",
          plan.tile_parts, "long_rows", plan.long_rows, "row_chunks", plan.row_chunks, "flags", plan.flags,
          flush=True)
    for seed in (3, 4, 5):              # new Q/K/V on the same plan, three calls in a row
        Q, K, V = numpy_qkv(H, L, d, dtype, 0.8, seed)
        dQ, dK, dV = to_device(Q, K, V)
        O_a, lse_a = sga.attention_forward(dQ, dK, dV, rp, ci, 0.11, workspace=ws_a, want_lse=True)
        O_b, lse_b = sga.attention_forward_prepared(dQ, dK, dV, rp, ci, 0.11, plan, ws_b, want_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(O_a, O_b), (name, seed)
        assert torch.equal(lse_a, lse_b), (name, seed)
    # the continuing form: the same state through both
    sga.attention_accumulate(dQ, dK, dV, rp, ci, 0.07, O_a, lse_a, workspace=ws_a)
    sga.attention_accumulate_prepared(dQ, dK, dV, rp, ci, 0.07, plan, ws_b, O_b, lse_b)
    torch.cuda.synchronize()
    assert torch.equal(O_a, O_b) and torch.equal(lse_a, lse_b), name


def test_prepared_plan_contents_and_oracle():
    """What the plan reports for masks whose structure is known, and one prepared result against
    the oracle itself."""
    L, H, d = 3001, 2, 64
    spec = MaskSpec(KIND_GLOBAL_LOCAL, L, window=40, n_global=40)
    rp, ci = sga.build_mask(spec)
    ws = sga.alloc_workspace(L, H, d, "f32", int(rp[-1]))
    plan = sga.graph_prepare(rp, ci, H, d, "f32", ws)
    assert plan.flags & sga.GRAPH_TILES_COVER_ALL and plan.tiles_left == 0
    assert plan.multi_tiles == 2 and plan.tile_parts >= 4      # the two tiles that hold the 40 global rows
    assert plan.long_rows == 0
    Q, K, V = numpy_qkv(H, L, d, "f32", 0.8, 21)
    dQ, dK, dV = to_device(Q, K, V)
    O, lse = sga.attention_forward_prepared(dQ, dK, dV, rp, ci, 0.125, plan, ws, want_lse=True)
    O_ref, lse_ref = R.attention_masked(Q, K, V, spec, 0.125)
    assert max_err(O.cpu().numpy(), O_ref) <= TOL["f32"]
    assert max_err(lse.cpu().numpy(), lse_ref) <= 1e-4
    # scattered mask: every tile is left to the per-row kernels
    dense = _bernoulli_csr(700, 0.02, 1)
    rp, ci = _csr(dense)
    ws = sga.alloc_workspace(700, 1, d, "f32", int(rp[-1]))
    plan = sga.graph_prepare(rp, ci, 1, d, "f32", ws)
    assert not (plan.flags & sga.GRAPH_TILES_COVER_ALL) and plan.tiles_left == (700 + 31) // 32
    # a workspace sized for fewer edges than the mask has is refused
    import torch
    small = torch.empty(sga.workspace_bytes(700, 1, d, "f32", 10), dtype=torch.uint8, device="cuda")
    with pytest.raises(sga.SgaError):
        sga.graph_prepare(rp, ci, 1, d, "f32", small)
    # the plan belongs to its buffers
    other = sga.alloc_workspace(700, 1, d, "f32", int(rp[-1]))
    Q, K, V = numpy_qkv(1, 700, d, "f32", 0.8, 22)
    dQ, dK, dV = to_device(Q, K, V)
    with pytest.raises(sga.SgaError):
        sga.attention_forward_prepared(dQ, dK, dV, rp, ci, 0.125, plan, other)


def test_prepared_forward_replays_from_a_hip_graph():
    """A prepared forward queues kernels only: captured once, replayed with new inputs and eager
    work in between, every replay equals the eager result bit for bit (the schedule counters of
    the fp32 kernel are put back by the kernel itself, not by a memset)."""
    import torch
    L, H, d = 3000, 2, 64
    spec = MaskSpec(KIND_GLOBAL_LOCAL, L, window=70, n_global=20)
    rp, ci = sga.build_mask(spec)
    ws = sga.alloc_workspace(L, H, d, "f32", int(rp[-1]))
    plan = sga.graph_prepare(rp, ci, H, d, "f32", ws)
    dev = "cuda:0"
    Q = torch.empty((H, L, d), dtype=torch.float32, device=dev)
    K, V, O = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    lse = torch.empty((H, L), dtype=torch.float32, device=dev)

    def fill(seed):
        q, k, v = numpy_qkv(H, L, d, "f32", 0.9, seed)
        Q.copy_(torch.from_numpy(q).to(dev))
        K.copy_(torch.from_numpy(k).to(dev))
        V.copy_(torch.from_numpy(v).to(dev))

    def step():
        sga.attention_forward_prepared(Q, K, V, rp, ci, 0.125, plan, ws, O=O, lse=lse)

    fill(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for seed in (2, 3, 4):
        fill(seed)
        step()
        torch.cuda.synchronize()
        want = (O.clone(), lse.clone())
        O.zero_()
        lse.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want[0]) and torch.equal(lse, want[1]), seed


@pytest.mark.parametrize("spec,dtype", [
    (MaskSpec(KIND_DILATED, 5000, window=64, stride=2), "f16"),      # K, then V, in one set of LDS blocks
    (MaskSpec(KIND_SLIDING, 5000, window=16), "f16"),                # K and V side by side
    (MaskSpec(KIND_SLIDING, 5000, window=300), "f16"),               # ring of blocks per workgroup
    (MaskSpec(KIND_SLIDING, 3000, window=100), "f32"),
], ids=lambda v: v if isinstance(v, str) else f"{v.name}-w{v.window}")
def test_implicit_forward_replays_from_a_hip_graph(spec, dtype):
    """The implicit forward needs no workspace and queues kernels only: captured once, every
    replay (new inputs and eager work in between) equals the eager result bit for bit."""
    import torch
    L, H, d = spec.L, 2, 64
    dev = "cuda:0"
    tdt = torch.float16 if dtype == "f16" else torch.float32
    Q = torch.empty((H, L, d), dtype=tdt, device=dev)
    K, V, O = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    lse = torch.empty((H, L), dtype=torch.float32, device=dev)

    def fill(seed):
        q, k, v = numpy_qkv(H, L, d, dtype, 0.7, seed)
        Q.copy_(torch.from_numpy(q).to(dev))
        K.copy_(torch.from_numpy(k).to(dev))
        V.copy_(torch.from_numpy(v).to(dev))

    def step():
        sga.attention_forward_implicit(Q, K, V, spec, 0.125, O=O, lse=lse)

    fill(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for seed in (2, 3, 4):
        fill(seed)
        step()
        torch.cuda.synchronize()
        want = (O.clone(), lse.clone())
        O.zero_()
        lse.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want[0]) and torch.equal(lse, want[1]), seed
