"""sga_attention_forward_static (the entry point that allocates nothing) against
sga_attention_forward, through the C ABI: two calls in a row on the library's own scratch array,
the second on a smaller input, each bit-identical to the existing entry point's result."""
import numpy as np
import pytest

import paper_2502_01659_amd as sga
from sga_inputs import MaskSpec, KIND_GLOBAL_LOCAL, KIND_SLIDING, numpy_qkv
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _both(spec, H, d, dtype, seed, path=0):
    import torch
    L = spec.L
    Q, K, V = numpy_qkv(H, L, d, dtype, 0.8, seed)
    dQ, dK, dV = to_device(Q, K, V)
    rp, ci = sga.build_mask(spec)
    nnz = int(rp[-1])
    code = 0 if dtype == "f32" else 1
    stream = torch.cuda.current_stream().cuda_stream
    # existing entry point, caller's workspace
    ws = sga.alloc_workspace(L, H, d, dtype, nnz)
    O_a = torch.full_like(dQ, 7.0)
    lse_a = torch.full((H, L), 7.0, dtype=torch.float32, device="cuda")
    st = sga.sga_attention_forward(dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), rp.data_ptr(), ci.data_ptr(),
                                   O_a.data_ptr(), L, H, d, 0.125, stream, code, lse_a.data_ptr(),
                                   ws.data_ptr(), ws.numel(), path)
    assert st == 0
    # new entry point: no workspace argument, the library's scratch array
    O_b = torch.full_like(dQ, 9.0)
    lse_b = torch.full((H, L), 9.0, dtype=torch.float32, device="cuda")
    st = sga.sga_attention_forward_static(dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), rp.data_ptr(),
                                          ci.data_ptr(), O_b.data_ptr(), L, H, d, 0.125, stream, code,
                                          lse_b.data_ptr(), nnz, path)
    assert st == 0, sga.sga_status_string(st)
    torch.cuda.synchronize()
    assert torch.equal(O_a, O_b), (spec, dtype)
    assert torch.equal(lse_a, lse_b), (spec, dtype)
    assert bool(torch.isfinite(O_b.float()).all())


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_static_scratch_forward_matches_forward(dtype):
    assert sga.sga_static_scratch_init() == 0
    assert sga.sga_static_scratch_bytes() == 64 << 20
    # first call: global rows long enough for multi-segment tiles (partial states, counters and
    # the tile graph all live in the scratch array) ...
    _both(MaskSpec(KIND_GLOBAL_LOCAL, 6001, window=40, n_global=40), H=2, d=64, dtype=dtype, seed=31)
    # ... then a smaller input on the same array, which still holds the first call's contents
    _both(MaskSpec(KIND_GLOBAL_LOCAL, 1500, window=20, n_global=3), H=1, d=64, dtype=dtype, seed=32)
    # and a window mask on the per-row kernels
    _both(MaskSpec(KIND_SLIDING, 700, window=9), H=3, d=64, dtype=dtype, seed=33, path=sga.PATH_GATHER)


def test_static_scratch_rejects_oversized_problems():
    ok = 0x1000
    f = sga.sga_attention_forward_static
    # workload 2 needs more workspace than the scratch array holds
    assert sga.workspace_bytes(65536, 8, 64, "f32", 18919024) > sga.sga_static_scratch_bytes()
    assert f(ok, ok, ok, ok, ok, ok, 65536, 8, 64, 0.125, None, 0, None, 18919024, 0) == -3
    assert f(ok, ok, ok, ok, ok, ok, 64, 1, 64, 0.125, None, 0, None, -1, 0) == -1
    assert f(ok, ok, ok, ok, ok, ok, 64, 1, 48, 0.125, None, 0, None, 64, 0) == -2
