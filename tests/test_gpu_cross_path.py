"""The tile kernels against the per-row kernels on seeded random shapes.

The two families share no kernel code (matrix-core tiles with block masks against one wavefront
per row walking the neighbour list), so their agreement on shapes nobody chose by hand (sequence
lengths that cut tiles, windows on both sides of every kernel switch, random block patterns)
is a property that holds at sizes the dense oracle does not reach.  Each path is compared with
the oracle itself in test_gpu_attention.py; here the bar is twice the oracle tolerance, relative
to 1 + |O|, and the lse of every row must agree, -inf included.  Prepared graphs must reproduce
the unprepared result bit for bit.
"""
import random

import pytest

import paper_2502_01659_amd as sga
from sga_inputs import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL, KIND_BIGBIRD, KIND_NONLOCAL,
                        KIND_DILATED_2D, torch_qkv)
from gpu_util import TOL, LSE_TOL

pytestmark = pytest.mark.gpu


def _agree(O1, l1, O2, l2, dtype, amp=1.0):
    import torch
    assert torch.isfinite(O1.float()).all() and torch.isfinite(O2.float()).all()
    err = ((O1.float() - O2.float()).abs() / (1.0 + O2.float().abs())).max().item()
    assert err <= 2 * TOL[dtype] * amp, err
    inf1, inf2 = ~torch.isfinite(l1), ~torch.isfinite(l2)
    assert torch.equal(inf1, inf2)
    if (~inf1).any():
        assert (l1[~inf1] - l2[~inf1]).abs().max().item() <= 2.5 * LSE_TOL[dtype] * amp


def _window_spec(rng):
    kind = rng.choice([KIND_SLIDING, KIND_DILATED, KIND_DILATED_2D])
    L = rng.choice([rng.randint(1, 300), rng.randint(300, 3000), rng.randint(3000, 20000)])
    if kind == KIND_DILATED_2D:
        stride = rng.randint(1, 4)
        block = rng.choice([rng.randint(1, 80), rng.randint(80, 300), rng.randint(30, 70) * stride])
        return MaskSpec(kind, L, block=block, stride=stride)
    stride = 1 if kind == KIND_SLIDING else rng.randint(2, 4)
    # both sides of the kernel switches at 32 (6 -> 7 key blocks per workgroup) and 64 (band kernel)
    W = rng.choice([rng.randint(0, 16), rng.randint(17, 32), rng.randint(33, 64), rng.randint(65, 200)])
    return MaskSpec(kind, L, window=W, stride=stride)


@pytest.mark.parametrize("seed", range(40))
def test_implicit_tiles_agree_with_row_kernels(seed):
    import torch
    rng = random.Random(1000 + seed)
    spec = _window_spec(rng)
    dtype = rng.choice(["f16", "f16", "f32"])
    H = rng.choice([1, 2, 3])
    sigma = rng.choice([0.3, 1.0, 3.0])
    scale = rng.choice([0.125, -0.125, 0.5])
    amp = max(1.0, sigma * sigma * abs(scale) * 8)      # rounding of the scores grows with their size
    print("case", seed, spec, dtype, "H", H, "sigma", sigma, "scale", scale, flush=True)
    Q, K, V = torch_qkv(H, spec.L, 64, dtype, sigma, seed, "cuda:0")
    O1, l1 = sga.attention_forward_implicit(Q, K, V, spec, scale, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward_implicit(Q, K, V, spec, scale, path=sga.PATH_GATHER, want_lse=True)
    torch.cuda.synchronize()
    _agree(O1, l1, O2, l2, dtype, amp)


def _explicit_spec(rng, seed):
    kind = rng.choice([KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL, KIND_BIGBIRD, KIND_NONLOCAL, KIND_DILATED_2D])
    L = rng.choice([rng.randint(1, 300), rng.randint(300, 3000), rng.randint(3000, 30000)])
    if kind == KIND_BIGBIRD:
        block = rng.choice([16, 32, 64, 128])
        nb = max(8, L // block)
        wb, ng = rng.randint(0, 2), rng.randint(0, 2)
        nr = rng.randint(0, max(0, min(3, nb - (2 * wb + 1) - ng - 1)))
        return MaskSpec(kind, nb * block, block=block, window_blocks=wb, n_global_blocks=ng, n_random_blocks=nr,
                        seed=seed)
    if kind == KIND_DILATED_2D:
        return MaskSpec(kind, L, block=rng.randint(1, 400), stride=rng.randint(1, 4))
    if kind in (KIND_GLOBAL_LOCAL, KIND_NONLOCAL):
        return MaskSpec(kind, L, window=rng.randint(0, 200), n_global=rng.randint(0, min(L, 70)))
    return MaskSpec(kind, L, window=rng.randint(0, 300), stride=1 if kind == KIND_SLIDING else rng.randint(2, 4))


@pytest.mark.parametrize("seed", range(40))
def test_explicit_tiles_agree_with_row_kernels_and_prepared_graphs(seed):
    import torch
    rng = random.Random(2000 + seed)
    spec = _explicit_spec(rng, seed)
    dtype = rng.choice(["f16", "f32"])
    H = rng.choice([1, 2, 4])
    sigma = rng.choice([0.3, 1.0])
    scale = rng.choice([0.125, -0.125, 0.3])
    print("case", seed, spec, dtype, "H", H, "sigma", sigma, "scale", scale, flush=True)
    L = spec.L
    Q, K, V = torch_qkv(H, L, 64, dtype, sigma, seed, "cuda:0")
    rp, ci = sga.build_mask(spec)
    nnz = int(rp[-1])
    ws = sga.alloc_workspace(L, H, 64, dtype, nnz)
    O1, l1 = sga.attention_forward(Q, K, V, rp, ci, scale, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward(Q, K, V, rp, ci, scale, path=sga.PATH_GATHER, want_lse=True)
    ws2 = sga.alloc_workspace(L, H, 64, dtype, nnz)
    ws2.fill_(0x5A)
    plan = sga.graph_prepare(rp, ci, H, 64, dtype, ws2)
    O3, l3 = sga.attention_forward_prepared(Q, K, V, rp, ci, scale, plan, ws2, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(O1, O3) and torch.equal(l1, l3)
    _agree(O1, l1, O2, l2, dtype)


@pytest.mark.parametrize("seed", range(36))
def test_implicit_nonlocal_tiles_agree_with_row_kernels(seed):
    """The implicit non-local mask (global tokens without their window): rows >= g and the g dense
    rows on the tile kernels against the per-row kernels, as a fresh call and continuing the state
    a local call left (the composition of Section V-F)."""
    import torch
    rng = random.Random(3000 + seed)
    L = rng.choice([rng.randint(1, 300), rng.randint(300, 3000), rng.randint(3000, 20000)])
    g = rng.choice([0, 1, rng.randint(1, 16), rng.randint(17, 32), rng.randint(33, 64)])
    W = rng.choice([0, rng.randint(1, 40), rng.randint(41, 200)])
    dtype = rng.choice(["f16", "f32"])
    H = rng.choice([1, 2, 3])
    d = rng.choice([64, 64, 128, 256])        # (128 and 256: one workgroup of d / 64 wavefronts per tile)
    scale = rng.choice([0.125, -0.125, 0.3]) * (64 / d) ** 0.5
    nl = MaskSpec(KIND_NONLOCAL, L, window=W, n_global=min(g, L))
    loc = MaskSpec(KIND_SLIDING, L, window=W)
    print("case", seed, nl, dtype, "H", H, "d", d, "scale", scale, flush=True)
    Q, K, V = torch_qkv(H, L, d, dtype, 0.8, seed, "cuda:0")
    ws = sga.alloc_workspace(L, H, d, dtype, -1)
    O1, l1 = sga.attention_forward_implicit(Q, K, V, nl, scale, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward_implicit(Q, K, V, nl, scale, workspace=ws, path=sga.PATH_GATHER, want_lse=True)
    torch.cuda.synchronize()
    _agree(O1, l1, O2, l2, dtype)
    # local first, then the non-local edges on the same state: both kernel families
    outs = []
    for path in (sga.PATH_TILE, sga.PATH_GATHER):
        O, lse = sga.attention_forward_implicit(Q, K, V, loc, scale, workspace=ws, path=path, want_lse=True)
        sga.attention_accumulate_implicit(Q, K, V, nl, scale, O, lse, workspace=ws, path=path)
        outs.append((O, lse))
    torch.cuda.synchronize()
    _agree(outs[0][0], outs[0][1], outs[1][0], outs[1][1], dtype, 2.0)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_implicit_nonlocal_tiles_at_length(dtype):
    """The same agreement where the g global rows span thousands of key blocks (128 ranges of 74
    blocks each) and row offsets pass 2^24."""
    import torch
    L, H, g, W = 300001, 2, 40, 77
    nl = MaskSpec(KIND_NONLOCAL, L, window=W, n_global=g)
    Q, K, V = torch_qkv(H, L, 64, dtype, 0.8, 5, "cuda:0")
    ws = sga.alloc_workspace(L, H, 64, dtype, -1)
    O1, l1 = sga.attention_forward_implicit(Q, K, V, nl, 0.125, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward_implicit(Q, K, V, nl, 0.125, workspace=ws, path=sga.PATH_GATHER, want_lse=True)
    torch.cuda.synchronize()
    _agree(O1, l1, O2, l2, dtype)
    # V = ones: every row with a neighbour returns exactly 1, the others the initial state
    ones = torch.ones_like(V)
    O3, l3 = sga.attention_forward_implicit(Q, K, ones, nl, 0.125, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    torch.cuda.synchronize()
    has = torch.isfinite(l3)
    assert torch.equal(has, torch.isfinite(l2))
    tol = 1e-6 if dtype == "f32" else 1e-3
    assert (O3[has].float() - 1.0).abs().max().item() <= tol
    assert (O3[~has].float() == 0).all()


def _scattered_mask(rng, seed, L):
    """A dense boolean mask of scattered columns drawn on the device: even or falling fill, column
    stripes, per-row fill, random blocks, or scattered columns next to dense rows, empty rows,
    a band and full columns."""
    import torch
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    u = torch.rand((L, L), generator=g, device="cuda:0")
    j = torch.arange(L, device="cuda:0")[None, :]
    i = torch.arange(L, device="cuda:0")[:, None]
    kind = rng.choice(["even", "falling", "stripes", "mixed", "rowvar", "blocks"])
    p = rng.choice([0.13, 0.2, 0.35, 0.5, 0.8, 0.97])
    if kind == "even":
        return kind, u < p
    if kind == "falling":
        return kind, u < p * (1 - j / L) ** rng.choice([1, 2, 4])
    if kind == "stripes":
        w = rng.choice([40, 333, 1024, 1500])
        return kind, (u < p) & ((j // w) % rng.choice([2, 3]) == 0)
    if kind == "rowvar":
        return kind, u < (p * ((i * 7919) % 97) / 97.0)
    if kind == "blocks":
        b = rng.choice([32, 64, 100])
        nb = (L + b - 1) // b
        ub = torch.rand((nb, nb), generator=g, device="cuda:0")
        return kind, (ub < 0.3).repeat_interleave(b, 0).repeat_interleave(b, 1)[:L, :L] & (u < max(p, 0.5))
    m = u < p
    for _ in range(rng.randint(1, 4)):
        m[rng.randrange(L)] = True
    for _ in range(rng.randint(1, 4)):
        r = rng.randrange(L)
        m[r:r + rng.randint(1, 40)] = False
    r = rng.randrange(max(1, L - 64))
    m[r:r + 64] = ((i - j).abs() <= rng.randint(0, 200))[r:r + 64]
    c = rng.randrange(L)
    m[:, c:c + rng.randint(1, 70)] = True
    return kind, m


@pytest.mark.parametrize("seed", range(30))
def test_scattered_masks_tiles_agree_with_row_kernels_and_prepared_graphs(seed):
    """Masks of scattered columns (the CSR -> tile pass builds their block words from an LDS
    bitmap once a list's first blocks show scattered columns), at lengths whose lists span up to
    nine windows of that walk, at d = 64 and 128."""
    import torch
    rng = random.Random(7000 + seed)
    L = rng.choice([rng.randint(100, 700), rng.randint(700, 3000), rng.randint(3000, 9000)])
    dtype = rng.choice(["f16", "f32"])
    H = rng.choice([1, 2, 3])
    d = rng.choice([64, 64, 128])
    kind, m = _scattered_mask(rng, seed, L)
    rp = torch.zeros(L + 1, dtype=torch.int64, device="cuda:0")
    rp[1:] = m.sum(dim=1).cumsum(0)
    ci = m.nonzero()[:, 1].to(torch.int32).contiguous()
    del m
    nnz = int(rp[-1])
    if nnz == 0:
        pytest.skip("empty mask")
    sigma = rng.choice([0.3, 1.0])
    scale = rng.choice([0.125, -0.125, 0.3]) * (64 / d) ** 0.5
    print("case", seed, kind, "L", L, dtype, "H", H, "d", d, "nnz", nnz, flush=True)
    Q, K, V = torch_qkv(H, L, d, dtype, sigma, seed, "cuda:0")
    ws = sga.alloc_workspace(L, H, d, dtype, nnz)
    O1, l1 = sga.attention_forward(Q, K, V, rp, ci, scale, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward(Q, K, V, rp, ci, scale, path=sga.PATH_GATHER, want_lse=True)
    ws2 = sga.alloc_workspace(L, H, d, dtype, nnz)
    ws2.fill_(0x5A)
    plan = sga.graph_prepare(rp, ci, H, d, dtype, ws2)
    O3, l3 = sga.attention_forward_prepared(Q, K, V, rp, ci, scale, plan, ws2, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(O1, O3) and torch.equal(l1, l3)
    _agree(O1, l1, O2, l2, dtype)


@pytest.mark.parametrize("case", range(11))
def test_d128_wide_bands_agree_with_row_kernels(case):
    """fp16, d = 128, windows wide enough and calls large enough for the kernel that gives a
    wavefront all 128 channels of its sub-tile: sliding, dilated and 2-D dilated masks, a
    negative scale, large scores, and a call that continues an earlier state."""
    import torch
    kind, L, H, kw, scale, sigma = [
        (KIND_SLIDING, 20011, 4, dict(window=333), 0.0884, 0.5),
        (KIND_SLIDING, 16384, 4, dict(window=65), -0.0884, 0.5),
        (KIND_SLIDING, 9000, 8, dict(window=9000), 0.0884, 0.3),
        (KIND_DILATED, 50000, 2, dict(window=100, stride=4), 0.0884, 1.0),
        (KIND_DILATED, 30000, 4, dict(window=2000, stride=2), 0.3, 1.0),
        (KIND_DILATED_2D, 48000, 4, dict(block=6000, stride=2), 0.0884, 0.5),
        (KIND_DILATED_2D, 40000, 6, dict(block=777, stride=1), 0.0884, 0.5),
        (KIND_SLIDING, 17000, 4, dict(window=200), 0.0884, 0.5),
        (KIND_SLIDING, 70001, 1, dict(window=16), 0.0884, 0.5),
        (KIND_DILATED, 33333, 4, dict(window=64, stride=2), 0.0884, 0.5),
        (KIND_SLIDING, 16500, 4, dict(window=0), 0.0884, 0.5),
    ][case]
    spec = MaskSpec(kind, L, **kw)
    print("case", case, spec, "H", H, flush=True)
    Q, K, V = torch_qkv(H, L, 128, "f16", sigma, 300 + case, "cuda:0")
    amp = max(1.0, sigma * sigma * abs(scale) * 11.3 * 8)
    O1, l1 = sga.attention_forward_implicit(Q, K, V, spec, scale, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward_implicit(Q, K, V, spec, scale, path=sga.PATH_GATHER, want_lse=True)
    torch.cuda.synchronize()
    _agree(O1, l1, O2, l2, "f16", amp)
    if case == 7:
        # the same window once more on the state of the first call: O unchanged, lse + ln 2
        O3, l3 = O1.clone(), l1.clone()
        sga.attention_accumulate_implicit(Q, K, V, spec, scale, O3, l3, path=sga.PATH_TILE)
        torch.cuda.synchronize()
        assert ((O3.float() - O1.float()).abs() / (1 + O1.float().abs())).max().item() <= 2 * TOL["f16"]
        assert (l3 - l1 - 0.6931472).abs().max().item() <= 2e-3


@pytest.mark.parametrize("seed", range(16))
def test_explicit_d128_tiles_agree_with_row_kernels_and_prepared_graphs(seed):
    """The explicit fp16 kernel at d = 128 (one wavefront per work item with all 128 channels) on
    the seeded masks of the d = 64 test: every mask family, multi-segment tiles (global rows,
    BigBird global blocks), ragged lengths, negative scales; prepared graphs bit for bit."""
    import torch
    rng = random.Random(5000 + seed)
    spec = _explicit_spec(rng, seed)
    H = rng.choice([1, 2, 4])
    sigma = rng.choice([0.3, 1.0])
    scale = rng.choice([0.0884, -0.0884, 0.2])
    print("case", seed, spec, "H", H, "sigma", sigma, "scale", scale, flush=True)
    L = spec.L
    Q, K, V = torch_qkv(H, L, 128, "f16", sigma, seed, "cuda:0")
    rp, ci = sga.build_mask(spec)
    nnz = int(rp[-1])
    ws = sga.alloc_workspace(L, H, 128, "f16", nnz)
    O1, l1 = sga.attention_forward(Q, K, V, rp, ci, scale, workspace=ws, path=sga.PATH_TILE, want_lse=True)
    O2, l2 = sga.attention_forward(Q, K, V, rp, ci, scale, path=sga.PATH_GATHER, want_lse=True)
    ws2 = sga.alloc_workspace(L, H, 128, "f16", nnz)
    ws2.fill_(0x5A)
    plan = sga.graph_prepare(rp, ci, H, 128, "f16", ws2)
    O3, l3 = sga.attention_forward_prepared(Q, K, V, rp, ci, scale, plan, ws2, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(O1, O3) and torch.equal(l1, l3)
    _agree(O1, l1, O2, l2, "f16", max(1.0, sigma * sigma * abs(scale) * 11.3 * 8))
    # a second call on the same state: O unchanged, lse + ln 2
    O4, l4 = O1.clone(), l1.clone()
    sga.attention_accumulate(Q, K, V, rp, ci, scale, O4, l4, workspace=ws, path=sga.PATH_TILE)
    torch.cuda.synchronize()
    fin = torch.isfinite(l1)
    assert ((O4.float() - O1.float()).abs() / (1 + O1.float().abs())).max().item() <= 2 * TOL["f16"]
    if fin.any():
        assert (l4[fin] - l1[fin] - 0.6931472).abs().max().item() <= 2e-3
