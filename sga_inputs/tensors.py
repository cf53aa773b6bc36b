"""Seeded Q/K/V generators.

Small problems are drawn with NumPy on the host (bit-reproducible anywhere) and
large ones with torch on the device in fixed-size chunks, so the stream of
values does not depend on how much memory happens to be free.  Values are cast
to the storage type here; both the oracle and the HIP path consume the *cast*
values.
"""
import numpy as np

DTYPE_F32 = "f32"
DTYPE_F16 = "f16"

_NP_DTYPE = {DTYPE_F32: np.float32, DTYPE_F16: np.float16}

# rows per device-side generation chunk (fixed: part of the recipe)
_CHUNK_ROWS = 1 << 22


def numpy_qkv(H, L, d, dtype, sigma, seed, dist="normal"):
    """Return (Q, K, V) as C-contiguous [H, L, d] arrays of the storage dtype.

    dist="normal": sigma * N(0, 1); dist="uniform": U[0, 1) (the distribution
    of the verification protocol in Section V-A).  Tensor t uses seed + t.
    """
    out = []
    for t in range(3):
        rng = np.random.default_rng(seed + t)
        if dist == "normal":
            x = rng.standard_normal((H, L, d)) * sigma
        elif dist == "uniform":
            x = rng.random((H, L, d))
        else:
            raise ValueError(dist)
        out.append(np.ascontiguousarray(x.astype(_NP_DTYPE[dtype])))
    return tuple(out)


def torch_qkv(H, L, d, dtype, sigma, seed, device):
    """Return (Q, K, V) as contiguous [H, L, d] torch tensors on `device`.

    Each tensor is filled chunk by chunk (fixed chunk of rows of the flattened
    [H*L, d] view) from a generator seeded with seed + t, in fp32, scaled by
    sigma and cast to the storage dtype.
    """
    import torch
    tdt = {DTYPE_F32: torch.float32, DTYPE_F16: torch.float16}[dtype]
    out = []
    rows = H * L
    for t in range(3):
        g = torch.Generator(device=device)
        g.manual_seed(seed + t)
        x = torch.empty((rows, d), dtype=tdt, device=device)
        for r0 in range(0, rows, _CHUNK_ROWS):
            r1 = min(rows, r0 + _CHUNK_ROWS)
            c = torch.randn((r1 - r0, d), generator=g, device=device,
                            dtype=torch.float32)
            if sigma != 1.0:
                c.mul_(sigma)
            x[r0:r1].copy_(c)
        out.append(x.view(H, L, d))
    return tuple(out)


def torch_random_csr(spec, device):
    """CSR (row_ptr int64 [L+1], col_idx int32 [nnz]) of a RandomMaskSpec on `device`: the mask
    is drawn row block by row block (fixed blocks of 2048 rows: part of the recipe) as
    rand(rows, L) < density from a generator seeded with spec.seed."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(spec.seed)
    L = spec.L
    counts, cols = [], []
    for r0 in range(0, L, 2048):
        r1 = min(L, r0 + 2048)
        dense = torch.rand((r1 - r0, L), generator=g, device=device) < spec.density
        counts.append(dense.sum(dim=1))
        cols.append(dense.nonzero()[:, 1].to(torch.int32))
        del dense
    row_ptr = torch.zeros(L + 1, dtype=torch.int64, device=device)
    row_ptr[1:] = torch.cat(counts).cumsum(0)
    col_idx = torch.cat(cols).contiguous()
    return row_ptr, col_idx
