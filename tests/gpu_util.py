"""Helpers for the GPU parity tests: move seeded inputs to the device, run the HIP path
through the C ABI binding, and evaluate the CPU oracle on the same stored values."""
import numpy as np

from sga_inputs import numpy_qkv
from oracle import reference as R
from oracle import rowscan as C

TOL = {"f32": 1e-5, "f16": 2e-3}   # max-abs-error bars: fp32, and fp16 storage with fp32 accumulate
# lse = m + ln l.  fp32 storage: fp32 rounding of a sum of up to 2^16 terms.  fp16 storage: l is the
# sum of the softmax numerators as the matrix cores use them, each rounded to fp16 (to nearest:
# relative error at most 2^-11 = 4.9e-4, reached when one neighbour dominates the row), so ln l is
# within 4.9e-4 of the exact value plus the fp32 noise of the other bar.
LSE_TOL = {"f32": 1e-4, "f16": 6e-4}


def to_device(*arrays):
    import torch
    return tuple(torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in arrays)


def small_inputs(wl, dist="normal"):
    return numpy_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, dist=dist)


def oracle_full(wl, Q, K, V):
    """Dense oracle on all rows (small L only)."""
    return R.attention_masked(Q, K, V, wl.mask, wl.scale)


def max_err(a, b):
    return float(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)).max())


def sample_rows(L, seed, n_random, edge=300, tiles=(32, 64, 128, 256), n_tile_idx=16):
    """Row sample for large problems: both ends, rows around tile boundaries, random rows."""
    rng = np.random.default_rng(seed)
    rows = [np.arange(0, min(edge, L)), np.arange(max(0, L - edge), L)]
    for T in tiles:
        nt = max(1, L // T)
        t = rng.integers(1, max(2, nt), size=n_tile_idx)
        rows.append(np.clip(t * T - 1, 0, L - 1))
        rows.append(np.clip(t * T, 0, L - 1))
    rows.append(rng.integers(0, L, size=n_random))
    return np.unique(np.concatenate(rows)).astype(np.int64)


def neighbor_lists(spec, rows):
    """Neighbour lists of `rows` from the oracle's predicate scan over all L keys of each row
    (one scan per row, rows spread over the host cores)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=max(1, C.num_threads())) as pool:
        return list(pool.map(lambda i: C.row_neighbors(spec, int(i)), rows))


def oracle_rows_gathered(spec, scale, rows, fetch_q, fetch_kv):
    """Row-sampled oracle for problems whose K/V do not fit on the host: neighbour lists by
    scanning the predicate over all keys, K/V rows fetched from the device by index only.
    fetch_q(rows)->[n,d] float32, fetch_kv(idx)->(K[idx], V[idx]) float32."""
    q = fetch_q(rows)
    out = np.zeros((len(rows), q.shape[1]))
    lse = np.zeros(len(rows))
    edges = 0
    for r, i in enumerate(rows):
        nb = C.row_neighbors(spec, int(i))
        Kg, Vg = fetch_kv(nb)
        out[r], lse[r] = C.attend_gathered(q[r], Kg, Vg, scale)
        edges += len(nb)
    return out, lse, edges
