"""CPU oracle for sparse graph attention -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this.  It shares no code with the HIP library and never calls it.

What it computes (all in float64, from the stored fp32/fp16 input values):

* the attention mask A (rows = queries, columns = keys) as a dense boolean
  matrix, straight from the predicates of Section II-C;
* masked attention by its plain definition (Eq. 1 with the entries outside the
  mask set to -inf before the row softmax, Section III "Efficient Sparse
  Attention Implementations"): S = scale * Q K^T, S[~A] = -inf,
  P = softmax_rows(S), O = P V;
* the CSR image of A (Section IV-B "CSR") by enumerating the dense predicate in
  row-major order;
* a second, sequential evaluator that follows Algorithm 1 step by step
  (Initialize, Get_Neighbors, Pull, running max m, running sum l, running
  normalised O), used to pin the recurrence and the merge of partial states.

Readings of the paper fixed here (the paper is silent or ambiguous):
  - window bounds are inclusive: |i - j| <= w   (the printed 1-D predicate uses
    a strict bound; the workloads are stated with the inclusive one);
  - dilation is given as the stride s between attended keys, s = r + 1 for the
    paper's dilation factor r:  (i - j) mod s == 0  and  |i - j| <= W * s;
  - the score is scale * (Q_i . K_j) with the caller's scale (Eq. 1 has
    1/sqrt(d_k); Algorithm 1 omits it);
  - a row with no neighbour returns O_i = 0 and lse_i = -inf (Algorithm 1's
    initial state), not NaN;
  - global tokens are positions 0..g-1 and are symmetric: they attend to and
    are attended by every token;
  - the "global (non-local)" mask is the global mask (i < g or j < g) minus the
    local window |i - j| <= w, as Section IV-B states for the kernel that runs
    after a local pass on the same (O, l, m) state;
  - the 2-D dilated predicate is printed with the segment id floor(i / (L / b)) but
    the in-block index i % b; the two agree only when L = b^2.  Here a block is b
    consecutive tokens (segment id floor(i / b)), "dilation factor r" is carried as
    the stride s = r + 1, and rows whose in-block index is not a multiple of s have
    no neighbour (in LongNet other segment/dilation pairs cover them);
  - the block mask is defined at block level: global blocks 0..G-1 (symmetric),
    a window of +-wb blocks, and R distinct random key blocks per non-global
    query block, drawn without replacement from blocks not already attended,
    by the counter-based generator in `bigbird_block_set`: query block b owns the
    stream key mix64(seed + GOLD*(b+1)); attempt a = 0, 1, 2, ... proposes key block
    mix64(key + GOLD*(a+1)) mod nb and is rejected if that block is already attended.

Parity pins for every function here are in tests/test_oracle_*.py.
"""
import math

import numpy as np

from sga_inputs.masks import (MaskSpec, KIND_SLIDING, KIND_DILATED,
                              KIND_GLOBAL_LOCAL, KIND_BIGBIRD, KIND_NONLOCAL,
                              KIND_DILATED_2D)

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15


# --------------------------------------------------------------------------
# Block selection for the BigBird-style mask
# --------------------------------------------------------------------------
def mix64(z: int) -> int:
    """splitmix64 output function (Steele, Lea, Flood 2014) on a 64-bit word."""
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def bigbird_block_set(spec: MaskSpec, b: int):
    """Sorted list of key blocks attended by query block b."""
    B = spec.block
    nb = spec.L // B
    G, wb, R = spec.n_global_blocks, spec.window_blocks, spec.n_random_blocks
    if b < G:
        return list(range(nb))
    chosen = set(range(G))
    for kb in range(b - wb, b + wb + 1):
        if 0 <= kb < nb:
            chosen.add(kb)
    stream = mix64(spec.seed + _GOLD * (b + 1))
    a = 0
    picked = 0
    while picked < R:
        cand = mix64(stream + _GOLD * (a + 1)) % nb
        a += 1
        if cand not in chosen:
            chosen.add(cand)
            picked += 1
    return sorted(chosen)


# --------------------------------------------------------------------------
# Dense predicates (Section II-C)
# --------------------------------------------------------------------------
def mask_rows(spec: MaskSpec, rows) -> np.ndarray:
    """Boolean [len(rows), L]: A[i, j] for the given query rows, all keys j."""
    L = spec.L
    i = np.asarray(rows, dtype=np.int64).reshape(-1, 1)
    j = np.arange(L, dtype=np.int64).reshape(1, -1)
    if spec.kind == KIND_SLIDING:
        return np.abs(i - j) <= spec.window
    if spec.kind == KIND_DILATED:
        diff = i - j
        return (np.abs(diff) <= spec.window * spec.stride) & (diff % spec.stride == 0)
    if spec.kind == KIND_GLOBAL_LOCAL:
        g = spec.n_global
        return (np.abs(i - j) <= spec.window) | (i < g) | (j < g)
    if spec.kind == KIND_NONLOCAL:
        # the global mask with the local mask taken out of it (Section IV-B, "Global
        # (non-local)"), so that a local pass and this pass never visit an edge twice
        g = spec.n_global
        return ((i < g) | (j < g)) & ~(np.abs(i - j) <= spec.window)
    if spec.kind == KIND_DILATED_2D:
        # blocks of b x b tokens on the diagonal; inside a block every stride-th row and
        # every stride-th column, counted from the block's first token, is kept
        b, s = spec.block, spec.stride
        return (i // b == j // b) & ((i % b) % s == 0) & ((j % b) % s == 0)
    if spec.kind == KIND_BIGBIRD:
        B = spec.block
        if L % B != 0:
            raise ValueError("block mask needs L divisible by the block size")
        nb = L // B
        out = np.zeros((i.shape[0], L), dtype=bool)
        cache = {}
        for r, ii in enumerate(i[:, 0]):
            b = int(ii) // B
            if b not in cache:
                blk = np.zeros(nb, dtype=bool)
                blk[bigbird_block_set(spec, b)] = True
                cache[b] = np.repeat(blk, B)
            out[r] = cache[b]
        return out
    raise ValueError(f"unknown mask kind {spec.kind}")


def dense_mask(spec: MaskSpec) -> np.ndarray:
    """The full L x L boolean mask."""
    return mask_rows(spec, np.arange(spec.L))


def csr_from_dense(mask: np.ndarray):
    """CSR (row offsets int64 [L+1], sorted column indices int32 [nnz]) of a 0/1 matrix."""
    L = mask.shape[0]
    deg = mask.sum(axis=1, dtype=np.int64)
    row_ptr = np.zeros(L + 1, dtype=np.int64)
    np.cumsum(deg, out=row_ptr[1:])
    _, cols = np.nonzero(mask)          # row-major order => sorted within a row
    return row_ptr, cols.astype(np.int32)


def sparsity_factor(mask: np.ndarray) -> float:
    """S_f = NNZ / TE  (Section II-D)."""
    return float(mask.sum(dtype=np.int64)) / float(mask.size)


# --------------------------------------------------------------------------
# Masked attention by definition
# --------------------------------------------------------------------------
def attention_dense(Q, K, V, mask, scale):
    """One head.  Q,K,V: [L, d] (any float dtype); mask: [Lq, L] boolean for the
    first Lq = mask.shape[0] query rows given in Q.  Returns (O [Lq, d], lse [Lq])
    in float64.  lse_i = log sum_j exp(S_ij) over the row's neighbours."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S = scale * (Q @ K.T)
    S = np.where(mask, S, -np.inf)
    M = S.max(axis=1)
    empty = ~np.isfinite(M)
    Msafe = np.where(empty, 0.0, M)
    P = np.exp(S - Msafe[:, None])
    Z = P.sum(axis=1)
    Zsafe = np.where(empty, 1.0, Z)
    O = (P / Zsafe[:, None]) @ V
    O[empty] = 0.0
    with np.errstate(divide="ignore"):
        lse = np.where(empty, -np.inf, Msafe + np.log(Zsafe))
    return O, lse


def attention_weights(Q, K, mask, scale):
    """Row-softmax weights P [Lq, L] (float64) of the masked scores."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    S = np.where(mask, scale * (Q @ K.T), -np.inf)
    M = S.max(axis=1, keepdims=True)
    M = np.where(np.isfinite(M), M, 0.0)
    P = np.exp(S - M)
    Z = P.sum(axis=1, keepdims=True)
    return P / np.where(Z == 0.0, 1.0, Z)


def attention_masked(Q, K, V, spec: MaskSpec, scale, rows=None):
    """All heads.  Q,K,V: [H, L, d].  rows: optional list of query rows (default
    all).  Returns (O [H, n, d], lse [H, n]) in float64."""
    H, L, d = Q.shape
    if rows is None:
        rows = np.arange(L)
    rows = np.asarray(rows, dtype=np.int64)
    mask = mask_rows(spec, rows)
    O = np.zeros((H, len(rows), V.shape[2]))
    lse = np.zeros((H, len(rows)))
    for h in range(H):
        O[h], lse[h] = attention_dense(Q[h][rows], K[h], V[h], mask, scale)
    return O, lse


# --------------------------------------------------------------------------
# Algorithm 1, followed step by step (sequential, float64)
# --------------------------------------------------------------------------
def algorithm1_row(q, K, V, neighbours, scale, state=None):
    """One query row through Algorithm 1's inner loop.

    state: optional (O_i, l_i, m_i) to continue from (the sequential composition
    of Section V-F runs several kernels on one shared state); default is the
    Initialize step: O_i = 0, l_i = 0, m_i = -inf.
    Returns (O_i, l_i, m_i) with O_i normalised after every neighbour, as printed.
    """
    d = len(q)
    if state is None:
        O = np.zeros(d)
        l = 0.0
        m = -math.inf
    else:
        O, l, m = np.array(state[0], dtype=np.float64), float(state[1]), float(state[2])
    q = np.asarray(q, dtype=np.float64)
    for j in neighbours:
        k = np.asarray(K[j], dtype=np.float64)          # Pull(K_j)
        W = scale * float(q @ k)
        m_new = max(m, W)
        carry = l * math.exp(m - m_new) if l != 0.0 else 0.0
        e = math.exp(W - m_new)
        l_new = carry + e
        v = np.asarray(V[j], dtype=np.float64)          # Pull(V_j)
        O = (carry * O + e * v) / l_new
        l, m = l_new, m_new
    return O, l, m


def algorithm1(Q, K, V, neighbour_lists, scale):
    """One head; neighbour_lists[i] is the iterable Get_Neighbors returns for row i."""
    L = len(neighbour_lists)
    d = Q.shape[1]
    O = np.zeros((L, d))
    l = np.zeros(L)
    m = np.full(L, -np.inf)
    for i in range(L):
        O[i], l[i], m[i] = algorithm1_row(Q[i], K, V, neighbour_lists[i], scale)
    return O, l, m


def partial_state(q, K, V, neighbours, scale):
    """Un-normalised partial (m, l, acc) of one chunk of a row's neighbours:
    m = max score, l = sum exp(s - m), acc = sum exp(s - m) V_j."""
    q = np.asarray(q, dtype=np.float64)
    nb = list(neighbours)
    d = len(q)
    if not nb:
        return -math.inf, 0.0, np.zeros(d)
    s = scale * (np.asarray(K, dtype=np.float64)[nb] @ q)
    m = float(s.max())
    p = np.exp(s - m)
    return m, float(p.sum()), p @ np.asarray(V, dtype=np.float64)[nb]


def merge_partials(parts):
    """Combine partial states of disjoint neighbour chunks: the running-max /
    running-sum update of Algorithm 1 applied to groups instead of single keys.
    Returns the normalised row O_i and its lse."""
    M = max(p[0] for p in parts)
    d = len(parts[0][2])
    if not math.isfinite(M):
        return np.zeros(d), -math.inf
    l = 0.0
    acc = np.zeros(d)
    for m, lp, a in parts:
        if lp == 0.0:
            continue
        w = math.exp(m - M)
        l += lp * w
        acc += a * w
    return acc / l, M + math.log(l)


# --------------------------------------------------------------------------
# Closed-form edge counts (S_f = NNZ / L^2, Section II-D) -- used as pins
# --------------------------------------------------------------------------
def nnz_sliding(L, w):
    """|i-j| <= w, valid for L >= 2w+1."""
    return L * (2 * w + 1) - w * (w + 1)


def nnz_dilated(L, W, s):
    """j = i + s*k, |k| <= W, valid for L >= 2*W*s+1."""
    return L * (2 * W + 1) - s * W * (W + 1)


def nnz_global_local(L, w, g):
    """|i-j| <= w or i < g or j < g, valid for g <= w+1 and L >= 2w+1+g."""
    return L * (2 * w + 1) - w * (w + 1) + 2 * g * L - g * g - g * (2 * w + 1)


def nnz_nonlocal(L, w, g):
    """(i < g or j < g) and |i-j| > w: the global+local count minus the window count."""
    return nnz_global_local(L, w, g) - nnz_sliding(L, w)


def nnz_dilated_2d(L, b, s):
    """Blocks of b tokens, every s-th row and column: sum over blocks of ceil(len/s)^2."""
    full, rest = divmod(L, b)
    return full * (-(-b // s)) ** 2 + (-(-rest // s)) ** 2


def nnz_bigbird_g2_w1(L, B, R):
    """Block mask with 2 global blocks, +-1 window, R random blocks."""
    nb = L // B
    G = 2
    return B * B * (G * nb + (nb - G) * (3 + G + R) - 2)
