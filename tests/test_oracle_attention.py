"""Pins for the oracle's masked attention (CPU only).

Nothing here re-types the oracle's formula.  The pins are:
  P1  softmax weights of a row sum to 1  (V = ones => O = ones);
  P2  a full mask reproduces dense attention computed by library routines
      (scipy softmax + matmul, and torch's scaled_dot_product_attention, the
      comparator of the verification protocol in Section V-A);
  P3  a single-neighbour row returns exactly that V row;
  P4  Q = 0 gives uniform weights: O_i is the mean of the neighbours' V rows,
      a moving average computed independently with prefix sums;
  P5  V[j] = j with Q = 0 returns the (clipped) window centre;
  P6  V = identity returns the weight vector, checked entry by entry with
      math.exp on a tiny problem;
  P7  adding one vector to every key leaves O unchanged; scores of magnitude
      ~100 give no inf/NaN;
  P8  the sequential evaluator that follows Algorithm 1 equals the two-pass
      definition, and merging partial (m, l, acc) states of any partition of a
      row's neighbours equals the unsplit row;
  P12 the verification protocol of Section V-A (L=256, d=32, U[0,1) inputs,
      Bernoulli masks of several sparsity factors, allclose atol 1e-8 rtol 1e-5,
      NaN == NaN) against torch's masked SDPA;
  P13 permuting a row's neighbour order changes nothing.
  Planted mistakes: a transposed operand, a dropped scale, a sign flip and an
  off-by-one window each break at least one pin (test_planted_mistakes_fail).
"""
import math

import numpy as np
import pytest
import scipy.special

from sga_inputs import (KIND_NONLOCAL, MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_GLOBAL_LOCAL,
                        KIND_BIGBIRD, numpy_qkv)
from oracle import reference as R


def _qkv(L, d, seed=0, dist="normal", dtype="f32", sigma=1.0, H=1):
    Q, K, V = numpy_qkv(H, L, d, dtype, sigma, seed, dist=dist)
    return Q, K, V


SPECS = [
    MaskSpec(KIND_SLIDING, 150, window=6),
    MaskSpec(KIND_DILATED, 150, window=5, stride=2),
    MaskSpec(KIND_GLOBAL_LOCAL, 150, window=7, n_global=3),
    MaskSpec(KIND_BIGBIRD, 160, block=8, window_blocks=1, n_global_blocks=2,
             n_random_blocks=3, seed=5),
]


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.name)
def test_p1_weights_sum_to_one(spec):
    Q, K, V = _qkv(spec.L, 16, seed=3)
    V = np.ones_like(V)
    O, lse = R.attention_masked(Q, K, V, spec, 0.25)
    assert np.abs(O - 1.0).max() < 1e-14
    P = R.attention_weights(Q[0], K[0], R.dense_mask(spec), 0.25)
    assert np.abs(P.sum(axis=1) - 1.0).max() < 1e-14
    assert (P[~R.dense_mask(spec)] == 0).all()


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.name)
def test_weights_match_library_softmax_row_by_row(spec):
    """attention_weights at value level: each row's weights equal scipy's softmax over that
    row's neighbours only (entry by entry), and weights @ V equals the output of the definition.
    A dropped or misplaced scale, a transposed operand or a wrong normaliser fails here."""
    Q, K, V = _qkv(spec.L, 16, seed=23)
    scale = 0.37
    A = R.dense_mask(spec)
    P = R.attention_weights(Q[0], K[0], A, scale)
    q, k, v = (x[0].astype(np.float64) for x in (Q, K, V))
    for i in range(spec.L):
        nb = np.flatnonzero(A[i])
        want = scipy.special.softmax(np.array([scale * float(q[i] @ k[j]) for j in nb]))
        assert np.abs(P[i, nb] - want).max() < 1e-14
    O, _ = R.attention_dense(Q[0], K[0], V[0], A, scale)
    assert np.abs(P @ v - O).max() < 1e-13


def test_p2_full_mask_is_dense_attention_scipy():
    L, d = 96, 24
    Q, K, V = _qkv(L, d, seed=11)
    scale = 1.0 / math.sqrt(d)
    full = np.ones((L, L), dtype=bool)
    O, lse = R.attention_dense(Q[0], K[0], V[0], full, scale)
    q, k, v = (x[0].astype(np.float64) for x in (Q, K, V))
    want = scipy.special.softmax(scale * (q @ k.T), axis=1) @ v
    assert np.abs(O - want).max() < 1e-13
    want_lse = scipy.special.logsumexp(scale * (q @ k.T), axis=1)
    assert np.abs(lse - want_lse).max() < 1e-12


def test_p2_full_window_equals_dense():
    # a window at least as wide as the sequence is the full mask
    L, d = 70, 8
    Q, K, V = _qkv(L, d, seed=2)
    spec = MaskSpec(KIND_SLIDING, L, window=L)
    O, _ = R.attention_masked(Q, K, V, spec, 0.3)
    q, k, v = (x[0].astype(np.float64) for x in (Q, K, V))
    want = scipy.special.softmax(0.3 * (q @ k.T), axis=1) @ v
    assert np.abs(O[0] - want).max() < 1e-13


@pytest.mark.parametrize("sf", [1.0, 0.5, 0.1, 0.01])
def test_p12_paper_verification_protocol_vs_torch_sdpa(sf):
    torch = pytest.importorskip("torch")
    L, d = 256, 32
    Q, K, V = _qkv(L, d, seed=21, dist="uniform")
    rng = np.random.default_rng(99)
    mask = rng.random((L, L)) < sf
    scale = 1.0 / math.sqrt(d)
    O, _ = R.attention_dense(Q[0], K[0], V[0], mask, scale)
    tq, tk, tv = (torch.from_numpy(x[0].astype(np.float64))[None, None] for x in (Q, K, V))
    want = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, attn_mask=torch.from_numpy(mask)[None, None], scale=scale)[0, 0].numpy()
    # rows with no neighbour: the oracle returns 0 (Algorithm 1's initial state);
    # SDPA yields NaN or 0 depending on the torch version (the protocol treats NaNs as equal)
    empty = ~mask.any(axis=1)
    if sf <= 0.01:
        assert empty.any()
    assert (np.isnan(want[empty]) | (want[empty] == 0)).all() and (O[empty] == 0).all()
    ok = ~empty
    assert np.allclose(O[ok], want[ok], atol=1e-8, rtol=1e-5)


def test_p3_single_neighbour_returns_that_row_exactly():
    L, d = 40, 16
    Q, K, V = _qkv(L, d, seed=8)
    mask = np.zeros((L, L), dtype=bool)
    perm = np.random.default_rng(1).permutation(L)
    mask[np.arange(L), perm] = True
    O, lse = R.attention_dense(Q[0], K[0], V[0], mask, 0.5)
    assert (O == V[0][perm].astype(np.float64)).all()
    # window 0 is the identity mask
    O2, _ = R.attention_masked(Q, K, V, MaskSpec(KIND_SLIDING, L, window=0), 0.5)
    assert (O2[0] == V[0].astype(np.float64)).all()


def _moving_average(V, w, s):
    """Mean of V[j] over j = i + s*k, |k| <= w, clipped to [0, L): prefix sums per residue class."""
    L, d = V.shape
    out = np.zeros((L, d))
    for p in range(s):
        idx = np.arange(p, L, s)
        cs = np.vstack([np.zeros((1, d)), np.cumsum(V[idx].astype(np.float64), axis=0)])
        n = len(idx)
        u = np.arange(n)
        lo = np.maximum(0, u - w)
        hi = np.minimum(n - 1, u + w)
        out[idx] = (cs[hi + 1] - cs[lo]) / (hi - lo + 1)[:, None]
    return out


@pytest.mark.parametrize("spec", SPECS[:2], ids=lambda s: s.name)
def test_p4_zero_query_gives_moving_average(spec):
    Q, K, V = _qkv(spec.L, 12, seed=4)
    Q = np.zeros_like(Q)
    O, lse = R.attention_masked(Q, K, V, spec, 0.125)
    want = _moving_average(V[0], spec.window, spec.stride)
    assert np.abs(O[0] - want).max() < 1e-13
    deg = R.dense_mask(spec).sum(axis=1)
    assert np.abs(lse[0] - np.log(deg)).max() < 1e-13


def test_p5_position_valued_v_returns_window_centre():
    L, w = 90, 7
    spec = MaskSpec(KIND_SLIDING, L, window=w)
    Q = np.zeros((1, L, 4), dtype=np.float32)
    K = np.ones((1, L, 4), dtype=np.float32)
    V = np.repeat(np.arange(L, dtype=np.float32)[None, :, None], 4, axis=2)
    O, _ = R.attention_masked(Q, K, V, spec, 1.0)
    i = np.arange(L)
    lo, hi = np.maximum(0, i - w), np.minimum(L - 1, i + w)
    assert np.abs(O[0][:, 0] - (lo + hi) / 2.0).max() < 1e-12
    assert np.abs(O[0][w:L - w, 0] - i[w:L - w]).max() < 1e-12


def test_p6_identity_v_returns_weights_entrywise():
    L = 12
    spec = MaskSpec(KIND_GLOBAL_LOCAL, L, window=2, n_global=1)
    Q, K, _ = _qkv(L, 5, seed=6)
    V = np.eye(L, dtype=np.float32)[None]
    O, _ = R.attention_masked(Q, K, V, spec, 0.7)
    for i in range(L):
        nb = [j for j in range(L) if abs(i - j) <= 2 or i < 1 or j < 1]
        s = [0.7 * sum(float(Q[0, i, c]) * float(K[0, j, c]) for c in range(5)) for j in nb]
        z = sum(math.exp(x) for x in s)
        for j in range(L):
            want = math.exp(s[nb.index(j)]) / z if j in nb else 0.0
            assert abs(O[0, i, j] - want) < 1e-14


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.name)
def test_p7_shift_invariance_and_large_scores(spec):
    d = 16
    Q, K, V = _qkv(spec.L, d, seed=9, sigma=1.0)
    t = np.random.default_rng(5).standard_normal(d).astype(np.float32) * 3
    O1, _ = R.attention_masked(Q, K, V, spec, 0.25)
    O2, _ = R.attention_masked(Q, (K.astype(np.float64) + t), V, spec, 0.25)
    assert np.abs(O1 - O2).max() < 1e-11
    Qb = Q * 30.0                      # scores of magnitude ~100
    O3, lse3 = R.attention_masked(Qb, K, V, spec, 0.25)
    assert np.isfinite(O3).all() and np.isfinite(lse3).all()
    assert np.abs(O3).max() <= np.abs(V).max() + 1e-12


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.name)
def test_p8_algorithm1_equals_definition(spec):
    d = 8
    Q, K, V = _qkv(spec.L, d, seed=12)
    mask = R.dense_mask(spec)
    nbrs = [list(np.nonzero(mask[i])[0]) for i in range(spec.L)]
    O_seq, l, m = R.algorithm1(Q[0], K[0], V[0], nbrs, 0.35)
    O_def, lse = R.attention_dense(Q[0], K[0], V[0], mask, 0.35)
    assert np.abs(O_seq - O_def).max() < 1e-12
    assert np.abs((m + np.log(l)) - lse).max() < 1e-12


def test_p8_merge_of_any_partition_equals_unsplit():
    L, d = 300, 8
    Q, K, V = _qkv(L, d, seed=13)
    rng = np.random.default_rng(3)
    full = np.ones((1, L), dtype=bool)
    O_def, lse = R.attention_dense(Q[0][:1], K[0], V[0], full, 0.4)
    for parts in (2, 5, 64):
        cuts = np.sort(rng.choice(np.arange(1, L), size=parts - 1, replace=False))
        chunks = np.split(rng.permutation(L), cuts)
        st = [R.partial_state(Q[0][0], K[0], V[0], c, 0.4) for c in chunks]
        st.append(R.partial_state(Q[0][0], K[0], V[0], [], 0.4))     # an empty chunk
        O, ls = R.merge_partials(st)
        assert np.abs(O - O_def[0]).max() < 1e-13
        assert abs(ls - lse[0]) < 1e-12
    # continuing Algorithm 1 from a saved state (sequential composition, Section V-F)
    a, b = list(range(0, 120)), list(range(120, L))
    s1 = R.algorithm1_row(Q[0][0], K[0], V[0], a, 0.4)
    s2 = R.algorithm1_row(Q[0][0], K[0], V[0], b, 0.4, state=s1)
    assert np.abs(s2[0] - O_def[0]).max() < 1e-13


def test_sequential_composition_local_then_nonlocal():
    """Section V-F runs a local kernel and then the global (non-local) kernel on one shared
    (O, l, m) state; because the two masks partition the global+local mask, the result is
    the single-mask result."""
    L, d, w, g = 90, 8, 6, 4
    Q, K, V = _qkv(L, d, seed=21)
    loc = R.dense_mask(MaskSpec(KIND_SLIDING, L, window=w))
    nl = R.dense_mask(MaskSpec(KIND_NONLOCAL, L, window=w, n_global=g))
    O_def, lse = R.attention_masked(Q, K, V, MaskSpec(KIND_GLOBAL_LOCAL, L, window=w, n_global=g), 0.3)
    for i in range(L):
        st = R.algorithm1_row(Q[0][i], K[0], V[0], np.nonzero(loc[i])[0], 0.3)
        st = R.algorithm1_row(Q[0][i], K[0], V[0], np.nonzero(nl[i])[0], 0.3, state=st)
        assert np.abs(st[0] - O_def[0][i]).max() < 1e-13
        assert abs(st[2] + math.log(st[1]) - lse[0][i]) < 1e-12


def test_p13_neighbour_order_does_not_matter():
    spec = SPECS[2]
    Q, K, V = _qkv(spec.L, 8, seed=14)
    mask = R.dense_mask(spec)
    rng = np.random.default_rng(0)
    nbrs = [list(rng.permutation(np.nonzero(mask[i])[0])) for i in range(spec.L)]
    O_seq, _, _ = R.algorithm1(Q[0], K[0], V[0], nbrs, 0.35)
    O_def, _ = R.attention_dense(Q[0], K[0], V[0], mask, 0.35)
    assert np.abs(O_seq - O_def).max() < 1e-12


def test_empty_row_reading():
    L, d = 10, 4
    Q, K, V = _qkv(L, d, seed=1)
    mask = np.zeros((L, L), dtype=bool)
    mask[3, 4] = True
    O, lse = R.attention_dense(Q[0], K[0], V[0], mask, 1.0)
    assert (O[0] == 0).all() and lse[0] == -np.inf
    assert (O[3] == V[0][4]).all()
    O1, l1, m1 = R.algorithm1_row(Q[0][0], K[0], V[0], [], 1.0)
    assert (O1 == 0).all() and l1 == 0 and m1 == -math.inf


def test_fp16_inputs_are_taken_as_stored():
    L, d = 64, 8
    Q, K, V = _qkv(L, d, seed=3, dtype="f16", sigma=0.5)
    spec = MaskSpec(KIND_SLIDING, L, window=4)
    O16, _ = R.attention_masked(Q, K, V, spec, 0.3)
    O32, _ = R.attention_masked(Q.astype(np.float32), K.astype(np.float32),
                                V.astype(np.float32), spec, 0.3)
    assert (O16 == O32).all()


# ---- planted mistakes: each must break at least one pin ---------------------
def _pins(att):
    """Run a reduced pin set against attention function att(Q,K,V,mask,scale)->O."""
    failures = []
    L, d = 48, 48      # square so that a transposed operand still has a valid shape
    Q, K, V = _qkv(L, d, seed=30)
    q, k, v = (x[0].astype(np.float64) for x in (Q, K, V))
    full = np.ones((L, L), dtype=bool)
    want = scipy.special.softmax(0.2 * (q @ k.T), axis=1) @ v
    if np.abs(att(q, k, v, full, 0.2) - want).max() > 1e-10:
        failures.append("P2")
    spec = MaskSpec(KIND_SLIDING, L, window=3)
    m = R.dense_mask(spec)
    if np.abs(att(np.zeros_like(q), k, v, m, 0.2) - _moving_average(v, 3, 1)).max() > 1e-10:
        failures.append("P4")
    if np.abs(att(q, k, np.ones_like(v), m, 0.2) - 1).max() > 1e-10:
        failures.append("P1")
    return failures


def test_planted_mistakes_fail():
    good = lambda q, k, v, m, s: R.attention_dense(q, k, v, m, s)[0]
    assert _pins(good) == []

    def transposed(q, k, v, m, s):
        S = np.where(m, s * (k @ q.T), -np.inf)       # K Q^T instead of Q K^T
        P = np.exp(S - S.max(1, keepdims=True))
        return (P / P.sum(1, keepdims=True)) @ v

    def no_scale(q, k, v, m, s):
        return R.attention_dense(q, k, v, m, 1.0)[0]

    def sign(q, k, v, m, s):
        return R.attention_dense(q, k, v, m, -s)[0]

    def unnormalised(q, k, v, m, s):
        S = np.where(m, s * (q @ k.T), -np.inf)
        return np.exp(S - S.max(1, keepdims=True)) @ v

    def off_by_one(q, k, v, m, s):
        m2 = m.copy()
        if not m.all():
            m2 = m & ~np.eye(len(m), k=3, dtype=bool)   # drops the last key of each window
        return R.attention_dense(q, k, v, m2, s)[0]

    for bad in (transposed, no_scale, sign, unnormalised, off_by_one):
        assert _pins(bad) != [], bad.__name__
