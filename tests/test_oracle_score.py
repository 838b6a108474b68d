"""Pins for the oracle's Global / Local accumulated attention scores (Sec. 3.2, Eq. 1).

None of these re-types the oracle's loop: they check it against the dense "three-step"
computation (App. A: QK^T, softmax, reduce-sum) done with library routines, against closed
forms, and against invariants a dropped term / wrong index / transposed operand would break.
"""
import numpy as np
import pytest
from scipy.special import softmax

import ems_inputs
from oracle import ems_ref
from oracle.ems_ref import RefParams


def three_step(q, k, window, scale=None):
    """Dense N x N route: matmul, masked softmax (scipy), column sums.  q [Hq,N,D]."""
    Hq, N, D = q.shape
    Hkv = k.shape[0]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    glo = np.zeros((Hkv, N))
    loc = np.zeros((Hkv, N))
    mask = np.triu(np.ones((N, N), bool), 1)
    for h in range(Hq):
        s = (q[h].astype(np.float64) @ k[h // G].astype(np.float64).T) * scale
        s[mask] = -np.inf
        a = softmax(s, axis=1)
        glo[h // G] += a.sum(axis=0)
        loc[h // G] += a[N - window:].sum(axis=0)
    return glo, loc


@pytest.mark.parametrize("hq,hkv,n,d,w", [(2, 2, 64, 16, 8), (4, 2, 97, 32, 13),
                                          (8, 2, 128, 64, 32), (3, 1, 33, 8, 1)])
def test_matches_three_step(hq, hkv, n, d, w):
    inp = ems_inputs.small(2, hq, hkv, d, n, seed=n)
    q, k = inp.f32("q"), inp.f32("k")
    p = RefParams(2, hq, hkv, d, n, w)
    glo, loc, lse = ems_ref.score(p, q, k, want_lse=True)
    for b in range(2):
        g2, l2 = three_step(q[b], k[b], w)
        np.testing.assert_allclose(glo[b], g2, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(loc[b], l2, rtol=1e-12, atol=1e-14)
    # lse against scipy's logsumexp of the masked logits, one head
    from scipy.special import logsumexp
    s = (q[0, 0].astype(np.float64) @ k[0, 0].astype(np.float64).T) / np.sqrt(d)
    s[np.triu(np.ones((n, n), bool), 1)] = -np.inf
    np.testing.assert_allclose(lse[0, 0], logsumexp(s, axis=1), rtol=1e-12)


def test_custom_scale_is_used():
    inp = ems_inputs.small(1, 2, 2, 16, 48, seed=5)
    q, k = inp.f32("q"), inp.f32("k")
    p = RefParams(1, 2, 2, 16, 48, 8, softmax_scale=0.37)
    glo, loc = ems_ref.score(p, q, k)
    g2, l2 = three_step(q[0], k[0], 8, scale=0.37)
    np.testing.assert_allclose(glo[0], g2, rtol=1e-12)
    np.testing.assert_allclose(loc[0], l2, rtol=1e-12)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_row_sum_invariant(hq, hkv):
    """Every causal softmax row sums to 1, so sum(s_glo) = G*N and sum(s_loc) = G*W per
    kv-head; the mean-alignment factor of Eq. 2 is therefore W/N."""
    n, w, d = 300, 20, 32
    inp = ems_inputs.small(1, hq, hkv, d, n, seed=3, scale=2.0)
    glo, loc = ems_ref.score(RefParams(1, hq, hkv, d, n, w), inp.f32("q"), inp.f32("k"))
    G = hq // hkv
    np.testing.assert_allclose(glo.sum(-1), G * n, rtol=1e-12)
    np.testing.assert_allclose(loc.sum(-1), G * w, rtol=1e-12)


def test_zero_queries_closed_form():
    """Q = 0 gives uniform rows A[i][j] = 1/(i+1): s_glo[j] = G*(H_N - H_j) with H the
    harmonic numbers, and s_loc[j] = G * sum_{i >= max(j, N-W)} 1/(i+1)."""
    hq, hkv, n, d, w = 4, 2, 257, 16, 19
    inp = ems_inputs.small(1, hq, hkv, d, n, seed=9)
    q = np.zeros_like(inp.f32("q"))
    glo, loc = ems_ref.score(RefParams(1, hq, hkv, d, n, w), q, inp.f32("k"))
    G = hq // hkv
    inv = 1.0 / np.arange(1, n + 1)
    tail = np.cumsum(inv[::-1])[::-1]            # tail[j] = sum_{i>=j} 1/(i+1)
    exp_glo = G * tail
    exp_loc = G * np.array([tail[max(j, n - w)] for j in range(n)])
    np.testing.assert_allclose(glo[0, 0], exp_glo, rtol=1e-12)
    np.testing.assert_allclose(glo[0, 1], exp_glo, rtol=1e-12)
    np.testing.assert_allclose(loc[0, 0], exp_loc, rtol=1e-12)


def test_window_equal_to_length_and_single_token():
    inp = ems_inputs.small(1, 2, 1, 16, 40, seed=1)
    q, k = inp.f32("q"), inp.f32("k")
    glo, loc = ems_ref.score(RefParams(1, 2, 1, 16, 40, 40), q, k)
    np.testing.assert_array_equal(glo, loc)
    g1, l1 = ems_ref.score(RefParams(1, 2, 1, 16, 1, 1), q[:, :, :1], k[:, :, :1])
    np.testing.assert_allclose(g1, 2.0)
    np.testing.assert_allclose(l1, 2.0)


def test_hard_attention_limit_is_a_histogram():
    """Keys = scaled identity rows, q_i = beta * e_{t(i)} with t(i) <= i: row i puts all of
    its weight on key t(i), so s_glo is the histogram of t and s_loc that of its tail."""
    n, w = 48, 10
    d = n
    rng = np.random.default_rng(4)
    t = np.array([rng.integers(0, i + 1) for i in range(n)])
    k = np.eye(n, dtype=np.float32)[None, None]
    q = np.zeros((1, 1, n, d), np.float32)
    q[0, 0, np.arange(n), t] = 400.0
    glo, loc = ems_ref.score(RefParams(1, 1, 1, d, n, w), q, k)
    np.testing.assert_allclose(glo[0, 0], np.bincount(t, minlength=n), atol=1e-9)
    np.testing.assert_allclose(loc[0, 0], np.bincount(t[n - w:], minlength=n), atol=1e-9)


def test_first_and_last_column_bounds_and_causality():
    hq, hkv, n, d, w = 4, 2, 120, 32, 16
    inp = ems_inputs.small(1, hq, hkv, d, n, seed=11)
    q, k = inp.f32("q"), inp.f32("k")
    glo, loc = ems_ref.score(RefParams(1, hq, hkv, d, n, w), q, k)
    G = hq // hkv
    assert (glo[..., 0] >= G - 1e-12).all()       # row 0 gives weight 1 to key 0
    assert (glo[..., -1] <= G + 1e-12).all()      # only the last row sees the last key
    assert (loc <= glo + 1e-12).all() and (loc >= 0).all()
    # causality: changing the last key/query must not change what earlier rows contribute,
    # i.e. scores from the first n-1 rows equal the scores of the truncated problem.
    g2, _ = ems_ref.score(RefParams(1, hq, hkv, d, n - 1, w), q[:, :, :n - 1], k[:, :, :n - 1])
    k_mod = k.copy(); k_mod[:, :, -1] += 5.0
    g3, _ = ems_ref.score(RefParams(1, hq, hkv, d, n, w), q, k_mod)
    # contribution of the last row is a probability vector: g - g2 (padded) sums to G
    diff = glo[..., :n - 1] - g2
    assert (diff >= -1e-12).all()
    np.testing.assert_allclose(diff.sum(-1) + glo[..., -1], G, rtol=1e-12)
    diff3 = g3[..., :n - 1] - g2
    np.testing.assert_allclose(diff3.sum(-1) + g3[..., -1], G, rtol=1e-12)


def test_key_shift_invariance():
    """Adding one vector c to every key adds the row constant q_i.c to row i of the logits;
    softmax rows are shift invariant, so no score moves."""
    hq, hkv, n, d, w = 2, 1, 90, 16, 12
    inp = ems_inputs.small(1, hq, hkv, d, n, seed=2)
    q, k = inp.f32("q"), inp.f32("k")
    c = np.linspace(-1, 1, d, dtype=np.float32) * 0.5   # exactly representable shifts
    c = ems_inputs.round_to_bf16(c)
    p = RefParams(1, hq, hkv, d, n, w)
    g1, l1 = ems_ref.score(p, q, k)
    g2, l2 = ems_ref.score(p, q, (k + c).astype(np.float32))
    np.testing.assert_allclose(g1, g2, rtol=1e-5, atol=1e-7)   # k+c rounds in float32
    np.testing.assert_allclose(l1, l2, rtol=1e-5, atol=1e-7)


def test_heads_and_batches_are_independent():
    inp = ems_inputs.small(2, 4, 2, 16, 70, seed=8)
    q, k = inp.f32("q"), inp.f32("k")
    glo, loc = ems_ref.score(RefParams(2, 4, 2, 16, 70, 9), q, k)
    g1, l1 = ems_ref.score(RefParams(1, 2, 1, 16, 70, 9), q[1:, 2:], k[1:, 1:])
    np.testing.assert_allclose(glo[1, 1], g1[0, 0], rtol=1e-13)
    np.testing.assert_allclose(loc[1, 1], l1[0, 0], rtol=1e-13)


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        ems_ref.score(RefParams(1, 3, 2, 8, 16, 4), np.zeros((1, 3, 16, 8), np.float32),
                      np.zeros((1, 2, 16, 8), np.float32))
    with pytest.raises(ValueError):
        ems_ref.score(RefParams(1, 2, 2, 8, 16, 17), np.zeros((1, 2, 16, 8), np.float32),
                      np.zeros((1, 2, 16, 8), np.float32))
