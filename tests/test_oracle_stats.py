"""Pins for the oracle's per-head statistics: sparsity rate (Eq. 3) and redundancy rate (Eq. 4)."""
import numpy as np
import pytest

import ems_inputs
from oracle import ems_ref
from oracle.ems_ref import RefParams


def _p(n, h=1, d=16, w=4, tau=0.6):
    return RefParams(1, h, h, d, n, w, tau=tau)


def _both(s):
    """s_glo = s_loc = s makes Eq. 2 return s itself (factor 1, max of equals)."""
    s = np.asarray(s, np.float64)[None, None]
    return s, s.copy()


# ------------------------------------------------------------------ Eq. 3
@pytest.mark.parametrize("zeta", [0.5, 0.9, 1.0 / 3.0, 1.0])
def test_uniform_scores_need_a_zeta_share_of_the_tokens(zeta):
    n = 60
    g, l = _both(np.full(n, 0.25))
    p_m, nk = ems_ref.sparsity(_p(n), zeta, g, l)
    assert nk[0, 0] == int(np.ceil(zeta * n - 1e-9))
    np.testing.assert_allclose(p_m[0, 0], 1 - nk[0, 0] / n, rtol=1e-15)


def test_one_hot_score_is_maximally_sparse():
    n = 50
    s = np.zeros(n); s[17] = 3.0
    p_m, nk = ems_ref.sparsity(_p(n), 0.95, *_both(s))
    assert nk[0, 0] == 1 and p_m[0, 0] == 1 - 1 / n


def test_geometric_scores_closed_form():
    """s_i = 2^-i (shuffled): the top k add up to 2 - 2^(1-k) of a total 2 - 2^(1-N)."""
    n = 40
    s = 2.0 ** -np.arange(n)
    rng = np.random.default_rng(0)
    for zeta in (0.5, 0.75, 0.9, 0.999):
        total = 2 - 2.0 ** (1 - n)
        k = next(k for k in range(1, n + 1) if 2 - 2.0 ** (1 - k) >= zeta * total)
        p_m, nk = ems_ref.sparsity(_p(n), zeta, *_both(rng.permutation(s)))
        assert nk[0, 0] == k


def test_sparsity_matches_numpy_on_the_global_local_score():
    n, h = 300, 3
    rng = np.random.default_rng(1)
    g = rng.gamma(0.3, 1.0, (1, h, n)); l = rng.gamma(0.3, 0.05, (1, h, n))
    l[0, :, ::17] *= 200                                   # both branches of the max occur
    p = _p(n, h=h)
    p_m, nk = ems_ref.sparsity(p, 0.8, g, l)
    for i in range(h):
        c = l[0, i].sum() / g[0, i].sum()
        s = np.maximum(g[0, i] * c, l[0, i])
        assert (g[0, i] * c > l[0, i]).any() and (g[0, i] * c < l[0, i]).any()
        cs = np.cumsum(np.sort(s)[::-1])
        want = int(np.searchsorted(cs, 0.8 * s.sum(), side="left")) + 1
        assert abs(nk[0, i] - want) <= 0                   # fp64 both sides, same summation order
        np.testing.assert_allclose(p_m[0, i], 1 - want / n)
    # s_glo alone would give another answer: the statistic is taken on Eq. 2's output
    alone = [int(np.searchsorted(np.cumsum(np.sort(g[0, i])[::-1]), 0.8 * g[0, i].sum())) + 1 for i in range(h)]
    assert any(a != b for a, b in zip(alone, nk[0]))


def test_sparsity_is_scale_and_permutation_invariant():
    n = 128
    rng = np.random.default_rng(2)
    g = rng.gamma(0.5, 1.0, (1, 1, n)); l = rng.gamma(0.5, 0.1, (1, 1, n))
    a = ems_ref.sparsity(_p(n), 0.7, g, l)
    b = ems_ref.sparsity(_p(n), 0.7, 4.0 * g, 4.0 * l)
    perm = rng.permutation(n)
    c = ems_ref.sparsity(_p(n), 0.7, g[..., perm], l[..., perm])
    assert a[1] == b[1] and abs(int(a[1][0, 0]) - int(c[1][0, 0])) <= 1   # the sum order changes with the permutation
    with pytest.raises(ValueError):
        ems_ref.sparsity(_p(n), 0.0, g, l)


# ------------------------------------------------------------------ Eq. 4
def _unit(x):
    x = x.astype(np.float64)
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def test_redundancy_matches_dense_numpy():
    n, h, d = 90, 2, 16
    inp = ems_inputs.small(1, h, h, d, n, seed=3)
    k, v = inp.f32("k").copy(), inp.f32("v").copy()
    rng = np.random.default_rng(3)
    for t in range(10, n, 9):                              # plant some near-copies of earlier tokens
        j = rng.integers(0, t)
        k[0, :, t] = 0.95 * k[0, :, j] + 0.2 * k[0, :, t]
        v[0, :, t] = 0.9 * v[0, :, j] + 0.25 * v[0, :, t]
    p = _p(n, h=h, d=d, tau=0.6)
    r, best = ems_ref.redundancy(p, k, v)
    for i in range(h):
        R = (_unit(k[0, i]) @ _unit(k[0, i]).T) * (_unit(v[0, i]) @ _unit(v[0, i]).T)
        R[np.triu_indices(n)] = -np.inf                    # only strictly earlier tokens count
        want = R.max(1)
        assert best[0, i, 0] == -np.inf
        np.testing.assert_allclose(best[0, i, 1:], want[1:], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(r[0, i], (want >= 0.6).mean(), rtol=1e-15)
    assert 0.05 < r.mean() < 0.5


def test_a_copy_is_redundant_but_its_original_is_not():
    n, d = 40, 16
    inp = ems_inputs.small(1, 1, 1, d, n, seed=4)
    k, v = inp.f32("k").copy(), inp.f32("v").copy()
    k[0, 0, 30], v[0, 0, 30] = 2.0 * k[0, 0, 7], 0.5 * v[0, 0, 7]
    r, best = ems_ref.redundancy(_p(n, d=d, tau=0.999), k, v)
    np.testing.assert_allclose(best[0, 0, 30], 1.0, rtol=1e-12)
    assert best[0, 0, 7] < 0.999                           # token 7 only sees tokens 0..6
    np.testing.assert_allclose(r[0, 0], 1 / n)


def test_redundancy_threshold_extremes_and_inclusive_comparison():
    n, d = 30, 16
    inp = ems_inputs.small(1, 1, 1, d, n, seed=5)
    k, v = inp.f32("k"), inp.f32("v")
    assert ems_ref.redundancy(_p(n, d=d, tau=1.5), k, v)[0][0, 0] == 0.0
    np.testing.assert_allclose(ems_ref.redundancy(_p(n, d=d, tau=-1.0), k, v)[0][0, 0], (n - 1) / n)
    # Eq. 4 compares with >=: a threshold equal to a token's best redundancy counts it
    _, best = ems_ref.redundancy(_p(n, d=d, tau=0.0), k, v)
    t = int(np.argmax(best[0, 0]))
    at = ems_ref.redundancy(_p(n, d=d, tau=float(best[0, 0, t])), k, v)[0][0, 0]
    above = ems_ref.redundancy(_p(n, d=d, tau=float(np.nextafter(best[0, 0, t], 2.0))), k, v)[0][0, 0]
    np.testing.assert_allclose(at, 1 / n)
    assert above == 0.0


def test_redundancy_at_is_the_same_loop_on_chosen_tokens():
    n, h, d = 70, 2, 16
    inp = ems_inputs.small(1, h, h, d, n, seed=6)
    k, v = inp.f32("k"), inp.f32("v")
    _, best = ems_ref.redundancy(_p(n, h=h, d=d), k, v)
    tokens = np.array([0, 1, 17, 69], np.int32)
    np.testing.assert_array_equal(ems_ref.redundancy_at(_p(n, h=h, d=d), k, v, tokens), best[..., tokens])
    with pytest.raises(ValueError):
        ems_ref.redundancy_at(_p(n, h=h, d=d), k, v, np.array([70], np.int32))


def test_redundancy_at_against_dense_cosine_products():
    """The sampled form on its own against Eq. 4 written out with numpy: for a chosen token t the best
    product of key and value cosines over the strictly earlier tokens (none for t = 0)."""
    n, h, d = 90, 2, 32
    inp = ems_inputs.small(1, h, h, d, n, seed=8)
    k, v = inp.f32("k").copy(), inp.f32("v").copy()
    k[0, :, 61], v[0, :, 61] = 3.0 * k[0, :, 12], 0.25 * v[0, :, 12]     # a scaled copy of an earlier token
    tokens = np.array([0, 1, 2, 40, 61, 89], np.int32)
    got = ems_ref.redundancy_at(_p(n, h=h, d=d), k, v, tokens)
    for i in range(h):
        uk, uv = _unit(k[0, i]), _unit(v[0, i])
        for c, t in enumerate(tokens):
            if t == 0:
                assert got[0, i, c] == -np.inf
                continue
            want = ((uk[:t] @ uk[t]) * (uv[:t] @ uv[t])).max()
            np.testing.assert_allclose(got[0, i, c], want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(got[0, :, 4], 1.0, rtol=1e-12)
