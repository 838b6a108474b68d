"""Pins for the oracle's Global-Local combination (Eq. 2), mean pooling and token
partition (Sec. 4.2)."""
import numpy as np
import pytest

from oracle import ems_ref
from oracle.ems_ref import RefParams


def _scores(rng, bh, n, w, g=1.0):
    glo = rng.random((1, bh, n)) * 3 + 0.01
    loc = rng.random((1, bh, n)) * 0.2
    return glo, loc


def test_pool_one_is_eq2_elementwise():
    rng = np.random.default_rng(0)
    n, w = 50, 8
    glo, loc = _scores(rng, 3, n, w)
    p = RefParams(1, 3, 3, 4, n, w, budget=16, pool_kernel=1)
    s = ems_ref.combine_pool(p, glo, loc)
    for h in range(3):
        c = loc[0, h].sum() / glo[0, h].sum()       # the two 1/N cancel
        np.testing.assert_allclose(s[0, h], np.maximum(glo[0, h] * c, loc[0, h]), rtol=1e-13)
    # the max is really element-wise and really a max: both branches occur
    assert ((glo * (loc.sum(-1, keepdims=True) / glo.sum(-1, keepdims=True))) > loc).any()
    assert ((glo * (loc.sum(-1, keepdims=True) / glo.sum(-1, keepdims=True))) < loc).any()


def test_alignment_makes_means_equal():
    """Eq. 2 rescales s_glo so that its mean equals the mean of s_loc: if s_loc is a
    multiple of s_glo the two arguments of the max coincide and the output is s_loc."""
    n = 64
    glo = np.linspace(5, 1, n)[None, None]
    loc = 0.25 * glo
    p = RefParams(1, 1, 1, 4, n, 4, budget=8, pool_kernel=1)
    s = ems_ref.combine_pool(p, glo, loc)
    np.testing.assert_allclose(s, loc, rtol=1e-13)
    # and if s_loc is far below the aligned s_glo everywhere but the means are forced equal,
    # the output keeps the mean of s_loc:  max(c*glo, 0) with loc == 0 except its total
    loc2 = np.zeros((1, 1, n)); loc2[0, 0, -1] = 3.0      # glo is smallest there
    s2 = ems_ref.combine_pool(p, glo, loc2)
    c = 3.0 / glo.sum()
    np.testing.assert_allclose(s2[0, 0, :-1], c * glo[0, 0, :-1], rtol=1e-13)
    assert s2[0, 0, -1] == 3.0


@pytest.mark.parametrize("pk", [3, 7, 9])
def test_pool_is_a_banded_matrix(pk):
    rng = np.random.default_rng(pk)
    n, w = 41, 5
    glo, loc = _scores(rng, 2, n, w)
    s1 = ems_ref.combine_pool(RefParams(1, 2, 2, 4, n, w, budget=8, pool_kernel=1), glo, loc)
    sp = ems_ref.combine_pool(RefParams(1, 2, 2, 4, n, w, budget=8, pool_kernel=pk), glo, loc)
    i, j = np.indices((n, n))
    band = (np.abs(i - j) <= (pk - 1) // 2) / pk        # zero padding, divisor always pk
    np.testing.assert_allclose(sp[0], s1[0] @ band.T, rtol=1e-13)


def test_pool_constant_input():
    n, pk = 30, 7
    glo = np.full((1, 1, n), 2.0)
    loc = np.full((1, 1, n), 2.0)
    s = ems_ref.combine_pool(RefParams(1, 1, 1, 4, n, 4, budget=8, pool_kernel=pk), glo, loc)
    np.testing.assert_allclose(s[0, 0, 3:-3], 2.0, rtol=1e-14)
    np.testing.assert_allclose(s[0, 0, :3], 2.0 * np.array([4, 5, 6]) / 7, rtol=1e-14)
    np.testing.assert_allclose(s[0, 0, -3:], 2.0 * np.array([6, 5, 4]) / 7, rtol=1e-14)


@pytest.mark.parametrize("n,w,nb,r", [(100, 10, 30, 0.5), (64, 8, 16, 3.0), (40, 4, 40, 2.0),
                                      (33, 1, 2, 0.0), (200, 32, 64, 10.0)])
def test_partition_matches_library_sort(n, w, nb, r):
    rng = np.random.default_rng(n)
    s = rng.random((2, 3, n))
    s[0, 0, 5:20] = 0.5                      # a run of exact ties across the cut
    p = RefParams(2, 3, 3, 4, n, w, budget=nb, merge_ratio=r)
    n_imp, n_tbm = ems_ref.sizes(p)
    assert n_imp == nb - w
    assert n_tbm == min(int(np.floor(r * nb)), n - nb)
    imp, tbm = ems_ref.partition(p, s)
    for b in range(2):
        for h in range(3):
            cand = s[b, h, :n - w]
            order = np.lexsort((np.arange(n - w), -cand))   # score desc, then position asc
            np.testing.assert_array_equal(imp[b, h], np.sort(order[:n_imp]))
            np.testing.assert_array_equal(tbm[b, h], np.sort(order[n_imp:n_imp + n_tbm]))
            # structure: disjoint, in range, ordered classes
            assert len(set(imp[b, h]) & set(tbm[b, h])) == 0
            assert imp[b, h].max(initial=-1) < n - w and tbm[b, h].max(initial=-1) < n - w
            rest = np.setdiff1d(np.arange(n - w), np.concatenate([imp[b, h], tbm[b, h]]))
            lo_imp = cand[imp[b, h]].min()
            if n_tbm:
                assert lo_imp >= cand[tbm[b, h]].max()
                if len(rest):
                    assert cand[tbm[b, h]].min() >= cand[rest].max()
            elif len(rest):
                assert lo_imp >= cand[rest].max()


def test_window_tokens_never_ranked():
    n, w, nb = 50, 10, 20
    s = np.zeros((1, 1, n)); s[0, 0, n - w:] = 100.0      # huge scores inside the window
    s[0, 0, :n - w] = np.linspace(0.1, 1.0, n - w)
    imp, tbm = ems_ref.partition(RefParams(1, 1, 1, 4, n, w, budget=nb, merge_ratio=0.5), s)
    assert imp.max() < n - w and tbm.max() < n - w
    np.testing.assert_array_equal(imp[0, 0], np.arange(n - w - 10, n - w))


def test_select_is_pool_then_partition():
    rng = np.random.default_rng(7)
    n, w, nb = 120, 12, 40
    glo, loc = _scores(rng, 2, n, w)
    p = RefParams(1, 2, 2, 4, n, w, budget=nb, merge_ratio=0.5, pool_kernel=7)
    pooled, imp, tbm = ems_ref.select(p, glo, loc)
    np.testing.assert_array_equal(pooled, ems_ref.combine_pool(p, glo, loc))
    i2, t2 = ems_ref.partition(p, pooled)
    np.testing.assert_array_equal(imp, i2)
    np.testing.assert_array_equal(tbm, t2)


def test_bad_params_rejected():
    s = np.zeros((1, 1, 16))
    for kw in (dict(budget=4, window=4), dict(budget=17, window=2), dict(budget=8, window=2,
               pool_kernel=4), dict(budget=8, window=2, merge_ratio=-1.0)):
        base = dict(batch=1, q_heads=1, kv_heads=1, head_dim=4, seq_len=16)
        base.update(kw)
        with pytest.raises(ValueError):
            ems_ref.partition(RefParams(**base), s)
