"""Pins for the oracle's paper-faithful merge variants: redundancy as key / value / key x value
cosine (Sec. 4.1, similarity ablation of App. B) and the score-weighted merge (Sec. 4.2)."""
import numpy as np
import pytest

from oracle import ems_ref
from test_oracle_merge import _case


def _unit(x):
    x = x.astype(np.float64)
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


# ------------------------------------------------------------------ similarity modes
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_dest_sim_matches_dense_numpy(mode):
    p, k, v, imp, tbm = _case(seed=11, tau=[0.45, 0.45, 0.15][mode])
    dest, sim, norm = ems_ref.dest_sim(p, mode, k, v, imp, tbm)
    n_imp, _ = ems_ref.sizes(p)
    for h in range(p.kv_heads):
        ck = _unit(k[0, h, tbm[0, h]]) @ _unit(k[0, h, imp[0, h]]).T
        cv = _unit(v[0, h, tbm[0, h]]) @ _unit(v[0, h, imp[0, h]]).T
        r = [ck, cv, ck * cv][mode]
        np.testing.assert_array_equal(dest[0, h], np.where(r.max(1) > p.tau, r.argmax(1), p.budget))
        np.testing.assert_allclose(sim[0, h], r.max(1), rtol=1e-12, atol=1e-15)
        # norms are key norms whatever the similarity
        np.testing.assert_allclose(norm[0, h, :n_imp], np.linalg.norm(k[0, h, imp[0, h]].astype(np.float64), axis=1), rtol=1e-14)
        np.testing.assert_allclose(norm[0, h, n_imp:], np.linalg.norm(k[0, h, tbm[0, h]].astype(np.float64), axis=1), rtol=1e-14)
    assert (dest == p.budget).any() and (dest < p.budget).any()


def test_key_mode_is_the_plain_destination():
    p, k, v, imp, tbm = _case(seed=12, tau=0.3)
    d0, s0, n0 = ems_ref.dest(p, k, imp, tbm)
    d1, s1, n1 = ems_ref.dest_sim(p, 0, k, v, imp, tbm)
    np.testing.assert_array_equal(d0, d1)
    np.testing.assert_allclose(s0, s1, rtol=1e-13)
    np.testing.assert_allclose(n0, n1, rtol=1e-15)


def test_value_mode_is_key_mode_on_swapped_tensors():
    p, k, v, imp, tbm = _case(seed=13, tau=0.2)
    dv, sv, _ = ems_ref.dest_sim(p, 1, k, v, imp, tbm)
    dk, sk, _ = ems_ref.dest_sim(p, 0, v, k, imp, tbm)
    np.testing.assert_array_equal(dv, dk)
    np.testing.assert_array_equal(sv, sk)


def test_product_reduces_to_key_cosine_when_values_are_parallel():
    """All values on one ray: every value cosine is 1, the product is the key cosine."""
    p, k, v, imp, tbm = _case(seed=14, tau=0.3)
    ray = np.random.default_rng(0).standard_normal(p.head_dim).astype(np.float32)
    scale = np.random.default_rng(1).uniform(0.5, 2.0, v.shape[:3]).astype(np.float32)
    v2 = scale[..., None] * ray
    d2, s2, _ = ems_ref.dest_sim(p, 2, k, v2, imp, tbm)
    d0, s0, _ = ems_ref.dest(p, k, imp, tbm)
    np.testing.assert_array_equal(d2, d0)
    np.testing.assert_allclose(s2, s0, rtol=1e-6)          # float32 ray: value cosine = 1 to rounding


def test_product_of_two_negative_cosines_is_positive():
    """The paper defines the redundancy as the plain product, signs included."""
    p, k, v, imp, tbm = _case(seed=15, tau=0.5, h=1)
    k, v = k.copy(), v.copy()
    t, c = tbm[0, 0, 2], imp[0, 0, 4]
    k[0, 0, t] = -1.5 * k[0, 0, c]
    v[0, 0, t] = -0.5 * v[0, 0, c]
    d, s, _ = ems_ref.dest_sim(p, 2, k, v, imp, tbm)
    assert d[0, 0, 2] == 4
    np.testing.assert_allclose(s[0, 0, 2], 1.0, rtol=1e-12)
    dk, sk, _ = ems_ref.dest_sim(p, 0, k, v, imp, tbm)
    assert dk[0, 0, 2] != 4 or sk[0, 0, 2] < 0            # key cosine alone never picks the antipode


def test_scaled_copy_in_both_tensors_has_redundancy_one():
    p, k, v, imp, tbm = _case(seed=16, tau=0.99)
    k, v = k.copy(), v.copy()
    for h in range(p.kv_heads):
        k[0, h, tbm[0, h, 1]] = 3.0 * k[0, h, imp[0, h, 7]]
        v[0, h, tbm[0, h, 1]] = 0.25 * v[0, h, imp[0, h, 7]]
    d, s, _ = ems_ref.dest_sim(p, 2, k, v, imp, tbm)
    assert (d[0, :, 1] == 7).all()
    np.testing.assert_allclose(s[0, :, 1], 1.0, rtol=1e-12)
    # a key-only copy is not enough for the product with a high threshold
    v[0, 0, tbm[0, 0, 1]] = np.random.default_rng(3).standard_normal(p.head_dim)
    d, s, _ = ems_ref.dest_sim(p, 2, k, v, imp, tbm)
    assert d[0, 0, 1] == p.budget


# ------------------------------------------------------------------ weighted merge
def _weights(p, seed):
    return np.random.default_rng(seed).uniform(0.1, 2.0, (p.batch, p.kv_heads, p.seq_len))


def test_constant_weights_give_the_plain_mean():
    p, k, v, imp, tbm = _case(seed=21, tau=0.1)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    ref = ems_ref.merge(p, k, v, imp, tbm, dest)
    for c in (1.0, 0.37):
        got = ems_ref.merge_weighted(p, k, v, np.full((p.batch, p.kv_heads, p.seq_len), c), imp, tbm, dest)
        np.testing.assert_allclose(got[0], ref[0], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(got[1], ref[1], rtol=1e-13, atol=1e-15)
        np.testing.assert_array_equal(got[2], ref[2])
        np.testing.assert_array_equal(got[3], ref[3])


def test_weighted_mean_recomputed_with_numpy():
    p, k, v, imp, tbm = _case(seed=22, tau=0.1)
    w = _weights(p, 5)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    ko, vo, kept, cnt = ems_ref.merge_weighted(p, k, v, w, imp, tbm, dest)
    n_imp, _ = ems_ref.sizes(p)
    joined = 0
    for h in range(p.kv_heads):
        kk, vv = k[0, h].astype(np.float64), v[0, h].astype(np.float64)
        for s in list(range(n_imp)) + [p.budget]:
            pos = ([] if s == p.budget else [imp[0, h, s]]) + list(tbm[0, h][dest[0, h] == s])
            if s != p.budget and len(pos) == 1:
                np.testing.assert_array_equal(ko[0, h, s], kk[pos[0]])
                np.testing.assert_array_equal(vo[0, h, s], vv[pos[0]])
                continue
            if not pos:
                assert not ko[0, h, s].any() and not vo[0, h, s].any()
                continue
            joined += 1
            ww = w[0, h, pos]
            np.testing.assert_allclose(vo[0, h, s], np.average(vv[pos], axis=0, weights=ww), rtol=1e-12, atol=1e-14)
            scale = 1.0 if s == p.budget else np.linalg.norm(kk[imp[0, h, s]])
            np.testing.assert_allclose(ko[0, h, s], scale * np.average(_unit(kk[pos]), axis=0, weights=ww),
                                       rtol=1e-12, atol=1e-14)
    assert joined > 4


def test_integer_weight_equals_repeated_token():
    """A member of weight 2 counts like two identical members of weight 1 (uniform merge of a
    sequence in which the token appears twice)."""
    p, k, v, imp, tbm = _case(seed=23, tau=-2.0, h=1)
    k, v = k.copy(), v.copy()
    a, b = tbm[0, 0, 0], tbm[0, 0, 1]
    k[0, 0, b], v[0, 0, b] = k[0, 0, a], v[0, 0, a]                # b is a copy of a
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    assert dest[0, 0, 0] == dest[0, 0, 1]                           # copies share a destination
    uni = ems_ref.merge(p, k, v, imp, tbm, dest)
    # weighted run: a carries weight 2 and its copy b weight 0
    w = np.ones((1, 1, p.seq_len)); w[0, 0, a] = 2.0; w[0, 0, b] = 0.0
    got = ems_ref.merge_weighted(p, k, v, w, imp, tbm, dest)
    s = dest[0, 0, 0]
    np.testing.assert_allclose(got[0][0, 0, s], uni[0][0, 0, s], rtol=1e-13)
    np.testing.assert_allclose(got[1][0, 0, s], uni[1][0, 0, s], rtol=1e-13)


def test_zero_weight_member_is_ignored():
    p, k, v, imp, tbm = _case(seed=24, tau=-2.0, h=1)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    w = _weights(p, 6)
    w[0, 0, tbm[0, 0, 4]] = 0.0
    got = ems_ref.merge_weighted(p, k, v, w, imp, tbm, dest)
    dest2 = dest.copy(); dest2[0, 0, 4] = p.budget                 # same thing: the token leaves its slot
    ref = ems_ref.merge_weighted(p, k, v, w, imp, tbm, dest2)
    s = dest[0, 0, 4]
    if ref[3][0, 0, s] > 1:                                         # slot still merged without it
        np.testing.assert_allclose(got[0][0, 0, s], ref[0][0, 0, s], rtol=1e-13)
        np.testing.assert_allclose(got[1][0, 0, s], ref[1][0, 0, s], rtol=1e-13)
    assert got[3][0, 0, s] == ref[3][0, 0, s] + 1                   # still counted as a member


def test_weight_scale_invariance_and_negative_as_zero():
    p, k, v, imp, tbm = _case(seed=25, tau=0.0)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    w = _weights(p, 7)
    a = ems_ref.merge_weighted(p, k, v, w, imp, tbm, dest)
    b = ems_ref.merge_weighted(p, k, v, 8.0 * w, imp, tbm, dest)     # power of two: exact
    np.testing.assert_array_equal(a[0], b[0]); np.testing.assert_array_equal(a[1], b[1])
    w0 = w.copy(); w0[..., ::3] = 0.0
    wn = w.copy(); wn[..., ::3] = -1.0
    a = ems_ref.merge_weighted(p, k, v, w0, imp, tbm, dest)
    b = ems_ref.merge_weighted(p, k, v, wn, imp, tbm, dest)
    np.testing.assert_array_equal(a[0], b[0]); np.testing.assert_array_equal(a[1], b[1])


def test_weighted_conservation():
    """sum over entries of (total weight) x (entry value) = sum of w_i v_i over all members."""
    p, k, v, imp, tbm = _case(seed=26, tau=0.15)
    w = _weights(p, 8)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    ko, vo, kept, cnt = ems_ref.merge_weighted(p, k, v, w, imp, tbm, dest)
    n_imp, _ = ems_ref.sizes(p)
    for h in range(p.kv_heads):
        tot = np.zeros(n_imp + 1)
        np.add.at(tot, np.arange(n_imp), w[0, h, imp[0, h]])
        np.add.at(tot, np.where(dest[0, h] == p.budget, n_imp, dest[0, h]), w[0, h, tbm[0, h]])
        rows = np.r_[np.arange(n_imp), p.budget]
        lhs = (tot[:, None] * vo[0, h, rows]).sum(0)
        members = np.r_[imp[0, h], tbm[0, h]]
        rhs = (w[0, h, members, None] * v[0, h, members].astype(np.float64)).sum(0)
        np.testing.assert_allclose(lhs, rhs, rtol=1e-11, atol=1e-12)


def test_all_zero_weights_keep_the_centres():
    p, k, v, imp, tbm = _case(seed=27, tau=-2.0)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    ko, vo, kept, cnt = ems_ref.merge_weighted(p, k, v, np.zeros((p.batch, p.kv_heads, p.seq_len)), imp, tbm, dest)
    n_imp, _ = ems_ref.sizes(p)
    for h in range(p.kv_heads):
        np.testing.assert_array_equal(ko[0, h, :n_imp], k[0, h, imp[0, h]].astype(np.float64))
        np.testing.assert_array_equal(vo[0, h, :n_imp], v[0, h, imp[0, h]].astype(np.float64))
        assert not ko[0, h, p.budget].any()


def test_weighted_rejects_bad_destination():
    p, k, v, imp, tbm = _case(seed=28)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    dest[0, 0, 0] = p.budget - 1                                    # a local-window row
    with pytest.raises(ValueError):
        ems_ref.merge_weighted(p, k, v, _weights(p, 1), imp, tbm, dest)
