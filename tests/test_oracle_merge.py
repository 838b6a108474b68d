"""Pins for the oracle's merge destination (Eq. 5 + threshold) and the segmented
evict-then-merge average (Sec. 4.2, App. A)."""
import numpy as np
import pytest

import ems_inputs
from oracle import ems_ref
from oracle.ems_ref import RefParams


def _case(seed=0, b=1, h=2, n=96, d=16, w=8, nb=24, r=1.5, tau=0.0):
    inp = ems_inputs.small(b, h, h, d, n, seed=seed)
    k, v = inp.f32("k"), inp.f32("v")
    p = RefParams(b, h, h, d, n, w, budget=nb, merge_ratio=r, tau=tau)
    rng = np.random.default_rng(seed)
    n_imp, n_tbm = ems_ref.sizes(p)
    imp = np.empty((b, h, n_imp), np.int32)
    tbm = np.empty((b, h, n_tbm), np.int32)
    for bi in range(b):
        for hi in range(h):
            perm = rng.permutation(n - w)
            imp[bi, hi] = np.sort(perm[:n_imp])
            tbm[bi, hi] = np.sort(perm[n_imp:n_imp + n_tbm])
    return p, k, v, imp, tbm


def test_dest_matches_dense_cosine():
    p, k, v, imp, tbm = _case(seed=1, tau=0.45)
    dest, sim, norm = ems_ref.dest(p, k, imp, tbm)
    n_imp, n_tbm = ems_ref.sizes(p)
    for h in range(p.kv_heads):
        kk = k[0, h].astype(np.float64)
        unit = kk / np.linalg.norm(kk, axis=1, keepdims=True)
        cos = unit[tbm[0, h]] @ unit[imp[0, h]].T           # library matmul, dense
        np.testing.assert_array_equal(np.where(cos.max(1) > p.tau, cos.argmax(1), p.budget),
                                      dest[0, h])
        np.testing.assert_allclose(sim[0, h], cos.max(1), rtol=1e-12)
        np.testing.assert_allclose(norm[0, h, :n_imp], np.linalg.norm(kk[imp[0, h]], axis=1),
                                   rtol=1e-14)
        np.testing.assert_allclose(norm[0, h, n_imp:], np.linalg.norm(kk[tbm[0, h]], axis=1),
                                   rtol=1e-14)
    assert (dest == p.budget).any() and (dest < p.budget).any()   # both branches taken


def test_duplicate_of_a_centre_goes_to_it():
    p, k, v, imp, tbm = _case(seed=2, tau=0.9)
    k = k.copy()
    k[0, 0, tbm[0, 0, 3]] = 2.0 * k[0, 0, imp[0, 0, 5]]      # same direction, other norm
    dest, sim, _ = ems_ref.dest(p, k, imp, tbm)
    assert dest[0, 0, 3] == 5
    np.testing.assert_allclose(sim[0, 0, 3], 1.0, rtol=1e-12)


def test_threshold_extremes():
    """tau >= 1: every TBM token is evicted (App. B, merge threshold); tau < -1: none is."""
    p, k, v, imp, tbm = _case(seed=3, tau=1.0)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    assert (dest == p.budget).all()
    p.tau = -1.5
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    assert (dest < ems_ref.sizes(p)[0]).all()


def test_strict_threshold_and_lowest_slot_tie_break():
    p, k, v, imp, tbm = _case(seed=4, tau=1.0)
    k = k.copy()
    k[0, 0, imp[0, 0, 2]] = k[0, 0, imp[0, 0, 7]]            # two identical centres
    k[0, 0, tbm[0, 0, 0]] = k[0, 0, imp[0, 0, 7]]
    p.tau = 0.5
    dest, sim, _ = ems_ref.dest(p, k, imp, tbm)
    assert dest[0, 0, 0] == 2                                # lower slot wins the tie
    p.tau = float(sim[0, 0, 0])                              # "exceeding": equal does not merge
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    assert dest[0, 0, 0] == p.budget


def test_merge_ratio_zero_is_a_gather():
    """gamma = 1 skips the unified merge: the cache is the top tokens plus the window."""
    p, k, v, imp, tbm = _case(seed=5, r=0.0)
    out = ems_ref.evict_merge(p, k, v, imp, tbm)
    n_imp, n_tbm = ems_ref.sizes(p)
    assert n_tbm == 0
    n, w = p.seq_len, p.window
    for h in range(p.kv_heads):
        kept = np.concatenate([imp[0, h], np.arange(n - w, n)])
        np.testing.assert_array_equal(out["kept_pos"][0, h], kept)
        np.testing.assert_array_equal(out["k_out"][0, h, :p.budget], k[0, h, kept].astype(np.float64))
        np.testing.assert_array_equal(out["v_out"][0, h, :p.budget], v[0, h, kept].astype(np.float64))
        assert (out["k_out"][0, h, p.budget] == 0).all() and out["slot_count"][0, h, -1] == 0
        assert (out["slot_count"][0, h, :-1] == 1).all()


def test_all_evicted_keeps_centres_and_fills_zero_class():
    p, k, v, imp, tbm = _case(seed=6, tau=1.0)
    out = ems_ref.evict_merge(p, k, v, imp, tbm)
    n_imp, n_tbm = ems_ref.sizes(p)
    for h in range(p.kv_heads):
        np.testing.assert_array_equal(out["k_out"][0, h, :n_imp], k[0, h, imp[0, h]].astype(np.float64))
        assert out["slot_count"][0, h, -1] == n_tbm
        np.testing.assert_allclose(out["v_out"][0, h, p.budget],
                                   v[0, h, tbm[0, h]].astype(np.float64).mean(0), rtol=1e-13)
        kk = k[0, h, tbm[0, h]].astype(np.float64)
        np.testing.assert_allclose(out["k_out"][0, h, p.budget],
                                   (kk / np.linalg.norm(kk, axis=1, keepdims=True)).mean(0),
                                   rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("tau", [-2.0, 0.0, 0.15])
def test_members_mean_and_conservation(tau):
    p, k, v, imp, tbm = _case(seed=7, b=2, h=3, n=150, nb=40, r=2.0, tau=tau)
    out = ems_ref.evict_merge(p, k, v, imp, tbm)
    n_imp, n_tbm = ems_ref.sizes(p)
    Nb = p.budget
    for b in range(p.batch):
        for h in range(p.kv_heads):
            kk, vv = k[b, h].astype(np.float64), v[b, h].astype(np.float64)
            unit = kk / np.linalg.norm(kk, axis=1, keepdims=True)
            dest, cnt = out["tbm_dest"][b, h], out["slot_count"][b, h]
            assert cnt.sum() == n_imp + n_tbm and (cnt[:-1] >= 1).all()
            tot_v = np.zeros(p.head_dim); tot_u = np.zeros(p.head_dim)
            for s in range(n_imp + 1):
                row = Nb if s == n_imp else s
                members = list(tbm[b, h][dest == row])
                if s < n_imp:
                    members = [imp[b, h, s]] + members
                assert cnt[s] == len(members)
                if not members:
                    continue
                np.testing.assert_allclose(out["v_out"][b, h, row], vv[members].mean(0),
                                           rtol=1e-12, atol=1e-14)
                scale = np.linalg.norm(kk[imp[b, h, s]]) if s < n_imp else 1.0
                np.testing.assert_allclose(out["k_out"][b, h, row], scale * unit[members].mean(0),
                                           rtol=1e-12, atol=1e-14)
                tot_v += cnt[s] * out["v_out"][b, h, row]
                tot_u += cnt[s] * out["k_out"][b, h, row] / scale
            everyone = np.concatenate([imp[b, h], tbm[b, h]])
            np.testing.assert_allclose(tot_v, vv[everyone].sum(0), rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(tot_u, unit[everyone].sum(0), rtol=1e-11, atol=1e-12)
            # local rows are copies, every head has budget rows + the zero-class row
            np.testing.assert_array_equal(out["k_out"][b, h, n_imp:Nb],
                                          kk[p.seq_len - p.window:])
            np.testing.assert_array_equal(out["v_out"][b, h, n_imp:Nb],
                                          vv[p.seq_len - p.window:])
    assert out["k_out"].shape == (p.batch, p.kv_heads, Nb + 1, p.head_dim)
    if tau < 0:
        assert (out["slot_count"][..., :-1] > 1).any()      # merging really happened


def test_tbm_order_does_not_matter():
    p, k, v, imp, tbm = _case(seed=8, tau=-2.0)
    dest, _, _ = ems_ref.dest(p, k, imp, tbm)
    a = ems_ref.merge(p, k, v, imp, tbm, dest)
    perm = np.random.default_rng(0).permutation(tbm.shape[-1])
    b = ems_ref.merge(p, k, v, imp, tbm[..., perm], dest[..., perm])
    np.testing.assert_allclose(a[0], b[0], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(a[3], b[3])


def test_merge_rejects_bad_destination():
    p, k, v, imp, tbm = _case(seed=9)
    dest = np.full(tbm.shape, ems_ref.sizes(p)[0], np.int32)   # N_imp is not a valid slot
    with pytest.raises(ValueError):
        ems_ref.merge(p, k, v, imp, tbm, dest)


def test_merged_key_keeps_centre_norm_when_members_are_parallel():
    """If every member points along the centre, the mean unit key is the centre's unit key
    and the stored key equals the centre's own key: the norm is preserved (Sec. 4.2)."""
    p, k, v, imp, tbm = _case(seed=10, tau=0.5)
    k = k.copy()
    c = imp[0, 1, 4]
    for t, f in zip(tbm[0, 1, :3], (0.5, 2.0, 4.0)):
        k[0, 1, t] = f * k[0, 1, c]
    out = ems_ref.evict_merge(p, k, v, imp, tbm)
    assert out["slot_count"][0, 1, 4] >= 4
    members = tbm[0, 1][out["tbm_dest"][0, 1] == 4]
    if set(members) == set(tbm[0, 1, :3]):
        np.testing.assert_allclose(out["k_out"][0, 1, 4], k[0, 1, c], rtol=1e-12)
