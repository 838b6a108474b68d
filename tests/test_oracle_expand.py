"""Pins for the oracle's shared-entry expansion (App. A; look-up-table of Sec. 4.2)."""
import numpy as np
import pytest

import ems_inputs
from oracle import ems_ref
from oracle.ems_ref import RefParams
from test_oracle_merge import _case


def _merged(seed, tau, **kw):
    p, k, v, imp, tbm = _case(seed=seed, tau=tau, **kw)
    out = ems_ref.evict_merge(p, k, v, imp, tbm)
    return p, k, v, imp, tbm, out


def test_layout_positions_and_evicted_rows():
    p, k, v, imp, tbm, out = _merged(3, 0.45, b=2, h=2, n=120, nb=32, r=1.0)
    n_imp, n_tbm = ems_ref.sizes(p)
    ke, ve, pos = ems_ref.expand(p, out["k_out"], out["v_out"], out["kept_pos"], tbm,
                                 out["tbm_dest"], out["k_norm"])
    E = n_imp + n_tbm + p.window
    assert ke.shape == (2, 2, E, p.head_dim) and pos.shape == (2, 2, E)
    np.testing.assert_array_equal(pos[..., :n_imp], imp)
    np.testing.assert_array_equal(pos[..., n_imp + n_tbm:],
                                  np.broadcast_to(np.arange(p.seq_len - p.window, p.seq_len), (2, 2, p.window)))
    evicted = out["tbm_dest"] == p.budget
    assert evicted.any() and (~evicted).any()
    np.testing.assert_array_equal(pos[..., n_imp:n_imp + n_tbm], np.where(evicted, -1, tbm))
    assert (ke[..., n_imp:n_imp + n_tbm, :][evicted] == 0).all()
    assert (ve[..., n_imp:n_imp + n_tbm, :][evicted] == 0).all()
    # centres and local tokens are their own entries
    np.testing.assert_array_equal(ke[..., :n_imp, :], out["k_out"][..., :n_imp, :])
    np.testing.assert_array_equal(ve[..., n_imp + n_tbm:, :], out["v_out"][..., n_imp:p.budget, :])


def test_expanded_tokens_share_value_and_direction_but_keep_their_norm():
    p, k, v, imp, tbm, out = _merged(5, -2.0, n=150, nb=40, r=2.0)     # everything merged
    n_imp, n_tbm = ems_ref.sizes(p)
    ke, ve, pos = ems_ref.expand(p, out["k_out"], out["v_out"], out["kept_pos"], tbm,
                                 out["tbm_dest"], out["k_norm"])
    for h in range(p.kv_heads):
        kk = k[0, h].astype(np.float64)
        for i in range(n_tbm):
            s = out["tbm_dest"][0, h, i]
            row = n_imp + i
            np.testing.assert_array_equal(ve[0, h, row], out["v_out"][0, h, s])
            # same direction as the entry (cosine 1), scaled by the token's own key norm
            ent = out["k_out"][0, h, s]
            cos = ke[0, h, row] @ ent / (np.linalg.norm(ke[0, h, row]) * np.linalg.norm(ent))
            np.testing.assert_allclose(cos, 1.0, rtol=1e-12)
            ratio = np.linalg.norm(ke[0, h, row]) / np.linalg.norm(ent)
            np.testing.assert_allclose(ratio, np.linalg.norm(kk[tbm[0, h, i]]) / np.linalg.norm(kk[imp[0, h, s]]),
                                       rtol=1e-12)


def test_parallel_members_are_reconstructed_exactly():
    """If every member of an entry is a multiple of the centre's key, expansion gives every
    member its own key back: the norm is what the look-up-table preserves (Sec. 4.2)."""
    p, k, v, imp, tbm = _case(seed=10, tau=0.5)
    k = k.copy()
    c = imp[0, 1, 4]
    for t, f in zip(tbm[0, 1, :3], (0.5, 2.0, 4.0)):
        k[0, 1, t] = f * k[0, 1, c]
    out = ems_ref.evict_merge(p, k, v, imp, tbm)
    members = np.nonzero(out["tbm_dest"][0, 1] == 4)[0]
    assert set(members) >= {0, 1, 2}
    if set(members) == {0, 1, 2}:
        n_imp, _ = ems_ref.sizes(p)
        ke, ve, pos = ems_ref.expand(p, out["k_out"], out["v_out"], out["kept_pos"], tbm,
                                     out["tbm_dest"], out["k_norm"])
        for i in (0, 1, 2):
            np.testing.assert_allclose(ke[0, 1, n_imp + i], k[0, 1, tbm[0, 1, i]].astype(np.float64), rtol=1e-12)


def test_no_merge_expansion_is_the_cache_itself():
    p, k, v, imp, tbm, out = _merged(6, 2.0)                           # all TBM tokens evicted
    n_imp, n_tbm = ems_ref.sizes(p)
    ke, ve, pos = ems_ref.expand(p, out["k_out"], out["v_out"], out["kept_pos"], tbm,
                                 out["tbm_dest"], out["k_norm"])
    keep = np.r_[0:n_imp, n_imp + n_tbm:n_imp + n_tbm + p.window]
    np.testing.assert_array_equal(ke[..., keep, :], out["k_out"][..., :p.budget, :])
    np.testing.assert_array_equal(ve[..., keep, :], out["v_out"][..., :p.budget, :])
    assert (pos[..., n_imp:n_imp + n_tbm] == -1).all()


def test_rejects_bad_destination():
    p, k, v, imp, tbm, out = _merged(7, 0.3)
    bad = out["tbm_dest"].copy(); bad[0, 0, 0] = ems_ref.sizes(p)[0]
    with pytest.raises(ValueError):
        ems_ref.expand(p, out["k_out"], out["v_out"], out["kept_pos"], tbm, bad, out["k_norm"])
