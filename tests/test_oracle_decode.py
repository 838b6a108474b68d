"""Pins for the decode-time oracle (Sec. 3.3 decoding paragraph; App. A "Evict-then-Merge
Details"): attention row against a dense softmax over the explicitly expanded cache, score
bookkeeping, window ring, threshold extremes, entries as plain means of everything they
absorbed (shadow bookkeeping on the raw tokens), table invariants."""
import numpy as np
import pytest
from scipy.special import softmax

import ems_inputs
from oracle import ems_decode_ref as dec
from oracle import ems_ref
from oracle.ems_ref import RefParams


class Case:
    """A small prompt compressed by the prefill oracle, one decode state per kv-head."""

    def __init__(self, seed=0, hq=4, hkv=2, n=96, d=16, w=8, nb=24, r=1.5, tau=0.3, pre_tau=0.3):
        self.p = p = RefParams(1, hq, hkv, d, n, w, budget=nb, merge_ratio=r, tau=pre_tau, pool_kernel=3)
        self.tau, self.g = tau, hq // hkv
        inp = ems_inputs.small(1, hq, hkv, d, n, seed=seed)
        self.q, self.k, self.v = inp.f32("q"), inp.f32("k"), inp.f32("v")
        self.s_glo, self.s_loc = ems_ref.score(p, self.q, self.k)
        _, self.imp, self.tbm = ems_ref.select(p, self.s_glo, self.s_loc)
        self.m = ems_ref.evict_merge(p, self.k, self.v, self.imp, self.tbm)
        self.n_imp, self.n_tbm = ems_ref.sizes(p)
        self.rng = np.random.default_rng(seed + 100)
        self.states = [self.init(h) for h in range(hkv)]
        self.raw = [{int(pos): (self.k[0, h, pos].astype(np.float64), self.v[0, h, pos].astype(np.float64))
                     for pos in range(n)} for h in range(hkv)]
        self.t = 0

    def init(self, h):
        m, p = self.m, self.p
        return dec.decode_init(p.seq_len, p.window, p.budget, p.merge_ratio, m["k_out"][0, h], m["v_out"][0, h],
                               m["kept_pos"][0, h], self.tbm[0, h], m["tbm_dest"][0, h], m["k_norm"][0, h],
                               m["slot_count"][0, h], self.s_glo[0, h], self.s_loc[0, h])

    def step(self, h, q=None, k=None, v=None):
        p = self.p
        q = self.rng.standard_normal((self.g, p.head_dim)) if q is None else q
        k = self.rng.standard_normal(p.head_dim) if k is None else k
        v = self.rng.standard_normal(p.head_dim) if v is None else v
        pos = p.seq_len + self.t
        self.raw[h][pos] = (k.copy(), v.copy())
        info = dec.decode_step(self.states[h], self.t, p.window, p.budget, self.tau, 0.0, q, k, v, pos)
        return q, k, v, info


def test_init_table_matches_the_prefill_outputs():
    c = Case(seed=1)
    for h, st in enumerate(c.states):
        E = c.n_imp + c.n_tbm
        np.testing.assert_array_equal(st["tok_pos"][:c.n_imp], c.imp[0, h])
        np.testing.assert_array_equal(st["tok_row"][:c.n_imp], np.arange(c.n_imp))
        dest = c.m["tbm_dest"][0, h]
        kept = dest < c.n_imp
        np.testing.assert_array_equal(st["tok_row"][c.n_imp:E], np.where(kept, dest, -1))
        np.testing.assert_array_equal(st["tok_pos"][c.n_imp:E][kept], c.tbm[0, h][kept])
        np.testing.assert_array_equal(st["tok_pos"][E:], np.arange(c.p.seq_len - c.p.window, c.p.seq_len))
        live = st["tok_row"] >= 0
        np.testing.assert_array_equal(st["tok_glo"][live], c.s_glo[0, h][st["tok_pos"][live]])
        np.testing.assert_array_equal(st["tok_past"][live], c.s_loc[0, h][st["tok_pos"][live]])
        assert not st["tok_cur"].any()
        np.testing.assert_allclose(st["tok_norm"][live], np.linalg.norm(c.k[0, h, st["tok_pos"][live]].astype(np.float64), axis=1), rtol=1e-13)
        assert kept.any() and (~kept).any()


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2)])
def test_attention_row_is_dense_softmax_over_the_expanded_cache(hq, hkv):
    """The run-time cache is the shared-entry expansion (pinned on its own) plus the new token."""
    c = Case(seed=2, hq=hq, hkv=hkv)
    p, m = c.p, c.m
    k_exp, _, pos_exp = ems_ref.expand(p, m["k_out"], m["v_out"], m["kept_pos"], c.tbm, m["tbm_dest"], m["k_norm"])
    for h in range(hkv):
        q, k, v, info = c.step(h)
        keys = np.vstack([k_exp[0, h], k[None]])
        logits = (q @ keys.T) / np.sqrt(p.head_dim)
        logits[:, :-1][:, pos_exp[0, h] < 0] = -np.inf
        np.testing.assert_allclose(info["attn"], softmax(logits, axis=1), rtol=1e-11, atol=1e-300)
        np.testing.assert_allclose(info["attn"].sum(1), 1.0, rtol=1e-13)


def test_scores_accumulate_the_attention_rows_and_swap_after_a_window():
    c = Case(seed=3, tau=-2.0)
    W, h = c.p.window, 0
    st = c.states[h]
    acc = {}
    past0 = {int(p_): x for p_, x in zip(st["tok_pos"], st["tok_past"]) if p_ >= 0}
    glo0 = {int(p_): x for p_, x in zip(st["tok_pos"], st["tok_glo"]) if p_ >= 0}
    for t in range(W):
        c.t = t
        pos_before = st["tok_pos"].copy()
        live_before = st["tok_row"] >= 0
        q, k, v, info = c.step(h)
        a = info["attn"].sum(0)
        for j in np.nonzero(live_before)[0]:
            acc[int(pos_before[j])] = acc.get(int(pos_before[j]), 0.0) + a[j]
        acc[c.p.seq_len + t] = a[-1]
        now = {int(p_): (g_, pa, cu) for p_, g_, pa, cu in
               zip(st["tok_pos"], st["tok_glo"], st["tok_past"], st["tok_cur"]) if p_ >= 0}
        for pos, (g_, pa, cu) in now.items():
            np.testing.assert_allclose(g_, glo0.get(pos, 0.0) + acc[pos], rtol=1e-12)
            if t < W - 1:
                np.testing.assert_allclose(cu, acc[pos], rtol=1e-12)
                assert pa == past0.get(pos, 0.0)
            else:                                            # the window of queries is complete
                np.testing.assert_allclose(pa, acc[pos], rtol=1e-12)
                assert cu == 0.0


def test_window_ring_holds_the_last_positions():
    c = Case(seed=4)
    W, n_imp, N = c.p.window, c.n_imp, c.p.seq_len
    st = c.states[1]
    E = c.n_imp + c.n_tbm
    for t in range(2 * W + 3):
        c.t = t
        c.step(1)
        np.testing.assert_array_equal(np.sort(st["tok_pos"][E:]), np.arange(N - W + t + 1, N + t + 1))
        for j in range(W):
            pos = int(st["tok_pos"][E + j])
            assert st["tok_row"][E + j] == n_imp + j
            np.testing.assert_array_equal(st["k_cache"][n_imp + j], c.raw[1][pos][0])
            np.testing.assert_array_equal(st["v_cache"][n_imp + j], c.raw[1][pos][1])


@pytest.mark.parametrize("tau", [2.0, -2.0])
def test_threshold_extremes(tau):
    """tau >= 1: the to-be-merged centre is always evicted and takes its followers with it;
    tau < -1: it is always merged and the number of live table elements stays constant."""
    c = Case(seed=5, tau=tau)
    st = c.states[0]
    E = c.n_imp + c.n_tbm
    for t in range(12):
        c.t = t
        rows_before = st["tok_row"][:E].copy()
        live_before = (rows_before >= 0).sum()
        _, _, _, info = c.step(0)
        s = info["tbm_entry"]
        followers = (rows_before == s).sum() - 1
        if tau >= 1:
            assert info["dest"] == -1
            assert (st["tok_row"][:E] >= 0).sum() == live_before - followers
            assert (st["tok_row"][:E] == s).sum() == 1       # only the new centre
        else:
            assert info["dest"] >= 0 and info["dest"] != s
            assert (st["tok_row"][:E] >= 0).sum() == live_before
            assert (st["tok_row"][:E] == info["dest"]).sum() == (rows_before == info["dest"]).sum() + followers


@pytest.mark.parametrize("tau", [0.25, -2.0])
def test_entries_are_plain_means_of_everything_they_absorbed(tau):
    """Shadow bookkeeping on the raw tokens: an entry's value is the mean of the raw values of
    all tokens averaged into it, its key the mean of their unit keys times the centre's norm."""
    c = Case(seed=6, tau=tau)
    h, p = 0, c.p
    st = c.states[h]
    absorbed = [[int(c.imp[0, h, s])] + [int(x) for x in c.tbm[0, h][c.m["tbm_dest"][0, h] == s]]
                for s in range(c.n_imp)]
    centre = [int(x) for x in c.imp[0, h]]
    merged_any = False
    for t in range(3 * p.window):
        c.t = t
        leaving = int(st["tok_pos"][c.n_imp + c.n_tbm + t % p.window])
        _, _, _, info = c.step(h)
        s, d = info["tbm_entry"], info["dest"]
        if d >= 0:
            absorbed[d] += absorbed[s]
            merged_any = True
        absorbed[s], centre[s] = [leaving], leaving
    assert merged_any
    for s in range(c.n_imp):
        ks = np.array([c.raw[h][x][0] for x in absorbed[s]])
        vs = np.array([c.raw[h][x][1] for x in absorbed[s]])
        assert st["entry_count"][s] == len(absorbed[s])
        if len(absorbed[s]) == 1:
            np.testing.assert_allclose(st["k_cache"][s], ks[0], rtol=1e-13)
            np.testing.assert_allclose(st["v_cache"][s], vs[0], rtol=1e-13)
            continue
        unit = ks / np.linalg.norm(ks, axis=1, keepdims=True)
        n_c = np.linalg.norm(c.raw[h][centre[s]][0])
        np.testing.assert_allclose(st["row_norm"][s], n_c, rtol=1e-13)
        np.testing.assert_allclose(st["v_cache"][s], vs.mean(0), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(st["k_cache"][s], n_c * unit.mean(0), rtol=1e-10, atol=1e-12)


def test_least_important_centre_is_the_one_merged():
    c = Case(seed=7, tau=2.0)
    st = c.states[0]
    for name in ("tok_glo", "tok_past"):
        st[name][:c.n_imp] += 50.0                           # every centre important ...
    victim = 5
    st["tok_glo"][victim] = st["tok_past"][victim] = 0.0      # ... but one
    _, _, _, info = c.step(0)
    assert info["tbm_entry"] == victim and info["dest"] == -1
    # exact tie between two centres: the lower slot goes first
    c2 = Case(seed=7, tau=2.0)
    st = c2.states[0]
    for name in ("tok_glo", "tok_past"):
        st[name][:c2.n_imp] += 50.0
    for s in (9, 3):
        st["tok_glo"][s] = st["tok_past"][s] = 0.0
        st["k_cache"][s] = 0.0                               # zero key: no attention difference either
        st["k_cache"][s, 0] = 1e-30
    st["tok_norm"][[3, 9]] = st["row_norm"][[3, 9]] = 1e-30
    _, _, _, info = c2.step(0)
    assert info["tbm_entry"] == 3


def test_parallel_entries_merge_with_similarity_one():
    c = Case(seed=8, tau=0.999)
    st = c.states[1]
    a, b = 2, 11
    alone = [s for s in range(c.n_imp) if st["entry_count"][s] == 1]
    a, b = alone[0], alone[-1]
    st["k_cache"][b] = 2.5 * st["k_cache"][a]
    st["row_norm"][b] = st["tok_norm"][b] = 2.5 * st["row_norm"][a]
    st["tok_glo"][:c.n_imp] += 50.0
    st["tok_glo"][a] = st["tok_past"][a] = 0.0
    kb, vb, va = st["k_cache"][b].copy(), st["v_cache"][b].copy(), st["v_cache"][a].copy()
    _, _, _, info = c.step(1)
    assert info["tbm_entry"] == a and info["dest"] == b
    np.testing.assert_allclose(info["sim"], 1.0, rtol=1e-12)
    np.testing.assert_allclose(st["k_cache"][b], kb, rtol=1e-12)          # same direction, b's norm
    np.testing.assert_allclose(st["v_cache"][b], 0.5 * (va + vb), rtol=1e-12)
    assert st["entry_count"][b] == 2 and st["entry_count"][a] == 1


def test_table_invariants_over_many_steps():
    c = Case(seed=9, tau=0.2)
    p = c.p
    E = c.n_imp + c.n_tbm
    for h in range(p.kv_heads):
        st = c.states[h]
        for t in range(40):
            c.t = t
            c.step(h)
            live = st["tok_row"] >= 0
            assert live[E:].all()
            assert (st["tok_row"][:E][live[:E]] < c.n_imp).all()
            pos = st["tok_pos"][live]
            assert len(np.unique(pos)) == len(pos)
            np.testing.assert_array_equal(st["tok_row"][st["entry_tok"]], np.arange(c.n_imp))
            assert (st["entry_count"] >= 1).all()
            assert (st["tok_glo"][live] > 0).all()
            # every stored entry key has norm <= its centre norm (a mean of unit vectors)
            assert (np.linalg.norm(st["k_cache"][:c.n_imp], axis=1) <= st["row_norm"][:c.n_imp] * (1 + 1e-12)).all()


@pytest.mark.parametrize("side", [-1, +1])
def test_threshold_is_applied_to_the_best_cosine(side):
    """tau just below the best cosine merges into the arg-max, just above evicts."""
    c = Case(seed=10)
    st = c.states[0]
    victim = 4
    st["tok_glo"][:c.n_imp] += 50.0
    st["tok_glo"][victim] = st["tok_past"][victim] = 0.0
    ek = st["k_cache"][:c.n_imp]
    unit = ek / np.linalg.norm(ek, axis=1, keepdims=True)
    cos = unit @ unit[victim]
    cos[victim] = -np.inf
    best = int(np.argmax(cos))
    c.tau = cos[best] + side * 1e-9
    _, _, _, info = c.step(0)
    assert info["tbm_entry"] == victim
    np.testing.assert_allclose(info["sim"], cos[best], rtol=1e-12)
    assert info["dest"] == (best if side < 0 else -1)
