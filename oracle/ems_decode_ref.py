"""CPU oracle for the decode-time update of the EMS cache (arXiv 2412.08521).

TEST INFRASTRUCTURE ONLY: plain numpy in fp64, one head at a time, steps in the paper's
order.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may import it;
it shares no code with the HIP library.

What the paper fixes (Sec. 3.3, decoding paragraph; App. A "Evict-then-Merge Details" and
"Shared Entry Expansion"; Sec. 5 "Memory analysis"):
  * every kept token carries scalars: s_Glo, s_Loc^past, s_Loc^cur, its key norm, and its
    place in the position look-up-table;
  * each generated token adds its attention row to s_Glo and s_Loc^cur; after L_win
    generated tokens s_Loc^cur becomes s_Loc^past and restarts from zero; s_Loc = past + cur;
  * after each step the token that leaves the local window becomes a class centre, the least
    important class centre becomes the single to-be-merged token, and per head it is merged
    into its most similar centre or -- similarity not above tau -- into the zero class
    (evicted); the merge happens at class-centre level, so the tokens that shared the entry
    follow it; the budget and the number of look-up-table elements stay constant: one
    element leaves the table and the new mapping takes its place.
What it leaves open, and the reading taken here (parity is pinned GIVEN these readings):
  * the attention row of the new query is taken over the expanded run-time cache (every
    live table element with key = own norm x entry direction), the window tokens and the
    new token itself; with grouped-query attention the rows of a group's q-heads are added;
  * importance of a centre = Eq. 2 on its centre token's scalars, the mean-alignment factor
    taken over all live tokens, no pooling (the kept tokens are not contiguous);
  * similarity = cosine of the stored entry keys; lowest slot wins ties, lowest score ties
    go to the lowest slot;
  * merging entry a into entry b keeps the entry a mean of all tokens averaged into it:
    count-weighted mean of the two values and of the two unit-key means, rescaled by b's
    centre norm; the tokens that pointed to a now point to b;
  * the table element that leaves is the merged / evicted centre's own element; the new
    centre takes that element and that entry.

State of one (batch, kv-head), n_imp entries, E = n_imp + n_tbm table elements, W = L_win:
    k_cache, v_cache [budget + 1, D]   rows 0..n_imp-1 entries, n_imp..budget-1 window ring
    row_norm   [budget]                centre key norm of every row (window rows: own norm)
    entry_count[n_imp]                 tokens averaged into the entry
    entry_tok  [n_imp]                 table index of the entry's centre token
    tok_pos, tok_row [E + W]           position; cache row or -1 (free element)
    tok_norm, tok_glo, tok_past, tok_cur [E + W]
Element E + t is the window ring's slot t.
"""
from __future__ import annotations

import numpy as np


def _sizes(n, window, budget, merge_ratio):
    n_imp = budget - window
    n_tbm = min(int(np.floor(float(merge_ratio) * budget)), n - budget)
    return n_imp, n_tbm


def decode_init(seq_len, window, budget, merge_ratio, k_cache, v_cache, kept_pos, tbm_idx,
                tbm_dest, k_norm, slot_count, s_glo, s_loc):
    """Table and scalars of ONE head from what the prefill compression returned for it.
    s_glo, s_loc are the prefill's accumulated scores over all N positions (Sec. 3.3: they
    are stored for the generation; the prefill's local score is the first s_Loc^past)."""
    n_imp, n_tbm = _sizes(seq_len, window, budget, merge_ratio)
    E, W = n_imp + n_tbm, window
    kc = np.array(k_cache, np.float64, copy=True)
    vc = np.array(v_cache, np.float64, copy=True)
    st = dict(k_cache=kc, v_cache=vc,
              row_norm=np.zeros(budget), entry_count=np.array(slot_count[:n_imp], np.int64),
              entry_tok=np.arange(n_imp, dtype=np.int64),
              tok_pos=np.full(E + W, -1, np.int64), tok_row=np.full(E + W, -1, np.int64),
              tok_norm=np.zeros(E + W), tok_glo=np.zeros(E + W), tok_past=np.zeros(E + W),
              tok_cur=np.zeros(E + W))
    for s in range(n_imp):
        st["tok_pos"][s], st["tok_row"][s], st["tok_norm"][s] = kept_pos[s], s, k_norm[s]
        st["row_norm"][s] = k_norm[s]
    for i in range(n_tbm):
        j = n_imp + i
        if 0 <= tbm_dest[i] < n_imp:
            st["tok_pos"][j], st["tok_row"][j], st["tok_norm"][j] = tbm_idx[i], tbm_dest[i], k_norm[n_imp + i]
    for t in range(W):
        j, row = E + t, n_imp + t
        nrm = np.sqrt((kc[row] ** 2).sum())
        st["tok_pos"][j], st["tok_row"][j], st["tok_norm"][j] = kept_pos[row], row, nrm
        st["row_norm"][row] = nrm
    live = st["tok_row"] >= 0
    st["tok_glo"][live] = np.asarray(s_glo, np.float64)[st["tok_pos"][live]]
    st["tok_past"][live] = np.asarray(s_loc, np.float64)[st["tok_pos"][live]]
    return st


def runtime_keys(st):
    """Shared-entry expansion of the table (App. A): one key per element, zeros if free."""
    T, D = len(st["tok_row"]), st["k_cache"].shape[1]
    keys = np.zeros((T, D))
    for j in range(T):
        r = st["tok_row"][j]
        if r >= 0:
            n_r = st["row_norm"][r]
            keys[j] = st["k_cache"][r] * (st["tok_norm"][j] / n_r if n_r > 0 else 0.0)
    return keys


def global_local(glo, loc):
    """Eq. 2 on the scalars of the live tokens (no pooling)."""
    c = loc.sum() / glo.sum() if glo.sum() > 0 else 0.0
    return np.maximum(glo * c, loc)


def decode_step(st, step, window, budget, tau, softmax_scale, q_new, k_new, v_new, pos_new):
    """One generated token for ONE head group: q_new [G, D]; k_new, v_new [D].  `step` counts
    the generated tokens before this one.  Updates `st` in place and returns what was
    decided: dict(attn [G, E+W+1], tbm_entry, dest (-1 = zero class), sim, and for diagnosis
    centre_score [n_imp] (Eq. 2 of every centre) and centre_sims [n_imp] (cosines to the
    to-be-merged entry))."""
    W, n_imp = window, budget - window
    T = len(st["tok_row"])
    E = T - W
    D = st["k_cache"].shape[1]
    q_new = np.asarray(q_new, np.float64).reshape(-1, D)
    k_new, v_new = np.asarray(k_new, np.float64), np.asarray(v_new, np.float64)
    scale = softmax_scale if softmax_scale > 0 else 1.0 / np.sqrt(D)
    live = st["tok_row"] >= 0

    # 1. attention row of the new query over the run-time cache and itself (Eq. 1)
    keys = np.vstack([runtime_keys(st), k_new[None]])
    mask = np.append(live, True)
    logits = scale * (q_new @ keys.T)                       # [G, T+1]
    logits[:, ~mask] = -np.inf
    attn = np.exp(logits - logits.max(1, keepdims=True))
    attn /= attn.sum(1, keepdims=True)
    a = attn.sum(0)                                         # summed over the group

    # 2. s_Glo and s_Loc^cur accumulate the new row (Sec. 3.3)
    st["tok_glo"][live] += a[:T][live]
    st["tok_cur"][live] += a[:T][live]
    new_glo = new_cur = a[T]

    # 3. the oldest window token leaves the window; the new token takes its ring slot
    ring = step % W
    jo, ro = E + ring, n_imp + ring
    old = dict(k=st["k_cache"][ro].copy(), v=st["v_cache"][ro].copy(), pos=st["tok_pos"][jo],
               norm=st["tok_norm"][jo], glo=st["tok_glo"][jo], past=st["tok_past"][jo],
               cur=st["tok_cur"][jo])
    st["k_cache"][ro], st["v_cache"][ro] = k_new, v_new
    n_new = np.sqrt((k_new ** 2).sum())
    st["row_norm"][ro] = n_new
    st["tok_pos"][jo], st["tok_row"][jo], st["tok_norm"][jo] = pos_new, ro, n_new
    st["tok_glo"][jo], st["tok_past"][jo], st["tok_cur"][jo] = new_glo, 0.0, new_cur

    # 4. least important class centre = the to-be-merged token (App. A); the token that left
    #    the window is tracked too, so it takes part in the mean alignment
    live = st["tok_row"] >= 0
    glo = np.append(st["tok_glo"][live], old["glo"])
    loc = np.append(st["tok_past"][live] + st["tok_cur"][live], old["past"] + old["cur"])
    c = loc.sum() / glo.sum() if glo.sum() > 0 else 0.0
    ct = st["entry_tok"]
    score = np.maximum(st["tok_glo"][ct] * c, st["tok_past"][ct] + st["tok_cur"][ct])
    s_star = int(np.argmin(score))                          # first minimum = lowest slot

    # 5. its destination among the other centres (Eq. 5, key cosine of the stored entries)
    ek = st["k_cache"][:n_imp]
    en = np.sqrt((ek ** 2).sum(1))
    sims = np.full(n_imp, -np.inf)
    for s in range(n_imp):
        if s == s_star:
            continue
        sims[s] = (ek[s] / en[s]) @ (ek[s_star] / en[s_star]) if en[s] > 0 and en[s_star] > 0 else 0.0
    if n_imp > 1:
        d = int(np.argmax(sims))
        sim = float(sims[d])
    else:
        d, sim = -1, -np.inf
    merged = n_imp > 1 and sim > tau
    members = (st["tok_row"][:E] == s_star)
    members[ct[s_star]] = False                             # the centre's own element leaves the table
    if merged:
        ca, cb = st["entry_count"][s_star], st["entry_count"][d]
        na, nb = st["row_norm"][s_star], st["row_norm"][d]
        dir_a = st["k_cache"][s_star] / na if na > 0 else np.zeros(D)
        dir_b = st["k_cache"][d] / nb if nb > 0 else np.zeros(D)
        st["k_cache"][d] = nb * ((cb * dir_b + ca * dir_a) / (ca + cb))
        st["v_cache"][d] = (cb * st["v_cache"][d] + ca * st["v_cache"][s_star]) / (ca + cb)
        st["entry_count"][d] = ca + cb
        st["tok_row"][:E][members] = d
    else:
        d = -1
        idx = np.nonzero(members)[0]
        st["tok_row"][idx] = -1
        st["tok_pos"][idx] = -1
        for name in ("tok_norm", "tok_glo", "tok_past", "tok_cur"):
            st[name][idx] = 0.0

    # 6. the token that left the window is the new centre of that entry and takes the
    #    departed centre's table element
    f = int(ct[s_star])
    st["k_cache"][s_star], st["v_cache"][s_star] = old["k"], old["v"]
    st["row_norm"][s_star] = old["norm"]
    st["entry_count"][s_star] = 1
    st["tok_pos"][f], st["tok_row"][f], st["tok_norm"][f] = old["pos"], s_star, old["norm"]
    st["tok_glo"][f], st["tok_past"][f], st["tok_cur"][f] = old["glo"], old["past"], old["cur"]

    # 7. window of scores: after L_win generated tokens cur becomes past (Sec. 3.3)
    if (step + 1) % W == 0:
        st["tok_past"] = st["tok_cur"].copy()
        st["tok_cur"] = np.zeros(T)
    return dict(attn=attn, tbm_entry=s_star, dest=d, sim=sim, centre_score=score, centre_sims=sims)
