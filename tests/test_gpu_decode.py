"""GPU parity of the decode-time path (ems_decode_init, ems_decode_step) against the numpy
oracle.  Every step is checked in isolation: the oracle starts from the GPU's own state before
the step, so that one flipped near-tie cannot hide or fake later differences."""
import sys

import numpy as np
import pytest
import torch

import ems_inputs
from gpu_util import dev_tensor, ref_params
from oracle import ems_decode_ref as dec
from oracle import ems_ref
from paper_2412_08521_amd import binding as B

pytestmark = pytest.mark.gpu

MODES = [B.EMS_BF16, B.EMS_F32]
SHAPES = [
    # (b, hq, hkv, d, n, w, budget, r)
    (1, 4, 2, 64, 600, 16, 48, 1.5),
    (2, 8, 2, 128, 1500, 32, 160, 2.0),
    (1, 2, 2, 128, 900, 8, 200, 3.0),
    (1, 8, 1, 64, 700, 8, 40, 1.0),
]


def _log(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


def _np(t):
    return t.float().cpu().numpy() if t.is_floating_point() else t.cpu().numpy()


def _prefill(shape, mode, tau, seed):
    """Prompt compressed by the library; returns params, device tensors and the state."""
    b, hq, hkv, d, n, w, nb, r = shape
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=seed)
    p = B.EmsParams(b, hq, hkv, d, n, w, nb, merge_ratio=r, tau=tau, pool_kernel=3, dtype=mode)
    q, k, v = (dev_tensor(getattr(inp, x), mode) for x in "qkv")
    s_glo, s_loc = B.ems_global_local_score(p, q, k)
    imp, tbm = B.ems_select(p, s_glo, s_loc)
    pre = B.EmsParams(b, hq, hkv, d, n, w, nb, merge_ratio=r, tau=0.25, pool_kernel=3, dtype=mode)
    merged = B.ems_evict_merge(pre, k, v, imp, tbm)
    st = B.ems_decode_init(p, merged, tbm, s_glo, s_loc)
    return p, merged, tbm, s_glo, s_loc, st


def _host_state(st, b, h):
    out = {}
    for name in B.STATE_FIELDS:
        if name == "step_count":
            continue
        a = _np(getattr(st, name)[b, h])
        out[name] = a.astype(np.int64) if a.dtype.kind == "i" else a.astype(np.float64)
    return out


def _new_token(p, rng, mode):
    def mk(heads):
        x = ems_inputs.f32_to_bf16_bits(rng.standard_normal((p.batch, heads, p.head_dim)).astype(np.float32))
        return x
    return mk(p.q_heads), mk(p.kv_heads), mk(p.kv_heads)


def run_and_check_step(p, st, t, qb, kb, vb, tau, units, mode):
    """One ems_decode_step on the GPU, checked in isolation for the given (batch, kv-head) units:
    the oracle takes the same step from the GPU's own state before it.  qb, kb, vb are bf16 bit
    patterns [B, heads, D].  Returns (decisions flipped inside float32 noise, merges, evictions)."""
    G, W = p.q_heads // p.kv_heads, p.window
    # merged rows: one bf16 rounding of the stored row; in f32 mode about ten float32 roundings with
    # cancellation between the two entries (the f32 bar of the prefill merge is the same 1e-5)
    cache_rtol = 2.0 ** -7 if mode == B.EMS_BF16 else 1e-5
    before = {u: _host_state(st, *u) for u in units}
    out = B.ems_decode_step(p, st, t, dev_tensor(qb, mode), dev_tensor(kb, mode), dev_tensor(vb, mode),
                            want_attn=True)
    attn, decision, sim = _np(out["attn"]), _np(out["decision"]), _np(out["sim"])
    qf, kf, vf = (ems_inputs.bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    n_flip = n_merge = n_evict = 0
    for (b, h) in units:
        ref = before[(b, h)]
        info = dec.decode_step(ref, t, W, p.budget, tau, 0.0, qf[b, h * G:(h + 1) * G], kf[b, h], vf[b, h],
                               p.seq_len + t)
        got = _host_state(st, b, h)
        np.testing.assert_allclose(attn[b, h * G:(h + 1) * G], info["attn"], rtol=2e-5, atol=1e-9)
        if tuple(decision[b, h]) != (info["tbm_entry"], info["dest"]):
            # a different decision is legitimate only inside float32 noise of a tie or of tau
            sc, sims = info["centre_score"], info["centre_sims"]
            gs, gd = int(decision[b, h, 0]), int(decision[b, h, 1])
            if gs != info["tbm_entry"]:
                assert abs(sc[gs] - sc[info["tbm_entry"]]) <= 1e-5 * np.abs(sc).max(), (t, b, h)
            elif gd >= 0 and info["dest"] >= 0:
                assert abs(sims[gd] - sims[info["dest"]]) < 2e-5, (t, b, h)
            else:
                assert abs(info["sim"] - tau) < 2e-5, (t, b, h)
            n_flip += 1
            continue
        n_merge += info["dest"] >= 0
        n_evict += info["dest"] < 0
        if np.isfinite(info["sim"]):
            assert abs(sim[b, h] - info["sim"]) < 1e-5
        for name in ("entry_count", "entry_tok", "tok_pos", "tok_row"):
            np.testing.assert_array_equal(got[name], ref[name], err_msg=f"{name} step {t}")
        for name in ("tok_norm", "tok_glo", "tok_past", "tok_cur", "row_norm"):
            np.testing.assert_allclose(got[name], ref[name], rtol=2e-5, atol=1e-9, err_msg=f"{name} step {t}")
        for name in ("k_cache", "v_cache"):
            want, have = ref[name][:p.budget], got[name][:p.budget]
            rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
            err = np.abs(have - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))
            assert err.max() <= cache_rtol, f"{name} step {t}: {err.max():.3e}"
    return n_flip, n_merge, n_evict


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", SHAPES[:3])
def test_decode_init_matches_oracle(shape, mode):
    _log("decode_init", shape, mode)
    p, merged, tbm, s_glo, s_loc, st = _prefill(shape, mode, 0.3, seed=5)
    m = {k_: _np(v_) for k_, v_ in merged.items()}
    for b in range(p.batch):
        for h in range(p.kv_heads):
            ref = dec.decode_init(p.seq_len, p.window, p.budget, p.merge_ratio, m["k_out"][b, h], m["v_out"][b, h],
                                  m["kept_pos"][b, h], _np(tbm)[b, h], m["tbm_dest"][b, h], m["k_norm"][b, h],
                                  m["slot_count"][b, h], _np(s_glo)[b, h], _np(s_loc)[b, h])
            got = _host_state(st, b, h)
            for name in ("entry_count", "entry_tok", "tok_pos", "tok_row"):
                np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
            for name in ("tok_glo", "tok_past", "tok_cur"):
                np.testing.assert_array_equal(got[name], ref[name], err_msg=name)   # gathers: exact
            np.testing.assert_allclose(got["tok_norm"], ref["tok_norm"], rtol=1e-6)
            np.testing.assert_allclose(got["row_norm"], ref["row_norm"], rtol=1e-6)
    assert (st.tok_row < 0).any() and (st.tok_row >= 0).any()


# a budget whose per-row staging does not fit in LDS: the kernel stages in the workspace instead
# large caches: in bf16 the step runs as four launches over row slices; BIG stages its row dots in the
# workspace (they do not fit in LDS), BIG_LDS in LDS
BIG = (1, 8, 1, 64, 4000, 8, 1800, 0.5)
BIG_LDS = (1, 8, 2, 128, 5000, 16, 1100, 0.5)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("tau", [0.3, -2.0, 2.0])
@pytest.mark.parametrize("shape", SHAPES + [BIG, BIG_LDS])
def test_decode_steps_match_oracle(shape, tau, mode):
    _log("decode_step", shape, "tau", tau, "mode", mode)
    p, merged, tbm, s_glo, s_loc, st = _prefill(shape, mode, tau, seed=shape[6])
    n_imp, n_tbm = B.ems_partition_sizes(p)
    G, W, D = p.q_heads // p.kv_heads, p.window, p.head_dim
    assert (shape == BIG) == (4 * (G + 1) * p.budget > 60 * 1024)
    rng = np.random.default_rng(17)
    n_merge = n_evict = n_flip = 0
    for t in range(W + 6):
        qb, kb, vb = _new_token(p, rng, mode)
        if t % 3 == 1:                                    # make some new keys similar to an entry
            src = ems_inputs.f32_to_bf16_bits(_np(st.k_cache[:, :, (3 * t) % n_imp]).astype(np.float32))
            kb = src
        units = [(b, h) for b in range(p.batch) for h in range(p.kv_heads)]
        c = run_and_check_step(p, st, t, qb, kb, vb, tau, units, mode)
        n_flip += c[0]; n_merge += c[1]; n_evict += c[2]
    total = (W + 6) * p.batch * p.kv_heads
    assert n_flip <= max(1, total // 20), (n_flip, total)
    if tau >= 1:
        assert n_merge == 0
    elif tau <= -1:
        assert n_evict == 0
    elif shape not in (BIG, BIG_LDS):                     # with a thousand random centres something is always similar
        assert n_merge > 0 and n_evict > 0, (n_merge, n_evict)


def test_decode_invariants_over_many_steps():
    shape = SHAPES[1]
    p, merged, tbm, s_glo, s_loc, st = _prefill(shape, B.EMS_BF16, 0.3, seed=3)
    n_imp, n_tbm = B.ems_partition_sizes(p)
    E, W, N = n_imp + n_tbm, p.window, p.seq_len
    g = torch.Generator(device="cpu").manual_seed(1)
    steps = 40 * W + 5                                  # long enough for every entry to be replaced several times
    qs = torch.randn((steps, p.batch, p.q_heads, p.head_dim), generator=g).to(torch.bfloat16).cuda()
    ks = torch.randn((steps, p.batch, p.kv_heads, p.head_dim), generator=g).to(torch.bfloat16).cuda()
    vs = torch.randn((steps, p.batch, p.kv_heads, p.head_dim), generator=g).to(torch.bfloat16).cuda()
    ws = torch.empty(max(B.ems_decode_workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")
    out = None
    for t in range(steps):
        out = B.ems_decode_step(p, st, t, qs[t], ks[t], vs[t], ws=ws, out=out)
    torch.cuda.synchronize()
    rows, pos = _np(st.tok_row), _np(st.tok_pos)
    for b in range(p.batch):
        for h in range(p.kv_heads):
            np.testing.assert_array_equal(np.sort(pos[b, h, E:]), np.arange(N + steps - W, N + steps))
            live = rows[b, h] >= 0
            assert (rows[b, h, :E][live[:E]] < n_imp).all()
            assert len(np.unique(pos[b, h][live])) == live.sum()
            np.testing.assert_array_equal(rows[b, h][_np(st.entry_tok)[b, h]], np.arange(n_imp))
            assert (_np(st.entry_count)[b, h] >= 1).all()
            assert np.isfinite(_np(st.k_cache)[b, h]).all() and np.isfinite(_np(st.tok_glo)[b, h]).all()
