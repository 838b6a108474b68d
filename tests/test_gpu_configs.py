"""GPU parity at the full sizes of the five benchmark configurations, in the launch
configuration bench.py times.  Where the fp64 oracle cannot do the whole layer in seconds it
does whole (batch, kv-head) units of it -- units are independent, which the small tests pin --
and every unit is additionally checked through properties that hold at any size and through
the oracle's cheap stages run on the GPU's own upstream output."""
import numpy as np
import pytest
import torch

import ems_inputs
from oracle import ems_ref
from paper_2412_08521_amd import binding as B
from gpu_util import (RTOL, RTOL_MERGE, assert_dest_valid, assert_rel, assert_sparsity_count_valid, check_band,
                      dev_tensor, ref_params)

pytestmark = pytest.mark.gpu


def _log(*a):
    print(*a, flush=True)


def _params(w, tau, mode=B.EMS_BF16):
    return B.EmsParams(w.batch, w.q_heads, w.kv_heads, w.head_dim, w.seq_len, w.window, w.budget,
                       merge_ratio=w.merge_ratio, tau=tau, pool_kernel=w.pool_kernel, dtype=mode)


def _upload(w, mode, layer=0):
    tdt = torch.float32 if mode == B.EMS_F32 else torch.bfloat16
    q = torch.empty((w.batch, w.q_heads, w.seq_len, w.head_dim), dtype=tdt, device="cuda")
    k = torch.empty((w.batch, w.kv_heads, w.seq_len, w.head_dim), dtype=tdt, device="cuda")
    v = torch.empty_like(k)
    host = []
    for b in range(w.batch):
        inp = ems_inputs.generate(w, layer=layer, batch_slice=slice(b, b + 1))
        q[b].copy_(dev_tensor(inp.q[0], mode)); k[b].copy_(dev_tensor(inp.k[0], mode))
        v[b].copy_(dev_tensor(inp.v[0], mode))
        host.append(inp)
    return q, k, v, host


def _run_chain(p, q, k, v):
    s_glo, s_loc = B.ems_global_local_score(p, q, k)
    imp, tbm, pooled = B.ems_select(p, s_glo, s_loc, want_pooled=True)
    out = B.ems_evict_merge(p, k, v, imp, tbm)
    torch.cuda.synchronize()
    return s_glo, s_loc, imp, tbm, pooled, out


def _check_unit_against_oracle(p, w, host_b, b, kvh, s_glo, s_loc, rtol):
    """Whole-unit element-wise score parity: the G q-heads of one (batch, kv-head)."""
    G = w.q_heads // w.kv_heads
    qf = host_b.f32("q")[:, kvh * G:(kvh + 1) * G]
    kf = host_b.f32("k")[:, kvh:kvh + 1]
    rp = ems_ref.RefParams(1, G, 1, w.head_dim, w.seq_len, w.window, softmax_scale=p.softmax_scale)
    o_glo, o_loc = ems_ref.score(rp, qf, kf)
    e1 = assert_rel(s_glo[b, kvh].cpu().numpy(), o_glo[0, 0], rtol, f"s_glo[{b},{kvh}]")
    e2 = assert_rel(s_loc[b, kvh].cpu().numpy(), o_loc[0, 0], rtol, f"s_loc[{b},{kvh}]")
    _log(f"  unit ({b},{kvh}): rel err glo {e1:.2e} loc {e2:.2e}")
    return o_glo[0, 0], o_loc[0, 0]


def _check_properties_all_units(p, w, host, s_glo, s_loc, imp, tbm, pooled, out, mode):
    """Holds at any size, checked on every (batch, kv-head)."""
    G = w.q_heads // w.kv_heads
    n_imp, n_tbm = B.ems_partition_sizes(p)
    # every causal softmax row sums to one
    np.testing.assert_allclose(s_glo.double().sum(-1).cpu().numpy(), G * w.seq_len, rtol=2e-4)
    np.testing.assert_allclose(s_loc.double().sum(-1).cpu().numpy(), G * w.window, rtol=2e-4)
    assert (s_loc <= s_glo * (1 + 1e-5) + 1e-12).all() and (s_loc >= 0).all()
    rp = ref_params(p)
    pooled_n = pooled.cpu().numpy()
    imp_n, tbm_n = imp.cpu().numpy(), tbm.cpu().numpy()
    # Eq. 2 + pooling of the GPU's own scores, then the partition of the GPU's own keys
    o_pooled = ems_ref.combine_pool(rp, s_glo.cpu().numpy(), s_loc.cpu().numpy())
    assert_rel(pooled_n, o_pooled, 1e-5, "pooled")
    x_imp, x_tbm = ems_ref.partition(rp, pooled_n.astype(np.float64))
    np.testing.assert_array_equal(imp_n, x_imp)
    np.testing.assert_array_equal(tbm_n, x_tbm)
    # evict-then-merge of every unit against the oracle's stages on the GPU's index sets
    kf = np.concatenate([h.f32("k") for h in host])
    vf = np.concatenate([h.f32("v") for h in host])
    ref = ems_ref.evict_merge(rp, kf, vf, imp_n, tbm_n)
    dest = out["tbm_dest"].cpu().numpy()
    np.testing.assert_allclose(out["tbm_sim"].cpu().numpy(), ref["tbm_sim"], rtol=0, atol=5e-6)
    # a destination may differ from the oracle's only where the decision is inside float32 noise
    n_diff = assert_dest_valid(dest, ref["tbm_dest"], kf, imp_n, tbm_n, p.tau, p.budget)
    assert n_diff <= max(1, dest.size // 200), n_diff
    k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge(rp, kf, vf, imp_n, tbm_n, dest)
    np.testing.assert_array_equal(out["kept_pos"].cpu().numpy(), kept_ref)
    np.testing.assert_array_equal(out["slot_count"].cpu().numpy(), cnt_ref)
    for name, want in (("k_out", k_ref), ("v_out", v_ref)):
        got = out[name].float().cpu().numpy()
        rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
        err = np.abs(got - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))
        assert err.max() <= RTOL_MERGE[mode], f"{name}: {err.max():.3e}"
    assert out["k_out"].shape == (w.batch, w.kv_heads, w.budget + 1, w.head_dim)
    assert cnt_ref.sum(-1).min() == n_imp + n_tbm == cnt_ref.sum(-1).max()
    return dest, ref


def _rel_rows(got, want):
    rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
    return (np.abs(got - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))).max()


def _host(d):
    return {n_: (t_.float().cpu().numpy() if t_.is_floating_point() else t_.cpu().numpy()) for n_, t_ in d.items()}


def _check_follow_up_calls(p, w, host, k, v, s_glo, s_loc, imp, tbm, pooled, out, units, steps=3):
    """The entry points that follow the compression, at the configuration's full shapes:
    shared-entry expansion, the key x value / score-weighted merge, and a few decode steps
    (each step checked in isolation on the given (batch, kv-head) units)."""
    from test_gpu_decode import run_and_check_step
    rp = ref_params(p)
    n_imp, n_tbm = B.ems_partition_sizes(p)
    imp_n, tbm_n = imp.cpu().numpy(), tbm.cpu().numpy()
    kf = np.concatenate([h.f32("k") for h in host])
    vf = np.concatenate([h.f32("v") for h in host])
    # expansion of the GPU's own compact cache
    k_exp, v_exp, pos = B.ems_expand(p, out, tbm)
    ho = _host(out)
    ko, vo, po = ems_ref.expand(rp, ho["k_out"], ho["v_out"], ho["kept_pos"], tbm_n, ho["tbm_dest"], ho["k_norm"])
    np.testing.assert_array_equal(pos.cpu().numpy(), po)
    np.testing.assert_array_equal(v_exp.float().cpu().numpy(), vo)
    assert _rel_rows(k_exp.float().cpu().numpy(), ko) <= 2.0 ** -8
    # paper-faithful merge variant: redundancy = key cosine x value cosine, weights = pooled score
    var = _host(B.ems_evict_merge_variant(p, B.EMS_SIM_KEY_VALUE, k, v, pooled, imp, tbm))
    d_ref, s_ref, n_ref = ems_ref.dest_sim(rp, 2, kf, vf, imp_n, tbm_n)
    np.testing.assert_allclose(var["tbm_sim"], s_ref, rtol=0, atol=1e-5)
    n_diff = assert_dest_valid(var["tbm_dest"], d_ref, kf, imp_n, tbm_n, p.tau, p.budget, vf=vf, tol=4e-5,
                               what="key x value tbm_dest")
    assert n_diff <= max(1, d_ref.size // 200), n_diff
    k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge_weighted(rp, kf, vf, pooled.cpu().numpy(), imp_n, tbm_n,
                                                             var["tbm_dest"])
    np.testing.assert_array_equal(var["slot_count"], cnt_ref)
    assert _rel_rows(var["k_out"], k_ref) <= RTOL_MERGE[B.EMS_BF16]
    assert _rel_rows(var["v_out"], v_ref) <= RTOL_MERGE[B.EMS_BF16]
    # per-head statistics: Eq. 3 against the oracle on the GPU's own scores, Eq. 4 on sampled tokens
    rate, nk = B.ems_sparsity_rate(p, 0.9, s_glo, s_loc)
    o_rate, o_nk = ems_ref.sparsity(rp, 0.9, s_glo.cpu().numpy(), s_loc.cpu().numpy())
    assert np.abs(nk.cpu().numpy() - o_nk).max() <= max(2, w.seq_len // 2000), (nk, o_nk)
    g_n, l_n, nk_n = s_glo.cpu().numpy(), s_loc.cpu().numpy(), nk.cpu().numpy()
    for b_ in range(w.batch):                              # both sides of the threshold, every head
        for h_ in range(w.kv_heads):
            assert_sparsity_count_valid(nk_n[b_, h_], g_n[b_, h_], l_n[b_, h_], 0.9)
    red, best = B.ems_redundancy_rate(p, k, v)
    tokens = np.array([0, 1, 31, 32, 1000, w.seq_len // 2 + 17, w.seq_len - 1], np.int32)
    o_best = ems_ref.redundancy_at(rp, kf, vf, tokens)
    np.testing.assert_allclose(best.cpu().numpy()[..., tokens][..., 1:], o_best[..., 1:], rtol=0, atol=1e-5)
    assert (best[..., 0] == -np.inf).all()
    np.testing.assert_array_equal(np.rint(red.cpu().numpy() * w.seq_len),
                                  (best >= p.tau).sum(-1).cpu().numpy())
    # decode steps on a copy of the cache
    merged = {n_: t_.clone() for n_, t_ in out.items()}
    st = B.ems_decode_init(p, merged, tbm, s_glo, s_loc)
    rng = np.random.default_rng(5)
    flips = 0
    for t in range(steps):
        qb = ems_inputs.f32_to_bf16_bits(rng.standard_normal((w.batch, w.q_heads, w.head_dim)).astype(np.float32))
        kb = ems_inputs.f32_to_bf16_bits(rng.standard_normal((w.batch, w.kv_heads, w.head_dim)).astype(np.float32))
        vb = ems_inputs.f32_to_bf16_bits(rng.standard_normal((w.batch, w.kv_heads, w.head_dim)).astype(np.float32))
        flips += run_and_check_step(p, st, t, qb, kb, vb, p.tau, units, B.EMS_BF16)[0]
    assert flips <= 1
    live = st.tok_row >= 0
    assert (st.tok_pos[live] >= 0).all() and torch.isfinite(st.tok_glo).all()
    _log(f"  follow-up calls checked: expand, key x value weighted merge, Eq. 3 / Eq. 4 statistics, "
         f"{steps} decode steps on {units}")


@pytest.mark.parametrize("mode", [B.EMS_BF16, B.EMS_F32])
def test_config2_llama2_7b_4k_full(mode):
    """32 heads MHA, D 128, N 4096, W 32, budget 256: the oracle does the whole layer."""
    w = ems_inputs.WORKLOADS["llama2_7b_4k"]
    q, k, v, host = _upload(w, mode)
    for tau in (0.6, 0.2):
        p = _params(w, tau, mode)
        s_glo, s_loc, imp, tbm, pooled, out = _run_chain(p, q, k, v)
        rp = ref_params(p)
        o_glo, o_loc = ems_ref.score(rp, host[0].f32("q"), host[0].f32("k"))
        e1 = assert_rel(s_glo.cpu().numpy(), o_glo, RTOL[mode], "s_glo")
        e2 = assert_rel(s_loc.cpu().numpy(), o_loc, RTOL[mode], "s_loc")
        _log(f"config 2 mode {mode} tau {tau}: rel err glo {e1:.2e} loc {e2:.2e}")
        o_pooled, o_imp, o_tbm = ems_ref.select(rp, o_glo, o_loc)
        for h in range(w.kv_heads):
            check_band(imp[0, h].cpu().numpy(), tbm[0, h].cpu().numpy(), o_pooled[0, h],
                       w.seq_len - w.window, RTOL[mode])
        if mode == B.EMS_F32:
            same = (imp.cpu().numpy() == o_imp).all(-1).mean()
            _log(f"  heads whose important set equals the fp64 oracle's exactly: {same:.2f}")
        dest, ref = _check_properties_all_units(p, w, host, s_glo, s_loc, imp, tbm, pooled, out, mode)
        if tau == 0.2:
            assert (dest < w.budget).any() and (dest == w.budget).any()


def test_config3_mistral_7b_16k():
    """32/8 GQA, N 16384: two whole kv-head groups against the oracle, properties on all."""
    w = ems_inputs.WORKLOADS["mistral_7b_16k"]
    q, k, v, host = _upload(w, B.EMS_BF16)
    p = _params(w, 0.6)
    s_glo, s_loc, imp, tbm, pooled, out = _run_chain(p, q, k, v)
    for kvh in (0, 5):
        _check_unit_against_oracle(p, w, host[0], 0, kvh, s_glo, s_loc, RTOL[B.EMS_BF16])
    _check_properties_all_units(p, w, host, s_glo, s_loc, imp, tbm, pooled, out, B.EMS_BF16)
    # f32 mode on one group (the same keys, four of the q-heads) to the 1e-5 bar
    G = w.q_heads // w.kv_heads
    p1 = B.EmsParams(1, G, 1, w.head_dim, w.seq_len, w.window, dtype=B.EMS_F32)
    g32, l32 = B.ems_global_local_score(p1, q[:, 2 * G:3 * G].float().contiguous(),
                                        k[:, 2:3].float().contiguous())
    rp = ems_ref.RefParams(1, G, 1, w.head_dim, w.seq_len, w.window)
    o_glo, o_loc = ems_ref.score(rp, host[0].f32("q")[:, 2 * G:3 * G], host[0].f32("k")[:, 2:3])
    e1 = assert_rel(g32.cpu().numpy(), o_glo, RTOL[B.EMS_F32], "f32 s_glo")
    e2 = assert_rel(l32.cpu().numpy(), o_loc, RTOL[B.EMS_F32], "f32 s_loc")
    _log(f"config 3 f32 mode group 2: rel err glo {e1:.2e} loc {e2:.2e}")


def test_config4_llama3_8b_32k():
    """Batch 4, 32/8 GQA, N 32768, W 64, budget 128 -- the benchmark workload."""
    w = ems_inputs.WORKLOADS["llama3_8b_32k"]
    q, k, v, host = _upload(w, B.EMS_BF16)
    p = _params(w, 0.6)
    s_glo, s_loc, imp, tbm, pooled, out = _run_chain(p, q, k, v)
    for b, kvh in ((0, 0), (3, 6)):
        o_glo, o_loc = _check_unit_against_oracle(p, w, host[b], b, kvh, s_glo, s_loc, RTOL[B.EMS_BF16])
        rp1 = ems_ref.RefParams(1, 1, 1, w.head_dim, w.seq_len, w.window, budget=w.budget,
                                merge_ratio=w.merge_ratio, pool_kernel=w.pool_kernel)
        o_pooled, _, _ = ems_ref.select(rp1, o_glo[None, None], o_loc[None, None])
        check_band(imp[b, kvh].cpu().numpy(), tbm[b, kvh].cpu().numpy(), o_pooled[0, 0],
                   w.seq_len - w.window, RTOL[B.EMS_BF16])
    _check_properties_all_units(p, w, host, s_glo, s_loc, imp, tbm, pooled, out, B.EMS_BF16)
    # a second run gives the same bits: which wave takes which work item varies from run to run, but
    # every float has one writer and a fixed summation order (atomics are integer counters only)
    again = _run_chain(p, q, k, v)
    assert torch.equal(again[0], s_glo) and torch.equal(again[1], s_loc)
    assert torch.equal(again[2], imp) and torch.equal(again[5]["k_out"], out["k_out"])
    # merge-heavy variant of the same workload
    p2 = _params(w, -2.0)
    out2 = B.ems_evict_merge(p2, k, v, imp, tbm)
    _check_properties_all_units(p2, w, host, s_glo, s_loc, imp, tbm, pooled, out2, B.EMS_BF16)
    assert (out2["slot_count"][..., -1] == 0).all()
    _check_follow_up_calls(p2, w, host, k, v, s_glo, s_loc, imp, tbm, pooled, out2, [(0, 0), (3, 6)])
    _check_follow_up_calls(p, w, host, k, v, s_glo, s_loc, imp, tbm, pooled, out, [(1, 3)], steps=2)


def test_config5_extreme_128k_two_layers():
    """32/8 GQA, N 131072, budget 2048: layers 0 and 31 of the 32 sequential layers (each
    layer has its own seeded inputs and is independent of the others)."""
    w = ems_inputs.WORKLOADS["extreme_128k"]
    for layer in (0, 31):
        _log(f"config 5 layer {layer}")
        q, k, v, host = _upload(w, B.EMS_BF16, layer=layer)
        p = _params(w, 0.6)
        s_glo, s_loc, imp, tbm, pooled, out = _run_chain(p, q, k, v)
        _check_properties_all_units(p, w, host, s_glo, s_loc, imp, tbm, pooled, out, B.EMS_BF16)
        if layer == 0:
            # one whole (batch, kv-head) unit of the benchmark launch itself -- the group sum over
            # its 4 q-heads, all row chunks and their reduction -- element by element at full length
            o_glo, o_loc = _check_unit_against_oracle(p, w, host[0], 0, 2, s_glo, s_loc, RTOL[B.EMS_BF16])
            rp1 = ems_ref.RefParams(1, 1, 1, w.head_dim, w.seq_len, w.window, budget=w.budget,
                                    merge_ratio=w.merge_ratio, pool_kernel=w.pool_kernel)
            o_pooled, _, _ = ems_ref.select(rp1, o_glo[None, None], o_loc[None, None])
            check_band(imp[0, 2].cpu().numpy(), tbm[0, 2].cpu().numpy(), o_pooled[0, 0],
                       w.seq_len - w.window, RTOL[B.EMS_BF16])
            p2 = _params(w, 0.15)
            out2 = B.ems_evict_merge(p2, k, v, imp, tbm)
            dest, _ = _check_properties_all_units(p2, w, host, s_glo, s_loc, imp, tbm, pooled, out2,
                                                  B.EMS_BF16)
            assert (dest < w.budget).any()
            _check_follow_up_calls(p2, w, host, k, v, s_glo, s_loc, imp, tbm, pooled, out2, [(0, 2)], steps=2)
        del q, k, v, host
        torch.cuda.empty_cache()
