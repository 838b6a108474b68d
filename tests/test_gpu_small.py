"""GPU parity, element by element, at sizes the oracle finishes in seconds: several tiles
and ragged tails, MHA and GQA, both head sizes, both modes, and the degenerate cases."""
import numpy as np
import pytest
import torch

import ems_inputs
from oracle import ems_ref
from paper_2412_08521_amd import binding as B
from gpu_util import (RTOL, RTOL_MERGE, assert_dest_valid, assert_rel, check_band, dev_tensor, is_sorted_unique,
                      ref_params)

pytestmark = pytest.mark.gpu

MODES = [B.EMS_BF16, B.EMS_F32]

# (batch, q_heads, kv_heads, head_dim, seq_len, window)
SCORE_SHAPES = [
    (1, 2, 2, 64, 1, 1),
    (1, 2, 1, 128, 31, 7),
    (2, 4, 2, 64, 777, 33),        # ragged tail, GQA
    (1, 2, 2, 128, 1000, 32),      # several key tiles + tail
    (1, 4, 1, 128, 300, 300),      # window == length
    (1, 8, 2, 128, 2500, 64),      # several row chunks in pass 2
    (1, 2, 2, 64, 4099, 70),       # window straddles a chunk boundary
    (1, 6, 3, 128, 6000, 64),      # heads that do not divide over the XCDs: pairs dealt by block index
]


def _log(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", SCORE_SHAPES)
def test_score_matches_oracle(shape, mode):
    b, hq, hkv, d, n, w = shape
    _log("score", shape, "mode", mode)
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=n + d)
    p = B.EmsParams(b, hq, hkv, d, n, w, dtype=mode)
    q, k = dev_tensor(inp.q, mode), dev_tensor(inp.k, mode)
    s_glo, s_loc, lse = B.ems_global_local_score(p, q, k, want_lse=True)
    torch.cuda.synchronize()
    o_glo, o_loc, o_lse = ems_ref.score(ref_params(p), inp.f32("q"), inp.f32("k"), want_lse=True)
    rtol = RTOL[mode]
    assert_rel(s_glo.cpu().numpy(), o_glo, rtol, "s_glo")
    assert_rel(s_loc.cpu().numpy(), o_loc, rtol, "s_loc")
    np.testing.assert_allclose(lse.cpu().numpy(), o_lse, rtol=0, atol=2e-5 if mode == B.EMS_F32 else 2e-2)
    # invariants that hold at any size: weights of every row sum to one
    G = hq // hkv
    np.testing.assert_allclose(s_glo.sum(-1).cpu().numpy(), G * n, rtol=1e-4)
    np.testing.assert_allclose(s_loc.sum(-1).cpu().numpy(), G * w, rtol=1e-4)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("group", [1, 2, 3, 4])
def test_score_every_remainder_of_interior_stages(group, mode):
    """The pipelined loops of both passes take whole trips of 4 stages (6 in f32 mode); what does not fill
    a trip goes through the masked loop.  Lengths 32 apart walk through every remainder, for every group size
    (the trip counts stages of all q-heads of a group), plus one ragged length."""
    lengths = [1312 + 32 * i for i in range(6 if mode == B.EMS_F32 else 4)] + [1333]
    for d in ([64, 128] if group in (1, 3) else [64]):
        for n in lengths:
            _log("score remainders: group", group, "d", d, "n", n, "mode", mode)
            inp = ems_inputs.small(1, group, 1, d, n, seed=n + group)
            p = B.EmsParams(1, group, 1, d, n, 32, dtype=mode)
            s_glo, s_loc, lse = B.ems_global_local_score(p, dev_tensor(inp.q, mode), dev_tensor(inp.k, mode), want_lse=True)
            torch.cuda.synchronize()
            o_glo, o_loc, o_lse = ems_ref.score(ref_params(p), inp.f32("q"), inp.f32("k"), want_lse=True)
            assert_rel(s_glo.cpu().numpy(), o_glo, RTOL[mode], f"s_glo n={n} d={d}")
            assert_rel(s_loc.cpu().numpy(), o_loc, RTOL[mode], f"s_loc n={n} d={d}")
            np.testing.assert_allclose(lse.cpu().numpy(), o_lse, rtol=0, atol=2e-5 if mode == B.EMS_F32 else 2e-2)


def test_score_custom_scale_and_large_logits():
    """Logits of magnitude ~40: the running maximum of pass 1 has to do its job."""
    b, hq, hkv, d, n, w = 1, 2, 2, 128, 600, 16
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=77, scale=2.0)
    for mode in MODES:
        p = B.EmsParams(b, hq, hkv, d, n, w, softmax_scale=0.3, dtype=mode)
        s_glo, s_loc = B.ems_global_local_score(p, dev_tensor(inp.q, mode), dev_tensor(inp.k, mode))
        o_glo, o_loc = ems_ref.score(ref_params(p), inp.f32("q"), inp.f32("k"))
        assert_rel(s_glo.cpu().numpy(), o_glo, max(RTOL[mode], 1e-4), "s_glo")
        assert_rel(s_loc.cpu().numpy(), o_loc, max(RTOL[mode], 1e-4), "s_loc")


def test_score_zero_queries_is_harmonic():
    """Closed form (uniform rows): s_glo[j] = G * sum_{i>=j} 1/(i+1), on the GPU itself."""
    b, hq, hkv, d, n, w = 1, 4, 2, 128, 1500, 40
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=5)
    p = B.EmsParams(b, hq, hkv, d, n, w)
    q = torch.zeros((b, hq, n, d), dtype=torch.bfloat16, device="cuda")
    s_glo, s_loc = B.ems_global_local_score(p, q, dev_tensor(inp.k, B.EMS_BF16))
    inv = 1.0 / np.arange(1, n + 1)
    tail = np.cumsum(inv[::-1])[::-1]
    np.testing.assert_allclose(s_glo[0, 0].cpu().numpy(), 2 * tail, rtol=1e-5)
    np.testing.assert_allclose(s_loc[0, 1].cpu().numpy(),
                               2 * np.array([tail[max(j, n - w)] for j in range(n)]), rtol=1e-5)


def test_score_runs_are_bit_identical_and_heads_independent():
    b, hq, hkv, d, n, w = 2, 8, 2, 128, 1300, 32
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=9)
    p = B.EmsParams(b, hq, hkv, d, n, w)
    q, k = dev_tensor(inp.q, B.EMS_BF16), dev_tensor(inp.k, B.EMS_BF16)
    a = B.ems_global_local_score(p, q, k)
    c = B.ems_global_local_score(p, q, k)
    assert torch.equal(a[0], c[0]) and torch.equal(a[1], c[1])
    p1 = B.EmsParams(1, 4, 1, d, n, w)
    one = B.ems_global_local_score(p1, q[1:, 4:].contiguous(), k[1:, 1:].contiguous())
    assert torch.equal(one[0][0, 0], a[0][1, 1]) and torch.equal(one[1][0, 0], a[1][1, 1])


# ---------------------------------------------------------------------------- select
SELECT_SHAPES = [
    # (bh, n, w, budget, r, pool)
    (3, 1024, 32, 64, 0.5, 7),
    (2, 4099, 32, 256, 0.5, 7),
    (2, 3000, 64, 128, 3.0, 1),
    (1, 200, 10, 190, 5.0, 3),       # N_tbm clamped, everything kept or merged
    (1, 70000, 64, 2048, 0.5, 7),    # long sequences: chunks of 2048 positions over many blocks per head
    (2, 33, 1, 2, 0.0, 1),
    (3, 8192, 32, 100, 0.5, 7),      # the longest sequence the one-block kernel takes
    (3, 8193, 32, 100, 0.5, 7),      # the shortest the chunked kernels take: a second chunk of one position
    (2, 20000, 2047, 4000, 1.0, 5),  # window ends inside a chunk; a large budget (many candidates)
    (1, 12288, 4096, 8000, 0.5, 63), # whole chunks inside the window; widest pooling kernel
    (2, 10000, 8, 9000, 0.5, 1),     # nearly everything kept: the candidate list is almost the whole head
    (1, 1000003, 64, 3000, 0.5, 7),  # 489 chunks: more than one chunk per thread when the factor is formed
    (1, 1 << 22, 64, 5000, 1.0, 7),  # the longest sequence the interface takes: 2048 chunks
]


def _rand_scores(bh, n, w, seed):
    rng = np.random.default_rng(seed)
    glo = (rng.random((1, bh, n)) ** 4 * 5 + 1e-3).astype(np.float32)
    loc = (rng.random((1, bh, n)) ** 6 * w / n * 20).astype(np.float32)
    return glo, loc


@pytest.mark.parametrize("shape", SELECT_SHAPES)
def test_select_matches_oracle(shape):
    bh, n, w, nb, r, pk = shape
    _log("select", shape)
    glo, loc = _rand_scores(bh, n, w, n)
    p = B.EmsParams(1, bh, bh, 128, n, w, nb, merge_ratio=r, pool_kernel=pk)
    imp, tbm, pooled = B.ems_select(p, torch.from_numpy(glo).cuda(), torch.from_numpy(loc).cuda(),
                                    want_pooled=True)
    imp, tbm, pooled = imp.cpu().numpy(), tbm.cpu().numpy(), pooled.cpu().numpy()
    rp = ref_params(p)
    o_pooled, o_imp, o_tbm = ems_ref.select(rp, glo, loc)
    assert_rel(pooled, o_pooled, 1e-5, "pooled score")
    # integer work is bit-exact given the keys: oracle partition of the GPU's own keys
    x_imp, x_tbm = ems_ref.partition(rp, pooled.astype(np.float64))
    np.testing.assert_array_equal(imp, x_imp)
    np.testing.assert_array_equal(tbm, x_tbm)
    # and against the full fp64 oracle with a band at the cuts
    for h in range(bh):
        check_band(imp[0, h], tbm[0, h], o_pooled[0, h], n - w, 1e-5)
        assert is_sorted_unique(imp[0, h]) and (tbm.shape[-1] == 0 or is_sorted_unique(tbm[0, h]))


@pytest.mark.parametrize("levels", [4, 1])
@pytest.mark.parametrize("n", [5000, 20000])
def test_select_exact_ties_rank_by_position(n, levels):
    """Scores quantised to a few levels (or all equal): almost everything ties, on the chunked path the
    candidate list is then most of the head; pooling off so the keys are exactly the inputs and the
    index sets must equal the oracle's exactly."""
    bh, w, nb = 2, 16, 300
    _log("select ties", n, levels)
    rng = np.random.default_rng(1)
    loc = rng.integers(1, levels + 1, (1, bh, n)).astype(np.float32)
    glo = np.full((1, bh, n), 1e-6, np.float32)      # aligned s_glo never wins the max
    p = B.EmsParams(1, bh, bh, 64, n, w, nb, merge_ratio=2.0, pool_kernel=1)
    imp, tbm = B.ems_select(p, torch.from_numpy(glo).cuda(), torch.from_numpy(loc).cuda())
    _, o_imp, o_tbm = ems_ref.select(ref_params(p), glo, loc)
    np.testing.assert_array_equal(imp.cpu().numpy(), o_imp)
    np.testing.assert_array_equal(tbm.cpu().numpy(), o_tbm)


# ---------------------------------------------------------------------------- evict-merge
MERGE_SHAPES = [
    # (b, hkv, d, n, w, budget, r)
    (1, 2, 64, 700, 16, 48, 1.5),
    (2, 2, 128, 1500, 32, 256, 0.5),
    (1, 3, 128, 4096, 64, 128, 3.0),
    (1, 1, 128, 3000, 32, 512, 2.0),       # centre list searched in 2 (bf16) / 4 (f32) slices
    (1, 2, 128, 12000, 32, 1100, 5.0),     # 5 / 9 slices; 5500 to-be-merged tokens: two LDS pieces in the merge
    (1, 1, 64, 9000, 16, 2300, 0.6),       # f32: 18 rounds of centres, two per slice
]


def _random_partition(p, seed):
    n_imp, n_tbm = B.ems_partition_sizes(p)
    rng = np.random.default_rng(seed)
    imp = np.empty((p.batch, p.kv_heads, n_imp), np.int32)
    tbm = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    for b in range(p.batch):
        for h in range(p.kv_heads):
            perm = rng.permutation(p.seq_len - p.window)
            imp[b, h] = np.sort(perm[:n_imp])
            tbm[b, h] = np.sort(perm[n_imp:n_imp + n_tbm])
    return imp, tbm


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("tau", [0.6, 0.22, -2.0, 2.0])
@pytest.mark.parametrize("shape", MERGE_SHAPES)
def test_evict_merge_matches_oracle(shape, tau, mode):
    b, hkv, d, n, w, nb, r = shape
    _log("evict_merge", shape, "tau", tau, "mode", mode)
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=nb)
    # plant near-duplicates so that tau = 0.6 merges something
    kf = inp.f32("k").copy()
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=tau, dtype=mode)
    imp, tbm = _random_partition(p, seed=nb + 1)
    rng = np.random.default_rng(3)
    for bb in range(b):
        for h in range(hkv):
            for t in tbm[bb, h, ::5]:
                c = imp[bb, h, rng.integers(0, imp.shape[-1])]
                kf[bb, h, t] = 0.8 * kf[bb, h, c] + 0.45 * kf[bb, h, t]
    inp.k = ems_inputs.f32_to_bf16_bits(kf)
    kf, vf = inp.f32("k"), inp.f32("v")

    out = B.ems_evict_merge(p, dev_tensor(inp.k, mode), dev_tensor(inp.v, mode),
                            torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda())
    out = {k_: v_.float().cpu().numpy() if v_.is_floating_point() else v_.cpu().numpy()
           for k_, v_ in out.items()}
    rp = ref_params(p)
    ref = ems_ref.evict_merge(rp, kf, vf, imp, tbm)
    n_imp, n_tbm = B.ems_partition_sizes(p)

    # destinations: equal except where the decision is inside float32 noise
    np.testing.assert_allclose(out["tbm_sim"], ref["tbm_sim"], rtol=0, atol=5e-6)
    np.testing.assert_allclose(out["k_norm"], ref["k_norm"], rtol=1e-6)
    n_diff = assert_dest_valid(out["tbm_dest"], ref["tbm_dest"], kf, imp, tbm, tau, nb)
    assert n_diff < 0.01 * ref["tbm_dest"].size
    # stage isolation: the oracle's average for the GPU's own destinations
    k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge(rp, kf, vf, imp, tbm, out["tbm_dest"])
    np.testing.assert_array_equal(out["kept_pos"], kept_ref)
    np.testing.assert_array_equal(out["slot_count"], cnt_ref)
    rtol = RTOL_MERGE[mode]
    for name, got, want in (("k_out", out["k_out"], k_ref), ("v_out", out["v_out"], v_ref)):
        # per-row floor: 1e-2 of the row's RMS
        rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
        err = np.abs(got - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))
        assert err.max() <= rtol, f"{name}: {err.max():.3e}"
    # rows nobody merged into, and the local rows, are bit-exact copies
    alone = cnt_ref[..., :n_imp] == 1
    src_k, src_v = (kf, vf)
    for bb in range(b):
        for h in range(hkv):
            rows = np.nonzero(alone[bb, h])[0]
            np.testing.assert_array_equal(out["k_out"][bb, h, rows], src_k[bb, h, imp[bb, h, rows]])
            np.testing.assert_array_equal(out["v_out"][bb, h, rows], src_v[bb, h, imp[bb, h, rows]])
            np.testing.assert_array_equal(out["k_out"][bb, h, n_imp:nb], src_k[bb, h, n - w:])
            np.testing.assert_array_equal(out["v_out"][bb, h, n_imp:nb], src_v[bb, h, n - w:])
    if tau >= 1:
        assert (out["tbm_dest"] == nb).all() and (out["slot_count"][..., -1] == n_tbm).all()
    if tau <= -1:
        assert (out["tbm_dest"] < n_imp).all() and (out["slot_count"][..., -1] == 0).all()
    if tau == 0.6:
        assert (out["tbm_dest"] < n_imp).any() and (out["tbm_dest"] == nb).any()


def test_evict_merge_many_centres():
    """12000 class centres (the destination search cuts them into 16 slices of three rounds each) and 6016
    to-be-merged tokens (two LDS pieces in the merge), checked like the small shapes."""
    test_evict_merge_matches_oracle((1, 1, 128, 40000, 32, 12032, 0.5), 0.22, B.EMS_BF16)


def test_merge_ratio_zero_is_bit_exact_gather():
    b, hkv, d, n, w, nb = 1, 2, 128, 900, 32, 100
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=4)
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=0.0)
    imp, tbm = _random_partition(p, seed=2)
    assert tbm.shape[-1] == 0
    k, v = dev_tensor(inp.k, B.EMS_BF16), dev_tensor(inp.v, B.EMS_BF16)
    out = B.ems_evict_merge(p, k, v, torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda())
    for h in range(hkv):
        kept = np.concatenate([imp[0, h], np.arange(n - w, n)])
        np.testing.assert_array_equal(out["kept_pos"][0, h].cpu().numpy(), kept)
        assert torch.equal(out["k_out"][0, h, :nb], k[0, h, torch.from_numpy(kept).cuda()])
        assert torch.equal(out["v_out"][0, h, :nb], v[0, h, torch.from_numpy(kept).cuda()])
        assert (out["k_out"][0, h, nb] == 0).all() and (out["v_out"][0, h, nb] == 0).all()
    assert (out["slot_count"][..., :-1] == 1).all() and (out["slot_count"][..., -1] == 0).all()


# ---------------------------------------------------------------------------- end to end
@pytest.mark.parametrize("mode", MODES)
def test_tiny_config_end_to_end(mode):
    """BASELINE config 1 (4 heads, D 64, N 1024, W 32, budget 64, r 0.5), full chain with
    every stage also checked in isolation on the GPU's own upstream output."""
    w = ems_inputs.WORKLOADS["tiny"]
    inp = ems_inputs.generate(w)
    for tau in (0.6, 0.3):
        p = B.EmsParams(w.batch, w.q_heads, w.kv_heads, w.head_dim, w.seq_len, w.window, w.budget,
                        merge_ratio=w.merge_ratio, tau=tau, pool_kernel=w.pool_kernel, dtype=mode)
        q, k, v = (dev_tensor(getattr(inp, x), mode) for x in "qkv")
        s_glo, s_loc = B.ems_global_local_score(p, q, k)
        imp, tbm, pooled = B.ems_select(p, s_glo, s_loc, want_pooled=True)
        out = B.ems_evict_merge(p, k, v, imp, tbm)
        out2 = B.ems_evict_merge(p, k, v, imp, tbm)
        for name in out:
            assert torch.equal(out[name], out2[name]), name        # reproducible bit for bit
        rp = ref_params(p)
        qf, kf, vf = inp.f32("q"), inp.f32("k"), inp.f32("v")
        o_glo, o_loc = ems_ref.score(rp, qf, kf)
        rtol = RTOL[mode]
        assert_rel(s_glo.cpu().numpy(), o_glo, rtol, "s_glo")
        assert_rel(s_loc.cpu().numpy(), o_loc, rtol, "s_loc")
        o_pooled, o_imp, o_tbm = ems_ref.select(rp, o_glo, o_loc)
        assert_rel(pooled.cpu().numpy(), o_pooled, rtol, "pooled")
        imp_n, tbm_n = imp.cpu().numpy(), tbm.cpu().numpy()
        for h in range(w.kv_heads):
            check_band(imp_n[0, h], tbm_n[0, h], o_pooled[0, h], w.seq_len - w.window, rtol)
        x_imp, x_tbm = ems_ref.partition(rp, pooled.cpu().numpy().astype(np.float64))
        np.testing.assert_array_equal(imp_n, x_imp)
        np.testing.assert_array_equal(tbm_n, x_tbm)
        ref = ems_ref.evict_merge(rp, kf, vf, imp_n, tbm_n)
        n_diff = assert_dest_valid(out["tbm_dest"].cpu().numpy(), ref["tbm_dest"], kf, imp_n, tbm_n, tau, w.budget)
        assert n_diff <= max(1, ref["tbm_dest"].size // 100)
        k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge(rp, kf, vf, imp_n, tbm_n,
                                                        out["tbm_dest"].cpu().numpy())
        np.testing.assert_array_equal(out["slot_count"].cpu().numpy(), cnt_ref)
        np.testing.assert_array_equal(out["kept_pos"].cpu().numpy(), kept_ref)
        for name, want in (("k_out", k_ref), ("v_out", v_ref)):
            got = out[name].float().cpu().numpy()
            rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
            err = np.abs(got - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))
            assert err.max() <= RTOL_MERGE[mode], f"{name}: {err.max():.3e}"
        assert out["k_out"].shape == (1, 4, w.budget + 1, w.head_dim)


@pytest.mark.parametrize("mode", MODES)
def test_score_split_calls_match_fused_call(mode):
    """Row log-sum-exp alone, then the column sums from it: same scores as the one call."""
    b, hq, hkv, d, n, w = 1, 4, 2, 128, 1111, 32
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=21)
    p = B.EmsParams(b, hq, hkv, d, n, w, dtype=mode)
    q, k = dev_tensor(inp.q, mode), dev_tensor(inp.k, mode)
    s_glo, s_loc, lse = B.ems_global_local_score(p, q, k, want_lse=True)
    lse2 = B.ems_attention_lse(p, q, k)
    assert torch.equal(lse, lse2)
    g2, l2 = B.ems_global_local_score_from_lse(p, q, k, lse2)
    assert_rel(g2.cpu().numpy(), s_glo.cpu().numpy(), 1e-5, "s_glo from lse")
    assert_rel(l2.cpu().numpy(), s_loc.cpu().numpy(), 1e-5, "s_loc from lse")
    # an lse computed by the oracle (as an attention kernel would hand over) works as well
    _, _, o_lse = ems_ref.score(ref_params(p), inp.f32("q"), inp.f32("k"), want_lse=True)
    o_glo, o_loc = ems_ref.score(ref_params(p), inp.f32("q"), inp.f32("k"))
    g3, l3 = B.ems_global_local_score_from_lse(p, q, k, torch.from_numpy(o_lse.astype(np.float32)).cuda())
    assert_rel(g3.cpu().numpy(), o_glo, max(RTOL[mode], 2e-5), "s_glo from oracle lse")
    assert_rel(l3.cpu().numpy(), o_loc, max(RTOL[mode], 2e-5), "s_loc from oracle lse")


# ---------------------------------------------------------------------------- expansion
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("tau", [0.6, -2.0, 2.0])
@pytest.mark.parametrize("shape", MERGE_SHAPES[:3])
def test_expand_matches_oracle(shape, tau, mode):
    """Shared-entry expansion of the GPU's own compact cache against the oracle's expansion
    of the same cache (App. A): positions exact, keys/values to the rounding of one product."""
    b, hkv, d, n, w, nb, r = shape
    _log("expand", shape, "tau", tau, "mode", mode)
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=nb + 7)
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=tau, dtype=mode)
    imp, tbm = _random_partition(p, seed=nb + 2)
    kf = inp.f32("k").copy()
    rng = np.random.default_rng(5)
    for bb in range(b):
        for h in range(hkv):
            for t in tbm[bb, h, ::4]:
                c = imp[bb, h, rng.integers(0, imp.shape[-1])]
                kf[bb, h, t] = 0.9 * kf[bb, h, c] + 0.4 * kf[bb, h, t]
    inp.k = ems_inputs.f32_to_bf16_bits(kf)
    tbm_d = torch.from_numpy(tbm).cuda()
    merged = B.ems_evict_merge(p, dev_tensor(inp.k, mode), dev_tensor(inp.v, mode),
                               torch.from_numpy(imp).cuda(), tbm_d)
    k_exp, v_exp, pos = B.ems_expand(p, merged, tbm_d)
    host = {k_: (v_.float().cpu().numpy() if v_.is_floating_point() else v_.cpu().numpy())
            for k_, v_ in merged.items()}
    ko, vo, po = ems_ref.expand(ref_params(p), host["k_out"], host["v_out"], host["kept_pos"], tbm,
                                host["tbm_dest"], host["k_norm"])
    np.testing.assert_array_equal(pos.cpu().numpy(), po)
    np.testing.assert_array_equal(v_exp.float().cpu().numpy(), vo)            # values are copies
    got = k_exp.float().cpu().numpy()
    rtol = 2.0 ** -8 if mode == B.EMS_BF16 else 1e-6                          # one rounding of n/n_c * k
    rms = np.sqrt((ko ** 2).mean(-1, keepdims=True))
    err = np.abs(got - ko) / np.maximum(np.abs(ko), 1e-2 * np.maximum(rms, 1e-30))
    assert err.max() <= rtol, err.max()
    n_imp, n_tbm = B.ems_partition_sizes(p)
    assert k_exp.shape == (b, hkv, n_imp + n_tbm + w, d)
    if tau >= 1:
        assert (pos[..., n_imp:n_imp + n_tbm] == -1).all()
    if tau == 0.6:
        sel = pos[..., n_imp:n_imp + n_tbm]
        assert (sel == -1).any() and (sel >= 0).any()


# ---------------------------------------------------------------------------- merge variants
def _unit64(x):
    x = x.astype(np.float64)
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("sim", [B.EMS_SIM_KEY, B.EMS_SIM_VALUE, B.EMS_SIM_KEY_VALUE])
@pytest.mark.parametrize("shape", MERGE_SHAPES[:3])
def test_evict_merge_variant_matches_oracle(shape, sim, weighted, mode):
    """Redundancy as key / value / key x value cosine (Sec. 4.1) and the score-weighted merge
    (Sec. 4.2) against the oracle's versions of both."""
    b, hkv, d, n, w, nb, r = shape
    tau = 0.5
    _log("variant", shape, "sim", sim, "weighted", weighted, "mode", mode)
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=nb + 11)
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=tau, dtype=mode)
    imp, tbm = _random_partition(p, seed=nb + 5)
    kf, vf = inp.f32("k").copy(), inp.f32("v").copy()
    rng = np.random.default_rng(9)
    for bb in range(b):
        for h in range(hkv):
            for t in tbm[bb, h, ::3]:                      # near-duplicates in keys AND values
                c = imp[bb, h, rng.integers(0, imp.shape[-1])]
                kf[bb, h, t] = 0.9 * kf[bb, h, c] + 0.3 * kf[bb, h, t]
                vf[bb, h, t] = 0.8 * vf[bb, h, c] + 0.35 * vf[bb, h, t]
    inp.k, inp.v = ems_inputs.f32_to_bf16_bits(kf), ems_inputs.f32_to_bf16_bits(vf)
    kf, vf = inp.f32("k"), inp.f32("v")
    wt = None
    if weighted:
        wt = rng.uniform(0.0, 2.0, (b, hkv, n)).astype(np.float32)
        wt[..., ::7] = 0.0
        wt[..., 3::11] = -0.5                               # counts as 0

    out = B.ems_evict_merge_variant(p, sim, dev_tensor(inp.k, mode), dev_tensor(inp.v, mode),
                                    None if wt is None else torch.from_numpy(wt).cuda(),
                                    torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda())
    out = {k_: v_.float().cpu().numpy() if v_.is_floating_point() else v_.cpu().numpy()
           for k_, v_ in out.items()}
    rp = ref_params(p)
    d_ref, s_ref, n_ref = ems_ref.dest_sim(rp, sim, kf, vf, imp, tbm)
    n_imp, n_tbm = B.ems_partition_sizes(p)
    np.testing.assert_allclose(out["tbm_sim"], s_ref, rtol=0, atol=1e-5)
    np.testing.assert_allclose(out["k_norm"], n_ref, rtol=1e-6)
    differ = out["tbm_dest"] != d_ref
    for bb, h, i in zip(*np.nonzero(differ)):
        ck = _unit64(kf[bb, h, imp[bb, h]]) @ _unit64(kf[bb, h, tbm[bb, h, i]])
        cv = _unit64(vf[bb, h, imp[bb, h]]) @ _unit64(vf[bb, h, tbm[bb, h, i]])
        top2 = np.sort([ck, cv, ck * cv][sim])[-2:]
        assert top2[1] - top2[0] < 4e-5 or abs(top2[1] - tau) < 4e-5, (bb, h, i, top2)
    assert differ.mean() < 0.01
    assert (out["tbm_dest"] < n_imp).any() and (out["tbm_dest"] == nb).any()

    if weighted:
        k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge_weighted(rp, kf, vf, wt, imp, tbm, out["tbm_dest"])
    else:
        k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge(rp, kf, vf, imp, tbm, out["tbm_dest"])
    np.testing.assert_array_equal(out["kept_pos"], kept_ref)
    np.testing.assert_array_equal(out["slot_count"], cnt_ref)
    for name, got, want in (("k_out", out["k_out"], k_ref), ("v_out", out["v_out"], v_ref)):
        rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
        err = np.abs(got - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))
        assert err.max() <= RTOL_MERGE[mode], f"{name}: {err.max():.3e}"


def test_variant_with_key_cosine_and_no_weights_is_evict_merge():
    b, hkv, d, n, w, nb, r = MERGE_SHAPES[1]
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=77)
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=0.2)
    imp, tbm = _random_partition(p, seed=78)
    k, v = dev_tensor(inp.k, B.EMS_BF16), dev_tensor(inp.v, B.EMS_BF16)
    i_d, t_d = torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda()
    a = B.ems_evict_merge(p, k, v, i_d, t_d)
    c = B.ems_evict_merge_variant(p, B.EMS_SIM_KEY, k, v, None, i_d, t_d)
    for name in a:
        assert torch.equal(a[name].view(torch.uint8), c[name].view(torch.uint8)), name
    # constant weights: same destinations, same averages up to the rounding of the weights' products
    ones = torch.full((b, hkv, n), 0.5, device="cuda")
    e = B.ems_evict_merge_variant(p, B.EMS_SIM_KEY, k, v, ones, i_d, t_d)
    assert torch.equal(a["tbm_dest"], e["tbm_dest"]) and torch.equal(a["slot_count"], e["slot_count"])
    torch.testing.assert_close(e["v_out"].float(), a["v_out"].float(), rtol=2e-2, atol=1e-3)


def test_all_zero_weights_keep_the_centres_on_gpu():
    b, hkv, d, n, w, nb, r = MERGE_SHAPES[0]
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=79)
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=-2.0)
    imp, tbm = _random_partition(p, seed=80)
    k, v = dev_tensor(inp.k, B.EMS_BF16), dev_tensor(inp.v, B.EMS_BF16)
    i_d, t_d = torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda()
    o = B.ems_evict_merge_variant(p, B.EMS_SIM_KEY_VALUE, k, v, torch.zeros((b, hkv, n), device="cuda"), i_d, t_d)
    n_imp, _ = B.ems_partition_sizes(p)
    for h in range(hkv):
        assert torch.equal(o["k_out"][0, h, :n_imp], k[0, h, i_d[0, h].long()])
        assert torch.equal(o["v_out"][0, h, :n_imp], v[0, h, i_d[0, h].long()])
    assert (o["slot_count"][..., :n_imp].sum(-1) == n_imp + (o["tbm_dest"] < n_imp).sum(-1)).all()


# ---------------------------------------------------------------------------- degenerate inputs
@pytest.mark.parametrize("mode", MODES)
def test_zero_keys_identical_keys_and_full_budget(mode):
    """Keys of norm 0 have similarity 0 and unit key 0; identical keys tie and go to the lowest
    slot; budget = N leaves nothing to merge or evict."""
    b, hkv, d, n, w, nb, r = 1, 2, 64, 400, 8, 40, 2.0
    inp = ems_inputs.small(b, hkv, hkv, d, n, seed=31)
    kf = inp.f32("k").copy()
    p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=-0.5, dtype=mode)
    imp, tbm = _random_partition(p, seed=32)
    kf[0, 0, tbm[0, 0, 3]] = 0.0                         # a to-be-merged key of norm 0
    kf[0, 0, imp[0, 0, 5]] = 0.0                         # a centre of norm 0
    kf[0, 1, :] = kf[0, 1, 0]                            # head 1: every key the same
    inp.k = ems_inputs.f32_to_bf16_bits(kf)
    kf, vf = inp.f32("k"), inp.f32("v")
    out = B.ems_evict_merge(p, dev_tensor(inp.k, mode), dev_tensor(inp.v, mode),
                            torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda())
    out = {k_: v_.float().cpu().numpy() if v_.is_floating_point() else v_.cpu().numpy() for k_, v_ in out.items()}
    rp = ref_params(p)
    ref = ems_ref.evict_merge(rp, kf, vf, imp, tbm)
    assert out["tbm_sim"][0, 0, 3] == 0.0 and out["k_norm"][0, 0, p.budget - w + 3] == 0.0
    np.testing.assert_allclose(out["tbm_sim"][0, 0], ref["tbm_sim"][0, 0], atol=5e-6)
    # head 1: all cosines are 1 up to rounding, so any slot is within noise; the merged rows must
    # still be the oracle's average for the kernel's own destinations
    np.testing.assert_allclose(out["tbm_sim"][0, 1], 1.0, atol=5e-6)
    k_ref, v_ref, kept_ref, cnt_ref = ems_ref.merge(rp, kf, vf, imp, tbm, out["tbm_dest"])
    np.testing.assert_array_equal(out["slot_count"], cnt_ref)
    for name, want in (("k_out", k_ref), ("v_out", v_ref)):
        rms = np.sqrt((want ** 2).mean(-1, keepdims=True))
        err = np.abs(out[name] - want) / np.maximum(np.abs(want), 1e-2 * np.maximum(rms, 1e-30))
        assert err.max() <= RTOL_MERGE[mode], f"{name}: {err.max():.3e}"
    assert np.isfinite(out["k_out"]).all() and np.isfinite(out["v_out"]).all()

    # budget = N: every position before the window is a centre, nothing is merged or evicted
    p2 = B.EmsParams(b, hkv, hkv, d, n, w, n, merge_ratio=3.0, tau=0.6, dtype=mode)
    assert B.ems_partition_sizes(p2) == (n - w, 0)
    s = torch.rand((b, hkv, n), device="cuda")
    imp2, tbm2 = B.ems_select(p2, s, s.clone())
    assert torch.equal(imp2, torch.arange(n - w, device="cuda", dtype=torch.int32).expand(b, hkv, -1))
    kd, vd = dev_tensor(inp.k, mode), dev_tensor(inp.v, mode)
    o2 = B.ems_evict_merge(p2, kd, vd, imp2, tbm2)
    assert torch.equal(o2["k_out"][:, :, :n], kd) and torch.equal(o2["v_out"][:, :, :n], vd)
    assert (o2["slot_count"][..., :-1] == 1).all() and (o2["slot_count"][..., -1] == 0).all()


def test_probe_kernels_run():
    """The benchmark's measurement kernels: the copy copies, the MFMA loop leaves finite values."""
    from paper_2412_08521_amd import bench_probe
    src = torch.randn(1 << 20, device="cuda")
    dst = torch.zeros_like(src)
    assert bench_probe.probe_copy(src, dst) == 2 * src.numel() * 4
    sink = torch.empty(8 * 256, dtype=torch.float32, device="cuda")
    assert bench_probe.probe_mfma(8, 10, sink) == 8 * 4 * 10 * 32 * 32768
    torch.cuda.synchronize()
    assert torch.equal(src, dst) and torch.isfinite(sink).all()
    ops = torch.randn(bench_probe.OPERAND_BYTES // 2, device="cuda").to(torch.bfloat16)
    bench_probe.probe_mfma(8, 100, sink, operands=ops)
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all()
