"""The prefill path under HIP graph capture: the library never allocates, frees or synchronises,
so score -> select -> evict_merge -> expand can be recorded once and replayed.  Every replay is
checked against the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import ems_inputs
from gpu_util import dev_tensor
from paper_2412_08521_amd import binding as B

pytestmark = pytest.mark.gpu


# the second shape is long enough for the score passes to run as resident waves that draw their work
# from queues (cursors cleared inside the recorded sequence) and for the chunked select
@pytest.mark.parametrize("shape", [(2, 4, 2, 128, 1500, 32, 160, 1.5), (1, 32, 8, 64, 32768, 64, 256, 0.5)])
def test_prefill_path_replays_bit_identically_from_a_graph(shape):
    b, hq, hkv, d, n, w, nb, r = shape
    p = B.EmsParams(b, hq, hkv, d, n, w, nb, merge_ratio=r, tau=0.25, pool_kernel=7)
    n_imp, n_tbm = B.ems_partition_sizes(p)
    ws_bytes = B.ems_workspace_bytes(p)
    ws = [torch.empty(max(x, 256), dtype=torch.uint8, device="cuda") for x in ws_bytes]
    q = torch.empty((b, hq, n, d), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((b, hkv, n, d), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    s_glo = torch.empty((b, hkv, n), dtype=torch.float32, device="cuda")
    s_loc = torch.empty_like(s_glo)
    imp = torch.empty((b, hkv, n_imp), dtype=torch.int32, device="cuda")
    tbm = torch.empty((b, hkv, n_tbm), dtype=torch.int32, device="cuda")
    outs = B.alloc_evict_merge_outputs(p, "cuda")
    n_exp = n_imp + n_tbm + w
    k_exp = torch.empty((b, hkv, n_exp, d), dtype=torch.bfloat16, device="cuda")
    v_exp = torch.empty_like(k_exp)
    pos_exp = torch.empty((b, hkv, n_exp), dtype=torch.int32, device="cuda")

    def load(seed):
        inp = ems_inputs.small(b, hq, hkv, d, n, seed=seed)
        q.copy_(dev_tensor(inp.q, B.EMS_BF16)); k.copy_(dev_tensor(inp.k, B.EMS_BF16))
        v.copy_(dev_tensor(inp.v, B.EMS_BF16))

    def run():
        B.ems_global_local_score(p, q, k, ws=ws[0], out=(s_glo, s_loc))
        B.ems_select(p, s_glo, s_loc, ws=ws[1], out=(imp, tbm))
        B.ems_evict_merge(p, k, v, imp, tbm, ws=ws[2], out=outs)
        B.ems_expand(p, outs, tbm, out=(k_exp, v_exp, pos_exp))

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (s_glo, s_loc, imp, tbm, k_exp, v_exp, pos_exp, *outs.values())]

    load(1)
    run()                                             # eager warm-up before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()

    for seed in (1, 2, 3, 2):
        load(seed)
        run()
        eager = snapshot()
        for t in (s_glo, s_loc, imp, tbm, k_exp, v_exp, pos_exp, *outs.values()):
            t.zero_()                                 # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        replayed = snapshot()
        for a_, b_ in zip(eager, replayed):
            assert torch.equal(a_.view(torch.uint8), b_.view(torch.uint8)), seed
    assert (imp >= 0).all() and (outs["slot_count"].sum(-1) == n_imp + n_tbm).all()


def test_decode_steps_replay_from_one_captured_launch():
    """One ems_decode_step recorded with EMS_STEP_FROM_STATE, replayed for token after token (new
    q/k/v copied into the same buffers), against the same steps enqueued eagerly with a host-side
    counter on a second copy of the state: every array identical bit for bit."""
    b, hq, hkv, d, n, w, nb, r = 2, 8, 2, 128, 1500, 16, 160, 2.0
    p = B.EmsParams(b, hq, hkv, d, n, w, nb, merge_ratio=r, tau=0.3, pool_kernel=3)
    inp = ems_inputs.small(b, hq, hkv, d, n, seed=11)
    q, k, v = (dev_tensor(getattr(inp, x), B.EMS_BF16) for x in "qkv")
    s_glo, s_loc = B.ems_global_local_score(p, q, k)
    imp, tbm = B.ems_select(p, s_glo, s_loc)
    merged = B.ems_evict_merge(p, k, v, imp, tbm)
    states = []
    for _ in range(2):
        states.append(B.ems_decode_init(p, {n_: t_.clone() for n_, t_ in merged.items()}, tbm, s_glo, s_loc))
    eager_st, graph_st = states
    steps = 2 * w + 3
    gen = torch.Generator(device="cuda").manual_seed(3)
    qs = torch.randn((steps, b, hq, d), device="cuda", generator=gen).bfloat16()
    ks = torch.randn((steps, b, hkv, d), device="cuda", generator=gen).bfloat16()
    vs = torch.randn((steps, b, hkv, d), device="cuda", generator=gen).bfloat16()
    ws = torch.empty(max(B.ems_decode_workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")
    res_e = B.ems_decode_step(p, eager_st, 0, qs[0], ks[0], vs[0], ws=ws)       # allocates the outputs once
    qb, kb, vb = qs[0].clone(), ks[0].clone(), vs[0].clone()
    res_g = {n_: (t_.clone() if t_ is not None else None) for n_, t_ in res_e.items()}
    B.ems_decode_step(p, graph_st, B.EMS_STEP_FROM_STATE, qb, kb, vb, ws=ws, out=res_g)   # eager, from the counter
    torch.cuda.synchronize()
    assert int(graph_st.step_count.item()) == 1 and int(eager_st.step_count.item()) == 1

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.ems_decode_step(p, graph_st, B.EMS_STEP_FROM_STATE, qb, kb, vb, ws=ws, out=res_g)
    torch.cuda.synchronize()
    assert int(graph_st.step_count.item()) == 1            # capturing does not run the step

    for t in range(1, steps):
        B.ems_decode_step(p, eager_st, t, qs[t], ks[t], vs[t], ws=ws, out=res_e)
        torch.cuda.synchronize()
        eager_dec = res_e["decision"].clone()
        qb.copy_(qs[t]); kb.copy_(ks[t]); vb.copy_(vs[t])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(eager_dec, res_g["decision"]), t
        for name in B.STATE_FIELDS:
            assert torch.equal(getattr(eager_st, name).view(torch.uint8), getattr(graph_st, name).view(torch.uint8)), (t, name)
    assert int(graph_st.step_count.item()) == steps
