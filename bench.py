#!/usr/bin/env python3
"""Benchmark of the EMS prefill compression path on one MI355X.

A "step" is one pass of the whole hot path -- Global/Local score, select, evict-then-merge --
over one layer's synthetic Q/K/V (already resident in HBM) of the named workload.  Prints ONE
JSON line: compressed tokens/s per layer, per-stage times, the roofline figures of the
dominant kernel (the key-stationary score pass) and the CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama3_8b_32k] [--tau 0.6]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_F32_MFMA_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_32k")
    ap.add_argument("--tau", type=float, default=0.6)
    ap.add_argument("--f32", action="store_true", help="validation mode (f32 MFMA)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--layers", type=int, default=1,
                    help="compress this many layers one after the other, each with its own seeded "
                         "inputs (the 128K workload is stated on 32): reports the per-layer median "
                         "and the total next to the headline figures, which stay those of --layer")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the timings of the entry points outside the headline step "
                         "(expansion, merge variants, decode-time update)")
    ap.add_argument("--decode-steps", type=int, default=64)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of Q (known size) so that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (every step is independent per "
                 "(batch, kv-head)); run with --gpus 1")

    import numpy as np
    import torch

    import ems_inputs
    from paper_2412_08521_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = ems_inputs.WORKLOADS[args.workload]
    mode = B.EMS_F32 if args.f32 else B.EMS_BF16
    p = B.EmsParams(w.batch, w.q_heads, w.kv_heads, w.head_dim, w.seq_len, w.window, w.budget,
                    merge_ratio=w.merge_ratio, tau=args.tau, pool_kernel=w.pool_kernel, dtype=mode)
    n_imp, n_tbm = B.ems_partition_sizes(p)

    # ---- synthetic inputs, generated on the host per batch entry and moved to HBM
    t0 = time.time()
    tdt = p.torch_dtype
    q = torch.empty((w.batch, w.q_heads, w.seq_len, w.head_dim), dtype=tdt, device="cuda")
    k = torch.empty((w.batch, w.kv_heads, w.seq_len, w.head_dim), dtype=tdt, device="cuda")
    v = torch.empty_like(k)
    sample = None
    for b in range(w.batch):
        inp = ems_inputs.generate(w, layer=args.layer, batch_slice=slice(b, b + 1))
        for name, dst in (("q", q), ("k", k), ("v", v)):
            bits = getattr(inp, name)
            if mode == B.EMS_F32:
                dst[b].copy_(torch.from_numpy(ems_inputs.bf16_bits_to_f32(bits[0])))
            else:
                dst[b].copy_(torch.from_numpy(bits[0].view(np.int16)).view(torch.bfloat16))
        if b == 0:
            G = w.q_heads // w.kv_heads
            sample = (inp.f32("q")[:, :G].copy(), inp.f32("k")[:, :1].copy(), inp.f32("v")[:, :1].copy())
        log(f"generated batch entry {b} ({time.time() - t0:.1f}s)")
        del inp

    # ---- everything the timed region touches is allocated up front
    ws_bytes = B.ems_workspace_bytes(p)
    ws_score = torch.empty(ws_bytes[0], dtype=torch.uint8, device="cuda")
    ws_select = torch.empty(ws_bytes[1], dtype=torch.uint8, device="cuda")
    ws_merge = torch.empty(ws_bytes[2], dtype=torch.uint8, device="cuda")
    s_glo = torch.empty((w.batch, w.kv_heads, w.seq_len), dtype=torch.float32, device="cuda")
    s_loc = torch.empty_like(s_glo)
    imp = torch.empty((w.batch, w.kv_heads, n_imp), dtype=torch.int32, device="cuda")
    tbm = torch.empty((w.batch, w.kv_heads, n_tbm), dtype=torch.int32, device="cuda")
    outs = B.alloc_evict_merge_outputs(p, "cuda")
    lse = torch.empty((w.batch, w.q_heads, w.seq_len), dtype=torch.float32, device="cuda")

    def score():
        B.ems_global_local_score(p, q, k, ws=ws_score, out=(s_glo, s_loc))

    def select():
        B.ems_select(p, s_glo, s_loc, ws=ws_select, out=(imp, tbm))

    def merge():
        B.ems_evict_merge(p, k, v, imp, tbm, ws=ws_merge, out=outs)

    def step():
        score(); select(); merge()

    def timed(fn, reps):
        """Average milliseconds per call over `reps` back-to-back calls (HIP events on the
        stream the kernels are launched on)."""
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b_.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b_) / reps

    if args.calibrate_copy:
        q_copy = torch.empty_like(q)
        q_copy.copy_(q)                      # reads and writes q.numel() * itemsize bytes
        torch.cuda.synchronize()
        log(f"calibration copy: {q.numel() * q.element_size()} bytes read and written")
        del q_copy
    for i in range(args.warmup):
        step()
        torch.cuda.synchronize()
        log(f"warmup {i} done")
    ms_step = timed(step, args.steps)
    log(f"timed {args.steps} steps: {ms_step:.3f} ms/step")

    K = args.steps
    stages = {"score": timed(score, K), "select": timed(select, K), "evict_merge": timed(merge, K)}
    ms_pass1 = timed(lambda: B.ems_attention_lse(p, q, k, ws=ws_score, out=lse), K)
    ms_pass2 = timed(lambda: B.ems_global_local_score_from_lse(p, q, k, lse, ws=ws_score,
                                                               out=(s_glo, s_loc)), K)
    log(f"stages ms: {stages}; pass1 {ms_pass1:.3f} pass2 {ms_pass2:.3f}")

    # ---- roofline of the dominant kernel: algorithmic flops = causal pairs only
    pairs = w.seq_len * (w.seq_len + 1) // 2
    flops_pass = 2.0 * w.head_dim * pairs * w.q_heads * w.batch
    peak = PEAK_F32_MFMA_TFLOPS if args.f32 else PEAK_BF16_TFLOPS
    achieved = flops_pass / (ms_pass2 * 1e-3) / 1e12
    # HBM traffic per launch comes from the committed rocprofv3 counter summary (two --pmc
    # runs, scaled by a plain copy); null when no summary exists for this workload
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"score_pass2_{w.name}.md")
    if os.path.exists(tpath) and not args.f32:
        import re
        m = re.search(r"hbm_bytes_per_launch:\s*([0-9.eE+]+)", open(tpath).read())
        traffic = float(m.group(1)) if m else None
    roofline = {"bound": "mfma", "kernel": "score_pass2_stream_kernel", "achieved": round(achieved, 2),
                "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": traffic,
                "traffic_source": (f"profiles/score_pass2_{w.name}.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                   "runs of this command, scaled by a plain copy; not measured by this process"
                                   if traffic is not None else None),
                "flops_per_launch": flops_pass,
                "ms_per_launch": round(ms_pass2, 4)}
    pass1 = {"kernel": "score_pass1_stream_kernel", "achieved": round(flops_pass / (ms_pass1 * 1e-3) / 1e12, 2),
             "unit": "TFLOP/s", "frac": round(flops_pass / (ms_pass1 * 1e-3) / 1e12 / peak, 4),
             "ms_per_launch": round(ms_pass1, 4)}

    # ---- the machine's own ceilings in the same process (bench-only library): a loop of bf16
    # MFMAs, 16 waves per compute unit, on operands that are all 1.0, on constants that differ
    # from lane to lane, and on random ones (the more bits toggle, the lower the clock the power
    # limit allows: the random-operand figure is the ceiling real inputs see), and a plain
    # 16-byte vector copy of Q
    from paper_2412_08521_amd import bench_probe
    sink = torch.empty(1024 * 256, dtype=torch.float32, device="cuda")
    ops = torch.randn(bench_probe.OPERAND_BYTES // 2, device="cuda").to(torch.bfloat16)
    bench_probe.probe_mfma(1024, 200, sink)
    torch.cuda.synchronize()
    probe_flops = 1024 * 4 * 2500 * 32 * 32768
    ms_mfma_const = timed(lambda: bench_probe.probe_mfma(1024, 2500, sink), 3)
    ms_mfma_rand = timed(lambda: bench_probe.probe_mfma(1024, 2500, sink, operands=ops), 3)
    ones = torch.ones(bench_probe.OPERAND_BYTES // 2, device="cuda", dtype=torch.bfloat16)
    ms_mfma_ones = timed(lambda: bench_probe.probe_mfma(1024, 2500, sink, operands=ones), 3)
    q_copy = torch.empty_like(q)
    bench_probe.probe_copy(q, q_copy)
    ms_copy = timed(lambda: bench_probe.probe_copy(q, q_copy), 5)
    copy_bytes = 2 * q.numel() * q.element_size()
    del q_copy
    ceilings = {"mfma_bf16_tflops_all_ones_operands": round(probe_flops / (ms_mfma_ones * 1e-3) / 1e12, 1),
                "mfma_bf16_tflops_constant_operands": round(probe_flops / (ms_mfma_const * 1e-3) / 1e12, 1),
                "mfma_bf16_tflops_random_operands": round(probe_flops / (ms_mfma_rand * 1e-3) / 1e12, 1),
                "copy_gbps": round(copy_bytes / (ms_copy * 1e-3) / 1e9, 1)}
    log(f"measured ceilings: {ceilings}")
    if not args.f32:
        roofline["frac_of_measured_ceiling"] = round(achieved / ceilings["mfma_bf16_tflops_random_operands"], 4)

    tokens = w.batch * w.seq_len
    result = {
        "metric": "compressed tokens/s per layer (score+evict+merge)",
        "value": round(tokens / (ms_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if args.f32 else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.q_heads,
                   "kv_heads": w.kv_heads, "head_dim": w.head_dim, "seq_len": w.seq_len,
                   "window": w.window, "budget": w.budget, "merge_ratio": w.merge_ratio,
                   "tau": args.tau, "pool_kernel": w.pool_kernel, "layer": args.layer},
        "stages_us": {k_: round(v_ * 1e3, 1) for k_, v_ in stages.items()},
        "roofline": roofline, "score_pass1": pass1, "ceilings": ceilings,
        # context, not the headline: what the step costs when the caller's attention kernel
        # hands over the row log-sum-exp and only the second pass runs (the paper's own design)
        "with_caller_lse": {"ms_per_step": round(ms_pass2 + stages["select"] + stages["evict_merge"], 4),
                            "value": round(tokens / ((ms_pass2 + stages["select"] + stages["evict_merge"]) * 1e-3), 1),
                            "unit": "tokens/s"},
    }

    # ---- several layers one after the other, each with its own seeded inputs
    if args.layers > 1:
        result["layers"] = run_layers(args, p, w, B, ems_inputs, torch, np, q, k, v, step,
                                      s_glo, s_loc, imp, tbm, outs, n_imp, n_tbm)
        log(f"layers: {result['layers']}")

    # ---- entry points outside the headline step, same shapes, reported on their own
    if not args.no_extras:
        result["extras_us"] = time_extras(args, p, w, B, torch, timed, k, v, s_glo, s_loc, imp, tbm,
                                          outs, ws_select, ws_merge)
        log(f"extras us: {result['extras_us']}")

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import ems_ref
        qs, ks, vs = sample
        G = w.q_heads // w.kv_heads
        rp = ems_ref.RefParams(1, G, 1, w.head_dim, w.seq_len, w.window, budget=w.budget,
                               merge_ratio=w.merge_ratio, tau=args.tau, pool_kernel=w.pool_kernel)
        t0 = time.time()
        o_glo, o_loc = ems_ref.score(rp, qs, ks)
        t_score = time.time() - t0
        t0 = time.time()
        _, o_imp, o_tbm = ems_ref.select(rp, o_glo, o_loc)
        ems_ref.evict_merge(rp, ks, vs, o_imp, o_tbm)
        t_rest = time.time() - t0
        t_layer = (t_score + t_rest) * w.batch * w.kv_heads
        result["cpu_baseline"] = {
            "value": round(tokens / t_layer, 2), "unit": "tokens/s", "cores": ems_ref.threads(),
            "kind": "oracle",
            "sample": (f"one of the {w.batch * w.kv_heads} (batch, kv-head) units at full length "
                       f"N={w.seq_len}: batch 0, kv-head 0 with its {G} q-heads (score "
                       f"{t_score:.2f}s, select+evict_merge {t_rest:.3f}s); layer time = unit "
                       f"time x {w.batch * w.kv_heads} (units are independent and cost the same)"),
        }
        log(f"cpu baseline: score {t_score:.2f}s rest {t_rest:.3f}s")

    print(json.dumps(result), flush=True)


def run_layers(args, p, w, B, ems_inputs, torch, np, q, k, v, step, s_glo, s_loc, imp, tbm, outs, n_imp, n_tbm):
    """One timed step per layer (HIP events), inputs of the layer generated on the host and moved
    to HBM before its timed region; afterwards, outside the timed region, the properties that hold
    at any size are asserted on the layer's outputs."""
    mode_f32 = p.dtype == B.EMS_F32
    G = w.q_heads // w.kv_heads
    per_layer = []
    for layer in range(args.layers):
        for b in range(w.batch):
            inp = ems_inputs.generate(w, layer=layer, batch_slice=slice(b, b + 1))
            for name, dst in (("q", q), ("k", k), ("v", v)):
                bits = getattr(inp, name)
                if mode_f32:
                    dst[b].copy_(torch.from_numpy(ems_inputs.bf16_bits_to_f32(bits[0])))
                else:
                    dst[b].copy_(torch.from_numpy(bits[0].view(np.int16)).view(torch.bfloat16))
            del inp
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        step()
        e1.record()
        torch.cuda.synchronize()
        per_layer.append(e0.elapsed_time(e1))
        # every causal softmax row sums to one; index sets are sorted, disjoint, in range; every
        # head emits budget rows that account for all N_imp + N_tbm tokens
        gs, ls = s_glo.double().sum(-1), s_loc.double().sum(-1)
        assert ((gs - G * w.seq_len).abs() <= 2e-4 * G * w.seq_len).all(), f"layer {layer}: s_glo row sums"
        assert ((ls - G * w.window).abs() <= 2e-4 * G * w.window).all(), f"layer {layer}: s_loc row sums"
        for idx, n in ((imp, n_imp), (tbm, n_tbm)):
            if n > 1:
                assert (idx[..., 1:] > idx[..., :-1]).all(), f"layer {layer}: index set not ascending"
            if n:
                assert int(idx.min()) >= 0 and int(idx.max()) < w.seq_len - w.window
        both = torch.cat([imp, tbm], -1).sort(-1).values
        assert (both[..., 1:] != both[..., :-1]).all(), f"layer {layer}: index sets overlap"
        assert (outs["slot_count"].sum(-1) == n_imp + n_tbm).all(), f"layer {layer}: slot counts"
        assert torch.isfinite(outs["k_out"].float()).all() and torch.isfinite(outs["v_out"].float()).all()
        log(f"layer {layer}: {per_layer[-1]:.3f} ms, invariants ok")
    total = float(sum(per_layer))
    return {"n": args.layers, "ms_per_layer_median": round(float(np.median(per_layer)), 4),
            "ms_per_layer_min": round(min(per_layer), 4), "ms_per_layer_max": round(max(per_layer), 4),
            "ms_total": round(total, 3),
            "tokens_per_s_over_all_layers": round(w.batch * w.seq_len * args.layers / (total * 1e-3), 1)}


def time_extras(args, p, w, B, torch, timed, k, v, s_glo, s_loc, imp, tbm, merged, ws_select, ws_merge):
    """Microseconds per call of ems_expand, ems_evict_merge_variant (key x value redundancy,
    score-weighted), ems_sparsity_rate, ems_redundancy_rate, ems_decode_init and ems_decode_step (average over --decode-steps
    consecutive generated tokens) on the workload's shapes; outputs allocated up front."""
    K = args.steps
    n_imp, n_tbm = B.ems_partition_sizes(p)
    n_exp = n_imp + n_tbm + w.window
    out = {}
    k_exp = torch.empty((w.batch, w.kv_heads, n_exp, w.head_dim), dtype=p.torch_dtype, device="cuda")
    v_exp = torch.empty_like(k_exp)
    pos_exp = torch.empty((w.batch, w.kv_heads, n_exp), dtype=torch.int32, device="cuda")
    out["expand"] = timed(lambda: B.ems_expand(p, merged, tbm, out=(k_exp, v_exp, pos_exp)), K) * 1e3
    pooled = B.ems_select(p, s_glo, s_loc, want_pooled=True, ws=ws_select)[2]
    outs2 = B.alloc_evict_merge_outputs(p, "cuda")
    out["evict_merge_kv_weighted"] = timed(
        lambda: B.ems_evict_merge_variant(p, B.EMS_SIM_KEY_VALUE, k, v, pooled, imp, tbm, ws=ws_merge,
                                          out=outs2), K) * 1e3
    out["sparsity_rate"] = timed(lambda: B.ems_sparsity_rate(p, 0.9, s_glo, s_loc), K) * 1e3
    out["redundancy_rate"] = timed(lambda: B.ems_redundancy_rate(p, k, v), max(1, K // 5)) * 1e3
    g = p.q_heads // p.kv_heads
    if g in (1, 2, 4, 8):
        B.ems_evict_merge(p, k, v, imp, tbm, ws=ws_merge, out=outs2)     # a cache the steps may overwrite
        state = [B.DecodeState(p, outs2["k_out"], outs2["v_out"])]
        out["decode_init"] = timed(lambda: B.ems_decode_init(p, outs2, tbm, s_glo, s_loc, state=state[0]), K) * 1e3
        n = args.decode_steps
        gen = torch.Generator(device="cuda").manual_seed(7)
        qn = torch.randn((n, w.batch, w.q_heads, w.head_dim), device="cuda", generator=gen).to(p.torch_dtype)
        kn = torch.randn((n, w.batch, w.kv_heads, w.head_dim), device="cuda", generator=gen).to(p.torch_dtype)
        vn = torch.randn((n, w.batch, w.kv_heads, w.head_dim), device="cuda", generator=gen).to(p.torch_dtype)
        ws = torch.empty(B.ems_decode_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        res = dict(decision=torch.empty((w.batch, w.kv_heads, 2), dtype=torch.int32, device="cuda"),
                   sim=torch.empty((w.batch, w.kv_heads), dtype=torch.float32, device="cuda"), attn=None)
        t = [0]

        def one():
            B.ems_decode_step(p, state[0], t[0], qn[t[0] % n], kn[t[0] % n], vn[t[0] % n], ws=ws, out=res)
            t[0] += 1
        for _ in range(4):
            one()
        out["decode_step"] = timed(one, n) * 1e3
        # the same step recorded once (step counter read from the state) and replayed from a HIP graph
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                B.ems_decode_step(p, state[0], B.EMS_STEP_FROM_STATE, qn[0], kn[0], vn[0], ws=ws, out=res)
        torch.cuda.synchronize()
        out["decode_step_graph_replay"] = timed(graph.replay, n) * 1e3
        e = 4 if args.f32 else 2
        per_head = (w.budget + n_imp) * w.head_dim * e + n_exp * 40
        out["decode_step_algorithmic_bytes"] = per_head * w.batch * w.kv_heads
    return {k_: round(v_, 1) for k_, v_ in out.items()}


if __name__ == "__main__":
    main()
