#!/usr/bin/env python3
"""Benchmark of the low-bit KV-cache decode hot path on one MI355X.

A "step" is one pass of the whole hot path of one layer over one batch: append the new
token's K/V to the residual ring, which fills it; trace outliers of the oldest group and
quantize it (these three in one launch, kvq_append_trace_quantize); decode attention over the
quantized cache + residual + pools (kvq_decode_attention).  Every step runs on its own copy of
the cache, so each one starts from the same state and reads from HBM rather than from the
256 MB last-level cache.

Prints ONE JSON line (metric = KV GB/s of algorithmic bytes; tokens/s alongside).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, vendor figure
# HBM bytes per decode launch from the FETCH_SIZE / WRITE_SIZE counters, scaled by what the same
# counters read for a plain device copy of known size (profiles/decode_kernel_<workload>.md).
MEASURED_TRAFFIC = {"llama2_7b_4k": 120_440_000}


def algorithmic_bytes(w, n_quant, n_res, pool_rows):
    """Bytes one decode step must move for one layer (compressed cache + full-precision rows +
    queries + outputs), and bytes of one group quantization (rows in, packed group out)."""
    hd, b, G, Gv = w.head_dim, w.bits, w.group_k, w.group_v
    g = w.q_heads // w.kv_heads
    per_tok = 2 * hd * b // 8 + 4 * hd // G + 4 * hd // Gv
    dec_unit = n_quant * per_tok + n_quant // 8 + n_res * 4 * hd + pool_rows * (4 * hd) + 2 * g * hd * 2
    quant_unit = G * hd * 4 + G * (2 * hd * b // 8 + 4 * hd // Gv) + 4 * hd + G // 8
    return dec_unit * w.units, quant_unit * w.units


def stream_mode(args, w):
    """Consecutive decode steps of one layer shape, the cadence of real decoding: every step appends a
    token and attends; every G-th also traces and quantizes a group.  Eight copies of the cache take
    turns (eight layers of a model, in effect), so that a step reads its cache from HBM."""
    import torch
    import kvq_synth as S
    from paper_2505_10938_amd import cache as KC
    G, steps, copies = w.group_k, args.stream, 8
    K, V = S.layer_kv(w, 0, w.context + steps)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + steps + G - 1) // G) * G, w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    base = KC.KVCache(cfg)
    base.prefill(0, Kd[:, :, :w.context].contiguous(), Vd[:, :, :w.context].contiguous())
    inst = [base] + [base.clone() for _ in range(copies - 1)]
    qd = torch.from_numpy(S.layer_queries(w, 0)).cuda()
    rows = [(Kd[:, :, w.context + s].contiguous(), Vd[:, :, w.context + s].contiguous()) for s in range(steps)]
    outs = [torch.empty_like(qd) for _ in inst]
    torch.cuda.synchronize()
    group_steps = 0
    t0 = time.perf_counter()
    for s in range(steps):
        for c, o in zip(inst, outs):
            before = c.n_quant[0]
            c.step(0, rows[s][0], rows[s][1], qd, o)
            group_steps += c.n_quant[0] != before
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us = dt * 1e6 / (steps * copies)
    n_mid = w.context + steps // 2
    nq_mid = G * ((n_mid - w.residual) // G)
    pool_rows = int(base.pool_count.view(torch.int32)[:w.units].sum().item()
                    + base.aux_count.view(torch.int32)[:w.units].sum().item()) / w.units
    dec_bytes, quant_bytes = algorithmic_bytes(w, nq_mid, n_mid - nq_mid, pool_rows)
    step_bytes = dec_bytes + quant_bytes * group_steps / (steps * copies)
    print(json.dumps({
        "metric": "decode_attention_kv_GBps_2bit_1xMI355X" if w.bits == 2 else "decode_attention_kv_GBps",
        "value": round(step_bytes / (us * 1e-6) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": steps * copies,
        "warmup": 0, "ms_per_step": round(us * 1e-3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {steps} consecutive decode steps from context {w.context} on each of "
                               f"{copies} cache copies in turn (batch {w.batch}, {w.q_heads} q / {w.kv_heads} kv heads, "
                               f"{w.bits}-bit, G={G}, R={w.residual}, N={w.outlier_budget}); {group_steps} of the "
                               f"{steps * copies} steps traced and quantized a group"},
        "tokens_per_s": round(w.batch / (us * 1e-6), 1),
        "frac_of_hbm_peak": round(step_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama2_7b_4k")
    ap.add_argument("--cpu-units", type=int, default=32, help="units of the workload the oracle is timed on")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--stream", type=int, default=0, metavar="STEPS",
                    help="instead of the step benchmark: STEPS consecutive decode steps (append + attention, a group "
                         "step whenever a ring fills) on each of 8 cache copies taken in turn, from a prompt of the "
                         "workload's context quantized in one call")
    ap.add_argument("--decode-only", type=int, default=0, metavar="N",
                    help="profiling aid: after set-up run N decode-attention launches over the cache copies and exit")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling aid: run 8 plain device copies of MIB MiB and exit (scales the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(units shard over batch x kv-head with no exchange between GPUs)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import kvq_synth as S
    from paper_2505_10938_amd import cache as KC

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "copies": 8}))
        return
    w = S.WORKLOADS[args.workload]
    assert w.layers == 1, "bench.py times one layer; multi-layer workloads are run layer by layer elsewhere"
    G = w.group_k
    if args.stream:
        stream_mode(args, w)
        return
    # the decode sees the context right after a group was quantized: the longest one of that kind
    # within the workload's context (for the default workload it is the workload's context itself)
    ctx = w.residual + G * ((w.context - w.residual) // G)
    nq_final, nres_final = ctx - w.residual, w.residual
    nq0 = nq_final - G                                        # state before the step: ring one short of full
    t_setup = time.time()
    K, V = S.layer_kv(w, 0)                                   # fp16 [B, Hkv, context, hd]
    Q = S.layer_queries(w, 0)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((ctx + G - 1) // G) * G, w.bits, G, w.group_v,
                         w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    base = KC.KVCache(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    for i in range(nq0 // G):
        base.load_residual(0, Kd[:, :, i * G:(i + 1) * G], Vd[:, :, i * G:(i + 1) * G])
        base.quantize_oldest(0)
    n_pre = w.residual + G - 1
    base.load_residual(0, Kd[:, :, nq0:nq0 + n_pre], Vd[:, :, nq0:nq0 + n_pre])
    k_new = Kd[:, :, nq0 + n_pre].contiguous()
    v_new = Vd[:, :, nq0 + n_pre].contiguous()
    qd = torch.from_numpy(Q).cuda()
    torch.cuda.synchronize()
    n_inst = args.steps + args.warmup
    inst = [base] + [base.clone() for _ in range(n_inst - 1)]
    outs = [torch.empty_like(qd) for _ in range(n_inst)]
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    if args.decode_only:
        for c in inst:                                        # bring every copy to the post-step state
            c.append(0, k_new, v_new)
        torch.cuda.synchronize()
        for i in range(args.decode_only):
            inst[i % n_inst].decode(0, qd, outs[i % n_inst])
        torch.cuda.synchronize()
        print(json.dumps({"decode_only_launches": args.decode_only, "workload": w.name}))
        return

    def step(c, out):
        quantized = c.append(0, k_new, v_new)                 # fills the ring -> trace + quantize
        assert quantized
        c.decode(0, qd, out)

    for i in range(args.warmup):
        step(inst[i], outs[i])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, n_inst):
        step(inst[i], outs[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    assert all(c.n_quant[0] == nq_final and c.n_res[0] == nres_final for c in inst)

    # dominant kernel: the decode-attention launch, timed back to back over the distinct
    # cache copies with events on the launch stream
    pool_rows = int(base.pool_count.view(torch.int32)[:w.units].sum().item()
                    + base.aux_count.view(torch.int32)[:w.units].sum().item()) / w.units
    dec_bytes, quant_bytes = algorithmic_bytes(w, nq_final, nres_final, pool_rows)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 3
    for i in range(min(4, n_inst)):
        inst[i].decode(0, qd, outs[i])
    torch.cuda.synchronize()
    dec_ms = 0.0
    for _ in range(reps):                                     # each pass over the copies is timed on its own
        e0.record()
        for i in range(n_inst):
            inst[i].decode(0, qd, outs[i])
        e1.record()
        torch.cuda.synchronize()
        dec_ms += e0.elapsed_time(e1)
    dec_us = dec_ms * 1e3 / (reps * n_inst)
    # same launch on ONE copy: served from the last-level cache, reported for context only
    e0.record()
    for _ in range(reps * 8):
        inst[0].decode(0, qd, outs[0])
    e1.record()
    torch.cuda.synchronize()
    hot_us = e0.elapsed_time(e1) * 1e3 / (reps * 8)

    # read bandwidth a trivial 16-byte-load kernel reaches on this device over a buffer larger than
    # the last-level cache (context for the roofline fraction, which stays quoted against 8 TB/s)
    from paper_2505_10938_amd import binding as KB
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    big.fill_(1)
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    for _ in range(2):
        KB.kvq_stream_read(big, big.numel(), sink)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        KB.kvq_stream_read(big, big.numel(), sink)
    e1.record()
    torch.cuda.synchronize()
    read_ceiling = 5 * big.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del big

    # the same entry point with the whole context held in full precision (residual ring as long as
    # the context, nothing quantized, no pool): the fp16 attention this cache replaces
    fp_cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, G, w.bits, G, w.group_v, ctx, 0, 0, w.head_dim)
    fp_inst = []
    for _ in range(3):
        c = KC.KVCache(fp_cfg)
        c.load_residual(0, Kd[:, :, :ctx], Vd[:, :, :ctx])
        fp_inst.append(c)
    for c in fp_inst:
        c.decode(0, qd, outs[0])
    torch.cuda.synchronize()
    e0.record()
    for _ in range(4):
        for c in fp_inst:
            c.decode(0, qd, outs[0])
    e1.record()
    torch.cuda.synchronize()
    fp_us = e0.elapsed_time(e1) * 1e3 / 12
    fp_bytes = w.units * (ctx * 4 * w.head_dim + 2 * (w.q_heads // w.kv_heads) * w.head_dim * 2)
    del fp_inst

    # a step on which the ring does not fill (G - 1 of G decode steps): the append rides in the
    # decode launch, one launch per layer.  Every copy takes one such step (its ring holds R rows).
    steady_out = torch.empty_like(qd)
    steady_us = None
    if G > 2:
        inst[0].step(0, k_new, v_new, qd, steady_out)
        torch.cuda.synchronize()
        e0.record()
        for c in inst[1:]:
            c.step(0, k_new, v_new, qd, steady_out)
        e1.record()
        torch.cuda.synchronize()
        steady_us = e0.elapsed_time(e1) * 1e3 / (n_inst - 1)
        assert all(c.n_res[0] == nres_final + 1 for c in inst)

    result = {
        "metric": "decode_attention_kv_GBps_2bit_1xMI355X" if w.bits == 2 else "decode_attention_kv_GBps",
        "value": round((dec_bytes + quant_bytes) / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{w.name}: 1 layer, batch {w.batch}, {w.q_heads} q / {w.kv_heads} kv heads, "
                               f"head_dim {w.head_dim}, context {ctx}, {w.bits}-bit, G={G}, Gv={w.group_v}, "
                               f"R={w.residual}, N={w.outlier_budget}, A={w.aux_capacity}; step = append + trace + "
                               f"quantize one group (one launch) + decode attention (one launch)",
                   "cache_copies": n_inst},
        "tokens_per_s": round(w.batch / (ms_per_step * 1e-3), 1),
        "frac_of_hbm_peak": round((dec_bytes + quant_bytes) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": {"bound": "hbm", "kernel": "decode attention (one launch of kvq_decode_attention)",
                     "achieved": round(dec_bytes / (dec_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(dec_bytes / (dec_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4), "traffic": MEASURED_TRAFFIC.get(w.name),
                     "algorithmic_bytes": int(dec_bytes), "us_per_launch": round(dec_us, 3),
                     "us_per_launch_cache_resident": round(hot_us, 3),
                     "measured_read_ceiling": round(read_ceiling, 1),
                     "frac_of_measured_read_ceiling": round(dec_bytes / (dec_us * 1e-6) / 1e9 / read_ceiling, 4)},
        "fp16_attention_same_entry_point": {
            "us_per_launch": round(fp_us, 3), "algorithmic_bytes": int(fp_bytes),
            "GBps": round(fp_bytes / (fp_us * 1e-6) / 1e9, 1),
            "speedup_of_quantized_decode": round(fp_us / dec_us, 3)},
        "setup_s": round(t_setup, 1),
    }
    if steady_us is not None:
        mean_us = (ms_per_step * 1e3 + (G - 1) * steady_us) / G
        result["step_without_group_quantize"] = {
            "us_per_step": round(steady_us, 3), "launches": 1,
            "mean_us_over_a_group_of_steps": round(mean_us, 3),
            "tokens_per_s_mean": round(w.batch / (mean_us * 1e-6), 1)}

    # parity spot check + CPU baseline on a bounded sample of units
    if not args.no_cpu:
        from oracle import kvq_oracle as O
        from tests import helpers as H
        try:
            from threadpoolctl import threadpool_limits
        except Exception:                                       # pragma: no cover
            threadpool_limits = None
        nu = min(args.cpu_units, w.units)
        units = [(u // w.kv_heads, u % w.kv_heads) for u in range(nu)]
        g = w.q_heads // w.kv_heads
        states = []
        for (b, h) in units:
            st = O.UnitState(w.head_dim, w.bits, G, w.group_v, w.outlier_budget, w.aux_capacity)
            for i in range(nq0 // G):
                st.append_group(K[b, h, i * G:(i + 1) * G], V[b, h, i * G:(i + 1) * G])
            states.append(st)
        import copy
        tp_limit = threadpool_limits(limits=1) if threadpool_limits else None
        t_cpu, reps_cpu, ref = 0.0, 0, None
        while t_cpu < 12.0 and reps_cpu < 400:
            sts = copy.deepcopy(states)
            t1 = time.perf_counter()
            ref = []
            for (b, h), st in zip(units, sts):
                st.append_group(K[b, h, nq0:nq0 + G], V[b, h, nq0:nq0 + G])          # trace + quantize
                o, _ = O.decode_attention(Q[b, h * g:(h + 1) * g], st, K[b, h, nq_final:ctx],
                                          V[b, h, nq_final:ctx])
                ref.append(o)
            t_cpu += time.perf_counter() - t1
            reps_cpu += 1
        if tp_limit is not None:
            tp_limit.__exit__(None, None, None)
        cpu_step_s = t_cpu / reps_cpu
        got = outs[-1].cpu().numpy().astype(np.float64)
        err = max(float(np.abs(got[b, h * g:(h + 1) * g] - o).max()) for (b, h), o in zip(units, ref))
        result["max_abs_err_vs_oracle"] = err
        frac_units = nu / w.units
        result["cpu_baseline"] = {
            "value": round((dec_bytes + quant_bytes) * frac_units / cpu_step_s / 1e9, 4), "unit": "GB/s",
            "cores": 1, "kind": "oracle",
            "sample": f"{nu} of {w.units} units of the same workload, full step (trace + quantize + decode), "
                      f"{reps_cpu} repetitions, numpy fp64 oracle, BLAS threads limited to 1",
            "tokens_per_s": round(w.batch * frac_units / cpu_step_s, 2),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
