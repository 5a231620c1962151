#!/usr/bin/env python3
"""Benchmark of the low-bit KV-cache decode hot path on one MI355X.

Workload: the 32-layer, batch-128 configuration (Mistral-7B shapes: 32 query / 8 kv heads, head_dim 128,
context 4096, 2-bit codes, G = Gv = 32, R = 128, N = 8).  A "step" is one decode step of the whole stack:
in every layer the new token's Key / Value rows join the cache and the attention over quantized cache +
residual ring + outlier pools is computed (one launch per layer, kvq_append_decode_attention); on the
steps on which the residual rings fill, every layer first traces and quantizes its oldest group
(kvq_append_trace_quantize) and then attends (kvq_decode_attention).  Steps are consecutive, as in real
decoding, and the start state is chosen so that one such group step falls into the timed region.  The
stack's cache (14.8 GB with 2-bit codes) is far larger than the last-level cache, so every launch reads
from HBM.  A workload of a single layer is run the same way on a stack of independent copies of that layer
(different contents), as many as it takes to exceed the last-level cache several times.

Cache contents come from a seeded generator on the device (same recipe as kvq_synth, which draws on the
host); the units the oracle checks are drawn on the host by kvq_synth and spliced in before the prompt is
quantized.  Prints ONE JSON line (metric = KV GB/s of algorithmic bytes; tokens/s alongside).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, vendor figure
DEFAULT_WORKLOAD = "mistral_7b_b128_4k"
# HBM bytes per decode launch from the FETCH_SIZE / WRITE_SIZE counters, scaled by what the same counters
# read for a plain device copy of known size; recorded values (profiles/decode_kernel_<workload>.md), the
# benchmark itself does not read hardware counters.
RECORDED_TRAFFIC = {"mistral_7b_b128_4k": 488_200_000, "llama2_7b_4k": 120_440_000}
SETTLE_PASSES = 10     # untimed passes of decode launches over the layers ahead of the warm-up steps
PAPER_CONTEXT = ("the paper reports 6.4x lower peak memory (A100 40G) and up to 2.3x end-to-end decoding throughput "
                 "(A800 80G) against fp16 for LLaMA-2-7B, no kernel-level figure")


def per_token_bytes(w):
    hd, b = w.head_dim, w.bits
    return 2 * hd * b // 8 + 4 * hd // w.group_k + 4 * hd // w.group_v


def decode_bytes(w, n_quant, n_res, pool_rows):
    """Algorithmic bytes of one layer's decode-attention launch: compressed cache, mask words, the
    full-precision rows (ring, pools), queries and outputs."""
    g = w.q_heads // w.kv_heads
    unit = n_quant * per_token_bytes(w) + n_quant // 8 + n_res * 4 * w.head_dim + pool_rows * 4 * w.head_dim \
        + 2 * g * w.head_dim * 2
    return unit * w.units


def group_step_bytes(w):
    """Algorithmic bytes of one layer's group step: G rows of K and V in, one packed group out."""
    hd, b, G = w.head_dim, w.bits, w.group_k
    return (G * hd * 4 + G * (2 * hd * b // 8 + 4 * hd // w.group_v) + 4 * hd + G // 8) * w.units


# ---- the oracle leg: worker processes (CPU only), forked before this process touches the GPU ------------------

def host_cores():
    n = len(os.sched_getaffinity(0))
    cap = int(os.environ.get("OMP_NUM_THREADS") or 16)       # the share of the host one GPU comes with
    return max(1, min(n, cap))


def _oracle_worker_init():
    global _BLAS_LIMIT
    try:
        from threadpoolctl import threadpool_limits
        _BLAS_LIMIT = threadpool_limits(limits=1)             # one thread per process: the processes fill the cores
    except Exception:                                         # pragma: no cover
        _BLAS_LIMIT = None


def _oracle_job(job):
    """One unit through the oracle: the prompt's groups, the reference output right after the prompt, the
    appended tokens (with the group steps the schedule asks for), the reference output of the last step, and
    a timed loop of decode-attention calls at that state."""
    import numpy as np
    import kvq_synth as S
    from oracle import kvq_oracle as O
    w = S.Workload(**job["workload"])
    layer, b, h, n0, n_steps, budget = job["layer"], job["b"], job["h"], job["n0"], job["n_steps"], job["budget"]
    G, R = w.group_k, w.residual
    K, V = S.unit_kv(w.seed, layer, b, h, n0 + n_steps, w.head_dim, w.rho)
    st = O.UnitState(w.head_dim, w.bits, G, w.group_v, w.outlier_budget, w.aux_capacity)
    nq = G * ((n0 - R) // G) if n0 >= R + G else 0
    for i in range(nq // G):
        st.append_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G])
    g = w.q_heads // w.kv_heads
    Q = S.layer_queries(w, layer, 0, "peaky")[b, h * g:(h + 1) * g]
    ref0, _ = O.decode_attention(Q, st, K[nq:n0], V[nq:n0])
    n, t_group, n_group = n0, 0.0, 0
    for _ in range(n_steps):
        n += 1
        if n - nq == R + G:
            t = time.perf_counter()
            st.append_group(K[nq:nq + G], V[nq:nq + G])
            t_group += time.perf_counter() - t
            n_group += 1
            nq += G
    ref1, _ = O.decode_attention(Q, st, K[nq:n], V[nq:n])
    reps, t0 = 0, time.perf_counter()
    elapsed = 0.0
    while elapsed < budget:
        O.decode_attention(Q, st, K[nq:n], V[nq:n])
        reps += 1
        elapsed = time.perf_counter() - t0
    return {"layer": layer, "b": b, "h": h, "ref0": ref0, "ref1": ref1, "reps": reps, "elapsed": elapsed,
            "t_group": t_group, "n_group": n_group, "pid": os.getpid(), "blas_limited": _BLAS_LIMIT is not None,
            "pool": len(st.pool) + len(st.aux)}


# ---- device-side synthetic inputs ---------------------------------------------------------------------------------

class DeviceSynth:
    """kvq_synth's recipe drawn with a seeded generator on the device: keys ~ N(0,1) with the (layer, kv
    head)'s four fixed channels x20 and each token an outlier token with probability rho (whole key row x10
    or x0.05), values ~ N(0,1).  The channels are kvq_synth's own; the draws are not (another generator)."""

    def __init__(self, w, device):
        import torch
        import kvq_synth as S
        self.w, self.S, self.torch = w, S, torch
        self.gen = torch.Generator(device=device)
        self.gen.manual_seed(1234 + w.seed)
        self.device = device

    def rows(self, layer, n):
        """fp16 [batch, kv_heads, n, head_dim] keys and values."""
        torch, w = self.torch, self.w
        shape = (w.batch, w.kv_heads, n, w.head_dim)
        K = torch.randn(shape, generator=self.gen, device=self.device, dtype=torch.float32)
        for h in range(w.kv_heads):
            ch = torch.from_numpy(self.S.outlier_channels(w.seed, layer, h, w.head_dim)).to(self.device)
            K[:, h, :, ch] *= 20.0
        is_out = torch.rand(shape[:3], generator=self.gen, device=self.device) < w.rho
        big = torch.rand(shape[:3], generator=self.gen, device=self.device) < 0.5
        scale = torch.where(is_out, torch.where(big, 10.0, 0.05), 1.0)
        K *= scale[..., None]
        V = torch.randn(shape, generator=self.gen, device=self.device, dtype=torch.float32)
        return K.to(torch.float16), V.to(torch.float16)


def run_stack(w, layers, steps, warmup, samples, pool, cpu_budget, label, value_per_step=0):
    """Consecutive decode steps over `layers` layer caches of workload w.  `samples`: (layer, b, h) units
    drawn on the host and checked against the oracle (through `pool`, a multiprocessing pool, or None).
    `value_per_step`: the schedule that quantizes Values at each step (needs a workload without tracing)."""
    import numpy as np
    import torch
    import kvq_synth as S
    from paper_2505_10938_amd import binding as KB
    from paper_2505_10938_amd import cache as KC

    dev = torch.device("cuda:0")
    G, R = w.group_k, w.residual
    total = steps + warmup
    # start state: the rings fill (a group step in every layer) in the middle of the timed steps, and the
    # quantized length right after it is the workload's
    # index of the step that fills the rings (a single timed step: right after it, so that the step timed is one
    # of the steps the roofline figure is taken from)
    fill_at = warmup + steps // 2 if steps >= 2 else warmup + 1
    nq_final = G * ((w.context - R) // G)
    n_fills = len([s for s in range(total) if s % G == fill_at % G])
    nq0 = nq_final - G * n_fills
    n_res0 = R + (G - 1 - fill_at) % G
    n0 = nq0 + n_res0
    assert nq0 >= 0 and n_res0 + fill_at % G + 1 == R + G
    max_seq = max(G, nq_final) + (G if value_per_step else 0)   # Values are quantized up to G - 1 tokens ahead of the Keys
    cfg = KC.make_config(layers, w.batch, w.q_heads, w.kv_heads, max_seq, w.bits, G, w.group_v, R, w.outlier_budget,
                         w.aux_capacity, w.head_dim, value_per_step=value_per_step)
    t_setup = time.time()
    jobs = None
    cache = KC.KVCache(cfg, device=dev)
    synth = DeviceSynth(w, dev)
    by_layer = {}
    for (l, b, h) in samples:
        by_layer.setdefault(l, []).append((b, h))
    new_k = torch.empty((total, layers, w.batch, w.kv_heads, w.head_dim), dtype=torch.float16, device=dev)
    new_v = torch.empty_like(new_k)
    for layer in range(layers):
        K, V = synth.rows(layer, n0 + total)
        for (b, h) in by_layer.get(layer, ()):                # host-drawn units, the ones the oracle sees
            k_host, v_host = S.unit_kv(w.seed, layer, b, h, n0 + total, w.head_dim, w.rho)
            K[b, h].copy_(torch.from_numpy(k_host))
            V[b, h].copy_(torch.from_numpy(v_host))
        cache.prefill(layer, K[:, :, :n0].contiguous(), V[:, :, :n0].contiguous())
        new_k[:, layer] = K[:, :, n0:].permute(2, 0, 1, 3)
        new_v[:, layer] = V[:, :, n0:].permute(2, 0, 1, 3)
        del K, V
    q = torch.stack([torch.from_numpy(S.layer_queries(w, layer, 0, "peaky")) for layer in range(layers)]).to(dev)
    out = torch.empty_like(q)
    torch.cuda.synchronize()
    assert cache.n_quant[0] == nq0 and cache.n_res[0] == n_res0
    # outputs right after the prompt (no append), for the parity check of the start state
    out0 = {}
    for layer in by_layer:
        out0[layer] = cache.decode(layer, q[layer]).cpu().numpy().astype(np.float64)
    pool_rows = float(cache.pool_count.view(torch.int32)[:layers * w.units].sum().item()
                      + cache.aux_count.view(torch.int32)[:layers * w.units].sum().item()) / (layers * w.units)
    t_setup = time.time() - t_setup

    def step(s):
        for layer in range(layers):
            cache.step(layer, new_k[s, layer], new_v[s, layer], q[layer], out[layer])

    # The device takes about ten such steps to settle after the set-up (the first ones run 5-8 % slower): plain
    # decode launches over the layers, which change no state, come before the warm-up steps asked for.
    for _ in range(SETTLE_PASSES):
        for layer in range(layers):
            cache.decode(layer, q[layer], out[layer])
    for s in range(warmup):
        step(s)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    step_bytes, step_kind, step_state = [], [], []
    t0 = time.perf_counter()
    for i in range(steps):
        marks[i].record()
        nq_before = cache.n_quant[0]
        step(warmup + i)
        grp = cache.n_quant[0] != nq_before
        step_kind.append(grp)
        step_state.append((cache.n_quant[0], cache.n_res[0]))
        step_bytes.append(layers * (decode_bytes(w, cache.n_quant[0], cache.n_res[0], pool_rows)
                                    + (group_step_bytes(w) if grp else 0)))
    marks[steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / steps
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    plain = [i for i in range(steps) if not step_kind[i]]
    # dominant kernel: the decode-attention launch.  A step without a group step is `layers` such launches
    # back to back and nothing else, so its duration / layers is the average launch (events on the launch stream)
    dec_us = sum(step_ms[i] for i in plain) * 1e3 / (len(plain) * layers)
    per_step_us = sorted(step_ms[i] * 1e3 / layers for i in plain)           # average launch of each such step
    dec_bytes = sum(step_bytes[i] for i in plain) / (len(plain) * layers)
    grp_steps = [i for i in range(steps) if step_kind[i]]
    assert cache.n_quant[0] == nq_final
    total_bytes = float(sum(step_bytes))
    g = w.q_heads // w.kv_heads
    res = {
        "label": label, "ms_per_step": ms_per_step, "value_GBps": total_bytes / dt / 1e9,
        "tokens_per_s": w.batch * steps * (1 if w.layers > 1 else layers) / dt, "dec_us": dec_us, "dec_bytes": dec_bytes,
        "group_steps": len(grp_steps), "setup_s": t_setup, "layers": layers,
        "context_range": [n0 + warmup + 1, n0 + total], "cache_GB": round(sum(
            getattr(cache, a).numel() for a in ("k_codes", "k_meta", "v_codes", "v_meta", "mask", "k_res", "v_res",
                                                 "pool_k", "pool_v")) / 1e9, 2),
        "launch_shape": KB.kvq_decode_launch_shape(cfg, 1, nq_final, R + 1 + w.outlier_budget + w.aux_capacity),
        "per_step": [(step_state[i][0], step_state[i][1], round(step_ms[i] * 1e3 / layers, 2), bool(step_kind[i]))
                     for i in range(steps)],
        "dec_us_median": per_step_us[len(per_step_us) // 2], "dec_us_min": per_step_us[0], "dec_us_max": per_step_us[-1],
    }
    if grp_steps:
        res["group_step_ms"] = sum(step_ms[i] for i in grp_steps) / len(grp_steps)
        res["plain_step_ms"] = sum(step_ms[i] for i in plain) / len(plain)
    if pool is not None and samples:
        # the oracle's processes start only now: while they run they take every host core, and the launches
        # of the timed region above must not wait for the host
        got1 = out.cpu().numpy().astype(np.float64)
        wd = {f: getattr(w, f) for f in w.__dataclass_fields__}
        jobs = pool.map_async(_oracle_job, [dict(workload=wd, layer=l, b=b, h=h, n0=n0, n_steps=total,
                                                 budget=cpu_budget) for (l, b, h) in samples], chunksize=1)
        results = jobs.get()
        from tests import helpers as H
        stats = H.AttStats()
        worst = 0.0
        for r in results:
            l, b, h = r["layer"], r["b"], r["h"]
            worst = max(worst, H.att_err(out0[l][b, h * g:(h + 1) * g], r["ref0"], stats),
                        H.att_err(got1[l, b, h * g:(h + 1) * g], r["ref1"], stats))
        res["parity"] = {"units": len(results), "elements": stats.n, "max_abs_err": stats.max_abs,
                         "elements_beyond_3.5": stats.relaxed, "worst_fp16_ulps_beyond_3.5": stats.worst_ulps,
                         "within_bar": bool(worst <= H.ATT_TOL)}
        if worst > H.ATT_TOL:
            print(f"bench.py: attention output differs from the oracle ({worst:.3e} in units of the bar)", file=sys.stderr)
        if cpu_budget > 0:
            by_pid = {}
            for r in results:
                by_pid[r["pid"]] = by_pid.get(r["pid"], 0.0) + r["elapsed"]
            wall = max(by_pid.values())                       # the busiest worker: the wall time of the timed loops
            unit_calls = sum(r["reps"] for r in results)
            unit_bytes = decode_bytes(w, nq_final, n0 + total - nq_final, pool_rows) / w.units
            t_dec = sum(r["elapsed"] for r in results) / unit_calls            # CPU seconds per unit and decode call
            t_grp = sum(r["t_group"] for r in results) / max(1, sum(r["n_group"] for r in results))
            res["cpu"] = {"decode_GBps": unit_bytes * unit_calls / wall / 1e9, "workers": len(by_pid),
                          "unit_calls": unit_calls, "wall_s": wall, "cpu_s_per_unit_decode": t_dec,
                          "cpu_s_per_unit_group_step": t_grp, "blas_limited": all(r["blas_limited"] for r in results),
                          "units": len(results)}
    del cache, new_k, new_v
    torch.cuda.empty_cache()
    return res


def fp16_attention(w, layers=3):
    """The same entry point with the whole context held in full precision (residual ring as long as the
    context, nothing quantized, no pool): the fp16 attention this cache replaces, one launch per layer."""
    import torch
    from paper_2505_10938_amd import cache as KC
    dev = torch.device("cuda:0")
    G = w.group_k
    cfg = KC.make_config(layers, w.batch, w.q_heads, w.kv_heads, G, w.bits, G, w.group_v, w.context, 0, 0, w.head_dim)
    cache = KC.KVCache(cfg, device=dev)
    synth = DeviceSynth(w, dev)
    for layer in range(layers):
        K, V = synth.rows(layer, w.context)
        cache.load_residual(layer, K, V)
        del K, V
    q = torch.randn((w.batch, w.q_heads, w.head_dim), device=dev).to(torch.float16)
    out = torch.empty_like(q)
    for layer in range(layers):
        cache.decode(layer, q, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 4
    e0.record()
    for _ in range(reps):
        for layer in range(layers):
            cache.decode(layer, q, out)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * layers)
    nbytes = w.units * (w.context * 4 * w.head_dim + 2 * (w.q_heads // w.kv_heads) * w.head_dim * 2)
    return {"us_per_launch": round(us, 3), "algorithmic_bytes": int(nbytes), "GBps": round(nbytes / (us * 1e-6) / 1e9, 1)}


def ragged_batch(copies=6):
    """A batch whose sequences differ in length (32 sequences of 128 .. 8192 tokens, 8 kv heads of 4 query
    heads, 2-bit): one decode-attention launch sized by the longest sequence, the same with a launch plan
    that deals the workgroups by length, and a batch of 32 sequences of the mean length for comparison.
    Each figure is the mean over `copies` caches taken in turn (more than the last-level cache holds)."""
    import torch
    import kvq_synth as S
    from paper_2505_10938_amd import cache as KC
    dev = torch.device("cuda:0")
    G, R, batch, qh, kvh = 32, 128, 32, 32, 8
    lengths = [128 + (8192 - 128) * i // (batch - 1) for i in range(batch)]
    mean_len = sum(lengths) // batch
    w = S.Workload("ragged_128_8192", layers=1, batch=batch, q_heads=qh, kv_heads=kvh, context=max(lengths), bits=2,
                   group_k=G, group_v=32, residual=R, outlier_budget=8, aux_capacity=32)
    synth = DeviceSynth(w, dev)
    K, V = synth.rows(0, max(lengths))

    def build(lens):
        cfg = KC.make_config(1, batch, qh, kvh, ((max(lens) + G - 1) // G) * G, 2, G, 32, R, 8, 32)
        caches = []
        for _ in range(copies):
            c = KC.RaggedKVCache(cfg, device=dev)
            for b, n in enumerate(lens):
                c.prefill_sequence(b, [K[b, :, :n].contiguous()], [V[b, :, :n].contiguous()])
            caches.append(c)
        return caches

    def timed(caches, planned):
        q = torch.randn((batch, qh, 128), device=dev).to(torch.float16)
        out = torch.empty_like(q)
        for c in caches:
            if planned:
                c.make_plan()
            c.decode(0, q, out, planned=planned)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 5
        e0.record()
        for _ in range(reps):
            for c in caches:
                c.decode(0, q, out, planned=planned)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * len(caches))

    def nbytes(lens):
        tot = 0
        for n in lens:
            nq = G * ((n - R) // G) if n >= R + G else 0
            tot += decode_bytes(w.with_(batch=1), nq, n - nq, 8)
        return tot

    ragged = build(lengths)
    t_plain, t_plan = timed(ragged, False), timed(ragged, True)
    del ragged
    torch.cuda.empty_cache()
    uniform = build([mean_len] * batch)
    t_mean = timed(uniform, False)
    del uniform, K, V
    torch.cuda.empty_cache()
    return {"sequences": batch, "tokens": f"{min(lengths)} .. {max(lengths)} (mean {mean_len})",
            "algorithmic_bytes": int(nbytes(lengths)),
            "decode_us_sized_by_the_longest": round(t_plain, 3), "decode_us_with_a_launch_plan": round(t_plan, 3),
            "decode_us_all_sequences_of_the_mean_length": round(t_mean, 3),
            "planned_over_mean_length": round(t_plan / t_mean, 3)}


def read_ceiling():
    """Read bandwidth a trivial 16-byte-load kernel reaches on this device over a buffer larger than the
    last-level cache (context for the roofline fraction, which stays quoted against 8 TB/s)."""
    import torch
    from paper_2505_10938_amd import binding as KB
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    big.fill_(1)
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    for _ in range(2):
        KB.kvq_stream_read(big, big.numel(), sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        KB.kvq_stream_read(big, big.numel(), sink)
    e1.record()
    torch.cuda.synchronize()
    return 5 * big.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9


def copies_for(w):
    """Layer caches a single-layer workload is run on, so that a pass reads several times the 256 MB
    last-level cache."""
    per_layer = decode_bytes(w, w.n_quant, w.n_res, w.outlier_budget)
    return max(8, min(64, math.ceil(2.5e9 / per_layer)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--cpu-seconds", type=float, default=20.0,
                    help="CPU work of the oracle's timed loops, summed over the sampled units, per host core")
    ap.add_argument("--no-cpu", action="store_true", help="no oracle leg (no parity check, no cpu_baseline)")
    ap.add_argument("--no-extras", action="store_true", help="only the workload itself: no 4-bit stack, no single-layer "
                                                              "line, no fp16 attention, no read ceiling")
    ap.add_argument("--decode-only", type=int, default=0, metavar="N",
                    help="profiling aid: after set-up run N passes of plain decode-attention launches over the layers "
                         "and exit")
    ap.add_argument("--prefill-only", type=int, default=0, metavar="N",
                    help="profiling aid: quantize one layer's prompt (kvq_prefill_quantize) N times into caches taken "
                         "in turn, print the time per call and exit")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling aid: run 8 plain device copies of MIB MiB and exit (scales the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(units shard over batch x kv-head with no exchange between GPUs)", file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.warmup < 0 or args.steps + args.warmup > 512:
        print("bench.py: 1 <= steps, 0 <= warmup, steps + warmup <= 512", file=sys.stderr)
        sys.exit(2)

    import kvq_synth as S
    w = S.WORKLOADS[args.workload]
    cores = host_cores()
    pool = None
    if not args.no_cpu and not args.decode_only and not args.copy_calibration and not args.prefill_only:
        import multiprocessing as mp
        # forked here, before anything initialises the GPU in this process; the workers never touch it
        pool = mp.get_context("fork").Pool(cores, initializer=_oracle_worker_init)

    import torch
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

    stacked = w.layers > 1
    layers = w.layers if stacked else copies_for(w)
    if args.decode_only:
        decode_only(w, layers, args.decode_only)
        return
    if args.prefill_only:
        prefill_only(w, args.prefill_only)
        return

    # units the oracle checks: three layers x three sequences x every kv head (fewer for a small workload)
    ls = sorted({0, layers // 2 + 1 if layers > 2 else 0, layers - 1})
    bs = sorted({0, w.batch // 2 - 1 if w.batch > 2 else 0, w.batch - 1})
    samples = [(l, b, h) for l in ls for b in bs for h in range(w.kv_heads)]
    if len(samples) > 96:
        samples = samples[::len(samples) // 72]
    # timed loops of about cpu_seconds per core in total
    budget = args.cpu_seconds * cores / len(samples)
    main_res = run_stack(w, layers, args.steps, args.warmup, samples if pool else [], pool, budget, w.name)

    frac = main_res["dec_bytes"] / (main_res["dec_us"] * 1e-6) / 1e9 / HBM_PEAK_GBPS
    # template arguments: query rows per kv head, bits, Value groups per token, paged cache, blocks per Key group
    kern = f"decode_kernel<{w.q_heads // w.kv_heads},{w.bits},{w.head_dim // w.group_v},false,{w.group_k // 32},false>"
    what = (f"{w.name}: {layers} layers" if stacked else f"{w.name}: {layers} independent copies of the layer")
    result = {
        "metric": "decode_attention_kv_GBps_2bit_1xMI355X" if w.bits == 2 else "decode_attention_kv_GBps",
        "value": round(main_res["value_GBps"], 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(main_res["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{what}, batch {w.batch}, {w.q_heads} q / {w.kv_heads} kv heads, head_dim {w.head_dim}, "
                               f"context {main_res['context_range'][0]}..{main_res['context_range'][1]}, {w.bits}-bit, "
                               f"G={w.group_k}, Gv={w.group_v}, R={w.residual}, N={w.outlier_budget}, A={w.aux_capacity}; "
                               f"step = one decode step of every layer (append + attention in one launch per layer; "
                               f"{main_res['group_steps']} of the {args.steps} timed steps first traced and quantized "
                               f"a group in every layer)",
                   "layers": layers, "cache_GB": main_res["cache_GB"], "settle_passes_before_warmup": SETTLE_PASSES,
                   "decode_launch_shape": dict(zip(("workgroups_per_unit", "wavefronts_per_workgroup",
                                                    "minichunks_per_workgroup"), main_res["launch_shape"]))},
        "tokens_per_s": round(main_res["tokens_per_s"], 1),
        "frac_of_hbm_peak": round(main_res["value_GBps"] / HBM_PEAK_GBPS, 4),
        "roofline": {"bound": "hbm", "kernel": kern + " (one launch of kvq_append_decode_attention)",
                     "achieved": round(main_res["dec_bytes"] / (main_res["dec_us"] * 1e-6) / 1e9, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(frac, 4),
                     "traffic": RECORDED_TRAFFIC.get(w.name),
                     "traffic_source": "recorded from rocprofv3 counter runs (profiles/), not measured in this run",
                     "algorithmic_bytes": int(main_res["dec_bytes"]), "us_per_launch": round(main_res["dec_us"], 3),
                     "us_per_launch_by_step": {"median": round(main_res["dec_us_median"], 3),
                                               "min": round(main_res["dec_us_min"], 3),
                                               "max": round(main_res["dec_us_max"], 3)}},
        "setup_s": round(main_res["setup_s"], 1),
    }
    if "group_step_ms" in main_res:
        result["step_with_group_quantize_ms"] = round(main_res["group_step_ms"], 4)
        result["step_without_group_quantize_ms"] = round(main_res["plain_step_ms"], 4)
    if "parity" in main_res:
        result["parity_vs_oracle"] = main_res["parity"]
        result["max_abs_err_vs_oracle"] = main_res["parity"]["max_abs_err"]
    if "cpu" in main_res:
        c = main_res["cpu"]
        # one decode step of the stack on the host: every unit's decode call, plus the group steps in the share
        # the timed region had
        units_total = layers * w.units
        cpu_step_s = units_total * (c["cpu_s_per_unit_decode"]
                                    + c["cpu_s_per_unit_group_step"] * main_res["group_steps"] / args.steps) / c["workers"]
        step_bytes = main_res["value_GBps"] * 1e9 * main_res["ms_per_step"] * 1e-3
        result["cpu_baseline"] = {
            "value": round(step_bytes / cpu_step_s / 1e9, 4), "unit": "GB/s", "cores": c["workers"], "kind": "oracle",
            "sample": f"{c['units']} of the {units_total} units (layers {ls}, sequences {bs}, every kv head), "
                      f"{c['unit_calls']} decode-attention calls of the numpy fp64 oracle in {c['workers']} processes "
                      f"(one per host core, BLAS threads per process "
                      f"{'limited to 1' if c['blas_limited'] else 'not limited'}), busiest process {c['wall_s']:.1f} s; "
                      f"the step's time is extrapolated from the sampled units to all {units_total} "
                      f"(x{units_total / c['units']:.0f}), group steps in the share of the timed region",
            "tokens_per_s": round(w.batch / cpu_step_s, 3),
            "decode_only_GBps": round(c["decode_GBps"], 4)}
    if pool is not None:
        pool.close()
        pool.join()

    if not args.no_extras:
        rc = read_ceiling()
        result["roofline"]["measured_read_ceiling"] = round(rc, 1)
        result["roofline"]["frac_of_measured_read_ceiling"] = round(frac * HBM_PEAK_GBPS / rc, 4)
        fp = fp16_attention(w)
        fp["speedup_of_quantized_decode"] = round(fp["us_per_launch"] / main_res["dec_us"], 3)
        result["fp16_attention_same_entry_point"] = fp
        extras = []
        if stacked and w.bits == 2:                            # the same stack with 4-bit codes
            extras.append((w.with_(name=w.name + "_4bit", bits=4), w.layers))
        if stacked and w.group_k == 32:
            # the same stack under the hyper-parameters of the paper's main tables (Experiments, "Details":
            # group size 128, residual length 32, 3 outlier tokens)
            extras.append((w.with_(name=w.name + "_g128_r32_n3", group_k=128, group_v=128, residual=32,
                                   outlier_budget=3), w.layers))
        if w.name == DEFAULT_WORKLOAD:                         # the single-layer MHA configuration, on copies
            w2 = S.WORKLOADS["llama2_7b_4k"]
            extras.append((w2, copies_for(w2)))
            # The two schedules the paper sets side by side (Experiments, "Details"; Efficiency comparison): Keys and
            # Values quantized together every G steps, against Values quantized at each step.  Same stack, same
            # data, no tracing in either (the per-step schedule is the one of the method without it).
            w0 = w.with_(name=w.name + "_no_tracing", outlier_budget=0, aux_capacity=0)
            ab = {}
            for key, vps in (("every_G_steps", 0), ("values_at_each_step", 1)):
                r = run_stack(w0, w.layers, args.steps, args.warmup, [], None, 0.0, key, value_per_step=vps)
                ab[key] = {"ms_per_step": round(r["ms_per_step"], 5), "tokens_per_s": round(r["tokens_per_s"], 1),
                           "step_without_group_quantize_ms": round(r.get("plain_step_ms", 0.0), 4),
                           "step_with_group_quantize_ms": round(r.get("group_step_ms", 0.0), 4),
                           "launches_per_layer_and_plain_step": 1 + vps}
            ab["slowdown_of_values_at_each_step"] = round(ab["values_at_each_step"]["ms_per_step"]
                                                          / ab["every_G_steps"]["ms_per_step"], 4)
            ab["value_launch_us_per_layer_and_step"] = round(
                (ab["values_at_each_step"]["step_without_group_quantize_ms"]
                 - ab["every_G_steps"]["step_without_group_quantize_ms"]) * 1e3 / w.layers, 3)
            ab["note"] = ("outlier_budget 0 in both; values_at_each_step adds one launch of kvq_quantize_value_tokens "
                          "per layer and step and its group steps quantize Keys only")
            result["value_schedule_ab"] = ab
            result["ragged_batch"] = ragged_batch()
        for (we, le) in extras:
            r = run_stack(we, le, args.steps, args.warmup, [], None, 0.0, we.name)
            result.setdefault("other_workloads", {})[we.name] = {
                "layers": le, "bits": we.bits, "group_k": we.group_k, "group_v": we.group_v, "residual": we.residual,
                "outlier_budget": we.outlier_budget, "ms_per_step": round(r["ms_per_step"], 5),
                "value_GBps": round(r["value_GBps"], 2), "tokens_per_s": round(r["tokens_per_s"], 1),
                "decode_us_per_launch": round(r["dec_us"], 3), "decode_algorithmic_bytes": int(r["dec_bytes"]),
                "decode_frac_of_hbm_peak": round(r["dec_bytes"] / (r["dec_us"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                "cache_GB": r["cache_GB"], "group_steps": r["group_steps"]}
    result["context"] = PAPER_CONTEXT
    print(json.dumps(result))


def decode_only(w, layers, passes):
    """Profiling aid: the stack's caches as the benchmark builds them, then `passes` passes of plain decode
    launches (kvq_decode_attention) over the layers."""
    import torch
    import kvq_synth as S
    from paper_2505_10938_amd import cache as KC
    dev = torch.device("cuda:0")
    G = w.group_k
    cfg = KC.make_config(layers, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G, w.group_v,
                         w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = KC.KVCache(cfg, device=dev)
    synth = DeviceSynth(w, dev)
    for layer in range(layers):
        K, V = synth.rows(layer, w.context)
        cache.prefill(layer, K, V)
        del K, V
    q = torch.stack([torch.from_numpy(S.layer_queries(w, layer, 0, "peaky")) for layer in range(layers)]).to(dev)
    out = torch.empty_like(q)
    torch.cuda.synchronize()
    for _ in range(passes):
        for layer in range(layers):
            cache.decode(layer, q[layer], out[layer])
    torch.cuda.synchronize()
    print(json.dumps({"decode_only_passes": passes, "layers": layers, "workload": w.name,
                      "n_quant": cache.n_quant[0], "n_res": cache.n_res[0]}))


def prefill_only(w, calls):
    """Profiling aid: one layer's prompt of the workload (its full batch and context) quantized `calls` times
    by kvq_prefill_quantize, each time into an empty cache of its own (the call expects empty pools); one
    untimed call ahead; the time per call from events around the calls."""
    import torch
    from paper_2505_10938_amd import cache as KC
    dev = torch.device("cuda:0")
    G = w.group_k
    calls = min(calls, 64)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G, w.group_v,
                         w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    caches = [KC.KVCache(cfg, device=dev) for _ in range(calls + 1)]
    K, V = DeviceSynth(w, dev).rows(0, w.context)
    caches[0].prefill(0, K, V)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for c in caches[1:]:
        c.prefill(0, K, V)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / calls
    fp16_bytes = 2 * K.numel() * 2
    print(json.dumps({"prefill_only_calls": calls, "workload": w.name, "units": w.batch * w.kv_heads,
                      "tokens": w.context, "us_per_call": round(us, 1),
                      "fp16_input_GBps": round(fp16_bytes / us / 1e3, 1),
                      "n_quant": caches[0].n_quant[0], "n_res": caches[0].n_res[0]}))


if __name__ == "__main__":
    main()
