"""Shared set-up for the GPU parity tests: build the same cache with the oracle (CPU) and
with the library (GPU) from the same seeded inputs, and compare them."""
from __future__ import annotations

import numpy as np

import kvq_synth as S
from oracle import kvq_oracle as O


ATT_TOL = 2e-3          # the bar on the attention output: max abs error against the oracle's fp64 result
ATT_ABS_LIMIT = 3.5     # |reference| up to which that bar is applied as it stands


class AttStats:
    """What the attention checks of one test saw."""

    def __init__(self):
        self.reset()

    def reset(self):
        self.n = self.relaxed = 0
        self.max_abs = self.worst_ulps = 0.0


ATT_STATS = AttStats()


def att_err(got, ref, stats: AttStats = ATT_STATS):
    """Error of an attention output (`got`: the kernel's fp16 values as float64, `ref`: the oracle's
    fp64 values), in units in which ATT_TOL is the bar.

    Where |ref| <= 3.5 it is the plain absolute error.  fp16 cannot hold a larger value to 2e-3 (half
    an ulp is 1.95e-3 in [4, 8)), so there the output is compared with the oracle's own result rounded
    to fp16 and must lie within one fp16 ulp of it: the error is counted in ulps and scaled so that
    one ulp equals ATT_TOL.  `stats` counts how many elements each branch judged; the tests bound the
    second branch's share."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    big = np.abs(ref) > ATT_ABS_LIMIT
    err_abs = np.abs(got - ref)
    stats.n += int(ref.size)
    stats.relaxed += int(big.sum())
    worst = float(err_abs[~big].max()) if (~big).any() else 0.0
    stats.max_abs = max(stats.max_abs, worst)
    if big.any():
        ref16 = ref[big].astype(np.float32).astype(np.float16)
        ulps = np.abs(got[big] - ref16.astype(np.float64)) / np.spacing(np.abs(ref16)).astype(np.float64)
        stats.worst_ulps = max(stats.worst_ulps, float(ulps.max()))
        worst = max(worst, float(ulps.max()) * ATT_TOL)
    return worst


def merged_partials(cache, w: S.Workload, n_quant: int, fp_rows: int):
    """The decode launch's result BEFORE the rounding of the output to fp16: the fp32 partial results
    (m, l, o) that the workgroups of a unit exchange through the workspace, merged here in fp64.  Only
    for launches that split a unit over several workgroups (they leave the partials in the workspace).
    Returns float64 [batch, q_heads, head_dim]."""
    import torch
    from paper_2505_10938_amd import binding as B
    splits, _, _ = B.kvq_decode_launch_shape(cache.cfg, 1, n_quant, fp_rows)
    assert splits > 1, "one workgroup per unit: no partials are written"
    upl, g, hd = w.batch * w.kv_heads, w.q_heads // w.kv_heads, w.head_dim
    off = ((upl * 4 + 255) // 256) * 256
    raw = cache.workspace[off:off + upl * splits * g * (hd + 2) * 4].view(torch.float32).cpu().numpy()
    part = raw.astype(np.float64).reshape(upl, splits, g, hd + 2)
    m, l, o = part[..., 0], part[..., 1], part[..., 2:]
    scale = np.exp2(m - m.max(axis=1, keepdims=True))               # scores are kept in the log2 domain
    out = (o * scale[..., None]).sum(axis=1) / (l * scale).sum(axis=1)[..., None]
    return out.reshape(w.batch, w.kv_heads * g, hd)


def oracle_states(w: S.Workload, K: np.ndarray, V: np.ndarray, n_quant: int, units=None):
    """K, V: fp16 [batch, kv_heads, n, hd] of one layer.  Streams the first n_quant tokens of
    every unit (or of the units listed, as indices b * kv_heads + h) through the oracle group
    by group.  Returns a flat list of UnitState, in the order of `units`."""
    states = []
    G = w.group_k
    for ui in (range(w.batch * w.kv_heads) if units is None else units):
        b, h = divmod(ui, w.kv_heads)
        st = O.UnitState(w.head_dim, w.bits, G, w.group_v, w.outlier_budget, w.aux_capacity)
        for i in range(n_quant // G):
            st.append_group(K[b, h, i * G:(i + 1) * G], V[b, h, i * G:(i + 1) * G])
        states.append(st)
    return states


def gpu_cache(w: S.Workload, K: np.ndarray, V: np.ndarray, n_quant: int, n_res: int, layer: int = 0,
              max_seq: int | None = None, cache=None):
    """Same stream through the library: groups are placed in the ring and quantized one by
    one, then the n_res residual rows are loaded."""
    import torch
    from paper_2505_10938_amd import cache as KC
    G = w.group_k
    if cache is None:
        ms = max_seq or max(G, ((n_quant + G - 1) // G) * G)
        cfg = KC.make_config(w.layers, w.batch, w.q_heads, w.kv_heads, ms, w.bits, G, w.group_v, w.residual,
                             w.outlier_budget, w.aux_capacity, w.head_dim)
        cache = KC.KVCache(cfg)
    Kd = torch.from_numpy(K).cuda()
    Vd = torch.from_numpy(V).cuda()
    for i in range(n_quant // G):
        cache.load_residual(layer, Kd[:, :, i * G:(i + 1) * G], Vd[:, :, i * G:(i + 1) * G])
        cache.quantize_oldest(layer)
    if n_res:
        cache.load_residual(layer, Kd[:, :, n_quant:n_quant + n_res], Vd[:, :, n_quant:n_quant + n_res])
    torch.cuda.synchronize()
    return cache


def compare_state(cache, states, w: S.Workload, n_quant: int, layer: int = 0, units=None):
    """Bit-exact comparison of packed codes, steps/zeros, mask words, pool / auxiliary sets
    (token index, score, K and V rows) and the frozen flag, unit by unit (`units`: the unit
    indices the states belong to; default all, in order).  Returns the unit list."""
    cfg, sz = cache.cfg, cache.sizes
    upl = w.batch * w.kv_heads
    u0 = layer * upl
    nb = n_quant // 32
    ng = n_quant // w.group_k
    bb = 512 * w.bits
    k_codes, k_meta, v_codes, v_meta, mask = (t.cpu().numpy() for t in cache.dense_quantized())
    nblk, ngrp = cfg.max_seq // 32, cfg.max_seq // w.group_k
    nv = w.head_dim // w.group_v
    kc = k_codes[:sz.units * nblk * bb].reshape(sz.units, nblk, bb)
    vc = v_codes[:sz.units * nblk * bb].reshape(sz.units, nblk, bb)
    km = k_meta.view(np.uint16)[:sz.units * ngrp * 2 * w.head_dim].reshape(sz.units, ngrp, 2, w.head_dim)
    vm = v_meta.view(np.uint16)[:sz.units * nblk * 64 * nv].reshape(sz.units, nblk, 64 * nv)
    mk = mask.view(np.uint32)[:sz.units * nblk].reshape(sz.units, nblk)
    slots = sz.pool_slots
    pk = cache.pool_k.cpu().numpy().view(np.uint16)[:sz.units * slots * w.head_dim].reshape(sz.units, slots, w.head_dim)
    pv = cache.pool_v.cpu().numpy().view(np.uint16)[:sz.units * slots * w.head_dim].reshape(sz.units, slots, w.head_dim)
    pidx = cache.pool_idx.cpu().numpy().view(np.int32)[:sz.units * slots].reshape(sz.units, slots)
    psc = cache.pool_score.cpu().numpy().view(np.float64)[:sz.units * slots].reshape(sz.units, slots)
    pcnt = cache.pool_count.cpu().numpy().view(np.int32)[:sz.units]
    acnt = cache.aux_count.cpu().numpy().view(np.int32)[:sz.units]
    frz = cache.frozen.cpu().numpy().view(np.int32)[:sz.units]
    N = w.outlier_budget
    unit_list = list(range(len(states))) if units is None else list(units)
    for i, st in zip(unit_list, states):
        u = u0 + i
        ref = O.packed_unit(st)
        assert np.array_equal(km[u, :ng], ref["k_meta"].view(np.uint16)), f"k_meta unit {i}"
        assert np.array_equal(vm[u, :nb], ref["v_meta"].view(np.uint16)), f"v_meta unit {i}"
        assert np.array_equal(kc[u, :nb], ref["k_codes"]), f"k_codes unit {i}"
        assert np.array_equal(vc[u, :nb], ref["v_codes"]), f"v_codes unit {i}"
        assert np.array_equal(mk[u, :nb], ref["mask"]), f"mask unit {i}"
        assert bool(frz[u]) == st.frozen, f"frozen unit {i}"
        assert pcnt[u] == len(st.pool) and acnt[u] == len(st.aux), f"pool counts unit {i}"
        for name, members, lo, cnt in (("pool", st.pool, 0, pcnt[u]), ("aux", st.aux, N, acnt[u])):
            got = sorted(range(lo, lo + cnt), key=lambda s: pidx[u, s])
            want = sorted(members, key=lambda m: m["idx"])
            assert [int(pidx[u, s]) for s in got] == [m["idx"] for m in want], f"{name} index set unit {i}"
            for s, m in zip(got, want):
                assert psc[u, s] == m["score"], f"{name} score unit {i}"
                assert np.array_equal(pk[u, s], m["k"].view(np.uint16)), f"{name} K row unit {i}"
                assert np.array_equal(pv[u, s], m["v"].view(np.uint16)), f"{name} V row unit {i}"


def oracle_attention(w: S.Workload, states, Q: np.ndarray, K: np.ndarray, V: np.ndarray, n_quant: int, n_res: int,
                     units=None):
    """fp64 [batch, q_heads, hd] reference outputs of one decode step (rows of units that are
    not listed stay NaN)."""
    g = w.q_heads // w.kv_heads
    out = np.full((w.batch, w.q_heads, w.head_dim), np.nan)
    unit_list = list(range(w.batch * w.kv_heads)) if units is None else list(units)
    for ui, st in zip(unit_list, states):
        b, h = divmod(ui, w.kv_heads)
        o, _ = O.decode_attention(Q[b, h * g:(h + 1) * g], st, K[b, h, n_quant:n_quant + n_res],
                                  V[b, h, n_quant:n_quant + n_res])
        out[b, h * g:(h + 1) * g] = o
    return out
