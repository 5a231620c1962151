"""GPU parity: the HIP path against the CPU oracle on the same seeded inputs, through the
C ABI.  Packed codes, steps/zeros, mask words, outlier/auxiliary sets: bit-exact.  Attention
output: max abs error <= 2e-3 against the oracle's fp64 result (fp16 output, fp32
accumulation on the GPU)."""
import numpy as np
import pytest

import kvq_synth as S
from paper_2505_10938_amd import binding as B
from tests import helpers as H

pytestmark = pytest.mark.gpu

ATT_TOL = H.ATT_TOL
att_err = H.att_err          # absolute error where |ref| <= 3.5, fp16 ulps of the rounded oracle result beyond


@pytest.fixture(autouse=True)
def relaxed_share(request):
    """Every test states how many output elements were judged on the relaxed branch of att_err (|ref| >
    3.5: within one fp16 ulp of the oracle's rounded result) and keeps that share below 0.1 % (a test
    whose inputs are scaled up on purpose says so with the `relaxed_share` marker; a test with few
    outputs may have three such elements)."""
    H.ATT_STATS.reset()
    yield
    st = H.ATT_STATS
    marker = request.node.get_closest_marker("relaxed_share")
    limit = marker.args[0] if marker else 1e-3
    if st.n:
        print(f"\n[attention check] {request.node.name}: {st.n} elements; max abs err {st.max_abs:.3e} on |ref| <= "
              f"{H.ATT_ABS_LIMIT}; {st.relaxed} elements ({100.0 * st.relaxed / st.n:.4f} %) beyond, worst "
              f"{st.worst_ulps:.2f} fp16 ulp from the rounded oracle result")
        assert st.relaxed <= max(3, limit * st.n), (st.relaxed, st.n)


def run_case(w: S.Workload, regimes=("peaky", "diffuse")):
    import torch
    K, V = S.layer_kv(w, 0)
    nq, nr = w.n_quant, w.n_res
    states = H.oracle_states(w, K, V, nq)
    cache = H.gpu_cache(w, K, V, nq, nr)
    H.compare_state(cache, states, w, nq)
    errs = {}
    for regime in regimes:
        Q = S.layer_queries(w, 0, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, nq, nr)
        out = cache.decode(0, torch.from_numpy(Q).cuda())
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        errs[regime] = att_err(got, ref)
        assert errs[regime] <= ATT_TOL, (regime, errs)
    return errs


def small(name, **kw):
    base = dict(layers=1, batch=2, q_heads=2, kv_heads=2, context=1024 + 77)
    base.update(kw)
    return S.Workload(name, **base)


def test_config1_small_mha():
    run_case(S.WORKLOADS["small_mha_1k"])


@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_gqa_ratios(g):
    run_case(small(f"g{g}", q_heads=2 * g, context=1500))


@pytest.mark.parametrize("g", [4, 8])
@pytest.mark.parametrize("Gv", [32, 64, 128])
def test_gqa_ratios_four_bit(g, Gv):
    # the kernel instances of four query heads per workgroup row with 4-bit codes (g = 8: two rows)
    run_case(small(f"g{g}b4v{Gv}", q_heads=2 * g, bits=4, group_v=Gv, context=1500))


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("G,Gv,R,N", [(32, 32, 128, 8), (64, 64, 32, 3), (128, 128, 32, 3), (32, 128, 0, 4)])
def test_hyper_parameter_grid(bits, G, Gv, R, N):
    run_case(small(f"b{bits}G{G}", bits=bits, group_k=G, group_v=Gv, residual=R, outlier_budget=N, q_heads=4,
                   context=1024 + 200))


def test_budget_zero_plain_group_quantization():
    run_case(small("n0", outlier_budget=0))


def test_short_sequence_nothing_quantized():
    w = small("short", context=100)
    assert w.n_quant == 0
    run_case(w)


def test_single_token():
    run_case(small("one", context=1))


def test_warmup_and_freeze_budget_equals_group():
    # N = G = 32 with many outlier tokens: the first group is all outliers, evictions fill the
    # auxiliary pool and tracing stops early
    w = small("freeze", outlier_budget=32, aux_capacity=32, rho=0.05, context=2048 + 128)
    K, V = S.layer_kv(w, 0)
    states = H.oracle_states(w, K, V, w.n_quant)
    assert any(st.frozen for st in states)
    run_case(w)


# ---- full-size configurations: every unit runs on the GPU, the oracle checks sampled units -----------

def run_sampled(w: S.Workload, units, regimes=("peaky", "diffuse")):
    import torch
    K, V = S.layer_kv(w, 0)
    nq, nr = w.n_quant, w.n_res
    states = H.oracle_states(w, K, V, nq, units)
    cache = H.gpu_cache(w, K, V, nq, nr)
    H.compare_state(cache, states, w, nq, units=units)
    g = w.q_heads // w.kv_heads
    for regime in regimes:
        Q = S.layer_queries(w, 0, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, nq, nr, units)
        out = cache.decode(0, torch.from_numpy(Q).cuda())
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        for ui in units:
            b, h = divmod(ui, w.kv_heads)
            err = att_err(got[b, h * g:(h + 1) * g], ref[b, h * g:(h + 1) * g])
            assert err <= ATT_TOL, (w.name, regime, ui, err)
    return cache


def paged_copy(cache, seed=5, spare=100):
    """The same cache contents in a paged cache whose pages are dealt at random."""
    import torch
    from paper_2505_10938_amd import cache as KC
    c = cache.cfg
    groups = c.max_seq // c.group_k
    other = KC.KVCache(c, n_pages=c.batch * groups + spare)
    deal = np.random.default_rng(seed).permutation(other.n_pages)[:c.batch * groups].reshape(c.batch, groups)
    other.page_table.copy_(torch.from_numpy(deal.astype(np.int32)))
    table = other.page_table.long()
    for name in ("k_codes", "k_meta", "v_codes", "v_meta", "mask"):
        dense, pool = getattr(cache, name), getattr(other, name)
        per_group = dense.numel() // (c.layers * c.batch * c.kv_heads * groups)
        pages = pool[:c.layers * c.kv_heads * other.n_pages * per_group].view(c.layers, c.kv_heads, other.n_pages, per_group)
        src = dense[:c.layers * c.batch * c.kv_heads * groups * per_group].view(c.layers, c.batch, c.kv_heads, groups, per_group)
        pages[:, :, table] = src.permute(0, 2, 1, 3, 4)
    for name in ("k_res", "v_res", "pool_k", "pool_v", "pool_idx", "pool_score", "pool_count", "aux_count", "frozen"):
        getattr(other, name).copy_(getattr(cache, name))
    other.n_quant, other.res_start, other.n_res = list(cache.n_quant), list(cache.res_start), list(cache.n_res)
    return other


def test_full_size_llama2_7b_4k_sampled_units():
    # the benchmark workload in the benchmark's launch shape (one workgroup of 8 wavefronts per unit)
    import torch
    w = S.WORKLOADS["llama2_7b_4k"]
    cache = run_sampled(w, [0, 37, 130, 255])
    # the same contents behind a page table (31 744 pages dealt at random): the same outputs, bit for bit
    q = torch.from_numpy(S.layer_queries(w, 0, 0, "peaky")).cuda()
    other = paged_copy(cache)
    assert all(torch.equal(x, y[:x.numel()]) for x, y in zip(cache.dense_quantized(), other.dense_quantized()))
    assert torch.equal(cache.decode(0, q), other.decode(0, q))


def test_full_size_long_32k_sampled_units():
    # long context, grouped queries, N = G: several workgroups per unit and the last-arrival merge
    import torch
    w = S.WORKLOADS["long_32k"]
    cache = run_sampled(w, [0, 31])
    assert B.kvq_decode_launch_shape(cache.cfg, 1, w.n_quant, w.n_res + 64)[0] == 8      # workgroups per unit
    # the result before the output is rounded to fp16, from the partial results the workgroups exchange
    units = [0, 13, 31]
    K, V = S.layer_kv(w, 0)
    states = H.oracle_states(w, K, V, w.n_quant, units)
    for regime in ("peaky", "diffuse"):
        Q = S.layer_queries(w, 0, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res, units)
        cache.decode(0, torch.from_numpy(Q).cuda())
        torch.cuda.synchronize()
        pre = H.merged_partials(cache, w, w.n_quant, w.n_res + 64)
        rows = np.isfinite(ref).all(axis=-1)
        err = float(np.abs(pre[rows] - ref[rows]).max())
        print(f"\n[before output rounding] long_32k {regime}: max abs err {err:.3e}")
        assert err <= 0.5 * ATT_TOL, (regime, err)


def test_full_size_llama3_8b_8k_sampled_units():
    # grouped queries at batch 16, context 8192: two workgroups per unit, four query heads each
    import torch
    w = S.WORKLOADS["llama3_8b_8k_stream"]
    cache = run_sampled(w, [0, 77, 127])
    assert B.kvq_decode_launch_shape(cache.cfg, 1, w.n_quant, w.n_res + 40)[:2] == (2, 8)
    q = torch.from_numpy(S.layer_queries(w, 0, 0, "peaky")).cuda()
    assert torch.equal(cache.decode(0, q), paged_copy(cache).decode(0, q))
    # the result before the output is rounded to fp16 (two workgroups per unit leave their partial results)
    units = [0, 77, 127]
    K, V = S.layer_kv(w, 0)
    states = H.oracle_states(w, K, V, w.n_quant, units)
    for regime in ("peaky", "diffuse"):
        Q = S.layer_queries(w, 0, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res, units)
        cache.decode(0, torch.from_numpy(Q).cuda())
        torch.cuda.synchronize()
        pre = H.merged_partials(cache, w, w.n_quant, w.n_res + 40)
        rows = np.isfinite(ref).all(axis=-1)
        err = float(np.abs(pre[rows] - ref[rows]).max())
        print(f"\n[before output rounding] llama3_8b_8k {regime}: max abs err {err:.3e}")
        assert err <= 0.5 * ATT_TOL, (regime, err)


@pytest.mark.parametrize("bits", [2, 4])
def test_batch_32_layer_shape_sampled_units(bits):
    # the 32-layer configuration's layer shape (8 kv heads, 4 query heads each) at a quarter of its batch
    # and a shorter context: 256 units, one workgroup of 8 wavefronts per unit
    w = S.WORKLOADS["mistral_7b_b128_4k_layer"].with_(name=f"b32_layer_{bits}bit", batch=32, context=1024 + 128,
                                                      bits=bits)
    cache = run_sampled(w, [0, 100, 255], regimes=("peaky",))
    assert B.kvq_decode_launch_shape(cache.cfg, 1, w.n_quant, w.n_res + 40)[:2] == (1, 8)


@pytest.mark.parametrize("bits,context", [(2, 4096), (4, 1024 + 128 + 19)])
def test_batch_128_stack_layer_sampled_units(bits, context):
    """The 32-layer, batch-128 configuration in the launch shape the benchmark times: 1024 units per layer, so
    every unit is one workgroup of TWO wavefronts that share its mini-chunks (2-bit: the full context of
    4096 tokens, 16 and 15 mini-chunks per wavefront).  The cache has four layers and the last one is used,
    so unit and plane offsets beyond the first layers are exercised.  Every unit runs on the GPU; units
    sampled across the batch are checked against the oracle, state bit for bit and attention in both query
    regimes."""
    import torch
    from paper_2505_10938_amd import cache as KC
    layer = 3
    w = S.WORKLOADS["mistral_7b_b128_4k"].with_(name=f"b128_stack_{bits}bit", layers=4, bits=bits, context=context)
    G = w.group_k
    cfg = KC.make_config(w.layers, w.batch, w.q_heads, w.kv_heads, ((w.n_quant + G - 1) // G) * G, w.bits, G, w.group_v,
                         w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    assert B.kvq_decode_launch_shape(cfg, 1, w.n_quant, w.n_res + 40)[:2] == (1, 2)
    units = [0, 7, 8 * 63 + 2, 8 * 100 + 5, 1023]
    K, V = S.layer_kv(w, layer)
    cache = KC.KVCache(cfg)
    cache.prefill(layer, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    states = H.oracle_states(w, K, V, w.n_quant, units)
    H.compare_state(cache, states, w, w.n_quant, layer=layer, units=units)
    g = w.q_heads // w.kv_heads
    for regime in ("peaky", "diffuse"):
        Q = S.layer_queries(w, layer, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res, units)
        got = cache.decode(layer, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        for ui in units:
            b, h = divmod(ui, w.kv_heads)
            err = att_err(got[b, h * g:(h + 1) * g], ref[b, h * g:(h + 1) * g])
            assert err <= ATT_TOL, (bits, regime, ui, err)
    # the other layers of the cache were not touched
    assert not cache.pool_count.view(torch.int32)[:3 * w.units].any()


@pytest.mark.parametrize("bits,G,Gv,N,use_pages", [
    (2, 32, 32, 8, False), (4, 32, 128, 8, False), (2, 64, 64, 3, False), (4, 64, 32, 8, False),
    (2, 128, 128, 3, False), (4, 128, 64, 40, False), (2, 32, 64, 0, False),
    (2, 32, 32, 8, True), (4, 64, 64, 8, True)])                       # through a page table
def test_prompts_of_many_groups_all_settings(bits, G, Gv, N, use_pages):
    """A prompt of 64 units x 16 groups in one call: from 1024 groups on the library quantizes with the kernel
    that gives a group two wavefronts (Keys / Values) instead of 1024 threads.  Every bit width, group size and
    value-group size; groups with and without flagged tokens (N = 40: most groups have several); sampled units
    against the oracle, state bit for bit and the attention."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = S.Workload("prompt", layers=1, batch=8, q_heads=8, kv_heads=8, context=32 + 16 * G + 5, bits=bits, group_k=G,
                   group_v=Gv, residual=32, outlier_budget=N, aux_capacity=32 if N else 0, rho=0.04)
    assert w.n_quant == 16 * G and w.batch * w.kv_heads * 16 >= 1024
    units = [0, 9, 31, 63]
    K, V = S.layer_kv(w, 0)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, w.n_quant, bits, G, Gv, w.residual, N, w.aux_capacity,
                         w.head_dim)
    cache = paged(cfg) if use_pages else KC.KVCache(cfg)
    cache.prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    states = H.oracle_states(w, K, V, w.n_quant, units)
    if N:
        assert any(len(st.pool) + len(st.aux) > 0 for st in states)
    H.compare_state(cache, states, w, w.n_quant, units=units)
    Q = S.layer_queries(w, 0, 0, "peaky")
    ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res, units)
    got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
    for ui in units:
        b, h = divmod(ui, w.kv_heads)
        assert att_err(got[b, h:h + 1], ref[b, h:h + 1]) <= ATT_TOL, ui


def test_four_bit_full_batch_sampled_units():
    w = S.WORKLOADS["llama2_7b_4k"].with_(name="llama2_7b_4k_4bit", bits=4, batch=4, context=2048 + 40)
    run_sampled(w, [3, 100])


def run_streaming(w: S.Workload, steps: int, fused: bool, check_every: int = 9, make_cache=None):
    """Tokens arrive one by one: the ring fills, a group is traced and quantized every G steps (in
    one launch if `fused`, else by the three separate calls), attention runs after appends."""
    import torch
    from paper_2505_10938_amd import cache as KC
    K, V = S.layer_kv(w, 0, w.context + steps)
    nq0, nr0 = w.n_quant, w.n_res
    G = w.group_k
    ms = ((w.context + steps + G - 1) // G) * G
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ms, w.bits, G, w.group_v, w.residual,
                         w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = H.gpu_cache(w, K, V, nq0, nr0, cache=(make_cache or KC.KVCache)(cfg))
    states = H.oracle_states(w, K, V, nq0)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    n, nq = w.context, nq0
    quantized = 0
    for s in range(steps):
        did = cache.append(0, Kd[:, :, n].contiguous(), Vd[:, :, n].contiguous(), fused=fused)
        n += 1
        if n - nq == w.residual + G:                       # the oracle's schedule: same rule, written again
            for ui, st in enumerate(states):
                b, h = divmod(ui, w.kv_heads)
                st.append_group(K[b, h, nq:nq + G], V[b, h, nq:nq + G])
            nq += G
            quantized += 1
            assert did
        assert cache.n_quant[0] == nq and cache.n_res[0] == n - nq
        if s % check_every == 0 or n - nq == w.residual:   # includes the steps right after a quantization
            Q = S.layer_queries(w, 0, s, "peaky")
            ref = H.oracle_attention(w, states, Q, K, V, nq, n - nq)
            got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
            assert att_err(got, ref) <= ATT_TOL, (s, n, nq)
    assert quantized >= 2
    H.compare_state(cache, states, w, nq)


@pytest.mark.parametrize("fused", [True, False])
def test_streaming_decode_matches_oracle_every_step(fused):
    run_streaming(small("stream", batch=2, q_heads=8, kv_heads=2, context=600), 70, fused)


@pytest.mark.parametrize("kw", [
    dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3),
    dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3),
    dict(bits=2, group_k=32, group_v=32, residual=0, outlier_budget=4),       # the new token closes the group
    dict(bits=4, group_k=32, group_v=128, residual=128, outlier_budget=0),    # no pool
    dict(bits=2, group_k=32, group_v=32, residual=64, outlier_budget=32, aux_capacity=32, rho=0.05),   # freezes
])
def test_fused_group_step_configurations(kw):
    w = small("fusedcfg", batch=2, q_heads=4, kv_heads=2, context=700, **kw)
    run_streaming(w, 2 * w.group_k + 5, True, check_every=17)


@pytest.mark.relaxed_share(1.0)
def test_large_magnitudes_stay_in_the_fp16_range_of_the_operands():
    """Keys 8 times and queries 4 times the usual size: Key steps of several hundred, |q| * step up
    to about 10^4, a quarter of what the fp16 operand rows can hold; Values 16 times the usual size."""
    import torch
    w = small("large", batch=2, q_heads=4, kv_heads=2, context=32 * 12 + 60, residual=32)
    K, V = S.layer_kv(w, 0)
    K, V = (K * np.float16(8)).astype(np.float16), (V * np.float16(16)).astype(np.float16)
    assert np.isfinite(K).all() and np.isfinite(V).all()
    states = H.oracle_states(w, K, V, w.n_quant)
    assert max(float(st.k_step.max()) for st in states) > 300
    cache = H.gpu_cache(w, K, V, w.n_quant, w.n_res)
    H.compare_state(cache, states, w, w.n_quant)
    Q = (S.layer_queries(w, 0, 0, "diffuse") * np.float16(4)).astype(np.float16)
    ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res)
    got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # outputs are 16 times larger than usual: most exceed 3.5 and are held to one fp16 ulp of the oracle's
    # rounded result, the others to the plain 2e-3
    assert att_err(got, ref) <= ATT_TOL


def test_first_layers_without_tracing():
    """Three layers, the first two with outlier budget 0 by configuration (the paper's setting for
    layers 0 and 1): they must equal plain group quantization, the third the traced cache."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = small("untraced", layers=3, batch=2, q_heads=4, kv_heads=2, context=32 * 10 + 50, residual=32, rho=0.05)
    G = w.group_k
    cfg = KC.make_config(w.layers, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim, untraced_layers=2)
    cache = KC.KVCache(cfg)
    selected_any = []
    for layer in range(3):
        K, V = S.layer_kv(w, layer)
        wl = w if layer >= 2 else w.with_(outlier_budget=0)
        states = H.oracle_states(wl, K, V, w.n_quant)
        H.gpu_cache(w, K, V, w.n_quant, w.n_res, layer=layer, cache=cache)
        H.compare_state(cache, states, wl, w.n_quant, layer=layer)
        selected_any.append(any(st.masked.any() for st in states))
        Q = S.layer_queries(w, layer, 0, "peaky")
        ref = H.oracle_attention(wl, states, Q, K, V, w.n_quant, w.n_res)
        got = cache.decode(layer, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
        assert att_err(got, ref) <= ATT_TOL, layer
    assert selected_any == [False, False, True]


def test_whole_context_in_full_precision():
    # residual ring as long as the context: nothing is quantized, every row takes the full-precision
    # path (the fp16 attention the benchmark sets beside the quantized one), several rows per wavefront
    w = small("allfp", residual=2048, outlier_budget=0, aux_capacity=0, context=1900, q_heads=4)
    assert w.n_quant == 0
    run_case(w)


def test_stream_read_reads_without_touching_the_buffer():
    import torch
    from paper_2505_10938_amd import binding as B
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda").view(torch.uint8)
    keep = buf.clone()
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    for n in (16, 4096, 32768 + 48, buf.numel()):
        B.kvq_stream_read(buf, n, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep)


# ---- whole-prompt quantization: the state that token-by-token appends would leave -----------------------

def run_prefill(w: S.Workload, regimes=("peaky",), make_cache=None):
    import torch
    from paper_2505_10938_amd import cache as KC
    K, V = S.layer_kv(w, 0)
    nq, nr = w.n_quant, w.n_res
    states = H.oracle_states(w, K, V, nq)
    G = w.group_k
    cfg = KC.make_config(w.layers, w.batch, w.q_heads, w.kv_heads, max(G, ((nq + G - 1) // G) * G), w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = (make_cache or KC.KVCache)(cfg)
    cache.prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    assert (cache.n_quant[0], cache.n_res[0], cache.res_start[0]) == (nq, nr, 0)
    H.compare_state(cache, states, w, nq)
    ring = cache.res_view("k").cpu().numpy()[:, :nr]
    assert np.array_equal(ring.view(np.uint16), K.reshape(-1, w.context, w.head_dim)[:, nq:].view(np.uint16))
    for regime in regimes:
        Q = S.layer_queries(w, 0, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, nq, nr)
        got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
        assert att_err(got, ref) <= ATT_TOL, regime
    return cache


@pytest.mark.parametrize("kw", [
    dict(),
    dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3),
    dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3),
    dict(residual=0, outlier_budget=4),
    dict(outlier_budget=0, group_v=128),
    dict(outlier_budget=32, aux_capacity=32, rho=0.05, context=2048 + 100),       # freezes on the way
    dict(context=100),                                                            # nothing to quantize
])
def test_prefill_equals_streaming(kw):
    base = dict(batch=2, q_heads=4, kv_heads=2, context=1024 + 77)
    base.update(kw)
    run_prefill(S.Workload("prefill", 1, **base))


@pytest.mark.parametrize("G,N,A", [(128, 64, 64), (64, 64, 20), (32, 5, 64), (128, 1, 0)])
def test_prefill_with_tied_scores_and_large_budgets(G, N, A):
    """The prompt's competitions on keys with many equal L1 scores (rows repeated, rows with permuted
    channels, signs flipped), so that the order falls back on the token index again and again, with
    budgets up to the largest supported and groups of up to two 64-token passes: the pools, flags,
    stop rule and codes are still those of the group-by-group competition."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = S.Workload("prefill_ties", 1, batch=2, q_heads=2, kv_heads=2, context=G * 9 + 40, bits=2, group_k=G,
                   group_v=32, residual=32, outlier_budget=N, aux_capacity=A)
    K, V = S.layer_kv(w, 0)
    rng = np.random.default_rng(5)
    for b in range(w.batch):
        for h in range(w.kv_heads):
            base_rows = K[b, h, :7].copy()
            for t in range(7, w.context):
                kind = rng.integers(0, 4)
                if kind == 0:
                    K[b, h, t] = base_rows[rng.integers(0, 7)]                       # the same row again
                elif kind == 1:
                    K[b, h, t] = -base_rows[rng.integers(0, 7)][rng.permutation(128)]  # same magnitudes
                elif kind == 2:
                    K[b, h, t] = K[b, h, t] * np.float16(0.05)                         # a small one
    nq, nr = w.n_quant, w.n_res
    states = H.oracle_states(w, K, V, nq)
    if N >= 64:                                               # members with equal scores: the index decided
        assert any(len({m["score"] for m in st.pool + st.aux}) < len(st.pool + st.aux) for st in states)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, nq, w.bits, G, w.group_v, w.residual, N, A, w.head_dim)
    cache = KC.KVCache(cfg)
    cache.prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    H.compare_state(cache, states, w, nq)
    Q = S.layer_queries(w, 0, 0, "diffuse")
    ref = H.oracle_attention(w, states, Q, K, V, nq, nr)
    got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
    assert att_err(got, ref) <= ATT_TOL


def test_prefill_then_stream():
    # a prompt quantized in one call, then tokens appended one by one (fused group steps)
    import torch
    w = small("prefill_stream", batch=2, q_heads=4, kv_heads=2, context=500)
    steps = 80
    K, V = S.layer_kv(w, 0, w.context + steps)
    from paper_2505_10938_amd import cache as KC
    G = w.group_k
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + steps + G - 1) // G) * G, w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = KC.KVCache(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    cache.prefill(0, Kd[:, :, :w.context].contiguous(), Vd[:, :, :w.context].contiguous())
    for s in range(steps):
        cache.append(0, Kd[:, :, w.context + s].contiguous(), Vd[:, :, w.context + s].contiguous())
    n = w.context + steps
    wf = w.with_(context=n)
    states = H.oracle_states(wf, K, V, wf.n_quant)
    assert cache.n_quant[0] == wf.n_quant and cache.n_res[0] == wf.n_res
    H.compare_state(cache, states, wf, wf.n_quant)
    Q = S.layer_queries(wf, 0, 0, "peaky")
    ref = H.oracle_attention(wf, states, Q, K, V, wf.n_quant, wf.n_res)
    got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
    assert att_err(got, ref) <= ATT_TOL


def ragged_lengths_state(n, G, R):
    nq = G * ((n - R) // G) if n >= R + G else 0
    return nq, n - nq


@pytest.mark.parametrize("kw,lengths", [
    (dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=4), [45, 300, 161, 96]),
    (dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3, q_heads=8), [1, 400, 95, 96]),
    (dict(bits=2, group_k=32, group_v=128, residual=0, outlier_budget=4), [32, 31, 257, 0]),
])
def test_ragged_batch_streaming(kw, lengths):
    run_ragged(kw, lengths)


def run_ragged(kw, lengths, make_cache=None, planned=False):
    """Sequences of different lengths in one batch: tokens are appended step by step to the
    sequences that are still growing (one launch per step and layer, the state kept on the device),
    then one decode launch serves all of them.  Every unit is compared with the oracle run on its
    own sequence alone."""
    import torch
    from paper_2505_10938_amd import cache as KC
    base = dict(layers=1, batch=len(lengths), q_heads=4, kv_heads=2, context=max(lengths))
    base.update(kw)
    w = S.Workload("ragged", **base)
    G, R = w.group_k, w.residual
    K, V = S.layer_kv(w, 0, max(lengths))
    ms = ((max(lengths) + G - 1) // G) * G
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ms, w.bits, G, w.group_v, R, w.outlier_budget,
                         w.aux_capacity, w.head_dim)
    cache = (make_cache or KC.RaggedKVCache)(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    for t in range(max(lengths)):
        cache.set_active([t < n for n in lengths])
        cache.append(0, Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
        cache.advance()
    torch.cuda.synchronize()
    state = cache.seq_state.cpu().numpy()
    Q = S.layer_queries(w, 0, 0, "peaky")
    if planned:                                              # workgroups dealt by length
        cache.make_plan()
    got = cache.decode(0, torch.from_numpy(Q).cuda(), planned=planned).cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    g = w.q_heads // w.kv_heads
    rows = cache.sizes.res_rows
    for b, n in enumerate(lengths):
        nq, nr = ragged_lengths_state(n, G, R)
        assert (state[b, 0], state[b, 2]) == (nq, nr), (b, state[b])
        assert state[b, 1] == nq % rows
        units = [b * w.kv_heads + h for h in range(w.kv_heads)]
        states = H.oracle_states(w, K, V, nq, units)
        H.compare_state(cache, states, w, nq, units=units)
        if n == 0:
            assert not got[b].any()                         # a sequence without tokens: zeros
            continue
        ref = H.oracle_attention(w, states, Q, K, V, nq, nr, units)
        err = att_err(got[b], ref[b])
        assert err <= ATT_TOL, (b, n, err)


@pytest.mark.parametrize("kw,lengths", [
    (dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=4), [45, 3000, 161, 96]),
    (dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3, q_heads=8), [1, 4000, 95, 960, 33, 2048]),
    (dict(bits=2, group_k=32, group_v=128, residual=0, outlier_budget=4), [32, 31, 2570, 0]),
    (dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3), [130, 2900, 700, 33, 161]),
])
def test_ragged_batch_with_a_launch_plan(kw, lengths):
    """The same batches through kvq_seq_plan + kvq_decode_attention_planned: the long sequences are split
    over several workgroups, the short ones have one, and every unit still matches the oracle."""
    run_ragged(kw, lengths, planned=True)


def test_launch_plan_contents():
    """What the plan holds: every sequence has consecutive entries, numbered 0 .. n-1, which together cover
    its mini-chunks exactly once and carry a copy of its state; there are no more entries than the launch has
    workgroups per kv head; longer sequences have more of them."""
    import torch
    from paper_2505_10938_amd import cache as KC
    lengths = [128 + (8192 - 128) * i // 31 for i in range(32)]
    G, R = 32, 128
    cfg = KC.make_config(1, 32, 32, 8, 8192, 2, G, 32, R, 8, 32)
    cache = KC.RaggedKVCache(cfg)
    st = torch.zeros(32, 4, dtype=torch.int32)
    for b, n in enumerate(lengths):
        nq, nr = ragged_lengths_state(n, G, R)
        st[b] = torch.tensor([nq, nq % cache.sizes.res_rows, nr, 1])
    cache.seq_state.copy_(st)
    cache.longest = max(lengths)
    cache.make_plan()
    plan = cache.plan.cpu().numpy()
    room = (len(plan) - 8) // 8
    n_entries = int(plan[0])
    assert 32 <= n_entries <= room
    entries = plan[8:8 + 8 * n_entries].reshape(n_entries, 8)
    per_seq = {}
    for i, e in enumerate(entries):
        b, split, n_splits, mc0, nq, rs, nr, mc1 = (int(x) for x in e)
        assert (nq, rs, nr) == tuple(int(x) for x in st[b, :3])
        per_seq.setdefault(b, []).append((split, n_splits, mc0, mc1, i))
    assert sorted(per_seq) == list(range(32))
    counts = []
    for b in range(32):
        parts = per_seq[b]
        n_mc = (int(st[b, 0]) + 127) // 128
        assert [p[0] for p in parts] == list(range(len(parts))) and all(p[1] == len(parts) for p in parts)
        assert [p[4] for p in parts] == list(range(parts[0][4], parts[0][4] + len(parts)))     # consecutive entries
        assert parts[0][2] == 0 and parts[-1][3] == n_mc
        assert all(parts[i][3] == parts[i + 1][2] for i in range(len(parts) - 1))              # no gap, no overlap
        counts.append(len(parts))
    assert counts == sorted(counts) and counts[0] == 1 and counts[-1] >= 2                      # lengths ascend with b


def test_full_size_ragged_batch_with_a_launch_plan_sampled_units():
    """The batch the benchmark's ragged lines run: 32 sequences of 128 .. 8192 tokens, 8 kv heads of 4 query
    heads, each sequence prefilled on its own.  Sampled units (the shortest, the longest, some between; one to
    four workgroups each under the plan) against the oracle, with and without the launch plan, in both query
    regimes; the two launches differ by no more than the rounding of the output."""
    import torch
    from paper_2505_10938_amd import cache as KC
    G, R, batch = 32, 128, 32
    lengths = [128 + (8192 - 128) * i // (batch - 1) for i in range(batch)]
    w = S.Workload("ragged_full", 1, batch=batch, q_heads=32, kv_heads=8, context=max(lengths), bits=2, group_k=G,
                   group_v=32, residual=R, outlier_budget=8, aux_capacity=32)
    cfg = KC.make_config(1, batch, w.q_heads, w.kv_heads, max(lengths), 2, G, 32, R, 8, 32)
    cache = KC.RaggedKVCache(cfg)
    sampled = [(0, 0), (0, 7), (9, 3), (16, 5), (24, 1), (31, 0), (31, 6)]       # (sequence, kv head)
    host = {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    for b, n in enumerate(lengths):
        k = torch.randn((w.kv_heads, n, 128), generator=gen, device="cuda", dtype=torch.float32).to(torch.float16)
        v = torch.randn((w.kv_heads, n, 128), generator=gen, device="cuda", dtype=torch.float32).to(torch.float16)
        for (sb, h) in sampled:
            if sb == b:                                   # units the oracle sees: kvq_synth's rows
                kh, vh = S.unit_kv(w.seed, 0, b, h, n, 128, w.rho)
                k[h].copy_(torch.from_numpy(kh))
                v[h].copy_(torch.from_numpy(vh))
                host[(b, h)] = (kh, vh)
        cache.prefill_sequence(b, [k.contiguous()], [v.contiguous()])
    cache.make_plan()
    plan = cache.plan.cpu().numpy()
    splits_of = {int(e[0]): int(e[2]) for e in plan[8:8 + 8 * int(plan[0])].reshape(-1, 8)}
    assert splits_of[0] == 1 and splits_of[31] >= 2
    g = w.q_heads // w.kv_heads
    from oracle import kvq_oracle as O
    for regime in ("peaky", "diffuse"):
        Q = S.layer_queries(w, 0, 0, regime)
        qd = torch.from_numpy(Q).cuda()
        plain = cache.decode(0, qd).cpu().numpy().astype(np.float64)
        planned = cache.decode(0, qd, planned=True).cpu().numpy().astype(np.float64)
        assert np.isfinite(planned).all()
        # (different splits of a sequence, different summation order: at most the output's rounding apart)
        assert np.abs(plain - planned).max() <= np.maximum(ATT_TOL, 2 * np.spacing(np.float16(np.abs(plain).max())))
        for (b, h), (kh, vh) in host.items():
            n = lengths[b]
            nq, nr = ragged_lengths_state(n, G, R)
            st = O.UnitState(128, 2, G, 32, 8, 32)
            for i in range(nq // G):
                st.append_group(kh[i * G:(i + 1) * G], vh[i * G:(i + 1) * G])
            ref, _ = O.decode_attention(Q[b, h * g:(h + 1) * g], st, kh[nq:n], vh[nq:n])
            for got in (plain, planned):
                assert att_err(got[b, h * g:(h + 1) * g], ref) <= ATT_TOL, (regime, b, h)


def test_ragged_equals_uniform_when_lengths_agree():
    """The ragged entry points on a batch whose sequences all have the same state give the bytes and
    the outputs of the uniform ones."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = small("ragged_uniform", q_heads=4, context=32 * 9 + 5, residual=64)
    G, R = w.group_k, w.residual
    K, V = S.layer_kv(w, 0)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G, w.group_v, R,
                         w.outlier_budget, w.aux_capacity, w.head_dim)
    a, b = KC.KVCache(cfg), KC.RaggedKVCache(cfg)
    b.set_active([1] * w.batch)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    for t in range(w.context):
        k, v = Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous()
        a.append(0, k, v)
        b.append(0, k, v)
        b.advance()
    q = torch.from_numpy(S.layer_queries(w, 0, 0, "peaky")).cuda()
    oa, ob = a.decode(0, q), b.decode(0, q)
    torch.cuda.synchronize()
    nb = a.n_quant[0] // 32
    for name in ("k_codes", "v_codes", "k_meta", "v_meta", "mask", "pool_idx", "pool_count", "aux_count"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    assert nb > 0 and torch.equal(oa, ob)


@pytest.mark.parametrize("g", [1, 4])
def test_decode_replayed_from_a_captured_graph(g):
    """The decode launch allocates nothing, synchronises nothing and leaves its workspace as it found
    it, so it can be captured into a graph; every replay, with eager launches between the replays,
    gives the eager result.  Few units: each is spread over several workgroups, so the replays
    also depend on the arrival counters being zero again after every launch."""
    import torch
    w = small(f"graph_g{g}", batch=1, q_heads=2 * g, context=1500)
    K, V = S.layer_kv(w, 0)
    cache = H.gpu_cache(w, K, V, w.n_quant, w.n_res)
    q = torch.from_numpy(S.layer_queries(w, 0, 0, "peaky")).cuda()
    q_other = torch.from_numpy(S.layer_queries(w, 0, 1, "diffuse")).cuda()
    eager = cache.decode(0, q).clone()
    eager_other = cache.decode(0, q_other).clone()
    out = torch.empty_like(q)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cache.decode(0, q, out)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cache.decode(0, q, out)
    for _ in range(4):
        out.zero_()
        assert torch.equal(cache.decode(0, q_other), eager_other)      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager)


@pytest.mark.parametrize("kw", [
    dict(bits=2, group_k=32, group_v=32, residual=128, outlier_budget=8),
    dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3, q_heads=8),
    dict(bits=2, group_k=32, group_v=128, residual=0, outlier_budget=4),      # every 32nd step fills the ring
])
def test_streaming_steps_with_the_append_inside_the_decode_launch(kw):
    """Token by token with KVCache.step: on the steps that do not fill the ring the new token's rows
    come with the decode launch, which attends to them and stores them; on the others the group step
    runs first.  The output of every step is compared with the oracle, so a row that the launch
    failed to store shows up in the following steps."""
    import torch
    from paper_2505_10938_amd import cache as KC
    base = dict(layers=1, batch=2, q_heads=2, kv_heads=2, context=300)
    base.update(kw)
    w = S.Workload("step", **base)
    steps = 2 * w.group_k + 9
    K, V = S.layer_kv(w, 0, w.context + steps)
    G = w.group_k
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + steps + G - 1) // G) * G, w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    nq, nr = w.n_quant, w.n_res
    cache = H.gpu_cache(w, K, V, nq, nr, cache=KC.KVCache(cfg))
    states = H.oracle_states(w, K, V, nq)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    n = w.context
    fused = 0
    for s in range(steps):
        Q = S.layer_queries(w, 0, s, "peaky")
        before = cache.n_quant[0]
        out = cache.step(0, Kd[:, :, n].contiguous(), Vd[:, :, n].contiguous(), torch.from_numpy(Q).cuda())
        n += 1
        if n - nq == w.residual + G:
            for ui, st in enumerate(states):
                b, h = divmod(ui, w.kv_heads)
                st.append_group(K[b, h, nq:nq + G], V[b, h, nq:nq + G])
            nq += G
            assert cache.n_quant[0] == before + G
        else:
            fused += 1
        assert cache.n_quant[0] == nq and cache.n_res[0] == n - nq
        ref = H.oracle_attention(w, states, Q, K, V, nq, n - nq)
        got = out.cpu().numpy().astype(np.float64)
        assert att_err(got, ref) <= ATT_TOL, (s, n, nq)
    assert fused >= steps - 3
    H.compare_state(cache, states, w, nq)


def rope_table(pos, hd=128, base=10000.0):
    """fp32 [hd]: the cosines of position `pos` at the usual frequencies base^(-2i/hd), then the sines."""
    ang = pos * base ** (-2.0 * np.arange(hd // 2, dtype=np.float64) / hd)
    return np.concatenate([np.cos(ang), np.sin(ang)]).astype(np.float32)


@pytest.mark.parametrize("kw,per_sequence", [
    (dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=8), False),
    (dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=8), True),
    (dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3, q_heads=8), True),   # four query heads
    (dict(bits=2, group_k=32, group_v=128, residual=0, outlier_budget=4), False),  # every 32nd step fills the ring
    (dict(bits=2, group_k=32, group_v=32, residual=40, outlier_budget=4, q_heads=16, batch=3), True),   # eight
    (dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3, context=300), False),  # four blocks per Key group
    (dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=8, q_heads=4, paged=True), True),  # behind a page table
])
def test_rotary_embedding_inside_the_decode_launch(kw, per_sequence):
    """Token by token with KVCache.step and a table of angles: the library rotates the query and the new
    Key itself (inside the decode launch; with the small launch on the steps that fill the ring).  The
    oracle rotates them with its own function and runs the unrotated path.  The rotated Key rows are
    compared bit for bit where they are stored (ring rows at the end; the codes and pool rows of the
    groups quantized on the way, which are made of rotated rows after the first residual + G steps), the
    attention output at every step."""
    import torch
    from oracle import kvq_oracle as O
    from paper_2505_10938_amd import cache as KC
    base = dict(layers=1, batch=2, q_heads=2, kv_heads=2, context=200)
    base.update(kw)
    use_pages = base.pop("paged", False)
    w = S.Workload("rope", **base)
    G = w.group_k
    steps = w.residual + 3 * G + 9
    K, V = S.layer_kv(w, 0, w.context + steps)
    K = K.copy()
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + steps + G - 1) // G) * G, w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    nq, nr = w.n_quant, w.n_res
    cache = H.gpu_cache(w, K, V, nq, nr, cache=paged(cfg) if use_pages else KC.KVCache(cfg))
    states = H.oracle_states(w, K, V, nq)
    raw_k = torch.from_numpy(K.copy()).cuda()
    Vd = torch.from_numpy(V).cuda()
    n = w.context
    fused = 0
    for s in range(steps):
        # the new token's position: the same for every sequence, or 1000 b further on for sequence b
        pos = [n + (1000 * b if per_sequence else 0) for b in range(w.batch)]
        tables = np.stack([rope_table(p) for p in pos])
        rope = torch.from_numpy(tables if per_sequence else tables[0]).cuda()
        Q = S.layer_queries(w, 0, s, "peaky")
        Qr = np.stack([O.rope_rotate(Q[b], tables[b, :64], tables[b, 64:]) for b in range(w.batch)])
        for b in range(w.batch):                                   # the oracle's token: rotated
            K[b, :, n] = O.rope_rotate(K[b, :, n], tables[b, :64], tables[b, 64:])
        out = cache.step(0, raw_k[:, :, n].contiguous(), Vd[:, :, n].contiguous(), torch.from_numpy(Q).cuda(),
                         rope=rope, rope_stride=w.head_dim if per_sequence else 0)
        n += 1
        if n - nq == w.residual + G:
            for ui, st in enumerate(states):
                b, h = divmod(ui, w.kv_heads)
                st.append_group(K[b, h, nq:nq + G], V[b, h, nq:nq + G])
            nq += G
        else:
            fused += 1
        assert cache.n_quant[0] == nq and cache.n_res[0] == n - nq
        ref = H.oracle_attention(w, states, Qr, K, V, nq, n - nq)
        got = out.cpu().numpy().astype(np.float64)
        assert att_err(got, ref) <= ATT_TOL, (s, n, nq)
    assert fused >= steps - 5 and nq >= w.context          # rotated rows have been quantized
    H.compare_state(cache, states, w, nq)
    ring = cache.res_view("k").cpu().numpy()
    rows = cache.sizes.res_rows
    for ui in range(w.batch * w.kv_heads):
        b, h = divmod(ui, w.kv_heads)
        at = [(cache.res_start[0] + i) % rows for i in range(n - nq)]
        assert np.array_equal(ring[ui, at].view(np.uint16), K[b, h, nq:n].view(np.uint16)), ui
    # the rotation changed the rows: the test would not pass on unrotated ones
    assert not np.array_equal(K[:, :, w.context:n], raw_k[:, :, w.context:n].cpu().numpy())


def test_rotation_on_its_own_equals_the_oracle_bit_for_bit():
    import torch
    from oracle import kvq_oracle as O
    from paper_2505_10938_amd import cache as KC
    cfg = KC.make_config(1, 5, 8, 2, 64, 2, 32, 32, 0, 0, 0, 128)
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((5, 8, 128)) * 4).astype(np.float16)
    x[0, 0, :4] = [0.0, -0.0, 65504.0, 6e-8]
    tables = np.stack([rope_table(31 * b + 3) for b in range(5)])
    xd = torch.from_numpy(x).cuda()
    out = torch.empty_like(xd)
    B.kvq_rope_rotate(cfg, xd, 8, torch.from_numpy(tables).cuda(), 128, out)
    want = np.stack([O.rope_rotate(x[b], tables[b, :64], tables[b, 64:]) for b in range(5)])
    assert np.array_equal(out.cpu().numpy().view(np.uint16), want.view(np.uint16))
    # one row for all sequences, in place
    B.kvq_rope_rotate(cfg, xd, 8, torch.from_numpy(tables[2]).cuda(), 0, xd)
    want = O.rope_rotate(x, tables[2, :64], tables[2, 64:])
    assert np.array_equal(xd.cpu().numpy().view(np.uint16), want.view(np.uint16))


# ---- paged quantized cache: pages of one Key group each, dealt to the sequences by a table ----------------

def paged(cfg, seed=11, spare=7, kind=None):
    """A paged cache whose pool has `spare` pages more than all sequences can fill, every group of
    every sequence assigned a page of its own in a seeded random order."""
    import torch
    from paper_2505_10938_amd import cache as KC
    groups = cfg.max_seq // cfg.group_k
    n_pages = cfg.batch * groups + spare
    cache = (kind or KC.KVCache)(cfg, n_pages=n_pages)
    deal = np.random.default_rng(seed).permutation(n_pages)[:cfg.batch * groups].reshape(cfg.batch, groups)
    assert len(set(deal.reshape(-1).tolist())) == deal.size
    cache.page_table.copy_(torch.from_numpy(deal.astype(np.int32)))
    return cache


@pytest.mark.parametrize("kw", [
    dict(bits=2, group_k=32, group_v=32, residual=128, outlier_budget=8),                 # four pages per mini-chunk
    dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3, q_heads=8),       # two
    dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3, q_heads=16),    # one; two workgroup rows
    # (the eight checked steps of this case see the same few dominant tokens with a Value element above 3.5: the
    # same 2 or 3 output elements are counted at every step, 18 of 12 288 in all)
    pytest.param(dict(bits=2, group_k=32, group_v=128, residual=0, outlier_budget=4, batch=3),
                 marks=pytest.mark.relaxed_share(2e-3)),
])
def test_paged_streaming(kw):
    """The streaming test on a paged cache: group steps write through the table, the decode launch
    reads through it; pages gathered through the table must be the oracle's bytes."""
    base = dict(batch=2, q_heads=4, kv_heads=2, context=1100)
    base.update(kw)
    w = small("paged", **base)
    run_streaming(w, 2 * w.group_k + 5, True, check_every=13, make_cache=paged)


@pytest.mark.parametrize("kw", [
    dict(),
    dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3),
    dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3, context=2048 + 300),
    dict(context=100),                                                            # nothing to quantize
])
def test_paged_prefill(kw):
    base = dict(batch=2, q_heads=4, kv_heads=2, context=1024 + 77)
    base.update(kw)
    run_prefill(S.Workload("paged_prefill", 1, **base), make_cache=paged)


def test_paged_ragged_batch():
    from paper_2505_10938_amd import cache as KC
    run_ragged(dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=4), [45, 300, 161, 96],
               make_cache=lambda cfg: paged(cfg, kind=KC.RaggedKVCache))


def test_paged_ragged_batch_with_a_launch_plan():
    """Sequences of different lengths behind a page table, the decode workgroups dealt by a launch plan."""
    from paper_2505_10938_amd import cache as KC
    run_ragged(dict(bits=2, group_k=64, group_v=32, residual=32, outlier_budget=4, q_heads=8), [45, 2100, 161, 700],
               make_cache=lambda cfg: paged(cfg, kind=KC.RaggedKVCache), planned=True)


def test_paged_equals_dense_bit_for_bit_second_layer():
    """Two layers, work on the second: a paged and a dense cache fed the same tokens hold the same
    bytes (pages gathered through the table) and give the same outputs, bit for bit; the pages of the
    first layer, and the pool's spare pages, stay untouched."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = small("paged_layers", layers=2, batch=2, q_heads=8, kv_heads=2, context=32 * 21 + 40, residual=32)
    K, V = S.layer_kv(w, 1)
    G = w.group_k
    cfg = KC.make_config(w.layers, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G,
                         w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    a = H.gpu_cache(w, K, V, w.n_quant, w.n_res, layer=1, cache=KC.KVCache(cfg))
    b = paged(cfg)
    b.k_codes.fill_(0xA5)
    b.v_codes.fill_(0xA5)
    b = H.gpu_cache(w, K, V, w.n_quant, w.n_res, layer=1, cache=b)
    for x, y, name in zip(a.dense_quantized(), b.dense_quantized(), ("k_codes", "k_meta", "v_codes", "v_meta", "mask")):
        per_unit = x.numel() // a.sizes.units
        n_used = {"k_codes": w.n_quant // 32 * 512 * w.bits, "v_codes": w.n_quant // 32 * 512 * w.bits}.get(name)
        xs, ys = x.view(a.sizes.units, per_unit), y[:x.numel()].view(a.sizes.units, per_unit)
        upl = w.batch * w.kv_heads
        sl = slice(None) if n_used is None else slice(0, n_used)
        assert torch.equal(xs[upl:, sl], ys[upl:, sl]), name
    # pages never written: the first layer's planes and the spare pages keep the fill pattern
    page_bytes = G // 32 * 512 * w.bits
    planes = b.k_codes[:cfg.layers * cfg.kv_heads * b.n_pages * page_bytes].view(cfg.layers, cfg.kv_heads, b.n_pages, page_bytes)
    assert bool((planes[0] == 0xA5).all())
    used = set(b.page_table.cpu().numpy()[:, :w.n_quant // G].reshape(-1).tolist())
    spare = [p for p in range(b.n_pages) if p not in used]
    assert len(spare) >= 7 and bool((planes[1][:, spare] == 0xA5).all())
    states = H.oracle_states(w, K, V, w.n_quant)
    H.compare_state(b, states, w, w.n_quant, layer=1)
    q = torch.from_numpy(S.layer_queries(w, 1, 0, "peaky")).cuda()
    oa, ob = a.decode(1, q), b.decode(1, q)
    torch.cuda.synchronize()
    assert torch.equal(oa, ob)
    ref = H.oracle_attention(w, states, S.layer_queries(w, 1, 0, "peaky"), K, V, w.n_quant, w.n_res)
    assert att_err(ob.cpu().numpy().astype(np.float64), ref) <= ATT_TOL


def test_paged_table_entries_out_of_range_are_clamped():
    """Entries of groups beyond a sequence's quantized part are never used, and an entry outside the
    pool is clamped: a table poisoned there must change nothing, and a decode over a table with
    wild entries for live groups must still finish without touching memory outside the pool."""
    import torch
    w = small("paged_poison", batch=2, q_heads=4, kv_heads=2, context=32 * 9 + 50, residual=32)
    K, V = S.layer_kv(w, 0)
    from paper_2505_10938_amd import cache as KC
    G = w.group_k
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, 32 * 40, w.bits, G, w.group_v, w.residual,
                         w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = H.gpu_cache(w, K, V, w.n_quant, w.n_res, cache=paged(cfg))
    q = torch.from_numpy(S.layer_queries(w, 0, 0, "peaky")).cuda()
    good = cache.decode(0, q).clone()
    cache.page_table[:, w.n_quant // G:] = 2 ** 30          # groups not yet quantized
    assert torch.equal(cache.decode(0, q), good)
    cache.page_table[:, 1] = -7                             # live groups: results change, accesses stay inside
    cache.page_table[:, 2] = 2 ** 30
    out = cache.decode(0, q)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())


@pytest.mark.parametrize("use_pages", [False, True])
def test_sequences_join_a_running_batch_by_their_own_prefill(use_pages):
    """Each sequence's prompt is quantized by its own call (different lengths; one slot is then
    taken over by a new sequence, which must not inherit the old one's pool or frozen flag), the
    batch decodes, streams a few tokens and decodes again; every unit is compared with the oracle
    run on its own sequence alone."""
    import torch
    from paper_2505_10938_amd import cache as KC
    lengths = [300, 45, 161, 0]                               # slot 3 stays empty
    steps = 40
    kw = dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=4, aux_capacity=4, rho=0.05)
    w = S.Workload("join", layers=1, batch=4, q_heads=4, kv_heads=2, context=max(lengths) + steps, **kw)
    G, R = w.group_k, w.residual
    K, V = S.layer_kv(w, 0)
    K2, V2 = S.layer_kv(w.with_(seed=w.seed + 1), 0)         # the sequence that takes slot 0 over
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G, w.group_v, R,
                         w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = paged(cfg, kind=KC.RaggedKVCache) if use_pages else KC.RaggedKVCache(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    for b, n in enumerate(lengths):
        if n:
            cache.prefill_sequence(b, [Kd[b, :, :n].contiguous()], [Vd[b, :, :n].contiguous()])
    # the first occupant of slot 0 froze its pools (small auxiliary pool, many outlier tokens) ...
    torch.cuda.synchronize()
    assert int(cache.frozen.view(torch.int32)[0].item()) == 1
    # ... and is replaced by a shorter sequence with other data
    n0 = 100
    K[0], V[0] = K2[0], V2[0]
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    cache.prefill_sequence(0, [Kd[0, :, :n0].contiguous()], [Vd[0, :, :n0].contiguous()])
    lengths[0] = n0

    def check(lengths, step):
        Q = S.layer_queries(w, 0, step, "peaky")
        got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
        state = cache.seq_state.cpu().numpy()
        for b, n in enumerate(lengths):
            if n == 0:
                assert not got[b].any()
                continue
            nq, nr = ragged_lengths_state(n, G, R)
            assert (state[b, 0], state[b, 2]) == (nq, nr), (b, state[b])
            units = [b * w.kv_heads + h for h in range(w.kv_heads)]
            states = H.oracle_states(w, K, V, nq, units)
            H.compare_state(cache, states, w, nq, units=units)
            ref = H.oracle_attention(w, states, Q, K, V, nq, nr, units)
            assert att_err(got[b], ref[b]) <= ATT_TOL, (b, n, step)

    check(lengths, 0)
    for t in range(steps):                                    # the three live sequences grow together
        cache.set_active([n > 0 for n in lengths])
        rows_k = torch.stack([Kd[b, :, n] for b, n in enumerate(lengths)]).contiguous()
        rows_v = torch.stack([Vd[b, :, n] for b, n in enumerate(lengths)]).contiguous()
        cache.append(0, rows_k, rows_v)
        cache.advance()
        lengths = [n + 1 if n > 0 else 0 for n in lengths]
    check(lengths, 1)


def test_full_size_llama3_8b_8k_128_consecutive_steps_sampled_units():
    """The third configuration as it is stated: batch 16, 32 query / 8 kv heads, context 8192, then 128
    consecutive decode steps with the group step on every 32nd (KVCache.step: one launch on the other
    steps).  The prompt is quantized in one call; sampled units are compared with the oracle streaming
    the same tokens, the attention output at every 8th step and after every group step."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = S.WORKLOADS["llama3_8b_8k_stream"]
    steps = 128
    units = [0, 77, 127]
    K, V = S.layer_kv(w, 0, w.context + steps)
    G, R = w.group_k, w.residual
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + steps + G - 1) // G) * G, w.bits, G,
                         w.group_v, R, w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = KC.KVCache(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    cache.prefill(0, Kd[:, :, :w.context].contiguous(), Vd[:, :, :w.context].contiguous())
    nq = w.n_quant
    assert cache.n_quant[0] == nq and cache.n_res[0] == w.n_res
    states = H.oracle_states(w, K, V, nq, units)
    n, quantized, checked = w.context, 0, 0
    for s in range(steps):
        Q = S.layer_queries(w, 0, s, "peaky")
        out = cache.step(0, Kd[:, :, n].contiguous(), Vd[:, :, n].contiguous(), torch.from_numpy(Q).cuda())
        n += 1
        closed = n - nq == R + G
        if closed:
            for ui, st in zip(units, states):
                b, h = divmod(ui, w.kv_heads)
                st.append_group(K[b, h, nq:nq + G], V[b, h, nq:nq + G])
            nq += G
            quantized += 1
        assert cache.n_quant[0] == nq and cache.n_res[0] == n - nq
        if closed or s % 8 == 0:
            ref = H.oracle_attention(w, states, Q, K, V, nq, n - nq, units)
            got = out.cpu().numpy().astype(np.float64)
            g = w.q_heads // w.kv_heads
            for ui in units:
                b, h = divmod(ui, w.kv_heads)
                err = att_err(got[b, h * g:(h + 1) * g], ref[b, h * g:(h + 1) * g])
                assert err <= ATT_TOL, (s, ui, err)
            checked += 1
    assert quantized == 4 and checked >= 16
    H.compare_state(cache, states, w, nq, units=units)


@pytest.mark.parametrize("kw,use_pages", [
    (dict(bits=2, group_k=32, group_v=32, residual=32, outlier_budget=8), False),
    (dict(bits=4, group_k=64, group_v=128, residual=32, outlier_budget=3), False),
    (dict(bits=2, group_k=128, group_v=64, residual=0, outlier_budget=4, rho=0.05), True),
])
def test_dequantized_rows_bit_exact(kw, use_pages):
    """kvq_dequantize against the oracle's fp16 rows: every token of the quantized segment, tokens
    held in the pools included (their stored rows), whole and as a window that starts inside it."""
    import torch
    from paper_2505_10938_amd import binding as B, cache as KC
    w = small("dequant", batch=2, q_heads=2, kv_heads=2, context=128 * 5 + 70, **kw)
    K, V = S.layer_kv(w, 0)
    nq = w.n_quant
    G = w.group_k
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ((w.context + G - 1) // G) * G, w.bits, G, w.group_v,
                         w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)
    cache = H.gpu_cache(w, K, V, nq, w.n_res, cache=paged(cfg) if use_pages else KC.KVCache(cfg))
    states = H.oracle_states(w, K, V, nq)
    assert any(st.masked.any() for st in states)
    units = w.batch * w.kv_heads
    for t0, n in ((0, nq), (96, nq - 160)):
        ko = torch.full((units, n + 8, w.head_dim), 7.0, dtype=torch.float16, device="cuda")   # padded stride
        vo = torch.full_like(ko, 7.0)
        B.kvq_dequantize(cfg, 0, cache.qcache, nq, cache.pool, t0, n, ko, vo, (n + 8) * w.head_dim)
        torch.cuda.synchronize()
        kg, vg = ko.cpu().numpy(), vo.cpu().numpy()
        for ui, st in enumerate(states):
            kr, vr = st.rows_fp16()
            assert np.array_equal(kg[ui, :n].view(np.uint16), kr[t0:t0 + n].view(np.uint16)), (ui, t0)
            assert np.array_equal(vg[ui, :n].view(np.uint16), vr[t0:t0 + n].view(np.uint16)), (ui, t0)
        assert (kg[:, n:] == 7.0).all() and (vg[:, n:] == 7.0).all()      # nothing written past the window


@pytest.mark.parametrize("g,tokens,kw", [
    (1, 2, dict()),
    (1, 4, dict(bits=4, group_k=64, group_v=64, residual=32, outlier_budget=3)),
    (2, 2, dict(group_v=128)),
    (1, 8, dict(residual=32)),                               # eight rows per kv head: two workgroup rows
    (4, 2, dict(residual=7, context=32 * 30 + 20)),          # the same, with grouped queries
    (2, 4, dict(context=8192 + 100, batch=1, kv_heads=2)),   # a long unit: several workgroups and the merge
    (2, 2, dict(bits=2, group_k=128, group_v=128, residual=32, outlier_budget=3, context=128 * 9 + 50)),  # one Key group per mini-chunk
    (1, 4, dict(bits=4, group_k=128, group_v=32, residual=32, outlier_budget=3, context=128 * 5 + 40)),
])
def test_several_query_tokens_at_once(g, tokens, kw):
    """kvq_decode_attention_multi: the `tokens` newest tokens of every sequence attend in one launch, each
    up to itself.  Every token's output is compared with the oracle's attention over the cache without
    the residual rows that follow the token."""
    import torch
    base = dict(batch=2, kv_heads=2, context=1024 + 77)
    base.update(kw)
    base["q_heads"] = g * base["kv_heads"]
    w = small("multi", **base)
    K, V = S.layer_kv(w, 0)
    nq, nr = w.n_quant, w.n_res
    assert nr >= tokens - 1
    states = H.oracle_states(w, K, V, nq)
    cache = H.gpu_cache(w, K, V, nq, nr)
    Q = np.stack([S.layer_queries(w, 0, i, "peaky" if i % 2 == 0 else "diffuse") for i in range(tokens)], axis=1)
    out = cache.decode_multi(0, torch.from_numpy(np.ascontiguousarray(Q)).cuda())
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert got.shape == (w.batch, tokens, w.q_heads, w.head_dim) and np.isfinite(got).all()
    for i in range(tokens):
        seen = nr - (tokens - 1 - i)
        ref = H.oracle_attention(w, states, Q[:, i], K, V, nq, seen)
        err = att_err(got[:, i], ref)
        assert err <= ATT_TOL, (i, err)
    # one query token through the same entry point is the plain decode step, bit for bit
    q1 = torch.from_numpy(np.ascontiguousarray(Q[:, -1])).cuda()
    assert torch.equal(cache.decode_multi(0, q1[:, None].contiguous())[:, 0], cache.decode(0, q1))


@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_configurations(seed):
    """Hyper-parameters, shapes and lengths drawn from a seeded generator (ragged tails, budgets from 0 to
    more than a group, every group size and bit width, every query-head ratio)."""
    g = np.random.default_rng(1000 + seed)
    G = int(g.choice([32, 64, 128]))
    kv_heads = int(g.choice([1, 2, 3]))
    ratio = int(g.choice([1, 2, 4, 8]))
    N = int(g.choice([0, 1, 3, 8, 17, 40]))
    kw = dict(bits=int(g.choice([2, 4])), group_k=G, group_v=int(g.choice([32, 64, 128])),
              residual=int(g.choice([0, 1, 31, 32, 100, 128])), outlier_budget=N,
              aux_capacity=int(g.choice([0, 4, 32, 64])) if N else 0,
              batch=int(g.choice([1, 2, 3])), kv_heads=kv_heads, q_heads=kv_heads * ratio,
              context=int(g.integers(1, 6 * G + 200)), rho=float(g.choice([0.0, 0.02, 0.1])))
    w = S.Workload(f"random{seed}", 1, seed=seed, **kw)
    run_case(w, regimes=("peaky",) if seed % 2 else ("diffuse",))


@pytest.mark.parametrize("seed", range(6))
def test_seeded_random_ragged_batches(seed):
    """Ragged batches with drawn lengths and hyper-parameters, on a dense or a paged cache."""
    from paper_2505_10938_amd import cache as KC
    g = np.random.default_rng(2000 + seed)
    G = int(g.choice([32, 64]))
    kw = dict(bits=int(g.choice([2, 4])), group_k=G, group_v=int(g.choice([32, 128])),
              residual=int(g.choice([0, 16, 32, 64])), outlier_budget=int(g.choice([0, 2, 6])),
              q_heads=int(g.choice([2, 4, 8])), rho=0.05)
    lengths = [int(x) for x in g.integers(0, 5 * G + 60, size=int(g.choice([2, 3, 5])))]
    if max(lengths) == 0:
        lengths[0] = 1
    make = (lambda cfg: paged(cfg, seed=seed, kind=KC.RaggedKVCache)) if seed % 2 else None
    run_ragged(kw, lengths, make_cache=make)


@pytest.mark.parametrize("bits", [2, 4])
def test_degenerate_groups(bits):
    """Groups whose range is zero (step 0, every code 0), fp16 subnormals, signed zeros, a channel and a
    token of large values: the quantizer's decisions must still be the oracle's bit for bit and the
    attention finite and within tolerance."""
    import torch
    w = small("degenerate", batch=1, q_heads=2, kv_heads=2, context=32 * 8 + 40, residual=32, bits=bits,
              outlier_budget=2)
    K, V = S.layer_kv(w, 0)
    K, V = K.copy(), V.copy()
    K[:, :, 32:64, :] = np.float16(0.5)                       # a Key group that is constant in every channel
    K[:, :, 64:96, 5] = np.float16(-3.0)                      # one constant channel in the next group
    V[:, :, 40:44, :] = np.float16(1.25)                      # Value rows that are constant
    V[:, :, 100, 32:64] = np.float16(0.0)                     # one constant value group of one token
    K[:, :, 96:128, 7] = np.float16(6e-8) * (np.arange(32) % 3).astype(np.float16)     # subnormal range
    V[:, :, 130, :] = np.where(np.arange(128) % 2 == 0, np.float16(0.0), -np.float16(0.0))   # signed zeros
    K[:, :, 160:192, 9] = (np.arange(32) * 30 - 400).astype(np.float16)                 # a wide channel
    V[:, :, 170, :] = (np.arange(128) * 4 - 250).astype(np.float16)                     # a wide token
    states = H.oracle_states(w, K, V, w.n_quant)
    assert any((st.k_step == 0).any() for st in states) and any((st.v_step == 0).any() for st in states)
    cache = H.gpu_cache(w, K, V, w.n_quant, w.n_res)
    H.compare_state(cache, states, w, w.n_quant)
    for regime in ("peaky", "diffuse"):
        Q = S.layer_queries(w, 0, 0, regime)
        ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res)
        got = cache.decode(0, torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        assert att_err(got, ref) <= ATT_TOL, regime                 # the wide token can dominate an output row


# ---- the per-step Value schedule (the paper's comparison: Keys every G steps, Values at each step) ----

def per_step_states(w, K, V, n):
    """Oracle units of the per-step schedule with n tokens in the cache, every unit of the layer."""
    from oracle import kvq_oracle as O
    states = []
    for ui in range(w.batch * w.kv_heads):
        b, h = divmod(ui, w.kv_heads)
        st = O.PerStepValueUnit(w.head_dim, w.bits, w.group_k, w.group_v)
        st.advance_to(K[b, h], V[b, h], n, w.residual)
        states.append(st)
    return states


def compare_per_step_values(cache, states, w, n, layer=0):
    """Bit-exact: the Value codes, steps and zeros of the tokens between the last closed Key group
    and the window (tokens n_quant .. n - R - 1, inside partly written blocks), and the ring's Value
    rows of those tokens, which hold the dequantized rows."""
    from oracle import kvq_oracle as O
    cfg, sz = cache.cfg, cache.sizes
    nq, nqv = states[0].n_quant, states[0].n_quant_v
    assert nqv == max(0, n - w.residual) and cache.n_quant[layer] == nq
    if nqv == nq:
        return
    bb, nv = 512 * w.bits, w.head_dim // w.group_v
    nblk = cfg.max_seq // 32
    _, _, v_codes, v_meta, _ = (t.cpu().numpy() for t in cache.dense_quantized())
    vc = v_codes[:sz.units * nblk * bb].reshape(sz.units, nblk, bb)
    vm = v_meta.view(np.uint16)[:sz.units * nblk * 64 * nv].reshape(sz.units, nblk, 64 * nv)
    ring = cache.res_view("v").cpu().numpy()
    levels = (1 << w.bits) - 1
    u0 = layer * w.batch * w.kv_heads
    for i, st in enumerate(states):
        u = u0 + i
        for blk in range(nq // 32, (nqv + 31) // 32):
            t0, t1 = 32 * blk, min(32 * blk + 32, nqv)
            codes = np.zeros((32, w.head_dim), np.uint8)
            codes[:t1 - t0] = st.v_codes[t0:t1]
            written = np.zeros((32, w.head_dim), np.uint8)
            written[:t1 - t0] = levels
            want, bits_written = O.pack_v_block(codes, w.bits), O.pack_v_block(written, w.bits)
            assert np.array_equal(vc[u, blk] & bits_written, want), f"v_codes unit {i} block {blk}"
            step = np.zeros((32, nv), np.float16)
            zero = np.zeros((32, nv), np.float16)
            step[:t1 - t0], zero[:t1 - t0] = st.v_step[t0:t1], st.v_zero[t0:t1]
            meta = O.pack_v_meta(step, zero).view(np.uint16)[0]
            there = O.pack_v_meta(np.where(written[:, :nv] > 0, 1, 0).astype(np.float16),
                                  np.where(written[:, :nv] > 0, 1, 0).astype(np.float16)).view(np.uint16)[0] != 0
            assert np.array_equal(vm[u, blk][there], meta[there]), f"v_meta unit {i} block {blk}"
        for t in range(nq, nqv):
            row = (cache.res_start[layer] + t - nq) % sz.res_rows
            assert np.array_equal(ring[u, row].view(np.uint16), st.v_hat[t].view(np.uint16)), f"ring row of token {t}"


@pytest.mark.parametrize("kw", [
    dict(bits=2, group_k=32, group_v=32, residual=32, q_heads=4, kv_heads=2),
    dict(bits=4, group_k=32, group_v=64, residual=40, q_heads=2, kv_heads=2),
    dict(bits=2, group_k=64, group_v=128, residual=1, q_heads=8, kv_heads=1),
    dict(bits=4, group_k=128, group_v=32, residual=128, q_heads=2, kv_heads=2),
    dict(bits=2, group_k=32, group_v=32, residual=32, q_heads=4, kv_heads=2, paged_cache=True),
    dict(bits=4, group_k=64, group_v=64, residual=20, q_heads=2, kv_heads=2, paged_cache=True),
])
def test_per_step_value_schedule_streaming(kw):
    """Prefill, then decode steps under the per-step Value schedule: the attention of every step
    against the oracle's, the Value codes written token by token and the ring rows that hold
    dequantized Values bit for bit, and at the end the closed groups bit for bit - which are those of
    the every-G-steps schedule without tracing."""
    import torch
    from paper_2505_10938_amd import cache as KC
    kw = dict(kw)
    paged_cache = kw.pop("paged_cache", False)
    w = small("per_step", batch=2, outlier_budget=0, aux_capacity=0, context=300, **kw)
    G, R = w.group_k, w.residual
    steps = 2 * G + 9
    n0 = w.context
    K, V = S.layer_kv(w, 0, n0 + steps)
    ms = ((n0 + steps + G - 1) // G) * G
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, ms, w.bits, G, w.group_v, R, 0, 0, w.head_dim,
                         value_per_step=1)
    cache = paged(cfg) if paged_cache else KC.KVCache(cfg)       # (paged: the Value words go through the page table)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    cache.prefill(0, Kd[:, :, :n0].contiguous(), Vd[:, :, :n0].contiguous())
    torch.cuda.synchronize()
    compare_per_step_values(cache, per_step_states(w, K, V, n0), w, n0)
    worst = 0.0
    for s in range(steps):
        n = n0 + s + 1
        Q = S.layer_queries(w, 0, s, "peaky" if s % 2 else "diffuse")
        got = cache.step(0, Kd[:, :, n - 1].contiguous(), Vd[:, :, n - 1].contiguous(), torch.from_numpy(Q).cuda())
        states = per_step_states(w, K, V, n)
        nq = states[0].n_quant
        assert cache.n_quant[0] == nq and cache.n_res[0] == n - nq
        ref = H.oracle_attention(w, states, Q, K, V, nq, n - nq)
        worst = max(worst, att_err(got.cpu().numpy().astype(np.float64), ref))
        if s % 7 == 0 or s == steps - 1:
            compare_per_step_values(cache, states, w, n)
    assert worst <= ATT_TOL, worst
    # the closed groups: what the every-G-steps schedule leaves without tracing
    H.compare_state(cache, states, w, nq)
    plain = H.oracle_states(w, K, V, nq)
    H.compare_state(cache, plain, w, nq)


def test_per_step_value_schedule_batch_128_layer_sampled_units():
    """The schedule comparison's stack shape (batch 128, 8 kv heads of 4 query heads, no tracing: 1024 units
    per layer, one workgroup of two wavefronts each), second layer of two: a prompt, then steps through a
    group step; sampled units against the oracle, attention at every step, Value words and ring rows at
    the end."""
    import torch
    from paper_2505_10938_amd import cache as KC
    layer = 1
    w = S.WORKLOADS["mistral_7b_b128_4k"].with_(name="b128_per_step", layers=2, context=1024 + 128 + 25, outlier_budget=0,
                                                aux_capacity=0)
    G, R = w.group_k, w.residual
    steps = 12
    n0 = w.context
    K, V = S.layer_kv(w, layer, n0 + steps)
    ms = ((n0 + steps + G - 1) // G) * G
    cfg = KC.make_config(2, w.batch, w.q_heads, w.kv_heads, ms, w.bits, G, w.group_v, R, 0, 0, w.head_dim, value_per_step=1)
    assert B.kvq_decode_launch_shape(cfg, 1, w.n_quant, w.n_res)[:2] == (1, 2)
    cache = KC.KVCache(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    cache.prefill(layer, Kd[:, :, :n0].contiguous(), Vd[:, :, :n0].contiguous())
    units = [0, 7, 8 * 63 + 2, 1023]
    from oracle import kvq_oracle as O
    g = w.q_heads // w.kv_heads
    states = {}
    for ui in units:
        b, h = divmod(ui, w.kv_heads)
        states[ui] = O.PerStepValueUnit(w.head_dim, w.bits, G, w.group_v)
    group_steps = 0
    for s in range(steps):
        n = n0 + s + 1
        Q = S.layer_queries(w, layer, s, "peaky" if s % 2 else "diffuse")
        nq_before = cache.n_quant[layer]
        got = cache.step(layer, Kd[:, :, n - 1].contiguous(), Vd[:, :, n - 1].contiguous(),
                         torch.from_numpy(Q).cuda()).cpu().numpy().astype(np.float64)
        group_steps += cache.n_quant[layer] != nq_before
        for ui in units:
            b, h = divmod(ui, w.kv_heads)
            st = states[ui]
            st.advance_to(K[b, h], V[b, h], n, R)
            assert cache.n_quant[layer] == st.n_quant
            ref, _ = O.decode_attention(Q[b, h * g:(h + 1) * g], st, K[b, h, st.n_quant:n], V[b, h, st.n_quant:n])
            assert att_err(got[b, h * g:(h + 1) * g], ref) <= ATT_TOL, (s, ui)
    assert group_steps == 1
    # the state at the end: closed groups, the Value words written token by token, the ring rows that hold
    # dequantized Values
    nq, nqv = states[units[0]].n_quant, states[units[0]].n_quant_v
    H.compare_state(cache, [states[ui] for ui in units], w, nq, layer=layer, units=units)
    sz = cache.sizes
    ring = cache.res_view("v").cpu().numpy()
    _, _, v_codes, _, _ = (t.cpu().numpy() for t in cache.dense_quantized())
    bb = 512 * w.bits
    vc = v_codes[:sz.units * (cfg.max_seq // 32) * bb].reshape(sz.units, cfg.max_seq // 32, bb)
    for ui in units:
        st = states[ui]
        u = layer * w.units + ui
        for t in range(nq, nqv):
            row = (cache.res_start[layer] + t - nq) % sz.res_rows
            assert np.array_equal(ring[u, row].view(np.uint16), st.v_hat[t].view(np.uint16)), (ui, t)
        blk = nq // 32
        codes = np.zeros((32, w.head_dim), np.uint8)
        written = np.zeros((32, w.head_dim), np.uint8)
        codes[:nqv - nq] = st.v_codes[nq:nqv]
        written[:nqv - nq] = (1 << w.bits) - 1
        assert np.array_equal(vc[u, blk] & O.pack_v_block(written, w.bits), O.pack_v_block(codes, w.bits)), ui
    assert not cache.v_codes[:w.units * (cfg.max_seq // 32) * bb].any()        # the first layer was not touched


def test_per_step_value_schedule_from_an_empty_cache():
    """No prompt: the first tokens stay inside the window, then Values start to leave it one by one
    before any Key group closes."""
    import torch
    from paper_2505_10938_amd import cache as KC
    w = small("per_step_empty", batch=1, q_heads=4, kv_heads=2, outlier_budget=0, aux_capacity=0, residual=16,
              context=0)
    G, R = w.group_k, w.residual
    steps = R + G + 5
    K, V = S.layer_kv(w, 0, steps)
    cfg = KC.make_config(1, w.batch, w.q_heads, w.kv_heads, 4 * G, w.bits, G, w.group_v, R, 0, 0, w.head_dim,
                         value_per_step=1)
    cache = KC.KVCache(cfg)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    for s in range(steps):
        n = s + 1
        Q = S.layer_queries(w, 0, s, "peaky")
        got = cache.step(0, Kd[:, :, s].contiguous(), Vd[:, :, s].contiguous(), torch.from_numpy(Q).cuda())
        states = per_step_states(w, K, V, n)
        nq = states[0].n_quant
        ref = H.oracle_attention(w, states, Q, K, V, nq, n - nq)
        assert att_err(got.cpu().numpy().astype(np.float64), ref) <= ATT_TOL, s
        compare_per_step_values(cache, states, w, n)
