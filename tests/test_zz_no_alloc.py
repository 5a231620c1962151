"""The decode entry point that allocates nothing (kvq_decode_attention_static): its output against
kvq_decode_attention's on the same cache, bit for bit, on two calls in a row that share the library's
static scratch array, the second with a smaller input and a different split."""
import numpy as np
import pytest

import kvq_synth as S
from paper_2505_10938_amd import binding as B
from paper_2505_10938_amd import cache as KC
from tests import helpers as H


def _config(w):
    G = w.group_k
    return KC.make_config(w.layers, w.batch, w.q_heads, w.kv_heads, max(G, ((w.n_quant + G - 1) // G) * G), w.bits, G,
                          w.group_v, w.residual, w.outlier_budget, w.aux_capacity, w.head_dim)


def test_problem_beyond_the_scratch_array_is_rejected_on_the_host():
    # 32768 units x 8 query rows x 520 bytes of partial results: far beyond 4 MiB; nothing is launched
    big = KC.make_config(1, 4096, 64, 8, 1024)
    assert B.kvq_decode_workspace_bytes(big, 1) > (4 << 20)
    lib = B.load_library()
    import ctypes as C
    st = lib.kvq_decode_attention_static(C.byref(big), 0, 256, B.kvq_qcache(256, 256, 256, 256, 256), 64,
                                         B.kvq_residual(256, 256), 0, 10, B.kvq_pool(256, 256, 256, 256, 256, 256, 256),
                                         256, None)
    assert st == B.KVQ_ERR_SCRATCH
    assert "scratch" in B.status_string(st)


@pytest.mark.gpu
def test_static_scratch_decode_equals_the_workspace_entry_point():
    import torch
    first = S.Workload("static_long", 1, 1, 8, 2, 6000 + 70, outlier_budget=8)           # 2 units, many workgroups each
    second = S.Workload("static_small", 1, 4, 8, 2, 1024 + 45, bits=4, outlier_budget=4)  # 8 units, fewer tokens
    third = S.Workload("static_one_workgroup", 1, 64, 8, 8, 512 + 40)                      # 512 units: no split
    shapes = []
    for w in (first, second, third, first):
        cfg = _config(w)
        K, V = S.layer_kv(w, 0)
        cache = KC.KVCache(cfg)
        cache.prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
        shapes.append(B.kvq_decode_launch_shape(cfg, 1, w.n_quant, w.n_res + w.outlier_budget + w.aux_capacity))
        for regime in ("peaky", "diffuse"):
            q = torch.from_numpy(S.layer_queries(w, 0, 0, regime)).cuda()
            want = cache.decode(0, q)
            got = torch.full_like(want, float("nan"))
            print(f"static-scratch decode: {w.name} {regime} shape {shapes[-1]}", flush=True)
            B.kvq_decode_attention_static(cfg, 0, q, cache.qcache, cache.n_quant[0], cache.res, cache.res_start[0],
                                          cache.n_res[0], cache.pool, got)
            torch.cuda.synchronize()
            assert torch.equal(got, want), (w.name, regime)
        # and against the oracle, on one unit, so that "equal" is not "equally wrong"
        states = H.oracle_states(w, K, V, w.n_quant, [1])
        Q = S.layer_queries(w, 0, 0, "peaky")
        ref = H.oracle_attention(w, states, Q, K, V, w.n_quant, w.n_res, [1])
        q = torch.from_numpy(Q).cuda()
        got = torch.empty_like(q)
        B.kvq_decode_attention_static(cfg, 0, q, cache.qcache, cache.n_quant[0], cache.res, cache.res_start[0],
                                      cache.n_res[0], cache.pool, got)
        g = w.q_heads // w.kv_heads
        b, h = divmod(1, w.kv_heads)
        err = H.att_err(got.cpu().numpy().astype(np.float64)[b, h * g:(h + 1) * g], ref[b, h * g:(h + 1) * g], H.AttStats())
        assert err <= H.ATT_TOL, (w.name, err)
    assert shapes[0][0] > 1 and shapes[1][0] > 1 and shapes[2][0] == 1, shapes
