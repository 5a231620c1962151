"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, reports
buffer sizes, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

import paper_2505_10938_amd as P
from paper_2505_10938_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def cfg(**kw):
    base = dict(layers=1, batch=2, q_heads=8, kv_heads=2, head_dim=128, max_seq=1024, bits=2, group_k=32,
                group_v=32, residual=128, outlier_budget=8, aux_capacity=32)
    base.update(kw)
    return P.kvq_config(**base)


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "kvq.h")).read()
    declared = set(re.findall(r"\b(kvq_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = P.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert P.kvq_version() >= 1
    assert P.status_string(0) == "ok" and "workspace" in P.status_string(B.KVQ_ERR_WORKSPACE)


def test_sizes():
    s = P.kvq_query_sizes(cfg())
    assert s.units == 4 and s.res_rows == 160 and s.pool_slots == 40
    assert s.k_codes_bytes == 4 * 1024 // 32 * 1024          # 2 bits: 1 KiB per 32-token block
    assert s.k_meta_bytes == 4 * (1024 // 32) * 128 * 4
    assert s.v_meta_bytes == 4 * 1024 * 4 * 4
    # bytes per quantized token per unit: 96 at 2-bit, G=32, Gv=32
    per_tok = (s.k_codes_bytes + s.v_codes_bytes + s.k_meta_bytes + s.v_meta_bytes) / (4 * 1024)
    assert per_tok == 96
    s4 = P.kvq_query_sizes(cfg(bits=4))
    assert (s4.k_codes_bytes + s4.v_codes_bytes + s4.k_meta_bytes + s4.v_meta_bytes) / (4 * 1024) == 160
    # residual ring is a whole number of groups: R=32, G=128 -> 256 rows
    assert P.kvq_query_sizes(cfg(group_k=128, residual=32, max_seq=1024)).res_rows == 256


@pytest.mark.parametrize("kw,status", [
    (dict(bits=3), B.KVQ_ERR_INVALID_ARG),
    (dict(group_k=48), B.KVQ_ERR_INVALID_ARG),
    (dict(group_v=16), B.KVQ_ERR_INVALID_ARG),
    (dict(max_seq=1000), B.KVQ_ERR_INVALID_ARG),
    (dict(q_heads=7), B.KVQ_ERR_INVALID_ARG),
    (dict(residual=-1), B.KVQ_ERR_INVALID_ARG),
    (dict(head_dim=64, group_v=32), B.KVQ_ERR_UNSUPPORTED),
    (dict(q_heads=6, kv_heads=2), B.KVQ_ERR_UNSUPPORTED),
    (dict(outlier_budget=100), B.KVQ_ERR_UNSUPPORTED),
])
def test_bad_config(kw, status):
    with pytest.raises(P.KvqError) as e:
        P.kvq_query_sizes(cfg(**kw))
    assert e.value.status == status


def test_bad_call_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    ws = P.kvq_query_sizes(c).workspace_bytes
    dec = lambda **k: lib.kvq_decode_attention(C.byref(c), k.get("layer", 0), k.get("q", 256), qc,
                                               k.get("n_quant", 64), res, k.get("res_start", 0),
                                               k.get("n_res", 10), pool, k.get("out", 256), k.get("ws", 512),
                                               k.get("wsb", ws), None)
    assert dec(layer=1) == B.KVQ_ERR_INVALID_ARG
    assert dec(q=None) == B.KVQ_ERR_INVALID_ARG
    assert dec(n_quant=33) == B.KVQ_ERR_INVALID_ARG
    assert dec(n_quant=2048) == B.KVQ_ERR_INVALID_ARG
    assert dec(n_res=161) == B.KVQ_ERR_INVALID_ARG
    assert dec(n_quant=0, n_res=0) == B.KVQ_ERR_INVALID_ARG
    assert dec(wsb=ws - 1) == B.KVQ_ERR_WORKSPACE
    assert dec(ws=None) == B.KVQ_ERR_WORKSPACE
    assert dec(ws=520) == B.KVQ_ERR_WORKSPACE                # not 256-byte aligned
    tr = lambda **k: lib.kvq_trace_outliers(C.byref(c), 0, k.get("gi", 0), k.get("kg", 256), 256,
                                            k.get("stride", 32 * 128), pool, k.get("sel", 256), None)
    assert tr(gi=32) == B.KVQ_ERR_INVALID_ARG
    assert tr(stride=100) == B.KVQ_ERR_INVALID_ARG
    assert tr(kg=258) == B.KVQ_ERR_INVALID_ARG
    assert tr(sel=None) == B.KVQ_ERR_INVALID_ARG
    qz = lambda **k: lib.kvq_quantize_group(C.byref(c), 0, k.get("gi", 0), k.get("kg", 256), 256, 32 * 128, None,
                                            k.get("qc", qc), None)
    assert qz(gi=-1) == B.KVQ_ERR_INVALID_ARG
    assert qz(qc=B.kvq_qcache(256, 0, 256, 256, 256)) == B.KVQ_ERR_INVALID_ARG
    ap = lambda **k: lib.kvq_append_residual(C.byref(c), 0, 256, 256, res, k.get("start", 0), k.get("n", 0), None)
    assert ap(start=160) == B.KVQ_ERR_INVALID_ARG
    assert ap(n=160) == B.KVQ_ERR_INVALID_ARG
    rd = lambda **k: lib.kvq_stream_read(k.get("buf", 256), k.get("n", 1024), k.get("sink", 256), None)
    assert rd(buf=None) == B.KVQ_ERR_INVALID_ARG
    assert rd(sink=None) == B.KVQ_ERR_INVALID_ARG
    assert rd(buf=260) == B.KVQ_ERR_INVALID_ARG
    assert rd(n=0) == B.KVQ_ERR_INVALID_ARG
    assert rd(n=1000) == B.KVQ_ERR_INVALID_ARG
    fz = lambda **k: lib.kvq_append_trace_quantize(C.byref(c), 0, 256, 256, res, k.get("start", 0), k.get("n", 159),
                                                   k.get("nq", 64), k.get("pool", pool), None, k.get("qc", qc), None)
    assert fz(n=100) == B.KVQ_ERR_INVALID_ARG                # ring not full after the append
    assert fz(start=16) == B.KVQ_ERR_INVALID_ARG             # oldest group not one contiguous block
    assert fz(nq=48) == B.KVQ_ERR_INVALID_ARG
    assert fz(nq=1024) == B.KVQ_ERR_INVALID_ARG              # no room for another group
    assert fz(qc=B.kvq_qcache(256, 256, 256, 256, 0)) == B.KVQ_ERR_INVALID_ARG
    assert fz(pool=B.kvq_pool(256, 256, 256, 256, 0, 256, 256)) == B.KVQ_ERR_INVALID_ARG
    pf = lambda **k: lib.kvq_prefill_quantize(C.byref(c), 0, k.get("kr", 256), 256, k.get("stride", 4096 * 128),
                                              k.get("n", 1000), k.get("pool", pool), k.get("sel", 256), qc, res, None)
    assert pf(n=0) == B.KVQ_ERR_INVALID_ARG
    assert pf(n=1024 + 128 + 32) == B.KVQ_ERR_INVALID_ARG     # more than max_seq + R + G - 1 tokens
    assert pf(stride=100) == B.KVQ_ERR_INVALID_ARG
    assert pf(kr=258) == B.KVQ_ERR_INVALID_ARG
    assert pf(sel=None) == B.KVQ_ERR_INVALID_ARG
    assert pf(pool=B.kvq_pool(256, 256, 256, 256, 256, 256, 0)) == B.KVQ_ERR_INVALID_ARG


def test_bad_ragged_call_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    ws = P.kvq_query_sizes(c).workspace_bytes
    dec = lambda **k: lib.kvq_decode_attention_ragged(C.byref(c), k.get("layer", 0), 256, k.get("qc", qc), res,
                                                      k.get("seq", 256), k.get("mq", 64), k.get("mr", 10), pool, 256,
                                                      k.get("ws", 512), ws, None)
    assert dec(seq=None) == B.KVQ_ERR_INVALID_ARG
    assert dec(seq=260) == B.KVQ_ERR_INVALID_ARG             # the state array is read 16 bytes at a time
    assert dec(mq=40) == B.KVQ_ERR_INVALID_ARG               # the bound is a multiple of the group size
    assert dec(mq=2048) == B.KVQ_ERR_INVALID_ARG
    assert dec(mr=161) == B.KVQ_ERR_INVALID_ARG
    assert dec(mq=0, mr=0) == B.KVQ_ERR_INVALID_ARG
    assert dec(layer=1) == B.KVQ_ERR_INVALID_ARG
    assert dec(qc=B.kvq_qcache(256, 256, 0, 256, 256)) == B.KVQ_ERR_INVALID_ARG
    assert dec(ws=None) == B.KVQ_ERR_WORKSPACE
    st = lambda **k: lib.kvq_append_trace_quantize_ragged(C.byref(c), k.get("layer", 0), k.get("kn", 256), 256, res,
                                                          k.get("seq", 256), k.get("pool", pool), None,
                                                          k.get("qc", qc), None)
    assert st(seq=None) == B.KVQ_ERR_INVALID_ARG
    assert st(seq=264) == B.KVQ_ERR_INVALID_ARG
    assert st(kn=None) == B.KVQ_ERR_INVALID_ARG
    assert st(layer=-1) == B.KVQ_ERR_INVALID_ARG
    assert st(qc=B.kvq_qcache(0, 256, 256, 256, 256)) == B.KVQ_ERR_INVALID_ARG
    assert st(pool=B.kvq_pool(256, 256, 256, 256, 256, 256, 0)) == B.KVQ_ERR_INVALID_ARG
    adv = lambda seq: lib.kvq_seq_advance(C.byref(c), seq, None)
    assert adv(None) == B.KVQ_ERR_INVALID_ARG
    assert adv(8) == B.KVQ_ERR_INVALID_ARG


def test_bad_append_decode_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    ws = P.kvq_query_sizes(c).workspace_bytes
    ad = lambda **k: lib.kvq_append_decode_attention(C.byref(c), 0, 256, k.get("kn", 256), k.get("vn", 256), qc,
                                                     k.get("nq", 64), k.get("res", res), 0, k.get("n", 10), pool, 256,
                                                     512, ws, None)
    assert ad(kn=None) == B.KVQ_ERR_INVALID_ARG
    assert ad(vn=None) == B.KVQ_ERR_INVALID_ARG
    assert ad(kn=258) == B.KVQ_ERR_INVALID_ARG               # rows are read 4 bytes at a time
    assert ad(n=159) == B.KVQ_ERR_INVALID_ARG                # the token would fill the ring: group step first
    assert ad(n=160) == B.KVQ_ERR_INVALID_ARG
    assert ad(nq=48) == B.KVQ_ERR_INVALID_ARG
    assert ad(res=B.kvq_residual(0, 256)) == B.KVQ_ERR_INVALID_ARG


def test_bad_page_tables_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    ws = P.kvq_query_sizes(c).workspace_bytes
    groups = c.max_seq // c.group_k
    paged = lambda table=256, stride=groups, pages=50: B.kvq_qcache(256, 256, 256, 256, 256, table, stride, pages)
    dec = lambda qc: lib.kvq_decode_attention(C.byref(c), 0, 256, qc, 64, res, 0, 10, pool, 256, 512, ws, None)
    step = lambda qc: lib.kvq_append_trace_quantize(C.byref(c), 0, 256, 256, res, 0, c.residual + c.group_k - 1, 64,
                                                    pool, None, qc, None)
    for call in (dec, step):
        assert call(paged(pages=0)) == B.KVQ_ERR_INVALID_ARG            # an empty pool
        assert call(paged(pages=-3)) == B.KVQ_ERR_INVALID_ARG
        assert call(paged(pages=(1 << 20) + 1)) == B.KVQ_ERR_INVALID_ARG
        assert call(paged(stride=groups - 1)) == B.KVQ_ERR_INVALID_ARG  # a table row shorter than a sequence can get
        assert call(paged(table=258)) == B.KVQ_ERR_INVALID_ARG          # int32 entries
    # a plane's codes must stay below 4 GiB (the kernels' block offsets are 32-bit): with 128-token groups
    # and 4-bit codes a page is 8 KiB of codes per plane, so 2^19 pages are one too many
    big = cfg(group_k=128, group_v=128, bits=4, max_seq=1024)
    ws_big = P.kvq_query_sizes(big).workspace_bytes
    for pages, want_ok in (((1 << 19) - 1, True), (1 << 19, False), (1 << 20, False)):
        qc = B.kvq_qcache(256, 256, 256, 256, 256, 256, big.max_seq // big.group_k, pages)
        # (a null workspace is looked at after the cache: it tells an accepted cache from a rejected one, no launch)
        st = lib.kvq_decode_attention(C.byref(big), 0, 256, qc, 128, res, 0, 10, pool, 256, 0, ws_big, None)
        assert st == (B.KVQ_ERR_WORKSPACE if want_ok else B.KVQ_ERR_INVALID_ARG), (pages, st)
    small_pages = cfg(group_k=32, bits=2)
    qc = B.kvq_qcache(256, 256, 256, 256, 256, 256, small_pages.max_seq // 32, 1 << 20)    # 1 GiB per plane: fine
    assert lib.kvq_decode_attention(C.byref(small_pages), 0, 256, qc, 64, res, 0, 10, pool, 256, 0, ws, None) == \
        B.KVQ_ERR_WORKSPACE
    # the quantized arrays are needed even with nothing quantized: the first block is always loaded
    assert lib.kvq_decode_attention(C.byref(c), 0, 256, B.kvq_qcache(0, 256, 256, 256, 256), 0, res, 0, 10, pool, 256,
                                    512, ws, None) == B.KVQ_ERR_INVALID_ARG


def test_misaligned_decode_buffers_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    ws = P.kvq_query_sizes(c).workspace_bytes
    def dec(q=256, qc=(256,) * 5, res=(256, 256), rows=(256, 256), out=256):
        pool = B.kvq_pool(rows[0], rows[1], 256, 256, 256, 256, 256)
        return lib.kvq_decode_attention(C.byref(c), 0, q, B.kvq_qcache(*qc), 64, B.kvq_residual(*res), 0, 10, pool, out,
                                        512, ws, None)
    bad = B.KVQ_ERR_INVALID_ARG
    assert dec(q=264) == bad                                  # rows are read 16 bytes at a time
    assert dec(res=(264, 256)) == bad and dec(res=(256, 260)) == bad
    assert dec(rows=(258, 256)) == bad and dec(rows=(256, 264)) == bad
    assert dec(qc=(264, 256, 256, 256, 256)) == bad and dec(qc=(256, 256, 260, 256, 256)) == bad
    assert dec(qc=(256, 258, 256, 256, 256)) == bad and dec(qc=(256, 256, 256, 256, 257)) == bad
    assert dec(out=257) == bad
    assert dec(rows=(0, 256)) == bad                          # pool slots exist (N + A > 0): their rows are read


def test_bad_sequence_prefill_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    pf = lambda seq=0, n=300, stride=300 * 128, k=256: lib.kvq_prefill_quantize_seq(
        C.byref(c), 0, seq, k, 256, stride, n, pool, 256, qc, res, None)
    assert pf(seq=-1) == B.KVQ_ERR_INVALID_ARG
    assert pf(seq=c.batch) == B.KVQ_ERR_INVALID_ARG
    assert pf(n=0) == B.KVQ_ERR_INVALID_ARG
    assert pf(stride=299 * 128) == B.KVQ_ERR_INVALID_ARG
    assert pf(k=264) == B.KVQ_ERR_INVALID_ARG
    assert lib.kvq_prefill_quantize_seq(None, 0, 0, 256, 256, 300 * 128, 300, pool, 256, qc, res, None) == B.KVQ_ERR_INVALID_ARG


def test_untraced_layers_must_fit_the_layer_count():
    assert P.load_library().kvq_query_sizes(C.byref(cfg(layers=3, untraced_layers=3)), C.byref(B.kvq_sizes())) == B.KVQ_OK
    for bad in (-1, 4):
        assert P.load_library().kvq_query_sizes(C.byref(cfg(layers=3, untraced_layers=bad)),
                                                C.byref(B.kvq_sizes())) == B.KVQ_ERR_INVALID_ARG


def test_per_step_value_schedule_configuration_and_arguments():
    lib = P.load_library()
    sz = B.kvq_sizes()
    ok = cfg(outlier_budget=0, aux_capacity=0, value_per_step=1)
    assert lib.kvq_query_sizes(C.byref(ok), C.byref(sz)) == B.KVQ_OK
    assert sz.v_codes_bytes == P.kvq_query_sizes(cfg(outlier_budget=0, aux_capacity=0)).v_codes_bytes
    assert lib.kvq_query_sizes(C.byref(cfg(outlier_budget=0, value_per_step=2)), C.byref(sz)) == B.KVQ_ERR_INVALID_ARG
    # the schedule of the method without tracing; the token that leaves the window must be in the ring
    assert lib.kvq_query_sizes(C.byref(cfg(value_per_step=1)), C.byref(sz)) == B.KVQ_ERR_UNSUPPORTED
    assert lib.kvq_query_sizes(C.byref(cfg(outlier_budget=0, residual=0, value_per_step=1)), C.byref(sz)) == B.KVQ_ERR_UNSUPPORTED
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    call = lambda c=ok, first=0, count=1, v=256, row=0, qc=qc: lib.kvq_quantize_value_tokens(
        C.byref(c), 0, first, count, v, row, qc, None)
    bad = B.KVQ_ERR_INVALID_ARG
    assert call(c=cfg(outlier_budget=0)) == bad                # the configuration quantizes Values with their group
    assert call(first=-1) == bad and call(count=0) == bad and call(count=161) == bad
    assert call(first=1024) == bad and call(first=1000, count=25) == bad   # past the quantized capacity
    assert call(row=-1) == bad and call(row=160) == bad
    assert call(v=None) == bad and call(v=258) == bad
    assert call(qc=B.kvq_qcache(256, 256, 0, 256, 256)) == bad
    # entry points that do not support the schedule
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    assert lib.kvq_append_trace_quantize_ragged(C.byref(ok), 0, 256, 256, res, 256, pool, None, qc, None) == B.KVQ_ERR_UNSUPPORTED
    assert lib.kvq_prefill_quantize_seq(C.byref(ok), 0, 0, 256, 256, 512 * 128, 512, pool, 256, qc, res, None) == B.KVQ_ERR_UNSUPPORTED


def test_launch_plan_sizes_and_arguments():
    lib = P.load_library()
    c = cfg(batch=32, q_heads=32, kv_heads=8, max_seq=8192)
    # 256 compute units x 2 workgroups of 4 wavefronts / 8 kv heads = 64 entries, twice the sequences
    assert B.kvq_seq_plan_bytes(c) == (8 + 8 * 64) * 4
    assert B.kvq_seq_plan_bytes(cfg(batch=2, q_heads=8, kv_heads=2)) == (8 + 8 * 128) * 4
    big = cfg(batch=2000, q_heads=8, kv_heads=8)
    assert lib.kvq_seq_plan_bytes(C.byref(big)) == B.KVQ_ERR_UNSUPPORTED           # more than 1024 sequences
    assert lib.kvq_seq_plan_bytes(C.byref(cfg(batch=600, q_heads=8, kv_heads=8))) == B.KVQ_ERR_UNSUPPORTED  # do not fit
    plan = lambda seq=256, nq=8192, nr=128, pl=512: lib.kvq_seq_plan(C.byref(c), seq, nq, nr, pl, None)
    bad = B.KVQ_ERR_INVALID_ARG
    assert plan(seq=None) == bad and plan(seq=260) == bad and plan(pl=None) == bad and plan(pl=520) == bad
    assert plan(nq=8200) == bad and plan(nq=8224) == bad and plan(nr=161) == bad and plan(nr=-1) == bad
    # the workspace the sizes report covers the planned launch: one partial result per entry and kv head
    s = P.kvq_query_sizes(c)
    assert s.workspace_bytes >= 64 * 8 * 4 * (128 + 2) * 4
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    dec = lambda pl=512, ws=s.workspace_bytes: lib.kvq_decode_attention_planned(
        C.byref(c), 0, 256, qc, res, pl, 8192, 128, pool, 256, 256, ws, None)
    assert dec(pl=None) == bad and dec(pl=516) == bad
    assert dec(ws=s.workspace_bytes - 1) == B.KVQ_ERR_WORKSPACE


def test_bad_rotary_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    ws = P.kvq_query_sizes(c).workspace_bytes
    dec = lambda k=256, v=256, rope=256, stride=0, n_res=10: lib.kvq_append_decode_attention_rope(
        C.byref(c), 0, 256, k, v, rope, stride, qc, 64, res, 0, n_res, pool, 256, 256, ws, None)
    bad = B.KVQ_ERR_INVALID_ARG
    assert dec(rope=None) == bad and dec(rope=264) == bad            # no table; not 16-byte aligned
    assert dec(k=None) == bad and dec(v=None) == bad                 # the rotation comes with the append only
    assert dec(stride=64) == bad and dec(stride=130) == bad and dec(stride=-128) == bad
    assert dec(n_res=c.residual + c.group_k - 1) == bad              # the ring would fill: not this entry point's step
    rot = lambda x=256, heads=8, rope=256, stride=128, out=512: lib.kvq_rope_rotate(
        C.byref(c), x, heads, rope, stride, out, None)
    assert rot(x=None) == bad and rot(out=None) == bad and rot(rope=None) == bad
    assert rot(x=258) == bad and rot(out=514) == bad and rot(rope=260) == bad
    assert rot(heads=0) == bad and rot(stride=100) == bad and rot(stride=126) == bad


def test_bad_dequantize_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    dq = lambda nq=256, t0=0, n=64, ko=256, stride=64 * 128, qc=qc, pool=pool: lib.kvq_dequantize(
        C.byref(c), 0, qc, nq, pool, t0, n, ko, 256, stride, None)
    bad = B.KVQ_ERR_INVALID_ARG
    assert dq(nq=250) == bad                                  # not a multiple of the group size
    assert dq(t0=16) == bad and dq(n=48) == bad and dq(n=0) == bad
    assert dq(t0=224, n=64) == bad                            # window past the quantized segment
    assert dq(ko=None) == bad and dq(ko=257) == bad
    assert dq(stride=64 * 128 - 1) == bad
    assert dq(qc=B.kvq_qcache(256, 0, 256, 256, 256)) == bad
    assert dq(pool=B.kvq_pool(256, 256, 0, 256, 256, 256, 256)) == bad     # token indices are needed


def test_bad_multi_token_decode_arguments_rejected_before_launch():
    lib = P.load_library()
    c = cfg()                                                  # 8 query heads on 2 kv heads: g = 4
    qc = B.kvq_qcache(256, 256, 256, 256, 256)
    pool = B.kvq_pool(256, 256, 256, 256, 256, 256, 256)
    res = B.kvq_residual(256, 256)
    ws = P.kvq_query_sizes(c).workspace_bytes
    assert P.kvq_decode_workspace_bytes(c, 1) == ws and P.kvq_decode_workspace_bytes(c, 2) >= ws
    assert lib.kvq_decode_workspace_bytes(C.byref(c), 3) == B.KVQ_ERR_UNSUPPORTED
    assert lib.kvq_decode_workspace_bytes(C.byref(c), 0) == B.KVQ_ERR_INVALID_ARG
    dm = lambda t, n_res=10, wsb=8 * ws: lib.kvq_decode_attention_multi(C.byref(c), 0, 256, t, qc, 64, res, 0, n_res,
                                                                        pool, 256, 512, wsb, None)
    assert dm(0) == B.KVQ_ERR_INVALID_ARG and dm(9) == B.KVQ_ERR_INVALID_ARG
    assert dm(3) == B.KVQ_ERR_UNSUPPORTED                     # 12 rows per kv head
    assert dm(4) == B.KVQ_ERR_UNSUPPORTED                     # 16 rows per kv head
    assert dm(2, n_res=0) == B.KVQ_ERR_INVALID_ARG            # the token to hide must be a residual row
    assert dm(2, wsb=ws // 2) == B.KVQ_ERR_WORKSPACE


def test_header_is_plain_c_and_cxx():
    """include/kvq.h compiles on its own as C99 and as C++11 (no torch or HIP types in the boundary)."""
    import shutil
    import subprocess
    header = os.path.join(ROOT, "include", "kvq.h")
    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("no host compiler")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", header],
                ["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", header]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
