"""Thin ctypes binding of libkvq.so: argument marshalling only.

Every function has the name and the argument order of its C entry point (see
include/kvq.h).  Tensors are torch CUDA tensors used as raw device memory; no
arithmetic of the method happens here.  The library must have been built
(`python -m paper_2505_10938_amd.build` or `__graft_entry__.build()`); a missing
library is an error, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libkvq.so")

KVQ_OK, KVQ_ERR_INVALID_ARG, KVQ_ERR_UNSUPPORTED, KVQ_ERR_WORKSPACE, KVQ_ERR_LAUNCH, KVQ_ERR_SCRATCH = 0, -1, -2, -3, -4, -5

INTERFACE_VERSION = 6       # kvq_version() of the library these structures and signatures match
EXPORTS = ["kvq_query_sizes", "kvq_append_residual", "kvq_trace_outliers", "kvq_quantize_group",
           "kvq_append_trace_quantize", "kvq_prefill_quantize", "kvq_prefill_quantize_seq", "kvq_decode_attention",
           "kvq_append_decode_attention", "kvq_append_decode_attention_rope", "kvq_rope_rotate",
           "kvq_append_trace_quantize_ragged", "kvq_seq_advance",
           "kvq_decode_attention_ragged", "kvq_decode_attention_multi", "kvq_decode_workspace_bytes",
           "kvq_decode_launch_shape", "kvq_decode_attention_static", "kvq_dequantize", "kvq_stream_read",
           "kvq_quantize_value_tokens", "kvq_seq_plan_bytes", "kvq_seq_plan", "kvq_decode_attention_planned",
           "kvq_status_string", "kvq_version"]


class kvq_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("layers", "batch", "q_heads", "kv_heads", "head_dim", "max_seq", "bits", "group_k",
                 "group_v", "residual", "outlier_budget", "aux_capacity", "untraced_layers", "value_per_step")]


class kvq_sizes(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("units", "res_rows", "pool_slots", "k_codes_bytes", "k_meta_bytes", "v_codes_bytes",
                 "v_meta_bytes", "mask_bytes", "res_bytes", "pool_rows_bytes", "pool_idx_bytes",
                 "pool_score_bytes", "counter_bytes", "selected_bytes", "workspace_bytes",
                 "prefill_selected_bytes")]


class kvq_qcache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_codes", "k_meta", "v_codes", "v_meta", "mask", "page_table")] + \
               [("table_stride", C.c_int32), ("n_pages", C.c_int32)]


class kvq_pool(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("pool_k", "pool_v", "pool_idx", "pool_score", "pool_count", "aux_count", "frozen")]


class kvq_residual(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_res", "v_res")]


class KvqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library() -> C.CDLL:
    """Load libkvq.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2505_10938_amd.build`")
    lib = C.CDLL(LIB_PATH)
    i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
    cfgp = C.POINTER(kvq_config)
    lib.kvq_version.restype = i32
    if lib.kvq_version() != INTERFACE_VERSION:          # the structures below would not match the library's
        raise RuntimeError(f"{LIB_PATH} has interface version {lib.kvq_version()}, this binding {INTERFACE_VERSION}: "
                           "rebuild with `python -m paper_2505_10938_amd.build`")
    lib.kvq_status_string.restype = C.c_char_p
    lib.kvq_status_string.argtypes = [i32]
    lib.kvq_query_sizes.restype = i32
    lib.kvq_query_sizes.argtypes = [cfgp, C.POINTER(kvq_sizes)]
    lib.kvq_stream_read.restype = i32
    lib.kvq_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
    lib.kvq_append_residual.restype = i32
    lib.kvq_append_residual.argtypes = [cfgp, i32, vp, vp, kvq_residual, i32, i32, vp]
    lib.kvq_trace_outliers.restype = i32
    lib.kvq_trace_outliers.argtypes = [cfgp, i32, i32, vp, vp, i64, kvq_pool, vp, vp]
    lib.kvq_quantize_group.restype = i32
    lib.kvq_quantize_group.argtypes = [cfgp, i32, i32, vp, vp, i64, vp, kvq_qcache, vp]
    lib.kvq_quantize_value_tokens.restype = i32
    lib.kvq_quantize_value_tokens.argtypes = [cfgp, i32, i32, i32, vp, i32, kvq_qcache, vp]
    lib.kvq_prefill_quantize.restype = i32
    lib.kvq_prefill_quantize.argtypes = [cfgp, i32, vp, vp, i64, i32, kvq_pool, vp, kvq_qcache, kvq_residual, vp]
    lib.kvq_prefill_quantize_seq.restype = i32
    lib.kvq_prefill_quantize_seq.argtypes = [cfgp, i32, i32, vp, vp, i64, i32, kvq_pool, vp, kvq_qcache, kvq_residual, vp]
    lib.kvq_append_trace_quantize.restype = i32
    lib.kvq_append_trace_quantize.argtypes = [cfgp, i32, vp, vp, kvq_residual, i32, i32, i32, kvq_pool, vp, kvq_qcache, vp]
    lib.kvq_decode_attention.restype = i32
    lib.kvq_decode_attention.argtypes = [cfgp, i32, vp, kvq_qcache, i32, kvq_residual, i32, i32, kvq_pool,
                                         vp, vp, C.c_size_t, vp]
    lib.kvq_decode_attention_static.restype = i32
    lib.kvq_decode_attention_static.argtypes = [cfgp, i32, vp, kvq_qcache, i32, kvq_residual, i32, i32, kvq_pool, vp, vp]
    lib.kvq_append_decode_attention.restype = i32
    lib.kvq_append_decode_attention.argtypes = [cfgp, i32, vp, vp, vp, kvq_qcache, i32, kvq_residual, i32, i32, kvq_pool,
                                                vp, vp, C.c_size_t, vp]
    lib.kvq_append_decode_attention_rope.restype = i32
    lib.kvq_append_decode_attention_rope.argtypes = [cfgp, i32, vp, vp, vp, vp, i64, kvq_qcache, i32, kvq_residual, i32,
                                                     i32, kvq_pool, vp, vp, C.c_size_t, vp]
    lib.kvq_rope_rotate.restype = i32
    lib.kvq_rope_rotate.argtypes = [cfgp, vp, i32, vp, i64, vp, vp]
    lib.kvq_append_trace_quantize_ragged.restype = i32
    lib.kvq_append_trace_quantize_ragged.argtypes = [cfgp, i32, vp, vp, kvq_residual, vp, kvq_pool, vp, kvq_qcache, vp]
    lib.kvq_decode_workspace_bytes.restype = i64
    lib.kvq_decode_workspace_bytes.argtypes = [cfgp, i32]
    lib.kvq_decode_launch_shape.restype = i32
    lib.kvq_decode_launch_shape.argtypes = [cfgp, i32, i32, i32] + [C.POINTER(i32)] * 3
    lib.kvq_decode_attention_multi.restype = i32
    lib.kvq_decode_attention_multi.argtypes = [cfgp, i32, vp, i32, kvq_qcache, i32, kvq_residual, i32, i32, kvq_pool,
                                               vp, vp, C.c_size_t, vp]
    lib.kvq_dequantize.restype = i32
    lib.kvq_dequantize.argtypes = [cfgp, i32, kvq_qcache, i32, kvq_pool, i32, i32, vp, vp, i64, vp]
    lib.kvq_seq_advance.restype = i32
    lib.kvq_seq_advance.argtypes = [cfgp, vp, vp]
    lib.kvq_decode_attention_ragged.restype = i32
    lib.kvq_decode_attention_ragged.argtypes = [cfgp, i32, vp, kvq_qcache, kvq_residual, vp, i32, i32, kvq_pool,
                                                vp, vp, C.c_size_t, vp]
    lib.kvq_seq_plan_bytes.restype = i64
    lib.kvq_seq_plan_bytes.argtypes = [cfgp]
    lib.kvq_seq_plan.restype = i32
    lib.kvq_seq_plan.argtypes = [cfgp, vp, i32, i32, vp, vp]
    lib.kvq_decode_attention_planned.restype = i32
    lib.kvq_decode_attention_planned.argtypes = [cfgp, i32, vp, kvq_qcache, kvq_residual, vp, i32, i32, kvq_pool,
                                                 vp, vp, C.c_size_t, vp]
    _lib = lib
    return lib


def _ptr(x):
    """Device (or null) pointer of a torch tensor / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def status_string(status: int) -> str:
    return load_library().kvq_status_string(status).decode()


def kvq_version() -> int:
    return load_library().kvq_version()


def kvq_query_sizes(cfg: kvq_config) -> kvq_sizes:
    out = kvq_sizes()
    st = load_library().kvq_query_sizes(C.byref(cfg), C.byref(out))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_query_sizes")
    return out


def kvq_append_residual(cfg, layer, k_new, v_new, res: kvq_residual, res_start, n_res, stream=None):
    st = load_library().kvq_append_residual(C.byref(cfg), layer, _ptr(k_new), _ptr(v_new), res, res_start, n_res,
                                            _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_append_residual")


def kvq_trace_outliers(cfg, layer, group_index, k_group, v_group, unit_stride, pool: kvq_pool, selected,
                       stream=None):
    st = load_library().kvq_trace_outliers(C.byref(cfg), layer, group_index, _ptr(k_group), _ptr(v_group),
                                           unit_stride, pool, _ptr(selected), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_trace_outliers")


def kvq_quantize_group(cfg, layer, group_index, k_group, v_group, unit_stride, selected, qcache: kvq_qcache,
                       stream=None):
    st = load_library().kvq_quantize_group(C.byref(cfg), layer, group_index, _ptr(k_group), _ptr(v_group),
                                           unit_stride, _ptr(selected), qcache, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_quantize_group")


def kvq_quantize_value_tokens(cfg, layer, first_token, count, v_res, ring_row, qcache: kvq_qcache, stream=None):
    st = load_library().kvq_quantize_value_tokens(C.byref(cfg), layer, first_token, count, _ptr(v_res), ring_row,
                                                  qcache, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_quantize_value_tokens")


def kvq_append_trace_quantize(cfg, layer, k_new, v_new, res: kvq_residual, res_start, n_res, n_quant, pool: kvq_pool,
                              selected, qcache: kvq_qcache, stream=None):
    st = load_library().kvq_append_trace_quantize(C.byref(cfg), layer, _ptr(k_new), _ptr(v_new), res, res_start,
                                                  n_res, n_quant, pool, _ptr(selected), qcache, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_append_trace_quantize")


def kvq_prefill_quantize(cfg, layer, k_rows, v_rows, unit_stride, n_tokens, pool: kvq_pool, selected,
                         qcache: kvq_qcache, res: kvq_residual, stream=None):
    st = load_library().kvq_prefill_quantize(C.byref(cfg), layer, _ptr(k_rows), _ptr(v_rows), unit_stride, n_tokens,
                                             pool, _ptr(selected), qcache, res, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_prefill_quantize")


def kvq_prefill_quantize_seq(cfg, layer, seq, k_rows, v_rows, unit_stride, n_tokens, pool: kvq_pool, selected,
                             qcache: kvq_qcache, res: kvq_residual, stream=None):
    st = load_library().kvq_prefill_quantize_seq(C.byref(cfg), layer, seq, _ptr(k_rows), _ptr(v_rows), unit_stride,
                                                 n_tokens, pool, _ptr(selected), qcache, res, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_prefill_quantize_seq")


def kvq_decode_workspace_bytes(cfg, q_tokens) -> int:
    n = load_library().kvq_decode_workspace_bytes(C.byref(cfg), q_tokens)
    if n < 0:
        raise KvqError(int(n), "kvq_decode_workspace_bytes")
    return int(n)


def kvq_decode_attention_static(cfg, layer, q, qcache: kvq_qcache, n_quant, res: kvq_residual, res_start, n_res,
                                pool: kvq_pool, out, stream=None):
    st = load_library().kvq_decode_attention_static(C.byref(cfg), layer, _ptr(q), qcache, n_quant, res, res_start,
                                                    n_res, pool, _ptr(out), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_attention_static")


def kvq_decode_launch_shape(cfg, q_tokens, n_quant, fp_rows):
    """(splits, waves, minichunks_per_split) of the decode launch for this state."""
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    st = load_library().kvq_decode_launch_shape(C.byref(cfg), q_tokens, n_quant, fp_rows, C.byref(a), C.byref(b),
                                                C.byref(c))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_launch_shape")
    return a.value, b.value, c.value


def kvq_decode_attention_multi(cfg, layer, q, q_tokens, qcache: kvq_qcache, n_quant, res: kvq_residual, res_start,
                               n_res, pool: kvq_pool, out, workspace, workspace_bytes, stream=None):
    st = load_library().kvq_decode_attention_multi(C.byref(cfg), layer, _ptr(q), q_tokens, qcache, n_quant, res,
                                                   res_start, n_res, pool, _ptr(out), _ptr(workspace),
                                                   workspace_bytes, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_attention_multi")


def kvq_dequantize(cfg, layer, qcache: kvq_qcache, n_quant, pool: kvq_pool, t0, n, k_out, v_out, out_unit_stride,
                   stream=None):
    st = load_library().kvq_dequantize(C.byref(cfg), layer, qcache, n_quant, pool, t0, n, _ptr(k_out), _ptr(v_out),
                                       out_unit_stride, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_dequantize")


def kvq_append_decode_attention(cfg, layer, q, k_new, v_new, qcache: kvq_qcache, n_quant, res: kvq_residual, res_start,
                                n_res, pool: kvq_pool, out, workspace, workspace_bytes, stream=None):
    st = load_library().kvq_append_decode_attention(C.byref(cfg), layer, _ptr(q), _ptr(k_new), _ptr(v_new), qcache,
                                                    n_quant, res, res_start, n_res, pool, _ptr(out), _ptr(workspace),
                                                    workspace_bytes, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_append_decode_attention")


def kvq_append_decode_attention_rope(cfg, layer, q, k_new, v_new, rope, rope_stride, qcache: kvq_qcache, n_quant,
                                     res: kvq_residual, res_start, n_res, pool: kvq_pool, out, workspace,
                                     workspace_bytes, stream=None):
    st = load_library().kvq_append_decode_attention_rope(C.byref(cfg), layer, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                         _ptr(rope), rope_stride, qcache, n_quant, res, res_start,
                                                         n_res, pool, _ptr(out), _ptr(workspace), workspace_bytes,
                                                         _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_append_decode_attention_rope")


def kvq_rope_rotate(cfg, x, heads, rope, rope_stride, out, stream=None):
    st = load_library().kvq_rope_rotate(C.byref(cfg), _ptr(x), heads, _ptr(rope), rope_stride, _ptr(out),
                                        _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_rope_rotate")


def kvq_append_trace_quantize_ragged(cfg, layer, k_new, v_new, res: kvq_residual, seq_state, pool: kvq_pool, selected,
                                     qcache: kvq_qcache, stream=None):
    st = load_library().kvq_append_trace_quantize_ragged(C.byref(cfg), layer, _ptr(k_new), _ptr(v_new), res,
                                                         _ptr(seq_state), pool, _ptr(selected), qcache,
                                                         _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_append_trace_quantize_ragged")


def kvq_seq_advance(cfg, seq_state, stream=None):
    st = load_library().kvq_seq_advance(C.byref(cfg), _ptr(seq_state), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_seq_advance")


def kvq_decode_attention_ragged(cfg, layer, q, qcache: kvq_qcache, res: kvq_residual, seq_state, max_n_quant,
                                max_n_res, pool: kvq_pool, out, workspace, workspace_bytes, stream=None):
    st = load_library().kvq_decode_attention_ragged(C.byref(cfg), layer, _ptr(q), qcache, res, _ptr(seq_state),
                                                    max_n_quant, max_n_res, pool, _ptr(out), _ptr(workspace),
                                                    workspace_bytes, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_attention_ragged")


def kvq_seq_plan_bytes(cfg) -> int:
    n = load_library().kvq_seq_plan_bytes(C.byref(cfg))
    if n < 0:
        raise KvqError(int(n), "kvq_seq_plan_bytes")
    return int(n)


def kvq_seq_plan(cfg, seq_state, max_n_quant, max_n_res, plan, stream=None):
    st = load_library().kvq_seq_plan(C.byref(cfg), _ptr(seq_state), max_n_quant, max_n_res, _ptr(plan), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_seq_plan")


def kvq_decode_attention_planned(cfg, layer, q, qcache: kvq_qcache, res: kvq_residual, plan, max_n_quant, max_n_res,
                                 pool: kvq_pool, out, workspace, workspace_bytes, stream=None):
    st = load_library().kvq_decode_attention_planned(C.byref(cfg), layer, _ptr(q), qcache, res, _ptr(plan),
                                                     max_n_quant, max_n_res, pool, _ptr(out), _ptr(workspace),
                                                     workspace_bytes, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_attention_planned")


def kvq_stream_read(buf, nbytes, sink, stream=None):
    st = load_library().kvq_stream_read(_ptr(buf), nbytes, _ptr(sink), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_stream_read")


def kvq_decode_attention(cfg, layer, q, qcache: kvq_qcache, n_quant, res: kvq_residual, res_start, n_res,
                         pool: kvq_pool, out, workspace, workspace_bytes, stream=None):
    st = load_library().kvq_decode_attention(C.byref(cfg), layer, _ptr(q), qcache, n_quant, res, res_start, n_res,
                                             pool, _ptr(out), _ptr(workspace), workspace_bytes, _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_attention")
