"""MI355X-native low-bit KV-cache decode attention with outlier-token tracing.

The computation lives in libkvq.so (HIP, gfx950; sources under csrc/); this
package is its Python binding.
"""
from . import binding
from .binding import (KvqError, kvq_append_decode_attention, kvq_append_residual, kvq_append_trace_quantize,
                      kvq_append_trace_quantize_ragged,
                      kvq_config, kvq_decode_attention, kvq_decode_attention_ragged, kvq_decode_attention_multi, kvq_decode_attention_static, kvq_decode_launch_shape,
                      kvq_decode_workspace_bytes, kvq_dequantize, kvq_pool, kvq_prefill_quantize,
                      kvq_qcache, kvq_seq_advance, kvq_prefill_quantize_seq,
                      kvq_quantize_group, kvq_query_sizes, kvq_residual, kvq_sizes, kvq_stream_read,
                      kvq_trace_outliers, kvq_version, load_library, status_string)

__all__ = ["binding", "KvqError", "kvq_append_decode_attention", "kvq_append_residual", "kvq_append_trace_quantize",
           "kvq_append_trace_quantize_ragged", "kvq_config", "kvq_decode_attention", "kvq_decode_attention_ragged", "kvq_decode_attention_multi", "kvq_decode_attention_static", "kvq_decode_launch_shape",
           "kvq_decode_workspace_bytes", "kvq_dequantize",
           "kvq_pool", "kvq_prefill_quantize", "kvq_prefill_quantize_seq", "kvq_seq_advance",
           "kvq_qcache", "kvq_quantize_group", "kvq_query_sizes", "kvq_residual", "kvq_sizes",
           "kvq_stream_read", "kvq_trace_outliers", "kvq_version", "load_library", "status_string"]
