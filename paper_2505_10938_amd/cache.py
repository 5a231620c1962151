"""Device buffers of one KV cache and the host-side schedule that drives the library.

Allocation (torch tensors as raw device memory) and the "quantize every G steps"
schedule (Method, "Quantization") live here; every computation is a call into
libkvq.so through `binding`.
"""
from __future__ import annotations

import torch

from . import binding as B


def make_config(layers, batch, q_heads, kv_heads, max_seq, bits=2, group_k=32, group_v=32, residual=128,
                outlier_budget=8, aux_capacity=32, head_dim=128, untraced_layers=0, value_per_step=0) -> B.kvq_config:
    return B.kvq_config(layers, batch, q_heads, kv_heads, head_dim, max_seq, bits, group_k, group_v, residual,
                        outlier_budget, aux_capacity, untraced_layers, value_per_step)


class KVCache:
    """All caller-owned buffers of kvq for one configuration, on one device.

    With `n_pages` the quantized arrays are a pool of that many pages (one Key group of one
    sequence each, for all layers and kv heads) and `page_table` (int32 [batch, max_seq / G], device)
    says which page holds which group of which sequence; the caller fills it before the group is
    quantized."""

    def __init__(self, cfg: B.kvq_config, device="cuda:0", n_pages=None):
        self.cfg = cfg
        self.sizes = sz = B.kvq_query_sizes(cfg)
        dev = torch.device(device)
        self.device = dev
        self.n_pages = n_pages
        self.page_table = None

        def raw(nbytes):
            return torch.zeros(max(int(nbytes), 16), dtype=torch.uint8, device=dev)

        qsz = sz
        if n_pages is not None:      # the pool is laid out as the dense cache of one sequence of n_pages groups
            qsz = B.kvq_query_sizes(make_config(cfg.layers, 1, cfg.kv_heads, cfg.kv_heads, n_pages * cfg.group_k,
                                                cfg.bits, cfg.group_k, cfg.group_v, cfg.residual, cfg.outlier_budget,
                                                cfg.aux_capacity, cfg.head_dim, 0, cfg.value_per_step))
            self.page_table = torch.zeros(cfg.batch, cfg.max_seq // cfg.group_k, dtype=torch.int32, device=dev)
        self.k_codes, self.k_meta = raw(qsz.k_codes_bytes), raw(qsz.k_meta_bytes)
        self.v_codes, self.v_meta = raw(qsz.v_codes_bytes), raw(qsz.v_meta_bytes)
        self.mask = raw(qsz.mask_bytes)
        self.k_res, self.v_res = raw(sz.res_bytes), raw(sz.res_bytes)
        self.pool_k, self.pool_v = raw(sz.pool_rows_bytes), raw(sz.pool_rows_bytes)
        self.pool_idx, self.pool_score = raw(sz.pool_idx_bytes), raw(sz.pool_score_bytes)
        self.pool_count, self.aux_count, self.frozen = (raw(sz.counter_bytes) for _ in range(3))
        self.selected = raw(sz.selected_bytes)
        self.workspace = raw(sz.workspace_bytes)
        self._bind()
        # per-layer schedule state (uniform over the batch)
        self.n_quant = [0] * cfg.layers
        self.res_start = [0] * cfg.layers
        self.n_res = [0] * cfg.layers

    def _bind(self):
        """The structures the library takes, from the tensors."""
        ptrs = [t.data_ptr() for t in (self.k_codes, self.k_meta, self.v_codes, self.v_meta, self.mask)]
        if self.page_table is None:
            self.qcache = B.kvq_qcache(*ptrs)
        else:
            self.qcache = B.kvq_qcache(*ptrs, self.page_table.data_ptr(), self.page_table.shape[1], self.n_pages)
        self.pool = B.kvq_pool(*(t.data_ptr() for t in (self.pool_k, self.pool_v, self.pool_idx, self.pool_score,
                                                        self.pool_count, self.aux_count, self.frozen)))
        self.res = B.kvq_residual(self.k_res.data_ptr(), self.v_res.data_ptr())

    # ---- views for tests / loaders -------------------------------------------------------------
    def dense_quantized(self):
        """The five quantized arrays in the dense layout [units, ...] (uint8 tensors): the arrays
        themselves, or, for a paged cache, its pages gathered through the table."""
        arrays = (self.k_codes, self.k_meta, self.v_codes, self.v_meta, self.mask)
        if self.page_table is None:
            return arrays
        c = self.cfg
        table = self.page_table.long().clamp(0, self.n_pages - 1)
        out = []
        for t in arrays:
            per_page = t.numel() // (c.layers * c.kv_heads * self.n_pages)
            pages = t[:c.layers * c.kv_heads * self.n_pages * per_page].view(c.layers, c.kv_heads, self.n_pages, per_page)
            out.append(pages[:, :, table].permute(0, 2, 1, 3, 4).reshape(-1))   # [layers, batch, kv_heads, groups, bytes]
        return tuple(out)

    @property
    def units_per_layer(self):
        return self.cfg.batch * self.cfg.kv_heads

    def res_view(self, which="k"):
        t = self.k_res if which == "k" else self.v_res
        return t.view(torch.float16).view(self.sizes.units, self.sizes.res_rows, self.cfg.head_dim)

    def _group_ptrs(self, layer, row0):
        hd = self.cfg.head_dim
        unit0 = layer * self.units_per_layer
        off = (unit0 * self.sizes.res_rows + row0) * hd * 2
        return self.k_res.data_ptr() + off, self.v_res.data_ptr() + off, self.sizes.res_rows * hd

    # ---- the schedule --------------------------------------------------------------------------------
    def _value_leaves_window(self, layer, stream=None):
        """The per-step Value schedule (cfg.value_per_step; Experiments, "Details": Values compressed at
        each step): ahead of a step's append, the Values of the token that the append pushes out of the
        window of the R most recent tokens are quantized."""
        cfg = self.cfg
        if not cfg.value_per_step:
            return
        tok = self.n_quant[layer] + self.n_res[layer] - cfg.residual
        if tok < 0:
            return
        row = (self.res_start[layer] + tok - self.n_quant[layer]) % self.sizes.res_rows
        B.kvq_quantize_value_tokens(cfg, layer, tok, 1, self.v_res, row, self.qcache, stream)

    def append(self, layer, k_new, v_new, stream=None, trace=True, fused=True):
        """Append one token (fp16 [batch, kv_heads, head_dim] each); when the ring then holds R + G
        tokens, trace and quantize the oldest G (in the same launch if `fused`, else with the three
        separate calls).  Returns True if a group was quantized."""
        cfg = self.cfg
        G = cfg.group_k
        self._value_leaves_window(layer, stream)
        fills = self.n_res[layer] + 1 == cfg.residual + G
        if fills and fused and trace:
            B.kvq_append_trace_quantize(cfg, layer, k_new, v_new, self.res, self.res_start[layer], self.n_res[layer],
                                        self.n_quant[layer], self.pool, self.selected, self.qcache, stream)
            self.n_quant[layer] += G
            self.n_res[layer] += 1 - G
            self.res_start[layer] = (self.res_start[layer] + G) % self.sizes.res_rows
            return True
        B.kvq_append_residual(cfg, layer, k_new, v_new, self.res, self.res_start[layer], self.n_res[layer], stream)
        self.n_res[layer] += 1
        if fills:
            self.quantize_oldest(layer, stream, trace)
            return True
        return False

    def quantize_oldest(self, layer, stream=None, trace=True):
        cfg = self.cfg
        G = cfg.group_k
        assert self.n_res[layer] >= G and self.n_quant[layer] + G <= cfg.max_seq
        gi = self.n_quant[layer] // G
        kp, vp, stride = self._group_ptrs(layer, self.res_start[layer])
        sel = None
        if trace and cfg.outlier_budget > 0:
            B.kvq_trace_outliers(cfg, layer, gi, kp, vp, stride, self.pool, self.selected, stream)
            sel = self.selected
        B.kvq_quantize_group(cfg, layer, gi, kp, vp, stride, sel, self.qcache, stream)
        self.n_quant[layer] += G
        self.n_res[layer] -= G
        self.res_start[layer] = (self.res_start[layer] + G) % self.sizes.res_rows

    def load_residual(self, layer, k_rows, v_rows):
        """Bulk-load rows (fp16 [batch, kv_heads, n, head_dim]) into an empty ring (test / benchmark
        set-up: a plain device copy, equivalent to n appends)."""
        n = k_rows.shape[2]
        rows = self.sizes.res_rows
        assert self.n_res[layer] == 0 and n <= rows
        u0, u1 = layer * self.units_per_layer, (layer + 1) * self.units_per_layer
        s = self.res_start[layer]
        first = min(n, rows - s)                      # the ring may wrap
        for view, src in ((self.res_view("k"), k_rows), (self.res_view("v"), v_rows)):
            src = src.reshape(-1, n, self.cfg.head_dim)
            view[u0:u1, s:s + first] = src[:, :first]
            if first < n:
                view[u0:u1, 0:n - first] = src[:, first:]
        self.n_res[layer] = n

    def prefill(self, layer, k_rows, v_rows, stream=None):
        """Quantize a whole prompt (fp16 [batch, kv_heads, n, head_dim], contiguous) into the empty cache
        of `layer`: the state that n appends would leave."""
        cfg = self.cfg
        n = k_rows.shape[2]
        assert self.n_quant[layer] == 0 and self.n_res[layer] == 0 and k_rows.is_contiguous() and v_rows.is_contiguous()
        if getattr(self, "prefill_selected", None) is None:
            self.prefill_selected = torch.zeros(max(int(self.sizes.prefill_selected_bytes), 16), dtype=torch.uint8,
                                                device=self.device)
        B.kvq_prefill_quantize(cfg, layer, k_rows, v_rows, n * cfg.head_dim, n, self.pool, self.prefill_selected,
                               self.qcache, self.res, stream)
        G, R = cfg.group_k, cfg.residual
        nq = G * ((n - R) // G) if n >= R + G else 0
        self.n_quant[layer], self.n_res[layer], self.res_start[layer] = nq, n - nq, 0

    def decode(self, layer, q, out=None, stream=None):
        """Attention output (fp16 [batch, q_heads, head_dim]) of one decode step."""
        if out is None:
            out = torch.empty_like(q)
        B.kvq_decode_attention(self.cfg, layer, q, self.qcache, self.n_quant[layer], self.res,
                               self.res_start[layer], self.n_res[layer], self.pool, out, self.workspace,
                               self.workspace.numel(), stream)
        return out

    def decode_multi(self, layer, q, out=None, stream=None):
        """Attention outputs of the q.shape[1] newest tokens at once (q: fp16 [batch, tokens, q_heads,
        head_dim]; their Keys and Values are in the cache already), each attending up to itself."""
        if out is None:
            out = torch.empty_like(q)
        tokens = q.shape[1]
        need = B.kvq_decode_workspace_bytes(self.cfg, tokens)
        if self.workspace.numel() < need:
            self.workspace = torch.zeros(need, dtype=torch.uint8, device=self.device)
        B.kvq_decode_attention_multi(self.cfg, layer, q, tokens, self.qcache, self.n_quant[layer], self.res,
                                     self.res_start[layer], self.n_res[layer], self.pool, out, self.workspace,
                                     self.workspace.numel(), stream)
        return out

    def step(self, layer, k_new, v_new, q, out=None, stream=None, rope=None, rope_stride=0):
        """One decode step of `layer`: the new token joins the cache and the attention output (fp16
        [batch, q_heads, head_dim]) over the cache including it is returned.  Two launches on the steps
        on which the ring fills (group step, then attention), one on all others; under the per-step
        Value schedule one more, ahead of them (the Values of the token that leaves the window).
        `rope` (fp32 device tensor: the head_dim/2 cosines, then the sines, of the new token's position;
        per sequence if rope_stride > 0): q and k_new are given unrotated and the library rotates them,
        inside the decode launch where there is one launch, with two small launches where the ring fills."""
        if out is None:
            out = torch.empty_like(q)
        if self.n_res[layer] + 1 == self.cfg.residual + self.cfg.group_k:
            if rope is not None:
                k_rot, q_rot = torch.empty_like(k_new), torch.empty_like(q)
                B.kvq_rope_rotate(self.cfg, k_new, self.cfg.kv_heads, rope, rope_stride, k_rot, stream)
                B.kvq_rope_rotate(self.cfg, q, self.cfg.q_heads, rope, rope_stride, q_rot, stream)
                k_new, q = k_rot, q_rot
            self.append(layer, k_new, v_new, stream)
            return self.decode(layer, q, out, stream)
        self._value_leaves_window(layer, stream)
        if rope is not None:
            B.kvq_append_decode_attention_rope(self.cfg, layer, q, k_new, v_new, rope, rope_stride, self.qcache,
                                               self.n_quant[layer], self.res, self.res_start[layer],
                                               self.n_res[layer], self.pool, out, self.workspace,
                                               self.workspace.numel(), stream)
        else:
            B.kvq_append_decode_attention(self.cfg, layer, q, k_new, v_new, self.qcache, self.n_quant[layer],
                                          self.res, self.res_start[layer], self.n_res[layer], self.pool, out,
                                          self.workspace, self.workspace.numel(), stream)
        self.n_res[layer] += 1
        return out

    def clone(self):
        """A second cache with the same contents in its own device memory."""
        other = KVCache.__new__(KVCache)
        other.cfg, other.sizes, other.device, other.n_pages = self.cfg, self.sizes, self.device, self.n_pages
        names = ("k_codes", "k_meta", "v_codes", "v_meta", "mask", "k_res", "v_res", "pool_k", "pool_v",
                 "pool_idx", "pool_score", "pool_count", "aux_count", "frozen", "selected", "workspace")
        for n in names:
            setattr(other, n, getattr(self, n).clone())
        other.page_table = None if self.page_table is None else self.page_table.clone()
        other._bind()
        other.n_quant, other.res_start, other.n_res = list(self.n_quant), list(self.res_start), list(self.n_res)
        other.prefill_selected = None
        return other


class RaggedKVCache(KVCache):
    """A cache whose sequences differ in length.  The per-sequence state {n_quant, res_start,
    n_res, active} is a device array that the library reads and advances; the host keeps only
    an upper bound of the longest sequence, which sizes the decode launch."""

    def __init__(self, cfg: B.kvq_config, device="cuda:0", n_pages=None):
        super().__init__(cfg, device, n_pages)
        self.seq_state = torch.zeros(cfg.batch, 4, dtype=torch.int32, device=self.device)
        self.longest = 0                                  # tokens of the longest sequence, at most

    def set_active(self, active):
        """active: bool / int tensor or list [batch]: the sequences that take part in the next steps."""
        self.seq_state[:, 3] = torch.as_tensor(active, device=self.device).to(torch.int32)

    def append(self, layer, k_new, v_new, stream=None):
        """One token per active sequence (fp16 [batch, kv_heads, head_dim] each; rows of inactive
        sequences are ignored) into `layer`; sequences whose ring fills have their oldest group
        traced and quantized in the same launch.  Call for every layer, then advance()."""
        B.kvq_append_trace_quantize_ragged(self.cfg, layer, k_new, v_new, self.res, self.seq_state, self.pool, None,
                                           self.qcache, stream)

    def prefill_sequence(self, b, k_rows, v_rows, active=True, stream=None):
        """A new sequence in slot `b`: its prompt (per layer: fp16 [kv_heads, n, head_dim], contiguous;
        `k_rows`, `v_rows` are lists over the layers) quantized in one call per layer, whatever the slot
        held before; the other sequences are not touched."""
        cfg = self.cfg
        n = k_rows[0].shape[1]
        G, R = cfg.group_k, cfg.residual
        nq = G * ((n - R) // G) if n >= R + G else 0
        if getattr(self, "prefill_selected", None) is None:
            self.prefill_selected = torch.zeros(max(int(self.sizes.prefill_selected_bytes), 16), dtype=torch.uint8,
                                                device=self.device)
        for layer in range(cfg.layers):
            k, v = k_rows[layer], v_rows[layer]
            assert k.shape == (cfg.kv_heads, n, cfg.head_dim) and k.is_contiguous() and v.is_contiguous()
            B.kvq_prefill_quantize_seq(cfg, layer, b, k, v, n * cfg.head_dim, n, self.pool, self.prefill_selected,
                                       self.qcache, self.res, stream)
        state = torch.tensor([nq, 0, n - nq, 1 if active else 0], dtype=torch.int32)
        self.seq_state[b].copy_(state.to(self.device), non_blocking=False)
        self.longest = max(self.longest, n)

    def advance(self, stream=None):
        """The sequences' states after the token just appended to every layer."""
        B.kvq_seq_advance(self.cfg, self.seq_state, stream)
        self.longest += 1

    def make_plan(self, stream=None):
        """Deal the decode launches of the next step by the sequences' current lengths (once per step,
        after advance(); then decode(..., planned=True) for every layer)."""
        if getattr(self, "plan", None) is None:
            self.plan = torch.zeros(B.kvq_seq_plan_bytes(self.cfg) // 4, dtype=torch.int32, device=self.device)
        nq, nr = self.bounds()
        B.kvq_seq_plan(self.cfg, self.seq_state, nq, nr, self.plan, stream)

    def bounds(self):
        """(max_n_quant, max_n_res) over all sequences, from the host's bound of the longest one."""
        G, R = self.cfg.group_k, self.cfg.residual
        n = self.longest
        nq = G * ((n - R) // G) if n >= R + G else 0
        return min(nq, self.cfg.max_seq), min(n, R + G - 1)

    def decode(self, layer, q, out=None, stream=None, planned=False):
        if out is None:
            out = torch.empty_like(q)
        nq, nr = self.bounds()
        if planned:
            B.kvq_decode_attention_planned(self.cfg, layer, q, self.qcache, self.res, self.plan, nq, nr, self.pool, out,
                                           self.workspace, self.workspace.numel(), stream)
            return out
        B.kvq_decode_attention_ragged(self.cfg, layer, q, self.qcache, self.res, self.seq_state, nq, nr, self.pool, out,
                                      self.workspace, self.workspace.numel(), stream)
        return out
