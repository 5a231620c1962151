// Host side of the C ABI: argument validation, buffer sizes, launches.
#include "kvq_common.h"

#include <mutex>

namespace {

using kvq::Dims;

int32_t check_config(const kvq_config* c) {
  if (!c) return KVQ_ERR_INVALID_ARG;
  if (c->layers < 1 || c->batch < 1 || c->kv_heads < 1 || c->q_heads < 1) return KVQ_ERR_INVALID_ARG;
  if (c->q_heads % c->kv_heads != 0) return KVQ_ERR_INVALID_ARG;
  if (c->bits != 2 && c->bits != 4) return KVQ_ERR_INVALID_ARG;
  if (c->group_k != 32 && c->group_k != 64 && c->group_k != 128) return KVQ_ERR_INVALID_ARG;
  if (c->head_dim < 32 || c->head_dim % 32 != 0) return KVQ_ERR_INVALID_ARG;
  if (c->group_v != 32 && c->group_v != 64 && c->group_v != 128) return KVQ_ERR_INVALID_ARG;
  if (c->head_dim % c->group_v != 0) return KVQ_ERR_INVALID_ARG;
  if (c->max_seq < c->group_k || c->max_seq % c->group_k != 0) return KVQ_ERR_INVALID_ARG;
  if (c->residual < 0 || c->outlier_budget < 0 || c->aux_capacity < 0) return KVQ_ERR_INVALID_ARG;
  if (c->untraced_layers < 0 || c->untraced_layers > c->layers) return KVQ_ERR_INVALID_ARG;
  if (c->residual > (1 << 20) || c->max_seq > (1 << 24)) return KVQ_ERR_INVALID_ARG;
  if (c->batch > 65535 || c->kv_heads > 32767) return KVQ_ERR_INVALID_ARG;   // grid y/z limits
  if (c->head_dim != kvq::kHeadDim) return KVQ_ERR_UNSUPPORTED;
  const int g = c->q_heads / c->kv_heads;
  if (g != 1 && g != 2 && g != 4 && g != 8) return KVQ_ERR_UNSUPPORTED;
  if (c->outlier_budget > 64 || c->aux_capacity > 64) return KVQ_ERR_UNSUPPORTED;
  if (c->value_per_step != 0 && c->value_per_step != 1) return KVQ_ERR_INVALID_ARG;
  // the per-step Value schedule is the one of the method without tracing; a token must be in the ring
  // when it leaves the window
  if (c->value_per_step && (c->outlier_budget != 0 || c->residual < 1)) return KVQ_ERR_UNSUPPORTED;
  return KVQ_OK;
}

int64_t res_rows_of(const kvq_config* c) {
  const int64_t G = c->group_k;
  return G * ((c->residual + G + G - 1) / G);
}

// Split of one unit's decode work over wavefronts and workgroups.  Quantized tokens go in
// mini-chunks of 128 (one wavefront each at a time), full-precision rows in groups of 16 that cost
// about half a mini-chunk.  As many wavefronts are wanted over the whole launch as fit on the chip
// at once (2 per SIMD by registers, fewer if a wavefront's LDS were larger), no more per unit than
// it has items; they form as few workgroups as fit (one workgroup per unit needs no exchange
// through memory).
struct Split {
  int32_t splits, nw, mc_per_split;
};
Split decode_split(int64_t units_per_layer, int g, int vgroups, int64_t n_quant, int64_t fp_rows) {
  Split s;
  const int64_t mc = (n_quant + kvq::kMiniChunk - 1) / kvq::kMiniChunk;
  const int64_t rg = (fp_rows + kvq::kFpGroupRows - 1) / kvq::kFpGroupRows;
  int64_t items = mc + (rg + 1) / 2;
  if (items < 1) items = 1;
  int64_t waves_per_cu = kvq::kLdsPerComputeUnit / kvq::decode_wave_lds_bytes(g, vgroups);
  const int64_t by_registers = 4 * kvq::kDecodeWavesPerSimd;
  if (waves_per_cu > by_registers) waves_per_cu = by_registers;
  if (waves_per_cu < 1) waves_per_cu = 1;
  int64_t wpu = kvq::kComputeUnits * waves_per_cu / units_per_layer;
  if (wpu > items) wpu = items;
  if (wpu < 1) wpu = 1;
  s.splits = (int32_t)((wpu + waves_per_cu - 1) / waves_per_cu);
  s.nw = (int32_t)((wpu + s.splits - 1) / s.splits);
  s.mc_per_split = (int32_t)((mc + s.splits - 1) / s.splits);
  return s;
}
constexpr int64_t kCounterBytes(int64_t upl) { return ((upl * 4 + 255) / 256) * 256; }

// Shape of a planned decode launch (sequences of different lengths dealt by length): wavefronts per
// workgroup and workgroups ("entries") per kv head.  All workgroups are to be resident at once, and there
// should be at least twice as many per kv head as sequences, so that a long sequence can have several
// while a short one has one: the workgroups are made smaller until that holds.  (Measured on 32 sequences
// of 128 .. 8192 tokens with 8 kv heads: 41.4 us with as many workgroups as sequences, 36.7 with twice,
// 36.8 with four times, 46.2 with eight times as many; sharing a large workgroup between several short
// sequences, one after the other, 61.8 us: every sequence then waits for its own first loads.)
// entries == 0: no such shape (more sequences than workgroups fit per kv head, or more than 1024).
struct PlanShape {
  int32_t nw, entries;
};
PlanShape plan_shape(const kvq_config* c) {
  const int g = c->q_heads / c->kv_heads;
  int64_t waves_per_cu = kvq::kLdsPerComputeUnit / kvq::decode_wave_lds_bytes(g, c->head_dim / c->group_v);
  const int64_t by_registers = 4 * kvq::kDecodeWavesPerSimd;
  if (waves_per_cu > by_registers) waves_per_cu = by_registers;
  if (waves_per_cu < 1) waves_per_cu = 1;
  PlanShape best = {0, 0};
  if (c->batch > 1024) return best;
  for (int nw = (int)waves_per_cu; nw >= 1; nw >>= 1) {
    const int64_t entries = kvq::kComputeUnits * (waves_per_cu / nw) / c->kv_heads;
    if (entries < c->batch) continue;
    best.nw = nw;
    best.entries = (int32_t)(entries > 4096 ? 4096 : entries);
    if (entries >= 2 * (int64_t)c->batch) break;
  }
  return best;
}
constexpr int64_t kPlanEntryWords = 8;
// Workgroup rows that share the query rows of a kv head.  Every supported count (1, 2, 4, 8) has a kernel
// instance of its own, so it is 1; the kernel still takes any divisor (a count without an instance would
// run as several rows of a smaller one, all reading the unit's cache).
constexpr int head_parts_of(int rows, int bits) { return (void)rows, (void)bits, 1; }

// Workspace of a decode launch whose kv heads have `rows` query rows each (rows = query heads per kv
// head times query tokens): arrival counters, then partial results for the largest split the launch
// shape can get.
int64_t decode_workspace_bytes(const kvq_config* cfg, int64_t rows) {
  const int64_t upl = (int64_t)cfg->batch * cfg->kv_heads, hd = cfg->head_dim;
  const int64_t hp = head_parts_of((int)rows, cfg->bits);
  const int64_t slots = (int64_t)cfg->outlier_budget + cfg->aux_capacity;
  const int64_t s_max =
      decode_split(upl * hp, (int)(rows / hp), (int)(hd / cfg->group_v), cfg->max_seq, res_rows_of(cfg) + slots).splits;
  int64_t slots_needed = upl * s_max;
  if (cfg->batch <= 1024) {                              // a planned launch: items per kv head
    const int64_t planned = (int64_t)plan_shape(cfg).entries * cfg->kv_heads;
    if (planned > slots_needed) slots_needed = planned;
  }
  return kCounterBytes(upl * hp) + slots_needed * rows * (hd + 2) * 4;
}


Dims make_dims(const kvq_config* c, int32_t layer) {
  Dims d;
  d.batch = c->batch;
  d.q_heads = c->q_heads;
  d.kv_heads = c->kv_heads;
  d.g = c->q_heads / c->kv_heads;
  d.bits = c->bits;
  d.G = c->group_k;
  d.Gv = c->group_v;
  // slots [0, outlier_budget) stay the outlier pool's in every layer (one layout for all buffers); a
  // layer that traces nothing has budget 0: no competition, and its pool never has a member
  d.N = layer < c->untraced_layers ? 0 : c->outlier_budget;
  d.A = c->aux_capacity;
  d.max_seq = c->max_seq;
  d.res_rows = (int32_t)res_rows_of(c);
  d.R = c->residual;
  d.pool_slots = c->outlier_budget + c->aux_capacity;
  d.units_per_layer = c->batch * c->kv_heads;
  d.unit0 = (int64_t)layer * d.units_per_layer;
  d.block_bytes = 512 * c->bits;
  d.blocks_per_unit = c->max_seq / kvq::kBlockTokens;
  d.groups_per_unit = c->max_seq / c->group_k;
  d.vgroups = c->head_dim / c->group_v;
  d.bpg_shift = c->group_k == 32 ? 0 : (c->group_k == 64 ? 1 : 2);
  d.page_table = nullptr;
  d.table_stride = 0;
  d.n_pages = 0;
  d.plane0 = (int64_t)layer * c->kv_heads;
  d.seq0 = 0;
  d.keys_only = c->value_per_step;
  return d;
}

// The five arrays and, for a paged cache, its table's shape.
bool qcache_ok(const kvq_config* c, const kvq_qcache& qc) {
  if (!qc.k_codes || !qc.k_meta || !qc.v_codes || !qc.v_meta || !qc.mask) return false;
  if (!qc.page_table) return true;
  // the kernels address the blocks of a plane with 32-bit byte offsets: a plane's codes stay below 4 GiB
  const int64_t plane_code_bytes = (int64_t)qc.n_pages * (c->group_k / 32) * 512 * c->bits;
  return qc.n_pages > 0 && qc.n_pages <= (1 << 20) && plane_code_bytes < (1ll << 32) &&
         qc.table_stride >= c->max_seq / c->group_k && (((uintptr_t)qc.page_table) & 3) == 0;
}
// Dims of a launch that reads or writes the quantized cache `qc`.
Dims make_dims(const kvq_config* c, int32_t layer, const kvq_qcache& qc) {
  Dims d = make_dims(c, layer);
  if (qc.page_table) {
    d.page_table = qc.page_table;
    d.table_stride = qc.table_stride;
    d.n_pages = qc.n_pages;
    d.groups_per_unit = qc.n_pages;
    d.blocks_per_unit = qc.n_pages << d.bpg_shift;
  }
  return d;
}

int32_t from_hip(hipError_t e) { return e == hipSuccess ? KVQ_OK : KVQ_ERR_LAUNCH; }

// Plain streaming read: a workgroup reads contiguous runs of 32 KB (8 loads of 16 bytes per thread in
// flight), the runs dealt round-robin to the workgroups.
constexpr int kReadUnroll = 8;
__global__ void __launch_bounds__(256) stream_read_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
  const size_t run = 256 * kReadUnroll;               // 16-byte words per workgroup step
  uint32_t acc = 0;
  size_t base = (size_t)blockIdx.x * run;
  for (; base + run <= n16; base += (size_t)gridDim.x * run) {
    uint4 v[kReadUnroll];
#pragma unroll
    for (int k = 0; k < kReadUnroll; ++k) {             // non-temporal: the data is read once
      typedef uint32_t u4v __attribute__((ext_vector_type(4)));
      const u4v t = __builtin_nontemporal_load((const u4v*)(p + base + k * 256 + threadIdx.x));
      v[k] = make_uint4(t.x, t.y, t.z, t.w);
    }
#pragma unroll
    for (int k = 0; k < kReadUnroll; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  for (size_t i = base + threadIdx.x; i < n16 && base < n16; i += 256) {   // the last, partial run
    if (i >= base + run) break;
    const uint4 a = p[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;      // keeps the loads alive; practically never taken
}

}  // namespace

extern "C" {

int32_t kvq_version(void) { return 6; }

int32_t kvq_stream_read(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)buf & 15) != 0) return KVQ_ERR_INVALID_ARG;
  hipLaunchKernelGGL(stream_read_kernel, dim3(kvq::kComputeUnits * 8), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)buf, bytes / 16, (uint32_t*)sink);
  return from_hip(hipGetLastError());
}

const char* kvq_status_string(int32_t status) {
  switch (status) {
    case KVQ_OK: return "ok";
    case KVQ_ERR_INVALID_ARG: return "invalid argument";
    case KVQ_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case KVQ_ERR_WORKSPACE: return "workspace too small";
    case KVQ_ERR_LAUNCH: return "HIP launch failed";
    case KVQ_ERR_SCRATCH: return "problem too large for the library's static scratch buffer";
    default: return "unknown status";
  }
}

int32_t kvq_query_sizes(const kvq_config* cfg, kvq_sizes* out) {
  if (!out) return KVQ_ERR_INVALID_ARG;
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  const int64_t units = (int64_t)cfg->layers * cfg->batch * cfg->kv_heads;
  const int64_t upl = (int64_t)cfg->batch * cfg->kv_heads;
  const int64_t hd = cfg->head_dim;
  const int64_t slots = (int64_t)cfg->outlier_budget + cfg->aux_capacity;
  const int64_t g = cfg->q_heads / cfg->kv_heads;
  out->units = units;
  out->res_rows = res_rows_of(cfg);
  out->pool_slots = slots;
  out->k_codes_bytes = units * (cfg->max_seq / 32) * 512 * cfg->bits;
  out->k_meta_bytes = units * (cfg->max_seq / cfg->group_k) * hd * 4;
  out->v_codes_bytes = out->k_codes_bytes;
  out->v_meta_bytes = units * cfg->max_seq * (hd / cfg->group_v) * 4;
  out->mask_bytes = units * (cfg->max_seq / 32) * 4;
  out->res_bytes = units * out->res_rows * hd * 2;
  // the decode kernel reads the pool slots 16 at a time: up to 15 rows past the last unit's last slot
  out->pool_rows_bytes = slots > 0 ? (units * slots + 15) * hd * 2 : 0;
  out->pool_idx_bytes = units * slots * 4;
  out->pool_score_bytes = units * slots * 8;
  out->counter_bytes = units * 4;
  out->selected_bytes = upl * cfg->group_k;
  // the split count grows with the amount of work: the largest is the one of a full cache
  const int hp = head_parts_of((int)g, cfg->bits);
  const int64_t s_max = decode_split(upl * hp, (int)g / hp, (int)(hd / cfg->group_v), cfg->max_seq, out->res_rows + slots).splits;
  out->workspace_bytes = decode_workspace_bytes(cfg, g);
  out->prefill_selected_bytes = upl * cfg->max_seq;
  return KVQ_OK;
}

int32_t kvq_append_residual(const kvq_config* cfg, int32_t layer, const void* k_new, const void* v_new,
                            kvq_residual res, int32_t res_start, int32_t n_res, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (!k_new || !v_new || !res.k_res || !res.v_res) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)k_new) | ((uintptr_t)v_new) | ((uintptr_t)res.k_res) | ((uintptr_t)res.v_res)) & 3)
    return KVQ_ERR_INVALID_ARG;                         // rows are copied 4 bytes at a time
  const int32_t rows = (int32_t)res_rows_of(cfg);
  if (res_start < 0 || res_start >= rows || n_res < 0 || n_res >= rows) return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer);
  return from_hip(kvq::launch_append(d, (const __half*)k_new, (const __half*)v_new, (__half*)res.k_res,
                                     (__half*)res.v_res, (res_start + n_res) % rows, (hipStream_t)stream));
}

int32_t kvq_trace_outliers(const kvq_config* cfg, int32_t layer, int32_t group_index, const void* k_group,
                           const void* v_group, int64_t unit_stride, kvq_pool pool, uint8_t* selected,
                           void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (group_index < 0 || group_index >= cfg->max_seq / cfg->group_k) return KVQ_ERR_INVALID_ARG;
  if (!k_group || !v_group || !selected) return KVQ_ERR_INVALID_ARG;
  if (unit_stride < (int64_t)cfg->group_k * cfg->head_dim || unit_stride % 8 != 0) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)k_group) | ((uintptr_t)v_group)) & 15) return KVQ_ERR_INVALID_ARG;
  if (!pool.pool_count || !pool.aux_count || !pool.frozen) return KVQ_ERR_INVALID_ARG;
  if (cfg->outlier_budget > 0 && (!pool.pool_k || !pool.pool_v || !pool.pool_idx || !pool.pool_score))
    return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer);
  return from_hip(kvq::launch_trace(d, group_index, (const __half*)k_group, (const __half*)v_group, unit_stride,
                                    pool, selected, (hipStream_t)stream));
}

int32_t kvq_quantize_group(const kvq_config* cfg, int32_t layer, int32_t group_index, const void* k_group,
                           const void* v_group, int64_t unit_stride, const uint8_t* selected, kvq_qcache qc,
                           void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (group_index < 0 || group_index >= cfg->max_seq / cfg->group_k) return KVQ_ERR_INVALID_ARG;
  if (!k_group || !v_group) return KVQ_ERR_INVALID_ARG;
  if (unit_stride < (int64_t)cfg->group_k * cfg->head_dim || unit_stride % 8 != 0) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)k_group) | ((uintptr_t)v_group)) & 15) return KVQ_ERR_INVALID_ARG;
  if (!qcache_ok(cfg, qc)) return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer, qc);
  return from_hip(kvq::launch_quantize(d, group_index, 1, (const __half*)k_group, (const __half*)v_group,
                                       unit_stride, selected, cfg->group_k, qc, (hipStream_t)stream));
}

namespace {

// Whole-prompt quantization of every sequence of the batch (seq < 0) or of sequence `seq` alone,
// whose pools are emptied first.
int32_t prefill_common(const kvq_config* cfg, int32_t layer, int32_t seq, const void* k_rows, const void* v_rows,
                       int64_t unit_stride, int32_t n_tokens, kvq_pool pool, uint8_t* selected, kvq_qcache qc,
                       kvq_residual res, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (!k_rows || !v_rows || !res.k_res || !res.v_res) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)k_rows) | ((uintptr_t)v_rows) | ((uintptr_t)res.k_res) | ((uintptr_t)res.v_res)) & 15)
    return KVQ_ERR_INVALID_ARG;
  const int32_t G = cfg->group_k, R = cfg->residual;
  if (n_tokens < 1 || (int64_t)n_tokens > (int64_t)cfg->max_seq + R + G - 1) return KVQ_ERR_INVALID_ARG;
  if (unit_stride < (int64_t)n_tokens * cfg->head_dim || unit_stride % 8 != 0) return KVQ_ERR_INVALID_ARG;
  const int32_t n_groups = n_tokens >= R + G ? (n_tokens - R) / G : 0;
  if ((int64_t)n_groups * G > cfg->max_seq) return KVQ_ERR_INVALID_ARG;
  if (!pool.pool_count || !pool.aux_count || !pool.frozen) return KVQ_ERR_INVALID_ARG;
  if (cfg->outlier_budget > 0 && (!pool.pool_k || !pool.pool_v || !pool.pool_idx || !pool.pool_score))
    return KVQ_ERR_INVALID_ARG;
  if (n_groups > 0 && (!selected || !qcache_ok(cfg, qc))) return KVQ_ERR_INVALID_ARG;
  if (n_groups > 65535) return KVQ_ERR_UNSUPPORTED;                    // grid limit of the quantization launch
  // per-step Value schedule: the Values of the tokens between the last whole group and the window of R
  // tokens are quantized as well (from the ring, after the tail rows are there)
  const int32_t n_more_values = cfg->value_per_step ? (n_tokens - R) - n_groups * G : 0;
  if (n_more_values > 0 && !qcache_ok(cfg, qc)) return KVQ_ERR_INVALID_ARG;
  if (cfg->value_per_step && seq >= 0) return KVQ_ERR_UNSUPPORTED;
  if (n_more_values > 0 && n_tokens - R > cfg->max_seq) return KVQ_ERR_INVALID_ARG;
  Dims d = (n_groups > 0 || n_more_values > 0) ? make_dims(cfg, layer, qc) : make_dims(cfg, layer);
  d.keys_only = 0;                                       // whole groups: Keys and Values in one pass
  hipStream_t s = (hipStream_t)stream;
  if (seq >= 0) {                                        // the launches cover the units of this sequence only
    d.unit0 += (int64_t)seq * cfg->kv_heads;
    d.units_per_layer = cfg->kv_heads;
    d.seq0 = seq;
    if (kvq::launch_reset_pools(d, pool, s) != hipSuccess) return KVQ_ERR_LAUNCH;
  }
  if (n_groups > 0) {
    hipError_t e = kvq::launch_prefill_trace(d, n_groups, (const __half*)k_rows, (const __half*)v_rows, unit_stride,
                                             pool, selected, s);
    if (e != hipSuccess) return KVQ_ERR_LAUNCH;
    // (the rows behind the last group go to the ring in the same launch)
    e = kvq::launch_quantize(d, 0, n_groups, (const __half*)k_rows, (const __half*)v_rows, unit_stride, selected,
                             (int64_t)n_groups * G, qc, s, n_tokens - n_groups * G, (__half*)res.k_res,
                             (__half*)res.v_res);
    if (e != hipSuccess) return KVQ_ERR_LAUNCH;
  }
  hipError_t e = n_groups > 0 ? hipSuccess
                              : kvq::launch_tail_copy(d, (const __half*)k_rows, (const __half*)v_rows, unit_stride, 0,
                                                      n_tokens, (__half*)res.k_res, (__half*)res.v_res, s);
  if (e == hipSuccess && n_more_values > 0)
    e = kvq::launch_value_tokens(d, n_groups * G, n_more_values, (__half*)res.v_res, 0, qc, s);
  return from_hip(e);
}

}  // namespace

int32_t kvq_prefill_quantize(const kvq_config* cfg, int32_t layer, const void* k_rows, const void* v_rows,
                             int64_t unit_stride, int32_t n_tokens, kvq_pool pool, uint8_t* selected, kvq_qcache qc,
                             kvq_residual res, void* stream) {
  return prefill_common(cfg, layer, -1, k_rows, v_rows, unit_stride, n_tokens, pool, selected, qc, res, stream);
}

int32_t kvq_prefill_quantize_seq(const kvq_config* cfg, int32_t layer, int32_t seq, const void* k_rows,
                                 const void* v_rows, int64_t unit_stride, int32_t n_tokens, kvq_pool pool,
                                 uint8_t* selected, kvq_qcache qc, kvq_residual res, void* stream) {
  if (!cfg || seq < 0 || seq >= cfg->batch) return KVQ_ERR_INVALID_ARG;
  return prefill_common(cfg, layer, seq, k_rows, v_rows, unit_stride, n_tokens, pool, selected, qc, res, stream);
}

int32_t kvq_append_trace_quantize(const kvq_config* cfg, int32_t layer, const void* k_new, const void* v_new,
                                  kvq_residual res, int32_t res_start, int32_t n_res, int32_t n_quant,
                                  kvq_pool pool, uint8_t* selected, kvq_qcache qc, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (!k_new || !v_new || !res.k_res || !res.v_res) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 3) return KVQ_ERR_INVALID_ARG;
  const int32_t rows = (int32_t)res_rows_of(cfg);
  const int32_t G = cfg->group_k;
  if (res_start < 0 || res_start >= rows || res_start % G != 0) return KVQ_ERR_INVALID_ARG;
  if (n_res + 1 != cfg->residual + G) return KVQ_ERR_INVALID_ARG;
  if (n_quant < 0 || n_quant % G != 0 || n_quant + G > cfg->max_seq) return KVQ_ERR_INVALID_ARG;
  if (!pool.pool_count || !pool.aux_count || !pool.frozen) return KVQ_ERR_INVALID_ARG;
  if (cfg->outlier_budget > 0 && (!pool.pool_k || !pool.pool_v || !pool.pool_idx || !pool.pool_score))
    return KVQ_ERR_INVALID_ARG;
  if (!qcache_ok(cfg, qc)) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)res.k_res) | ((uintptr_t)res.v_res)) & 15) return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer, qc);
  return from_hip(kvq::launch_group_step(d, n_quant / G, (const __half*)k_new, (const __half*)v_new,
                                         (__half*)res.k_res, (__half*)res.v_res, (res_start + n_res) % rows,
                                         res_start, nullptr, pool, selected, qc, (hipStream_t)stream));
}

int32_t kvq_append_trace_quantize_ragged(const kvq_config* cfg, int32_t layer, const void* k_new, const void* v_new,
                                         kvq_residual res, const int32_t* seq_state, kvq_pool pool,
                                         uint8_t* selected, kvq_qcache qc, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (cfg->value_per_step) return KVQ_ERR_UNSUPPORTED;
  if (!k_new || !v_new || !res.k_res || !res.v_res || !seq_state) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 3) return KVQ_ERR_INVALID_ARG;
  if (((uintptr_t)seq_state) & 15) return KVQ_ERR_INVALID_ARG;
  if (!pool.pool_count || !pool.aux_count || !pool.frozen) return KVQ_ERR_INVALID_ARG;
  if (cfg->outlier_budget > 0 && (!pool.pool_k || !pool.pool_v || !pool.pool_idx || !pool.pool_score))
    return KVQ_ERR_INVALID_ARG;
  if (!qcache_ok(cfg, qc)) return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)res.k_res) | ((uintptr_t)res.v_res)) & 15) return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer, qc);
  return from_hip(kvq::launch_group_step(d, 0, (const __half*)k_new, (const __half*)v_new, (__half*)res.k_res,
                                         (__half*)res.v_res, 0, 0, seq_state, pool, selected, qc,
                                         (hipStream_t)stream));
}

int32_t kvq_quantize_value_tokens(const kvq_config* cfg, int32_t layer, int32_t first_token, int32_t count,
                                  void* v_res, int32_t ring_row, kvq_qcache qc, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (!cfg->value_per_step) return KVQ_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  const int32_t rows = (int32_t)res_rows_of(cfg);
  if (first_token < 0 || count < 1 || count > rows || (int64_t)first_token + count > cfg->max_seq)
    return KVQ_ERR_INVALID_ARG;
  if (ring_row < 0 || ring_row >= rows) return KVQ_ERR_INVALID_ARG;
  if (!v_res || (((uintptr_t)v_res) & 3)) return KVQ_ERR_INVALID_ARG;
  if (!qcache_ok(cfg, qc)) return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer, qc);
  return from_hip(kvq::launch_value_tokens(d, first_token, count, (__half*)v_res, ring_row, qc, (hipStream_t)stream));
}

int32_t kvq_dequantize(const kvq_config* cfg, int32_t layer, kvq_qcache qc, int32_t n_quant, kvq_pool pool,
                       int32_t t0, int32_t n, void* k_out, void* v_out, int64_t out_unit_stride, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  if (n_quant < 0 || n_quant > cfg->max_seq || n_quant % cfg->group_k != 0) return KVQ_ERR_INVALID_ARG;
  if (t0 < 0 || n < 1 || t0 % kvq::kBlockTokens != 0 || n % kvq::kBlockTokens != 0 || (int64_t)t0 + n > n_quant)
    return KVQ_ERR_INVALID_ARG;
  if (!k_out || !v_out || ((((uintptr_t)k_out) | ((uintptr_t)v_out)) & 1)) return KVQ_ERR_INVALID_ARG;
  if (out_unit_stride < (int64_t)n * cfg->head_dim) return KVQ_ERR_INVALID_ARG;
  if (!qcache_ok(cfg, qc) || !pool.pool_count || !pool.aux_count) return KVQ_ERR_INVALID_ARG;
  if (cfg->outlier_budget > 0 && (!pool.pool_k || !pool.pool_v || !pool.pool_idx)) return KVQ_ERR_INVALID_ARG;
  const Dims d = make_dims(cfg, layer, qc);
  const int64_t n_blocks = n / kvq::kBlockTokens;
  if (n_blocks * d.units_per_layer > 0x7FFFFFFFll) return KVQ_ERR_UNSUPPORTED;
  return from_hip(kvq::launch_dequantize(d, t0 / kvq::kBlockTokens, (int32_t)n_blocks, qc, pool, (__half*)k_out,
                                         (__half*)v_out, out_unit_stride, (hipStream_t)stream));
}

int32_t kvq_seq_advance(const kvq_config* cfg, int32_t* seq_state, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (!seq_state || (((uintptr_t)seq_state) & 15)) return KVQ_ERR_INVALID_ARG;
  return from_hip(kvq::launch_seq_advance(make_dims(cfg, 0), seq_state, (hipStream_t)stream));
}

namespace {

// Scratch of kvq_decode_attention_static: the decode launch's workspace (arrival counters, partial
// results) for callers that cannot hand one over.  One array per device, held until the process ends;
// its device address is looked up once per device and kept.  In host code the array's NAME is not
// a device address: only the looked-up pointer is ever passed to a kernel.
constexpr size_t kScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int32_t scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVQ_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KVQ_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return KVQ_OK;
}

// (a fill kernel and not a memset: a memset node in a captured graph has replayed wrongly on this stack)
__global__ void zero_words_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// The decode launch, shared by the two entry points: `seq_state` null = every sequence has the
// state given; otherwise n_quant and n_res are upper bounds and each sequence brings its own.
int32_t decode_common(const kvq_config* cfg, int32_t layer, const void* q, int32_t q_tokens, kvq_qcache qc,
                      int32_t n_quant, kvq_residual res, int32_t res_start, int32_t n_res, const int32_t* seq_state,
                      const void* k_new, const void* v_new, kvq_pool pool, void* out, void* workspace,
                      size_t workspace_bytes, void* stream, bool static_scratch = false,
                      const int32_t* plan = nullptr, const float* rope = nullptr, int64_t rope_stride = 0) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (layer < 0 || layer >= cfg->layers) return KVQ_ERR_INVALID_ARG;
  const int32_t g = cfg->q_heads / cfg->kv_heads;
  if (q_tokens < 1 || q_tokens > 8) return KVQ_ERR_INVALID_ARG;
  const int32_t qrows = q_tokens * g;                    // query rows per kv head: 1, 2, 4 or 8
  if (qrows != 1 && qrows != 2 && qrows != 4 && qrows != 8) return KVQ_ERR_UNSUPPORTED;
  // a token must not see the tokens after it: those are hidden as the newest residual rows
  if (q_tokens > 1 && (seq_state || k_new || n_res < q_tokens - 1)) return KVQ_ERR_INVALID_ARG;
  if (!q || !out) return KVQ_ERR_INVALID_ARG;
  // rows are read 16 bytes at a time (the query rows too: they stand in for rows past the last pool slot)
  if ((((uintptr_t)q) | ((uintptr_t)res.k_res) | ((uintptr_t)res.v_res) | ((uintptr_t)pool.pool_k) |
       ((uintptr_t)pool.pool_v) | ((uintptr_t)qc.k_codes) | ((uintptr_t)qc.v_codes)) & 15)
    return KVQ_ERR_INVALID_ARG;
  if ((((uintptr_t)out) & 1) || ((((uintptr_t)qc.k_meta) | ((uintptr_t)qc.v_meta) | ((uintptr_t)qc.mask)) & 3))
    return KVQ_ERR_INVALID_ARG;
  if (n_quant < 0 || n_quant > cfg->max_seq || n_quant % cfg->group_k != 0) return KVQ_ERR_INVALID_ARG;
  const int32_t rows = (int32_t)res_rows_of(cfg);
  if (n_res < 0 || n_res > rows || res_start < 0 || res_start >= rows) return KVQ_ERR_INVALID_ARG;
  if (res_start % 16 != 0) return KVQ_ERR_INVALID_ARG;     // residual rows are read 16 at a time, without wrapping
  if (n_quant + n_res + (k_new ? 1 : 0) < 1) return KVQ_ERR_INVALID_ARG;
  if ((k_new != nullptr) != (v_new != nullptr)) return KVQ_ERR_INVALID_ARG;
  if (k_new) {                                          // the new token must leave the ring short of full
    if (n_res + 1 >= cfg->residual + cfg->group_k || !res.k_res || !res.v_res) return KVQ_ERR_INVALID_ARG;
    if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 3) return KVQ_ERR_INVALID_ARG;
  }
  if (rope) {                                            // rows of head_dim floats, read 8 bytes at a time
    if (!k_new || (((uintptr_t)rope) & 15)) return KVQ_ERR_INVALID_ARG;
    if (rope_stride != 0 && (rope_stride < cfg->head_dim || rope_stride % 4 != 0)) return KVQ_ERR_INVALID_ARG;
  }
  // the arrays are needed even when nothing is quantized yet: every workgroup issues the loads of a
  // first block (the last one, or block 0) whether or not it has quantized tokens to work on
  if (!qcache_ok(cfg, qc)) return KVQ_ERR_INVALID_ARG;
  if (n_res > 0 && (!res.k_res || !res.v_res)) return KVQ_ERR_INVALID_ARG;
  if (!pool.pool_count || !pool.aux_count) return KVQ_ERR_INVALID_ARG;
  // every pool slot is read, filled or not, so the rows must exist whenever there are slots
  if (cfg->outlier_budget + cfg->aux_capacity > 0 && (!pool.pool_k || !pool.pool_v)) return KVQ_ERR_INVALID_ARG;
  if (static_scratch) {                                  // the library's own array stands in for the workspace
    if (decode_workspace_bytes(cfg, qrows) > (int64_t)kScratchBytes) return KVQ_ERR_SCRATCH;
    const int32_t got = scratch_of_current_device(&workspace);
    if (got != KVQ_OK) return got;
    workspace_bytes = kScratchBytes;
  }
  if (!workspace || ((uintptr_t)workspace & 255) != 0) return KVQ_ERR_WORKSPACE;
  if ((int64_t)workspace_bytes < decode_workspace_bytes(cfg, qrows)) return KVQ_ERR_WORKSPACE;

  kvq::DecodeArgs a;
  a.d = make_dims(cfg, layer, qc);
  a.q = (const __half*)q;
  a.k_codes = (const uint8_t*)qc.k_codes;
  a.k_meta = (const uint32_t*)qc.k_meta;
  a.v_codes = (const uint8_t*)qc.v_codes;
  a.v_meta = (const uint32_t*)qc.v_meta;
  a.mask = (const uint32_t*)qc.mask;
  a.k_res = (const __half*)res.k_res;
  a.v_res = (const __half*)res.v_res;
  a.pool_k = (const __half*)pool.pool_k;
  a.pool_v = (const __half*)pool.pool_v;
  a.pool_count = pool.pool_count;
  a.aux_count = pool.aux_count;
  a.out = (__half*)out;
  a.counters = (int32_t*)workspace;
  a.partials = (float*)((unsigned char*)workspace + kCounterBytes((int64_t)a.d.units_per_layer * head_parts_of(qrows, cfg->bits)));
  a.n_quant = n_quant;
  a.res_start = res_start;
  a.n_res = n_res;
  a.seq = seq_state;
  a.k_new = (const __half*)k_new;
  a.v_new = (const __half*)v_new;
  a.head_parts = head_parts_of(qrows, cfg->bits);
  a.q_tokens = q_tokens;
  a.g_shift = g == 1 ? 0 : g == 2 ? 1 : g == 4 ? 2 : 3;
  const Split sp = decode_split((int64_t)a.d.units_per_layer * a.head_parts, qrows / a.head_parts, a.d.vgroups, n_quant,
                                (int64_t)n_res + (k_new ? 1 : 0) + a.d.pool_slots);
  a.splits = sp.splits;
  a.nw = sp.nw;
  a.mc_per_split = sp.mc_per_split;
  a.plan = nullptr;
  a.plan_entries = 0;
  a.rope = rope;
  a.rope_stride = rope_stride;
  if (plan) {                                            // the plan's own shape; splits are per sequence
    const PlanShape ps = plan_shape(cfg);
    if (ps.entries == 0 || q_tokens != 1 || k_new) return KVQ_ERR_UNSUPPORTED;
    a.plan = plan;
    a.plan_entries = ps.entries;
    a.nw = ps.nw;
    a.splits = 1;
    a.seq = nullptr;
  }
  if (static_scratch && sp.splits > 1) {
    // The array is shared by every call on this device, whatever its shape: where this launch keeps its
    // arrival counters an earlier one may have left partial results.  They must start at zero.
    const int words = (int)(kCounterBytes((int64_t)a.d.units_per_layer * a.head_parts) / 4);
    hipLaunchKernelGGL(zero_words_kernel, dim3((words + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       (uint32_t*)workspace, words);
    if (hipGetLastError() != hipSuccess) return KVQ_ERR_LAUNCH;
  }
  return from_hip(kvq::launch_decode(a, (hipStream_t)stream));
}

}  // namespace

int32_t kvq_decode_attention(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qc, int32_t n_quant,
                             kvq_residual res, int32_t res_start, int32_t n_res, kvq_pool pool, void* out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(cfg, layer, q, 1, qc, n_quant, res, res_start, n_res, nullptr, nullptr, nullptr, pool, out,
                       workspace, workspace_bytes, stream);
}

int32_t kvq_decode_attention_static(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qc, int32_t n_quant,
                                    kvq_residual res, int32_t res_start, int32_t n_res, kvq_pool pool, void* out,
                                    void* stream) {
  return decode_common(cfg, layer, q, 1, qc, n_quant, res, res_start, n_res, nullptr, nullptr, nullptr, pool, out,
                       nullptr, 0, stream, true);
}

int64_t kvq_decode_workspace_bytes(const kvq_config* cfg, int32_t q_tokens) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  const int64_t rows = (int64_t)q_tokens * (cfg->q_heads / cfg->kv_heads);
  if (q_tokens < 1 || q_tokens > 8) return KVQ_ERR_INVALID_ARG;
  if (rows != 1 && rows != 2 && rows != 4 && rows != 8) return KVQ_ERR_UNSUPPORTED;
  return decode_workspace_bytes(cfg, rows);
}

int32_t kvq_decode_launch_shape(const kvq_config* cfg, int32_t q_tokens, int32_t n_quant, int32_t fp_rows,
                                int32_t* splits, int32_t* waves, int32_t* minichunks_per_split) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (!splits || !waves || !minichunks_per_split) return KVQ_ERR_INVALID_ARG;
  if (q_tokens < 1 || q_tokens > 8 || fp_rows < 0) return KVQ_ERR_INVALID_ARG;
  const int32_t qrows = q_tokens * (cfg->q_heads / cfg->kv_heads);
  if (qrows != 1 && qrows != 2 && qrows != 4 && qrows != 8) return KVQ_ERR_UNSUPPORTED;
  if (n_quant < 0 || n_quant > cfg->max_seq || n_quant % cfg->group_k != 0) return KVQ_ERR_INVALID_ARG;
  const int hp = head_parts_of(qrows, cfg->bits);
  const Split sp = decode_split((int64_t)cfg->batch * cfg->kv_heads * hp, qrows / hp, cfg->head_dim / cfg->group_v,
                                n_quant, fp_rows);
  *splits = sp.splits;
  *waves = sp.nw;
  *minichunks_per_split = sp.mc_per_split;
  return KVQ_OK;
}

int32_t kvq_decode_attention_multi(const kvq_config* cfg, int32_t layer, const void* q, int32_t q_tokens,
                                   kvq_qcache qc, int32_t n_quant, kvq_residual res, int32_t res_start,
                                   int32_t n_res, kvq_pool pool, void* out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return decode_common(cfg, layer, q, q_tokens, qc, n_quant, res, res_start, n_res, nullptr, nullptr, nullptr, pool,
                       out, workspace, workspace_bytes, stream);
}

int32_t kvq_append_decode_attention(const kvq_config* cfg, int32_t layer, const void* q, const void* k_new,
                                    const void* v_new, kvq_qcache qc, int32_t n_quant, kvq_residual res,
                                    int32_t res_start, int32_t n_res, kvq_pool pool, void* out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  if (!k_new || !v_new) return KVQ_ERR_INVALID_ARG;
  return decode_common(cfg, layer, q, 1, qc, n_quant, res, res_start, n_res, nullptr, k_new, v_new, pool, out,
                       workspace, workspace_bytes, stream);
}

int32_t kvq_append_decode_attention_rope(const kvq_config* cfg, int32_t layer, const void* q, const void* k_new,
                                         const void* v_new, const float* rope, int64_t rope_stride, kvq_qcache qc,
                                         int32_t n_quant, kvq_residual res, int32_t res_start, int32_t n_res,
                                         kvq_pool pool, void* out, void* workspace, size_t workspace_bytes,
                                         void* stream) {
  if (!k_new || !v_new || !rope) return KVQ_ERR_INVALID_ARG;
  return decode_common(cfg, layer, q, 1, qc, n_quant, res, res_start, n_res, nullptr, k_new, v_new, pool, out,
                       workspace, workspace_bytes, stream, false, nullptr, rope, rope_stride);
}

int32_t kvq_rope_rotate(const kvq_config* cfg, const void* x, int32_t heads, const float* rope, int64_t rope_stride,
                        void* out, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  if (!x || !out || !rope || heads < 1 || heads > 65536) return KVQ_ERR_INVALID_ARG;
  if (((((uintptr_t)x) | ((uintptr_t)out)) & 3) || (((uintptr_t)rope) & 15)) return KVQ_ERR_INVALID_ARG;
  if (rope_stride != 0 && (rope_stride < cfg->head_dim || rope_stride % 4 != 0)) return KVQ_ERR_INVALID_ARG;
  return from_hip(kvq::launch_rope((const __half*)x, (int64_t)cfg->batch * heads, heads, rope, rope_stride,
                                   (__half*)out, (hipStream_t)stream));
}

int64_t kvq_seq_plan_bytes(const kvq_config* cfg) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  const PlanShape ps = plan_shape(cfg);
  if (ps.entries == 0) return KVQ_ERR_UNSUPPORTED;
  return (8 + kPlanEntryWords * (int64_t)ps.entries) * 4;
}

int32_t kvq_seq_plan(const kvq_config* cfg, const int32_t* seq_state, int32_t max_n_quant, int32_t max_n_res,
                     int32_t* plan, void* stream) {
  const int32_t st = check_config(cfg);
  if (st != KVQ_OK) return st;
  const PlanShape ps = plan_shape(cfg);
  if (ps.entries == 0) return KVQ_ERR_UNSUPPORTED;
  if (!seq_state || (((uintptr_t)seq_state) & 15) || !plan || (((uintptr_t)plan) & 15)) return KVQ_ERR_INVALID_ARG;
  if (max_n_quant < 0 || max_n_quant > cfg->max_seq || max_n_quant % cfg->group_k != 0) return KVQ_ERR_INVALID_ARG;
  if (max_n_res < 0 || max_n_res > (int32_t)res_rows_of(cfg)) return KVQ_ERR_INVALID_ARG;
  return from_hip(kvq::launch_seq_plan(make_dims(cfg, 0), seq_state, max_n_quant, max_n_res, ps.entries, plan,
                                       (hipStream_t)stream));
}

int32_t kvq_decode_attention_planned(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qc,
                                     kvq_residual res, const int32_t* plan, int32_t max_n_quant, int32_t max_n_res,
                                     kvq_pool pool, void* out, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  if (!plan || (((uintptr_t)plan) & 15)) return KVQ_ERR_INVALID_ARG;
  return decode_common(cfg, layer, q, 1, qc, max_n_quant, res, 0, max_n_res, nullptr, nullptr, nullptr, pool, out,
                       workspace, workspace_bytes, stream, false, plan);
}

int32_t kvq_decode_attention_ragged(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qc,
                                    kvq_residual res, const int32_t* seq_state, int32_t max_n_quant,
                                    int32_t max_n_res, kvq_pool pool, void* out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  if (!seq_state || (((uintptr_t)seq_state) & 15)) return KVQ_ERR_INVALID_ARG;
  return decode_common(cfg, layer, q, 1, qc, max_n_quant, res, 0, max_n_res, seq_state, nullptr, nullptr, pool, out,
                       workspace, workspace_bytes, stream);
}

}  // extern "C"
