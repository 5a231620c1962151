// Internal declarations shared by the host entry points and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "kvq.h"

namespace kvq {

constexpr int kHeadDim = 128;      // the only head size built
constexpr int kBlockTokens = 32;   // tokens per packed block
constexpr int kMiniChunk = 128;     // quantized tokens one wavefront handles at a time
constexpr int kComputeUnits = 256;      // of the device this build targets
constexpr int kLdsPerComputeUnit = 160 * 1024;
// Wavefronts per SIMD the decode kernel is compiled and launched for: two, with half of the
// register file each.  Measured against three (a third of the file): no spills in any instance,
// and 3 to 45 % shorter launches, the more query heads per kv head the more.
constexpr int kDecodeWavesPerSimd = 2;
constexpr int kFpGroupRows = 16;   // full-precision rows one wavefront handles at a time
constexpr float kNegBig = -1.0e30f;

// Everything a kernel needs to find a unit's data, derived once on the host.
struct Dims {
  int32_t batch, q_heads, kv_heads, g;       // g = q_heads / kv_heads
  int32_t bits, G, Gv, N, A;
  int32_t max_seq, res_rows, pool_slots;
  int32_t R;                                  // residual length (the ring is full at R + G rows)
  int32_t units_per_layer;                    // batch * kv_heads
  int64_t unit0;                              // first unit of the layer being processed
  int32_t block_bytes;                        // 512 * bits
  int32_t blocks_per_unit;                    // max_seq / 32; paged: blocks per plane = n_pages * G / 32
  int32_t groups_per_unit;                    // max_seq / G;  paged: n_pages
  int32_t vgroups;                            // head_dim / Gv
  int32_t bpg_shift;                          // log2(G / 32): blocks per Key group
  // Paged quantized cache (page_table != null): the quantized arrays hold, per plane (layer, kv head),
  // n_pages pages of one Key group each; group j of sequence b is page page_table[b * table_stride + j].
  const int32_t* page_table;
  int32_t table_stride;
  int32_t n_pages;
  int64_t plane0;                             // layer * kv_heads
  // A launch over the units of ONE sequence (units_per_layer = kv_heads, unit0 includes the sequence):
  int32_t seq0;                               // that sequence (0 for launches over the whole batch)
  int32_t keys_only;                          // group quantization leaves the Value arrays alone (Values are
                                              // quantized token by token, at each step)
};

// Where group `group` of local unit ul = b * kv_heads + h is stored: `row` indexes runs of
// groups_per_unit groups (blocks_per_unit blocks), `slot` the group inside the run.  A page number
// outside [0, n_pages) is clamped, so that whatever the table holds the access stays inside the pool.
struct GroupPlace {
  int64_t row;
  int32_t slot;
};
__device__ inline GroupPlace place_of_group(const Dims& d, int ul, int group) {
  if (!d.page_table) return {d.unit0 + ul, group};
  const int b = ul / d.kv_heads, h = ul - b * d.kv_heads;
  const int page = d.page_table[(int64_t)(d.seq0 + b) * d.table_stride + group];
  return {d.plane0 + h, min(max(page, 0), d.n_pages - 1)};
}

struct DecodeArgs {
  Dims d;
  const __half* q;
  const uint8_t* k_codes;
  const uint32_t* k_meta;
  const uint8_t* v_codes;
  const uint32_t* v_meta;
  const uint32_t* mask;
  const __half* k_res;
  const __half* v_res;
  const __half* pool_k;
  const __half* pool_v;
  const int32_t* pool_count;
  const int32_t* aux_count;
  __half* out;
  float* partials;      // [units_per_layer][splits][g][head_dim + 2]
  int32_t* counters;    // [units_per_layer], zero on entry and on exit
  int32_t n_quant, res_start, n_res;   // the batch's state; with `seq`, upper bounds of n_quant and n_res
  const int32_t* seq;   // per-sequence state [batch][4] = {n_quant, res_start, n_res, active}, or null
  const __half* k_new;  // [batch][kv_heads][head_dim] rows of the token being decoded, not yet in the ring (it is
  const __half* v_new;  // attended as the newest residual row, and stored in the ring by the launch), or null
  int32_t splits;       // workgroups per unit
  int32_t nw;           // wavefronts per workgroup
  int32_t head_parts;   // workgroup rows that share a kv head's query rows (the host passes 1: every row count has its instance)
  int32_t q_tokens;     // consecutive query tokens attended at once (1 in a plain decode step); the rows of a
  int32_t g_shift;      // kv head are its q_tokens * g (token, query head) pairs, token-major; g = 1 << g_shift
  int32_t mc_per_split; // 128-token mini-chunks of the quantized segment per workgroup
  // A launch plan (sequences of different lengths dealt by length), or null.  int32: [0] = entries in use;
  // from [8] on the entries, 8 words each: {sequence, split, splits of the sequence, first mini-chunk,
  // n_quant, res_start, n_res, end of the mini-chunks}.  The entries of a sequence are consecutive.  With a
  // plan the grid is (plan_entries, kv heads, 1): workgroup x does entry x; `seq`, `splits` and
  // `mc_per_split` are not used.
  const int32_t* plan;
  int32_t plan_entries;     // entries the plan has room for (the grid's x extent)
  // Rotary position embedding of the query rows and of the new Key row inside the launch (null: none):
  // fp32 cosines of the head_dim / 2 angles of the new token's position, then their sines; sequence b's
  // row starts rope_stride elements after sequence b - 1's (0: one row for all).
  const float* rope;
  int64_t rope_stride;
};

hipError_t launch_append(const Dims& d, const __half* k_new, const __half* v_new, __half* k_res, __half* v_res,
                         int32_t row, hipStream_t s);
hipError_t launch_dequantize(const Dims& d, int32_t block0, int32_t n_blocks, const kvq_qcache& qc, const kvq_pool& pool,
                             __half* k_out, __half* v_out, int64_t out_unit_stride, hipStream_t s);
hipError_t launch_reset_pools(const Dims& d, const kvq_pool& pool, hipStream_t s);
hipError_t launch_trace(const Dims& d, int32_t group_index, const __half* k_group, const __half* v_group,
                        int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s);
hipError_t launch_quantize(const Dims& d, int32_t group_index, int32_t n_groups, const __half* k_group,
                           const __half* v_group, int64_t unit_stride, const uint8_t* selected,
                           int64_t selected_unit_stride, const kvq_qcache& qc, hipStream_t s, int32_t tail_n = 0,
                           __half* k_res = nullptr, __half* v_res = nullptr);
hipError_t launch_prefill_trace(const Dims& d, int32_t n_groups, const __half* k_rows, const __half* v_rows,
                                int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s);
hipError_t launch_tail_copy(const Dims& d, const __half* k_rows, const __half* v_rows, int64_t unit_stride, int32_t n0,
                            int32_t n, __half* k_res, __half* v_res, hipStream_t s);
hipError_t launch_group_step(const Dims& d, int32_t group_index, const __half* k_new, const __half* v_new, __half* k_res,
                             __half* v_res, int32_t append_row, int32_t group_row0, const int32_t* seq,
                             const kvq_pool& pool, uint8_t* selected, const kvq_qcache& qc, hipStream_t s);
hipError_t launch_seq_advance(const Dims& d, int32_t* seq, hipStream_t s);
hipError_t launch_seq_plan(const Dims& d, const int32_t* seq, int32_t max_n_quant, int32_t max_n_res, int32_t entries,
                           int32_t* plan, hipStream_t s);
hipError_t launch_value_tokens(const Dims& d, int32_t first_token, int32_t count, __half* v_res, int32_t ring_row,
                               const kvq_qcache& qc, hipStream_t s);
hipError_t launch_decode(const DecodeArgs& a, hipStream_t s);
hipError_t launch_rope(const __half* x, int64_t rows, int32_t rows_per_seq, const float* rope, int64_t rope_stride,
                       __half* out, hipStream_t s);
int decode_wave_lds_bytes(int g, int vgroups);   // LDS one decode wavefront needs

// ---- exchanges inside a row of 16 lanes on the DPP path (no LDS traffic) -----------------------
// Step s of a butterfly over 2, 4, 8, 16 adjacent lanes: the value of lane ^ 1, of lane ^ 2, then of
// the mirror lane inside 8 and inside 16.  The mirrors pair a lane with one of the other half; they
// stand for lane ^ 4 and lane ^ 8 in a reduction because by then all lanes of a half hold the same
// partial result.  Any commutative, associative and exact combination (min, max, exact sums) may use it.
template <int STEP>
__device__ __forceinline__ uint32_t row_partner_u32(uint32_t v) {
  constexpr int ctrl = STEP == 0 ? 0xB1 /* quad_perm [1,0,3,2] */ : STEP == 1 ? 0x4E /* quad_perm [2,3,0,1] */
                       : STEP == 2 ? 0x141 /* row_half_mirror */ : 0x140 /* row_mirror */;
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, 0xf, 0xf, false);
}
template <int STEP>
__device__ __forceinline__ float row_partner(float v) {
  return __uint_as_float(row_partner_u32<STEP>(__float_as_uint(v)));
}
template <int STEP>
__device__ __forceinline__ double row_partner(double v) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  const unsigned long long lo = row_partner_u32<STEP>((uint32_t)b), hi = row_partner_u32<STEP>((uint32_t)(b >> 32));
  return __longlong_as_double((long long)((hi << 32) | lo));
}

// ---- packed layout ---------------------------------------------------------------------------
// Byte offset (inside a block) of the u32 word that holds field f of lane l, and the bit
// offset of code x = 2v + e inside that word.  A code occupies bits code_bit .. code_bit + bits - 1
// taken modulo 32 (one 4-bit code wraps around the end of its word): it is put in place with a
// rotation.  Positions are chosen so that the word (for half of the fields: the word rotated right
// by 8) holds a field's codes at bits 2..9 of each 16-bit half, the top of an fp16 significand.
__host__ __device__ inline int word_byte(int bits, int lane, int f) {
  return bits == 2 ? 16 * lane + 4 * (f >> 1) : 1024 * (f >> 2) + 16 * lane + 4 * (f & 3);
}
__host__ __device__ inline int code_bit(int bits, int f, int x) {
  const int v = x >> 1, e = x & 1;
  return (bits == 2 ? 16 * e + 2 * (v + 1) + 8 * (f & 1) : 16 * e + 2 + 4 * (v & 1) + 8 * (v >> 1)) & 31;
}
__host__ __device__ inline uint32_t place_code(uint32_t code, int bit) { return (code << bit) | (code >> ((32 - bit) & 31)); }
// Key block: (token t in 0..31, channel c) -> (lane, field, x)
__host__ __device__ inline void k_pos(int t, int c, int& lane, int& f, int& x) {
  lane = 16 * ((c & 31) >> 3) + (t & 15);
  f = 4 * (t >> 4) + (c >> 5);
  x = c & 7;
}
// Value block: (token t in 0..31, channel c) -> (lane, field, x)
__host__ __device__ inline void v_pos(int t, int c, int& lane, int& f, int& x) {
  lane = 16 * (t >> 3) + (c & 15);
  f = c >> 4;
  x = t & 7;
}

}  // namespace kvq
