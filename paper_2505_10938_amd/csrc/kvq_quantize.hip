// Residual append and group quantization (mean replacement, Eq. 2 per group, packing), and the
// fused group step (append + outlier competition + quantization in one launch).
#include "kvq_common.h"
#include "kvq_trace_core.h"

#include <type_traits>

// The integer code decisions must not depend on how the compiler fuses multiplies and adds.
#pragma clang fp contract(off)

namespace kvq {

namespace {

// ---- residual append: one row of 128 fp16 per unit, K and V -----------------------------------
__global__ void __launch_bounds__(128) append_kernel(Dims d, const __half* __restrict__ k_new,
                                                     const __half* __restrict__ v_new, __half* __restrict__ k_res,
                                                     __half* __restrict__ v_res, int32_t row) {
  const int ul = blockIdx.x;                       // unit inside the layer
  const int64_t u = d.unit0 + ul;
  const int tid = threadIdx.x;                     // 64 threads for K, 64 for V, 4 bytes each
  const int which = tid >> 6, lane = tid & 63;
  const uint32_t* src = (const uint32_t*)((which ? v_new : k_new) + (int64_t)ul * kHeadDim);
  uint32_t* dst = (uint32_t*)((which ? v_res : k_res) + (u * d.res_rows + row) * kHeadDim);
  dst[lane] = src[lane];
}

// ---- Eq. 2 for one value against its group's (min, step) -------------------------------------
// step is the fp16-rounded step as float; code = number of thresholds (k + 1/2) * step reached
// by fl32(x - mn).  The products are exact in fp32, so the decision is IEEE-reproducible.
__device__ inline uint32_t quant_code(float x, float mn, float step, int levels) {
  if (step == 0.0f) return 0u;
  const float t = x - mn;
  uint32_t code = 0;
  for (int k = 0; k < levels; ++k) {
    const float thr = ((float)k + 0.5f) * step;
    code += (t >= thr) ? 1u : 0u;
  }
  return code;
}

// The same decision as quant_code, as a binary search: code k is reached when fl32(x - mn) >= (2k - 1) * h
// with h = step / 2 (exact products again: 2k - 1 has 5 bits, h 11).  Returns 2 * code as a float.  A group
// whose step is zero passes h = +infinity: no threshold is reached, the code is 0.
template <int BITS>
__device__ __forceinline__ float quant_code_twice(float x, float mn, float h) {
  const float t = x - mn;
  float acc = 0.0f;
#pragma unroll
  for (int l = BITS - 1; l >= 0; --l) {
    const float c = (float)(2 << l);
    const float w = acc + (c - 1.0f);
    acc = (t >= w * h) ? acc + c : acc;
  }
  return acc;
}
__device__ __forceinline__ float half_step_of(__half st) {
  const float s = __half2float(st);
  return s == 0.0f ? __uint_as_float(0x7F800000u) : 0.5f * s;
}
// 2 * code (as returned above) put at bit position p of a packed word (a compile-time position of the
// first field of a word; bits beyond 31 wrap around)
template <int BITS>
__device__ __forceinline__ uint32_t place_twice(float acc, int p) {
  const uint32_t b = (uint32_t)acc;
  return (b << (p - 1)) | (p + BITS > 32 ? b >> (33 - p) : 0u);
}

// fp16 step from a group's min and max: fl32(fl32(max - min) * c_b) rounded to nearest even.
__device__ inline __half step_of(float mn, float mx, int bits) {
  const float c = bits == 2 ? __uint_as_float(0x3EAAAAABu) : __uint_as_float(0x3D888889u);  // 1/3, 1/15
  const float d = mx - mn;
  float s32 = d * c;
  // Keep the fp32 product as its own rounding step: without this the compiler merges the
  // multiply and the fp16 conversion into one instruction with a single rounding.
  asm volatile("" : "+v"(s32));
  return __float2half_rn(s32);
}

constexpr int kRowB = 272;   // LDS row: 128 fp16 + 16 bytes of padding (spreads rows over the banks)

__device__ inline float half_at(const unsigned char* p) { return __half2float(*(const __half*)p); }
__device__ inline float lo_half(uint32_t w) { return __half2float(__ushort_as_half((unsigned short)(w & 0xFFFFu))); }
__device__ inline float hi_half(uint32_t w) { return __half2float(__ushort_as_half((unsigned short)(w >> 16))); }

constexpr int kQuantThreads = 1024;
constexpr int64_t kPromptGroups = 1024;   // from this many groups in one launch on, prompt_quantize_kernel takes them

// Minimum and maximum over groups of `n` adjacent lanes (n = 4, 8 or 16).
__device__ inline void team_minmax(float& mn, float& mx, int n) {
  mn = fminf(mn, row_partner<0>(mn));
  mx = fmaxf(mx, row_partner<0>(mx));
  mn = fminf(mn, row_partner<1>(mn));
  mx = fmaxf(mx, row_partner<1>(mx));
  if (n > 4) {
    mn = fminf(mn, row_partner<2>(mn));
    mx = fmaxf(mx, row_partner<2>(mx));
  }
  if (n > 8) {
    mn = fminf(mn, row_partner<3>(mn));
    mx = fmaxf(mx, row_partner<3>(mx));
  }
}

// LDS of the quantization: the whole group (G x 128, K and V) and its meta.
template <int G>
struct QuantLds {
  unsigned char* sk;     // [G] rows of kRowB bytes
  unsigned char* sv;     // [G] rows
  float2* skm;           // [128] K meta: {zero, step / 2 (+infinity for a zero step)}
  float2* svm;           // [vgroups][G] V meta, the same pair
  uint8_t* ssel;         // [G] selected flags
  __device__ QuantLds(unsigned char* smem, int vgroups) {
    sk = smem;
    sv = sk + G * kRowB;
    skm = (float2*)(sv + G * kRowB);
    svm = skm + kHeadDim;
    ssel = (uint8_t*)(svm + G * vgroups);
  }
};
template <int G>
size_t quant_lds_bytes(int vgroups) { return (size_t)2 * G * kRowB + kHeadDim * 8 + (size_t)G * vgroups * 8 + G; }

// The group's rows, 16 bytes per thread: K rows first, then V rows.
template <int G>
struct GroupRows {
  static constexpr int kLoads = 2 * G * 16 / kQuantThreads;   // 1, 2 or 4
  uint4 rw[kLoads];
};
template <int G>
__device__ __forceinline__ void rows_issue(GroupRows<G>& r, const __half* gk, const __half* gv, int tid) {
#pragma unroll
  for (int q = 0; q < GroupRows<G>::kLoads; ++q) {
    const int e = q * kQuantThreads + tid;
    const int kv = e / (G * 16), rem = e % (G * 16);
    r.rw[q] = *(const uint4*)((kv ? gv : gk) + (rem >> 4) * kHeadDim + (rem & 15) * 8);
  }
}
template <int G>
__device__ __forceinline__ void rows_to_lds(const GroupRows<G>& r, const QuantLds<G>& L, int tid) {
#pragma unroll
  for (int q = 0; q < GroupRows<G>::kLoads; ++q) {
    const int e = q * kQuantThreads + tid;
    const int kv = e / (G * 16), rem = e % (G * 16);
    *(uint4*)((kv ? L.sv : L.sk) + (rem >> 4) * kRowB + (rem & 15) * 16) = r.rw[q];
  }
}

// Quantization of the group held in LDS (rows stored, not yet synchronized): mean replacement of
// the rows flagged (`flag` = this thread's token, threads below G), meta, codes, mask words.
// Every thread of the 1024-thread workgroup calls it.  (u, group_index) say where the group is stored
// (place_of_group): the unit and the group's index, or, in a paged cache, the plane and the page.
template <int BITS, int G>
__device__ __forceinline__ void quantize_body(const Dims& d, int64_t u, int32_t group_index, const QuantLds<G>& L,
                                              uint8_t flag, uint8_t* __restrict__ k_codes,
                                              uint32_t* __restrict__ k_meta, uint8_t* __restrict__ v_codes,
                                              uint32_t* __restrict__ v_meta, uint32_t* __restrict__ mask, int tid) {
  unsigned char* sk = L.sk;
  unsigned char* sv = L.sv;
  float2* skm = L.skm;
  float2* svm = L.svm;
  uint8_t* ssel = L.ssel;
  const int gv_shift = 31 - __clz(d.Gv);             // Gv is a power of two
  if (tid < G) ssel[tid] = flag;
  const int any = __syncthreads_or(flag);

  // mean replacement: per-channel mean of the original rows of all G tokens, exact fp64 sum,
  // scaled by the power of two 1/G, rounded to fp32 then fp16.
  if (any) {
    // four adjacent lanes per (matrix, channel), each summing every fourth token (the adds are exact,
    // so the split changes nothing), then each replacing the flagged ones among its own tokens
    const int part = tid & 3, c = (tid >> 2) & 127;
    unsigned char* rows = (tid < 512) ? sk : sv;
    double sum = 0.0;
#pragma unroll 8
    for (int t = part; t < G; t += 4) sum += (double)half_at(rows + t * kRowB + 2 * c);
    sum += row_partner<0>(sum);
    sum += row_partner<1>(sum);
    const float m32 = (float)(sum / (double)G);
    const __half m16 = __float2half_rn(m32);
    for (int t = part; t < G; t += 4)
      if (ssel[t]) *(__half*)(rows + t * kRowB + 2 * c) = m16;
    __syncthreads();
  }

  // K meta: 8 adjacent lanes share a channel, each taking every 8th token.
  {
    const int c = tid >> 3, part = tid & 7;
    float mn = half_at(sk + part * kRowB + 2 * c), mx = mn;
#pragma unroll
    for (int t = part + 8; t < G; t += 8) {
      const float x = half_at(sk + t * kRowB + 2 * c);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    team_minmax(mn, mx, 8);
    mn += 0.0f;                                        // a zero minimum is stored as +0 (-0 + +0 = +0)
    if (part == 0) {
      const __half st = step_of(mn, mx, BITS);
      skm[c] = make_float2(mn, half_step_of(st));      // (mn is an fp16 value)
      // global layout of a group's Key meta: fp16 step[128], then fp16 zero[128]
      __half* gm = (__half*)(k_meta + (u * d.groups_per_unit + group_index) * kHeadDim);
      gm[c] = st;
      gm[kHeadDim + c] = __float2half_rn(mn);
    }
  }
  // V meta: Gv / 8 adjacent lanes share a (token, channel group), 8 channels each.
  if (!d.keys_only) {
    const int lanes = d.Gv >> 3;                       // 4, 8 or 16
#pragma unroll 1
    for (int e = tid; e < G * 16; e += kQuantThreads) {
      const int t = e >> 4, c8 = e & 15;               // 8 channels from 8 * c8 on
      const uint4 w = *(const uint4*)(sv + t * kRowB + c8 * 16);
      const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
      float mn = lo_half(ww[0]), mx = mn;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float x0 = lo_half(ww[k]), x1 = hi_half(ww[k]);
        mn = fminf(mn, fminf(x0, x1));
        mx = fmaxf(mx, fmaxf(x0, x1));
      }
      team_minmax(mn, mx, lanes);
      mn += 0.0f;                                      // a zero minimum is stored as +0
      if ((c8 & (lanes - 1)) == 0) {
        const int j = (c8 * 8) >> gv_shift;
        const __half st = step_of(mn, mx, BITS);
        svm[j * G + t] = make_float2(mn, half_step_of(st));
        // global layout of a 32-token block's Value meta (NV = value groups per token):
        // fp16 step[16 token pairs][NV][2], then fp16 zero[16 token pairs][NV][2]
        const int64_t tok = (int64_t)group_index * G + t;
        const int tb = (int)(tok & 31);
        __half* gm = (__half*)(v_meta + (u * d.blocks_per_unit + (tok >> 5)) * 32 * d.vgroups);
        gm[((tb >> 1) * d.vgroups + j) * 2 + (tb & 1)] = st;
        gm[32 * d.vgroups + ((tb >> 1) * d.vgroups + j) * 2 + (tb & 1)] = __float2half_rn(mn);
      }
    }
  }
  __syncthreads();

  // codes: one field (8 codes) of one packed u32 word of K or V per thread step.  Word w of lane l
  // of block blk holds 4/BITS fields; with two fields per word, adjacent lanes hold them.
  constexpr int kWordsPerBlock = 128 * BITS;          // 512*BITS bytes / 4
  constexpr int kFieldsPerWord = 4 / BITS;            // 2 (2-bit) or 1 (4-bit)
  constexpr int nblk = G / kBlockTokens;
  constexpr int kItems = 2 * nblk * kWordsPerBlock * kFieldsPerWord;   // a multiple of 1024
  const int first_block = group_index * nblk;
  const int n_items = d.keys_only ? kItems / 2 : kItems;          // Key words first, then Value words
#pragma unroll 1
  for (int e = tid; e < n_items; e += kQuantThreads) {
    const int kv = e / (kItems / 2);
    const int wf = e % (kItems / 2);
    const int i = wf / kFieldsPerWord, ff = wf % kFieldsPerWord;
    const int blk = i / kWordsPerBlock;
    const int wi = i - blk * kWordsPerBlock;
    // invert word_byte(): byte = 4*wi
    int lane, f0;
    if (BITS == 2) {
      lane = wi >> 2;
      f0 = (wi & 3) * 2;
    } else {
      const int half = wi >> 8;                        // 256 words per 1 KiB half
      lane = (wi & 255) >> 2;
      f0 = half * 4 + (wi & 3);
    }
    const int r = lane >> 4, mn_ = lane & 15;
    const int f = f0 + ff;
    // the word as if the field were the first of its word; the second field of a 2-bit word sits 8 bits up
    uint32_t word = 0;
    float2 ms[8];
    float val[8];
    if (kv == 0) {  // Key: lane = 16 r + m, field = 4 th + cb: 8 consecutive channels of one token
      const int t = 16 * (f >> 2) + mn_;
      const int c0 = 32 * (f & 3) + 8 * r;
      const uint4 xv = *(const uint4*)(sk + (blk * kBlockTokens + t) * kRowB + 2 * c0);
      const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int x = 0; x < 8; x += 2) {
        const float4 m2 = *(const float4*)(skm + c0 + x);
        ms[x] = make_float2(m2.x, m2.y);
        ms[x + 1] = make_float2(m2.z, m2.w);
      }
#pragma unroll
      for (int x = 0; x < 8; ++x) val[x] = (x & 1) ? hi_half(xs[x >> 1]) : lo_half(xs[x >> 1]);
    } else {        // Value: lane = 16 r + n, field = ct: one channel of 8 consecutive tokens
      const int c = 16 * f + mn_;
      const int t0 = blk * kBlockTokens + 8 * r;
      const float2* pm = svm + (c >> gv_shift) * G + t0;
#pragma unroll
      for (int x = 0; x < 8; x += 2) {
        const float4 m2 = *(const float4*)(pm + x);
        ms[x] = make_float2(m2.x, m2.y);
        ms[x + 1] = make_float2(m2.z, m2.w);
      }
#pragma unroll
      for (int x = 0; x < 8; ++x) val[x] = half_at(sv + (t0 + x) * kRowB + 2 * c);
    }
#pragma unroll
    for (int x = 0; x < 8; ++x)
      word |= place_twice<BITS>(quant_code_twice<BITS>(val[x], ms[x].x, ms[x].y), code_bit(BITS, 0, x));
    if (ff) word = (word << 8) | (word >> 24);
    if (kFieldsPerWord == 2) word |= row_partner_u32<0>(word);      // the word's other field (the adjacent lane)
    if (ff == 0) {
      const int64_t boff = (u * d.blocks_per_unit + first_block + blk) * (int64_t)d.block_bytes;
      ((uint32_t*)((kv ? v_codes : k_codes) + boff))[wi] = word;
    }
  }

  // mask words
  if (tid < nblk) {
    uint32_t w = 0;
    for (int t = 0; t < 32; ++t) w |= (ssel[tid * 32 + t] ? 1u : 0u) << t;
    mask[u * d.blocks_per_unit + first_block + tid] = w;
  }
}

// One workgroup of 16 wavefronts per unit.  Every global load of the kernel is issued before the
// first wait, so a launch costs one trip to memory; the work after it is spread over all 1024
// threads because nothing else hides latency.  LDS: 2 * G * 272 bytes (<= 68 KB) + meta.
template <int BITS, int G>
__global__ void __launch_bounds__(kQuantThreads) quantize_kernel(
    Dims d, int32_t group_index, const __half* __restrict__ k_group, const __half* __restrict__ v_group,
    int64_t unit_stride, const uint8_t* __restrict__ selected, int64_t selected_unit_stride,
    uint8_t* __restrict__ k_codes, uint32_t* __restrict__ k_meta, uint8_t* __restrict__ v_codes,
    uint32_t* __restrict__ v_meta, uint32_t* __restrict__ mask, int32_t n_groups, int32_t tail_n,
    __half* __restrict__ k_res, __half* __restrict__ v_res) {
  // grid (units, groups + tail blocks): workgroup (ul, gy) with gy < n_groups quantizes the G rows from row
  // gy * G of the unit's rows as group group_index + gy; its flags are
  // selected[ul * selected_unit_stride + gy * G ..].  The workgroups behind them copy the tail_n rows that
  // follow the last group into ring rows 0 .. of the unit (a whole prompt: the rows that stay in full
  // precision), 16 bytes of K and of V per thread.
  extern __shared__ __align__(16) unsigned char smem[];
  const QuantLds<G> L(smem, d.vgroups);
  const int tid = threadIdx.x;
  const int ul = blockIdx.x, gy = blockIdx.y;
  if (gy >= n_groups) {
    const int i = (gy - n_groups) * kQuantThreads + tid;
    if (i < tail_n * 16) {
      const int64_t src = (int64_t)ul * unit_stride + (int64_t)n_groups * G * kHeadDim;
      const int64_t dst = (d.unit0 + ul) * d.res_rows * kHeadDim;
      ((uint4*)(k_res + dst))[i] = ((const uint4*)(k_group + src))[i];
      ((uint4*)(v_res + dst))[i] = ((const uint4*)(v_group + src))[i];
    }
    return;
  }
  GroupRows<G> rows;
  const int64_t row0 = (int64_t)ul * unit_stride + (int64_t)gy * G * kHeadDim;
  rows_issue<G>(rows, k_group + row0, v_group + row0, tid);
  uint8_t flag = 0;
  if (tid < G && selected) flag = selected[(int64_t)ul * selected_unit_stride + gy * G + tid];
  const GroupPlace at = place_of_group(d, ul, group_index + gy);
  rows_to_lds<G>(rows, L, tid);
  quantize_body<BITS, G>(d, at.row, at.slot, L, flag, k_codes, k_meta, v_codes, v_meta, mask, tid);
}

// ---- many groups per launch (a prompt): one workgroup of two wavefronts per group -------------------------
// The kernel above spreads one group over 1024 threads because a decode step waits for it.  A prompt has
// thousands of groups, and what counts is the instructions spent per group.  Here wavefront 0 quantizes the
// group's Keys and wavefront 1 its Values, each with a lane-to-element mapping in which the packed words fall
// out of the lanes that computed the codes:
//   Keys:   a lane owns one channel pair for all tokens, so minimum and maximum over the tokens are packed
//           fp16 operations inside the lane (exact: they only select).  The 8 (2-bit) or 4 (4-bit) lanes
//           whose codes share a packed word are adjacent (for 2-bit the lanes are numbered accordingly) and
//           combine it with 3 or 2 cross-lane ORs; over 8 or 4 tokens each of them keeps one word, then all
//           store.
//   Values: minimum and maximum per (token, channel group) with 8 channels per lane and a butterfly over
//           Gv / 8 lanes on the packed pair {min, -max}; the rows and their {zero, step / 2} then go through
//           LDS into the mapping in which a lane owns the two channels of one packed word for 8 tokens.
// Results are those of quantize_body bit for bit (same roundings in the same order; minimum, maximum and
// the exact fp64 sums do not depend on the order they are taken in).
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ h2 as_h2(uint32_t w) { return __builtin_bit_cast(h2, w); }
__device__ __forceinline__ uint32_t as_u32(h2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ uint32_t rotl32(uint32_t w, int n) { return __builtin_amdgcn_alignbit(w, w, (32 - n) & 31); }
__device__ __forceinline__ uint32_t half_bits(float x) { return (uint32_t)__half_as_ushort(__float2half_rn(x)); }
__device__ __forceinline__ uint32_t mean_half_bits(double sum, int G) { return half_bits((float)(sum / (double)G)); }
__device__ __forceinline__ void lds_order() {   // LDS traffic of one wavefront executes in order; this holds the compiler to it
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int BITS, int G>
__global__ void __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(4, 8))) prompt_quantize_kernel(
    Dims d, int32_t group_index, const __half* __restrict__ k_rows, const __half* __restrict__ v_rows,
    int64_t unit_stride, const uint8_t* __restrict__ selected, int64_t selected_unit_stride,
    uint8_t* __restrict__ k_codes, uint32_t* __restrict__ k_meta, uint8_t* __restrict__ v_codes,
    uint32_t* __restrict__ v_meta, uint32_t* __restrict__ mask, int32_t n_groups, int32_t tail_n,
    __half* __restrict__ k_res, __half* __restrict__ v_res) {
  // grid (units, groups + tail blocks), as quantize_kernel's
  __shared__ uint4 vrow[32 * 16];                      // 32 Value rows of 128 fp16 (mean-replaced where flagged)
  __shared__ float2 vms[32 * 4];                       // their {zero, step / 2} per channel group
  __shared__ uint32_t vpr[32 * 4];                     // and before that {minimum, -maximum} as an fp16 pair
  const int tid = threadIdx.x;
  const int ul = blockIdx.x, gy = blockIdx.y;
  if (gy >= n_groups) {
    const int i = (gy - n_groups) * 128 + tid;
    if (i < tail_n * 16) {
      const int64_t src = (int64_t)ul * unit_stride + (int64_t)n_groups * G * kHeadDim;
      const int64_t dst = (d.unit0 + ul) * d.res_rows * kHeadDim;
      ((uint4*)(k_res + dst))[i] = ((const uint4*)(k_rows + src))[i];
      ((uint4*)(v_res + dst))[i] = ((const uint4*)(v_rows + src))[i];
    }
    return;
  }
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row0 = (int64_t)ul * unit_stride + (int64_t)gy * G * kHeadDim;
  const GroupPlace at = place_of_group(d, ul, group_index + gy);
  constexpr int nblk = G / kBlockTokens;
  const int64_t block0 = at.row * d.blocks_per_unit + (int64_t)at.slot * nblk;   // the group's first packed block
  // the flags of the group's tokens as bit masks (uniform)
  constexpr int kSelWords = (G + 63) / 64;
  unsigned long long sel[kSelWords];
  bool any = false;
#pragma unroll
  for (int w = 0; w < kSelWords; ++w) {
    const int t = 64 * w + lane;
    const bool f = selected && t < G && selected[(int64_t)ul * selected_unit_stride + (int64_t)gy * G + t] != 0;
    sel[w] = __ballot(f);
    any |= sel[w] != 0;
  }
  auto is_sel = [&](int t) -> bool { return (sel[kSelWords == 1 ? 0 : t >> 6] >> (t & 63)) & 1ull; };

  if (wave == 0) {
    // ---- Keys ------------------------------------------------------------------------------------------
    const int v = lane & 3;
    int cp, r, hi = 0, p = 0, cb = 0;                  // cp: the lane's channel pair (channels 2 cp, 2 cp + 1)
    if (BITS == 2) {
      hi = lane >> 5, r = (lane >> 3) & 3, p = (lane >> 2) & 1;
      cp = 16 * (2 * hi + p) + 4 * r + v;
    } else {
      cp = lane, cb = lane >> 4, r = (lane >> 2) & 3;
    }
    const uint32_t* kr = (const uint32_t*)(k_rows + row0) + cp;        // token t: kr[64 t]
    // Where the lane's two codes of a token sit in the packed word: bit pos0 (channel 2 cp) and pos0 + 16
    // (channel 2 cp + 1), the whole turned left by 8 for the odd fields of a 2-bit word.
    const int pos0 = BITS == 2 ? 2 * (v + 1) : 2 + 4 * (v & 1) + 8 * (v >> 1);
    const int turn = BITS == 2 ? 8 * p : 0;
    const uint32_t bit_a0 = rotl32(1u << pos0, turn), bit_a1 = rotl32(2u << pos0, turn);         // 2-bit codes: their
    const uint32_t bit_b0 = rotl32(1u << (pos0 + 16), turn), bit_b1 = rotl32(2u << (pos0 + 16), turn);   // two bits each
    constexpr int J = BITS == 2 ? 8 : 4;               // lanes that share a word
    const int j = lane & (J - 1);
    auto keys = [&](auto any_c) {
      constexpr bool ANY = decltype(any_c)::value;     // some token of the group is flagged (uniform)
      uint32_t y[32];
      h2 mn = {(_Float16)__builtin_inff(), (_Float16)__builtin_inff()};
      h2 mx = {(_Float16)(-__builtin_inff()), (_Float16)(-__builtin_inff())};
      double s0 = 0.0, s1 = 0.0;
#pragma unroll 1
      for (int blk = 0; blk < nblk; ++blk) {
#pragma unroll
        for (int t = 0; t < 32; ++t) y[t] = kr[(blk * 32 + t) * 64];
#pragma unroll
        for (int t = 0; t < 32; ++t) {
          const h2 x = as_h2(y[t]);
          if (ANY) {
            const bool s = is_sel(blk * 32 + t);
            mn = s ? mn : __builtin_elementwise_min(mn, x);
            mx = s ? mx : __builtin_elementwise_max(mx, x);
          } else {
            mn = __builtin_elementwise_min(mn, x);
            mx = __builtin_elementwise_max(mx, x);
          }
        }
        if (ANY) {                                     // the exact sums of ALL rows as they came (two chains of
#pragma unroll                                         // dependent additions: few conversions in flight at a time)
          for (int t = 0; t < 32; ++t) {
            s0 += (double)lo_half(y[t]);
            asm volatile("" : "+v"(s0));
            s1 += (double)hi_half(y[t]);
            asm volatile("" : "+v"(s1));
          }
        }
      }
      uint32_t mean = 0;
      if (ANY) {
        mean = mean_half_bits(s0, G) | (mean_half_bits(s1, G) << 16);
        mn = __builtin_elementwise_min(mn, as_h2(mean));
        mx = __builtin_elementwise_max(mx, as_h2(mean));
      }
      const float mn0 = (float)mn[0] + 0.0f, mn1 = (float)mn[1] + 0.0f;   // a zero minimum is stored as +0
      const __half st0 = step_of(mn0, (float)mx[0], BITS), st1 = step_of(mn1, (float)mx[1], BITS);
      const float h0 = half_step_of(st0), h1 = half_step_of(st1);
      {
        uint32_t* gm = k_meta + (at.row * d.groups_per_unit + at.slot) * kHeadDim;   // fp16 step[128], then zero[128]
        gm[cp] = (uint32_t)__half_as_ushort(st0) | ((uint32_t)__half_as_ushort(st1) << 16);
        gm[64 + cp] = half_bits(mn0) | (half_bits(mn1) << 16);
      }
      // 2-bit: the thresholds (2k - 1) h themselves (exact: h has 11 bits)
      const float h0x3 = 3.0f * h0, h0x5 = 5.0f * h0, h1x3 = 3.0f * h1, h1x5 = 5.0f * h1;
#pragma unroll 1
      for (int blk = 0; blk < nblk; ++blk) {
        if (nblk > 1) {
#pragma unroll
          for (int t = 0; t < 32; ++t) y[t] = kr[(blk * 32 + t) * 64];
        }
        uint8_t* kb = k_codes + (block0 + blk) * (int64_t)d.block_bytes;
        if (ANY) {                                     // the flagged rows become the mean row
#pragma unroll
          for (int t = 0; t < 32; ++t) y[t] = is_sel(blk * 32 + t) ? mean : y[t];
        }
        uint32_t keep = 0;
#pragma unroll
        for (int t = 0; t < 32; ++t) {
          const uint32_t x = y[t];
          uint32_t w;
          if (BITS == 2) {
            // code = [t >= 3h] * 2 + [t >= (5h if so, else h)]: the number of thresholds h, 3h, 5h reached
            const float ta = lo_half(x) - mn0, tb = hi_half(x) - mn1;
            const bool a1 = ta >= h0x3, b1 = tb >= h1x3;
            const bool a0 = ta >= (a1 ? h0x5 : h0), b0 = tb >= (b1 ? h1x5 : h1);
            w = (a1 ? bit_a1 : 0u) | (a0 ? bit_a0 : 0u) | (b1 ? bit_b1 : 0u) | (b0 ? bit_b0 : 0u);
          } else {
            const uint32_t ca = (uint32_t)quant_code_twice<BITS>(lo_half(x), mn0, h0);   // 2 * code
            const uint32_t cb2 = (uint32_t)quant_code_twice<BITS>(hi_half(x), mn1, h1);
            w = (ca << (pos0 - 1)) | rotl32(cb2 << (pos0 - 1), 16);
          }
          w |= row_partner_u32<0>(w);
          w |= row_partner_u32<1>(w);
          if (BITS == 2) w |= row_partner_u32<2>(w);
          keep = (t & (J - 1)) == j ? w : keep;
          if ((t & (J - 1)) == J - 1) {                // every lane now holds the word of token t - (J - 1) + j
            const int tt = t - (J - 1) + j, m = tt & 15, th = tt >> 4;
            const int byte = BITS == 2 ? 16 * (16 * r + m) + 4 * (2 * th + hi) : 1024 * th + 16 * (16 * r + m) + 4 * cb;
            *(uint32_t*)(kb + byte) = keep;
          }
        }
        if (lane == 0) {
          const uint32_t mw = (uint32_t)(sel[kSelWords == 1 ? 0 : (blk * 32) >> 6] >> ((blk * 32) & 63));
          mask[block0 + blk] = mw;
        }
      }
    };
    if (any) keys(std::true_type{});
    else keys(std::false_type{});
    return;
  }

  // ---- Values ----------------------------------------------------------------------------------------------
  const int gv_shift = 31 - __clz(d.Gv);
  const int lanes = d.Gv >> 3;                          // lanes per (token, channel group) in the first mapping
  const int NV = d.vgroups;
  const int nv_shift = NV == 4 ? 2 : NV == 2 ? 1 : 0;
  const int t4 = lane >> 4, c16 = lane & 15;            // first mapping: token 4 i + t4, channels 8 c16 .. + 7
  const __half* vr = v_rows + row0 + 8 * c16;
  const int n = lane & 15, q = lane >> 4;               // second mapping: channels 32 q + n and 32 q + 16 + n
  const int jq = (32 * q) >> gv_shift;                  // their channel group
  auto values = [&](auto any_c) {
    constexpr bool ANY = decltype(any_c)::value;
    uint32_t mean4[4] = {0u, 0u, 0u, 0u};
    if (ANY) {                                          // per-channel means of the group's Value rows, exact
      double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
      for (int t = t4; t < G; t += 4) {
        const uint4 w = *(const uint4*)(vr + t * kHeadDim);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[2 * k] += (double)lo_half(ww[k]);
          acc[2 * k + 1] += (double)hi_half(ww[k]);
        }
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        acc[k] += __shfl_xor(acc[k], 16);
        acc[k] += __shfl_xor(acc[k], 32);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) mean4[k] = mean_half_bits(acc[2 * k], G) | (mean_half_bits(acc[2 * k + 1], G) << 16);
    }
#pragma unroll 1
    for (int blk = 0; blk < nblk; ++blk) {
      uint4 w[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) w[i] = *(const uint4*)(vr + (blk * 32 + 4 * i + t4) * kHeadDim);
      lds_order();                                      // the previous block's reads are done
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = 4 * i + t4, T = blk * 32 + t;
        if (ANY && ((sel[kSelWords == 1 ? 0 : T >> 6] >> (T & 63)) & 1ull))
          w[i] = make_uint4(mean4[0], mean4[1], mean4[2], mean4[3]);
        const h2 a = __builtin_elementwise_min(__builtin_elementwise_min(as_h2(w[i].x), as_h2(w[i].y)),
                                               __builtin_elementwise_min(as_h2(w[i].z), as_h2(w[i].w)));
        const h2 b = __builtin_elementwise_max(__builtin_elementwise_max(as_h2(w[i].x), as_h2(w[i].y)),
                                               __builtin_elementwise_max(as_h2(w[i].z), as_h2(w[i].w)));
        // the two halves against each other with the same instructions (they order -0 below +0, as the
        // scalar minimum and maximum of the other kernel do; a comparison would not)
        const h2 a2 = __builtin_elementwise_min(a, as_h2(rotl32(as_u32(a), 16)));
        const h2 b2 = __builtin_elementwise_max(b, as_h2(rotl32(as_u32(b), 16)));
        h2 pr = {a2[0], (_Float16)(-b2[0])};            // {min, -max}: one packed minimum reduces both
        pr = __builtin_elementwise_min(pr, as_h2(row_partner_u32<0>(as_u32(pr))));
        pr = __builtin_elementwise_min(pr, as_h2(row_partner_u32<1>(as_u32(pr))));
        if (lanes > 4) pr = __builtin_elementwise_min(pr, as_h2(row_partner_u32<2>(as_u32(pr))));
        if (lanes > 8) pr = __builtin_elementwise_min(pr, as_h2(row_partner_u32<3>(as_u32(pr))));
        vrow[t * 16 + c16] = w[i];
        if ((c16 & (lanes - 1)) == 0) vpr[t * 4 + ((8 * c16) >> gv_shift)] = as_u32(pr);
      }
      lds_order();
      // steps and zeros of the block's 32 NV (token, channel group) pairs: one lane per (token pair, group),
      // which is also one dword of each half of the block's meta (fp16 step[16 token pairs][NV][2], then
      // fp16 zero[16 token pairs][NV][2])
      if (lane < 16 * NV) {
        const int tp = lane >> nv_shift, jv = lane & (NV - 1);
        uint32_t stw = 0, zw = 0;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          const h2 pr = as_h2(vpr[(2 * tp + k) * 4 + jv]);
          const float mnf = (float)pr[0] + 0.0f, mxf = -(float)pr[1];
          const __half st = step_of(mnf, mxf, BITS);
          vms[(2 * tp + k) * 4 + jv] = make_float2(mnf, half_step_of(st));
          stw |= (uint32_t)__half_as_ushort(st) << (16 * k);
          zw |= half_bits(mnf) << (16 * k);
        }
        uint32_t* gm = v_meta + (block0 + blk) * 32 * NV;
        gm[lane] = stw;
        gm[16 * NV + lane] = zw;
      }
      lds_order();
      uint8_t* vb = v_codes + (block0 + blk) * (int64_t)d.block_bytes;
      const __half* rows = (const __half*)vrow;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        uint32_t wa = 0, wb = 0;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const int t = 8 * r + x;
          const float2 ms = vms[t * 4 + jq];
          const _Float16 ha = ((const _Float16*)rows)[t * kHeadDim + 32 * q + n];
          const _Float16 hb = ((const _Float16*)rows)[t * kHeadDim + 32 * q + 16 + n];
          const float xa = (float)ha, xb = (float)hb;
          if (BITS == 2) {
            constexpr uint32_t one = 1u;
            const int pos = code_bit(2, 0, x);          // at most 24: both bits fit
            const float ta = xa - ms.x, tb = xb - ms.x, h3 = 3.0f * ms.y, h5 = 5.0f * ms.y;
            const bool a1 = ta >= h3, b1 = tb >= h3;
            const bool a0 = ta >= (a1 ? h5 : ms.y), b0 = tb >= (b1 ? h5 : ms.y);
            wa |= (a1 ? one << (pos + 1) : 0u) | (a0 ? one << pos : 0u);
            wb |= (b1 ? one << (pos + 1) : 0u) | (b0 ? one << pos : 0u);
          } else {
            wa |= place_twice<BITS>(quant_code_twice<BITS>(xa, ms.x, ms.y), code_bit(BITS, 0, x));
            wb |= place_twice<BITS>(quant_code_twice<BITS>(xb, ms.x, ms.y), code_bit(BITS, 0, x));
          }
        }
        if (BITS == 2) {                                // fields 2 q and 2 q + 1: word q of the packed lane, the odd field 8 bits up
          ((uint32_t*)(vb + 16 * (16 * r + n)))[q] = wa | rotl32(wb, 8);
        } else {                                        // words 2 (q & 1), 2 (q & 1) + 1 of half q >> 1
          *(uint2*)(vb + 1024 * (q >> 1) + 16 * (16 * r + n) + 8 * (q & 1)) = make_uint2(wa, wb);
        }
      }
    }
  };
  if (any) values(std::true_type{});
  else values(std::false_type{});
}

// Rows n0 .. n0 + n - 1 of every unit's rows into ring rows 0 .. n - 1 (16 bytes per thread).
__global__ void __launch_bounds__(256) tail_copy_kernel(Dims d, const __half* __restrict__ k_rows,
                                                        const __half* __restrict__ v_rows, int64_t unit_stride,
                                                        int32_t n0, int32_t n, __half* __restrict__ k_res,
                                                        __half* __restrict__ v_res) {
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  const uint4* sk = (const uint4*)(k_rows + (int64_t)ul * unit_stride + (int64_t)n0 * kHeadDim);
  const uint4* sv = (const uint4*)(v_rows + (int64_t)ul * unit_stride + (int64_t)n0 * kHeadDim);
  uint4* dk = (uint4*)(k_res + u * d.res_rows * kHeadDim);
  uint4* dv = (uint4*)(v_res + u * d.res_rows * kHeadDim);
  for (int i = blockIdx.y * 256 + threadIdx.x; i < n * 16; i += gridDim.y * 256) {
    dk[i] = sk[i];
    dv[i] = sv[i];
  }
}

// The whole group step of one unit in one launch: append the new token's row to the ring, run the
// outlier competition on the oldest G rows, quantize them.  The ring must be full after the
// append (R + G rows), its oldest G rows starting at ring row `group_row0`.
template <int BITS, int G>
__global__ void __launch_bounds__(kQuantThreads) group_step_kernel(
    Dims d, int32_t group_index, const __half* __restrict__ k_new, const __half* __restrict__ v_new, __half* k_res,
    __half* v_res, int32_t append_row, int32_t group_row0, const int32_t* __restrict__ seq, __half* pool_k,
    __half* pool_v, int32_t* pool_idx,
    double* pool_score, int32_t* pool_count, int32_t* aux_count, int32_t* frozen, uint8_t* selected,
    uint8_t* __restrict__ k_codes, uint32_t* __restrict__ k_meta, uint8_t* __restrict__ v_codes,
    uint32_t* __restrict__ v_meta, uint32_t* __restrict__ mask) {
  extern __shared__ __align__(16) unsigned char smem[];
  const QuantLds<G> L(smem, d.vgroups);
  const int tid = threadIdx.x;
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  __half* kring = k_res + u * d.res_rows * kHeadDim;
  __half* vring = v_res + u * d.res_rows * kHeadDim;
  bool close_group = true;
  if (seq) {
    // A batch of sequences of different lengths: the unit's sequence says where its new row goes
    // and whether its ring is full with it.  A sequence that is inactive, or whose state does not
    // fit the buffers, is left alone; all of this is uniform over the workgroup.
    const int4 own = *(const int4*)(seq + 4 * (ul / d.kv_heads));
    const int nq = own.x, rs = own.y, nr = own.z;
    if (!own.w || nq < 0 || rs < 0 || rs >= d.res_rows || nr < 0 || nr >= d.res_rows) return;
    append_row = rs + nr;
    append_row -= append_row >= d.res_rows ? d.res_rows : 0;
    group_row0 = rs;
    group_index = nq / G;
    close_group = nr + 1 == d.R + G && rs % G == 0 && nq % G == 0 && nq + G <= d.max_seq;
  }
  if (tid < 128) {                                   // the new row: 64 threads for K, 64 for V, 4 bytes each
    const int which = tid >> 6, lane = tid & 63;
    const uint32_t* src = (const uint32_t*)((which ? v_new : k_new) + (int64_t)ul * kHeadDim);
    ((uint32_t*)((which ? vring : kring) + append_row * kHeadDim))[lane] = src[lane];
  }
  if (!close_group) return;
  const GroupPlace at = place_of_group(d, ul, group_index);        // where the group's codes and meta go
  if (append_row >= group_row0 && append_row < group_row0 + G) {   // R = 0: the new token closes the group
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  const __half* gk = kring + group_row0 * kHeadDim;
  const __half* gv = vring + group_row0 * kHeadDim;
  GroupRows<G> rows;
  rows_issue<G>(rows, gk, gv, tid);
  uint8_t* sel = selected ? selected + (int64_t)ul * G : nullptr;
  if (d.N > 0) {
    const trace_core::UnitPool p =
        trace_core::unit_pool(d, u, pool_k, pool_v, pool_idx, pool_score, pool_count, aux_count, frozen);
    trace_core::Loaded<G> in;
    const bool ahead = d.N <= trace_core::kPoolRowsAhead;
    trace_core::load<G>(in, d, p, gk, tid, ahead);
    rows_to_lds<G>(rows, L, tid);
    trace_core::compete<G>(in, d, group_index, p, gk, gv, sel, L.ssel, tid, L.sk, L.sv, kRowB, ahead);
  } else {
    rows_to_lds<G>(rows, L, tid);
    if (tid < G) {
      L.ssel[tid] = 0;
      if (sel) sel[tid] = 0;
    }
  }
  __syncthreads();                                   // the flags are in LDS
  const uint8_t flag = tid < G ? L.ssel[tid] : (uint8_t)0;
  quantize_body<BITS, G>(d, at.row, at.slot, L, flag, k_codes, k_meta, v_codes, v_meta, mask, tid);
}

template <int BITS, int G>
hipError_t launch_quantize_one(const Dims& d, int32_t group_index, int32_t n_groups, const __half* k_group,
                               const __half* v_group, int64_t unit_stride, const uint8_t* selected,
                               int64_t selected_unit_stride, const kvq_qcache& qc, int32_t tail_n, __half* k_res,
                               __half* v_res, hipStream_t s) {
  // many groups (a prompt): the kernel that spends the fewest instructions per group; few: the one that is
  // done with a group soonest
  if ((int64_t)d.units_per_layer * n_groups >= kPromptGroups && !d.keys_only) {
    const int tail_blocks = (tail_n * 16 + 127) / 128;
    hipLaunchKernelGGL((prompt_quantize_kernel<BITS, G>), dim3(d.units_per_layer, n_groups + tail_blocks), dim3(128), 0,
                       s, d, group_index, k_group, v_group, unit_stride, selected, selected_unit_stride,
                       (uint8_t*)qc.k_codes, (uint32_t*)qc.k_meta, (uint8_t*)qc.v_codes, (uint32_t*)qc.v_meta,
                       (uint32_t*)qc.mask, n_groups, tail_n, k_res, v_res);
    return hipGetLastError();
  }
  const size_t smem = quant_lds_bytes<G>(d.vgroups);
  if (smem > 48 * 1024) {  // more than the default limit of dynamic LDS per workgroup
    hipError_t e = hipFuncSetAttribute((const void*)quantize_kernel<BITS, G>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
    if (e != hipSuccess) return e;
  }
  const int tail_blocks = (tail_n * 16 + kQuantThreads - 1) / kQuantThreads;
  hipLaunchKernelGGL((quantize_kernel<BITS, G>), dim3(d.units_per_layer, n_groups + tail_blocks), dim3(kQuantThreads),
                     smem, s, d, group_index, k_group, v_group, unit_stride, selected, selected_unit_stride,
                     (uint8_t*)qc.k_codes, (uint32_t*)qc.k_meta, (uint8_t*)qc.v_codes, (uint32_t*)qc.v_meta,
                     (uint32_t*)qc.mask, n_groups, tail_n, k_res, v_res);
  return hipGetLastError();
}

template <int BITS>
hipError_t launch_quantize_bits(const Dims& d, int32_t group_index, int32_t n_groups, const __half* k_group,
                                const __half* v_group, int64_t unit_stride, const uint8_t* selected,
                                int64_t selected_unit_stride, const kvq_qcache& qc, int32_t tail_n, __half* k_res,
                                __half* v_res, hipStream_t s) {
  switch (d.G) {
    case 32: return launch_quantize_one<BITS, 32>(d, group_index, n_groups, k_group, v_group, unit_stride, selected, selected_unit_stride, qc, tail_n, k_res, v_res, s);
    case 64: return launch_quantize_one<BITS, 64>(d, group_index, n_groups, k_group, v_group, unit_stride, selected, selected_unit_stride, qc, tail_n, k_res, v_res, s);
    default: return launch_quantize_one<BITS, 128>(d, group_index, n_groups, k_group, v_group, unit_stride, selected, selected_unit_stride, qc, tail_n, k_res, v_res, s);
  }
}

}  // namespace

hipError_t launch_append(const Dims& d, const __half* k_new, const __half* v_new, __half* k_res, __half* v_res,
                         int32_t row, hipStream_t s) {
  hipLaunchKernelGGL(append_kernel, dim3(d.units_per_layer), dim3(128), 0, s, d, k_new, v_new, k_res, v_res, row);
  return hipGetLastError();
}

namespace {

template <int BITS, int G>
hipError_t launch_group_step_one(const Dims& d, int32_t group_index, const __half* k_new, const __half* v_new,
                                 __half* k_res, __half* v_res, int32_t append_row, int32_t group_row0,
                                 const int32_t* seq, const kvq_pool& pool, uint8_t* selected, const kvq_qcache& qc,
                                 hipStream_t s) {
  const size_t smem = quant_lds_bytes<G>(d.vgroups);
  if (smem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)group_step_kernel<BITS, G>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((group_step_kernel<BITS, G>), dim3(d.units_per_layer), dim3(kQuantThreads), smem, s, d,
                     group_index, k_new, v_new, k_res, v_res, append_row, group_row0, seq, (__half*)pool.pool_k,
                     (__half*)pool.pool_v, pool.pool_idx, pool.pool_score, pool.pool_count, pool.aux_count,
                     pool.frozen, selected, (uint8_t*)qc.k_codes, (uint32_t*)qc.k_meta, (uint8_t*)qc.v_codes,
                     (uint32_t*)qc.v_meta, (uint32_t*)qc.mask);
  return hipGetLastError();
}

template <int BITS>
hipError_t launch_group_step_bits(const Dims& d, int32_t group_index, const __half* k_new, const __half* v_new,
                                  __half* k_res, __half* v_res, int32_t append_row, int32_t group_row0,
                                  const int32_t* seq, const kvq_pool& pool, uint8_t* selected, const kvq_qcache& qc,
                                  hipStream_t s) {
  switch (d.G) {
    case 32: return launch_group_step_one<BITS, 32>(d, group_index, k_new, v_new, k_res, v_res, append_row, group_row0, seq, pool, selected, qc, s);
    case 64: return launch_group_step_one<BITS, 64>(d, group_index, k_new, v_new, k_res, v_res, append_row, group_row0, seq, pool, selected, qc, s);
    default: return launch_group_step_one<BITS, 128>(d, group_index, k_new, v_new, k_res, v_res, append_row, group_row0, seq, pool, selected, qc, s);
  }
}

}  // namespace

// ---- per-step Value quantization ---------------------------------------------------------------
// One workgroup of 128 threads (thread = channel) per unit; the tokens of the call one after the
// other.  Per token: minimum and maximum of each group of Gv channels, step and zero, codes (Eq. 2,
// the same device functions as the group quantization), the dequantized row back into the ring, the
// steps and zeros to their places in the block's meta, and the token's 2 or 4 bits of 64 or 128
// packed words replaced (the words also hold the block's other tokens of the same 8).
template <int BITS>
__global__ void __launch_bounds__(128) value_tokens_kernel(Dims d, int32_t first_token, int32_t count,
                                                           __half* __restrict__ v_res, int32_t ring_row,
                                                           uint8_t* __restrict__ v_codes,
                                                           uint32_t* __restrict__ v_meta) {
  constexpr int kLevels = (1 << BITS) - 1;
  constexpr int kWords = 32 * BITS;                     // packed words that hold one token's codes
  __shared__ float s_mn[2], s_mx[2];
  __shared__ uint32_t s_words[kWords];
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  const int c = threadIdx.x;                            // channel
  const int gv_shift = 31 - __clz(d.Gv);
  const int nblk_shift = d.bpg_shift;                   // blocks per Key group
  __half* ring = v_res + u * d.res_rows * kHeadDim;
  for (int i = 0; i < count; ++i) {
    const int tok = first_token + i;
    int row = ring_row + i;
    row -= row >= d.res_rows ? d.res_rows : 0;
    const float x = __half2float(ring[row * kHeadDim + c]);
    float mn = x, mx = x;
    const int team = d.Gv < 64 ? d.Gv : 64;
    for (int off = 1; off < team; off <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, off));
      mx = fmaxf(mx, __shfl_xor(mx, off));
    }
    if (d.Gv == 128) {                                  // the group spans both wavefronts
      if ((c & 63) == 0) {
        s_mn[c >> 6] = mn;
        s_mx[c >> 6] = mx;
      }
      __syncthreads();
      mn = fminf(s_mn[0], s_mn[1]);
      mx = fmaxf(s_mx[0], s_mx[1]);
    }
    mn += 0.0f;                                         // a zero minimum is stored as +0
    const __half st = step_of(mn, mx, BITS);
    const float stf = __half2float(st);
    const uint32_t code = quant_code(x, mn, stf, kLevels);
    const float prod = (float)code * stf;               // exact
    ring[row * kHeadDim + c] = __float2half_rn(mn + prod);
    // where the token's block is stored
    const GroupPlace at = place_of_group(d, ul, tok / d.G);
    const int64_t blk = at.row * d.blocks_per_unit + ((int64_t)at.slot << nblk_shift) + ((tok % d.G) >> 5);
    const int tb = tok & 31;
    if ((c & (d.Gv - 1)) == 0) {
      const int j = c >> gv_shift;
      __half* gm = (__half*)(v_meta + blk * 32 * d.vgroups);
      gm[((tb >> 1) * d.vgroups + j) * 2 + (tb & 1)] = st;
      gm[32 * d.vgroups + ((tb >> 1) * d.vgroups + j) * 2 + (tb & 1)] = __float2half_rn(mn);
    }
    // codes: channel c = 16 f + n of token tb = 8 r + xx lives in lane 16 r + n, field f, code xx
    const int n = c & 15, f = c >> 4, xx = tb & 7, r = tb >> 3;
    const int slot = BITS == 2 ? n * 4 + (f >> 1) : (f >> 2) * 64 + n * 4 + (f & 3);
    __syncthreads();                                    // the previous token's words have been used
    if (c < kWords) s_words[c] = 0;
    __syncthreads();
    atomicOr(&s_words[slot], place_code(code, code_bit(BITS, f, xx)));
    __syncthreads();
    if (c < kWords) {
      const int half = BITS == 2 ? 0 : c >> 6, nn = (c & 63) >> 2, w = c & 3;
      const uint32_t clear = BITS == 2 ? (place_code(3u, code_bit(2, 0, xx)) | place_code(3u, code_bit(2, 1, xx)))
                                       : place_code(15u, code_bit(4, 0, xx));
      uint32_t* gw = (uint32_t*)(v_codes + blk * d.block_bytes + 1024 * half + 16 * (16 * r + nn) + 4 * w);
      *gw = (*gw & ~clear) | s_words[c];
    }
  }
}

hipError_t launch_value_tokens(const Dims& d, int32_t first_token, int32_t count, __half* v_res, int32_t ring_row,
                               const kvq_qcache& qc, hipStream_t s) {
  if (d.bits == 2)
    hipLaunchKernelGGL(value_tokens_kernel<2>, dim3(d.units_per_layer), dim3(128), 0, s, d, first_token, count, v_res,
                       ring_row, (uint8_t*)qc.v_codes, (uint32_t*)qc.v_meta);
  else
    hipLaunchKernelGGL(value_tokens_kernel<4>, dim3(d.units_per_layer), dim3(128), 0, s, d, first_token, count, v_res,
                       ring_row, (uint8_t*)qc.v_codes, (uint32_t*)qc.v_meta);
  return hipGetLastError();
}

// The state of every active sequence after one token has been appended to it (and its oldest group
// quantized if that filled its ring): the rule group_step_kernel applies, applied to the array.
__global__ void seq_advance_kernel(Dims d, int32_t* seq) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= d.batch) return;
  int4 own = *(const int4*)(seq + 4 * b);
  if (!own.w || own.x < 0 || own.y < 0 || own.y >= d.res_rows || own.z < 0 || own.z >= d.res_rows) return;
  const bool close_group =
      own.z + 1 == d.R + d.G && own.y % d.G == 0 && own.x % d.G == 0 && own.x + d.G <= d.max_seq;
  own.z += 1;
  if (close_group) {
    own.x += d.G;
    own.z -= d.G;
    own.y += d.G;
    own.y -= own.y >= d.res_rows ? d.res_rows : 0;
  }
  *(int4*)(seq + 4 * b) = own;
}

// A launch plan for the decode attention of sequences of different lengths: `entries` workgroups per kv
// head are dealt to the sequences by the work each has (mini-chunks of quantized tokens, groups of
// full-precision rows at half a mini-chunk each), every sequence at least one; a sequence's workgroups
// share its mini-chunks equally.  The share m of one workgroup is the smallest for which the sequences'
// workgroups, ceil(work / m) each, are at most `entries` in all (found by bisection: that count does not
// grow with m).  One workgroup, one thread per sequence.
__global__ void __launch_bounds__(1024) seq_plan_kernel(Dims d, const int32_t* __restrict__ seq, int32_t max_nq,
                                                         int32_t max_nres, int32_t entries, int32_t* __restrict__ plan) {
  __shared__ int s_acc;
  __shared__ int s_wave[16];
  const int b = threadIdx.x;
  const bool live = b < d.batch;
  int nq = 0, rs = 0, nr = 0, w = 0, mc = 0;
  if (live) {
    const int4 own = *(const int4*)(seq + 4 * b);
    nq = min(max(own.x, 0), max_nq) & ~(kBlockTokens - 1);
    rs = (own.y >= 0 && own.y < d.res_rows) ? own.y & ~15 : 0;
    nr = min(max(own.z, 0), max_nres);
    mc = (nq + kMiniChunk - 1) / kMiniChunk;
    w = 2 * mc + ((nr + kFpGroupRows - 1) / kFpGroupRows) + ((d.pool_slots + kFpGroupRows - 1) / kFpGroupRows);
  }
  auto block_sum = [&](int v) {
    if (threadIdx.x == 0) s_acc = 0;
    __syncthreads();
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if ((threadIdx.x & 63) == 0) atomicAdd(&s_acc, v);
    __syncthreads();
    const int r = s_acc;
    __syncthreads();
    return r;
  };
  auto block_max = [&](int v) {
    if (threadIdx.x == 0) s_acc = 0;
    __syncthreads();
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
    if ((threadIdx.x & 63) == 0) atomicMax(&s_acc, v);
    __syncthreads();
    const int r = s_acc;
    __syncthreads();
    return r;
  };
  auto splits_for = [&](int m) { return live ? min(max((w + m - 1) / m, 1), max(mc, 1)) : 0; };
  int lo = 1, hi = max(block_max(w), 1);                // at m = hi every sequence has one workgroup: entries >= batch
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (block_sum(splits_for(mid)) <= entries) hi = mid;
    else lo = mid + 1;
  }
  const int sp = splits_for(lo);
  // exclusive prefix of the sequences' workgroup counts
  int incl = sp;
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if ((threadIdx.x & 63) >= off) incl += up;
  }
  if ((threadIdx.x & 63) == 63) s_wave[threadIdx.x >> 6] = incl;
  __syncthreads();
  int before = 0;
  for (int k = 0; k < (int)(threadIdx.x >> 6); ++k) before += s_wave[k];
  const int first = before + incl - sp;
  if (threadIdx.x == 1023) plan[0] = min(first + sp, entries);
  if (live) {
    const int per = (mc + sp - 1) / sp;                  // mini-chunks per workgroup of this sequence
    for (int k = 0; k < sp && first + k < entries; ++k) {
      int4* e = (int4*)(plan + 8 + 8 * (first + k));
      e[0] = make_int4(b, k, sp, min(k * per, mc));
      e[1] = make_int4(nq, rs, nr, min((k + 1) * per, mc));
    }
  }
}

hipError_t launch_seq_plan(const Dims& d, const int32_t* seq, int32_t max_n_quant, int32_t max_n_res, int32_t entries,
                           int32_t* plan, hipStream_t s) {
  hipLaunchKernelGGL(seq_plan_kernel, dim3(1), dim3(1024), 0, s, d, seq, max_n_quant, max_n_res, entries, plan);
  return hipGetLastError();
}

hipError_t launch_seq_advance(const Dims& d, int32_t* seq, hipStream_t s) {
  hipLaunchKernelGGL(seq_advance_kernel, dim3((d.batch + 255) / 256), dim3(256), 0, s, d, seq);
  return hipGetLastError();
}

hipError_t launch_group_step(const Dims& d, int32_t group_index, const __half* k_new, const __half* v_new,
                             __half* k_res, __half* v_res, int32_t append_row, int32_t group_row0,
                             const int32_t* seq, const kvq_pool& pool, uint8_t* selected, const kvq_qcache& qc,
                             hipStream_t s) {
  return d.bits == 2 ? launch_group_step_bits<2>(d, group_index, k_new, v_new, k_res, v_res, append_row, group_row0, seq, pool, selected, qc, s)
                     : launch_group_step_bits<4>(d, group_index, k_new, v_new, k_res, v_res, append_row, group_row0, seq, pool, selected, qc, s);
}

hipError_t launch_quantize(const Dims& d, int32_t group_index, int32_t n_groups, const __half* k_group,
                           const __half* v_group, int64_t unit_stride, const uint8_t* selected,
                           int64_t selected_unit_stride, const kvq_qcache& qc, hipStream_t s, int32_t tail_n,
                           __half* k_res, __half* v_res) {
  return d.bits == 2 ? launch_quantize_bits<2>(d, group_index, n_groups, k_group, v_group, unit_stride, selected, selected_unit_stride, qc, tail_n, k_res, v_res, s)
                     : launch_quantize_bits<4>(d, group_index, n_groups, k_group, v_group, unit_stride, selected, selected_unit_stride, qc, tail_n, k_res, v_res, s);
}

hipError_t launch_tail_copy(const Dims& d, const __half* k_rows, const __half* v_rows, int64_t unit_stride, int32_t n0,
                            int32_t n, __half* k_res, __half* v_res, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int by = (n * 16 + 255) / 256;
  hipLaunchKernelGGL(tail_copy_kernel, dim3(d.units_per_layer, by > 16 ? 16 : by), dim3(256), 0, s, d, k_rows, v_rows,
                     unit_stride, n0, n, k_res, v_res);
  return hipGetLastError();
}

}  // namespace kvq
