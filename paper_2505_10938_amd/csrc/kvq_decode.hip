// Decode-step attention (Eq. 1) over the quantized cache, the residual ring and the outlier
// pools, for gfx950.  One kernel launch per call.
//
// Work split: grid = (splits, kv heads, batch), 1 to 8 wavefronts per workgroup.  The quantized
// tokens of a unit are cut into mini-chunks of 128 tokens (4 packed blocks).  A workgroup owns a
// contiguous range of mini-chunks; its wavefronts take them round-robin, each keeping a running
// (max, sum, weighted values) and loading its next mini-chunk into registers while it computes
// the current one.  The full-precision rows (residual ring, outlier pool, auxiliary pool) are
// dealt to the same wavefronts in groups of 16, starting from the wavefronts with the fewest
// mini-chunks, and are processed first, while the first quantized loads are in flight.  Every
// workgroup merges its wavefronts' results through LDS.  With one workgroup per unit (the usual
// case when there are many units) that is the output; otherwise it is a partial, and the last
// workgroup of a unit to arrive (per-unit counter) merges the partials and writes the output.
//
// Arithmetic: every contraction runs on the matrix cores (v_mfma_f32_16x16x32_f16).
//  * q.K^T:  A = q * step, split in fp16 hi + lo rows (two matrix rows per query head, so the
//            split costs no extra instruction), B = the packed codes themselves.
//  * P.V:    A = p * step (hi + lo rows), B = the packed codes.
//  * zero points: sum_c q_c z_c (one scalar per group and head) is A = q (hi/lo) times B = the
//            fp16 zeros of the group; sum_t p_t z_t (one scalar per head and value group) and
//            sum_t p_t are A = p (hi/lo) times B = [zeros | ones].
// A packed code becomes an fp16 operand with ONE `and`: masked in place, a 2-bit code at bits
// [p, p+2) of a half-word is the fp16 subnormal code * 2^(p-24), and the factor 2^(-p) is folded
// into the other operand.  The matrix cores take a subnormal input at its value, but they align
// the products of one instruction as if its exponent were that of the smallest normal number and
// drop what falls below their window: measured, the sum is off by up to 2^-15 of the largest
// product with codes at bits 0..7 and by 2^-18 with codes at bits 2..9 (2^-23 with normal numbers),
// so the packed format keeps every code as high in the significand as one rotation allows.
// Scores live in the log2 domain: s = (q . k) * log2(e) / sqrt(d).
#include "kvq_common.h"

#include <type_traits>

namespace kvq {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowBytes = 272;   // LDS row of 128 fp16 + 16 bytes of padding (bank spread)
// The operands q*step and p*step are formed from q (p) scaled by 2^(kSh - pos) and split in fp16 hi + lo
// (pos = bit position of the code they meet, 2..8).  The largest factor, 2^(kSh - 2), bounds what fits
// fp16: |q| * step * log2(e)/sqrt(d) < 2^12 and Value steps < 2^12.  The smallest, 2^(kSh - 8), pushes
// the lo parts of small elements into fp16 subnormals (spacing 2^-24): an absolute error of up to
// 2^(pos - 25 - kSh) * step * code per element in score units, 1e-5 for a Key step of 40 at pos = 8,
// and 2^(pos - 25 - kSh) * code per token in output units.
constexpr int kShK = 6;
constexpr int kShV = 6;

__device__ inline float h2f_bits(uint32_t bits16) { return __half2float(__ushort_as_half((unsigned short)bits16)); }

// Order LDS traffic between lanes of one wavefront (DS operations of a wave execute in order;
// this only stops the compiler from moving them across).
__device__ inline void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Wave-wide reductions on the DPP path (no LDS traffic), N values at once: 4 steps inside each row
// of 16 lanes, then row 0->1, 2->3 and rows {0,1}->{2,3}; the totals are in lane 63 and are
// broadcast from there.  Written as instructions, one per value and step, operating in place (the
// compiler's own form takes four).  A DPP operand must not be read sooner than two issue slots
// after it was written: with four values the other three chains fill the slots, with fewer an
// s_nop does.  Lanes a step does not write (rows outside row_mask) keep their value.
#define KVQ_DPP_CTRL0 "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf"
#define KVQ_DPP_CTRL1 "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
#define KVQ_DPP_CTRL2 "row_half_mirror row_mask:0xf bank_mask:0xf"
#define KVQ_DPP_CTRL3 "row_mirror row_mask:0xf bank_mask:0xf"
#define KVQ_DPP_CTRL4 "row_bcast:15 row_mask:0xa bank_mask:0xf"
#define KVQ_DPP_CTRL5 "row_bcast:31 row_mask:0xc bank_mask:0xf"
#define KVQ_DPP_STEP1(OP, C) "s_nop 1\n\t" OP " %0, %0, %0 " C "\n\t"
#define KVQ_DPP_STEP2(OP, C) "s_nop 0\n\t" OP " %0, %0, %0 " C "\n\t" OP " %1, %1, %1 " C "\n\t"
#define KVQ_DPP_STEP4(OP, C) \
  OP " %0, %0, %0 " C "\n\t" OP " %1, %1, %1 " C "\n\t" OP " %2, %2, %2 " C "\n\t" OP " %3, %3, %3 " C "\n\t"
#define KVQ_DPP_ALL(STEP, OP)                                                                               \
  STEP(OP, KVQ_DPP_CTRL0) STEP(OP, KVQ_DPP_CTRL1) STEP(OP, KVQ_DPP_CTRL2) STEP(OP, KVQ_DPP_CTRL3) \
  STEP(OP, KVQ_DPP_CTRL4) STEP(OP, KVQ_DPP_CTRL5)
__device__ inline float from_lane63(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
#define KVQ_WAVE_REDUCE(NAME, OP)                                                                      \
  __device__ inline void NAME(float (&v)[1]) {                                                         \
    asm(KVQ_DPP_ALL(KVQ_DPP_STEP1, OP) : "+v"(v[0]));                                                  \
    v[0] = from_lane63(v[0]);                                                                          \
  }                                                                                                    \
  __device__ inline void NAME(float (&v)[2]) {                                                         \
    asm("s_nop 0\n\t" KVQ_DPP_ALL(KVQ_DPP_STEP2, OP) : "+v"(v[0]), "+v"(v[1]));                        \
    v[0] = from_lane63(v[0]);                                                                          \
    v[1] = from_lane63(v[1]);                                                                          \
  }                                                                                                    \
  __device__ inline void NAME(float (&v)[4]) {                                                         \
    asm("s_nop 1\n\t" KVQ_DPP_ALL(KVQ_DPP_STEP4, OP) : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3])); \
    v[0] = from_lane63(v[0]);                                                                          \
    v[1] = from_lane63(v[1]);                                                                          \
    v[2] = from_lane63(v[2]);                                                                          \
    v[3] = from_lane63(v[3]);                                                                          \
  }
KVQ_WAVE_REDUCE(wave_max, "v_max_f32_dpp")
KVQ_WAVE_REDUCE(wave_sum, "v_add_f32_dpp")
// eight values: two chains of four
#define KVQ_WAVE_REDUCE8(NAME)                                              \
  __device__ inline void NAME(float (&v)[8]) {                                \
    float a[4] = {v[0], v[1], v[2], v[3]}, b[4] = {v[4], v[5], v[6], v[7]};   \
    NAME(a);                                                                  \
    NAME(b);                                                                  \
    for (int i = 0; i < 4; ++i) {                                             \
      v[i] = a[i];                                                            \
      v[4 + i] = b[i];                                                        \
    }                                                                         \
  }
KVQ_WAVE_REDUCE8(wave_max)
KVQ_WAVE_REDUCE8(wave_sum)
// The same inside each row of 16 lanes only (the first four steps): every lane of a row ends up with the
// row's result (the mirrors stand for lane ^ 4 and lane ^ 8 because by then the lanes of a half hold the
// same partial result), which needs no broadcast.
#define KVQ_DPP_ROW(STEP, OP) STEP(OP, KVQ_DPP_CTRL0) STEP(OP, KVQ_DPP_CTRL1) STEP(OP, KVQ_DPP_CTRL2) STEP(OP, KVQ_DPP_CTRL3)
#define KVQ_ROW_REDUCE(NAME, OP)                                                                       \
  __device__ inline void NAME(float (&v)[1]) { asm(KVQ_DPP_ROW(KVQ_DPP_STEP1, OP) : "+v"(v[0])); }     \
  __device__ inline void NAME(float (&v)[2]) {                                                         \
    asm("s_nop 0\n\t" KVQ_DPP_ROW(KVQ_DPP_STEP2, OP) : "+v"(v[0]), "+v"(v[1]));                        \
  }                                                                                                    \
  __device__ inline void NAME(float (&v)[4]) {                                                         \
    asm("s_nop 1\n\t" KVQ_DPP_ROW(KVQ_DPP_STEP4, OP) : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3])); \
  }                                                                                                    \
  __device__ inline void NAME(float (&v)[8]) {                                                         \
    float a[4] = {v[0], v[1], v[2], v[3]}, b[4] = {v[4], v[5], v[6], v[7]};                            \
    NAME(a);                                                                                           \
    NAME(b);                                                                                           \
    for (int i = 0; i < 4; ++i) {                                                                      \
      v[i] = a[i];                                                                                     \
      v[4 + i] = b[i];                                                                                 \
    }                                                                                                  \
  }
KVQ_ROW_REDUCE(row16_max, "v_max_f32_dpp")
KVQ_ROW_REDUCE(row16_sum, "v_add_f32_dpp")

// fp16 hi/lo split of two floats: hi = fp16(x), lo = fp16(x - hi), both rounded to nearest, so that
// hi + lo = x (1 + e) with |e| <= 2^-22 and no bias (truncating hi instead leaves 2^-21, one-sided);
// packed pairs.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
__device__ inline void split_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  const half2v h = __builtin_convertvector(float2v{x0, x1}, half2v);
  const half2v l = __builtin_convertvector(float2v{x0 - (float)h[0], x1 - (float)h[1]}, half2v);
  hi = __builtin_bit_cast(uint32_t, h);
  lo = __builtin_bit_cast(uint32_t, l);
}

// Product of an unevaluated sum ah + al (packed fp16 pairs) with packed fp16 b, again as an
// unevaluated sum: hi = fp16(ah*b); the rounding error ah*b - hi is exact in fp16 (a product of
// two 11-bit significands has 22 bits) and joins al*b in lo.  Three packed instructions.
__device__ inline void mul_split(half2v ah, half2v al, half2v b, uint32_t& hi, uint32_t& lo) {
  const half2v h = ah * b;
  const half2v e = __builtin_elementwise_fma(ah, b, -h);
  const half2v l = __builtin_elementwise_fma(al, b, e);
  hi = __builtin_bit_cast(uint32_t, h);
  lo = __builtin_bit_cast(uint32_t, l);
}
__device__ inline half2v as_half2(uint32_t w) { return __builtin_bit_cast(half2v, w); }

// Rotary position embedding of one lane's channel pair (2*lane, 2*lane + 1).  Channel i < 64 forms a
// plane with channel i + 64, so a lane's partner is lane ^ 32 and both use the angles of pair lane & 31:
//     y_i = x_i cos_i - x_{i+64} sin_i,   y_{i+64} = x_{i+64} cos_i + x_i sin_i
// (Su et al., "RoFormer", Eq. 34, in the half-split pairing).  Each product and the sum are rounded to
// fp32 on their own and the result once to fp16: the rotated Key row is stored, and what is stored must
// not depend on how a compiler contracts the expression.
__device__ inline uint32_t rope_word(uint32_t own, uint32_t partner, float2 c, float2 s, bool upper) {
#pragma clang fp contract(off)
  const float o0 = h2f_bits(own & 0xFFFFu), o1 = h2f_bits(own >> 16);
  const float p0 = h2f_bits(partner & 0xFFFFu), p1 = h2f_bits(partner >> 16);
  const float a0 = o0 * c.x, a1 = o1 * c.y, b0 = p0 * s.x, b1 = p1 * s.y;
  const float y0 = upper ? a0 + b0 : a0 - b0;
  const float y1 = upper ? a1 + b1 : a1 - b1;
  return (uint32_t)__half_as_ushort(__float2half_rn(y0)) | ((uint32_t)__half_as_ushort(__float2half_rn(y1)) << 16);
}

// Exponent of the power of two carried by pair v (v = lane & 3 on the producing side) of a
// field: a masked code at pair v is worth code * 2^(pos(v) - 24).
template <int BITS>
__device__ inline int pair_pos(int v) { return BITS == 2 ? 2 + 2 * v : 2 + 4 * (v & 1); }

// One matrix-core operand (8 fp16 = 4 dwords) from field f of a lane's packed words.  The codes of
// a field sit at bits 2..9 of each half-word, of the word itself or of the word rotated by 8.
template <int BITS>
__device__ inline half8 field_operand(const uint32_t (&w)[2 * BITS], int f) {
  u32x4 o;
  if (BITS == 2) {
    const uint32_t x = (f & 1) ? __builtin_amdgcn_alignbit(w[f >> 1], w[f >> 1], 8) : w[f >> 1];
    o[0] = x & 0x000C000Cu;
    o[1] = x & 0x00300030u;
    o[2] = x & 0x00C000C0u;
    o[3] = x & 0x03000300u;
  } else {
    const uint32_t x = w[f], y = __builtin_amdgcn_alignbit(w[f], w[f], 8);
    o[0] = x & 0x003C003Cu;
    o[1] = x & 0x03C003C0u;
    o[2] = y & 0x003C003Cu;
    o[3] = y & 0x03C003C0u;
  }
  return __builtin_bit_cast(half8, o);
}

// Device-scope (all compute dies) relaxed accesses for data exchanged between workgroups.
__device__ inline void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float coherent_load(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline half8 lds_operand(const unsigned char* row, int byte) {
  return __builtin_bit_cast(half8, *(const u32x4*)(row + byte));
}

// Registers one wavefront loads for one mini-chunk (4 blocks), per lane.
template <int BITS, int NV>
struct McRegs {
  uint32_t kc[4][2 * BITS];  // Key codes: this lane's 16 (32) bytes of each block
  uint32_t vc[4][2 * BITS];  // Value codes
  uint32_t ksp[4];         // Key steps of channels 2*lane, 2*lane+1 of each block's group
  uint32_t ksz[4];         // Key zeros, same channels
  uint32_t vsp[NV];        // Value steps of this lane's tokens (2*lane, 2*lane+1 of the 128), per value group
  uint32_t vsz[NV];        // Value zeros, same tokens
  uint32_t mkw;            // mask word of this lane's block
  bool mk_valid;           // false for a block past the end (every token of it is masked)
};

// LDS of one wavefront.  The first group of arrays is used while scores are formed, the second
// afterwards; they share storage.  The scores of a mini-chunk are written while the first group is in
// use and read before the second buffer of the p*step rows is first written: they lie behind the
// first group, over that second buffer.
template <int GQ, int NV>
struct WaveLds {
  struct KeyPart {
    unsigned char aop[2][2 * GQ][kRowBytes];      // q*step rows of one block; two buffers, taken in turn
    unsigned char zk[4][kRowBytes];               // Key zeros per block, 128 channels
  };
  struct ValuePart {
    unsigned char pp[2 * GQ][kRowBytes];          // p rows (hi/lo per head), 128 tokens
    unsigned char zv[NV + 1][kRowBytes];          // Value zeros per value group, 128 tokens; row NV = ones
    unsigned char ps[2][2 * GQ][kRowBytes];       // p*step rows of one value group; two buffers, taken in turn
  };
  static constexpr int kSecondBuffer = (2 * GQ + NV + 1 + 2 * GQ) * kRowBytes;   // offset of ps[1]
  static constexpr int kScores = (int)sizeof(KeyPart) > kSecondBuffer ? (int)sizeof(KeyPart) : kSecondBuffer;
  static constexpr int kSharedBytes =
      (int)sizeof(ValuePart) > kScores + GQ * 128 * 4 ? (int)sizeof(ValuePart) : kScores + GQ * 128 * 4;
  unsigned char q0[2 * GQ][kRowBytes];            // q rows (hi/lo per head), no step; written once
  union {
    KeyPart k;
    ValuePart v;
    unsigned char shared[kSharedBytes];
  };
  float qz[4][GQ];                                // sum_c q_c z_c per (block, head)
  // scores of the 128 tokens, [GQ][128]
  __device__ __forceinline__ float (&sc())[GQ][128] { return *(float (*)[GQ][128])(shared + kScores); }
};

// Results handed to the workgroup merge, laid over the wavefronts' storage once they are done
// with it: slots 0..nw-1 = the wavefronts' quantized parts, slots nw..2nw-1 = their
// full-precision parts.
template <int GQ, int NV>
struct MergeView {
  float* o;   // [2 nw][GQ][kHeadDim]
  float* m;   // [2 nw][GQ]
  float* l;   // [2 nw][GQ]
  float* z;   // [nw][GQ][NV]: sum_t p_t z_t per value group (quantized parts)
  __device__ MergeView(unsigned char* base, int nw) {
    o = (float*)base;
    m = o + 2 * nw * GQ * kHeadDim;
    l = m + 2 * nw * GQ;
    z = l + 2 * nw * GQ;
  }
};
template <int GQ, int NV>
constexpr int merge_bytes_per_wave() { return (2 * GQ * kHeadDim + 4 * GQ + GQ * NV) * 4; }

// Uniform (per wavefront) base pointers of the unit's quantized cache; loads add 32-bit offsets.
// Block i of a dense cache is the unit's i-th block.  In a paged cache the blocks of Key group j
// are those of page table[j] of the plane (layer, kv head) the pointers address; the physical
// block numbers of the mini-chunk about to be loaded are kept in `pb`.
template <bool PAGED>
struct UnitPtrs {
  const unsigned char* kc;    // Key codes
  const unsigned char* vc;    // Value codes
  const unsigned char* km;    // Key meta
  const unsigned char* vm;    // Value meta
  const unsigned char* mask;
  int nblocks;                // quantized blocks of the unit
  int last_block;             // the last of them (0 if there is none: the cache holds at least one block)
  int bpg_shift;
  uint32_t block_bytes;
  const int32_t* table;       // paged: the sequence's row of the page table
  int n_pages;                // paged: pages per plane
  uint32_t pb0, pb1, pb2, pb3;  // paged: where the four blocks of the mini-chunk being loaded are stored
  uint32_t pbl;               // paged: the same for block lane >> 4 (per lane)

  // block i of mini-chunk mc, as stored (a block past the end is replaced by the last one)
  __device__ __forceinline__ uint32_t block(int mc, int i) const {
    if constexpr (PAGED) return i == 0 ? pb0 : i == 1 ? pb1 : i == 2 ? pb2 : pb3;
    else return (uint32_t)min(mc * 4 + i, last_block);
  }
  // the block of this lane's token pair: block lane >> 4 of the mini-chunk
  __device__ __forceinline__ uint32_t lane_block(int mc, int lane) const {
    if constexpr (PAGED) return pbl;
    else return (uint32_t)min(mc * 4 + (lane >> 4), last_block);
  }
  // Page-table entries of mini-chunk mc: that of block lane & 3 (lanes 0..3 are read out to scalar
  // registers) and that of the lane's own block lane >> 4.  Vector loads: they take their turn among
  // the other loads in flight.  `resolve` turns them into block numbers.  An entry outside
  // [0, n_pages) is clamped: whatever the table holds, accesses stay inside the pool.
  struct Pages {
    uint32_t of_block, of_lane;
  };
  __device__ __forceinline__ Pages fetch_pages(int mc, int lane) const {
    const uint32_t b0 = (uint32_t)min(mc * 4 + (lane & 3), last_block);
    const uint32_t b1 = (uint32_t)min(mc * 4 + (lane >> 4), last_block);
    return {(uint32_t)table[b0 >> bpg_shift], (uint32_t)table[b1 >> bpg_shift]};
  }
  __device__ __forceinline__ uint32_t stored_block(uint32_t logical, uint32_t entry) const {
    const int page = min(max((int)entry, 0), n_pages - 1);
    return ((uint32_t)page << bpg_shift) | (logical & ((1u << bpg_shift) - 1u));
  }
  __device__ __forceinline__ void resolve(int mc, Pages e, int lane) {
    pb0 = stored_block((uint32_t)min(mc * 4 + 0, last_block), __builtin_amdgcn_readlane(e.of_block, 0));
    pb1 = stored_block((uint32_t)min(mc * 4 + 1, last_block), __builtin_amdgcn_readlane(e.of_block, 1));
    pb2 = stored_block((uint32_t)min(mc * 4 + 2, last_block), __builtin_amdgcn_readlane(e.of_block, 2));
    pb3 = stored_block((uint32_t)min(mc * 4 + 3, last_block), __builtin_amdgcn_readlane(e.of_block, 3));
    pbl = stored_block((uint32_t)min(mc * 4 + (lane >> 4), last_block), e.of_lane);
  }
};
// The cache is read once per launch: its loads are non-temporal, which keeps them from displacing each
// other in the caches on their way through (measured: a plain streaming read reaches 7.0 TB/s with
// such loads against 6.2 TB/s without, and the kernel gains 8-12 %).
template <typename T>
__device__ __forceinline__ T ld(const unsigned char* base, uint32_t off);
template <>
__device__ __forceinline__ uint32_t ld<uint32_t>(const unsigned char* base, uint32_t off) {
  return __builtin_nontemporal_load((const uint32_t*)(base + off));
}
template <>
__device__ __forceinline__ uint4 ld<uint4>(const unsigned char* base, uint32_t off) {
  const u32x4 t = __builtin_nontemporal_load((const u32x4*)(base + off));
  return make_uint4(t[0], t[1], t[2], t[3]);
}

// Loads of one mini-chunk, in the four parts the compute phases consume.  A block past the end of
// the quantized segment is replaced by the last block with every token masked, so that every
// wave runs the same straight-line code.
template <int BITS, int NV, class PT>
__device__ __forceinline__ void load_k_meta_block(McRegs<BITS, NV>& R, const PT& P, int mc, int i, int lane) {
  // uniform base (scalar registers) + one lane offset shared by all loads
  const unsigned char* gp = P.km + (P.block(mc, i) >> P.bpg_shift) * 512u;
  // (ordinary loads: with groups of more than 32 tokens the blocks of a mini-chunk share these rows, and
  // non-temporal loads were measured slower here even without sharing)
  R.ksp[i] = *(const uint32_t*)(gp + lane * 4u);
  R.ksz[i] = *(const uint32_t*)(gp + 256 + lane * 4u);
}
// (SB: how many consecutive blocks of a mini-chunk lie in one Key group - 1, 2 or 4 for groups of 32, 64 or
// 128 tokens - and share its steps and zeros: those are loaded, and the operand rows made of them are
// formed, once per group, by the group's first block)
template <int BITS, int NV, int SB, class PT>
__device__ __forceinline__ void load_k_meta(McRegs<BITS, NV>& R, const PT& P, int mc, int lane) {
#pragma unroll
  for (int i = 0; i < 4; i += SB) load_k_meta_block(R, P, mc, i, lane);
}
template <int BITS, class PT>
__device__ __forceinline__ void load_codes_block(uint32_t (&w)[4][2 * BITS], const unsigned char* codes,
                                                 const PT& P, int mc, int i, int lane) {
  const unsigned char* bp = codes + P.block(mc, i) * P.block_bytes;   // uniform
#pragma unroll
  for (int hf = 0; hf < BITS / 2; ++hf) {
    const uint4 t = ld<uint4>(bp + hf * 1024, lane * 16u);
    w[i][4 * hf + 0] = t.x;
    w[i][4 * hf + 1] = t.y;
    w[i][4 * hf + 2] = t.z;
    w[i][4 * hf + 3] = t.w;
  }
}
template <int BITS, class PT>
__device__ __forceinline__ void load_codes(uint32_t (&w)[4][2 * BITS], const unsigned char* codes, const PT& P,
                                           int mc, int lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) load_codes_block<BITS>(w, codes, P, mc, i, lane);
}
template <int BITS, int NV, class PT>
__device__ __forceinline__ void load_v_meta(McRegs<BITS, NV>& R, const PT& P, int mc, int lane) {
  // this lane's tokens are 2*lane, 2*lane+1 of the 128: pair lane&15 of block lane>>4
  const int myblk = mc * 4 + (lane >> 4);
  const uint32_t blk = P.lane_block(mc, lane);
  // the loaded word is not touched here: any use would make this point wait for the load
  R.mkw = ld<uint32_t>(P.mask, blk * 4u);
  R.mk_valid = myblk < P.nblocks;
  const uint32_t off = blk * (128u * NV) + (lane & 15) * (4u * NV);
#pragma unroll
  for (int jv = 0; jv < NV; ++jv) {
    R.vsp[jv] = ld<uint32_t>(P.vm, off + 4u * jv);
    R.vsz[jv] = ld<uint32_t>(P.vm, off + 64u * NV + 4u * jv);
  }
}

// Running state of one wavefront over its mini-chunks.
template <int GQ>
struct WaveAcc {
  float4v O[8];      // weighted values: 8 channel tiles; rows = heads (hi, lo)
  float4v Dz;        // columns < NV: sum_t p_t z_t per value group; column NV: sum_t p_t
  float m[GQ];       // running maximum per head (log2 domain)
};

template <int GQ, int BITS, int NV, int SB, bool more, class PT>
__device__ __forceinline__ void compute_minichunk(McRegs<BITS, NV>& R, WaveAcc<GQ>& S, WaveLds<GQ, NV>& L,
                                                  const half2v (&qh)[GQ], const half2v (&ql)[GQ], int lane,
                                                  const PT& P, int mc_next) {
  // Each group of registers is reloaded for the wave's next mini-chunk (mc_next, if `more`) right
  // after its last use here, so those loads are in flight during the rest of this mini-chunk.
  // `more` is a template parameter so that every path has a fixed number of loads in flight and
  // the waits on them can be exact.
  // Operand rows that depend on a block (q*step) or on a value group (p*step) are formed right
  // before the products that read them, in two buffers taken in turn: LDS operations of a
  // wavefront execute in program order, so a buffer can be rewritten as soon as the reads of its
  // previous contents have been issued, and the vector work of the next rows runs under the
  // matrix instructions of the current ones.
  const int m16 = lane & 15, r = lane >> 4;
  constexpr int R2 = 2 * GQ;
  const int arow = m16 % R2;          // rows beyond 2*GQ repeat valid rows (their results are unused)
  auto key_rows = [&](int i) {          // q*step (hi/lo per head) of the Key group that block i begins
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      uint32_t hi, lo;
      mul_split(qh[j], ql[j], as_half2(R.ksp[i]), hi, lo);
      ((uint32_t*)L.k.aop[(i / SB) & 1][2 * j])[lane] = hi;
      ((uint32_t*)L.k.aop[(i / SB) & 1][2 * j + 1])[lane] = lo;
    }
  };

  wave_sync();                          // the previous mini-chunk is done with the shared storage
#pragma unroll
  for (int i = 0; i < 4; i += SB) ((uint32_t*)L.k.zk[i])[lane] = R.ksz[i];
  key_rows(0);
  if (more) load_k_meta_block(R, P, mc_next, 0, lane);
  wave_sync();

  // ---- sum_c q_c z_c of the 4 blocks: column n of B = zeros of block n & 3 --------------------------
  {
    float4v Dq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
      Dq = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds_operand(L.q0[arow], cb * 64 + r * 16),
                                                  lds_operand(L.k.zk[(m16 & 3) & ~(SB - 1)], cb * 64 + r * 16), Dq, 0, 0, 0);
    if (m16 < 4) {
      if (2 * r < GQ) L.qz[m16][2 * r] = Dq[0] + Dq[1];
      if (2 * r + 1 < GQ) L.qz[m16][(2 * r + 1) % GQ] = Dq[2] + Dq[3];
    }
  }
  // ---- scores (left in units of 2^-(24 - kShK); the softmax scales them) -----------------------------
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i + 1 < 4 && (i + 1) % SB == 0) {
      key_rows(i + 1);
      if (more) load_k_meta_block(R, P, mc_next, i + 1, lane);
    }
    // both 16-token halves of the block share each operand row read
    float4v D0 = {0.f, 0.f, 0.f, 0.f}, D1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      const half8 aq = lds_operand(L.k.aop[(i / SB) & 1][arow], cb * 64 + r * 16);
      D0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(aq, field_operand<BITS>(R.kc[i], cb), D0, 0, 0, 0);
      D1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(aq, field_operand<BITS>(R.kc[i], 4 + cb), D1, 0, 0, 0);
    }
    if (more) load_codes_block<BITS>(R.kc, P.kc, P, mc_next, i, lane);
    const int tl = i * 32 + m16;
    if (2 * r < GQ) {
      L.sc()[2 * r][tl] = D0[0] + D0[1];
      L.sc()[2 * r][tl + 16] = D1[0] + D1[1];
    }
    if (2 * r + 1 < GQ) {
      L.sc()[(2 * r + 1) % GQ][tl] = D0[2] + D0[3];
      L.sc()[(2 * r + 1) % GQ][tl + 16] = D1[2] + D1[3];
    }
    if ((i + 1) % SB == 0) wave_sync();  // the next group's rows, at last the scores, are visible
  }

  // ---- softmax numerators of the 128 tokens against the running maximum; operand rows ---------------
  half2v ph[GQ], pl[GQ];                // p of this lane's two tokens, hi + lo
  half2v vs[NV];                        // their Value steps, scaled for the fp16 split
  auto value_rows = [&](int jv) {       // p*step (hi/lo per head) of value group jv
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      uint32_t hi, lo;
      mul_split(ph[j], pl[j], vs[jv], hi, lo);
      ((uint32_t*)L.v.ps[jv & 1][2 * j])[lane] = hi;
      ((uint32_t*)L.v.ps[jv & 1][2 * j + 1])[lane] = lo;
    }
  };
  {
    const float post_k = __builtin_amdgcn_exp2f((float)(24 - kShK));
    const int bi = lane >> 4;                         // block of this lane's tokens (2*lane, 2*lane+1)
    uint32_t mword = R.mkw;
    asm volatile("" : "+v"(mword) :: "memory");       // first use of the loaded word stays here
    mword = R.mk_valid ? mword : 0xFFFFFFFFu;
    const int bit = (2 * lane) & 31;
    const bool ok0 = !((mword >> bit) & 1u);
    const bool ok1 = !((mword >> (bit + 1)) & 1u);
    const _Float16 fv = (_Float16)__builtin_amdgcn_exp2f((float)(kShV - pair_pos<BITS>(lane & 3)));
    // The Value codes, which were asked for right after the steps and zeros used next, are waited for here
    // as well and not block by block between the matrix instructions that read them (measured: 0.5 %).
    asm volatile("" ::"v"(R.vc[3][2 * BITS - 1]));
#pragma unroll
    for (int jv = 0; jv < NV; ++jv) vs[jv] = as_half2(R.vsp[jv]) * half2v{fv, fv};
    float alpha[GQ], x0[GQ], x1[GQ], mx[GQ];
    bool above = false;                                 // does a score here exceed its head's running maximum?
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      const float2 s2 = *(const float2*)&L.sc()[j][2 * lane];
      const float qz = L.qz[bi][j];
      x0[j] = ok0 ? __builtin_fmaf(s2.x, post_k, qz) : kNegBig;
      x1[j] = ok1 ? __builtin_fmaf(s2.y, post_k, qz) : kNegBig;
      mx[j] = fmaxf(x0[j], x1[j]);
      above |= mx[j] > S.m[j];
      alpha[j] = 1.f;
    }
    // The wave-wide maxima are needed only if some score exceeds a running maximum (always in a
    // wavefront's first mini-chunk, ever more rarely afterwards): otherwise nothing moves.
    const bool rescale = __any(above);                  // wave-uniform
    if (rescale) {
      wave_max(mx);
#pragma unroll
      for (int j = 0; j < GQ; ++j) {
        const float m = fmaxf(S.m[j], mx[j]);
        alpha[j] = __builtin_amdgcn_exp2f(S.m[j] - m);
        S.m[j] = m;
      }
    }
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      const float m = S.m[j];
      const float p0 = ok0 ? __builtin_amdgcn_exp2f(x0[j] - m) : 0.f;
      const float p1 = ok1 ? __builtin_amdgcn_exp2f(x1[j] - m) : 0.f;
      uint32_t hi, lo;
      split_pair(p0, p1, hi, lo);
      ((uint32_t*)L.v.pp[2 * j])[lane] = hi;
      ((uint32_t*)L.v.pp[2 * j + 1])[lane] = lo;
      ph[j] = as_half2(hi);
      pl[j] = as_half2(lo);
    }
#pragma unroll
    for (int jv = 0; jv < NV; ++jv) ((uint32_t*)L.v.zv[jv])[lane] = R.vsz[jv];
    ((uint32_t*)L.v.zv[NV])[lane] = 0x3C003C00u;      // fp16 ones
    value_rows(0);
    // the running maximum moved (wave-uniform, rare after the first mini-chunks): rescale
    if (rescale) {
      float a0 = 1.f, a1 = 1.f;
#pragma unroll
      for (int j = 0; j < GQ; ++j) {
        a0 = (j == 2 * r) ? alpha[j] : a0;
        a1 = (j == 2 * r + 1) ? alpha[j] : a1;
      }
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        S.O[ct][0] *= a0;
        S.O[ct][1] *= a0;
        S.O[ct][2] *= a1;
        S.O[ct][3] *= a1;
      }
      S.Dz[0] *= a0;
      S.Dz[1] *= a0;
      S.Dz[2] *= a1;
      S.Dz[3] *= a1;
    }
  }
  wave_sync();

  // ---- weighted values; sum_t p_t z_t and sum_t p_t ride along as one more product -------------------
  const int zrow = m16 < NV ? m16 : NV;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    S.Dz = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds_operand(L.v.pp[arow], i * 64 + r * 16),
                                                  lds_operand(L.v.zv[zrow], i * 64 + r * 16), S.Dz, 0, 0, 0);
#pragma unroll
  for (int jv = 0; jv < NV; ++jv) {
    if (jv + 1 < NV) value_rows(jv + 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {                     // the channel tiles of one value group share an operand row
      const half8 ap = lds_operand(L.v.ps[jv & 1][arow], i * 64 + r * 16);
#pragma unroll
      for (int ct = jv * (8 / NV); ct < (jv + 1) * (8 / NV); ++ct)
        S.O[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ap, field_operand<BITS>(R.vc[i], ct), S.O[ct], 0, 0, 0);
    }
    if (jv + 1 < NV) wave_sync();                     // the next value group's rows are visible
  }
  // (the Value steps, zeros and mask word are reloaded here and not right after their last use:
  // held in flight across the products above they were moved to other registers at the end of
  // every pass, and such a move waits for the load)
  if (more) load_v_meta(R, P, mc_next, lane);
  if (more) load_codes<BITS>(R.vc, P.vc, P, mc_next, lane);
}

// Full-precision rows (residual ring, then outlier-pool slots, then auxiliary slots) in groups of
// 16: q.k^T on the matrix cores (a K row is a B operand as it is), the weighted values on the
// vector units (row-major V has the wrong operand shape).  Lane = channel pair for the values.
template <int GQ>
struct FpAcc {
  float m[GQ], l[GQ];
  float o[GQ][2];
};

// The state of the sequence a workgroup works on: the batch's (kernel arguments), or its own.
struct Seq {
  int n_quant, res_start, n_res;
  int n_ring;   // residual rows that are in the ring; n_res - n_ring (0 or 1) newest row comes with the call
};

struct FpRegs {
  uint4 kf[4];       // K row of token first + (lane & 15): channels 32cb + 8(lane >> 4) ..
  uint32_t vw[16];   // V rows of the 16 tokens: this lane's channel pair
  int group;
};

// The full-precision rows of a unit, in groups of 16 that are each one contiguous run of rows in memory,
// so that a group is loaded from one base address with constant offsets (no work per row):
//   groups 0 .. ring_groups-1 : the residual tokens in ring order, 16 per group.  The ring starts at a
//       multiple of 16 and has a multiple of 16 rows, so a group never wraps; the last group may reach past
//       the newest token (those rows are ring rows that hold no live token and are masked).  The token
//       being decoded, if it comes with the call, is the newest of them: its ring row is not written yet,
//       its Key row is read from the caller's buffer by the lanes that own it and its Value words are put
//       in place from the registers every wavefront has loaded them into.
//   then pool_groups groups  : the outlier-pool and auxiliary-pool slots, 16 per group; the last group may
//       reach up to 15 rows past the unit's last slot (the next unit's slots, or the padding behind the
//       last unit's: kvq_query_sizes counts it), masked as well.
struct FpLayout {
  int ring_groups, pool_groups;
  int new_group, new_t;    // where the token being decoded sits (new_group < 0: it does not come with the call)
  __device__ __forceinline__ int groups() const { return ring_groups + pool_groups; }
};
__device__ __forceinline__ FpLayout fp_layout(const DecodeArgs& a, const Seq& sq) {
  FpLayout f;
  f.ring_groups = (sq.n_res + 15) >> 4;
  f.pool_groups = (a.d.pool_slots + 15) >> 4;
  f.new_group = sq.n_res > sq.n_ring ? sq.n_ring >> 4 : -1;
  f.new_t = sq.n_ring & 15;
  return f;
}

// Issue the loads of group g (a wavefront without a group passes one that exists: the same loads are then
// in flight on every path; the ring always has a first group of 16 rows).  Every pool slot is read, filled or
// not: the slot counts are looked at only when the data is used, so that these loads do not wait for them.
__device__ __forceinline__ void fp_load(FpRegs& X, const DecodeArgs& a, const Seq& sq, const FpLayout& f, int64_t u,
                                        const __half* k_new_row, int g, int lane) {
  const Dims& d = a.d;
  const int m16 = lane & 15, r = lane >> 4;
  const bool is_ring = g < f.ring_groups;                            // uniform
  int ring0 = sq.res_start + 16 * (is_ring ? g : 0);
  ring0 -= ring0 >= d.res_rows ? d.res_rows : 0;
  const int slot0 = 16 * (g - f.ring_groups);
  const int64_t row0 = is_ring ? u * d.res_rows + ring0 : u * d.pool_slots + slot0;
  const unsigned char* kb = (const unsigned char*)((is_ring ? a.k_res : a.pool_k) + row0 * kHeadDim);
  const unsigned char* vb = (const unsigned char*)((is_ring ? a.v_res : a.pool_v) + row0 * kHeadDim);
  X.group = g;
  // Keys: lane (row m16, quarter r) reads its 16 bytes of each 64-byte run of its row
  const bool is_new = g == f.new_group && m16 == f.new_t;
  const unsigned char* kp = is_new ? (const unsigned char*)k_new_row + r * 16 : kb + m16 * (2 * kHeadDim) + r * 16;
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) X.kf[cb] = ld<uint4>(kp, cb * 64u);
  // Values: every lane its channel pair of each of the 16 rows
  const unsigned char* vp = vb + lane * 4;
#pragma unroll
  for (int t = 0; t < 16; ++t) X.vw[t] = ld<uint32_t>(vp, t * (2u * kHeadDim));
}

// Does row m16 of group g hold a token?
__device__ __forceinline__ bool fp_row_ok(const DecodeArgs& a, const Seq& sq, const FpLayout& f, int g, int m16,
                                          int n_pool, int n_aux) {
  if (g < f.ring_groups) return 16 * g + m16 < sq.n_res;
  const int slot = 16 * (g - f.ring_groups) + m16;
  return slot < a.d.N ? (slot < n_pool) : (slot < a.d.pool_slots && slot - a.d.N < n_aux);
}

template <int GQ, int NV, bool ROPE>
__device__ __forceinline__ void fp_compute(FpRegs& X, FpAcc<GQ>& F, WaveLds<GQ, NV>& L, const DecodeArgs& a,
                                           const Seq& sq, const FpLayout& f, int n_pool, int n_aux, int r0,
                                           uint32_t k_new_word, uint32_t v_new_word, int lane) {
  const int m16 = lane & 15, r = lane >> 4;
  const bool okk = fp_row_ok(a, sq, f, X.group, m16, n_pool, n_aux);
  if (X.group == f.new_group) {                                    // uniform, one group of the unit
#pragma unroll
    for (int t = 0; t < 16; ++t) X.vw[t] = t == f.new_t ? v_new_word : X.vw[t];
    if constexpr (ROPE) {
      // The new Key row was loaded as the caller gave it; the rotated one exists as one word per lane
      // (channels 2*lane, 2*lane + 1).  The lanes that own the row take their 16-byte pieces (channels
      // 32 cb + 8 r ..) from the lanes that hold them: words 16 cb + 4 r .. + 3.
      const bool mine = m16 == f.new_t;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const uint32_t w0 = (uint32_t)__shfl((int)k_new_word, 16 * cb + 4 * r + 0);
        const uint32_t w1 = (uint32_t)__shfl((int)k_new_word, 16 * cb + 4 * r + 1);
        const uint32_t w2 = (uint32_t)__shfl((int)k_new_word, 16 * cb + 4 * r + 2);
        const uint32_t w3 = (uint32_t)__shfl((int)k_new_word, 16 * cb + 4 * r + 3);
        X.kf[cb] = mine ? make_uint4(w0, w1, w2, w3) : X.kf[cb];
      }
    }
  }
  // Several query tokens at once: token i of q_tokens does not see the q_tokens - 1 - i tokens after it,
  // which are the newest residual rows (one query token: nothing is hidden).  Row j of this workgroup
  // belongs to token (r0 + j) >> g_shift.
  auto seen_by = [&](int j) {
    const int after = a.q_tokens - 1 - ((r0 + j) >> a.g_shift);
    const int row = 16 * X.group + m16;                              // its place among the residual tokens
    return okk && !(X.group < f.ring_groups && row >= sq.n_res - after);
  };
  // which of the 16 rows hold a token, as a wave-uniform bit mask (lanes 0..15 are rows 0..15)
  const uint32_t ok_rows = (uint32_t)__ballot(okk) & 0xFFFFu;
  constexpr int R2 = 2 * GQ;
  const int arow = m16 % R2;
  float4v D = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
    D = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds_operand(L.q0[arow], cb * 64 + r * 16),
                                                __builtin_bit_cast(half8, X.kf[cb]), D, 0, 0, 0);
  wave_sync();                                                     // earlier readers of sc are done
  if (2 * r < GQ) L.sc()[2 * r][m16] = seen_by(2 * r) ? D[0] + D[1] : kNegBig;
  if (2 * r + 1 < GQ) L.sc()[(2 * r + 1) % GQ][m16] = seen_by(2 * r + 1) ? D[2] + D[3] : kNegBig;
  // a row that holds no token may hold anything, a NaN too: its Value words are cleared (most groups are
  // full: one uniform test)
  if (ok_rows != 0xFFFFu) {
#pragma unroll
    for (int t = 0; t < 16; ++t) X.vw[t] = ((ok_rows >> t) & 1u) ? X.vw[t] : 0u;
  }
  wave_sync();
  float alpha[GQ], x[GQ], red[GQ];
#pragma unroll
  for (int j = 0; j < GQ; ++j) red[j] = x[j] = L.sc()[j][m16];      // every row of 16 lanes: the 16 scores
  row16_max(red);
#pragma unroll
  for (int j = 0; j < GQ; ++j) {
    const float m = fmaxf(F.m[j], red[j]);
    alpha[j] = __builtin_amdgcn_exp2f(F.m[j] - m);
    F.m[j] = m;
    x[j] = x[j] > 0.5f * kNegBig ? __builtin_amdgcn_exp2f(x[j] - m) : 0.f;   // now p
    red[j] = x[j];
    if (lane < 16) L.sc()[j][16 + lane] = x[j];
  }
  row16_sum(red);
#pragma unroll
  for (int j = 0; j < GQ; ++j) F.l[j] = F.l[j] * alpha[j] + red[j];
  wave_sync();
#pragma unroll
  for (int j = 0; j < GQ; ++j) {
    F.o[j][0] *= alpha[j];
    F.o[j][1] *= alpha[j];
  }
  // (newest row first: loads return in order, so the wait for the last row's word covers all of them)
#pragma unroll
  for (int t = 15; t >= 0; --t) {
    const float v0 = h2f_bits(X.vw[t] & 0xFFFFu), v1 = h2f_bits(X.vw[t] >> 16);
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      const float p = L.sc()[j][16 + t];
      F.o[j][0] += p * v0;
      F.o[j][1] += p * v1;
    }
  }
}

// One unit (or one split of it) on the calling workgroup.  `entry` < 0: the grid's coordinates say which;
// otherwise entry `entry` of the launch plan does (a batch of sequences of different lengths dealt by
// length).  The plan is device data: what is read from it is clamped to bounds the host has checked
// against the buffers.
// (ROPE: the launch rotates the query rows and the new Key row - an instance of its own, so that the others
// carry nothing of it: with a run-time test instead they measured 0.3 % slower)
template <int GQ, int BITS, int NV, bool PAGED, int SB, bool ROPE>
__device__ __forceinline__ void decode_item(const DecodeArgs& a, unsigned char* smem, int& s_last, int entry) {
  const Dims& d = a.d;
  // Every argument the loads below depend on is fetched here, in one round trip (left to
  // itself the compiler fetches an argument where it is first used, and each such place waits
  // for everything that is in flight on the scalar side).
  asm volatile("" ::"s"(a.nw), "s"(a.splits), "s"(a.head_parts), "s"(a.mc_per_split), "s"(a.n_quant), "s"(a.res_start),
               "s"(a.n_res), "s"(d.kv_heads), "s"(d.q_heads), "s"(d.unit0), "s"(d.pool_slots), "s"(d.res_rows), "s"(d.N),
               "s"(d.bpg_shift), "s"(d.block_bytes), "s"(d.blocks_per_unit), "s"(d.groups_per_unit), "s"(a.q),
               "s"(a.k_codes), "s"(a.k_meta), "s"(a.v_codes), "s"(a.v_meta), "s"(a.mask), "s"(a.k_res), "s"(a.v_res),
               "s"(a.pool_k), "s"(a.pool_v), "s"(a.pool_count), "s"(a.aux_count), "s"(a.seq));
  asm volatile("" ::"s"(a.k_new), "s"(a.v_new), "s"(d.page_table), "s"(d.table_stride), "s"(d.n_pages), "s"(d.plane0),
               "s"(a.q_tokens), "s"(a.g_shift));
  if constexpr (ROPE) asm volatile("" ::"s"(a.rope), "s"(a.rope_stride));
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nw = a.nw;
  const int nthreads = nw * 64;
  const int m16 = lane & 15, r = lane >> 4;
  // the query heads of a kv head may be dealt to `head_parts` workgroup rows (part-major in
  // blockIdx.y, so that the parts of one kv head tend to land on the same compute die)
  const int h = blockIdx.y % d.kv_heads, part = blockIdx.y / d.kv_heads;
  int split = blockIdx.x, b = blockIdx.z, n_splits = a.splits;
  int64_t part_first = -1;                               // first slot of the unit's partial results (plan only)
  int4 planned = {0, 0, 0, 0};
  int plan_mc_begin = 0, plan_mc_end = 0;
  if (entry >= 0) {
    const int32_t* e = a.plan + 8 + 8 * entry;
    const int4 e0 = *(const int4*)e;
    planned = *(const int4*)(e + 4);
    b = min(max(e0.x, 0), d.batch - 1);
    n_splits = min(max(e0.z, 1), a.plan_entries);
    split = min(max(e0.y, 0), n_splits - 1);
    plan_mc_begin = e0.w;
    plan_mc_end = planned.w;
    part_first = (int64_t)blockIdx.y * a.plan_entries + min(max(entry - split, 0), a.plan_entries - n_splits);
  }
  const int ul = b * d.kv_heads + h;                     // the unit whose cache is read
  const int wl = ul * a.head_parts + part;               // its slice of the workspace
  // The rows handled here: GQ consecutive (query token, query head) pairs of the kv head, token-major
  // (a plain decode step has one token: the rows are the kv head's query heads).
  const int r0 = part * GQ;
  auto row_elem = [&](int j) -> int64_t {                // element offset of row j's query and output row
    const int r = r0 + j, tj = r >> a.g_shift, hj = r & ((1 << a.g_shift) - 1);
    return (((int64_t)b * a.q_tokens + tj) * d.q_heads + (h << a.g_shift) + hj) * kHeadDim;
  };
  const int64_t u = d.unit0 + ul;
  const float qscale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
  WaveLds<GQ, NV>& L = ((WaveLds<GQ, NV>*)smem)[wave];
  const __half* qbase = a.q + row_elem(0);               // also stands in for rows that do not exist
  // A batch of sequences of different lengths: each sequence's own state, read from memory.  The
  // arguments' values bound it (the host has checked them against the buffers), so that whatever
  // the array holds every access below stays inside the buffers.
  Seq sq = {a.n_quant, a.res_start, a.n_res, a.n_res};
  if (a.k_new) sq.n_res += 1;                            // the token being decoded: the newest residual row
  if (a.seq || entry >= 0) {
    const int4 own = entry >= 0 ? planned : *(const int4*)(a.seq + 4 * b);   // uniform: one scalar load
    sq.n_quant = min(max(own.x, 0), a.n_quant) & ~(kBlockTokens - 1);
    sq.res_start = (own.y >= 0 && own.y < d.res_rows) ? own.y & ~15 : 0;   // (a row group of 16 must not wrap)
    sq.n_res = min(max(own.z, 0), a.n_res);
    sq.n_ring = sq.n_res;
  }

  UnitPtrs<PAGED> P;
  P.nblocks = sq.n_quant >> 5;
  P.last_block = max(P.nblocks - 1, 0);
  P.bpg_shift = d.bpg_shift;
  P.block_bytes = (uint32_t)d.block_bytes;
  P.table = PAGED ? d.page_table + (int64_t)b * d.table_stride : nullptr;
  P.n_pages = d.n_pages;
  // the mini-chunks of the quantized segment that are this workgroup's: [mc_begin, mc_end)
  const int n_mc = (sq.n_quant + kMiniChunk - 1) / kMiniChunk;
  const int mc_begin = entry >= 0 ? min(max(plan_mc_begin, 0), n_mc) : split * a.mc_per_split;
  const int mc_end = entry >= 0 ? min(max(plan_mc_end, mc_begin), n_mc) : min(n_mc, (split + 1) * a.mc_per_split);
  int mc = mc_begin + wave;
  // A paged cache: the page numbers of the wave's first two mini-chunks are asked for before
  // everything else, so that the loads of the first mini-chunk can follow as soon as possible
  // (from then on the entries of a mini-chunk are fetched one mini-chunk ahead of its loads).
  typename UnitPtrs<PAGED>::Pages pages_now = {0, 0}, pages_next = {0, 0};
  if constexpr (PAGED) {
    pages_now = P.fetch_pages(mc, lane);
    pages_next = P.fetch_pages(mc + nw, lane);
  }

  // Loads go out in the order their data is needed, and all of them before anything is waited
  // on: the query, the wave's first group of full-precision rows, its first quantized mini-chunk.
  uint32_t qw[GQ];
#pragma unroll
  for (int j = 0; j < GQ; ++j) qw[j] = ((const uint32_t*)(a.q + row_elem(j)))[lane];
  // The rows of the token being decoded, if they come with the call: one wavefront of the unit
  // stores them in the ring at the end (every wavefront loads them, so that all issue the same
  // loads; without such rows the query row is read instead).
  const __half* k_new_row = a.k_new ? a.k_new + (int64_t)ul * kHeadDim : qbase;
  const __half* v_new_row = a.k_new ? a.v_new + (int64_t)ul * kHeadDim : qbase;
  uint32_t k_new_word = ((const uint32_t*)k_new_row)[lane];
  const uint32_t v_new_word = ((const uint32_t*)v_new_row)[lane];
  // the angles of the new token's position, if the launch is to rotate the query and the new Key
  float2 rope_cos = {1.f, 1.f}, rope_sin = {0.f, 0.f};
  if constexpr (ROPE) {
    const float* rope_row = a.rope + (int64_t)b * a.rope_stride;
    rope_cos = ((const float2*)rope_row)[lane & 31];
    rope_sin = ((const float2*)rope_row)[32 + (lane & 31)];
  }

  // full-precision row groups go to the unit's wavefronts from the last one backwards (the
  // first wavefronts of a workgroup are the ones that may hold one more mini-chunk)
  const FpLayout fl = fp_layout(a, sq);
  const int n_rg = fl.groups();
  const int unit_waves = n_splits * nw;
  int rg = unit_waves - 1 - (split * nw + wave);
  const bool has_fp = rg < n_rg;                         // uniform over the wave
  // The unit's slot counts come through the vector memory path, ahead of the rows they qualify:
  // a scalar load in flight would hold up the next wait on the scalar side, which comes before
  // the quantized loads below.
  // Every wavefront issues the same loads, whether or not it has rows or a mini-chunk to work on
  // (a wavefront without a row group loads the unit's first one, one without a mini-chunk the unit's
  // last block): only then are the loads in flight the same on every path, and only then can the
  // waits leave the younger ones in flight.
  FpRegs X;
  int64_t uv = u;
  asm("" : "+v"(uv));                                    // a vector address: a vector load
  int n_pool = a.pool_count[uv];
  int n_aux = a.aux_count[uv];
  if (n_rg > 0) {                                        // (no residual token and no pool slot at all: nothing to load)
    fp_load(X, a, sq, fl, u, k_new_row, has_fp ? rg : 0, lane);
  }

  // Quantized arrays: a dense cache keeps the blocks of unit u together, a paged one those of the
  // plane (layer, kv head); there d.blocks_per_unit and d.groups_per_unit are the plane's.
  const int64_t uq = PAGED ? d.plane0 + h : u;
  P.kc = a.k_codes + uq * d.blocks_per_unit * (int64_t)d.block_bytes;
  P.vc = a.v_codes + uq * d.blocks_per_unit * (int64_t)d.block_bytes;
  P.km = (const unsigned char*)(a.k_meta + uq * d.groups_per_unit * kHeadDim);
  P.vm = (const unsigned char*)a.v_meta + uq * d.blocks_per_unit * (int64_t)(128 * NV);
  P.mask = (const unsigned char*)(a.mask + uq * d.blocks_per_unit);
  const bool has_q = mc < mc_end;                        // uniform over the wave
  McRegs<BITS, NV> R;
  if constexpr (PAGED) P.resolve(mc, pages_now, lane);
  load_k_meta<BITS, NV, SB>(R, P, mc, lane);
  load_codes<BITS>(R.kc, P.kc, P, mc, lane);
  load_v_meta(R, P, mc, lane);
  load_codes<BITS>(R.vc, P.vc, P, mc, lane);

  if constexpr (ROPE) {
#pragma unroll
    for (int j = 0; j < GQ; ++j)
      qw[j] = rope_word(qw[j], (uint32_t)__shfl_xor((int)qw[j], 32), rope_cos, rope_sin, lane >= 32);
    k_new_word = rope_word(k_new_word, (uint32_t)__shfl_xor((int)k_new_word, 32), rope_cos, rope_sin, lane >= 32);
  }
  // this lane's two channels (2*lane, 2*lane+1) of every query head, log2-domain scaled
  float qa[GQ][2];
#pragma unroll
  for (int j = 0; j < GQ; ++j) {
    qa[j][0] = h2f_bits(qw[j] & 0xFFFFu) * qscale;
    qa[j][1] = h2f_bits(qw[j] >> 16) * qscale;
  }

  // ---- full-precision part, while the first quantized loads are in flight --------------------------
  FpAcc<GQ> F;
#pragma unroll
  for (int j = 0; j < GQ; ++j) {
    F.m[j] = kNegBig;
    F.l[j] = 0.f;
    F.o[j][0] = F.o[j][1] = 0.f;
  }
#pragma unroll
  for (int j = 0; j < GQ; ++j) {                         // the query rows, for both parts
    uint32_t hi, lo;
    split_pair(qa[j][0], qa[j][1], hi, lo);
    ((uint32_t*)L.q0[2 * j])[lane] = hi;
    ((uint32_t*)L.q0[2 * j + 1])[lane] = lo;
  }
  wave_sync();
  if (has_fp) {
    n_pool = __builtin_amdgcn_readfirstlane(n_pool);
    n_aux = __builtin_amdgcn_readfirstlane(n_aux);
    fp_compute<GQ, NV, ROPE>(X, F, L, a, sq, fl, n_pool, n_aux, r0, k_new_word, v_new_word, lane);
    for (rg += unit_waves; rg < n_rg; rg += unit_waves) {          // the wavefront's further groups
      fp_load(X, a, sq, fl, u, k_new_row, rg, lane);
      fp_compute<GQ, NV, ROPE>(X, F, L, a, sq, fl, n_pool, n_aux, r0, k_new_word, v_new_word, lane);
    }
  }

  WaveAcc<GQ> S;
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) S.O[ct] = float4v{0.f, 0.f, 0.f, 0.f};
  S.Dz = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < GQ; ++j) S.m[j] = kNegBig;
  if (has_q) {
    // q of this lane's channel pair, scaled for the fp16 split of q*step, as hi + lo
    half2v qh[GQ], ql[GQ];
    const float fs = __builtin_amdgcn_exp2f((float)(kShK - pair_pos<BITS>(lane & 3)));
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      uint32_t hi, lo;
      split_pair(qa[j][0] * fs, qa[j][1] * fs, hi, lo);
      qh[j] = as_half2(hi);
      ql[j] = as_half2(lo);
    }
    // Two wavefronts share a SIMD, and with equal priorities the older of them is served first whenever
    // both have an instruction ready: it runs up to a fifth faster than the younger one, ends early and
    // leaves the SIMD to a single wavefront, which cannot fill it.  Measured on the batch-128 layer: of the
    // four workgroups of a compute unit, the one whose two wavefronts are both the older ones on their SIMDs
    // ended after 67 us, the other three after 82 us.  So the younger wavefront (the one in the second wave
    // slot of its SIMD) takes, from one mini-chunk to the next, a priority above the older one's for three
    // mini-chunks and one below it for two (a mini-chunk at the lower priority lasts longer, so the two
    // spend about the same time favoured): ends of 75 and 81 us, the launch 3 % shorter.  Results do not
    // depend on it: the work of a wavefront is what it was.
    uint32_t wave_slot;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID, 0, 4)" : "=s"(wave_slot));
    const bool younger = wave_slot != 0;
    if (!younger) __builtin_amdgcn_s_setprio(1);
    int turn = 0;
    for (; mc + nw < mc_end; mc += nw) {
      if (younger) {
        if (turn < 3) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(0);
        turn = turn == 4 ? 0 : turn + 1;
      }
      if constexpr (PAGED) {
        const auto pages_after = P.fetch_pages(mc + 2 * nw, lane);
        P.resolve(mc + nw, pages_next, lane);
        pages_next = pages_after;
      }
      compute_minichunk<GQ, BITS, NV, SB, true>(R, S, L, qh, ql, lane, P, mc + nw);
    }
    compute_minichunk<GQ, BITS, NV, SB, false>(R, S, L, qh, ql, lane, P, mc);
  }
  const float post_v = __builtin_amdgcn_exp2f((float)(24 - kShV));
  if (a.k_new && split == 0 && part == 0 && wave == 0) {     // append: the ring row after the live ones
    int row = sq.res_start + sq.n_ring;
    row -= row >= d.res_rows ? d.res_rows : 0;
    ((uint32_t*)(const_cast<__half*>(a.k_res) + (u * d.res_rows + row) * kHeadDim))[lane] = k_new_word;
    ((uint32_t*)(const_cast<__half*>(a.v_res) + (u * d.res_rows + row) * kHeadDim))[lane] = v_new_word;
  }

  // ---- hand both results of the wave to the merge buffer ---------------------------------------------
  __syncthreads();                                       // every wave is done with its WaveLds
  const MergeView<GQ, NV> mg(smem, nw);
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const int j = 2 * r + jj;
    if (j < GQ) {
#pragma unroll
      for (int ct = 0; ct < 8; ++ct)
        mg.o[(wave * GQ + j % GQ) * kHeadDim + 16 * ct + m16] = (S.O[ct][2 * jj] + S.O[ct][2 * jj + 1]) * post_v;
      const float zsum = S.Dz[2 * jj] + S.Dz[2 * jj + 1];
      if (m16 < NV) mg.z[(wave * GQ + j % GQ) * NV + m16 % NV] = zsum;
      if (m16 == NV) mg.l[wave * GQ + j % GQ] = zsum;
    }
  }
#pragma unroll
  for (int j = 0; j < GQ; ++j) {
    *(float2*)&mg.o[((nw + wave) * GQ + j) * kHeadDim + 2 * lane] = float2{F.o[j][0], F.o[j][1]};
    if (lane == 0) {
      mg.m[wave * GQ + j] = S.m[j];
      mg.m[(nw + wave) * GQ + j] = F.m[j];
      mg.l[(nw + wave) * GQ + j] = F.l[j];
    }
  }

  // ---- merge the 2 nw results: the output itself if this workgroup is the unit's only one, else its partial
  __syncthreads();
  const int64_t part_slot0 = part_first >= 0 ? part_first : (int64_t)wl * n_splits;
  float* part_out = a.partials + (part_slot0 + split) * GQ * (kHeadDim + 2);
  for (int i = tid; i < GQ * kHeadDim; i += nthreads) {
    const int j = i / kHeadDim, c = i % kHeadDim;
    const int jv = c / (kHeadDim / NV);
    float m = kNegBig;
    for (int w = 0; w < 2 * nw; ++w) m = fmaxf(m, mg.m[w * GQ + j]);
    float o = 0.f, l = 0.f;
    for (int w = 0; w < nw; ++w) {                       // quantized parts carry their zero-point sums
      const float f = __builtin_amdgcn_exp2f(mg.m[w * GQ + j] - m);
      o += (mg.o[(w * GQ + j) * kHeadDim + c] + mg.z[(w * GQ + j) * NV + jv]) * f;
      l += mg.l[w * GQ + j] * f;
    }
    for (int w = nw; w < 2 * nw; ++w) {
      const float f = __builtin_amdgcn_exp2f(mg.m[w * GQ + j] - m);
      o += mg.o[(w * GQ + j) * kHeadDim + c] * f;
      l += mg.l[w * GQ + j] * f;
    }
    if (n_splits == 1) {
      a.out[row_elem(j) + c] = __float2half_rn(l > 0.f ? o / l : 0.f);
    } else {
      coherent_store(&part_out[j * (kHeadDim + 2) + 2 + c], o);
      if (c == 0) {
        coherent_store(&part_out[j * (kHeadDim + 2) + 0], m);
        coherent_store(&part_out[j * (kHeadDim + 2) + 1], l);
      }
    }
  }
  if (n_splits == 1) return;

  // ---- the last workgroup of the unit to arrive merges the unit's partials ---------------------------
  // Partials and the counter are accessed with device-scope atomic operations (they go to the
  // point where the compute dies' L2 caches agree), so no cache write-back or invalidate is
  // needed.  What orders them is explicit: every thread waits until its own partial stores have
  // been acknowledged at that point (vector-memory counter at zero), then the barrier, then one
  // thread bumps the counter.  A workgroup that finds the counter at n_splits - 1 therefore finds
  // every other workgroup's partials in place; its loads are device-scope too and are issued after
  // the barrier that follows the counter's return.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (tid == 0) {
    const int old = __hip_atomic_fetch_add(&a.counters[wl], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (old == n_splits - 1);
  }
  __syncthreads();
  if (s_last) {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const float* pu = a.partials + part_slot0 * GQ * (kHeadDim + 2);
    constexpr int kBatch = 8;                            // partials fetched per round trip
    for (int i = tid; i < GQ * kHeadDim; i += nthreads) {
      const int j = i / kHeadDim, c = i % kHeadDim;
      const float* pj = pu + j * (kHeadDim + 2);
      float m = kNegBig, l = 0.f, o = 0.f;
      for (int s0 = 0; s0 < n_splits; s0 += kBatch) {
        float pm[kBatch], pl[kBatch], po[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
          const int sidx = min(s0 + k, n_splits - 1);
          const float* ps = pj + (int64_t)sidx * GQ * (kHeadDim + 2);
          pm[k] = coherent_load(&ps[0]);
          pl[k] = coherent_load(&ps[1]);
          po[k] = coherent_load(&ps[2 + c]);
        }
        float mb = m;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) mb = fmaxf(mb, pm[k]);
        const float fo = __builtin_amdgcn_exp2f(m - mb);
        l *= fo;
        o *= fo;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
          const float w = (s0 + k < n_splits) ? __builtin_amdgcn_exp2f(pm[k] - mb) : 0.f;
          l += pl[k] * w;
          o += po[k] * w;
        }
        m = mb;
      }
      a.out[row_elem(j) + c] = __float2half_rn(l > 0.f ? o / l : 0.f);
    }
    if (tid == 0)                                        // leave the counter as it was found
      __hip_atomic_store(&a.counters[wl], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// grid (splits, kv_heads * head_parts, batch), or with a launch plan (entries, kv_heads, 1); 64 * a.nw threads
// (a.nw at most what one compute unit holds of this instance), a.nw * sizeof(WaveLds) bytes of dynamic LDS.
template <int GQ, int BITS, int NV, bool PAGED, int SB, bool ROPE>
__global__ void __launch_bounds__(64 * 4 * kDecodeWavesPerSimd) __attribute__((amdgpu_waves_per_eu(kDecodeWavesPerSimd)))
decode_kernel(DecodeArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_last;
  int entry = -1;
  if (a.plan) {
    entry = blockIdx.x;
    if (entry >= min(a.plan[0], a.plan_entries)) return;
  }
  decode_item<GQ, BITS, NV, PAGED, SB, ROPE>(a, smem, s_last, entry);
}

template <int GQ, int BITS, int NV, bool PAGED, int SB, bool ROPE>
void launch_instance(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  const size_t lds = (size_t)a.nw * sizeof(WaveLds<GQ, NV>);
  static_assert(merge_bytes_per_wave<GQ, NV>() <= (int)sizeof(WaveLds<GQ, NV>), "merge view must fit");
  if (lds > 48 * 1024)     // more than the default limit of dynamic LDS: raise it (cheap, idempotent)
    (void)hipFuncSetAttribute((const void*)decode_kernel<GQ, BITS, NV, PAGED, SB, ROPE>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL((decode_kernel<GQ, BITS, NV, PAGED, SB, ROPE>), grid, dim3(64 * a.nw), lds, s, a);
}
template <int GQ, int BITS, int NV, bool PAGED, int SB>
void launch_shared(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  if (a.rope) launch_instance<GQ, BITS, NV, PAGED, SB, true>(a, grid, s);
  else launch_instance<GQ, BITS, NV, PAGED, SB, false>(a, grid, s);
}
template <int GQ, int BITS, int NV, bool PAGED>
void launch_paged(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  // blocks per Key group: a mini-chunk (four blocks, starting at a multiple of 128 tokens) is four, two or one group
  if (a.d.bpg_shift == 2) launch_shared<GQ, BITS, NV, PAGED, 4>(a, grid, s);
  else if (a.d.bpg_shift == 1) launch_shared<GQ, BITS, NV, PAGED, 2>(a, grid, s);
  else launch_shared<GQ, BITS, NV, PAGED, 1>(a, grid, s);
}
template <int GQ, int BITS, int NV>
void launch_one(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  if (a.d.page_table) launch_paged<GQ, BITS, NV, true>(a, grid, s);
  else launch_paged<GQ, BITS, NV, false>(a, grid, s);
}

template <int GQ, int BITS>
void launch_nv(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  switch (a.d.vgroups) {
    case 4: launch_one<GQ, BITS, 4>(a, grid, s); break;
    case 2: launch_one<GQ, BITS, 2>(a, grid, s); break;
    default: launch_one<GQ, BITS, 1>(a, grid, s); break;
  }
}

template <int GQ>
void launch_bits(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  if (a.d.bits == 2)
    launch_nv<GQ, 2>(a, grid, s);
  else
    launch_nv<GQ, 4>(a, grid, s);
}

// The rotation on its own, for the steps on which the decode launch cannot apply it (a ring that fills:
// the new Key goes through the group step first): one wavefront per row of 128 channels.  A wavefront
// has read its whole row before it writes any of it, so out may be x.
__global__ void __launch_bounds__(256) rope_kernel(const __half* __restrict__ x, int64_t rows, int rows_per_seq,
                                                   const float* __restrict__ rope, int64_t rope_stride,
                                                   __half* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float* rr = rope + (row / rows_per_seq) * rope_stride;
  const float2 c = ((const float2*)rr)[lane & 31], sn = ((const float2*)rr)[32 + (lane & 31)];
  const uint32_t own = ((const uint32_t*)(x + row * kHeadDim))[lane];
  const uint32_t y = rope_word(own, (uint32_t)__shfl_xor((int)own, 32), c, sn, lane >= 32);
  ((uint32_t*)(out + row * kHeadDim))[lane] = y;
}

}  // namespace

hipError_t launch_rope(const __half* x, int64_t rows, int32_t rows_per_seq, const float* rope, int64_t rope_stride,
                       __half* out, hipStream_t s) {
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x, rows, rows_per_seq, rope,
                     rope_stride, out);
  return hipGetLastError();
}

int decode_wave_lds_bytes(int g, int nv) {
  auto of_g = [&](auto gq) -> int {
    constexpr int GQ = decltype(gq)::value;
    return nv == 4 ? (int)sizeof(WaveLds<GQ, 4>) : nv == 2 ? (int)sizeof(WaveLds<GQ, 2>) : (int)sizeof(WaveLds<GQ, 1>);
  };
  switch (g) {
    case 1: return of_g(std::integral_constant<int, 1>{});
    case 2: return of_g(std::integral_constant<int, 2>{});
    case 8: return of_g(std::integral_constant<int, 8>{});
    default: return of_g(std::integral_constant<int, 4>{});
  }
}

hipError_t launch_decode(const DecodeArgs& a, hipStream_t s) {
  const dim3 grid(a.plan ? a.plan_entries : a.splits, a.d.kv_heads * a.head_parts, a.plan ? 1 : a.d.batch);
  switch ((a.q_tokens << a.g_shift) / a.head_parts) {
    case 1: launch_bits<1>(a, grid, s); break;
    case 2: launch_bits<2>(a, grid, s); break;
    case 8: launch_bits<8>(a, grid, s); break;
    default: launch_bits<4>(a, grid, s); break;
  }
  return hipGetLastError();
}

}  // namespace kvq
