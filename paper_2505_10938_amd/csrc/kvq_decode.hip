// Decode-step attention (Eq. 1) over the quantized cache, the residual ring and the outlier
// pools, for gfx950.
//
// Work split: grid = (chunks, kv heads, batch).  A quantized chunk is 512 tokens = 16 packed
// blocks; each of the 4 wavefronts of a workgroup owns 4 blocks (128 tokens) and produces its
// own (max, sum, weighted values); the 4 results are merged through LDS and written as one
// partial per (unit, chunk).  Full-precision chunks (64 rows of residual / pool / auxiliary
// pool) produce partials of the same form.  A second small kernel merges the partials.
//
// Arithmetic: every contraction runs on the matrix cores (v_mfma_f32_16x16x32_f16).
//  * q.K^T:  A = q * step, split in fp16 hi + lo rows (two matrix rows per query head, so the
//            split costs no extra instruction), B = the packed codes themselves.
//  * P.V:    A = p * step (hi + lo rows), B = the packed codes.
//  * zero points: sum_c q_c z_c (one scalar per group and head) is A = q (hi/lo) times B = the
//            fp16 zero plane of the group; sum_t p_t z_t (one scalar per head and value group)
//            and sum_t p_t are A = p (hi/lo) times B = [zero plane | ones].
// A packed code becomes an fp16 operand with ONE `and`: masked in place, a 2-bit code at bits
// [2v, 2v+2) of a half-word is the fp16 subnormal code * 2^(2v-24) (the matrix cores take
// subnormal inputs exactly), and the factor 2^(-2v) is folded into the other operand.
// Scores live in the log2 domain: s = (q . k) * log2(e) / sqrt(d).
#include "kvq_common.h"

namespace kvq {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowBytes = 272;   // LDS row of 128 fp16 + 16 bytes of padding (bank spread)
constexpr int kShK = 6;          // q*step operand is scaled by 2^(kShK - pos) before the fp16 split
constexpr int kShV = 8;          // p*step operand likewise

__device__ inline float h2f_bits(uint32_t bits16) { return __half2float(__ushort_as_half((unsigned short)bits16)); }

// Order LDS traffic between lanes of one wavefront (DS operations of a wave execute in order;
// this only stops the compiler from moving them across).
__device__ inline void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Wave-wide reductions on the DPP path (no LDS traffic): 4 steps inside each row of 16 lanes,
// then row 0->1, 2->3 and rows {0,1}->{2,3}; the total is in lane 63 and is broadcast from there.
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_f(float old, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v),
                                                               CTRL, ROW_MASK, 0xF, false));
}
__device__ inline float wave_max(float v) {
  v = fmaxf(v, dpp_f<0xB1, 0xF>(v, v));    // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_f<0x4E, 0xF>(v, v));    // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp_f<0x141, 0xF>(v, v));   // row_half_mirror
  v = fmaxf(v, dpp_f<0x140, 0xF>(v, v));   // row_mirror
  v = fmaxf(v, dpp_f<0x142, 0xA>(v, v));   // row_bcast:15 into rows 1 and 3
  v = fmaxf(v, dpp_f<0x143, 0xC>(v, v));   // row_bcast:31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ inline float wave_sum(float v) {
  v += dpp_f<0xB1, 0xF>(0.f, v);
  v += dpp_f<0x4E, 0xF>(0.f, v);
  v += dpp_f<0x141, 0xF>(0.f, v);
  v += dpp_f<0x140, 0xF>(0.f, v);
  v += dpp_f<0x142, 0xA>(0.f, v);
  v += dpp_f<0x143, 0xC>(0.f, v);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// fp16 hi/lo split of two floats: hi = fp16(x) (toward zero), lo = fp16(x - hi); packed pairs.
__device__ inline void split_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  const auto h = __builtin_amdgcn_cvt_pkrtz(x0, x1);
  const auto l = __builtin_amdgcn_cvt_pkrtz(x0 - (float)h[0], x1 - (float)h[1]);
  hi = __builtin_bit_cast(uint32_t, h);
  lo = __builtin_bit_cast(uint32_t, l);
}

// Exponent of the power of two carried by pair v (v = lane & 3 on the producing side) of a
// field: a masked code at pair v is worth code * 2^(pos(v) - 24).
template <int BITS>
__device__ inline int pair_pos(int v) { return BITS == 2 ? 2 * v : 4 * (v & 1); }

// One matrix-core operand (8 fp16 = 4 dwords) from field f of a lane's packed words.
template <int BITS>
__device__ inline half8 field_operand(const uint4 (&w)[BITS / 2], int f) {
  u32x4 o;
  const uint32_t* p = (const uint32_t*)&w[0];
  if (BITS == 2) {
    const uint32_t x = (f & 1) ? (p[f >> 1] >> 8) : p[f >> 1];
    o[0] = x & 0x00030003u;
    o[1] = x & 0x000C000Cu;
    o[2] = x & 0x00300030u;
    o[3] = x & 0x00C000C0u;
  } else {
    const uint32_t x = p[f], y = p[f] >> 8;
    o[0] = x & 0x000F000Fu;
    o[1] = x & 0x00F000F0u;
    o[2] = y & 0x000F000Fu;
    o[3] = y & 0x00F000F0u;
  }
  return __builtin_bit_cast(half8, o);
}

__device__ inline half8 lds_operand(const unsigned char* row, int byte) {
  return __builtin_bit_cast(half8, *(const u32x4*)(row + byte));
}

template <int GQ, int NV>
struct WaveLds {
  union {                                      // aop is dead once the scores are written
    unsigned char aop[2 * GQ][kRowBytes];      // q-side operand rows: hi/lo per head, 128 channels
    unsigned char pp[2 * GQ][kRowBytes];       // p rows (hi/lo per head), 128 tokens
  };
  unsigned char ps[NV][2 * GQ][kRowBytes];     // p*step rows per value group (hi/lo per head), 128 tokens
  float sc[GQ][128];                           // scores of the wave's 128 tokens
  float qz[4][GQ];                             // sum_c q_c z_c per (block, head)
};

template <int GQ, int NV>
struct MergeLds {
  float m[4][GQ], l[4][GQ];
  float z[4][GQ][NV];                          // sum_t p_t z_t per value group
  float o[4][GQ][kHeadDim];
};

template <int GQ, int NV>
union DecodeLds {
  WaveLds<GQ, NV> w[4];
  MergeLds<GQ, NV> mg;
};

// ---- merge the 4 wavefronts' results and write the chunk partial --------------------------------
template <int GQ, int NV>
__device__ inline void merge_and_store(MergeLds<GQ, NV>& mg, float* part, int tid) {
  __syncthreads();
  for (int i = tid; i < GQ * kHeadDim; i += 256) {
    const int j = i / kHeadDim, c = i % kHeadDim;
    const int jv = c / (kHeadDim / NV);
    const float m = fmaxf(fmaxf(mg.m[0][j], mg.m[1][j]), fmaxf(mg.m[2][j], mg.m[3][j]));
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = __builtin_amdgcn_exp2f(mg.m[w][j] - m);
      o += (mg.o[w][j][c] + mg.z[w][j][jv]) * f;
      l += mg.l[w][j] * f;
    }
    part[j * (kHeadDim + 2) + 2 + c] = o;
    if (c == 0) {
      part[j * (kHeadDim + 2) + 0] = m;
      part[j * (kHeadDim + 2) + 1] = l;
    }
  }
}

// grid (chunks_q + chunks_fp, kv_heads, batch), 256 threads
template <int GQ, int BITS, int NV>
__global__ void __launch_bounds__(256) decode_partial_kernel(DecodeArgs a) {
  __shared__ __align__(16) DecodeLds<GQ, NV> lds;
  const Dims& d = a.d;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m16 = lane & 15, r = lane >> 4;
  const int chunk = blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z;
  const int ul = b * d.kv_heads + h;
  const int64_t u = d.unit0 + ul;
  const float qscale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
  constexpr int R2 = 2 * GQ;                  // operand rows in use
  const int arow = m16 % R2;                  // rows beyond 2*GQ repeat valid rows (their results are unused)
  WaveLds<GQ, NV>& L = lds.w[wave];
  const __half* qbase = a.q + ((int64_t)b * d.q_heads + (int64_t)h * GQ) * kHeadDim;
  float* part = a.partials + ((int64_t)ul * (a.chunks_q + a.chunks_fp) + chunk) * GQ * (kHeadDim + 2);

  // this lane's two channels (2*lane, 2*lane+1) of every query head, log2-domain scaled
  float qa[GQ][2];
#pragma unroll
  for (int j = 0; j < GQ; ++j) {
    const uint32_t w2 = ((const uint32_t*)(qbase + j * kHeadDim))[lane];
    qa[j][0] = h2f_bits(w2 & 0xFFFFu) * qscale;
    qa[j][1] = h2f_bits(w2 >> 16) * qscale;
  }

  if (chunk < a.chunks_q) {
    // =================================== quantized chunk ===================================
    const int nblocks = a.n_quant >> 5;
    const int blk0 = chunk * (kChunkTokens / 32) + wave * 4;          // first block of this wave
    // Blocks past the end are replaced by the last block with every token masked, so that all
    // waves run the same straight-line code.
    int blk[4];
    uint32_t mk[4];
    uint4 kc[4][BITS / 2], vc[4][BITS / 2];
    uint32_t ksp[4];                                                  // this lane's two Key steps
    const unsigned char* kmeta_g[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = blk0 + i < nblocks;
      blk[i] = min(blk0 + i, nblocks - 1);
      const int64_t gb = u * d.blocks_per_unit + blk[i];
      const uint4* kp = (const uint4*)(a.k_codes + gb * d.block_bytes) + lane;
      const uint4* vp = (const uint4*)(a.v_codes + gb * d.block_bytes) + lane;
#pragma unroll
      for (int hf = 0; hf < BITS / 2; ++hf) {
        kc[i][hf] = kp[hf * 64];
        vc[i][hf] = vp[hf * 64];
      }
      kmeta_g[i] = (const unsigned char*)(a.k_meta + (u * d.groups_per_unit + (blk[i] >> d.bpg_shift)) * kHeadDim);
      ksp[i] = ((const uint32_t*)kmeta_g[i])[lane];
      const uint32_t mw_ = a.mask[gb];
      mk[i] = ok ? mw_ : 0xFFFFFFFFu;
    }
    // Value steps of this lane's two tokens (pair lane&15 of block lane>>4): NV dwords (s_t0, s_t1)
    uint32_t vsp[NV];
    const unsigned char* vmeta_b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      vmeta_b[i] = (const unsigned char*)a.v_meta + (u * d.blocks_per_unit + blk[i]) * (int64_t)(128 * NV);
    {
      const int bi = lane >> 4;
      const unsigned char* vb = bi == 0 ? vmeta_b[0] : (bi == 1 ? vmeta_b[1] : (bi == 2 ? vmeta_b[2] : vmeta_b[3]));
      const uint32_t* p = (const uint32_t*)(vb + (lane & 15) * 4 * NV);
#pragma unroll
      for (int jv = 0; jv < NV; ++jv) vsp[jv] = p[jv];
    }

    // ---- q rows (hi/lo, no step) -> sum_c q_c z_c of the 4 blocks in one pass: column n of the
    //      B operand is the zero plane of block n's group -----------------------------------------
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      uint32_t hi, lo;
      split_pair(qa[j][0], qa[j][1], hi, lo);
      ((uint32_t*)L.aop[2 * j])[lane] = hi;
      ((uint32_t*)L.aop[2 * j + 1])[lane] = lo;
    }
    wave_sync();
    {
      float4v Dq = {0.f, 0.f, 0.f, 0.f};
      const unsigned char* zg = m16 == 0 ? kmeta_g[0] : (m16 == 1 ? kmeta_g[1] : (m16 == 2 ? kmeta_g[2] : kmeta_g[3]));
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const uint4 zz = m16 < 4 ? *(const uint4*)(zg + 256 + cb * 64 + r * 16) : uint4{0, 0, 0, 0};
        Dq = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds_operand(L.aop[arow], cb * 64 + r * 16),
                                                    __builtin_bit_cast(half8, zz), Dq, 0, 0, 0);
      }
      if (m16 < 4) {
        if (2 * r < GQ) L.qz[m16][2 * r] = Dq[0] + Dq[1];
        if (2 * r + 1 < GQ) L.qz[m16][(2 * r + 1) % GQ] = Dq[2] + Dq[3];
      }
    }

    // ---- scores of the wave's 4 blocks ------------------------------------------------------------
    const float post_k = __builtin_amdgcn_exp2f((float)(24 - kShK));
    {
      const float fs = __builtin_amdgcn_exp2f((float)(kShK - pair_pos<BITS>(lane & 3)));
      float qaf[GQ][2];
#pragma unroll
      for (int j = 0; j < GQ; ++j) {
        qaf[j][0] = qa[j][0] * fs;
        qaf[j][1] = qa[j][1] * fs;
      }
      half8 aq[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if ((i & ((1 << d.bpg_shift) - 1)) == 0) {      // first block of a Key group: new q*step rows
          const float s0 = h2f_bits(ksp[i] & 0xFFFFu), s1 = h2f_bits(ksp[i] >> 16);
          wave_sync();                                   // earlier reads of aop are done
#pragma unroll
          for (int j = 0; j < GQ; ++j) {
            uint32_t hi, lo;
            split_pair(qaf[j][0] * s0, qaf[j][1] * s1, hi, lo);
            ((uint32_t*)L.aop[2 * j])[lane] = hi;
            ((uint32_t*)L.aop[2 * j + 1])[lane] = lo;
          }
          wave_sync();
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) aq[cb] = lds_operand(L.aop[arow], cb * 64 + r * 16);
        }
#pragma unroll
        for (int th = 0; th < 2; ++th) {
          float4v D = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            D = __builtin_amdgcn_mfma_f32_16x16x32_f16(aq[cb], field_operand<BITS>(kc[i], 4 * th + cb), D, 0, 0, 0);
          const int tl = i * 32 + th * 16 + m16;
          if (2 * r < GQ) L.sc[2 * r][tl] = (D[0] + D[1]) * post_k;
          if (2 * r + 1 < GQ) L.sc[(2 * r + 1) % GQ][tl] = (D[2] + D[3]) * post_k;
        }
      }
    }
    wave_sync();

    // ---- softmax numerators of the wave's 128 tokens; p and p*step operand rows ----------------
    float mw[GQ];
    {
      const int bi = lane >> 4;                         // block of this lane's tokens (2*lane, 2*lane+1)
      const uint32_t mword = bi == 0 ? mk[0] : (bi == 1 ? mk[1] : (bi == 2 ? mk[2] : mk[3]));
      const int bit = (2 * lane) & 31;
      const bool ok0 = !((mword >> bit) & 1u);
      const bool ok1 = !((mword >> (bit + 1)) & 1u);
      const float fv = __builtin_amdgcn_exp2f((float)(kShV - pair_pos<BITS>(lane & 3)));
#pragma unroll
      for (int j = 0; j < GQ; ++j) {
        const float2 s2 = *(const float2*)&L.sc[j][2 * lane];
        const float qz = L.qz[bi][j];
        const float x0 = ok0 ? s2.x + qz : kNegBig;
        const float x1 = ok1 ? s2.y + qz : kNegBig;
        const float m = wave_max(fmaxf(x0, x1));
        const float p0 = ok0 ? __builtin_amdgcn_exp2f(x0 - m) : 0.f;
        const float p1 = ok1 ? __builtin_amdgcn_exp2f(x1 - m) : 0.f;
        mw[j] = m;
        uint32_t hi, lo;
        split_pair(p0, p1, hi, lo);
        ((uint32_t*)L.pp[2 * j])[lane] = hi;
        ((uint32_t*)L.pp[2 * j + 1])[lane] = lo;
        const float p0f = p0 * fv, p1f = p1 * fv;
#pragma unroll
        for (int jv = 0; jv < NV; ++jv) {
          split_pair(p0f * h2f_bits(vsp[jv] & 0xFFFFu), p1f * h2f_bits(vsp[jv] >> 16), hi, lo);
          ((uint32_t*)L.ps[jv][2 * j])[lane] = hi;
          ((uint32_t*)L.ps[jv][2 * j + 1])[lane] = lo;
        }
      }
    }
    wave_sync();

    // ---- weighted values; sum_t p_t z_t and sum_t p_t ride along as one more product ---------------
    float4v O[8];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) O[ct] = float4v{0.f, 0.f, 0.f, 0.f};
    float4v Dz = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // B operand of the side product: column n < NV = zeros of value group n (8 tokens 8r..8r+7),
      // column NV = ones, other columns 0
      const uint4 zz = m16 < NV ? *(const uint4*)(vmeta_b[i] + 64 * NV + m16 * 64 + r * 16)
                                : (m16 == NV ? uint4{0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u}
                                             : uint4{0, 0, 0, 0});
      Dz = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds_operand(L.pp[arow], i * 64 + r * 16),
                                                  __builtin_bit_cast(half8, zz), Dz, 0, 0, 0);
      half8 ap[NV];
#pragma unroll
      for (int jv = 0; jv < NV; ++jv) ap[jv] = lds_operand(L.ps[jv][arow], i * 64 + r * 16);
#pragma unroll
      for (int ct = 0; ct < 8; ++ct)
        O[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ap[ct * NV / 8], field_operand<BITS>(vc[i], ct), O[ct], 0, 0, 0);
    }
    const float post_v = __builtin_amdgcn_exp2f((float)(24 - kShV));

    // ---- hand the wave's result to the merge buffer --------------------------------------------------
    __syncthreads();                                     // every wave is done with its WaveLds
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int j = 2 * r + jj;
      if (j < GQ) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) lds.mg.o[wave][j % GQ][16 * ct + m16] = (O[ct][2 * jj] + O[ct][2 * jj + 1]) * post_v;
        const float zsum = Dz[2 * jj] + Dz[2 * jj + 1];
        if (m16 < NV) lds.mg.z[wave][j % GQ][m16 % NV] = zsum;
        if (m16 == NV) lds.mg.l[wave][j % GQ] = zsum;
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < GQ; ++j) lds.mg.m[wave][j] = mw[j];
    }
    merge_and_store<GQ, NV>(lds.mg, part, tid);
  } else {
    // ============================== full-precision chunk ===============================
    // 64 rows per workgroup, 16 per wavefront: residual ring rows, then pool slots, then
    // auxiliary slots.  q.k^T on the matrix cores (K rows are the B operand as they are);
    // the weighted values on the vector units (row-major V has the wrong operand shape).
    const int row0 = (chunk - a.chunks_q) * kFpChunkRows + wave * 16;
    const int n_pool = a.pool_count[u], n_aux = a.aux_count[u];
    // Row index -> element offset of the row inside (k_res | pool_k), or -1 for an empty slot.
    // Branch-free so that all 16 + 4 loads of the wave are issued before anything is waited on.
    const int64_t res_base = u * d.res_rows, pool_base = u * d.pool_slots;
    auto row_off = [&](int row, bool& in_res) -> int64_t {
      in_res = row < a.n_res;
      int ring = a.res_start + row;
      ring -= ring >= d.res_rows ? d.res_rows : 0;
      const int slot = row - a.n_res;
      const bool ok = in_res || (slot < d.N ? (slot < n_pool) : (slot < d.pool_slots && slot - d.N < n_aux));
      const int64_t off = in_res ? (res_base + ring) * kHeadDim : (pool_base + slot) * kHeadDim;
      return ok ? off : (int64_t)-1;
    };
    // K row of this lane's token (row0 + m16): 4 x 16 bytes, channels 32cb + 8r ..
    bool kres;
    const int64_t koff = row_off(row0 + m16, kres);
    const __half* krow = (kres ? a.k_res : a.pool_k) + (koff < 0 ? 0 : koff);
    uint4 kf[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) kf[cb] = koff >= 0 ? *(const uint4*)(krow + cb * 32 + r * 8) : uint4{0, 0, 0, 0};
    // V rows of the wave's 16 tokens, this lane's channel pair (2*lane, 2*lane+1)
    uint32_t vw[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      bool vres;
      const int64_t voff = row_off(row0 + t, vres);                 // uniform over the wave
      const __half* vrow = (vres ? a.v_res : a.pool_v) + (voff < 0 ? 0 : voff);
      vw[t] = voff >= 0 ? ((const uint32_t*)vrow)[lane] : 0u;
    }
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      uint32_t hi, lo;
      split_pair(qa[j][0], qa[j][1], hi, lo);
      ((uint32_t*)L.aop[2 * j])[lane] = hi;
      ((uint32_t*)L.aop[2 * j + 1])[lane] = lo;
    }
    wave_sync();
    float4v D = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
      D = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds_operand(L.aop[arow], cb * 64 + r * 16),
                                                  __builtin_bit_cast(half8, kf[cb]), D, 0, 0, 0);
    if (2 * r < GQ) L.sc[2 * r][m16] = D[0] + D[1];
    if (2 * r + 1 < GQ) L.sc[(2 * r + 1) % GQ][m16] = D[2] + D[3];
    wave_sync();
    // softmax numerators of the 16 rows (lanes 0..15 hold one row each), kept in LDS as fp32
    const bool okrow = (koff >= 0) && lane < 16;         // for lanes 0..15, m16 == lane
    float mw[GQ], lw[GQ];
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      const float x = okrow ? L.sc[j][lane & 15] : kNegBig;
      const float m = wave_max(x);
      const float p = okrow ? __builtin_amdgcn_exp2f(x - m) : 0.f;
      mw[j] = m;
      lw[j] = wave_sum(p);
      if (lane < 16) L.sc[j][16 + lane] = p;
    }
    wave_sync();
    // weighted values: lane = channel pair (2*lane, 2*lane+1); empty slots have p = 0 and v = 0
    float ov[GQ][2];
#pragma unroll
    for (int j = 0; j < GQ; ++j) ov[j][0] = ov[j][1] = 0.f;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const float v0 = h2f_bits(vw[t] & 0xFFFFu), v1 = h2f_bits(vw[t] >> 16);
#pragma unroll
      for (int j = 0; j < GQ; ++j) {
        const float p = L.sc[j][16 + t];
        ov[j][0] += p * v0;
        ov[j][1] += p * v1;
      }
    }
    __syncthreads();                                     // every wave is done with its WaveLds
#pragma unroll
    for (int j = 0; j < GQ; ++j) {
      *(float2*)&lds.mg.o[wave][j][2 * lane] = float2{ov[j][0], ov[j][1]};
      if (lane < NV) lds.mg.z[wave][j][lane % NV] = 0.f;
      if (lane == 0) {
        lds.mg.m[wave][j] = mw[j];
        lds.mg.l[wave][j] = lw[j];
      }
    }
    merge_and_store<GQ, NV>(lds.mg, part, tid);
  }
}

// grid (g, units_per_layer), 128 threads: merge chunk partials of one query head.
__global__ void __launch_bounds__(128) decode_combine_kernel(DecodeArgs a) {
  const Dims& d = a.d;
  const int j = blockIdx.x, ul = blockIdx.y, c = threadIdx.x;
  const int b = ul / d.kv_heads, h = ul - b * d.kv_heads;
  const int n_chunks = a.chunks_q + a.chunks_fp;
  const float* part = a.partials + (int64_t)ul * n_chunks * d.g * (kHeadDim + 2) + j * (kHeadDim + 2);
  const int64_t stride = (int64_t)d.g * (kHeadDim + 2);
  float m = kNegBig;
  for (int i = 0; i < n_chunks; ++i) m = fmaxf(m, part[i * stride]);
  float l = 0.f, o = 0.f;
  for (int i = 0; i < n_chunks; ++i) {
    const float w = exp2f(part[i * stride] - m);
    l += part[i * stride + 1] * w;
    o += part[i * stride + 2 + c] * w;
  }
  a.out[((int64_t)b * d.q_heads + h * d.g + j) * kHeadDim + c] = __float2half_rn(o / l);
}

template <int GQ, int BITS>
void launch_partial_nv(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  switch (a.d.vgroups) {
    case 4: hipLaunchKernelGGL((decode_partial_kernel<GQ, BITS, 4>), grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((decode_partial_kernel<GQ, BITS, 2>), grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((decode_partial_kernel<GQ, BITS, 1>), grid, dim3(256), 0, s, a); break;
  }
}

template <int GQ>
void launch_partial_bits(const DecodeArgs& a, dim3 grid, hipStream_t s) {
  if (a.d.bits == 2)
    launch_partial_nv<GQ, 2>(a, grid, s);
  else
    launch_partial_nv<GQ, 4>(a, grid, s);
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, hipStream_t s) {
  const dim3 grid(a.chunks_q + a.chunks_fp, a.d.kv_heads, a.d.batch);
  switch (a.d.g) {
    case 1: launch_partial_bits<1>(a, grid, s); break;
    case 2: launch_partial_bits<2>(a, grid, s); break;
    case 4: launch_partial_bits<4>(a, grid, s); break;
    default: launch_partial_bits<8>(a, grid, s); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_combine_kernel, dim3(a.d.g, a.d.units_per_layer), dim3(128), 0, s, a);
  return hipGetLastError();
}

}  // namespace kvq
