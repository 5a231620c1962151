// Decode-step attention (Eq. 1) over the quantized cache, the residual ring and the outlier
// pools, for gfx950.
//
// Work split: grid = (chunks, units of the layer).  A quantized chunk is 512 tokens = 16 packed
// blocks; each of the 4 wavefronts of a workgroup owns 4 blocks (128 tokens) and produces its
// own (max, sum, weighted values); the 4 results are merged through LDS and written as one
// partial per (unit, chunk).  Full-precision chunks (64 rows of residual / pool / auxiliary
// pool) produce partials of the same form.  A second small kernel merges the partials.
//
// Arithmetic: both contractions run on the matrix cores (v_mfma_f32_16x16x32_f16).
//  * q.K^T:  A = q * step, split in fp16 hi + lo rows (two matrix rows per query head, so the
//            split costs no extra instruction), B = the packed codes themselves.
//  * P.V:    A = p * step (hi + lo rows), B = the packed codes.
// A packed code becomes an fp16 operand with ONE `and`: masked in place, a 2-bit code at bits
// [2v, 2v+2) of a half-word is the fp16 subnormal code * 2^(2v-24) (the matrix cores take
// subnormal inputs exactly), and the factor 2^(-2v) is folded into the other operand.  Zero
// points never touch the codes: sum_c q_c z_c is one scalar per (group, head) and
// sum_t p_t z_t one scalar per (head, value group).
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

__device__ inline float wave_max(float v) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
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
  if (BITS == 2) {
    const uint32_t* p = (const uint32_t*)&w[0];
    const uint32_t x = (f & 1) ? (p[f >> 1] >> 8) : p[f >> 1];
    o[0] = x & 0x00030003u;
    o[1] = x & 0x000C000Cu;
    o[2] = x & 0x00300030u;
    o[3] = x & 0x00C000C0u;
  } else {
    const uint32_t* p = (const uint32_t*)&w[0];
    const uint32_t x = p[f], y = p[f] >> 8;
    o[0] = x & 0x000F000Fu;
    o[1] = x & 0x00F000F0u;
    o[2] = y & 0x000F000Fu;
    o[3] = y & 0x00F000F0u;
  }
  return __builtin_bit_cast(half8, o);
}

template <int GQ, int NV>
struct WaveLds {
  unsigned char aop[2 * GQ][kRowBytes];        // q-side operand rows: hi/lo per head, 128 channels
  float sc[GQ][128];                           // scores of the wave's 128 tokens
  unsigned char ps[NV][2 * GQ][kRowBytes];     // p*step operand rows per value group: 128 tokens
  float qz[4][GQ];                             // sum_c q_c z_c per (block, head)
};

template <int GQ>
struct MergeLds {
  float m[4][GQ], l[4][GQ];
  float o[4][GQ][kHeadDim];
};

template <int GQ, int NV>
union DecodeLds {
  WaveLds<GQ, NV> w[4];
  MergeLds<GQ> mg;
};

// ---- merge the 4 wavefronts' results and write the chunk partial --------------------------------
template <int GQ>
__device__ inline void merge_and_store(MergeLds<GQ>& mg, float* part, int tid) {
  __syncthreads();
  for (int i = tid; i < GQ * kHeadDim; i += 256) {
    const int j = i / kHeadDim, c = i - j * kHeadDim;
    const float m = fmaxf(fmaxf(mg.m[0][j], mg.m[1][j]), fmaxf(mg.m[2][j], mg.m[3][j]));
    float o = 0.f, l = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float f = exp2f(mg.m[w][j] - m);
      o += mg.o[w][j][c] * f;
      l += mg.l[w][j] * f;
    }
    part[j * (kHeadDim + 2) + 2 + c] = o;
    if (c == 0) {
      part[j * (kHeadDim + 2) + 0] = m;
      part[j * (kHeadDim + 2) + 1] = l;
    }
  }
}

// grid (chunks_q + chunks_fp, units_per_layer), 256 threads
template <int GQ, int BITS, int NV>
__global__ void __launch_bounds__(256) decode_partial_kernel(DecodeArgs a) {
  __shared__ __align__(16) DecodeLds<GQ, NV> lds;
  const Dims& d = a.d;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m16 = lane & 15, r = lane >> 4;
  const int chunk = blockIdx.x;
  const int ul = blockIdx.y;
  const int64_t u = d.unit0 + ul;
  const int b = ul / d.kv_heads, h = ul - b * d.kv_heads;
  const float qscale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
  constexpr int R2 = 2 * GQ;                  // operand rows in use
  const int arow = m16 % R2;                  // rows beyond 2*GQ repeat valid rows (their results are unused)
  WaveLds<GQ, NV>& L = lds.w[wave];
  const __half* qbase = a.q + ((int64_t)b * d.q_heads + (int64_t)h * GQ) * kHeadDim;

  // per-wave results in the matrix-core output layout: lane (n = m16, r) holds rows 4r..4r+3,
  // i.e. heads 2r (hi, lo) and 2r+1 (hi, lo), for column n of each of the 8 channel tiles
  float4v O[8];
  for (int ct = 0; ct < 8; ++ct) O[ct] = float4v{0.f, 0.f, 0.f, 0.f};
  float mw[GQ], lw[GQ];
  float ozero[2][NV];                          // sum_t p_t z_t of heads 2r, 2r+1 per value group
  for (int jj = 0; jj < 2; ++jj)
    for (int jv = 0; jv < NV; ++jv) ozero[jj][jv] = 0.f;
  float post_v = 1.f;

  if (chunk < a.chunks_q) {
    // =================================== quantized chunk ===================================
    const int blk0 = chunk * (kChunkTokens / 32) + wave * 4;          // first block of this wave
    const int nb = max(0, min(4, a.n_quant / 32 - blk0));             // blocks that exist
    const int bpg = d.G / 32;                                         // blocks per Key group
    const int t0w = blk0 * 32;                                        // first token of this wave

    // ---- issue every global load of the wave up front ----------------------------------------
    uint4 kc[4][BITS / 2], vc[4][BITS / 2];
    uint2 km[4];
    uint32_t mk[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = i < nb;
      const int64_t blk = (u * d.blocks_per_unit + blk0 + (ok ? i : 0));
      const uint4* kp = (const uint4*)(a.k_codes + blk * d.block_bytes) + lane;
      const uint4* vp = (const uint4*)(a.v_codes + blk * d.block_bytes) + lane;
      for (int hf = 0; hf < BITS / 2; ++hf) {
        kc[i][hf] = ok ? kp[hf * 64] : uint4{0, 0, 0, 0};
        vc[i][hf] = ok ? vp[hf * 64] : uint4{0, 0, 0, 0};
      }
      const int gidx = (blk0 + (ok ? i : 0)) / bpg;
      km[i] = ok ? ((const uint2*)(a.k_meta + (u * d.groups_per_unit + gidx) * kHeadDim))[lane] : uint2{0, 0};
      mk[i] = ok ? a.mask[u * d.blocks_per_unit + blk0 + i] : 0xFFFFFFFFu;
    }
    // Value meta of this lane's two tokens (2*lane, 2*lane + 1 of the wave's 128)
    uint32_t vm[2][NV];
    {
      const bool ok = (lane >> 4) < nb;
      const uint32_t* p = a.v_meta + (u * d.max_seq + t0w + 2 * lane) * NV;
      for (int e = 0; e < 2; ++e)
        for (int jv = 0; jv < NV; ++jv) vm[e][jv] = ok ? p[e * NV + jv] : 0u;
    }
    // this lane's two channels (2*lane, 2*lane+1) of every query head, for the operand rows
    float qa[GQ][2], qaf[GQ][2];
    {
      const float fs = exp2f((float)(kShK - pair_pos<BITS>(lane & 3)));
      for (int j = 0; j < GQ; ++j) {
        const uint32_t w2 = ((const uint32_t*)(qbase + j * kHeadDim))[lane];
        qa[j][0] = h2f_bits(w2 & 0xFFFFu) * qscale;
        qa[j][1] = h2f_bits(w2 >> 16) * qscale;
        qaf[j][0] = qa[j][0] * fs;
        qaf[j][1] = qa[j][1] * fs;
      }
    }

    // ---- scores of the wave's blocks ------------------------------------------------------------
    const float post_k = exp2f((float)(24 - kShK));
    half8 aq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i >= nb) continue;
      if (i % bpg == 0) {
        const float s0 = h2f_bits(km[i].x & 0xFFFFu), z0 = h2f_bits(km[i].x >> 16);
        const float s1 = h2f_bits(km[i].y & 0xFFFFu), z1 = h2f_bits(km[i].y >> 16);
        wave_sync();                                   // earlier reads of aop are done
        for (int j = 0; j < GQ; ++j) {
          uint32_t hi, lo;
          split_pair(qaf[j][0] * s0, qaf[j][1] * s1, hi, lo);
          ((uint32_t*)L.aop[2 * j])[lane] = hi;
          ((uint32_t*)L.aop[2 * j + 1])[lane] = lo;
          const float zs = wave_sum(qa[j][0] * z0 + qa[j][1] * z1);
          for (int k = i; k < i + bpg && k < 4; ++k)
            if (lane == 0) L.qz[k][j] = zs;
        }
        wave_sync();
        for (int cb = 0; cb < 4; ++cb)
          aq[cb] = __builtin_bit_cast(half8, *(const u32x4*)(L.aop[arow] + cb * 64 + r * 16));
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
    wave_sync();

    // ---- softmax numerators of the wave's 128 tokens; p*step operand rows ---------------------
    {
      const int bi = lane >> 4;                         // block of this lane's tokens
      const bool inb = bi < nb;
      const uint32_t mword = mk[0] * (bi == 0) + mk[1] * (bi == 1) + mk[2] * (bi == 2) + mk[3] * (bi == 3);
      const int bit = (2 * lane) & 31;
      const bool ok0 = inb && !((mword >> bit) & 1u);
      const bool ok1 = inb && !((mword >> (bit + 1)) & 1u);
      const float fv = exp2f((float)(kShV - pair_pos<BITS>(lane & 3)));
      float sv[2][NV], zv[2][NV];
      for (int e = 0; e < 2; ++e)
        for (int jv = 0; jv < NV; ++jv) {
          sv[e][jv] = h2f_bits(vm[e][jv] & 0xFFFFu) * fv;
          zv[e][jv] = h2f_bits(vm[e][jv] >> 16);
        }
      float pz[GQ][NV];
      for (int j = 0; j < GQ; ++j) {
        const float2 s2 = *(const float2*)&L.sc[j][2 * lane];
        const float qz = inb ? L.qz[bi][j] : 0.f;
        const float x0 = ok0 ? s2.x + qz : kNegBig;
        const float x1 = ok1 ? s2.y + qz : kNegBig;
        const float m = wave_max(fmaxf(x0, x1));
        const float p0 = ok0 ? exp2f(x0 - m) : 0.f;
        const float p1 = ok1 ? exp2f(x1 - m) : 0.f;
        mw[j] = m;
        lw[j] = wave_sum(p0 + p1);
        for (int jv = 0; jv < NV; ++jv) {
          uint32_t hi, lo;
          split_pair(p0 * sv[0][jv], p1 * sv[1][jv], hi, lo);
          ((uint32_t*)L.ps[jv][2 * j])[lane] = hi;
          ((uint32_t*)L.ps[jv][2 * j + 1])[lane] = lo;
          pz[j][jv] = wave_sum(p0 * zv[0][jv] + p1 * zv[1][jv]);
        }
      }
      for (int jj = 0; jj < 2; ++jj)
        for (int jv = 0; jv < NV; ++jv) {
          float z = 0.f;
          for (int j = 0; j < GQ; ++j) z = (j == 2 * r + jj) ? pz[j][jv] : z;
          ozero[jj][jv] = z;
        }
    }
    wave_sync();

    // ---- weighted values --------------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i >= nb) continue;
      half8 ap[NV];
      for (int jv = 0; jv < NV; ++jv)
        ap[jv] = __builtin_bit_cast(half8, *(const u32x4*)(L.ps[jv][arow] + i * 64 + r * 16));
#pragma unroll
      for (int ct = 0; ct < 8; ++ct)
        O[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ap[ct * NV / 8], field_operand<BITS>(vc[i], ct), O[ct], 0, 0, 0);
    }
    post_v = exp2f((float)(24 - kShV));
  } else {
    // ============================== full-precision chunk ===============================
    // 64 rows per workgroup, 16 per wavefront: residual ring rows, then pool slots, then
    // auxiliary slots.  q.k^T on the matrix cores (K rows are the B operand as they are);
    // the weighted values on the vector units (row-major V has the wrong operand shape).
    const int row0 = (chunk - a.chunks_q) * kFpChunkRows + wave * 16;
    const int n_pool = a.pool_count[u], n_aux = a.aux_count[u];
    auto row_ptr = [&](int row, const __half*& kr, const __half*& vr) {
      kr = nullptr;
      vr = nullptr;
      if (row < a.n_res) {
        const int64_t ring = (a.res_start + row) % d.res_rows;
        kr = a.k_res + (u * d.res_rows + ring) * kHeadDim;
        vr = a.v_res + (u * d.res_rows + ring) * kHeadDim;
      } else {
        const int slot = row - a.n_res;
        const bool ok = slot < d.N ? (slot < n_pool) : (slot < d.pool_slots && slot - d.N < n_aux);
        if (ok) {
          kr = a.pool_k + (u * d.pool_slots + slot) * kHeadDim;
          vr = a.pool_v + (u * d.pool_slots + slot) * kHeadDim;
        }
      }
    };
    // K rows of this lane's token (row0 + m16): 4 x 16 bytes, channels 32cb + 8r ..
    const __half *krow, *vrow_unused;
    row_ptr(row0 + m16, krow, vrow_unused);
    uint4 kf[4];
    for (int cb = 0; cb < 4; ++cb) kf[cb] = krow ? *(const uint4*)(krow + cb * 32 + r * 8) : uint4{0, 0, 0, 0};
    // q operand rows (hi/lo of q * log2e/sqrt(d)), no group scale
    for (int j = 0; j < GQ; ++j) {
      const uint32_t w2 = ((const uint32_t*)(qbase + j * kHeadDim))[lane];
      uint32_t hi, lo;
      split_pair(h2f_bits(w2 & 0xFFFFu) * qscale, h2f_bits(w2 >> 16) * qscale, hi, lo);
      ((uint32_t*)L.aop[2 * j])[lane] = hi;
      ((uint32_t*)L.aop[2 * j + 1])[lane] = lo;
    }
    wave_sync();
    float4v D = {0.f, 0.f, 0.f, 0.f};
    for (int cb = 0; cb < 4; ++cb) {
      const half8 aqv = __builtin_bit_cast(half8, *(const u32x4*)(L.aop[arow] + cb * 64 + r * 16));
      D = __builtin_amdgcn_mfma_f32_16x16x32_f16(aqv, __builtin_bit_cast(half8, kf[cb]), D, 0, 0, 0);
    }
    if (2 * r < GQ) L.sc[2 * r][m16] = D[0] + D[1];
    if (2 * r + 1 < GQ) L.sc[(2 * r + 1) % GQ][m16] = D[2] + D[3];
    wave_sync();
    // softmax numerators of the 16 rows (lanes 0..15 hold one row each), kept in LDS as fp32
    const __half *kr2, *vr2;
    row_ptr(row0 + (lane & 15), kr2, vr2);
    const bool okrow = kr2 != nullptr;
    for (int j = 0; j < GQ; ++j) {
      const float x = (okrow && lane < 16) ? L.sc[j][lane] : kNegBig;
      const float m = wave_max(x);
      const float p = (okrow && lane < 16) ? exp2f(x - m) : 0.f;
      mw[j] = m;
      lw[j] = wave_sum(p);
      wave_sync();
      if (lane < 16) L.sc[j][16 + lane] = p;
    }
    wave_sync();
    // weighted values: lane = channel pair (2*lane, 2*lane+1); results go to LDS directly
    float ov[GQ][2];
    for (int j = 0; j < GQ; ++j) ov[j][0] = ov[j][1] = 0.f;
    for (int t = 0; t < 16; ++t) {
      const __half *kr3, *vr3;
      row_ptr(row0 + t, kr3, vr3);                       // uniform over the wave
      if (!vr3) continue;
      const uint32_t w2 = ((const uint32_t*)vr3)[lane];
      const float v0 = h2f_bits(w2 & 0xFFFFu), v1 = h2f_bits(w2 >> 16);
      for (int j = 0; j < GQ; ++j) {
        const float p = L.sc[j][16 + t];
        ov[j][0] += p * v0;
        ov[j][1] += p * v1;
      }
    }
    __syncthreads();                                     // every wave is done with its WaveLds
    for (int j = 0; j < GQ; ++j) {
      lds.mg.o[wave][j][2 * lane] = ov[j][0];
      lds.mg.o[wave][j][2 * lane + 1] = ov[j][1];
      if (lane == 0) {
        lds.mg.m[wave][j] = mw[j];
        lds.mg.l[wave][j] = lw[j];
      }
    }
    float* part = a.partials + ((int64_t)ul * (a.chunks_q + a.chunks_fp) + chunk) * GQ * (kHeadDim + 2);
    merge_and_store<GQ>(lds.mg, part, tid);
    return;
  }

  // ---- quantized chunk: hand the wave's result to the merge buffer ------------------------------
  __syncthreads();                                       // every wave is done with its WaveLds
  for (int jj = 0; jj < 2; ++jj) {
    const int j = 2 * r + jj;
    if (j < GQ) {
      for (int ct = 0; ct < 8; ++ct)
        lds.mg.o[wave][j][16 * ct + m16] = (O[ct][2 * jj] + O[ct][2 * jj + 1]) * post_v + ozero[jj][ct * NV / 8];
    }
  }
  if (lane == 0)
    for (int j = 0; j < GQ; ++j) {
      lds.mg.m[wave][j] = mw[j];
      lds.mg.l[wave][j] = lw[j];
    }
  float* part = a.partials + ((int64_t)ul * (a.chunks_q + a.chunks_fp) + chunk) * GQ * (kHeadDim + 2);
  merge_and_store<GQ>(lds.mg, part, tid);
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
  const dim3 grid(a.chunks_q + a.chunks_fp, a.d.units_per_layer);
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
