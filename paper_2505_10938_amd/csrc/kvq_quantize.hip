// Residual append and group quantization (mean replacement, Eq. 2 per group, packing).
#include "kvq_common.h"

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

// One workgroup per unit: the whole group (G x 128, K and V) lives in LDS.
// LDS: 2 * G * 128 * 2 bytes (<= 64 KB) + meta.
template <int BITS>
__global__ void __launch_bounds__(256) quantize_kernel(Dims d, int32_t group_index, const __half* __restrict__ k_group,
                                                       const __half* __restrict__ v_group, int64_t unit_stride,
                                                       const uint8_t* __restrict__ selected, uint8_t* __restrict__ k_codes,
                                                       uint32_t* __restrict__ k_meta, uint8_t* __restrict__ v_codes,
                                                       uint32_t* __restrict__ v_meta, uint32_t* __restrict__ mask) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int G = d.G;
  __half* sk = (__half*)smem;                        // [G][128]
  __half* sv = sk + G * kHeadDim;                    // [G][128]
  uint32_t* skm = (uint32_t*)(sv + G * kHeadDim);    // [128] K meta
  uint32_t* svm = skm + kHeadDim;                    // [G][vgroups] V meta
  uint8_t* ssel = (uint8_t*)(svm + G * d.vgroups);   // [G]
  __shared__ int s_any;

  const int tid = threadIdx.x;
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  const __half* gk = k_group + (int64_t)ul * unit_stride;
  const __half* gv = v_group + (int64_t)ul * unit_stride;

  if (tid == 0) s_any = 0;
  __syncthreads();
  // load rows (16 bytes per thread per step), selected flags
  const int n16 = G * kHeadDim / 8;
  for (int i = tid; i < n16; i += 256) {
    ((uint4*)sk)[i] = ((const uint4*)gk)[i];
    ((uint4*)sv)[i] = ((const uint4*)gv)[i];
  }
  if (tid < G) {
    const uint8_t f = selected ? selected[(int64_t)ul * G + tid] : (uint8_t)0;
    ssel[tid] = f;
    if (f) s_any = 1;
  }
  __syncthreads();

  // mean replacement: per-channel mean of the original rows of all G tokens, exact fp64 sum,
  // scaled by the power of two 1/G, rounded to fp32 then fp16.
  if (s_any) {
    const int c = tid & 127;
    __half* rows = (tid < 128) ? sk : sv;
    double sum = 0.0;
    for (int t = 0; t < G; ++t) sum += (double)__half2float(rows[t * kHeadDim + c]);
    const float m32 = (float)(sum / (double)G);
    const __half m16 = __float2half_rn(m32);
    for (int t = 0; t < G; ++t)
      if (ssel[t]) rows[t * kHeadDim + c] = m16;
  }
  __syncthreads();

  // K meta: one channel per thread (threads 0..127); V meta: one (token, channel group) per
  // thread step (threads 128..255).
  if (tid < 128) {
    const int c = tid;
    float mn = __half2float(sk[c]), mx = mn;
    for (int t = 1; t < G; ++t) {
      const float x = __half2float(sk[t * kHeadDim + c]);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    const __half st = step_of(mn, mx, BITS);
    const uint32_t m = (uint32_t)__half_as_ushort(st) | ((uint32_t)__half_as_ushort(__float2half_rn(mn)) << 16);
    skm[c] = m;
    // global layout of a group's Key meta: fp16 step[128], then fp16 zero[128]
    __half* gm = (__half*)(k_meta + (u * d.groups_per_unit + group_index) * kHeadDim);
    gm[c] = st;
    gm[kHeadDim + c] = __float2half_rn(mn);
  } else {
    const int nvg = G * d.vgroups;
    for (int i = tid - 128; i < nvg; i += 128) {
      const int t = i / d.vgroups, j = i - t * d.vgroups;
      const __half* p = sv + t * kHeadDim + j * d.Gv;
      float mn = __half2float(p[0]), mx = mn;
      for (int c = 1; c < d.Gv; ++c) {
        const float x = __half2float(p[c]);
        mn = fminf(mn, x);
        mx = fmaxf(mx, x);
      }
      const __half st = step_of(mn, mx, BITS);
      const uint32_t m = (uint32_t)__half_as_ushort(st) | ((uint32_t)__half_as_ushort(__float2half_rn(mn)) << 16);
      svm[i] = m;
      // global layout of a 32-token block's Value meta (NV = value groups per token):
      // fp16 step[16 token pairs][NV][2], then fp16 zero[16 token pairs][NV][2]
      const int64_t tok = (int64_t)group_index * G + t;
      const int tb = (int)(tok & 31);
      __half* gm = (__half*)(v_meta + (u * d.blocks_per_unit + (tok >> 5)) * 32 * d.vgroups);
      gm[((tb >> 1) * d.vgroups + j) * 2 + (tb & 1)] = st;
      gm[32 * d.vgroups + ((tb >> 1) * d.vgroups + j) * 2 + (tb & 1)] = __float2half_rn(mn);
    }
  }
  __syncthreads();

  // codes: one packed u32 word per thread step.  Word w of lane l of block blk holds
  // 32/BITS codes of 32/BITS/8 fields.
  constexpr int kLevels = (1 << BITS) - 1;
  constexpr int kWordsPerBlock = 128 * BITS;          // 512*BITS bytes / 4
  constexpr int kFieldsPerWord = 4 / BITS;            // 2 (2-bit) or 1 (4-bit)
  const int nblk = G / kBlockTokens;
  const int first_block = group_index * nblk;
  for (int i = tid; i < nblk * kWordsPerBlock; i += 256) {
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
    uint32_t kw = 0, vw = 0;
    for (int ff = 0; ff < kFieldsPerWord; ++ff) {
      const int f = f0 + ff;
      for (int x = 0; x < 8; ++x) {
        const int bit = code_bit(BITS, f, x);
        {  // Key: lane = 16 r + m, field = 4 th + cb
          const int t = 16 * (f >> 2) + mn_;
          const int c = 32 * (f & 3) + 8 * r + x;
          const uint32_t meta = skm[c];
          const float st = __half2float(__ushort_as_half((unsigned short)(meta & 0xFFFFu)));
          const float zr = __half2float(__ushort_as_half((unsigned short)(meta >> 16)));
          const float xv = __half2float(sk[(blk * kBlockTokens + t) * kHeadDim + c]);
          kw |= quant_code(xv, zr, st, kLevels) << bit;
        }
        {  // Value: lane = 16 r + n, field = ct
          const int t = 8 * r + x;
          const int c = 16 * f + mn_;
          const int tg = blk * kBlockTokens + t;
          const uint32_t meta = svm[tg * d.vgroups + c / d.Gv];
          const float st = __half2float(__ushort_as_half((unsigned short)(meta & 0xFFFFu)));
          const float zr = __half2float(__ushort_as_half((unsigned short)(meta >> 16)));
          const float xv = __half2float(sv[tg * kHeadDim + c]);
          vw |= quant_code(xv, zr, st, kLevels) << bit;
        }
      }
    }
    const int64_t boff = (u * d.blocks_per_unit + first_block + blk) * (int64_t)d.block_bytes;
    ((uint32_t*)(k_codes + boff))[wi] = kw;
    ((uint32_t*)(v_codes + boff))[wi] = vw;
  }

  // mask words
  if (tid < nblk) {
    uint32_t w = 0;
    for (int t = 0; t < 32; ++t) w |= (ssel[tid * 32 + t] ? 1u : 0u) << t;
    mask[u * d.blocks_per_unit + first_block + tid] = w;
  }
}

}  // namespace

hipError_t launch_append(const Dims& d, const __half* k_new, const __half* v_new, __half* k_res, __half* v_res,
                         int32_t row, hipStream_t s) {
  hipLaunchKernelGGL(append_kernel, dim3(d.units_per_layer), dim3(128), 0, s, d, k_new, v_new, k_res, v_res, row);
  return hipGetLastError();
}

hipError_t launch_quantize(const Dims& d, int32_t group_index, const __half* k_group, const __half* v_group,
                           int64_t unit_stride, const uint8_t* selected, const kvq_qcache& qc, hipStream_t s) {
  const size_t smem = (size_t)2 * d.G * kHeadDim * 2 + kHeadDim * 4 + (size_t)d.G * d.vgroups * 4 + d.G;
  if (smem > 64 * 1024) {  // G = 128 needs a little more than the default per-workgroup limit
    hipError_t e = hipFuncSetAttribute(d.bits == 2 ? (const void*)quantize_kernel<2> : (const void*)quantize_kernel<4>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  if (d.bits == 2) {
    hipLaunchKernelGGL(quantize_kernel<2>, dim3(d.units_per_layer), dim3(256), smem, s, d, group_index, k_group, v_group,
                       unit_stride, selected, (uint8_t*)qc.k_codes, (uint32_t*)qc.k_meta, (uint8_t*)qc.v_codes,
                       (uint32_t*)qc.v_meta, (uint32_t*)qc.mask);
  } else {
    hipLaunchKernelGGL(quantize_kernel<4>, dim3(d.units_per_layer), dim3(256), smem, s, d, group_index, k_group, v_group,
                       unit_stride, selected, (uint8_t*)qc.k_codes, (uint32_t*)qc.k_meta, (uint8_t*)qc.v_codes,
                       (uint32_t*)qc.v_meta, (uint32_t*)qc.mask);
  }
  return hipGetLastError();
}

}  // namespace kvq
