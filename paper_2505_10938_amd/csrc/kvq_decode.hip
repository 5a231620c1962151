// Decode-step attention over the quantized cache, the residual ring and the outlier pools.
// First version: straightforward per-element dequantization, one workgroup per chunk, partial
// (max, sum, weighted values) per chunk, then a combine kernel.
#include "kvq_common.h"

namespace kvq {

namespace {

__device__ inline float h2f_bits(uint32_t bits16) { return __half2float(__ushort_as_half((unsigned short)bits16)); }

__device__ inline uint32_t read_code(const uint8_t* block, int bits, int lane, int f, int x) {
  const uint32_t w = *(const uint32_t*)(block + word_byte(bits, lane, f));
  return (w >> code_bit(bits, f, x)) & ((1u << bits) - 1u);
}

__device__ inline float block_max(float v, float* red, int tid) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ inline float block_sum(float v, float* red, int tid) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// grid (chunks_q + chunks_fp, units_per_layer), 256 threads.
// Scores are kept in the log2 domain: s = (q . k) * log2(e) / sqrt(d).
template <int GQ>
__global__ void __launch_bounds__(256) decode_partial_kernel(DecodeArgs a) {
  __shared__ float sq[GQ][kHeadDim];
  __shared__ float ssc[GQ][kChunkTokens];
  __shared__ float so[2][GQ][kHeadDim];
  __shared__ float red[4];
  const Dims& d = a.d;
  const int tid = threadIdx.x;
  const int chunk = blockIdx.x;
  const int ul = blockIdx.y;
  const int64_t u = d.unit0 + ul;
  const int b = ul / d.kv_heads, h = ul - b * d.kv_heads;
  const float qscale = 1.4426950408889634f / sqrtf((float)kHeadDim);

  for (int i = tid; i < GQ * kHeadDim; i += 256) {
    const int j = i / kHeadDim, c = i - j * kHeadDim;
    sq[j][c] = __half2float(a.q[((int64_t)b * d.q_heads + h * GQ + j) * kHeadDim + c]) * qscale;
  }
  __syncthreads();

  const bool quant = chunk < a.chunks_q;
  int count;          // tokens (rows) of this chunk
  int t0;             // first token / row
  if (quant) {
    t0 = chunk * kChunkTokens;
    count = min(kChunkTokens, a.n_quant - t0);
  } else {
    t0 = (chunk - a.chunks_q) * kFpChunkRows;
    count = max(0, min(kFpChunkRows, a.n_res + d.pool_slots - t0));
  }
  const int n_pool = a.pool_count[u], n_aux = a.aux_count[u];

  // row pointers of a full-precision row (or null when the slot is empty)
  auto fp_row = [&](int row, const __half*& kr, const __half*& vr) {
    kr = nullptr; vr = nullptr;
    if (row < a.n_res) {
      const int64_t ring = (a.res_start + row) % d.res_rows;
      kr = a.k_res + (u * d.res_rows + ring) * kHeadDim;
      vr = a.v_res + (u * d.res_rows + ring) * kHeadDim;
    } else {
      const int slot = row - a.n_res;
      const bool ok = slot < d.N ? (slot < n_pool) : (slot - d.N < n_aux);
      if (ok) {
        kr = a.pool_k + (u * d.pool_slots + slot) * kHeadDim;
        vr = a.pool_v + (u * d.pool_slots + slot) * kHeadDim;
      }
    }
  };

  // ---- scores -------------------------------------------------------------------------------
  for (int tl = tid; tl < kChunkTokens; tl += 256) {
    float s[GQ];
    bool valid = tl < count;
    for (int j = 0; j < GQ; ++j) s[j] = 0.f;
    if (valid) {
      if (quant) {
        const int t = t0 + tl;
        const int blk = t >> 5, tb = t & 31;
        valid = ((a.mask[u * d.blocks_per_unit + blk] >> tb) & 1u) == 0u;
        if (valid) {
          const uint8_t* kb = a.k_codes + (u * d.blocks_per_unit + blk) * (int64_t)d.block_bytes;
          const uint32_t* km = a.k_meta + (u * d.groups_per_unit + t / d.G) * kHeadDim;
          for (int c = 0; c < kHeadDim; ++c) {
            int lane, f, x;
            k_pos(tb, c, lane, f, x);
            const uint32_t m = km[c];
            const float kv = h2f_bits(m >> 16) + (float)read_code(kb, d.bits, lane, f, x) * h2f_bits(m & 0xFFFFu);
            for (int j = 0; j < GQ; ++j) s[j] += sq[j][c] * kv;
          }
        }
      } else {
        const __half *kr, *vr;
        fp_row(t0 + tl, kr, vr);
        valid = kr != nullptr;
        if (valid)
          for (int c = 0; c < kHeadDim; ++c) {
            const float kv = __half2float(kr[c]);
            for (int j = 0; j < GQ; ++j) s[j] += sq[j][c] * kv;
          }
      }
    }
    for (int j = 0; j < GQ; ++j) ssc[j][tl] = valid ? s[j] : kNegBig;
  }
  __syncthreads();

  // ---- chunk softmax statistics ---------------------------------------------------------------
  float mj[GQ], lj[GQ];
  for (int j = 0; j < GQ; ++j) {
    const float m = block_max(fmaxf(ssc[j][tid], ssc[j][tid + 256]), red, tid);
    float psum = 0.f;
    for (int tl = tid; tl < kChunkTokens; tl += 256) {
      const float s = ssc[j][tl];
      const float p = (s > 0.5f * kNegBig) ? exp2f(s - m) : 0.f;
      ssc[j][tl] = p;
      psum += p;
    }
    mj[j] = m;
    lj[j] = block_sum(psum, red, tid);
  }
  __syncthreads();

  // ---- weighted values: thread = (channel, half of the tokens) -----------------------------------
  {
    const int c = tid & 127, half = tid >> 7;
    float o[GQ];
    for (int j = 0; j < GQ; ++j) o[j] = 0.f;
    for (int tl = half; tl < count; tl += 2) {
      float vv;
      bool any = false;
      for (int j = 0; j < GQ; ++j) any |= ssc[j][tl] != 0.f;
      if (!any) continue;
      if (quant) {
        const int t = t0 + tl;
        const int blk = t >> 5, tb = t & 31;
        const uint8_t* vb = a.v_codes + (u * d.blocks_per_unit + blk) * (int64_t)d.block_bytes;
        int lane, f, x;
        v_pos(tb, c, lane, f, x);
        const uint32_t m = a.v_meta[(u * d.max_seq + t) * d.vgroups + c / d.Gv];
        vv = h2f_bits(m >> 16) + (float)read_code(vb, d.bits, lane, f, x) * h2f_bits(m & 0xFFFFu);
      } else {
        const __half *kr, *vr;
        fp_row(t0 + tl, kr, vr);
        vv = __half2float(vr[c]);
      }
      for (int j = 0; j < GQ; ++j) o[j] += ssc[j][tl] * vv;
    }
    for (int j = 0; j < GQ; ++j) so[half][j][c] = o[j];
  }
  __syncthreads();
  const int n_chunks = a.chunks_q + a.chunks_fp;
  float* part = a.partials + ((int64_t)ul * n_chunks + chunk) * GQ * (kHeadDim + 2);
  for (int i = tid; i < GQ * kHeadDim; i += 256) {
    const int j = i / kHeadDim, c = i - j * kHeadDim;
    part[j * (kHeadDim + 2) + 2 + c] = so[0][j][c] + so[1][j][c];
  }
  if (tid < GQ) {
    part[tid * (kHeadDim + 2) + 0] = mj[tid];
    part[tid * (kHeadDim + 2) + 1] = lj[tid];
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

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, hipStream_t s) {
  const dim3 grid(a.chunks_q + a.chunks_fp, a.d.units_per_layer);
  switch (a.d.g) {
    case 1: hipLaunchKernelGGL(decode_partial_kernel<1>, grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL(decode_partial_kernel<2>, grid, dim3(256), 0, s, a); break;
    case 4: hipLaunchKernelGGL(decode_partial_kernel<4>, grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL(decode_partial_kernel<8>, grid, dim3(256), 0, s, a); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_combine_kernel, dim3(a.d.g, a.d.units_per_layer), dim3(128), 0, s, a);
  return hipGetLastError();
}

}  // namespace kvq
