// The quantized segment as fp16 rows: x^ = X_min + Q * q, the inverse of Eq. 2 (Preliminaries,
// "Quantization"), for consumers that need the cache as a matrix.  A token that lives in the outlier or
// auxiliary pool comes out as its stored full-precision row (Method, "Decoding": such a token is
// never represented by its codes).  Not on the decode path; one workgroup per (32-token block, unit).
#include "kvq_common.h"

namespace kvq {

namespace {

constexpr int kDequantThreads = 256;

__device__ inline uint32_t code_at(const uint32_t* words, int bits, int lane, int f, int x) {
  const uint32_t w = words[word_byte(bits, lane, f) >> 2];
  const int bit = code_bit(bits, f, x);
  return ((w >> bit) | (w << ((32 - bit) & 31))) & ((1u << bits) - 1u);     // the code was rotated into place
}

__global__ void __launch_bounds__(kDequantThreads) dequant_kernel(
    Dims d, int32_t block0, int32_t n_blocks, const uint8_t* __restrict__ k_codes, const uint32_t* __restrict__ k_meta,
    const uint8_t* __restrict__ v_codes, const uint32_t* __restrict__ v_meta, const uint32_t* __restrict__ mask,
    const __half* __restrict__ pool_k, const __half* __restrict__ pool_v, const int32_t* __restrict__ pool_idx,
    const int32_t* __restrict__ pool_count, const int32_t* __restrict__ aux_count, __half* __restrict__ k_out,
    __half* __restrict__ v_out, int64_t out_unit_stride) {
  __shared__ uint32_t sk[512], sv[512];              // the block's packed Key and Value codes (4-bit: 2 KB each)
  __shared__ int32_t s_slot[kBlockTokens];           // pool slot of a masked token, -1 otherwise
  const int tid = threadIdx.x;
  const int ul = blockIdx.x / n_blocks;              // grid: units x blocks, flattened (x has the widest limit)
  const int blk = block0 + blockIdx.x % n_blocks;    // logical block of the sequence
  const int64_t u = d.unit0 + ul;
  const GroupPlace at = place_of_group(d, ul, blk >> d.bpg_shift);
  const int64_t pblk = at.row * d.blocks_per_unit + ((int64_t)at.slot << d.bpg_shift) + (blk & ((1 << d.bpg_shift) - 1));
  const int words = d.block_bytes >> 2;
  const uint32_t* gk = (const uint32_t*)(k_codes + pblk * d.block_bytes);
  const uint32_t* gv = (const uint32_t*)(v_codes + pblk * d.block_bytes);
  for (int i = tid; i < words; i += kDequantThreads) {
    sk[i] = gk[i];
    sv[i] = gv[i];
  }
  // masked tokens: the slot whose token index is theirs
  const uint32_t mword = mask[pblk];
  if (tid < kBlockTokens) {
    int slot = -1;
    if ((mword >> tid) & 1u) {
      const int token = blk * kBlockTokens + tid;
      const int n_pool = min(max(pool_count[u], 0), d.N), n_aux = min(max(aux_count[u], 0), d.A);
      for (int s = 0; s < n_pool; ++s)
        if (pool_idx[u * d.pool_slots + s] == token) slot = s;
      for (int s = d.N; s < d.N + n_aux; ++s)
        if (pool_idx[u * d.pool_slots + s] == token) slot = s;
    }
    s_slot[tid] = slot;
  }
  __syncthreads();

  const __half* km = (const __half*)k_meta + (at.row * d.groups_per_unit + at.slot) * (2 * kHeadDim);
  const __half* vm = (const __half*)v_meta + pblk * (64 * d.vgroups);
  const int gv_shift = 31 - __clz(d.Gv);
  __half* ko = k_out + (int64_t)ul * out_unit_stride + (int64_t)(blk - block0) * kBlockTokens * kHeadDim;
  __half* vo = v_out + (int64_t)ul * out_unit_stride + (int64_t)(blk - block0) * kBlockTokens * kHeadDim;
  for (int e = tid; e < kBlockTokens * kHeadDim; e += kDequantThreads) {
    const int t = e >> 7, c = e & (kHeadDim - 1);
    const int slot = s_slot[t];
    if (slot >= 0) {                                  // the token's stored row (128 consecutive threads agree)
      ko[e] = pool_k[(u * d.pool_slots + slot) * kHeadDim + c];
      vo[e] = pool_v[(u * d.pool_slots + slot) * kHeadDim + c];
      continue;
    }
    int lane, f, x;
    k_pos(t, c, lane, f, x);
    const float kc = (float)code_at(sk, d.bits, lane, f, x);
    ko[e] = __float2half_rn(__fmaf_rn(kc, __half2float(km[c]), __half2float(km[kHeadDim + c])));
    v_pos(t, c, lane, f, x);
    const float vc = (float)code_at(sv, d.bits, lane, f, x);
    const int j = c >> gv_shift;
    const int mi = ((t >> 1) * d.vgroups + j) * 2 + (t & 1);
    vo[e] = __float2half_rn(__fmaf_rn(vc, __half2float(vm[mi]), __half2float(vm[32 * d.vgroups + mi])));
  }
}

}  // namespace

hipError_t launch_dequantize(const Dims& d, int32_t block0, int32_t n_blocks, const kvq_qcache& qc, const kvq_pool& pool,
                             __half* k_out, __half* v_out, int64_t out_unit_stride, hipStream_t s) {
  hipLaunchKernelGGL(dequant_kernel, dim3((uint32_t)(n_blocks * d.units_per_layer)), dim3(kDequantThreads), 0, s, d,
                     block0, n_blocks,
                     (const uint8_t*)qc.k_codes, (const uint32_t*)qc.k_meta, (const uint8_t*)qc.v_codes,
                     (const uint32_t*)qc.v_meta, (const uint32_t*)qc.mask, (const __half*)pool.pool_k,
                     (const __half*)pool.pool_v, pool.pool_idx, pool.pool_count, pool.aux_count, k_out, v_out,
                     out_unit_stride);
  return hipGetLastError();
}

}  // namespace kvq
