// Outlier-token competition: L1 scores, ranking of pool + group, pool / auxiliary-pool update.
#include "kvq_common.h"

namespace kvq {

namespace {

constexpr int kMaxCand = 64 + 128;   // pool (N <= 64) + group (G <= 128)

__device__ inline double wave_sum_f64(double v) {
  // fp64 adds of multiples of 2^-24 below 2^23 are exact, so the order does not matter.
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// copy one 128 x fp16 row with 64 lanes (4 bytes each)
__device__ inline void copy_row(__half* dst, const __half* src, int lane) {
  ((uint32_t*)dst)[lane] = ((const uint32_t*)src)[lane];
}

// One workgroup (4 wavefronts) per unit.
__global__ void __launch_bounds__(256) trace_kernel(Dims d, int32_t group_index, const __half* __restrict__ k_group,
                                                    const __half* __restrict__ v_group, int64_t unit_stride,
                                                    __half* pool_k, __half* pool_v, int32_t* pool_idx,
                                                    double* pool_score, int32_t* pool_count, int32_t* aux_count,
                                                    int32_t* frozen, uint8_t* __restrict__ selected) {
  __shared__ double c_score[kMaxCand];
  __shared__ int32_t c_idx[kMaxCand];
  __shared__ int32_t c_rank[kMaxCand];
  __shared__ int32_t ev_slots[64];       // old pool slots that fall out, ascending
  __shared__ int32_t s_nev, s_nnew;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  const int G = d.G, N = d.N, A = d.A;
  uint8_t* sel = selected + (int64_t)ul * G;

  const bool active = (N > 0) && (frozen[u] == 0);     // uniform over the workgroup
  if (!active) {
    if (tid < G) sel[tid] = 0;
    return;
  }
  const __half* gk = k_group + (int64_t)ul * unit_stride;
  const __half* gv = v_group + (int64_t)ul * unit_stride;
  __half* pk = pool_k + u * d.pool_slots * kHeadDim;
  __half* pv = pool_v + u * d.pool_slots * kHeadDim;
  int32_t* pidx = pool_idx + u * d.pool_slots;
  double* psc = pool_score + u * d.pool_slots;
  const int n_old = pool_count[u];
  const int n_aux = aux_count[u];
  const int n_cand = n_old + G;

  // candidates: old pool members first (stored score), then the group's tokens
  if (tid < n_old) {
    c_score[tid] = psc[tid];
    c_idx[tid] = pidx[tid];
  }
  for (int t = wave; t < G; t += 4) {
    const uint32_t w = ((const uint32_t*)(gk + (int64_t)t * kHeadDim))[lane];
    const float a = fabsf(__half2float(__ushort_as_half((unsigned short)(w & 0xFFFFu))));
    const float b = fabsf(__half2float(__ushort_as_half((unsigned short)(w >> 16))));
    const double s = wave_sum_f64((double)a + (double)b);
    if (lane == 0) {
      c_score[n_old + t] = s;
      c_idx[n_old + t] = group_index * G + t;
    }
  }
  if (tid == 0) { s_nev = 0; s_nnew = 0; }
  __syncthreads();

  // rank by counting: (score, token index) ascending; indices are unique, so ranks are too
  const int keep = min(N, n_cand);
  bool is_ev = false, is_new = false;
  if (tid < n_cand) {
    const double s = c_score[tid];
    const int32_t ix = c_idx[tid];
    int rank = 0;
    for (int j = 0; j < n_cand; ++j) {
      const double sj = c_score[j];
      rank += (sj < s || (sj == s && c_idx[j] < ix)) ? 1 : 0;
    }
    c_rank[tid] = rank;
    is_ev = (tid < n_old) && (rank >= keep);
    is_new = (tid >= n_old) && (rank < keep);
    if (is_ev) atomicAdd(&s_nev, 1);
    if (is_new) atomicAdd(&s_nnew, 1);
  }
  __syncthreads();
  const int n_ev = s_nev;

  // stop rule: evicted members must all fit in the auxiliary pool, else freeze and change nothing
  if (n_aux + n_ev > A) {
    if (tid == 0) frozen[u] = 1;
    if (tid < G) sel[tid] = 0;
    return;
  }

  // order of evicted members (by old slot) and of new members (by token index = candidate order)
  int my_order = 0;
  if (is_ev) {
    for (int j = 0; j < tid; ++j) my_order += (c_rank[j] >= keep) ? 1 : 0;
    ev_slots[my_order] = tid;
  }
  if (is_new) {
    for (int j = n_old; j < tid; ++j) my_order += (c_rank[j] < keep) ? 1 : 0;
  }
  // c_rank[] is reused below as "destination slot" (-1 = none); make ranks dead first
  __syncthreads();
  int dst = -1;
  if (is_ev) dst = N + n_aux + my_order;
  if (is_new) dst = (my_order < n_ev) ? ev_slots[my_order] : (n_old - n_ev + my_order);
  __syncthreads();
  if (tid < n_cand) c_rank[tid] = dst;
  __syncthreads();

  // phase 1: evicted rows -> auxiliary slots (reads of pool rows finish before phase 2 overwrites)
  for (int i = wave; i < n_old; i += 4) {
    const int to = c_rank[i];
    if (to >= 0) {
      copy_row(pk + (int64_t)to * kHeadDim, pk + (int64_t)i * kHeadDim, lane);
      copy_row(pv + (int64_t)to * kHeadDim, pv + (int64_t)i * kHeadDim, lane);
      if (lane == 0) {
        pidx[to] = c_idx[i];
        psc[to] = c_score[i];
      }
    }
  }
  __syncthreads();
  // phase 2: new members -> pool slots
  for (int t = wave; t < G; t += 4) {
    const int to = c_rank[n_old + t];
    if (to >= 0) {
      copy_row(pk + (int64_t)to * kHeadDim, gk + (int64_t)t * kHeadDim, lane);
      copy_row(pv + (int64_t)to * kHeadDim, gv + (int64_t)t * kHeadDim, lane);
      if (lane == 0) {
        pidx[to] = c_idx[n_old + t];
        psc[to] = c_score[n_old + t];
      }
    }
    if (lane == 0) sel[t] = (to >= 0) ? 1 : 0;
  }
  if (tid == 0) {
    pool_count[u] = n_old - n_ev + s_nnew;
    aux_count[u] = n_aux + n_ev;
  }
}

}  // namespace

hipError_t launch_trace(const Dims& d, int32_t group_index, const __half* k_group, const __half* v_group,
                        int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s) {
  hipLaunchKernelGGL(trace_kernel, dim3(d.units_per_layer), dim3(256), 0, s, d, group_index, k_group, v_group,
                     unit_stride, (__half*)pool.pool_k, (__half*)pool.pool_v, pool.pool_idx, pool.pool_score,
                     pool.pool_count, pool.aux_count, pool.frozen, selected);
  return hipGetLastError();
}

}  // namespace kvq
