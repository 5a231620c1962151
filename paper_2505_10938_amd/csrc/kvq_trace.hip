// Outlier-token competition as kernels of its own: one group per launch, or the groups of a whole
// prompt one after the other (one workgroup of 4 wavefronts per unit in both).
#include "kvq_common.h"
#include "kvq_trace_core.h"

namespace kvq {

namespace {

// All loads of the first phase (state, stored scores, the group's K rows) go out together; the
// rows that move (evicted -> auxiliary pool, new -> pool) are loaded together in a second phase.
template <int G>
__global__ void __launch_bounds__(trace_core::kWorkers) trace_kernel(
    Dims d, int32_t group_index, const __half* __restrict__ k_group, const __half* __restrict__ v_group,
    int64_t unit_stride, __half* pool_k, __half* pool_v, int32_t* pool_idx, double* pool_score, int32_t* pool_count,
    int32_t* aux_count, int32_t* frozen, uint8_t* __restrict__ selected) {
  const int tid = threadIdx.x;
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  uint8_t* sel = selected + (int64_t)ul * G;
  if (d.N == 0) {                                      // no pool: nothing is ever selected
    if (tid < G) sel[tid] = 0;
    return;
  }
  const __half* gk = k_group + (int64_t)ul * unit_stride;
  const __half* gv = v_group + (int64_t)ul * unit_stride;
  const trace_core::UnitPool p =
      trace_core::unit_pool(d, u, pool_k, pool_v, pool_idx, pool_score, pool_count, aux_count, frozen);
  trace_core::Loaded<G> in;
  trace_core::load<G>(in, d, p, gk, tid);
  trace_core::compete<G>(in, d, group_index, p, gk, gv, sel, nullptr, tid);
}

// The competitions of a whole prompt: the groups of a unit one after the other in one workgroup
// (each depends on the pool the previous one left).  Flags go to selected[unit][group][G].
template <int G>
__global__ void __launch_bounds__(trace_core::kWorkers) prefill_trace_kernel(
    Dims d, int32_t n_groups, const __half* __restrict__ k_rows, const __half* __restrict__ v_rows,
    int64_t unit_stride, __half* pool_k, __half* pool_v, int32_t* pool_idx, double* pool_score, int32_t* pool_count,
    int32_t* aux_count, int32_t* frozen, uint8_t* __restrict__ selected) {
  const int tid = threadIdx.x;
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  uint8_t* sel = selected + (int64_t)ul * n_groups * G;
  if (d.N == 0) {                                      // no pool: nothing is ever selected
    for (int i = tid; i < n_groups * G; i += trace_core::kWorkers) sel[i] = 0;
    return;
  }
  const __half* gk = k_rows + (int64_t)ul * unit_stride;
  const __half* gv = v_rows + (int64_t)ul * unit_stride;
  const trace_core::UnitPool p =
      trace_core::unit_pool(d, u, pool_k, pool_v, pool_idx, pool_score, pool_count, aux_count, frozen);
  trace_core::Loaded<G> in;
  trace_core::load<G>(in, d, p, gk, tid);
  for (int gi = 0; gi < n_groups; ++gi) {
    if (in.is_frozen) {                                // uniform: tracing has stopped for good
      for (int i = gi * G + tid; i < n_groups * G; i += trace_core::kWorkers) sel[i] = 0;
      return;
    }
    trace_core::compete<G>(in, d, gi, p, gk + (int64_t)gi * G * kHeadDim, gv + (int64_t)gi * G * kHeadDim,
                           sel + gi * G, nullptr, tid);
    if (gi + 1 < n_groups) {
      // this group's stores are complete and ordered before the next group's loads (same
      // compute unit, one vector cache), and nobody still reads the shared arrays
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      trace_core::load_next<G>(in, d, p, gk + (int64_t)(gi + 1) * G * kHeadDim, tid);
    }
  }
}

}  // namespace

hipError_t launch_prefill_trace(const Dims& d, int32_t n_groups, const __half* k_rows, const __half* v_rows,
                                int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s) {
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(d.units_per_layer), dim3(trace_core::kWorkers), 0, s, d, n_groups, k_rows, v_rows,
                       unit_stride, (__half*)pool.pool_k, (__half*)pool.pool_v, pool.pool_idx, pool.pool_score,
                       pool.pool_count, pool.aux_count, pool.frozen, selected);
  };
  switch (d.G) {
    case 32: go(prefill_trace_kernel<32>); break;
    case 64: go(prefill_trace_kernel<64>); break;
    default: go(prefill_trace_kernel<128>); break;
  }
  return hipGetLastError();
}

// Empty pools for the units of the launch (a new sequence in a slot that held another).
__global__ void reset_pools_kernel(Dims d, int32_t* pool_count, int32_t* aux_count, int32_t* frozen) {
  const int ul = blockIdx.x * blockDim.x + threadIdx.x;
  if (ul >= d.units_per_layer) return;
  pool_count[d.unit0 + ul] = 0;
  aux_count[d.unit0 + ul] = 0;
  frozen[d.unit0 + ul] = 0;
}
hipError_t launch_reset_pools(const Dims& d, const kvq_pool& pool, hipStream_t s) {
  hipLaunchKernelGGL(reset_pools_kernel, dim3((d.units_per_layer + 63) / 64), dim3(64), 0, s, d, pool.pool_count,
                     pool.aux_count, pool.frozen);
  return hipGetLastError();
}

hipError_t launch_trace(const Dims& d, int32_t group_index, const __half* k_group, const __half* v_group,
                        int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s) {
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(d.units_per_layer), dim3(trace_core::kWorkers), 0, s, d, group_index, k_group,
                       v_group, unit_stride, (__half*)pool.pool_k, (__half*)pool.pool_v, pool.pool_idx,
                       pool.pool_score, pool.pool_count, pool.aux_count, pool.frozen, selected);
  };
  switch (d.G) {
    case 32: go(trace_kernel<32>); break;
    case 64: go(trace_kernel<64>); break;
    default: go(trace_kernel<128>); break;
  }
  return hipGetLastError();
}

}  // namespace kvq
