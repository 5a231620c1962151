// Outlier-token competition: L1 scores, ranking of pool + group, pool / auxiliary-pool update.
#include "kvq_common.h"

namespace kvq {

namespace {

constexpr int kMaxCand = 64 + 128;   // pool (N <= 64) + group (G <= 128)

// Sum over the 16 lanes of a row team.  fp64 adds of multiples of 2^-24 below 2^23 are exact,
// so the order does not matter.
__device__ inline double team_sum_f64(double v) {
  for (int off = 8; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ inline double abs_sum8(uint4 w) {
  const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    s += (double)fabsf(__half2float(__ushort_as_half((unsigned short)(ws[k] & 0xFFFFu))));
    s += (double)fabsf(__half2float(__ushort_as_half((unsigned short)(ws[k] >> 16))));
  }
  return s;
}

constexpr int kMaxMovesPerTeam = (64 + 64) / 16;   // at most N evicted + N new rows, dealt to 16 teams

// One workgroup (4 wavefronts) per unit.  Rows are handled by teams of 16 lanes (16 bytes per lane).
// All loads of the first phase (state, stored scores, the group's K rows) go out together; the
// rows that move (evicted -> auxiliary pool, new -> pool) are loaded together in a second phase.
template <int G>
__global__ void __launch_bounds__(256) trace_kernel(Dims d, int32_t group_index, const __half* __restrict__ k_group,
                                                    const __half* __restrict__ v_group, int64_t unit_stride,
                                                    __half* pool_k, __half* pool_v, int32_t* pool_idx,
                                                    double* pool_score, int32_t* pool_count, int32_t* aux_count,
                                                    int32_t* frozen, uint8_t* __restrict__ selected) {
  __shared__ double c_score[kMaxCand];
  __shared__ int32_t c_idx[kMaxCand];
  __shared__ int32_t ev_slots[64];       // old pool slots that fall out, ascending
  __shared__ int32_t mv_src[128];        // rows that move: source (>= 0: pool slot, < 0: -(group row) - 1)
  __shared__ int32_t mv_dst[128];        //                 destination slot
  __shared__ int32_t s_nev, s_wnew[4];

  const int tid = threadIdx.x;
  const int team = tid >> 4, sub = tid & 15;
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  const int N = d.N, A = d.A;
  uint8_t* sel = selected + (int64_t)ul * G;
  if (N == 0) {                                        // no pool: nothing is ever selected
    if (tid < G) sel[tid] = 0;
    return;
  }
  const __half* gk = k_group + (int64_t)ul * unit_stride;
  const __half* gv = v_group + (int64_t)ul * unit_stride;
  __half* pk = pool_k + u * d.pool_slots * kHeadDim;
  __half* pv = pool_v + u * d.pool_slots * kHeadDim;
  int32_t* pidx = pool_idx + u * d.pool_slots;
  double* psc = pool_score + u * d.pool_slots;

  // ---- phase 1 loads ---------------------------------------------------------------------------
  const int is_frozen = frozen[u];
  const int n_old = pool_count[u];
  const int n_aux = aux_count[u];
  double old_score = 0.0;
  int32_t old_idx = 0;
  if (tid < N) {                                       // every pool slot is valid memory, filled or not
    old_score = psc[tid];
    old_idx = pidx[tid];
  }
  constexpr int P = G / 16;
  uint4 kr[P];
#pragma unroll
  for (int p = 0; p < P; ++p) kr[p] = *(const uint4*)(gk + (p * 16 + team) * kHeadDim + sub * 8);

  if (is_frozen) {                                     // uniform over the workgroup
    if (tid < G) sel[tid] = 0;
    return;
  }
  const int n_cand = n_old + G;

  // candidates: old pool members first (stored score), then the group's tokens (L1 norm of the key)
  if (tid < n_old) {
    c_score[tid] = old_score;
    c_idx[tid] = old_idx;
  }
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const double sc = team_sum_f64(abs_sum8(kr[p]));
    if (sub == 0) {
      const int t = p * 16 + team;
      c_score[n_old + t] = sc;
      c_idx[n_old + t] = group_index * G + t;
    }
  }
  __syncthreads();

  // rank by counting: (score, token index) ascending; indices are unique, so ranks are too.
  // Scores are non-negative, so their bit patterns order like the values.  Each wavefront holds
  // 64 candidates at a time in registers and broadcasts them one by one (no memory in the loop).
  const int lane = tid & 63, wave = tid >> 6;
  const int keep = min(N, n_cand);
  bool is_ev = false, is_new = false;
  if (wave * 64 < n_cand) {                            // uniform over the wavefront
    const int me = min(tid, n_cand - 1);
    const unsigned long long sme = (unsigned long long)__double_as_longlong(c_score[me]);
    const int32_t ix = c_idx[me];
    int rank = 0;
    for (int base = 0; base < n_cand; base += 64) {
      const int jn = min(64, n_cand - base);
      const int jl = min(base + lane, n_cand - 1);
      const unsigned long long sl = (unsigned long long)__double_as_longlong(c_score[jl]);
      const int32_t il = c_idx[jl];
      for (int j = 0; j < jn; ++j) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)sl, j);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(sl >> 32), j);
        const int32_t ij = __builtin_amdgcn_readlane(il, j);
        const unsigned long long sj = ((unsigned long long)hi << 32) | lo;
        rank += (sj < sme || (sj == sme && ij < ix)) ? 1 : 0;
      }
    }
    is_ev = (tid < n_old) && (rank >= keep);
    is_new = (tid >= n_old) && (tid < n_cand) && (rank < keep);
  }
  // order of evicted members (by old slot: all of them sit in wavefront 0) and of new members
  // (by token index = candidate order, over up to 4 wavefronts)
  const unsigned long long bal_ev = __ballot(is_ev), bal_new = __ballot(is_new);
  const unsigned long long below = (1ull << lane) - 1ull;
  int my_order = __popcll((is_ev ? bal_ev : bal_new) & below);
  if (is_ev) ev_slots[my_order] = tid;
  if (lane == 0) {
    s_wnew[wave] = __popcll(bal_new);
    if (wave == 0) s_nev = __popcll(bal_ev);
  }
  __syncthreads();
  const int n_ev = s_nev;
  const int n_new = s_wnew[0] + s_wnew[1] + s_wnew[2] + s_wnew[3];
  if (is_new)
    for (int w = 0; w < wave; ++w) my_order += s_wnew[w];

  // stop rule: evicted members must all fit in the auxiliary pool, else freeze and change nothing
  if (n_aux + n_ev > A) {
    if (tid == 0) frozen[u] = 1;
    if (tid < G) sel[tid] = 0;
    return;
  }

  // list of moves: evicted rows first (-> auxiliary slots), then new members (-> freed, then free slots)
  if (is_ev) {
    mv_src[my_order] = tid;
    mv_dst[my_order] = N + n_aux + my_order;
  }
  if (is_new) {
    mv_src[n_ev + my_order] = -(tid - n_old) - 1;
    mv_dst[n_ev + my_order] = (my_order < n_ev) ? ev_slots[my_order] : (n_old - n_ev + my_order);
  }
  if (tid >= n_old && tid < n_cand) sel[tid - n_old] = is_new ? 1 : 0;
  __syncthreads();

  // ---- phase 2: load every moving row, then (all loads complete) store them -----------------------
  const int n_moves = n_ev + n_new;
  uint4 mk[kMaxMovesPerTeam], mvv[kMaxMovesPerTeam];
#pragma unroll
  for (int q = 0; q < kMaxMovesPerTeam; ++q) {
    const int m = q * 16 + team;
    if (m < n_moves) {
      const int src = mv_src[m];
      const __half* rk = src >= 0 ? pk + (int64_t)src * kHeadDim : gk + (int64_t)(-src - 1) * kHeadDim;
      const __half* rv = src >= 0 ? pv + (int64_t)src * kHeadDim : gv + (int64_t)(-src - 1) * kHeadDim;
      mk[q] = *(const uint4*)(rk + sub * 8);
      mvv[q] = *(const uint4*)(rv + sub * 8);
    }
  }
  // a destination may be another move's source: every load must have returned before any store
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kMaxMovesPerTeam; ++q) {
    const int m = q * 16 + team;
    if (m < n_moves) {
      const int src = mv_src[m], to = mv_dst[m];
      *(uint4*)(pk + (int64_t)to * kHeadDim + sub * 8) = mk[q];
      *(uint4*)(pv + (int64_t)to * kHeadDim + sub * 8) = mvv[q];
      if (sub == 0) {
        const int ci = src >= 0 ? src : n_old + (-src - 1);
        pidx[to] = c_idx[ci];
        psc[to] = c_score[ci];
      }
    }
  }
  if (tid == 0) {
    pool_count[u] = n_old - n_ev + n_new;
    aux_count[u] = n_aux + n_ev;
  }
}

}  // namespace

hipError_t launch_trace(const Dims& d, int32_t group_index, const __half* k_group, const __half* v_group,
                        int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s) {
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(d.units_per_layer), dim3(256), 0, s, d, group_index, k_group, v_group, unit_stride,
                       (__half*)pool.pool_k, (__half*)pool.pool_v, pool.pool_idx, pool.pool_score, pool.pool_count,
                       pool.aux_count, pool.frozen, selected);
  };
  switch (d.G) {
    case 32: go(trace_kernel<32>); break;
    case 64: go(trace_kernel<64>); break;
    default: go(trace_kernel<128>); break;
  }
  return hipGetLastError();
}

}  // namespace kvq
