// Outlier-token competition as kernels of its own: one group per launch (one workgroup of 4 wavefronts
// per unit), or the groups of a whole prompt (scores in parallel, then one wavefront per unit).
#include "kvq_common.h"
#include "kvq_trace_core.h"

#include <type_traits>

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

// ---- the competitions of a whole prompt -----------------------------------------------------------
// One workgroup of 4 wavefronts per unit.  The L1 scores of the tokens are computed 1024 tokens at a time
// into one of two LDS buffers; ONE wavefront walks the groups of a chunk in order on those scores while
// the other three compute the next chunk's.  The pool is a sorted list held one entry per lane of that
// wavefront; a stretch of tokens is looked at with one comparison per token against the pool's largest
// key, and only tokens below it are inserted, one at a time (the N smallest of pool and group do not
// depend on the order of insertion).  At the end the wavefront copies the rows of the final members from
// the prompt.  The result is the state the group-by-group competitions leave: same index sets, scores,
// rows, counts and flags (slot order is not part of it).

__device__ inline double lane_value(double v, int l) {     // v of lane l (uniform l)
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, l);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), l);
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// The value of lane - 1 (lane 0 keeps its own), as a DPP move over the whole wavefront: no LDS traffic.
__device__ __forceinline__ uint32_t from_lane_below_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x138 /* wave_shr:1 */, 0xf, 0xf, false);
}
__device__ __forceinline__ double from_lane_below(double v) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  const unsigned long long lo = from_lane_below_u32((uint32_t)b), hi = from_lane_below_u32((uint32_t)(b >> 32));
  return __longlong_as_double((long long)((hi << 32) | lo));
}
// (score, token index) ascending: the order of the competition
__device__ inline bool key_less(double as, int ai, double bs, int bi) { return as < bs || (as == bs && ai < bi); }

constexpr int kScoreChunk = 1024;                      // scores staged in LDS at a time
// wavefronts per unit: one walks the groups, the others score ahead.  Measured on a 4096-token prompt: 4 / 8 / 16
// wavefronts 91 / 80 / 79 us for 256 units (the whole prompt 233 / 218 / 220 us), 810 / 811 .. 822 / 865 us for the
// whole prompt of 1024 units.  With 8 the scores are ready well ahead and the walk itself, about 75 us, is what
// remains; a raised priority for the walking wavefront changes nothing.
constexpr int kTraceWaves = 8;

// Requires empty pools on entry (a prompt starts a sequence).
template <int G>
__global__ void __launch_bounds__(64 * kTraceWaves) prefill_trace_kernel(
    Dims d, int32_t n_groups, const __half* __restrict__ k_rows, const __half* __restrict__ v_rows,
    int64_t unit_stride, __half* pool_k, __half* pool_v, int32_t* pool_idx, double* pool_score, int32_t* pool_count,
    int32_t* aux_count, int32_t* frozen, uint8_t* __restrict__ selected) {
  __shared__ double s_buf[2][kScoreChunk];
  __shared__ double s_aux_score[64];
  __shared__ int32_t s_aux_idx[64];
  __shared__ int32_t s_stop[2];                         // set by the wavefront that holds the pool; slot = chunk parity
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ul = blockIdx.x;
  const int64_t u = d.unit0 + ul;
  const int n_tok = n_groups * G;
  uint8_t* sel = selected + (int64_t)ul * n_tok;
  const int N = d.N, A = d.A;
  if (N == 0) {                                        // no pool: nothing is ever selected
    for (int i = tid; i < n_tok; i += 64 * kTraceWaves) sel[i] = 0;
    return;
  }
  constexpr int kRounds = (G + 63) / 64;               // a group is looked at 64 tokens at a time
  constexpr int kPer = kScoreChunk / 64;
  // fp64 L1 scores of the chunk's tokens into `buf`, by the wavefronts w0 .. kTraceWaves - 1: 16 lanes per row, 4 rows
  // per load instruction, eight of them in flight per wavefront
  const __half* rows = k_rows + (int64_t)ul * unit_stride;
  auto score_chunk = [&](int c0, double* buf, int w0) {
    const int nw = kTraceWaves - w0;
    const int n_here = min(kScoreChunk, n_tok - c0);
    const int team = lane >> 4, sub = lane & 15;
    for (int i0 = 0; ((wave - w0) + nw * i0) * 4 < n_here; i0 += 8) {
      uint4 w[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int r = min(((wave - w0) + nw * (i0 + q)) * 4 + team, n_here - 1);
        w[q] = *(const uint4*)(rows + (int64_t)(c0 + r) * kHeadDim + sub * 8);
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int r = ((wave - w0) + nw * (i0 + q)) * 4 + team;
        const double sc = trace_core::team_sum_f64(trace_core::abs_sum8(w[q]));
        if (sub == 0 && r < n_here) buf[r] = sc;
      }
    }
  };
  if (tid < 2) s_stop[tid] = 0;
  score_chunk(0, s_buf[0], 0);
  __syncthreads();
  const double kInf = __longlong_as_double(0x7FF0000000000000ll);
  double ps = kInf;                                    // the pool, ascending by key: entry `lane`, lanes below P
  int pi = 0x7FFFFFFF;
  int P = 0, aux_n = 0;
  bool stopped = false;
  int gi = 0;                                          // the next group
  // One group on the sorted pool: tokens that belong to the N smallest keys seen so far are inserted one
  // at a time, the largest key falling out each time the pool is full.
  auto do_group = [&](int gl, const double* s_sc) {
    const int first = gi * G;                          // the group's first token
    const double ps0 = ps;                             // the pool before the group, should tracing stop here
    const int pi0 = pi, P0 = P;
    int E = 0;                                         // members of the old pool that fall out
    unsigned long long selm[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) selm[r] = 0;
    // (the rounds as calls with a constant round number: as a loop around the insertions it is not unrolled)
    auto round = [&](auto round_number) {
      constexpr int r = decltype(round_number)::value;
      const int t = r * 64 + lane;
      const double s = s_sc[gl * G + min(t, G - 1)];
      const int idx = first + t;
      bool pending = t < G;
      while (true) {
        // all tokens while the pool has room, else those below its largest key
        const double max_s = lane_value(ps, max(P - 1, 0));
        const int max_i = __builtin_amdgcn_readlane(pi, max(P - 1, 0));
        const bool in = pending && (P < N || key_less(s, idx, max_s, max_i));
        const unsigned long long m = __ballot(in);
        if (m == 0) break;
        const int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)m) - 1);
        const double cs = lane_value(s, l);
        const int ci = first + r * 64 + l;
        if (lane == l) pending = false;
        const int pos = __popcll(__ballot(lane < P && key_less(ps, pi, cs, ci)));
        if (P == N) {                                  // the largest key falls out
          if (max_i < first) {                         // a member of the old pool: to the auxiliary pool
            if (aux_n + E < A && lane == 0) {
              s_aux_score[aux_n + E] = max_s;
              s_aux_idx[aux_n + E] = max_i;
            }
            ++E;
          } else {                                     // a token of this group that got in a moment ago
            const int tt = max_i - first;
#pragma unroll
            for (int rr = 0; rr < kRounds; ++rr)
              if ((tt >> 6) == rr) selm[rr] &= ~(1ull << (tt & 63));
          }
        }
        const double up_s = from_lane_below(ps);
        const int up_i = (int)from_lane_below_u32((uint32_t)pi);
        if (lane > pos) {
          ps = up_s;
          pi = up_i;
        } else if (lane == pos) {
          ps = cs;
          pi = ci;
        }
        if (P < N) ++P;
        selm[r] |= 1ull << l;
      }
    };
    round(std::integral_constant<int, 0>{});
    if constexpr (kRounds > 1) round(std::integral_constant<int, 1>{});
    if (aux_n + E > A) {                               // they do not fit: tracing stops, nothing changes
      ps = ps0;
      pi = pi0;
      P = P0;
      stopped = true;
#pragma unroll
      for (int r = 0; r < kRounds; ++r) selm[r] = 0;
    } else {
      aux_n += E;
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
      if (r * 64 + lane < G) sel[first + r * 64 + lane] = (uint8_t)((selm[r] >> lane) & 1ull);
    ++gi;
  };
  constexpr int kSpanTok = G > 64 ? G : 64;            // tokens that are ruled out together: whole groups, whole masks
  constexpr int kMasksPerSpan = kSpanTok / 64, kGroupsPerSpan = kSpanTok / G;
  // the groups of one chunk (the wavefront that holds the pool)
  auto compete_chunk = [&](int c0, const double* s_sc) {
    const int here = min(kScoreChunk, n_tok - c0) / G;
    // Which tokens of the chunk lie below the pool's largest key as it is now (64 per mask, mask k kept by
    // lane k): that key only falls, so tokens that are not below it now cannot change anything later, and
    // most stretches of a long prompt hold no such token.
    uint32_t below_lo = 0, below_hi = 0;
    auto look = [&]() {
      const double max_s = lane_value(ps, max(P - 1, 0));
      const int max_i = __builtin_amdgcn_readlane(pi, max(P - 1, 0));
      double v[kPer];
#pragma unroll
      for (int k = 0; k < kPer; ++k) v[k] = s_sc[k * 64 + lane];
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        const int t = c0 + k * 64 + lane;
        const unsigned long long b = __ballot(t < n_tok && (P < N || key_less(v[k], t, max_s, max_i)));
        below_lo = lane == k ? (uint32_t)b : below_lo;
        below_hi = lane == k ? (uint32_t)(b >> 32) : below_hi;
      }
    };
    look();
    for (int gl = 0; gl < here && !stopped;) {
      const int k0 = (gl * G) >> 6;                    // the span's first mask
      uint32_t any = 0;
#pragma unroll
      for (int m = 0; m < kMasksPerSpan; ++m)
        any |= (uint32_t)__builtin_amdgcn_readlane((int)below_lo, k0 + m) |
               (uint32_t)__builtin_amdgcn_readlane((int)below_hi, k0 + m);
      const int n_here = min(kGroupsPerSpan, here - gl);
      if (any == 0) {
#pragma unroll
        for (int m = 0; m < kMasksPerSpan; ++m) {
          const int t = c0 + (k0 + m) * 64 + lane;
          if (t < c0 + (gl + n_here) * G) sel[t] = 0;
        }
        gl += n_here;
        gi += n_here;
        continue;
      }
      for (int g2 = 0; g2 < n_here && !stopped; ++g2) do_group(gl + g2, s_sc);
      gl += n_here;
    }
  };
  int buf = 0;
  for (int c0 = 0; c0 < n_tok; c0 += kScoreChunk, buf ^= 1) {
    if (wave == 0) {
      compete_chunk(c0, s_buf[buf]);
      if (stopped && lane == 0) s_stop[buf] = 1;
    } else if (c0 + kScoreChunk < n_tok) {
      score_chunk(c0 + kScoreChunk, s_buf[buf ^ 1], 1);
    }
    __syncthreads();
    if (s_stop[buf]) break;                            // (written before the barrier; the slot is not written again
                                                       // before every wavefront has passed the next one)
  }
  if (wave != 0) return;
  for (int i = gi * G + lane; i < n_tok; i += 64) sel[i] = 0;      // groups after the stop select nothing
  // lane 0's writes of the auxiliary list, read by the other lanes below
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // the unit's state
  const int64_t slot0 = u * d.pool_slots;
  if (lane < P) {
    pool_idx[slot0 + lane] = pi;
    pool_score[slot0 + lane] = ps;
  }
  if (lane < aux_n) {
    pool_idx[slot0 + N + lane] = s_aux_idx[lane];
    pool_score[slot0 + N + lane] = s_aux_score[lane];
  }
  if (lane == 0) {
    pool_count[u] = P;
    aux_count[u] = aux_n;
    frozen[u] = stopped ? 1 : 0;
  }
  // (3) the members' rows, bit for bit, from the prompt: 4 bytes per lane and row
  const uint32_t* kr = (const uint32_t*)(k_rows + (int64_t)ul * unit_stride);
  const uint32_t* vr = (const uint32_t*)(v_rows + (int64_t)ul * unit_stride);
  uint32_t* pk = (uint32_t*)(pool_k + slot0 * kHeadDim);
  uint32_t* pv = (uint32_t*)(pool_v + slot0 * kHeadDim);
  // (eight rows' loads in flight at a time; a row's destination is its slot)
  const int n_rows = P + aux_n;
  for (int j0 = 0; j0 < n_rows; j0 += 8) {
    uint32_t kw[8], vw[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int j = min(j0 + q, n_rows - 1);
      const int idx = j < P ? __builtin_amdgcn_readlane(pi, min(j, 63)) : s_aux_idx[max(j - P, 0)];
      const int64_t src = (int64_t)idx * (kHeadDim / 2) + lane;
      kw[q] = kr[src];
      vw[q] = vr[src];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int j = j0 + q;
      if (j < n_rows) {
        const int slot = j < P ? j : N + (j - P);
        pk[slot * (kHeadDim / 2) + lane] = kw[q];
        pv[slot * (kHeadDim / 2) + lane] = vw[q];
      }
    }
  }
}

}  // namespace

hipError_t launch_prefill_trace(const Dims& d, int32_t n_groups, const __half* k_rows, const __half* v_rows,
                                int64_t unit_stride, const kvq_pool& pool, uint8_t* selected, hipStream_t s) {
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(d.units_per_layer), dim3(64 * kTraceWaves), 0, s, d, n_groups, k_rows, v_rows, unit_stride,
                       (__half*)pool.pool_k, (__half*)pool.pool_v, pool.pool_idx, pool.pool_score, pool.pool_count,
                       pool.aux_count, pool.frozen, selected);
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
