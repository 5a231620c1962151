// Outlier-token competition for one unit, as device code shared by the stand-alone trace kernel
// and the fused group step: L1 scores, ranking of pool + group, pool / auxiliary-pool update
// (Method, "Quantization"; Appendix, "Competition Mechanism").
#pragma once

#include "kvq_common.h"

namespace kvq {
namespace trace_core {

constexpr int kMaxCand = 64 + 128;                 // pool (N <= 64) + group (G <= 128)
constexpr int kWorkers = 256;                      // threads of the workgroup that do the work
constexpr int kMaxMovesPerTeam = (64 + 64) / 16;   // at most N evicted + N new rows, dealt to 16 teams

// Sum over the 16 lanes of a row team.  fp64 adds of multiples of 2^-24 below 2^23 are exact,
// so the order does not matter.
__device__ inline double team_sum_f64(double v) {
  v += row_partner<0>(v);
  v += row_partner<1>(v);
  v += row_partner<2>(v);
  v += row_partner<3>(v);
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

// The unit's pool, already offset to the unit.
struct UnitPool {
  __half* pk;
  __half* pv;
  int32_t* pidx;
  double* psc;
  int32_t* pool_count;
  int32_t* aux_count;
  int32_t* frozen;
};

__device__ inline UnitPool unit_pool(const Dims& d, int64_t u, __half* pool_k, __half* pool_v, int32_t* pool_idx,
                                     double* pool_score, int32_t* pool_count, int32_t* aux_count, int32_t* frozen) {
  UnitPool p;
  p.pk = pool_k + u * d.pool_slots * kHeadDim;
  p.pv = pool_v + u * d.pool_slots * kHeadDim;
  p.pidx = pool_idx + u * d.pool_slots;
  p.psc = pool_score + u * d.pool_slots;
  p.pool_count = pool_count + u;
  p.aux_count = aux_count + u;
  p.frozen = frozen + u;
  return p;
}

// What the first phase loads.
template <int G>
struct Loaded {
  int is_frozen, n_old, n_aux;
  double old_score;
  int32_t old_idx;
  uint4 kr[G / 16];      // Key rows 16p + team, this lane's 8 channels (threads below kWorkers)
  uint4 pool_kr, pool_vr;   // pool slot `team`'s Key and Value row, same 8 channels (see kPoolRowsAhead)
};

// A budget of at most this many tokens has its pool rows fetched with the first loads, so that a
// member that falls out can be moved to the auxiliary pool without a second trip to memory.
constexpr int kPoolRowsAhead = 16;

// Issue every load of the first phase (state, stored scores, the group's Key rows); nothing is
// waited for here.  Rows are handled by teams of 16 lanes (16 bytes per lane).  Requires N > 0.
template <int G>
__device__ __forceinline__ void load(Loaded<G>& in, const Dims& d, const UnitPool& p, const __half* gk, int tid,
                                     bool pool_rows_ahead = false) {
  in.is_frozen = *p.frozen;
  in.n_old = *p.pool_count;
  in.n_aux = *p.aux_count;
  in.old_score = 0.0;
  in.old_idx = 0;
  if (tid < d.N) {                                     // every pool slot is valid memory, filled or not
    in.old_score = p.psc[tid];
    in.old_idx = p.pidx[tid];
  }
  const int team = (tid & (kWorkers - 1)) >> 4, sub = tid & 15;
  if (tid < kWorkers) {
#pragma unroll
    for (int q = 0; q < G / 16; ++q) in.kr[q] = *(const uint4*)(gk + (q * 16 + team) * kHeadDim + sub * 8);
    if (pool_rows_ahead && team < d.N) {               // d.N <= kPoolRowsAhead: one slot per team
      in.pool_kr = *(const uint4*)(p.pk + (int64_t)team * kHeadDim + sub * 8);
      in.pool_vr = *(const uint4*)(p.pv + (int64_t)team * kHeadDim + sub * 8);
    }
  }
}

// The competition and the pool update.  Every thread of the workgroup must call it (it holds
// barriers); the work is done by threads 0 .. kWorkers-1.  Writes the group's selected flags to
// `sel` (global, may be null) and `sel_lds` (LDS, may be null), and leaves the unit's new state
// (frozen flag, member counts) in `in`.  Requires N > 0.
// `staged_k`, `staged_v` (may be null): the group's rows in LDS, row t at byte t * staged_pitch; with them,
// and with the pool rows fetched ahead (`pool_rows_ahead`, as passed to load()), no moving row is read
// from memory.
template <int G>
__device__ __forceinline__ void compete(Loaded<G>& in, const Dims& d, int group_index, const UnitPool& p,
                                        const __half* gk, const __half* gv, uint8_t* sel, uint8_t* sel_lds, int tid,
                                        const unsigned char* staged_k = nullptr, const unsigned char* staged_v = nullptr,
                                        int staged_pitch = 0, bool pool_rows_ahead = false) {
  __shared__ uint4 s_pool_k[kPoolRowsAhead][16], s_pool_v[kPoolRowsAhead][16];
  __shared__ double c_score[kMaxCand];
  __shared__ int32_t c_idx[kMaxCand];
  __shared__ int32_t c_rank[kMaxCand];
  __shared__ int32_t ev_slots[64];       // old pool slots that fall out, ascending
  __shared__ int32_t mv_src[128];        // rows that move: source (>= 0: pool slot, < 0: -(group row) - 1)
  __shared__ int32_t mv_dst[128];        //                 destination slot
  __shared__ int32_t s_nev, s_wnew[4];

  const bool worker = tid < kWorkers;
  const int team = (tid & (kWorkers - 1)) >> 4, sub = tid & 15;
  const int N = d.N, A = d.A;
  auto none_selected = [&]() {
    if (tid < G) {
      if (sel) sel[tid] = 0;
      if (sel_lds) sel_lds[tid] = 0;
    }
  };
  if (in.is_frozen) {                                  // uniform over the workgroup
    none_selected();
    return;
  }
  const int n_old = in.n_old, n_aux = in.n_aux;
  const int n_cand = n_old + G;

  // candidates: old pool members first (stored score), then the group's tokens (L1 norm of the key)
  if (tid < n_old) {
    c_score[tid] = in.old_score;
    c_idx[tid] = in.old_idx;
  }
  if (tid < n_cand) c_rank[tid] = 0;
  if (worker && pool_rows_ahead && team < N) {
    s_pool_k[team][sub] = in.pool_kr;
    s_pool_v[team][sub] = in.pool_vr;
  }
  if (worker) {
#pragma unroll
    for (int q = 0; q < G / 16; ++q) {
      const double sc = team_sum_f64(abs_sum8(in.kr[q]));
      if (sub == 0) {
        const int t = q * 16 + team;
        c_score[n_old + t] = sc;
        c_idx[n_old + t] = group_index * G + t;
      }
    }
  }
  __syncthreads();

  // rank by counting: (score, token index) ascending; indices are unique, so ranks are too.
  // Scores are non-negative, so their bit patterns order like the values.  Lane = candidate
  // (64 at a time), the wavefronts share the candidates to compare against; partial counts are
  // added up in LDS (integer adds: any order).
  const int lane = tid & 63, wave = tid >> 6;
  const int n_waves = (int)(blockDim.x >> 6);
  const int keep = min(N, n_cand);
  for (int base = 0; base < n_cand; base += 64) {
    const int me = min(base + lane, n_cand - 1);
    const unsigned long long sme = (unsigned long long)__double_as_longlong(c_score[me]);
    const int32_t ix = c_idx[me];
    int cnt = 0;
#pragma unroll 4
    for (int j = wave; j < n_cand; j += n_waves) {
      const unsigned long long sj = (unsigned long long)__double_as_longlong(c_score[j]);
      cnt += (sj < sme || (sj == sme && c_idx[j] < ix)) ? 1 : 0;
    }
    if (base + lane < n_cand && cnt) atomicAdd(&c_rank[base + lane], cnt);
  }
  __syncthreads();
  bool is_ev = false, is_new = false;
  if (tid < n_cand) {
    const int rank = c_rank[tid];
    is_ev = (tid < n_old) && (rank >= keep);
    is_new = (tid >= n_old) && (rank < keep);
  }
  // order of evicted members (by old slot: all of them sit in wavefront 0) and of new members
  // (by token index = candidate order; they sit in the first 4 wavefronts)
  const unsigned long long bal_ev = __ballot(is_ev), bal_new = __ballot(is_new);
  const unsigned long long below = (1ull << lane) - 1ull;
  int my_order = __popcll((is_ev ? bal_ev : bal_new) & below);
  if (is_ev) ev_slots[my_order] = tid;
  if (lane == 0 && wave < 4) {
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
    if (tid == 0) *p.frozen = 1;
    in.is_frozen = 1;
    none_selected();
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
  if (tid >= n_old && tid < n_cand) {
    if (sel) sel[tid - n_old] = is_new ? 1 : 0;
    if (sel_lds) sel_lds[tid - n_old] = is_new ? 1 : 0;
  }
  __syncthreads();

  // ---- load every moving row, then (all loads complete) store them ---------------------------------
  const int n_moves = n_ev + n_new;
  uint4 mk[kMaxMovesPerTeam], mvv[kMaxMovesPerTeam];
#pragma unroll
  for (int q = 0; q < kMaxMovesPerTeam; ++q) {
    const int m = q * 16 + team;
    if (worker && m < n_moves) {
      const int src = mv_src[m];
      if (src >= 0 && pool_rows_ahead) {               // a member that falls out: its row was fetched ahead
        mk[q] = s_pool_k[src][sub];
        mvv[q] = s_pool_v[src][sub];
      } else if (src < 0 && staged_k) {                // a new member: its row is staged in LDS
        mk[q] = *(const uint4*)(staged_k + (-src - 1) * staged_pitch + sub * 16);
        mvv[q] = *(const uint4*)(staged_v + (-src - 1) * staged_pitch + sub * 16);
      } else {
        const __half* rk = src >= 0 ? p.pk + (int64_t)src * kHeadDim : gk + (int64_t)(-src - 1) * kHeadDim;
        const __half* rv = src >= 0 ? p.pv + (int64_t)src * kHeadDim : gv + (int64_t)(-src - 1) * kHeadDim;
        mk[q] = *(const uint4*)(rk + sub * 8);
        mvv[q] = *(const uint4*)(rv + sub * 8);
      }
    }
  }
  // A destination may be another move's source: every load from memory must have returned before any
  // store.  Rows taken from LDS copies have no such hazard (uniform over the workgroup).
  if (!(pool_rows_ahead && staged_k)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
#pragma unroll
  for (int q = 0; q < kMaxMovesPerTeam; ++q) {
    const int m = q * 16 + team;
    if (worker && m < n_moves) {
      const int src = mv_src[m], to = mv_dst[m];
      *(uint4*)(p.pk + (int64_t)to * kHeadDim + sub * 8) = mk[q];
      *(uint4*)(p.pv + (int64_t)to * kHeadDim + sub * 8) = mvv[q];
      if (sub == 0) {
        const int ci = src >= 0 ? src : n_old + (-src - 1);
        p.pidx[to] = c_idx[ci];
        p.psc[to] = c_score[ci];
      }
    }
  }
  if (tid == 0) {
    *p.pool_count = n_old - n_ev + n_new;
    *p.aux_count = n_aux + n_ev;
  }
  in.n_old = n_old - n_ev + n_new;
  in.n_aux = n_aux + n_ev;
}

// Loads for the next group of the same unit inside one kernel: the stored scores and indices as
// they stand after the previous competition (whose stores were completed and ordered by the
// caller) and the next group's Key rows; the counts and the frozen flag are carried in `in`.
template <int G>
__device__ __forceinline__ void load_next(Loaded<G>& in, const Dims& d, const UnitPool& p, const __half* gk, int tid) {
  in.old_score = 0.0;
  in.old_idx = 0;
  if (tid < d.N) {
    in.old_score = __hip_atomic_load(&p.psc[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    in.old_idx = __hip_atomic_load(&p.pidx[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  const int team = (tid & (kWorkers - 1)) >> 4, sub = tid & 15;
  if (tid < kWorkers) {
#pragma unroll
    for (int q = 0; q < G / 16; ++q) in.kr[q] = *(const uint4*)(gk + (q * 16 + team) * kHeadDim + sub * 8);
  }
}

}  // namespace trace_core
}  // namespace kvq
