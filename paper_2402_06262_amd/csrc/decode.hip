// RoCo decode step on gfx950 (section 4.3 of the paper; Fig. 1: one key/value pair is deleted before the
// next token's is appended; section 5.3: decoding is I/O-bounded).
//
// The victim of step t+1 depends only on the statistics as they stand after step t, so it is chosen at the
// end of step t, while the updated statistics are still in registers, and kept in `next_slot[unit]` (part
// of the cache state).  A step is then two kernels on the caller's stream:
//
//   decode_attend : grid (splits, units).  The slot the new token goes to is next_slot[u] when the buffer is
//     full, else n_used[u].  Streams K and V of its slot range once with 128-bit loads; the one row that is
//     being overwritten is taken from k_new / v_new instead (and written into the cache in passing).  Keeps
//     an online softmax per 16-lane group, stores every base-2 logit, writes one partial (max, sum, weighted
//     V sum) per split.  HBM-bound: no matrix cores.
//   decode_finish : one workgroup per unit.  Merges the partials in split order (fixed order: results do not
//     depend on scheduling), writes the attention output, adds p, p^2 and 1 into the three statistics planes
//     (the overwritten slot starts from zero), records pos / n_used / evicted_*, and, if the buffer is now
//     full, selects the next victim: scope = the `scope` slots of lowest variance, victim = lowest mean
//     attention score inside it.
//
//   select_victims : the selection alone (for a cache whose statistics were produced elsewhere).
#include <cstdlib>
#include "kernels.hpp"
#include "profile.hpp"
#include "stream.hpp"

namespace roco {
namespace {

constexpr int kAttendThreads = 256;
constexpr int kAttendWaves = kAttendThreads / kWave;
constexpr int kFinishThreads = kDecodeSelectThreads;
constexpr int kFusedThreads = 256;  // with 8 rows in flight per lane group: two workgroups per compute unit

// ------------------------------------------------------------------------------------------------
// BIAS: a recency bias is in force; STREAMING: non-temporal loads.  They are template parameters, not branches inside
// one kernel, to keep each kernel's code (the unrolled, software-pipelined stream) small.
template <int DT, int D, int U, bool BIAS, bool STREAMING>
__global__ __launch_bounds__(kAttendThreads) void decode_attend(DecodeArgs a) {
  using G = RowGeom<DT, D>;
  constexpr int STREAMS = kAttendWaves;  // one merged stream per wave reaches LDS
  constexpr int PASS = kAttendWaves * U * G::R;
  __shared__ float sm_m[STREAMS], sm_l[STREAMS];
  __shared__ float sm_acc[STREAMS][D];

  const int u = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int c = lane % G::LPR;
  const int n0 = a.n_used[u];
  const bool full = n0 >= a.B;
  const int slot = full ? min(max(a.next_slot[u], 0), a.B - 1) : n0;  // where the new token goes
  const int n = full ? a.B : n0 + 1;
  const int row0 = split * a.rows_per_split;
  const int row1 = min(n, row0 + a.rows_per_split);

  const size_t in_off = static_cast<size_t>(u) * G::ROW_BYTES + c * 16;
  float qf[G::EPL];
  unpack16<DT>(load16(static_cast<const char*>(a.q) + in_off), qf);
#pragma unroll
  for (int e = 0; e < G::EPL; ++e) qf[e] *= a.scale_log2;

  char* Kb = static_cast<char*>(a.K) + static_cast<size_t>(u) * a.B * G::ROW_BYTES;
  char* Vb = static_cast<char*>(a.V) + static_cast<size_t>(u) * a.B * G::ROW_BYTES;
  float* z = a.z + static_cast<size_t>(u) * a.B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * a.B;
  const int qp = a.qpos[u];
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;

  FlashState<G::EPL> st;
  st.reset();
  auto bias = [&](int row, int row_pos) -> float {
    const int dlt = (row == slot) ? 0 : qp - row_pos;
    return (dlt >= 0 && dlt < w) ? rb : 0.0f;
  };
  // in-place overwrite of the slot the new token takes: the cache never grows past B
  auto fix_k = [&](int row, uint4& kw, int col) {
    if (row == slot && row < row1) {
      kw = load16(static_cast<const char*>(a.k_new) + in_off);
      *reinterpret_cast<uint4*>(Kb + static_cast<size_t>(row) * G::ROW_BYTES + col * 16) = kw;
    }
  };
  auto fix_v = [&](int row, uint4& vw, int col) {
    if (row == slot && row < row1) {
      vw = load16(static_cast<const char*>(a.v_new) + in_off);
      *reinterpret_cast<uint4*>(Vb + static_cast<size_t>(row) * G::ROW_BYTES + col * 16) = vw;
    }
  };
  const int span = row1 - row0;
  const int passes = span > 0 ? (span + PASS - 1) / PASS : 0;
  const int rot = passes > 0 ? static_cast<int>((static_cast<unsigned>(u) * 5u + static_cast<unsigned>(split) * 3u) %
                                                static_cast<unsigned>(passes))
                             : 0;
  stream_attend<DT, D, U, BIAS, STREAMING>(qf, Kb, Vb, row0, row1, passes, a.rotate ? rot : 0, PASS, wave * (U * G::R),
                                           bias, pos, z, slot, fix_k, fix_v, st);
  merge_groups_in_wave<DT, D>(st);

  if (lane < G::LPR) {
    if (lane == 0) { sm_m[wave] = st.m; sm_l[wave] = st.l; }
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) sm_acc[wave][lane * G::EPL + e] = st.acc[e];
  }
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < STREAMS; ++s) M = fmaxf(M, sm_m[s]);
  const size_t pidx = static_cast<size_t>(u) * a.splits + split;
  if (tid < D) {
    float o = 0.0f, l = 0.0f;
#pragma unroll
    for (int s = 0; s < STREAMS; ++s) {
      const float wgt = (sm_m[s] > -INFINITY) ? fast_exp2(sm_m[s] - M) : 0.0f;
      l += sm_l[s] * wgt;
      o += sm_acc[s][tid] * wgt;
    }
    a.part_o[pidx * D + tid] = o;
    if (tid == 0) { a.part_m[pidx] = M; a.part_l[pidx] = l; }
  }
}

// Adds this step's probabilities p_j = 2^(z_j - M) / L to the three statistics of slots [0, n) (the slot that
// just received the new token starts from zero) and, when the unit is full, writes the ranking keys of the
// updated statistics.  z may live in global memory or in LDS.
// What the ranking keys of a step need besides the statistics: the policy, the slots' positions (read only by
// policies that rank by position) and the position of the token that has just taken `slot`.
struct StepKeys {
  Policy pol;
  const int32_t* pos;
  int qpos;
};

// The update of four adjacent slots j .. j + 3 whose statistics are already in registers.
__device__ __forceinline__ void update_four(float4& a1, float4& a2, float4& cc, const float4 zz, int j, int n, int slot,
                                            float M, float inv, bool full, uint32_t* mas_key, uint32_t* var_key,
                                            const StepKeys& sk) {
  const float zv[4] = {zz.x, zz.y, zz.z, zz.w};
  int pv[4] = {0, 0, 0, 0};
  if (full && sk.pol.needs_pos()) {
    const int4 pp = *reinterpret_cast<const int4*>(sk.pos + j);
    pv[0] = pp.x; pv[1] = pp.y; pv[2] = pp.z; pv[3] = pp.w;
  }
  float s1[4] = {a1.x, a1.y, a1.z, a1.w}, s2[4] = {a2.x, a2.y, a2.z, a2.w}, sc[4] = {cc.x, cc.y, cc.z, cc.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int jj = j + e;
    if (jj < n) {
      if (jj == slot) { s1[e] = 0.0f; s2[e] = 0.0f; sc[e] = 0.0f; }
      const float p = fast_exp2(zv[e] - M) * inv;
      s1[e] += p;
      s2[e] = sk.pol.second_statistic(s2[e], p, static_cast<float>(n));
      sc[e] += 1.0f;
      if (full) ranking_keys(s1[e], s2[e], sc[e], jj == slot ? sk.qpos : pv[e], sk.pol, mas_key[jj], var_key[jj]);
    }
  }
  a1 = make_float4(s1[0], s1[1], s1[2], s1[3]);
  a2 = make_float4(s2[0], s2[1], s2[2], s2[3]);
  cc = make_float4(sc[0], sc[1], sc[2], sc[3]);
}

// Statistics of the first PF groups of four slots of this thread, loaded ahead of their use: issued before the
// K / V stream, they arrive while it runs, so that the update after the stream does not wait on memory.
template <int NT, int PF> struct StatsAhead {
  float4 a1[PF], a2[PF], cc[PF];
  __device__ __forceinline__ void load(const float* acc, const float* acc2, const float* cnt, int n) {
#pragma unroll
    for (int k = 0; k < PF; ++k) {
      const int j = (k * NT + static_cast<int>(threadIdx.x)) * 4;
      const int jc = j < n ? j : 0;  // a group past the end is never used; keep its address inside the planes
      a1[k] = *reinterpret_cast<const float4*>(acc + jc);
      a2[k] = *reinterpret_cast<const float4*>(acc2 + jc);
      cc[k] = *reinterpret_cast<const float4*>(cnt + jc);
    }
  }
};

template <int NT, int PF>
__device__ __forceinline__ void update_statistics(float* acc, float* acc2, float* cnt, const float* z, int n, int B,
                                                  int slot, float M, float inv, bool full, uint32_t* mas_key,
                                                  uint32_t* var_key, StatsAhead<NT, PF>* ahead, const StepKeys& sk) {
  const int tid = threadIdx.x;
  if ((B & 3) == 0) {
    // four adjacent slots per thread, 128-bit accesses on every plane
    if (ahead != nullptr) {
#pragma unroll
      for (int k = 0; k < PF; ++k) {
        const int j = (k * NT + tid) * 4;
        if (j < n) {
          update_four(ahead->a1[k], ahead->a2[k], ahead->cc[k], *reinterpret_cast<const float4*>(z + j), j, n, slot, M,
                      inv, full, mas_key, var_key, sk);
          *reinterpret_cast<float4*>(acc + j) = ahead->a1[k];
          *reinterpret_cast<float4*>(acc2 + j) = ahead->a2[k];
          *reinterpret_cast<float4*>(cnt + j) = ahead->cc[k];
        }
      }
    }
    for (int j = ((ahead != nullptr ? PF * NT : 0) + tid) * 4; j < n; j += NT * 4) {
      float4 a1 = *reinterpret_cast<const float4*>(acc + j);
      float4 a2 = *reinterpret_cast<const float4*>(acc2 + j);
      float4 cc = *reinterpret_cast<const float4*>(cnt + j);
      update_four(a1, a2, cc, *reinterpret_cast<const float4*>(z + j), j, n, slot, M, inv, full, mas_key, var_key, sk);
      *reinterpret_cast<float4*>(acc + j) = a1;
      *reinterpret_cast<float4*>(acc2 + j) = a2;
      *reinterpret_cast<float4*>(cnt + j) = cc;
    }
  } else {
    for (int j = tid; j < n; j += NT) {
      float s1 = acc[j], s2 = acc2[j], sc = cnt[j];
      if (j == slot) { s1 = 0.0f; s2 = 0.0f; sc = 0.0f; }
      const float p = fast_exp2(z[j] - M) * inv;
      s1 += p;
      s2 = sk.pol.second_statistic(s2, p, static_cast<float>(n));
      sc += 1.0f;
      acc[j] = s1; acc2[j] = s2; cnt[j] = sc;
      if (full) ranking_keys(s1, s2, sc, j == slot ? sk.qpos : (sk.pol.needs_pos() ? sk.pos[j] : 0), sk.pol, mas_key[j], var_key[j]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
template <int DT, int D, int NT>
__global__ __launch_bounds__(NT) void decode_finish(DecodeArgs a) {
  extern __shared__ uint32_t lds_keys[];  // [2][B] when B <= kMaxDecodeBudgetLds
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  __shared__ unsigned long long best_sh[NT / kWave];
  __shared__ float mrg_m[kMaxSplits], mrg_l[kMaxSplits];
  __shared__ float mrg_o[NT / D][D];
  static_assert(NT >= kMaxSplits && NT % D == 0, "one thread per split, whole groups per dimension");

  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B, S = a.splits;
  const int n0 = a.n_used[u];
  const bool was_full = n0 >= B;
  const int slot = was_full ? min(max(a.next_slot[u], 0), B - 1) : n0;
  const int n = was_full ? B : n0 + 1;
  const bool full = n >= B;

  // The partial normalisers come in with one load per thread and are merged from LDS, by every thread, in split
  // order; a loop of dependent trips to global memory here would cost more than the rest of the kernel when a
  // unit has many splits.
  if (tid < S) {
    mrg_m[tid] = a.part_m[static_cast<size_t>(u) * S + tid];
    mrg_l[tid] = a.part_l[static_cast<size_t>(u) * S + tid];
  }
  __syncthreads();
  float M = -INFINITY;
  for (int s = 0; s < S; ++s) M = fmaxf(M, mrg_m[s]);
  float Lsum = 0.0f;
  for (int s = 0; s < S; ++s) Lsum += (mrg_m[s] > -INFINITY) ? mrg_l[s] * fast_exp2(mrg_m[s] - M) : 0.0f;
  const float inv = 1.0f / Lsum;

  // output: the threads form NT / D groups, group g sums the splits g, g + NT / D, ... of its dimension
  {
    constexpr int G = NT / D;
    const int g = tid / D, dd = tid % D;
    const float* po = a.part_o + static_cast<size_t>(u) * S * D;
    float o = 0.0f;
    for (int s = g; s < S; s += G) o += (mrg_m[s] > -INFINITY) ? po[s * D + dd] * fast_exp2(mrg_m[s] - M) : 0.0f;
    mrg_o[g][dd] = o;
    __syncthreads();
    if (tid < D) {
      float sum = mrg_o[0][tid];
#pragma unroll
      for (int k = 1; k < G; ++k) sum += mrg_o[k][tid];
      store_elem<DT>(a.out, static_cast<size_t>(u) * D + tid, sum * inv);
    }
  }

  float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  float* acc2 = acc + B;
  float* cnt = acc2 + B;
  const float* z = a.z + static_cast<size_t>(u) * B;
  int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  uint32_t* var_key = (B <= kMaxDecodeBudgetLds) ? lds_keys : a.keys + static_cast<size_t>(u) * 2 * B;
  uint32_t* mas_key = var_key + B;

  // Bookkeeping first: the load counter is in order, so a load issued after the statistics stores could only be
  // waited for together with them, and every wave would sit at the barrier below for the stores' round trip.
  if (tid == 0) {
    const int old_pos = pos[slot];
    pos[slot] = a.qpos[u];
    a.n_used[u] = n;
    if (a.evicted_slot) a.evicted_slot[u] = was_full ? slot : -1;
    if (a.evicted_pos) a.evicted_pos[u] = was_full ? old_pos : -1;
  }
  const StepKeys sk = {a.pol, pos, a.qpos[u]};
  update_statistics<NT, 1>(acc, acc2, cnt, z, n, B, slot, M, inv, full, mas_key, var_key, nullptr, sk);
  if (full) {
    __syncthreads();
    const int victim = select_victim_block<NT>(var_key, mas_key, B, a.pol.scope_size(a.scope, B), sel_sh, best_sh);
    if (tid == 0) a.next_slot[u] = victim;
  }
}

// ------------------------------------------------------------------------------------------------
// The whole step of a unit in one workgroup: stream the unit's K and V once (the new token's rows go into their
// slot on the way), merge the waves' online-softmax states through LDS, write the output, update the
// statistics from the logits kept in LDS and choose the next victim.  Nothing but the final results is written
// to global memory and no second launch is needed; the price is that a workgroup's selection phase does not
// stream, so this shape is used when there are at least about two units per compute unit to overlap with.
template <int DT, int D, int U, bool BIAS, bool STREAMING>
__global__ __launch_bounds__(kFusedThreads) void decode_fused(DecodeArgs a) {
  using G = RowGeom<DT, D>;
  constexpr int NT = kFusedThreads, WAVES = NT / kWave;
  constexpr int PASS = WAVES * U * G::R;
  extern __shared__ __attribute__((aligned(16))) uint32_t lds_dyn[];  // [2][B] ranking keys, then [B] base-2 logits
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  __shared__ unsigned long long best_sh[WAVES];
  __shared__ float sm_m[WAVES], sm_l[WAVES];
  __shared__ float sm_acc[WAVES][D];

  const int u = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int c = lane % G::LPR;
  const int B = a.B;
  const int n0 = a.n_used[u];
  const bool was_full = n0 >= B;
  const int slot = was_full ? min(max(a.next_slot[u], 0), B - 1) : n0;  // where the new token goes
  const int n = was_full ? B : n0 + 1;
  const bool full = n >= B;
  uint32_t* var_key = lds_dyn;
  uint32_t* mas_key = var_key + B;
  float* z = reinterpret_cast<float*>(lds_dyn + 2 * static_cast<size_t>(B));

  const size_t in_off = static_cast<size_t>(u) * G::ROW_BYTES + c * 16;
  float qf[G::EPL];
  unpack16<DT>(load16(static_cast<const char*>(a.q) + in_off), qf);
#pragma unroll
  for (int e = 0; e < G::EPL; ++e) qf[e] *= a.scale_log2;

  char* Kb = static_cast<char*>(a.K) + static_cast<size_t>(u) * B * G::ROW_BYTES;
  char* Vb = static_cast<char*>(a.V) + static_cast<size_t>(u) * B * G::ROW_BYTES;
  int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  const int qp = a.qpos[u];
  const int old_pos = pos[slot];
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;

  float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  constexpr int PF = 512 / NT;  // covers B <= 2048; larger budgets load the rest after the stream
  StatsAhead<NT, PF> ahead;
  const bool vec = (B & 3) == 0;
  if (vec) ahead.load(acc, acc + B, acc + 2 * static_cast<size_t>(B), n);

  FlashState<G::EPL> st;
  st.reset();
  auto bias = [&](int row, int row_pos) -> float {
    const int dlt = (row == slot) ? 0 : qp - row_pos;
    return (dlt >= 0 && dlt < w) ? rb : 0.0f;
  };
  auto fix_k = [&](int row, uint4& kw, int col) {
    if (row == slot && row < n) {
      kw = load16(static_cast<const char*>(a.k_new) + in_off);
      *reinterpret_cast<uint4*>(Kb + static_cast<size_t>(row) * G::ROW_BYTES + col * 16) = kw;
    }
  };
  auto fix_v = [&](int row, uint4& vw, int col) {
    if (row == slot && row < n) {
      vw = load16(static_cast<const char*>(a.v_new) + in_off);
      *reinterpret_cast<uint4*>(Vb + static_cast<size_t>(row) * G::ROW_BYTES + col * 16) = vw;
    }
  };
  const int passes = (n + PASS - 1) / PASS;
  const int rot = a.rotate ? static_cast<int>((static_cast<unsigned>(u) * 5u) % static_cast<unsigned>(passes)) : 0;
  stream_attend<DT, D, U, BIAS, STREAMING>(qf, Kb, Vb, 0, n, passes, rot, PASS, wave * (U * G::R), bias, pos, z, slot,
                                           fix_k, fix_v, st);
  merge_groups_in_wave<DT, D>(st);

  if (lane < G::LPR) {
    if (lane == 0) { sm_m[wave] = st.m; sm_l[wave] = st.l; }
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) sm_acc[wave][lane * G::EPL + e] = st.acc[e];
  }
  __syncthreads();  // also orders the waves' logit stores before the reads below
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < WAVES; ++s) M = fmaxf(M, sm_m[s]);
  float Lsum = 0.0f;
#pragma unroll
  for (int s = 0; s < WAVES; ++s) Lsum += (sm_m[s] > -INFINITY) ? sm_l[s] * fast_exp2(sm_m[s] - M) : 0.0f;
  const float inv = 1.0f / Lsum;
  if (tid < D) {
    float o = 0.0f;
#pragma unroll
    for (int s = 0; s < WAVES; ++s) o += (sm_m[s] > -INFINITY) ? sm_acc[s][tid] * fast_exp2(sm_m[s] - M) : 0.0f;
    store_elem<DT>(a.out, static_cast<size_t>(u) * D + tid, o * inv);
  }

  // (bookkeeping before the statistics stores: no load may follow them, see decode_finish)
  if (tid == 0) {
    pos[slot] = qp;
    a.n_used[u] = n;
    if (a.evicted_slot) a.evicted_slot[u] = was_full ? slot : -1;
    if (a.evicted_pos) a.evicted_pos[u] = was_full ? old_pos : -1;
  }
  update_statistics<NT, PF>(acc, acc + B, acc + 2 * static_cast<size_t>(B), z, n, B, slot, M, inv, full, mas_key,
                            var_key, vec ? &ahead : nullptr, StepKeys{a.pol, pos, qp});
  if (full) {
    __syncthreads();
    const int victim = select_victim_block<NT>(var_key, mas_key, B, a.pol.scope_size(a.scope, B), sel_sh, best_sh);
    if (tid == 0) a.next_slot[u] = victim;
  }
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kFinishThreads) void select_victims(DecodeArgs a) {
  constexpr int NT = kFinishThreads;
  extern __shared__ uint32_t lds_keys[];
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  __shared__ unsigned long long best_sh[NT / kWave];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B;
  if (a.n_used[u] < B) {
    if (tid == 0) a.next_slot[u] = -1;
    return;
  }
  const float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  const float* acc2 = acc + B;
  const float* cnt = acc2 + B;
  uint32_t* var_key = (B <= kMaxDecodeBudgetLds) ? lds_keys : a.keys + static_cast<size_t>(u) * 2 * B;
  uint32_t* mas_key = var_key + B;
  const bool by_pos = a.pol.needs_pos();
  const int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  for (int i = tid; i < B; i += NT)
    ranking_keys(acc[i], acc2[i], cnt[i], by_pos ? pos[i] : 0, a.pol, mas_key[i], var_key[i]);
  __syncthreads();
  const int victim = select_victim_block<NT>(var_key, mas_key, B, a.pol.scope_size(a.scope, B), sel_sh, best_sh);
  if (tid == 0) a.next_slot[u] = victim;
}

// Benchmark aid: the memory side of decode_attend alone.  Same grid, same rows per workgroup, same 128-bit
// loads in the same order, no arithmetic beyond an xor that keeps the loads alive: what this kernel reaches is
// the read bandwidth the access pattern can get on the machine at hand.
template <int ROW_BYTES, int U, bool STREAMING>
__global__ __launch_bounds__(kAttendThreads) void cache_read_probe(DecodeArgs a) {
  constexpr int LPR = ROW_BYTES / 16, R = kWave / LPR, PASS = kAttendWaves * U * R;
  const int u = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int g = lane / LPR, c = lane % LPR;
  const int row0 = split * a.rows_per_split;
  const int row1 = min(a.B, row0 + a.rows_per_split);
  const char* Kb = static_cast<const char*>(a.K) + static_cast<size_t>(u) * a.B * ROW_BYTES;
  const char* Vb = static_cast<const char*>(a.V) + static_cast<size_t>(u) * a.B * ROW_BYTES;
  uint32_t x = 0;
  for (int base = row0 + wave * (U * R); base < row1; base += PASS) {
    uint4 kw[U], vw[U];
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int row = base + i * R + g;
      const size_t off = static_cast<size_t>(row < row1 ? row : row0) * ROW_BYTES + c * 16;
      kw[i] = STREAMING ? load16_streaming(Kb + off) : load16(Kb + off);
      vw[i] = STREAMING ? load16_streaming(Vb + off) : load16(Vb + off);
    }
#pragma unroll
    for (int i = 0; i < U; ++i)
      x ^= kw[i].x ^ kw[i].y ^ kw[i].z ^ kw[i].w ^ vw[i].x ^ vw[i].y ^ vw[i].z ^ vw[i].w;
  }
  if (x == 0x9e3779b9u) a.part_m[static_cast<size_t>(u) * a.splits + split] = 1.0f;  // practically never taken
}

template <int DT, int D, int U>
void launch_attend(const DecodeArgs& a, hipStream_t s) {
  ProfScope ps(kProfDecodeAttend, s);
  const dim3 grid(a.splits, a.units), block(kAttendThreads);
  const bool bias = a.recency_window > 0, nt = a.streaming != 0;
  if (bias && nt) hipLaunchKernelGGL((decode_attend<DT, D, U, true, true>), grid, block, 0, s, a);
  else if (bias) hipLaunchKernelGGL((decode_attend<DT, D, U, true, false>), grid, block, 0, s, a);
  else if (nt) hipLaunchKernelGGL((decode_attend<DT, D, U, false, true>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((decode_attend<DT, D, U, false, false>), grid, block, 0, s, a);
}

template <int DT, int D>
hipError_t launch_decode_t(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = key_lds_bytes(a.B);
  if (a.fused) {  // requires B <= kMaxFusedBudget (checked by the host)
    ProfScope ps(kProfDecodeAttend, s);
    const size_t lds3 = static_cast<size_t>(a.B) * 3 * sizeof(uint32_t);
    const dim3 grid(a.units), block(kFusedThreads);
    const bool bias = a.recency_window > 0, nt = a.streaming != 0;
    if (bias && nt) hipLaunchKernelGGL((decode_fused<DT, D, 8, true, true>), grid, block, lds3, s, a);
    else if (bias) hipLaunchKernelGGL((decode_fused<DT, D, 8, true, false>), grid, block, lds3, s, a);
    else if (nt) hipLaunchKernelGGL((decode_fused<DT, D, 8, false, true>), grid, block, lds3, s, a);
    else hipLaunchKernelGGL((decode_fused<DT, D, 8, false, false>), grid, block, lds3, s, a);
    return hipGetLastError();
  }
  switch (a.unroll) {
    case 2: launch_attend<DT, D, 2>(a, s); break;
    case 8: launch_attend<DT, D, 8>(a, s); break;
    default: launch_attend<DT, D, 4>(a, s); break;
  }
  {
    ProfScope ps(kProfDecodeFinish, s);
    // A unit's statistics and selection are one workgroup's work: 1024 threads when there is at most one unit per
    // compute unit and enough slots to share out (measured: faster from 1024 slots on, e.g. 34 -> 28 us per step at
    // 40 units x 4096 slots, 78 -> 64 at 64 x 8192), else 256.
    if (a.B >= 1024 && a.units <= 256) {
      if (!allow_key_lds(reinterpret_cast<const void*>(decode_finish<DT, D, 1024>), lds)) return hipErrorInvalidValue;
      hipLaunchKernelGGL((decode_finish<DT, D, 1024>), dim3(a.units), dim3(1024), lds, s, a);
    } else {
      if (!allow_key_lds(reinterpret_cast<const void*>(decode_finish<DT, D, kFinishThreads>), lds))
        return hipErrorInvalidValue;
      hipLaunchKernelGGL((decode_finish<DT, D, kFinishThreads>), dim3(a.units), dim3(kFinishThreads), lds, s, a);
    }
  }
  return hipGetLastError();
}

}  // namespace

// Rows one decode_attend workgroup covers per pass over its waves, for the given shape and unroll; the host
// picks rows_per_split as a multiple of it.
int decode_rows_per_pass(int dtype, int head_dim, int unroll) {
  const int epl = dtype == kBF16 ? 8 : 4;
  const int lpr = head_dim / epl;
  return kAttendWaves * unroll * (kWave / lpr);
}

hipError_t launch_decode(int dtype, int head_dim, const DecodeArgs& a, hipStream_t s) {
  if (dtype == kF32 && head_dim == 64) return launch_decode_t<kF32, 64>(a, s);
  if (dtype == kF32 && head_dim == 128) return launch_decode_t<kF32, 128>(a, s);
  if (dtype == kBF16 && head_dim == 64) return launch_decode_t<kBF16, 64>(a, s);
  if (dtype == kBF16 && head_dim == 128) return launch_decode_t<kBF16, 128>(a, s);
  return hipErrorInvalidValue;
}

hipError_t launch_cache_read_probe(int dtype, int head_dim, const DecodeArgs& a, hipStream_t s) {
  const int row_bytes = head_dim * (dtype == kBF16 ? 2 : 4);
  const dim3 grid(a.splits, a.units);
  ProfScope ps(kProfReadProbe, s);
  switch (row_bytes) {
    case 128:
      if (a.streaming) hipLaunchKernelGGL((cache_read_probe<128, 8, true>), grid, dim3(kAttendThreads), 0, s, a);
      else hipLaunchKernelGGL((cache_read_probe<128, 8, false>), grid, dim3(kAttendThreads), 0, s, a);
      break;
    case 256:
      if (a.streaming) hipLaunchKernelGGL((cache_read_probe<256, 8, true>), grid, dim3(kAttendThreads), 0, s, a);
      else hipLaunchKernelGGL((cache_read_probe<256, 8, false>), grid, dim3(kAttendThreads), 0, s, a);
      break;
    case 512:
      if (a.streaming) hipLaunchKernelGGL((cache_read_probe<512, 8, true>), grid, dim3(kAttendThreads), 0, s, a);
      else hipLaunchKernelGGL((cache_read_probe<512, 8, false>), grid, dim3(kAttendThreads), 0, s, a);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_select_victims(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = key_lds_bytes(a.B);
  if (!allow_key_lds(reinterpret_cast<const void*>(select_victims), lds)) return hipErrorInvalidValue;
  ProfScope ps(kProfDecodeSelect, s);
  hipLaunchKernelGGL(select_victims, dim3(a.units), dim3(kFinishThreads), lds, s, a);
  return hipGetLastError();
}

}  // namespace roco
