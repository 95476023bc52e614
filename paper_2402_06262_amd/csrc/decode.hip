// RoCo decode step on gfx950: victim selection + in-place slot overwrite, split-K attention over the
// budgeted cache, and the combine that also updates Acc / Acc2 / Count (section 4.3 of the paper; Fig. 1:
// one key/value pair is deleted before the next token's is appended).
//
// Three kernels per step, all on the caller's stream:
//   1. decode_select_update : one workgroup per unit.  If the unit's buffer is full, rank the slots by
//      attention variance, take the `scope` lowest as the eviction scope and pick the slot of lowest mean
//      attention score inside it; then write k_new / v_new / qpos into the slot and zero its statistics.
//   2. decode_attend        : grid (splits, units).  Streams K and V of its slot range once with 128-bit
//      loads, keeps an online softmax per lane group, stores every base-2 logit, writes one partial
//      (max, sum, weighted V sum) per split.  HBM-bound: no matrix cores.
//   3. decode_combine_stats : grid (slot blocks, units).  Merges the partials in split order (fixed order:
//      results do not depend on scheduling), writes the attention output, and adds p, p^2 and 1 into the
//      three statistics planes.
#include "kernels.hpp"
#include "profile.hpp"
#include "stream.hpp"

namespace roco {
namespace {

constexpr int kAttendThreads = 256;
constexpr int kAttendWaves = kAttendThreads / kWave;
constexpr int kAttendUnroll = 4;
constexpr int kCombineThreads = 256;
constexpr int kCombineSlots = 1024;  // slots per combine workgroup

// ------------------------------------------------------------------------------------------------
template <int DT, int D>
__global__ __launch_bounds__(kDecodeSelectThreads) void decode_select_update(DecodeArgs a) {
  constexpr int NT = kDecodeSelectThreads;
  using G = RowGeom<DT, D>;
  extern __shared__ uint32_t lds_keys[];  // [2][B] when B <= kMaxDecodeBudgetLds
  __shared__ uint32_t sel_sh[256 + NT / kWave + 3];
  __shared__ unsigned long long best_sh[NT / kWave];
  __shared__ int slot_sh;

  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B;
  const int n = a.n_used[u];
  float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  float* acc2 = acc + B;
  float* cnt = acc2 + B;
  int32_t* pos = a.pos + static_cast<size_t>(u) * B;

  int slot, ev_slot = -1, ev_pos = -1;
  if (n < B) {
    slot = n;
  } else {
    uint32_t* var_key = (B <= kMaxDecodeBudgetLds) ? lds_keys : a.keys + static_cast<size_t>(u) * 2 * B;
    uint32_t* mas_key = var_key + B;
    for (int i = tid; i < B; i += NT) {
      uint32_t mk, vk;
      ranking_keys(acc[i], acc2[i], cnt[i], mk, vk);
      var_key[i] = vk;
      mas_key[i] = mk;
    }
    __syncthreads();
    const KSmallest sc = select_k_smallest<NT>([&](int i) { return var_key[i]; }, B,
                                               static_cast<uint32_t>(a.scope), sel_sh);
    // lowest mean attention score inside the scope; equal scores go to the lowest slot
    unsigned long long best = ~0ull;
    for (int i = tid; i < B; i += NT) {
      if (sc.has(var_key[i], i)) {
        const unsigned long long cand = (static_cast<unsigned long long>(mas_key[i]) << 32) | static_cast<uint32_t>(i);
        best = cand < best ? cand : best;
      }
    }
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
      const unsigned long long o = __shfl_xor(best, m, kWave);
      best = o < best ? o : best;
    }
    if ((tid & (kWave - 1)) == 0) best_sh[tid / kWave] = best;
    __syncthreads();
    if (tid == 0) {
      unsigned long long b = best_sh[0];
      for (int w = 1; w < NT / kWave; ++w) b = best_sh[w] < b ? best_sh[w] : b;
      slot_sh = static_cast<int>(b & 0xffffffffu);
    }
    __syncthreads();
    slot = slot_sh;
    ev_slot = slot;
    ev_pos = pos[slot];
  }
  __syncthreads();  // every thread has read pos[slot] / n_used before they change

  // overwrite the slot in place: the cache never grows past B and is never reallocated
  const size_t row = (static_cast<size_t>(u) * B + slot) * G::ROW_BYTES;
  const size_t in_row = static_cast<size_t>(u) * G::ROW_BYTES;
  if (tid < G::LPR) {
    *reinterpret_cast<uint4*>(static_cast<char*>(a.K) + row + tid * 16) =
        load16(static_cast<const char*>(a.k_new) + in_row + tid * 16);
  } else if (tid >= kWave && tid < kWave + G::LPR) {
    const int t = tid - kWave;
    *reinterpret_cast<uint4*>(static_cast<char*>(a.V) + row + t * 16) =
        load16(static_cast<const char*>(a.v_new) + in_row + t * 16);
  } else if (tid == 2 * kWave) {
    pos[slot] = a.qpos[u];
    acc[slot] = 0.0f;
    acc2[slot] = 0.0f;
    cnt[slot] = 0.0f;
    if (n < B) a.n_used[u] = n + 1;
    if (a.evicted_slot) a.evicted_slot[u] = ev_slot;
    if (a.evicted_pos) a.evicted_pos[u] = ev_pos;
  }
}

// ------------------------------------------------------------------------------------------------
template <int DT, int D>
__global__ __launch_bounds__(kAttendThreads) void decode_attend(DecodeArgs a) {
  using G = RowGeom<DT, D>;
  constexpr int U = kAttendUnroll;
  constexpr int STREAMS = kAttendWaves;  // one merged stream per wave reaches LDS
  __shared__ float sm_m[STREAMS], sm_l[STREAMS];
  __shared__ float sm_acc[STREAMS][D];

  const int u = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int c = lane % G::LPR;
  const int n = a.n_used[u];
  const int row0 = split * a.rows_per_split;
  const int row1 = min(n, row0 + a.rows_per_split);

  float qf[G::EPL];
  {
    const uint4 qw = load16(static_cast<const char*>(a.q) + static_cast<size_t>(u) * G::ROW_BYTES + c * 16);
    unpack16<DT>(qw, qf);
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) qf[e] *= a.scale_log2;
  }
  const char* Kb = static_cast<const char*>(a.K) + static_cast<size_t>(u) * a.B * G::ROW_BYTES;
  const char* Vb = static_cast<const char*>(a.V) + static_cast<size_t>(u) * a.B * G::ROW_BYTES;
  float* z = a.z + static_cast<size_t>(u) * a.B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * a.B;
  const int qp = a.qpos[u];
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;

  FlashState<G::EPL> st;
  st.reset();
  auto bias = [&](int row) -> float {
    if (w <= 0) return 0.0f;
    const int dlt = qp - pos[row];
    return (dlt >= 0 && dlt < w) ? rb : 0.0f;
  };
  auto zstore = [&](int row, float t) { z[row] = t; };
  stream_attend<DT, D, U>(qf, Kb, Vb, row0 + wave * (U * G::R), row1, kAttendWaves * U * G::R, bias, zstore, st);
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
      const float wgt = (sm_m[s] > -INFINITY) ? exp2f(sm_m[s] - M) : 0.0f;
      l += sm_l[s] * wgt;
      o += sm_acc[s][tid] * wgt;
    }
    a.part_o[pidx * D + tid] = o;
    if (tid == 0) { a.part_m[pidx] = M; a.part_l[pidx] = l; }
  }
}

// ------------------------------------------------------------------------------------------------
template <int DT, int D>
__global__ __launch_bounds__(kCombineThreads) void decode_combine_stats(DecodeArgs a) {
  const int u = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
  const int B = a.B, S = a.splits;
  const int n = a.n_used[u];
  const float* pm = a.part_m + static_cast<size_t>(u) * S;
  const float* pl = a.part_l + static_cast<size_t>(u) * S;

  // every thread merges the (few) partial normalisers in split order
  float M = -INFINITY;
  for (int s = 0; s < S; ++s) M = fmaxf(M, pm[s]);
  float Lsum = 0.0f;
  for (int s = 0; s < S; ++s) Lsum += (pm[s] > -INFINITY) ? pl[s] * exp2f(pm[s] - M) : 0.0f;
  const float inv = 1.0f / Lsum;

  if (blk == 0 && tid < D) {
    const float* po = a.part_o + static_cast<size_t>(u) * S * D;
    float o = 0.0f;
    for (int s = 0; s < S; ++s) o += (pm[s] > -INFINITY) ? po[s * D + tid] * exp2f(pm[s] - M) : 0.0f;
    store_elem<DT>(a.out, static_cast<size_t>(u) * D + tid, o * inv);
  }

  float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  float* acc2 = acc + B;
  float* cnt = acc2 + B;
  const float* z = a.z + static_cast<size_t>(u) * B;
  const int lo = blk * kCombineSlots;
  const int hi = min(n, lo + kCombineSlots);
  for (int j = lo + tid; j < hi; j += kCombineThreads) {
    const float p = exp2f(z[j] - M) * inv;
    acc[j] += p;
    acc2[j] += p * p;
    cnt[j] += 1.0f;
  }
}

template <int DT, int D>
hipError_t launch_decode_t(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = (a.B <= kMaxDecodeBudgetLds) ? static_cast<size_t>(a.B) * 2 * sizeof(uint32_t) : 0;
  {
    ProfScope ps(kProfDecodeSelect, s);
    hipLaunchKernelGGL((decode_select_update<DT, D>), dim3(a.units), dim3(kDecodeSelectThreads), lds, s, a);
  }
  {
    ProfScope ps(kProfDecodeAttend, s);
    hipLaunchKernelGGL((decode_attend<DT, D>), dim3(a.splits, a.units), dim3(kAttendThreads), 0, s, a);
  }
  {
    ProfScope ps(kProfDecodeCombine, s);
    hipLaunchKernelGGL((decode_combine_stats<DT, D>),
                       dim3((a.B + kCombineSlots - 1) / kCombineSlots, a.units), dim3(kCombineThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace

// Rows one decode_attend workgroup covers per pass over its waves, for the given shape; the host picks
// rows_per_split as a multiple of it.
int decode_rows_per_pass(int dtype, int head_dim) {
  const int epl = dtype == kBF16 ? 8 : 4;
  const int lpr = head_dim / epl;
  return kAttendWaves * kAttendUnroll * (kWave / lpr);
}

hipError_t launch_decode(int dtype, int head_dim, const DecodeArgs& a, hipStream_t s) {
  if (dtype == kF32 && head_dim == 64) return launch_decode_t<kF32, 64>(a, s);
  if (dtype == kF32 && head_dim == 128) return launch_decode_t<kF32, 128>(a, s);
  if (dtype == kBF16 && head_dim == 64) return launch_decode_t<kBF16, 64>(a, s);
  if (dtype == kBF16 && head_dim == 128) return launch_decode_t<kBF16, 128>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace roco
