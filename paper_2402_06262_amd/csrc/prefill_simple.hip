// Prefill attention statistics on the plain vector ALUs, for every supported dtype / head_dim.
//
// This is the general path (fp32 storage, head_dim 64) and the cross-check for the matrix-core path.
// Two passes, because a column statistic needs the final normaliser of every row it sums over:
//   pass 1: one wave per query row i streams keys 0..i with an online softmax and stores the row's base-2
//           log-sum-exp (and the attention output, if asked)                     (section 2.1, eq. 1; causal)
//   pass 2: one wave per key column j streams queries j..len-1, recomputes the logit and accumulates
//           Acc[j] = sum_i P[i,j] and Acc2[j] = sum_i P[i,j]^2 in fp32            (section 4.3)
// Count[j] = len - j has a closed form and is not accumulated.  The L x L matrix is never stored.
#include "kernels.hpp"
#include "profile.hpp"
#include "stream.hpp"

namespace roco {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kUnroll = 4;

template <int DT, int D>
__global__ __launch_bounds__(kThreads) void prefill_rows_simple(PrefillArgs a) {
  using G = RowGeom<DT, D>;
  const int uq = blockIdx.y;       // (unit, query head)
  const int uk = uq / a.group;     // the unit: its keys, values and length
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int c = lane % G::LPR;
  const int i = blockIdx.x * kWaves + wave;
  const int len = a.len[uk];
  if (i >= len) return;
  const size_t ubase = static_cast<size_t>(uq) * a.L_max;
  const size_t kbase = static_cast<size_t>(uk) * a.L_max;
  float qf[G::EPL];
  unpack16<DT>(load16(static_cast<const char*>(a.Q) + (ubase + i) * G::ROW_BYTES + c * 16), qf);
#pragma unroll
  for (int e = 0; e < G::EPL; ++e) qf[e] *= a.scale_log2;
  const char* Kb = static_cast<const char*>(a.K) + kbase * G::ROW_BYTES;
  const char* Vb = static_cast<const char*>(a.V) + kbase * G::ROW_BYTES;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  FlashState<G::EPL> st;
  st.reset();
  auto bias = [&](int row, int) -> float { return (i - row < w) ? rb : 0.0f; };  // row <= i here
  auto fix = [](int, uint4&, int) {};
  constexpr int PASS = kUnroll * G::R;
  if (w > 0)
    stream_attend<DT, D, kUnroll, true, false>(qf, Kb, Vb, 0, i + 1, (i + PASS) / PASS, 0, PASS, 0, bias, nullptr, nullptr, -1, fix, fix, st);
  else
    stream_attend<DT, D, kUnroll, false, false>(qf, Kb, Vb, 0, i + 1, (i + PASS) / PASS, 0, PASS, 0, bias, nullptr, nullptr, -1, fix, fix, st);
  merge_groups_in_wave<DT, D>(st);
  if (lane == 0) a.lse[ubase + i] = st.m + log2f(st.l);
  if (a.O != nullptr && lane < G::LPR) {
    const float inv = 1.0f / st.l;
#pragma unroll
    for (int e = 0; e < G::EPL; ++e)
      store_elem<DT>(a.O, (ubase + i) * D + lane * G::EPL + e, st.acc[e] * inv);
  }
}

template <int DT, int D>
__global__ __launch_bounds__(kThreads) void prefill_columns_simple(PrefillArgs a) {
  using G = RowGeom<DT, D>;
  constexpr int U = kUnroll;
  const int u = blockIdx.y;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / G::LPR, c = lane % G::LPR;
  const int j = blockIdx.x * kWaves + wave;
  const int len = a.len[u];
  if (j >= len) return;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  float kf[G::EPL];
  unpack16<DT>(load16(static_cast<const char*>(a.K) + (ubase + j) * G::ROW_BYTES + c * 16), kf);
#pragma unroll
  for (int e = 0; e < G::EPL; ++e) kf[e] *= a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const float inv_heads = 1.0f / static_cast<float>(a.group);
  float s1 = 0.0f, s2 = 0.0f;
  for (int base = j; base < len; base += U * G::R) {
    float pbar[U];  // sum over the unit's query heads of P[row, j] (one head without grouped-query attention)
#pragma unroll
    for (int x = 0; x < U; ++x) pbar[x] = 0.0f;
    for (int h = 0; h < a.group; ++h) {
      const size_t qbase = (static_cast<size_t>(u) * a.group + h) * a.L_max;
      const char* Qb = static_cast<const char*>(a.Q) + qbase * G::ROW_BYTES;
      const float* lse = a.lse + qbase;
      uint4 qw[U];
      float ls[U];
#pragma unroll
      for (int x = 0; x < U; ++x) {
        const int row = base + x * G::R + g;
        const int r = row < len ? row : j;
        qw[x] = load16(Qb + static_cast<size_t>(r) * G::ROW_BYTES + c * 16);
        ls[x] = lse[r];
      }
#pragma unroll
      for (int x = 0; x < U; ++x) {
        const int row = base + x * G::R + g;
        float qf[G::EPL];
        unpack16<DT>(qw[x], qf);
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) dot = fmaf(qf[e], kf[e], dot);
        dot = group_sum<G::LPR>(dot);
        if (row < len) {
          const float t = dot + ((row - j < w) ? rb : 0.0f);
          pbar[x] += exp2f(t - ls[x]);
        }
      }
    }
#pragma unroll
    for (int x = 0; x < U; ++x) {
      const float p = pbar[x] * inv_heads;  // rows past the end contribute exactly zero
      s1 += p;
      if (a.pol.counts_above_average()) s2 += (p * static_cast<float>(base + x * G::R + g + 1) > 1.0f) ? 1.0f : 0.0f;
      else s2 = fmaf(p, p, s2);
    }
  }
#pragma unroll
  for (int m = G::LPR; m < kWave; m <<= 1) {
    s1 += __shfl_xor(s1, m, kWave);
    s2 += __shfl_xor(s2, m, kWave);
  }
  if (lane == 0) {
    a.acc[ubase + j] = s1;
    a.acc2[ubase + j] = s2;
  }
}

template <int DT, int D>
hipError_t launch_t(const PrefillArgs& a, hipStream_t s) {
  const dim3 grid((a.L_max + kWaves - 1) / kWaves, a.units);
  if (!a.skip_rows) {
    ProfScope ps(kProfPrefillRows, s);
    const dim3 rows_grid(grid.x, static_cast<unsigned>(a.units) * a.group);
    hipLaunchKernelGGL((prefill_rows_simple<DT, D>), rows_grid, dim3(kThreads), 0, s, a);
  }
  {
    ProfScope ps(kProfPrefillColumns, s);
    hipLaunchKernelGGL((prefill_columns_simple<DT, D>), grid, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

// The attention row of the last prompt token, P[len-1, j] for every key j, written over Acc2: the second
// statistic of the last-token importance score (section 4.1, LTAS).  One workgroup per unit; a lane group owns
// a key row, as in the passes above.  Needs the row normalisers of pass 1.
template <int DT, int D>
__global__ __launch_bounds__(kThreads) void prefill_last_row(PrefillArgs a) {
  using G = RowGeom<DT, D>;
  const int u = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / G::LPR, c = lane % G::LPR;
  const int len = a.len[u];
  const int last = len - 1;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Kb = static_cast<const char*>(a.K) + ubase * G::ROW_BYTES;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const float inv_heads = 1.0f / static_cast<float>(a.group);
  constexpr int U = 4;  // key rows in flight per lane group: the loop is bound by load latency, not by bytes
  // the last token's query, scaled, and its normaliser: loaded once when the unit has a single head
  float q0[G::EPL];
  float lse0 = 0.0f;
  auto load_query = [&](int h, float* qs, float& lse_h) {
    const size_t qbase = (static_cast<size_t>(u) * a.group + h) * a.L_max;
    float qf[G::EPL];
    unpack16<DT>(load16(static_cast<const char*>(a.Q) + (qbase + last) * G::ROW_BYTES + c * 16), qf);
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) qs[e] = qf[e] * a.scale_log2;
    lse_h = a.lse[qbase + last];
  };
  if (a.group == 1) load_query(0, q0, lse0);
  for (int base = wave * G::R; base < len; base += kWaves * G::R * U) {
    float kf[U][G::EPL];
    int jc[U];
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const int j = base + r * kWaves * G::R + g;
      jc[r] = j < len ? j : last;
      unpack16<DT>(load16(Kb + static_cast<size_t>(jc[r]) * G::ROW_BYTES + c * 16), kf[r]);
    }
    float pbar[U] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int h = 0; h < a.group; ++h) {  // the unit's query heads (one without grouped-query attention)
      float qh[G::EPL];
      float lse_h = lse0;
      if (a.group == 1) {
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) qh[e] = q0[e];
      } else {
        load_query(h, qh, lse_h);
      }
#pragma unroll
      for (int r = 0; r < U; ++r) {
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) dot = fmaf(qh[e], kf[r][e], dot);
        dot = group_sum<G::LPR>(dot);
        if (w > 0 && last - jc[r] < w) dot += rb;
        pbar[r] += fast_exp2(dot - lse_h);
      }
    }
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const int j = base + r * kWaves * G::R + g;
      if (c == 0 && j < len) a.acc2[ubase + j] = pbar[r] * inv_heads;
    }
  }
}

// Row normalisers handed in as natural logarithms, rescaled to the base-2 form the passes use.
__global__ __launch_bounds__(kThreads) void lse_to_base2(const float* in, float* out, size_t n) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i < n) out[i] = in[i] * 1.4426950408889634f;
}

}  // namespace

hipError_t launch_lse_to_base2(const float* lse_ln, float* lse_log2, size_t n, hipStream_t s) {
  const size_t blocks = (n + kThreads - 1) / kThreads;
  if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(lse_to_base2, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, s, lse_ln, lse_log2, n);
  return hipGetLastError();
}

hipError_t launch_prefill_last_row(int dtype, int head_dim, const PrefillArgs& a, hipStream_t s) {
  const dim3 grid(a.units), block(kThreads);
  if (dtype == kF32 && head_dim == 64) hipLaunchKernelGGL((prefill_last_row<kF32, 64>), grid, block, 0, s, a);
  else if (dtype == kF32 && head_dim == 128) hipLaunchKernelGGL((prefill_last_row<kF32, 128>), grid, block, 0, s, a);
  else if (dtype == kBF16 && head_dim == 64) hipLaunchKernelGGL((prefill_last_row<kBF16, 64>), grid, block, 0, s, a);
  else if (dtype == kBF16 && head_dim == 128) hipLaunchKernelGGL((prefill_last_row<kBF16, 128>), grid, block, 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_prefill_attention_simple(int dtype, int head_dim, const PrefillArgs& a, hipStream_t s) {
  if (dtype == kF32 && head_dim == 64) return launch_t<kF32, 64>(a, s);
  if (dtype == kF32 && head_dim == 128) return launch_t<kF32, 128>(a, s);
  if (dtype == kBF16 && head_dim == 64) return launch_t<kBF16, 64>(a, s);
  if (dtype == kBF16 && head_dim == 128) return launch_t<kBF16, 128>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace roco
