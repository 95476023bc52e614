// Prefill attention statistics on the gfx950 matrix cores: bf16 storage, head_dim 128.
//
// Two passes over the causal score matrix (a column statistic needs the final normaliser of every row it
// sums over), neither of which stores the L x L matrix:
//   pass 1  prefill_rows_mfma    : row normalisers -- base-2 log-sum-exp of every query row (section 2.1 eq. 1)
//   pass 2  prefill_columns_mfma : Acc[j] = sum_i P[i,j], Acc2[j] = sum_i P[i,j]^2 in fp32 (section 4.3)
//
// Both passes have the same shape.  A workgroup owns 128 rows of one operand (queries in pass 1, keys in
// pass 2), 32 per wave, held in registers as the B operand of v_mfma_f32_32x32x16_bf16; the other operand is
// streamed through LDS in tiles of 64 rows (A operand).  The 32x32 result tile then has the *owned* row in the
// lane (column = lane % 32) and the streamed rows in the 16 accumulator registers, so the reduction the pass
// needs (over keys in pass 1, over queries in pass 2) runs down the registers of a lane: no cross-lane traffic
// per tile, no atomics, a fixed summation order.
//
// Operand layout of the 32x32x16 instruction, as used here: lane l supplies row (l % 32) and the 8
// consecutive k-elements starting at 8 * (l / 32) of each 16-wide k-step, for A and for B alike; register r
// of the result belongs to A-row 8 * (r / 4) + 4 * (l / 32) + (r % 4) and B-row (l % 32).
#include "kernels.hpp"
#include "profile.hpp"
#include "stream.hpp"

namespace roco {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kOwn = 32 * kWaves;        // owned rows per workgroup
constexpr int kTile = 64;                // streamed rows per LDS tile
constexpr int kRowBytes = D * 2;         // 256
constexpr int kLdsRow = kRowBytes + 16;  // padded: 16 lanes x 16 B then hit distinct bank groups
constexpr int kKSteps = D / 16;          // 8 matrix instructions per 32x32 tile

struct Staged {
  uint4 w[4];  // this thread's 64 bytes of a 64 x 256 B tile
};

// Thread t of 256 copies bytes [t*16 + i*4096, +16) of the tile, i < 4: row = (t + 256 i) / 16, column chunk t % 16.
__device__ __forceinline__ void tile_load(Staged& s, const char* base, int row0, int last_row) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = row0 + (t >> 4) + 16 * i;
    row = row < last_row ? row : last_row;  // clamp: rows past the end are masked by the caller
    s.w[i] = load16(base + static_cast<size_t>(row) * kRowBytes + (t & 15) * 16);
  }
}
__device__ __forceinline__ void tile_store(const Staged& s, char* lds) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<uint4*>(lds + ((t >> 4) + 16 * i) * kLdsRow + (t & 15) * 16) = s.w[i];
}

// One 32x32 score tile: streamed rows [sub*32, sub*32+32) of the LDS tile against this wave's owned rows.
__device__ __forceinline__ f32x16 score_tile(const char* lds, int sub, const uint4* own) {
  const int lane = threadIdx.x & (kWave - 1);
  const char* p = lds + (sub * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
  f32x16 acc = {0};
#pragma unroll
  for (int kk = 0; kk < kKSteps; ++kk) {
    const uint4 a = *reinterpret_cast<const uint4*>(p + kk * 32);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, own[kk]),
                                                  acc, 0, 0, 0);
  }
  return acc;
}

__device__ __forceinline__ void load_owned(uint4* own, const char* base, int row, int last_row) {
  const int lane = threadIdx.x & (kWave - 1);
  row = row < last_row ? row : last_row;
#pragma unroll
  for (int kk = 0; kk < kKSteps; ++kk)
    own[kk] = load16(base + static_cast<size_t>(row) * kRowBytes + kk * 32 + (lane >> 5) * 16);
}

// ------------------------------------------------------------------------------------------------
// pass 1: lse[i] = log2 sum_{j<=i} 2^(t_ij),  t_ij = scale*log2(e) * q_i.k_j + bias
__global__ __launch_bounds__(kThreads) void prefill_rows_mfma(PrefillArgs a) {
  __shared__ __attribute__((aligned(16))) char lds[2][kTile * kLdsRow];
  const int u = blockIdx.y;
  const int len = a.len[u];
  const int q0 = (gridDim.x - 1 - blockIdx.x) * kOwn;  // long rows first
  if (q0 >= len) return;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Qb = static_cast<const char*>(a.Q) + ubase * kRowBytes;
  const char* Kb = static_cast<const char*>(a.K) + ubase * kRowBytes;
  const int qw0 = q0 + 32 * wave;      // first query of this wave
  const int qi = qw0 + (lane & 31);    // this lane's query
  const int half = lane >> 5;
  uint4 own[kKSteps];
  load_owned(own, Qb, qi, len - 1);

  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  float m = -INFINITY, l = 0.0f;

  const int last_key = min(len, q0 + kOwn) - 1;  // keys 0..last_key are visible to some query of the block
  const int n_tiles = last_key / kTile + 1;
  Staged st;
  tile_load(st, Kb, 0, len - 1);
  for (int t = 0; t < n_tiles; ++t) {
    tile_store(st, lds[t & 1]);
    __syncthreads();
    if (t + 1 < n_tiles) tile_load(st, Kb, (t + 1) * kTile, len - 1);
    const int k0 = t * kTile;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = k0 + sub * 32;
      if (kb > qw0 + 31) continue;  // wholly above the diagonal for every query of this wave
      const f32x16 s = score_tile(lds[t & 1], sub, own);
      const bool diag = kb + 31 > qw0;  // some (key, query) pairs of the tile violate key <= query
      float tv[16];
      float mb = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kb + 8 * (r >> 2) + 4 * half + (r & 3);
        float x = s[r] * sc;
        if (w > 0 && qi - key < w) x += rb;
        if (diag && key > qi) x = -INFINITY;
        tv[r] = x;
        mb = fmaxf(mb, x);
      }
      const float m_new = fmaxf(m, mb);
      if (m_new > -INFINITY) {
        float sum = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += fast_exp2(tv[r] - m_new);
        l = l * fast_exp2(m - m_new) + sum;
        m = m_new;
      }
    }
  }
  // the two lane halves hold different keys of the same query
  const float m_o = __shfl_xor(m, 32, kWave), l_o = __shfl_xor(l, 32, kWave);
  const float m_new = fmaxf(m, m_o);
  const float tot = (m > -INFINITY ? l * fast_exp2(m - m_new) : 0.0f) + (m_o > -INFINITY ? l_o * fast_exp2(m_o - m_new) : 0.0f);
  if (half == 0 && qi < len) a.lse[ubase + qi] = m_new + log2f(tot);
}

// ------------------------------------------------------------------------------------------------
// pass 2: Acc[j] = sum_{i>=j} 2^(t_ij - lse_i),  Acc2[j] = sum_{i>=j} (same)^2
__global__ __launch_bounds__(kThreads) void prefill_columns_mfma(PrefillArgs a) {
  __shared__ __attribute__((aligned(16))) char lds[2][kTile * kLdsRow];
  __shared__ __attribute__((aligned(16))) float lse_s[2][kTile];
  const int u = blockIdx.y;
  const int len = a.len[u];
  const int j0 = blockIdx.x * kOwn;  // low key blocks have the longest columns and come first
  if (j0 >= len) return;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Qb = static_cast<const char*>(a.Q) + ubase * kRowBytes;
  const char* Kb = static_cast<const char*>(a.K) + ubase * kRowBytes;
  const float* lse = a.lse + ubase;
  const int kw0 = j0 + 32 * wave;
  const int kj = kw0 + (lane & 31);  // this lane's key
  const int half = lane >> 5;
  uint4 own[kKSteps];
  load_owned(own, Kb, kj, len - 1);

  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  float s1 = 0.0f, s2 = 0.0f;

  const int t_first = j0 / kTile;            // first query tile with a query >= j0
  const int t_last = (len - 1) / kTile;
  Staged st;
  tile_load(st, Qb, t_first * kTile, len - 1);
  float lse_st = 0.0f;
  if (threadIdx.x < kTile) lse_st = lse[min(t_first * kTile + static_cast<int>(threadIdx.x), len - 1)];
  for (int t = t_first; t <= t_last; ++t) {
    const int b = (t - t_first) & 1;
    tile_store(st, lds[b]);
    if (threadIdx.x < kTile) lse_s[b][threadIdx.x] = lse_st;
    __syncthreads();
    if (t < t_last) {
      tile_load(st, Qb, (t + 1) * kTile, len - 1);
      if (threadIdx.x < kTile) lse_st = lse[min((t + 1) * kTile + static_cast<int>(threadIdx.x), len - 1)];
    }
    const int i0 = t * kTile;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int ib = i0 + sub * 32;
      if (ib + 31 < kw0) continue;  // every query of the tile precedes every key of this wave
      const f32x16 s = score_tile(lds[b], sub, own);
      const bool edge = ib < kw0 + 31 || ib + 31 >= len;  // diagonal tile, or the ragged end of the prompt
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const float4 ls = *reinterpret_cast<const float4*>(&lse_s[b][sub * 32 + 8 * g4 + 4 * half]);
        const float lv[4] = {ls.x, ls.y, ls.z, ls.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int qi = ib + 8 * g4 + 4 * half + e;
          float x = fmaf(s[4 * g4 + e], sc, -lv[e]);
          if (w > 0 && qi - kj < w) x += rb;
          float p = fast_exp2(x);
          if (edge && (qi < kj || qi >= len)) p = 0.0f;
          s1 += p;
          s2 = fmaf(p, p, s2);
        }
      }
    }
  }
  s1 += __shfl_xor(s1, 32, kWave);
  s2 += __shfl_xor(s2, 32, kWave);
  if (half == 0 && kj < len) {
    a.acc[ubase + kj] = s1;
    a.acc2[ubase + kj] = s2;
  }
}

}  // namespace

hipError_t launch_prefill_attention_mfma(const PrefillArgs& a, hipStream_t s) {
  if (a.O != nullptr) return launch_prefill_attention_simple(kBF16, D, a, s);  // attention output: general path
  const dim3 grid((a.L_max + kOwn - 1) / kOwn, a.units);
  {
    ProfScope ps(kProfPrefillRows, s);
    hipLaunchKernelGGL(prefill_rows_mfma, grid, dim3(kThreads), 0, s, a);
  }
  {
    ProfScope ps(kProfPrefillColumns, s);
    hipLaunchKernelGGL(prefill_columns_mfma, grid, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace roco
