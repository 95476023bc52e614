// Device helpers shared by the RoCo kernels (gfx950, 64-wide wavefronts).
#pragma once
#include "kernels.hpp"
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace roco {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

enum : int { kF32 = 0, kBF16 = 1 };

// ---------------------------------------------------------------- element types
template <int DT> struct Elem;
template <> struct Elem<kF32> {
  using type = float;
  static constexpr int per16 = 4;  // elements in one 16-byte lane load
};
template <> struct Elem<kBF16> {
  using type = uint16_t;
  static constexpr int per16 = 8;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}
// round to nearest even; inputs are finite attention outputs
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

template <int DT> __device__ __forceinline__ void unpack16(const uint4& w, float* f);
template <> __device__ __forceinline__ void unpack16<kF32>(const uint4& w, float* f) {
  f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
  f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
}
template <> __device__ __forceinline__ void unpack16<kBF16>(const uint4& w, float* f) {
  f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
  f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
  f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
  f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
}

template <int DT> __device__ __forceinline__ void store_elem(void* base, size_t idx, float v);
template <> __device__ __forceinline__ void store_elem<kF32>(void* base, size_t idx, float v) {
  static_cast<float*>(base)[idx] = v;
}
template <> __device__ __forceinline__ void store_elem<kBF16>(void* base, size_t idx, float v) {
  static_cast<uint16_t*>(base)[idx] = f32_to_bf16(v);
}

__device__ __forceinline__ uint4 load16(const void* p) { return *static_cast<const uint4*>(p); }
// Streaming variant: data that is touched once per kernel and should not displace what the caches hold.
typedef uint32_t uint4_vec __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_streaming(const void* p) {
  const uint4_vec v = __builtin_nontemporal_load(static_cast<const uint4_vec*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// ---------------------------------------------------------------- cross-lane
// Lane exchange inside a 16-lane row through the data-parallel-primitive path of the vector ALU (no LDS
// traffic).  CTRL: 0xB1 = swap neighbours, 0x4E = swap pairs, 0x141 = mirror each 8 lanes, 0x140 = mirror
// each 16 lanes.  After the two swaps every lane of a quad holds the quad's value, so the two mirrors act
// as the xor-4 and xor-8 steps of a butterfly.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// All-reduce (sum) over aligned groups of LANES lanes (LANES a power of two <= 64).
template <int LANES> __device__ __forceinline__ float group_sum(float v) {
  if (LANES >= 2) v += dpp_move<0xB1>(v);
  if (LANES >= 4) v += dpp_move<0x4E>(v);
  if (LANES >= 8) v += dpp_move<0x141>(v);
  if (LANES >= 16) v += dpp_move<0x140>(v);
#pragma unroll
  for (int m = 16; m < LANES; m <<= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
template <int LANES> __device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int m = 1; m < LANES; m <<= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wave on the vector ALU's lane-shift path: four shifted adds inside
// each row of 16 lanes, then the last lane of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  auto shr = [](uint32_t x, auto ctrl, auto row_mask) {
    return static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(x), decltype(ctrl)::value, decltype(row_mask)::value, 0xF, false));
  };
  using std::integral_constant;
  v += shr(v, integral_constant<int, 0x111>{}, integral_constant<int, 0xF>{});  // row_shr:1
  v += shr(v, integral_constant<int, 0x112>{}, integral_constant<int, 0xF>{});  // row_shr:2
  v += shr(v, integral_constant<int, 0x114>{}, integral_constant<int, 0xF>{});  // row_shr:4
  v += shr(v, integral_constant<int, 0x118>{}, integral_constant<int, 0xF>{});  // row_shr:8
  v += shr(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});  // row_bcast:15 into rows 1, 3
  v += shr(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});  // row_bcast:31 into rows 2, 3
  return v;
}

// Exclusive prefix sum of one value per thread over the whole block, in thread order.
// `sh` needs NT/64 + 1 words; returns the block total through `total`.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* sh, uint32_t& total) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  uint32_t incl = wave_inclusive_scan(v);
  __syncthreads();  // protects `sh` against readers of a previous call
  if (lane == kWave - 1) sh[wave] = incl;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NT / kWave; ++w) {
    uint32_t s = sh[w];
    if (w < wave) off += s;
    tot += s;
  }
  total = tot;
  return off + incl - v;
}

// ---------------------------------------------------------------- k-smallest selection
// Non-negative IEEE floats order like their bit patterns read as uint32, so selection runs on
// integers and is exact.  radix_select finds the k-th smallest key (k is 1-based, 1 <= k <= n) among
// key_of(0..n-1), 8-bit digits from the top; it also returns how many keys are strictly smaller and how
// many are equal.  Two histograms alternate (the idle one is cleared while the other is scanned), which
// leaves three barriers per digit; and as soon as the chosen bin holds no more keys than a wave has lanes the
// remaining digits are not counted: one wave ranks those keys directly.  `sh` needs kSelectLdsWords words of
// LDS.  All threads of the block call it.
constexpr int kSelectLdsWords = 2 * 256 + 12;

template <int NT, class KeyFn>
__device__ void radix_select(KeyFn key_of, int n, uint32_t k, uint32_t* sh,
                             uint32_t& kth, uint32_t& n_less, uint32_t& n_equal) {
  static_assert(NT >= 256 && NT % kWave == 0, "one thread per histogram bin");
  uint32_t* wtot = sh + 512;  // inclusive totals of the four scanning waves
  uint32_t* res = sh + 516;   // bin, keys below the bin, keys in the bin, the key itself and a counter (early exit)
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  __syncthreads();  // `sh` may still be in use by a previous call
  if (tid < 256) sh[tid] = 0;
  __syncthreads();
  uint32_t prefix = 0, mask = 0, kk = k, less = 0, neq = 0;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    uint32_t* hist = sh + ((pass & 1) ? 256 : 0);
    uint32_t* idle = sh + ((pass & 1) ? 0 : 256);
    for (int i = tid; i < n; i += NT) {
      const uint32_t key = key_of(i);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    uint32_t h = 0;
    if (tid < 256) {
      h = hist[tid];
      idle[tid] = 0;  // ready for the next digit
    }
    uint32_t incl = wave_inclusive_scan(h);
    if (tid < 256 && lane == kWave - 1) wtot[wave] = incl;
    __syncthreads();
    if (tid < 256) {
      for (int w = 0; w < wave; ++w) incl += wtot[w];
      const uint32_t excl = incl - h;
      if (excl < kk && kk <= incl) { res[0] = tid; res[1] = excl; res[2] = h; res[4] = 0; }
    }
    __syncthreads();
    prefix |= res[0] << shift;
    mask |= 255u << shift;
    less += res[1];
    kk -= res[1];
    neq = res[2];
    if (neq <= kWave && pass < 3) {
      // At most a wave's worth of candidates is left: they are gathered (into the idle histogram, which is clear)
      // and ranked by one wave directly, every lane counting the candidates below and equal to its own.
      uint32_t* cand = idle;
      for (int i = tid; i < n; i += NT) {
        const uint32_t key = key_of(i);
        if ((key & mask) == prefix) cand[atomicAdd(&res[4], 1u)] = key;
      }
      __syncthreads();
      if (tid < kWave) {
        const uint32_t mine = tid < neq ? cand[tid] : 0xffffffffu;
        uint32_t lt = 0, eq = 0;
        for (uint32_t m = 0; m < neq; ++m) {
          const uint32_t other = cand[m];
          lt += other < mine ? 1u : 0u;
          eq += other == mine ? 1u : 0u;
        }
        if (tid < neq && lt < kk && kk <= lt + eq) { res[1] = lt; res[2] = eq; res[3] = mine; }  // equal lanes agree
      }
      __syncthreads();
      prefix = res[3];
      less += res[1];
      neq = res[2];
      break;
    }
  }
  kth = prefix;
  n_less = less;
  n_equal = neq;
}

// The k smallest keys, equal keys taken in index order: element i is selected iff
//   key < kth  ||  (key == kth && i <= index_limit).
struct KSmallest {
  uint32_t kth;
  uint32_t index_limit;
  __device__ __forceinline__ bool has(uint32_t key, uint32_t i) const {
    return key < kth || (key == kth && i <= index_limit);
  }
};

template <int NT, class KeyFn>
__device__ KSmallest select_k_smallest(KeyFn key_of, int n, uint32_t k, uint32_t* sh) {
  // everything is wanted (the policies whose scope is the whole cache, say): nothing to select
  if (k >= static_cast<uint32_t>(n)) return KSmallest{0xffffffffu, 0xffffffffu};
  KSmallest r;
  uint32_t n_less, n_equal;
  radix_select<NT>(key_of, n, k, sh, r.kth, n_less, n_equal);
  const uint32_t take = k - n_less;  // how many of the keys equal to kth belong to the selection
  if (take == n_equal) {
    r.index_limit = 0xffffffffu;
  } else {
    // ties straddle the boundary: the `take` lowest indices among the equal keys win
    const uint32_t kth = r.kth;
    uint32_t lim, a, b;
    radix_select<NT>([&](int i) { return key_of(i) == kth ? static_cast<uint32_t>(i) : 0xffffffffu; },
                     n, take, sh, lim, a, b);
    r.index_limit = lim;
  }
  return r;
}

// Scope = `scope` lowest variance keys among [0, B); returns the slot of lowest MAS key inside it (lowest
// slot on equal keys).  Every thread of the block calls it and gets the same answer.
template <int NT>
__device__ int select_victim_block(const uint32_t* var_key, const uint32_t* mas_key, int B, int scope,
                                   uint32_t* sel_sh, unsigned long long* best_sh) {
  const int tid = threadIdx.x;
  const KSmallest sc = select_k_smallest<NT>([&](int i) { return var_key[i]; }, B,
                                             static_cast<uint32_t>(scope), sel_sh);
  unsigned long long best = ~0ull;
  for (int i = tid; i < B; i += NT) {
    if (sc.has(var_key[i], i)) {
      const unsigned long long cand =
          (static_cast<unsigned long long>(mas_key[i]) << 32) | static_cast<uint32_t>(i);
      best = cand < best ? cand : best;
    }
  }
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) {
    const unsigned long long o = __shfl_xor(best, m, kWave);
    best = o < best ? o : best;
  }
  __syncthreads();
  if ((tid & (kWave - 1)) == 0) best_sh[tid / kWave] = best;
  __syncthreads();
  unsigned long long b = best_sh[0];
#pragma unroll
  for (int w = 1; w < NT / kWave; ++w) b = best_sh[w] < b ? best_sh[w] : b;
  return static_cast<int>(b & 0xffffffffu);
}

// Ranking keys of one cached token: the token of lowest importance key among the tokens of lowest scope key
// is evicted; keys are compared as unsigned integers (non-negative floats order like their bit patterns).
// For RoCo these are the mean attention score and the attention variance, each operation rounded on its own
// (no fused multiply-add), so that a single observation gives a variance of exactly zero:
//   MAS = Acc/Count,  Var = max(0, Acc2/Count - MAS^2)          (section 4.3 of the paper)
// A protected sink position gets the largest importance key below the marker 0xffffffff that the selections
// use for "outside the scope".
__device__ __forceinline__ void ranking_keys(float acc, float acc2, float count, int pos, const Policy& pol,
                                             uint32_t& mas_key, uint32_t& var_key) {
  if (pol.importance == kImpMas) {
    mas_key = __float_as_uint(__fdiv_rn(acc, count));
  } else if (pol.importance == kImpAas) {
    mas_key = acc > 0.0f ? __float_as_uint(acc) : 0u;
  } else if (pol.importance == kImpLast || pol.importance == kImpCount) {
    mas_key = acc2 > 0.0f ? __float_as_uint(acc2) : 0u;
  } else {
    mas_key = pos < pol.sinks ? 0xfffffffeu : static_cast<uint32_t>(pos);
  }
  if (pol.scope_kind == kScopeStd) {
    const float mas = __fdiv_rn(acc, count);
    const float ex2 = __fdiv_rn(acc2, count);
    const float var = __fsub_rn(ex2, __fmul_rn(mas, mas));
    var_key = var > 0.0f ? __float_as_uint(var) : 0u;
  } else if (pol.scope_kind == kScopeWindow) {
    var_key = static_cast<uint32_t>(pos);
  } else {
    var_key = 0u;
  }
}

}  // namespace roco
