// Device helpers shared by the RoCo kernels (gfx950, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    uint32_t o = __shfl_up(v, d, kWave);
    if (lane >= d) v += o;
  }
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
// key_of(0..n-1), four 8-bit digits from the top; it also returns how many keys are strictly smaller
// and how many are equal.  `sh` needs 256 + NT/64 + 3 words of LDS.  All threads of the block call it.
template <int NT, class KeyFn>
__device__ void radix_select(KeyFn key_of, int n, uint32_t k, uint32_t* sh,
                             uint32_t& kth, uint32_t& n_less, uint32_t& n_equal) {
  static_assert(NT >= 256 && NT % kWave == 0, "one thread per histogram bin");
  uint32_t* hist = sh;
  uint32_t* wtot = sh + 256;
  uint32_t* res = wtot + NT / kWave;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  uint32_t prefix = 0, mask = 0, kk = k, less = 0, neq = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    __syncthreads();
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) {
      const uint32_t key = key_of(i);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    const uint32_t h = (tid < 256) ? hist[tid] : 0u;
    uint32_t incl = wave_inclusive_scan(h);
    if (tid < 256 && lane == kWave - 1) wtot[wave] = incl;
    __syncthreads();
    if (tid < 256) {
      for (int w = 0; w < wave; ++w) incl += wtot[w];
      const uint32_t excl = incl - h;
      if (excl < kk && kk <= incl) { res[0] = tid; res[1] = excl; res[2] = h; }
    }
    __syncthreads();
    prefix |= res[0] << shift;
    mask |= 255u << shift;
    less += res[1];
    kk -= res[1];
    neq = res[2];
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

// Mean attention score and attention variance as ranking keys, each operation rounded on its own
// (no fused multiply-add), so that a single observation gives a variance of exactly zero:
//   MAS = Acc/Count,  Var = max(0, Acc2/Count - MAS^2)          (section 4.3 of the paper)
__device__ __forceinline__ void ranking_keys(float acc, float acc2, float count,
                                             uint32_t& mas_key, uint32_t& var_key) {
  const float mas = __fdiv_rn(acc, count);
  const float ex2 = __fdiv_rn(acc2, count);
  const float var = __fsub_rn(ex2, __fmul_rn(mas, mas));
  mas_key = __float_as_uint(mas);
  var_key = var > 0.0f ? __float_as_uint(var) : 0u;
}

}  // namespace roco
