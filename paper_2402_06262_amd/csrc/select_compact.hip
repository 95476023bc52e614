// Prefill eviction step and cache compaction (one eviction step that frees E = len - B tokens; section 5.3
// "Overhead", block-wise evict-and-encode with the prompt as one block).
//
// Rule (section 4.3 applied E times with the statistics frozen, in closed form): among the s + E - 1
// tokens of lowest attention variance, evict the E tokens of lowest mean attention score; equal keys go to
// the lowest position.  The retained tokens keep ascending position order in the compacted cache.
//
//   prefill_select  : one workgroup per unit.  Two exact k-smallest selections on the fp32 bit patterns
//                     (radix select, no sorting), then an ordered prefix sum assigns cache slots and writes
//                     pos[], the three statistics planes and n_used.
//   prefill_gather  : grid (row blocks, units): copies the retained K / V rows into the cache, 16 bytes per
//                     lane.
#include "kernels.hpp"
#include "profile.hpp"
#include "stream.hpp"

namespace roco {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kGatherThreads = 256;
constexpr int kGatherRows = 64;  // cache rows per gather workgroup

__global__ __launch_bounds__(kSelThreads) void prefill_select(PrefillArgs a) {
  constexpr int NT = kSelThreads;
  extern __shared__ uint32_t lds_keys[];  // [2][L_max] ranking keys when L_max <= kMaxDecodeBudgetLds
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  __shared__ uint32_t scan_sh[NT / kWave + 1];
  __shared__ unsigned long long best_sh[NT / kWave];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B;
  const int n = a.len[u];
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const float* acc = a.acc + ubase;
  const float* acc2 = a.acc2 + ubase;
  // every radix pass reads every key: in LDS they cost a fraction of a trip to the L2 each
  const bool keys_in_lds = a.L_max <= kMaxDecodeBudgetLds;
  uint32_t* var_key = keys_in_lds ? lds_keys : a.var_key + ubase;
  uint32_t* mas_key = keys_in_lds ? lds_keys + a.L_max : a.mas_key + ubase;
  float* oacc = a.stats + static_cast<size_t>(u) * 3 * B;
  float* oacc2 = oacc + B;
  float* ocnt = oacc2 + B;
  int32_t* pos = a.pos + static_cast<size_t>(u) * B;

  const int kept = n < B ? n : B;
  if (n <= B) {
    for (int i = tid; i < n; i += NT) {
      pos[i] = i;
      oacc[i] = acc[i];
      oacc2[i] = acc2[i];
      ocnt[i] = static_cast<float>(n - i);
    }
  } else {
    const uint32_t E = static_cast<uint32_t>(n - B);
    const uint32_t m = min(static_cast<uint32_t>(n), static_cast<uint32_t>(a.pol.scope_size(a.scope, n)) + E - 1u);
    for (int i = tid; i < n; i += NT) {
      uint32_t mk, vk;
      ranking_keys(acc[i], acc2[i], static_cast<float>(n - i), i, a.pol, mk, vk);
      var_key[i] = vk;
      mas_key[i] = mk;
    }
    __syncthreads();
    const KSmallest scope = select_k_smallest<NT>([&](int i) { return var_key[i]; }, n, m, sel_sh);
    auto key2 = [&](int i) -> uint32_t { return scope.has(var_key[i], i) ? mas_key[i] : 0xffffffffu; };
    const KSmallest out = select_k_smallest<NT>(key2, n, E, sel_sh);
    // ordered compaction: thread t owns the contiguous positions [t*c, (t+1)*c)
    const int c = (n + NT - 1) / NT;
    const int lo = min(n, tid * c), hi = min(n, lo + c);
    uint32_t mine = 0;
    for (int i = lo; i < hi; ++i) mine += out.has(key2(i), i) ? 0u : 1u;
    uint32_t total;
    uint32_t dst = block_exclusive_scan<NT>(mine, scan_sh, total);
    for (int i = lo; i < hi; ++i) {
      if (!out.has(key2(i), i) && dst < static_cast<uint32_t>(B)) {
        pos[dst] = i;
        oacc[dst] = acc[i];
        oacc2[dst] = acc2[i];
        ocnt[dst] = static_cast<float>(n - i);
        ++dst;
      }
    }
  }
  for (int i = kept + tid; i < B; i += NT) {
    pos[i] = -1;
    oacc[i] = 0.0f;
    oacc2[i] = 0.0f;
    ocnt[i] = 0.0f;
  }
  if (tid == 0) a.n_used[u] = kept;
  // the first decode step on a full cache needs its victim: choose it now, from the compacted statistics
  if (kept == B) {
    __syncthreads();  // the compacted planes written above are visible to the whole block
    for (int i = tid; i < B; i += NT) ranking_keys(oacc[i], oacc2[i], ocnt[i], pos[i], a.pol, mas_key[i], var_key[i]);
    __syncthreads();
    const KSmallest sc = select_k_smallest<NT>([&](int i) { return var_key[i]; }, B,
                                               static_cast<uint32_t>(a.pol.scope_size(a.scope, B)), sel_sh);
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
    if (tid == 0) {
      unsigned long long b = best_sh[0];
      for (int w = 1; w < NT / kWave; ++w) b = best_sh[w] < b ? best_sh[w] : b;
      a.next_slot[u] = static_cast<int>(b & 0xffffffffu);
    }
  } else if (tid == 0) {
    a.next_slot[u] = -1;
  }
}

template <int ROW_BYTES>
__global__ __launch_bounds__(kGatherThreads) void prefill_gather(PrefillArgs a) {
  constexpr int LPR = ROW_BYTES / 16;
  constexpr int RPP = kGatherThreads / LPR;  // rows per pass
  const int u = blockIdx.y, tid = threadIdx.x;
  const int B = a.B;
  const int n = a.len[u];
  const int kept = n < B ? n : B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  const char* Kin = static_cast<const char*>(a.K) + static_cast<size_t>(u) * a.L_max * ROW_BYTES;
  const char* Vin = static_cast<const char*>(a.V) + static_cast<size_t>(u) * a.L_max * ROW_BYTES;
  char* Kout = static_cast<char*>(a.K_cache) + static_cast<size_t>(u) * B * ROW_BYTES;
  char* Vout = static_cast<char*>(a.V_cache) + static_cast<size_t>(u) * B * ROW_BYTES;
  const int r = tid / LPR, c = tid % LPR;
  const int first = blockIdx.x * kGatherRows;
  const int last = min(kept, first + kGatherRows);
  for (int slot = first + r; slot < last; slot += RPP) {
    const int p = pos[slot];
    if (p < 0 || p >= n) continue;  // never read outside the prompt, whatever pos[] holds
    const size_t src = static_cast<size_t>(p) * ROW_BYTES + c * 16;
    const size_t dst = static_cast<size_t>(slot) * ROW_BYTES + c * 16;
    *reinterpret_cast<uint4*>(Kout + dst) = load16_streaming(Kin + src);  // prompt rows are not needed again
    *reinterpret_cast<uint4*>(Vout + dst) = load16_streaming(Vin + src);
  }
}

// Which cached tokens survive one eviction step that shrinks a unit to `keep` tokens: the closed form of the
// rule above on the statistics as they stand, nothing modified.  mask[u][j] = 1 for survivors, 0 for victims and
// for empty slots.
__global__ __launch_bounds__(kSelThreads) void select_retained(DecodeArgs a, int keep, int32_t* mask_out) {
  constexpr int NT = kSelThreads;
  extern __shared__ uint32_t lds_keys[];  // [2][B] when B <= kMaxDecodeBudgetLds
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B;
  const int n = min(a.n_used[u], B);
  const float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  const float* acc2 = acc + B;
  const float* cnt = acc2 + B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  int32_t* mask = mask_out + static_cast<size_t>(u) * B;
  uint32_t* var_key = (B <= kMaxDecodeBudgetLds) ? lds_keys : a.keys + static_cast<size_t>(u) * 2 * B;
  uint32_t* mas_key = var_key + B;
  if (n <= keep) {
    for (int i = tid; i < B; i += NT) mask[i] = i < n ? 1 : 0;
    return;
  }
  const uint32_t E = static_cast<uint32_t>(n - keep);
  const uint32_t m = min(static_cast<uint32_t>(n), static_cast<uint32_t>(a.pol.scope_size(a.scope, n)) + E - 1u);
  const bool by_pos = a.pol.needs_pos();
  for (int i = tid; i < n; i += NT)
    ranking_keys(acc[i], acc2[i], cnt[i], by_pos ? pos[i] : 0, a.pol, mas_key[i], var_key[i]);
  __syncthreads();
  const KSmallest scope = select_k_smallest<NT>([&](int i) { return var_key[i]; }, n, m, sel_sh);
  auto key2 = [&](int i) -> uint32_t { return scope.has(var_key[i], i) ? mas_key[i] : 0xffffffffu; };
  const KSmallest out = select_k_smallest<NT>(key2, n, E, sel_sh);
  for (int i = tid; i < B; i += NT) mask[i] = (i < n && !out.has(key2(i), i)) ? 1 : 0;
}

// Overlap of two sets of cached tokens per unit (what section 4.1's consistency study compares): set X holds the
// positions pos_x[j] of the slots j < n_x with mask_x[j] != 0 (no mask: every such slot).  Positions inside a cache
// are distinct, so |A and B| is the number of B's members whose bit A has set in an LDS bitmap over [0, max_pos).
__global__ __launch_bounds__(256) void set_overlap(int slots_a, const int32_t* pos_a, const int32_t* mask_a,
                                                   const int32_t* n_a, int slots_b, const int32_t* pos_b,
                                                   const int32_t* mask_b, const int32_t* n_b, int max_pos,
                                                   int32_t* inter_out, int32_t* union_out) {
  extern __shared__ uint32_t bits[];  // (max_pos + 31) / 32 words, then the three counters
  const int u = blockIdx.x, tid = threadIdx.x;
  const int words = (max_pos + 31) / 32;
  uint32_t* const cnt = bits + words;  // |A|, |B|, |A and B|
  for (int i = tid; i < words; i += 256) bits[i] = 0u;
  if (tid < 3) cnt[tid] = 0u;
  __syncthreads();
  const int na = min(n_a[u], slots_a), nb = min(n_b[u], slots_b);
  uint32_t mine_a = 0, mine_b = 0, mine_i = 0;
  for (int j = tid; j < na; j += 256) {
    const int p = pos_a[static_cast<size_t>(u) * slots_a + j];
    if ((mask_a == nullptr || mask_a[static_cast<size_t>(u) * slots_a + j] != 0) && p >= 0 && p < max_pos) {
      atomicOr(&bits[p >> 5], 1u << (p & 31));
      ++mine_a;
    }
  }
  __syncthreads();
  for (int j = tid; j < nb; j += 256) {
    const int p = pos_b[static_cast<size_t>(u) * slots_b + j];
    if ((mask_b == nullptr || mask_b[static_cast<size_t>(u) * slots_b + j] != 0) && p >= 0 && p < max_pos) {
      ++mine_b;
      mine_i += (bits[p >> 5] >> (p & 31)) & 1u;
    }
  }
  atomicAdd(&cnt[0], mine_a);
  atomicAdd(&cnt[1], mine_b);
  atomicAdd(&cnt[2], mine_i);
  __syncthreads();
  if (tid == 0) {
    inter_out[u] = static_cast<int32_t>(cnt[2]);
    union_out[u] = static_cast<int32_t>(cnt[0] + cnt[1] - cnt[2]);
  }
}

}  // namespace

hipError_t launch_set_overlap(int units, int slots_a, const int32_t* pos_a, const int32_t* mask_a, const int32_t* n_a,
                              int slots_b, const int32_t* pos_b, const int32_t* mask_b, const int32_t* n_b, int max_pos,
                              int32_t* inter, int32_t* uni, hipStream_t s) {
  // the bitmap (the host keeps it within 64 KiB) and three counters: the largest range needs the raised limit
  const size_t lds = (static_cast<size_t>((max_pos + 31) / 32) + 3) * sizeof(uint32_t);
  if (!allow_key_lds(reinterpret_cast<const void*>(set_overlap), lds)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(set_overlap, dim3(units), dim3(256), lds, s, slots_a, pos_a, mask_a, n_a, slots_b, pos_b, mask_b, n_b,
                     max_pos, inter, uni);
  return hipGetLastError();
}

hipError_t launch_select_retained(const DecodeArgs& a, int keep, int32_t* mask, hipStream_t s) {
  const size_t lds = key_lds_bytes(a.B);
  if (!allow_key_lds(reinterpret_cast<const void*>(select_retained), lds)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(select_retained, dim3(a.units), dim3(kSelThreads), lds, s, a, keep, mask);
  return hipGetLastError();
}

hipError_t launch_prefill_select_compact(int dtype, int head_dim, const PrefillArgs& a, hipStream_t s) {
  {
    ProfScope ps(kProfPrefillSelect, s);
    const size_t key_lds = key_lds_bytes(a.L_max);  // the budget's keys for the first decode victim fit too: B < L_max
    if (!allow_key_lds(reinterpret_cast<const void*>(prefill_select), key_lds)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(prefill_select, dim3(a.units), dim3(kSelThreads), key_lds, s, a);
  }
  ProfScope ps(kProfPrefillGather, s);
  const int row_bytes = head_dim * (dtype == kBF16 ? 2 : 4);
  const dim3 grid((a.B + kGatherRows - 1) / kGatherRows, a.units);
  switch (row_bytes) {
    case 128: hipLaunchKernelGGL((prefill_gather<128>), grid, dim3(kGatherThreads), 0, s, a); break;
    case 256: hipLaunchKernelGGL((prefill_gather<256>), grid, dim3(kGatherThreads), 0, s, a); break;
    case 512: hipLaunchKernelGGL((prefill_gather<512>), grid, dim3(kGatherThreads), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace roco
