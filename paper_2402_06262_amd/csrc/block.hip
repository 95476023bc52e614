// Block-wise evict-and-encode on gfx950 (section 5.3 "Overhead" and appendix B of the paper: the number of
// tokens freed and encoded within one eviction step is a block size b; b = 1 is the token-wise scheme).
//
// With n tokens cached, E = max(0, n + b - B) tokens are evicted in one step (E single evictions by the rule of
// section 4.3 with frozen statistics = the E lowest mean attention scores among the s + E - 1 lowest variances),
// the block's tokens go in order to the ascending list of freed and still-empty slots, query i of the block
// attends every retained token and the block's tokens 0..i, and every attended token gets p, p^2 and 1 added to
// its statistics.  The point of the scheme is that K and V are streamed once per block instead of once per token:
// the step stays HBM-bound, so encoding b tokens costs about what encoding one does.
//
//   block_prepare : one workgroup per unit.  Victims (two exact radix selects), ordered slot assignment,
//                   K / V rows of the block written into their slots, pos / statistics of those slots reset.
//   block_attend  : grid (splits, units), two waves.  64-slot K and V tiles through LDS, each wave scores 32
//                   slots against the block's queries on the matrix cores (score tile = K . Q^T, the query in
//                   the lane; one or two tiles of 32 query rows, every K and V^T fragment read from LDS feeding
//                   both), stores the base-2 logits, keeps an online softmax per query and accumulates
//                   O^T = V^T . P^T with V^T fragments from the LDS transpose read.
//   block_attend_shared : the same for fp32 and head_dim 64, on the vector ALUs (see there).
//   block_finish  : one workgroup per unit.  Merges the partials per query, writes the outputs, adds the
//                   statistics of all rows to every slot and chooses the victim a following single-token step
//                   would take.
//
// The same three kernels serve grouped-query attention (section 5.3, "Extension to Grouped-Query Attention"):
// g query heads share the unit's keys and values, the query rows are (token, head) pairs, and the statistics
// receive, once per token, the mean of its g heads' probabilities (BlockArgs::heads).
#include <cstdlib>

#include "kernels.hpp"
#include "mfma.hpp"
#include "profile.hpp"
#include "stream.hpp"

namespace roco {
namespace {

using namespace mfma;

constexpr int kPrepThreads = 1024;  // 512 when the units outnumber the compute units (see launch_block)
constexpr int kAttThreads = 128;  // two waves: one 32-slot half of a 64-slot tile each
constexpr int kFinThreads = 1024;
constexpr int kQ = 32;            // query rows per matrix tile
static_assert(kMaxBlock == 2 * kQ, "a step holds at most two tiles of query rows");

// ------------------------------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(NT) void block_prepare(BlockArgs a) {
  extern __shared__ uint32_t lds_keys[];  // [2][B] when B <= kMaxDecodeBudgetLds
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  __shared__ uint32_t scan_sh[NT / kWave + 1];
  __shared__ int slot_of[kMaxBlock];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B, b = a.block;
  const int n = a.n_used[u];
  const int E = max(0, n + b - B);
  const int n_new = min(B, n + b);
  float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  float* acc2 = acc + B;
  float* cnt = acc2 + B;
  int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  int32_t* bidx = a.blk_idx + static_cast<size_t>(u) * B;
  uint32_t* var_key = (B <= kMaxDecodeBudgetLds) ? lds_keys : a.keys + static_cast<size_t>(u) * 2 * B;
  uint32_t* mas_key = var_key + B;

  if (tid < kMaxBlock) slot_of[tid] = 0;
  KSmallest scope = {0u, 0u}, out = {0u, 0u};
  // one eviction from a full cache: the victim was already chosen when the statistics were last updated
  const int hint = (E == 1 && n == B) ? a.next_slot[u] : -1;
  if (E > 0 && hint < 0) {
    for (int i = tid; i < n; i += NT) ranking_keys(acc[i], acc2[i], cnt[i], pos[i], a.pol, mas_key[i], var_key[i]);
    __syncthreads();
    const uint32_t m = min(static_cast<uint32_t>(n), static_cast<uint32_t>(a.pol.scope_size(a.scope, n)) + static_cast<uint32_t>(E) - 1u);
    scope = select_k_smallest<NT>([&](int i) { return var_key[i]; }, n, m, sel_sh);
    out = select_k_smallest<NT>(
        [&](int i) -> uint32_t { return scope.has(var_key[i], i) ? mas_key[i] : 0xffffffffu; }, n,
        static_cast<uint32_t>(E), sel_sh);
  }
  auto is_target = [&](int j) -> bool {
    if (j >= n) return j < n_new;  // still-empty slot taken by the block
    if (E == 0) return false;
    if (hint >= 0) return j == hint;
    const uint32_t k2 = scope.has(var_key[j], j) ? mas_key[j] : 0xffffffffu;
    return out.has(k2, j);
  };
  // ordered assignment: thread t owns the contiguous slots [t*c, (t+1)*c); the i-th target gets block token i
  const int c = (B + NT - 1) / NT;
  const int lo = min(B, tid * c), hi = min(B, lo + c);
  uint32_t mine = 0;
  for (int j = lo; j < hi; ++j) mine += (j < n_new && is_target(j)) ? 1u : 0u;
  uint32_t total;
  uint32_t rank = block_exclusive_scan<NT>(mine, scan_sh, total);
  const int qp0 = a.qpos0[u];
  for (int j = lo; j < hi; ++j) {
    int bi = -1;
    if (j < n_new && is_target(j) && rank < static_cast<uint32_t>(b)) {
      bi = static_cast<int>(rank++);
      slot_of[bi] = j;
      const bool held = j < n;  // the slot held a token that is now evicted
      if (a.evicted_slot) a.evicted_slot[static_cast<size_t>(u) * b + bi] = held ? j : -1;
      if (a.evicted_pos) a.evicted_pos[static_cast<size_t>(u) * b + bi] = held ? pos[j] : -1;
      pos[j] = qp0 + bi;
      acc[j] = 0.0f;
      acc2[j] = 0.0f;
      cnt[j] = 0.0f;
    }
    bidx[j] = bi;
  }
  __syncthreads();
  // the block's K / V rows go into their slots: 16 bytes per lane
  const int lpr = a.row_bytes / 16;  // lanes per row: 8, 16 or 32
  const size_t in_base = static_cast<size_t>(u) * b * a.row_bytes;
  for (int i = tid / lpr; i < b; i += NT / lpr) {
    const size_t dst = (static_cast<size_t>(u) * B + slot_of[i]) * a.row_bytes + (tid % lpr) * 16;
    const size_t src = in_base + static_cast<size_t>(i) * a.row_bytes + (tid % lpr) * 16;
    *reinterpret_cast<uint4*>(static_cast<char*>(a.K) + dst) = load16(static_cast<const char*>(a.k_new) + src);
    *reinterpret_cast<uint4*>(static_cast<char*>(a.V) + dst) = load16(static_cast<const char*>(a.v_new) + src);
  }
  if (tid == 0) a.n_used[u] = n_new;
}

// ------------------------------------------------------------------------------------------------
struct StagedKV {
  uint4 k[8], v[8];  // this thread's 128 bytes of a 64 x 256 B tile of K and of V (128 threads)
};
// `fresh` (or -1) is a slot whose row is taken from knew / vnew instead of the cache: the token a single-token step
// is about to write there.  The address is selected, not the load, so there is no control flow around the loads.
template <bool STREAMING>
__device__ __forceinline__ void kv_load(StagedKV& s, const char* Kb, const char* Vb, int row0, int last_row,
                                        int fresh, const char* knew, const char* vnew) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int row = row0 + (t >> 4) + 8 * i;
    row = row < last_row ? row : last_row;  // slots past the end are masked by the caller
    const size_t off = static_cast<size_t>(row) * kRowBytes + (t & 15) * 16;
    const char* kp = row == fresh ? knew + (t & 15) * 16 : Kb + off;
    const char* vp = row == fresh ? vnew + (t & 15) * 16 : Vb + off;
    s.k[i] = STREAMING ? load16_streaming(kp) : load16(kp);
    s.v[i] = STREAMING ? load16_streaming(vp) : load16(vp);
  }
}
__device__ __forceinline__ void kv_store(const StagedKV& s, char* tileK, char* tileV) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    *reinterpret_cast<uint4*>(tileK + ((t >> 4) + 8 * i) * kLdsRow + (t & 15) * 16) = s.k[i];
    *reinterpret_cast<uint4*>(tileV + ((t >> 4) + 8 * i) * kLdsRowV + (t & 15) * 16) = s.v[i];
  }
}

// NQT: tiles of 32 query rows (1 or 2).  The workspace planes are addressed with a.qrows = 32 NQT rows per unit.
template <int NQT>
__global__ __launch_bounds__(kAttThreads) void block_attend(BlockArgs a) {
  constexpr int QR = NQT * kQ;
  extern __shared__ __attribute__((aligned(16))) char lds_dyn[];  // K[2] and V[2] tiles; reused for the merge
  __shared__ __attribute__((aligned(16))) int32_t bidx_s[2][kTile];
  __shared__ __attribute__((aligned(16))) int32_t pos_s[2][kTile];
  __shared__ float merge_m[QR], merge_l[QR];
  const int u = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int half = lane >> 5, qi = lane & 31;  // this lane's query row inside a tile
  const int B = a.B, b = a.queries;
  // Usually block_prepare has run: n_used counts the block's tokens and their rows are in the cache.  A single-token
  // step skips it (BlockArgs::single): the token's slot is known from the state, its row is read from k_new / v_new
  // and written into the cache by the workgroup that streams that slot, as in the token-wise decode kernels.
  int n = a.n_used[u];
  int fresh = -1;
  if (a.single) {
    const bool was_full = n >= B;
    fresh = was_full ? min(max(a.next_slot[u], 0), B - 1) : n;
    n = was_full ? B : n + 1;
  }
  const char* knew = static_cast<const char*>(a.k_new) + static_cast<size_t>(u) * kRowBytes;
  const char* vnew = static_cast<const char*>(a.v_new) + static_cast<size_t>(u) * kRowBytes;
  const int row0 = split * a.rows_per_split;
  const int row1 = min(n, row0 + a.rows_per_split);
  const size_t pidx = static_cast<size_t>(u) * a.splits + split;
  char* Kb = static_cast<char*>(a.K) + static_cast<size_t>(u) * B * kRowBytes;
  char* Vb = static_cast<char*>(a.V) + static_cast<size_t>(u) * B * kRowBytes;
  const int32_t* bidx = a.blk_idx + static_cast<size_t>(u) * B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  float* z = a.z + static_cast<size_t>(u) * QR * B;
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  int ti[NQT], qp[NQT];  // this lane's block token per tile; the heads of a group share its position
#pragma unroll
  for (int t2 = 0; t2 < NQT; ++t2) {
    ti[t2] = (kQ * t2 + qi) / a.heads;
    qp[t2] = a.qpos0[u] + ti[t2];
  }

  // B operand: the block's queries (lanes beyond the block reuse its last query; their results are dropped)
  uint4 own[NQT][kKSteps];
#pragma unroll
  for (int t2 = 0; t2 < NQT; ++t2) {
    const char* qrow = static_cast<const char*>(a.q) + (static_cast<size_t>(u) * b + min(kQ * t2 + qi, b - 1)) * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < kKSteps; ++kk) own[t2][kk] = load16(qrow + kk * 32 + half * 16);
  }
  float m[NQT], l[NQT];
  f32x16 o[NQT][4];
#pragma unroll
  for (int t2 = 0; t2 < NQT; ++t2) {
    m[t2] = -INFINITY;
    l[t2] = 0.0f;
#pragma unroll
    for (int db = 0; db < 4; ++db) o[t2][db] = f32x16{0};
  }
  const int tr_off = transposed_fragment_offset();

  const int n_tiles = row1 > row0 ? (row1 - row0 + kTile - 1) / kTile : 0;
  StagedKV st;
  int32_t st_bidx = -1, st_pos = 0;
  // Tiles are visited from a start that differs between workgroups, so that workgroups running side by side do
  // not walk the memory channels in lock step (the online softmax does not care about the order).
  const int rot = n_tiles > 0 ? static_cast<int>((static_cast<unsigned>(u) * 5u + static_cast<unsigned>(split) * 3u) %
                                                 static_cast<unsigned>(n_tiles))
                              : 0;
  auto tile_row = [&](int t) { return row0 + (t + rot < n_tiles ? t + rot : t + rot - n_tiles) * kTile; };
  auto fetch = [&](int t) {
    const int tr0 = tile_row(t);
    if (a.streaming) kv_load<true>(st, Kb, Vb, tr0, n - 1, fresh, knew, vnew);
    else kv_load<false>(st, Kb, Vb, tr0, n - 1, fresh, knew, vnew);
    if (fresh >= tr0 && fresh < min(tr0 + kTile, row1)) {  // this tile holds the new token's slot: put the row there
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (tr0 + (tid >> 4) + 8 * i == fresh) {
          const size_t off = static_cast<size_t>(fresh) * kRowBytes + (tid & 15) * 16;
          *reinterpret_cast<uint4*>(Kb + off) = st.k[i];
          *reinterpret_cast<uint4*>(Vb + off) = st.v[i];
        }
      }
    }
    if (tid < kTile) {
      const int slot = min(tr0 + tid, n - 1);
      st_bidx = a.single ? -1 : bidx[slot];
      st_pos = slot == fresh ? a.qpos0[u] : pos[slot];
    }
  };
  if (n_tiles > 0) fetch(0);
  for (int t = 0; t < n_tiles; ++t) {
    char* const tileK = lds_dyn + (t & 1) * kTileBytes;
    char* const tileV = lds_dyn + 2 * kTileBytes + (t & 1) * kTileBytesV;
    kv_store(st, tileK, tileV);
    if (tid < kTile) { bidx_s[t & 1][tid] = st_bidx; pos_s[t & 1][tid] = st_pos; }
    __syncthreads();
    if (t + 1 < n_tiles) fetch(t + 1);
    const int tr0 = tile_row(t);
    const int sb = tr0 + 32 * wave;  // first slot of this wave's half-tile
    if (sb < row1) {                               // wave-uniform
    // ---- scores of 32 slots x 32 NQT queries: every K fragment feeds one accumulator chain per query tile
    f32x16 sacc[NQT];
    {
      const char* p = tileK + (32 * wave + (lane & 31)) * kLdsRow + half * 16;
      const f32x16 zero = {0};
#pragma unroll
      for (int kk = 0; kk < kKSteps; ++kk) {
        const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p + kk * 32));
#pragma unroll
        for (int t2 = 0; t2 < NQT; ++t2)
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, __builtin_bit_cast(bf16x8, own[t2][kk]),
                                                             kk == 0 ? zero : sacc[t2], 0, 0, 0);
      }
    }
    bf16x8 pfrag[NQT][2];
#pragma unroll
    for (int t2 = 0; t2 < NQT; ++t2) {
    // ---- base-2 logits: a slot is visible if it exists and does not hold a later token of the block
    const int q = kQ * t2 + qi;
    float tv[16];
    float mb = -INFINITY;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int base = 32 * wave + 8 * g4 + 4 * half;  // index inside the tile of 4 consecutive slots
      const int4 bi = *reinterpret_cast<const int4*>(&bidx_s[t & 1][base]);
      const int4 ps = *reinterpret_cast<const int4*>(&pos_s[t & 1][base]);
      const int biv[4] = {bi.x, bi.y, bi.z, bi.w};
      const int psv[4] = {ps.x, ps.y, ps.z, ps.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int slot = tr0 + base + e;
        float x = sacc[t2][4 * g4 + e] * sc;
        if (w > 0) {
          const int dlt = qp[t2] - psv[e];
          if (dlt >= 0 && dlt < w) x += rb;
        }
        if (slot >= row1 || biv[e] > ti[t2]) x = -INFINITY;
        tv[4 * g4 + e] = x;
        mb = fmaxf(mb, x);
      }
      const int slot0 = tr0 + base;
      if (q < b && slot0 < row1) {  // logits of real queries and real slots are kept for the statistics
        *reinterpret_cast<float4*>(z + static_cast<size_t>(q) * B + slot0) =
            make_float4(tv[4 * g4], tv[4 * g4 + 1], tv[4 * g4 + 2], tv[4 * g4 + 3]);
      }
    }
    mb = fmaxf(mb, __shfl_xor(mb, 32, kWave));  // both lane halves feed one matrix product
    const float m_new = fmaxf(m[t2], mb);
    if (__any(m_new > m[t2])) {
      const float alpha = (m_new > -INFINITY) ? fast_exp2(m[t2] - m_new) : 1.0f;
      l[t2] *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t2][db][r] *= alpha;
    }
    m[t2] = m_new;
    float sum = 0.0f;
    const float ref = (m_new > -INFINITY) ? m_new : 0.0f;  // nothing visible yet: every term is 2^-inf = 0
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pv = fast_exp2(tv[r] - ref);
      sum += pv;
      pfrag[t2][r >> 3][r & 7] = static_cast<__bf16>(pv);
    }
    l[t2] += sum;
    }
    // ---- O^T += V^T . P^T
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const char* vt = tileV + (32 * wave + ks * 16) * kLdsRowV + tr_off;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const uint2 lo = lds_read_transposed(vt + db * 64);
        const uint2 hi = lds_read_transposed(vt + 8 * kLdsRowV + db * 64);
        const bf16x8 afrag = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
        for (int t2 = 0; t2 < NQT; ++t2)
          o[t2][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, pfrag[t2][ks], o[t2][db], 0, 0, 0);
      }
    }
    }
  }
#pragma unroll
  for (int t2 = 0; t2 < NQT; ++t2) l[t2] += __shfl_xor(l[t2], 32, kWave);  // the lane halves summed different slots

  // ---- merge the two waves (wave 1 hands its state to wave 0 through LDS), then write the split's partial
  __syncthreads();  // everybody is done with the tiles
  float* mo = reinterpret_cast<float*>(lds_dyn);  // [QR query rows][128 dims]
  if (wave == 1) {
#pragma unroll
    for (int t2 = 0; t2 < NQT; ++t2) {
      const int q = kQ * t2 + qi;
      if (half == 0) { merge_m[q] = m[t2]; merge_l[q] = l[t2]; }
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) mo[q * D + db * 32 + 8 * (r >> 2) + 4 * half + (r & 3)] = o[t2][db][r];
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int t2 = 0; t2 < NQT; ++t2) {
      const int q = kQ * t2 + qi;
      if (q >= b) continue;  // lanes beyond the step's query rows repeated its last query: nothing of theirs is kept
      const float m1 = merge_m[q], l1 = merge_l[q];
      const float M = fmaxf(m[t2], m1);
      const float w0 = (m[t2] > -INFINITY) ? fast_exp2(m[t2] - M) : 0.0f;
      const float w1 = (m1 > -INFINITY) ? fast_exp2(m1 - M) : 0.0f;
      if (half == 0) {
        a.part_m[pidx * QR + q] = M;
        a.part_l[pidx * QR + q] = l[t2] * w0 + l1 * w1;
      }
      float* po = a.part_o + (pidx * QR + q) * D;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int d0 = db * 32 + 8 * g4 + 4 * half;
          float4 r4;
          const float4 other = (w1 > 0.0f) ? *reinterpret_cast<const float4*>(mo + q * D + d0)
                                           : make_float4(0.0f, 0.0f, 0.0f, 0.0f);  // wave 1 saw nothing: ignore LDS
          r4.x = o[t2][db][4 * g4 + 0] * w0 + other.x * w1;
          r4.y = o[t2][db][4 * g4 + 1] * w0 + other.y * w1;
          r4.z = o[t2][db][4 * g4 + 2] * w0 + other.z * w1;
          r4.w = o[t2][db][4 * g4 + 3] * w0 + other.w * w1;
          *reinterpret_cast<float4*>(po + d0) = r4;
        }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// The attention of the block-wise / grouped-query step for the shapes the matrix-core kernel is not built for
// (fp32, head_dim 64), on the vector ALUs: grid (splits, units), four waves.  K and V are streamed once for all
// query rows of the step, as on the matrix-core path: a tile of 64 slots goes through LDS (as fp32), then
//   scores : a wave takes every fourth query row.  Its lanes form QS groups; a lane owns QS slots of the tile (one
//            lane of every group per slot) and the queries of its group, so that every K or Q value read from LDS
//            feeds several multiply-adds (a register block of QS slots x QL queries per lane: with one slot per
//            lane the broadcast reads of Q, not the arithmetic, set the pace).  The group keeps an online softmax
//            per query row (maximum and sum over the tile by lane reductions inside the group), stores the base-2
//            logits and leaves the tile's probabilities and the factor that rescales the running output in LDS.
//   output : a thread owns four output dimensions of every NG-th query row: O[q][d] = O[q][d] alpha[q] +
//            sum_r P[q][r] V[r][d], four slots at a time (one 16-byte read of P per row, of V per slot).
// The vector work grows with the number of query rows while the bytes do not: a step of many rows is bound by the
// ALUs, and still reads the cache once instead of once per row.  Produces what block_attend produces.
template <int D> struct SharedTile {
  static constexpr int kRows = 64;        // slots per tile
  static constexpr int kStride = D + 4;   // floats per K row in LDS: lanes that read consecutive rows hit different banks
  static size_t lds_bytes(int qmax) {     // K tile, V tile, probabilities, queries, rescale factors
    return (static_cast<size_t>(kRows) * kStride + static_cast<size_t>(kRows) * D + static_cast<size_t>(qmax) * kRows +
            static_cast<size_t>(qmax) * D + qmax) * sizeof(float);
  }
};

// QMAX: most query rows the instantiation takes (8, 16, 32 or 64).  The smaller ones need fewer registers and less LDS,
// so more workgroups fit a compute unit, and they keep two tiles in flight per workgroup instead of one.
template <int DT, int D, int QMAX>
__global__ __launch_bounds__(256, (D == 64 ? 2 : 1)) void block_attend_shared(BlockArgs a) {
  using G = RowGeom<DT, D>;
  using T = SharedTile<D>;
  constexpr int TR = T::kRows, KS = T::kStride, WAVES = 4;
  constexpr int KQ = QMAX / WAVES;       // query rows per wave: wave + 4 k
  constexpr int QS = KQ >= 4 ? 4 : KQ;   // lane groups of a wave = slots per lane
  constexpr int RG = kWave / QS;         // lanes per group; lane rg owns slots rg + RG i, i < QS
  constexpr int QL = KQ / QS;            // query rows per lane: k = qs + QS jq
  constexpr int DQ = D / 4;              // output phase: threads per query row, four dimensions each
  constexpr int NG = 256 / DQ;           // ... and groups of threads: group og takes rows og + NG k
  constexpr int OQ = QMAX >= NG ? QMAX / NG : 1;
  constexpr int CH = TR * G::LPR / 256;  // 16-byte pieces of a tile per thread and operand
  constexpr int PF = (QMAX <= 8 || (QMAX <= 32 && D == 64)) ? 2 : 1;  // tiles in flight
  static_assert(CH >= 1 && TR * G::LPR % 256 == 0, "a tile is dealt evenly to the threads");
  static_assert(QMAX % WAVES == 0 && KQ % QS == 0 && QS * RG == kWave && RG * QS == TR && QMAX <= kMaxBlock, "query rows and slots are dealt evenly");
  extern __shared__ __attribute__((aligned(16))) float lds_f[];
  __shared__ int32_t bidx_s[TR], pos_s[TR];
  float* const Kt = lds_f;                 // [TR][KS]
  float* const Vt = Kt + TR * KS;          // [TR][D]
  float* const Pt = Vt + TR * D;           // [QMAX][TR] probabilities of the tile against the running reference
  float* const Qs = Pt + QMAX * TR;        // [QMAX][D]  queries times scale * log2(e)
  float* const al = Qs + QMAX * D;         // [QMAX]     factor for the running output of a query row
  const int u = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int B = a.B, nq = a.queries, QR = a.qrows;  // QR: rows per unit of the workspace planes
  const int n = a.n_used[u];  // block_prepare has run: the block's rows are in the cache and counted
  const int row0 = split * a.rows_per_split;
  const int row1 = min(n, row0 + a.rows_per_split);
  const size_t pidx = static_cast<size_t>(u) * a.splits + split;
  const char* Kb = static_cast<const char*>(a.K) + static_cast<size_t>(u) * B * G::ROW_BYTES;
  const char* Vb = static_cast<const char*>(a.V) + static_cast<size_t>(u) * B * G::ROW_BYTES;
  const int32_t* bidx = a.blk_idx + static_cast<size_t>(u) * B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  float* z = a.z + static_cast<size_t>(u) * QR * B;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const int qp0 = a.qpos0[u];

  for (int idx = tid; idx < QMAX * G::LPR; idx += 256) {  // the step's queries, scaled, as fp32; zeros beyond them
    const int q = idx / G::LPR, c = idx % G::LPR;
    float f[G::EPL];
    unpack16<DT>(load16(static_cast<const char*>(a.q) + (static_cast<size_t>(u) * nq + min(q, nq - 1)) * G::ROW_BYTES + c * 16), f);
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) Qs[q * D + c * G::EPL + e] = q < nq ? f[e] * a.scale_log2 : 0.0f;
  }

  const int rg = lane % RG, qs = lane / RG;
  int qrow[QL];        // this lane's query rows (may lie beyond the step's: those compute on zeros and store nothing)
  float m[QL], l[QL];  // their online softmax (the same in every lane of the group)
#pragma unroll
  for (int jq = 0; jq < QL; ++jq) {
    qrow[jq] = wave + WAVES * (qs + QS * jq);
    m[jq] = -INFINITY;
    l[jq] = 0.0f;
  }
  const int dq = tid % DQ, og = tid / DQ;
  float4 o[OQ];
#pragma unroll
  for (int k = 0; k < OQ; ++k) o[k] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

  const int n_tiles = row1 > row0 ? (row1 - row0 + TR - 1) / TR : 0;
  uint4 pk[PF][CH], pv[PF][CH];
  int32_t st_bidx[PF], st_pos[PF];  // first wave: of slot `lane` of the tiles on their way
  auto fetch = [&](int t, uint4* fk, uint4* fv, int32_t& fb, int32_t& fp) {
    const int tr0 = row0 + t * TR;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int idx = tid + 256 * i;
      const int row = min(tr0 + idx / G::LPR, n - 1);  // slots past the end are masked below
      const size_t off = static_cast<size_t>(row) * G::ROW_BYTES + (idx % G::LPR) * 16;
      fk[i] = a.streaming ? load16_streaming(Kb + off) : load16(Kb + off);
      fv[i] = a.streaming ? load16_streaming(Vb + off) : load16(Vb + off);
    }
    if (tid < TR) {
      const int slot = min(tr0 + tid, n - 1);
      fb = bidx[slot];
      fp = pos[slot];
    }
  };
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    st_bidx[j] = -1;
    st_pos[j] = 0;
    if (j < n_tiles) fetch(j, pk[j], pv[j], st_bidx[j], st_pos[j]);
  }
  for (int t0 = 0; t0 < n_tiles; t0 += PF) {
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      const int t = t0 + j;
      if (t >= n_tiles) break;
      const int tr0 = row0 + t * TR;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const int idx = tid + 256 * i;
        const int r = idx / G::LPR, c = idx % G::LPR;
        float fk[G::EPL], fv[G::EPL];
        unpack16<DT>(pk[j][i], fk);
        unpack16<DT>(pv[j][i], fv);
#pragma unroll
        for (int e = 0; e < G::EPL; e += 4) {
          *reinterpret_cast<float4*>(Kt + r * KS + c * G::EPL + e) = make_float4(fk[e], fk[e + 1], fk[e + 2], fk[e + 3]);
          *reinterpret_cast<float4*>(Vt + r * D + c * G::EPL + e) = make_float4(fv[e], fv[e + 1], fv[e + 2], fv[e + 3]);
        }
      }
      if (tid < TR) { bidx_s[tid] = st_bidx[j]; pos_s[tid] = st_pos[j]; }
      __syncthreads();  // the tile (and, the first time, the queries) are in LDS
      if (t + PF < n_tiles) fetch(t + PF, pk[j], pv[j], st_bidx[j], st_pos[j]);

      // ---- scores: QS slots x QL query rows per lane (a wave whose first query row lies beyond the step's has none)
      if (wave < nq) {
      float part[QS][QL];
#pragma unroll
      for (int i = 0; i < QS; ++i)
#pragma unroll
        for (int jq = 0; jq < QL; ++jq) part[i][jq] = 0.0f;
#pragma unroll 2  // (fully unrolled, the compiler hoists every LDS read of the tile and runs out of registers)
      for (int c0 = 0; c0 < D; c0 += 8) {
        float4 kc[QS][2];
#pragma unroll
        for (int i = 0; i < QS; ++i) {
          kc[i][0] = *reinterpret_cast<const float4*>(Kt + (rg + RG * i) * KS + c0);
          kc[i][1] = *reinterpret_cast<const float4*>(Kt + (rg + RG * i) * KS + c0 + 4);
        }
#pragma unroll
        for (int jq = 0; jq < QL; ++jq) {
          const int q = min(qrow[jq], QMAX - 1);
          const float4 qa = *reinterpret_cast<const float4*>(Qs + q * D + c0);
          const float4 qb = *reinterpret_cast<const float4*>(Qs + q * D + c0 + 4);
#pragma unroll
          for (int i = 0; i < QS; ++i) {
            float s = part[i][jq];
            s = fmaf(kc[i][0].x, qa.x, s); s = fmaf(kc[i][0].y, qa.y, s);
            s = fmaf(kc[i][0].z, qa.z, s); s = fmaf(kc[i][0].w, qa.w, s);
            s = fmaf(kc[i][1].x, qb.x, s); s = fmaf(kc[i][1].y, qb.y, s);
            s = fmaf(kc[i][1].z, qb.z, s); s = fmaf(kc[i][1].w, qb.w, s);
            part[i][jq] = s;
          }
        }
      }
#pragma unroll
      for (int jq = 0; jq < QL; ++jq) {
        const int q = qrow[jq];
        const bool live = q < nq;   // uniform inside a group of lanes, not inside the wave
        const int ti = q / a.heads;  // the heads of a group share the token's position
        float x[QS];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < QS; ++i) {
          const int r = rg + RG * i, slot = tr0 + r;
          float v = part[i][jq];
          const int dlt = qp0 + ti - pos_s[r];
          if (w > 0 && dlt >= 0 && dlt < w) v += rb;
          if (slot >= row1 || bidx_s[r] > ti) v = -INFINITY;  // no such slot, or a later token of the block
          if (live && slot < row1) z[static_cast<size_t>(q) * B + slot] = v;  // kept for the statistics
          x[i] = v;
          mx = fmaxf(mx, v);
        }
        const float m_new = fmaxf(m[jq], group_max<RG>(mx));
        const float ref = (m_new > -INFINITY) ? m_new : 0.0f;  // nothing visible yet: every term is 2^-inf = 0
        const float alpha = (m_new > -INFINITY) ? fast_exp2(m[jq] - m_new) : 1.0f;
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < QS; ++i) {
          const float pr = fast_exp2(x[i] - ref);
          sum += pr;
          if (live) Pt[q * TR + rg + RG * i] = pr;
        }
        l[jq] = fmaf(l[jq], alpha, group_sum<RG>(sum));
        m[jq] = m_new;
        if (live && rg == 0) al[q] = alpha;
      }
      }
      __syncthreads();  // the tile's probabilities are in LDS

      // ---- O[q][d] = O[q][d] alpha[q] + sum_r P[q][r] V[r][d] (a wave whose first query row is beyond the step's: idle)
      if ((wave * kWave) / DQ < nq) {
#pragma unroll
      for (int k = 0; k < OQ; ++k) {
        const int q = og + NG * k;
        if (q < nq) {
          const float f = al[q];
          o[k].x *= f; o[k].y *= f; o[k].z *= f; o[k].w *= f;
        }
      }
      for (int r = 0; r < TR; r += 4) {
        const float4 v0 = *reinterpret_cast<const float4*>(Vt + r * D + 4 * dq);
        const float4 v1 = *reinterpret_cast<const float4*>(Vt + (r + 1) * D + 4 * dq);
        const float4 v2 = *reinterpret_cast<const float4*>(Vt + (r + 2) * D + 4 * dq);
        const float4 v3 = *reinterpret_cast<const float4*>(Vt + (r + 3) * D + 4 * dq);
#pragma unroll
        for (int k = 0; k < OQ; ++k) {
          const int q = og + NG * k;
          if (q < nq) {
            const float4 p4 = *reinterpret_cast<const float4*>(Pt + q * TR + r);
            o[k].x = fmaf(p4.x, v0.x, o[k].x); o[k].y = fmaf(p4.x, v0.y, o[k].y);
            o[k].z = fmaf(p4.x, v0.z, o[k].z); o[k].w = fmaf(p4.x, v0.w, o[k].w);
            o[k].x = fmaf(p4.y, v1.x, o[k].x); o[k].y = fmaf(p4.y, v1.y, o[k].y);
            o[k].z = fmaf(p4.y, v1.z, o[k].z); o[k].w = fmaf(p4.y, v1.w, o[k].w);
            o[k].x = fmaf(p4.z, v2.x, o[k].x); o[k].y = fmaf(p4.z, v2.y, o[k].y);
            o[k].z = fmaf(p4.z, v2.z, o[k].z); o[k].w = fmaf(p4.z, v2.w, o[k].w);
            o[k].x = fmaf(p4.w, v3.x, o[k].x); o[k].y = fmaf(p4.w, v3.y, o[k].y);
            o[k].z = fmaf(p4.w, v3.z, o[k].z); o[k].w = fmaf(p4.w, v3.w, o[k].w);
          }
        }
      }
      }
      __syncthreads();  // everybody is done with the tile before the next one overwrites it
    }
  }

  // ---- this split's partial: reference, sum and unnormalised output per query row
#pragma unroll
  for (int jq = 0; jq < QL; ++jq) {
    const int q = qrow[jq];
    if (q < nq && rg == 0) {
      a.part_m[pidx * QR + q] = m[jq];
      a.part_l[pidx * QR + q] = l[jq];
    }
  }
#pragma unroll
  for (int k = 0; k < OQ; ++k) {
    const int q = og + NG * k;
    if (q < nq) *reinterpret_cast<float4*>(a.part_o + (pidx * QR + q) * D + 4 * dq) = o[k];
  }
}

// ------------------------------------------------------------------------------------------------
// One workgroup per unit: it walks all slots of the unit two per thread and sweep, keeps the ranking keys in LDS and
// chooses the next victim itself.  (Spreading the update over slot chunks and selecting in a launch of its own
// measured slower for every number of query rows: the extra launch costs more than the longer sweep.)
// CHUNKED: the logits of four query rows are loaded at a time (chosen by the host where it measured faster: grouped
// queries, and more than 32 rows).
template <int DT, int D, bool CHUNKED>
__global__ __launch_bounds__(kFinThreads) void block_finish(BlockArgs a) {
  constexpr int NT = kFinThreads;
  constexpr int kSlots = 2 * NT;  // slots per sweep
  extern __shared__ uint32_t lds_keys[];  // [2][B] ranking keys when B <= kMaxDecodeBudgetLds
  __shared__ uint32_t sel_sh[kSelectLdsWords];
  __shared__ unsigned long long best_sh[NT / kWave];
  __shared__ float Mq[kMaxBlock], invq[kMaxBlock];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int B = a.B, nq = a.queries, S = a.splits, QR = a.qrows;
  int n = a.n_used[u];
  int fresh = -1;  // single-token step without block_prepare: the slot the token took, which this kernel books
  bool evicted = false;
  if (a.single) {
    evicted = n >= B;
    fresh = evicted ? min(max(a.next_slot[u], 0), B - 1) : n;
    n = evicted ? B : n + 1;
  }
  const int heads = a.heads;
  const float inv_heads = 1.0f / static_cast<float>(heads);
  const float* pm = a.part_m + static_cast<size_t>(u) * S * QR;
  const float* pl = a.part_l + static_cast<size_t>(u) * S * QR;
  const float* po = a.part_o + static_cast<size_t>(u) * S * QR * D;

  if (tid < nq) {  // per query row: merge the splits' normalisers in split order
    float M = -INFINITY;
    for (int s = 0; s < S; ++s) M = fmaxf(M, pm[s * QR + tid]);
    float L = 0.0f;
    for (int s = 0; s < S; ++s) {
      const float ms = pm[s * QR + tid];
      L += (ms > -INFINITY) ? pl[s * QR + tid] * fast_exp2(ms - M) : 0.0f;
    }
    Mq[tid] = M;
    invq[tid] = 1.0f / L;
  }
  __syncthreads();  // every thread has read n_used and next_slot
  if (a.single && tid == 0) {
    int32_t* pos = a.pos + static_cast<size_t>(u) * B;
    const int old_pos = pos[fresh];
    pos[fresh] = a.qpos0[u];
    a.n_used[u] = n;
    if (a.evicted_slot) a.evicted_slot[u] = evicted ? fresh : -1;
    if (a.evicted_pos) a.evicted_pos[u] = evicted ? old_pos : -1;
  }
  // outputs of this workgroup's query rows
  for (int idx = tid; idx < nq * D; idx += NT) {
    const int q = idx / D, dd = idx % D;
    float o = 0.0f;
    for (int s = 0; s < S; ++s) {
      const float ms = pm[s * QR + q];
      o += (ms > -INFINITY) ? po[(static_cast<size_t>(s) * QR + q) * D + dd] * fast_exp2(ms - Mq[q]) : 0.0f;
    }
    store_elem<DT>(a.out, (static_cast<size_t>(u) * nq + q) * D + dd, o * invq[q]);
  }
  // statistics: every slot receives, per block token that attended it, the head-mean of the probabilities
  float* acc = a.stats + static_cast<size_t>(u) * 3 * B;
  float* acc2 = acc + B;
  float* cnt = acc2 + B;
  const float* z = a.z + static_cast<size_t>(u) * QR * B;
  const bool full = n >= B;
  uint32_t* var_key = (B <= kMaxDecodeBudgetLds) ? lds_keys : a.keys + static_cast<size_t>(u) * 2 * B;
  uint32_t* mas_key = var_key + B;
  const bool by_pos = a.pol.needs_pos();
  // B is a multiple of 4 on this path, so a pair of slots is inside [0, B).
  for (int j = tid * 2; j < n; j += kSlots) {
  const int2 bi = a.single ? make_int2(-1, -1)
                                       : *reinterpret_cast<const int2*>(a.blk_idx + static_cast<size_t>(u) * B + j);
  const float2 a1 = *reinterpret_cast<const float2*>(acc + j);
  const float2 a2 = *reinterpret_cast<const float2*>(acc2 + j);
  const float2 cc = *reinterpret_cast<const float2*>(cnt + j);
  float s1[2] = {a1.x, a1.y}, s2[2] = {a2.x, a2.y}, sc[2] = {cc.x, cc.y};
  const int biv[2] = {bi.x, bi.y};
#pragma unroll
  for (int e = 0; e < 2; ++e)
    if (j + e == fresh) { s1[e] = 0.0f; s2[e] = 0.0f; sc[e] = 0.0f; }  // the new token starts from zero
  auto book = [&](const float* mean, int t) {  // token t of the block has attended: its head-mean goes to the slots
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      if (j + e < n && biv[e] <= t) {  // older tokens have index -1: attended by every row
        const float p = mean[e] * inv_heads;  // group-wise averaged probability (exact for one head)
        s1[e] += p;
        s2[e] = a.pol.second_statistic(s2[e], p, static_cast<float>(n - a.block + t + 1));  // what row t attended
        sc[e] += 1.0f;
      }
    }
  };
  if (!CHUNKED) {
    for (int t = 0; t < a.block; ++t) {
      float mean[2] = {0.0f, 0.0f};  // sum over the token's query heads of p
      for (int h = 0; h < heads; ++h) {
        const int q = t * heads + h;
        const float2 zz = *reinterpret_cast<const float2*>(z + static_cast<size_t>(q) * B + j);
        const float M = Mq[q], inv = invq[q];
        mean[0] += fast_exp2(zz.x - M) * inv;
        mean[1] += fast_exp2(zz.y - M) * inv;
      }
      book(mean, t);
    }
  } else {
    // The query rows (token-major, a token's heads side by side) are taken four at a time, so that four logit
    // loads are in flight per thread instead of one.
    float mean[2] = {0.0f, 0.0f};  // sum over the query heads of the token under way of p
    int t = 0, h = 0;
    for (int q0 = 0; q0 < nq; q0 += 4) {
      float2 zz[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        zz[i] = *reinterpret_cast<const float2*>(z + static_cast<size_t>(min(q0 + i, nq - 1)) * B + j);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int q = q0 + i;
        if (q < nq) {
          const float M = Mq[q], inv = invq[q];
          mean[0] += fast_exp2(zz[i].x - M) * inv;
          mean[1] += fast_exp2(zz[i].y - M) * inv;
          if (++h == heads) {  // the token's last head
            book(mean, t);
            mean[0] = mean[1] = 0.0f;
            h = 0;
            ++t;
          }
        }
      }
    }
  }
  *reinterpret_cast<float2*>(acc + j) = make_float2(s1[0], s1[1]);
  *reinterpret_cast<float2*>(acc2 + j) = make_float2(s2[0], s2[1]);
  *reinterpret_cast<float2*>(cnt + j) = make_float2(sc[0], sc[1]);
  if (full) {
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (j + e < n)
        ranking_keys(s1[e], s2[e], sc[e],
                     j + e == fresh ? a.qpos0[u] : (by_pos ? a.pos[static_cast<size_t>(u) * B + j + e] : 0), a.pol,
                     mas_key[j + e], var_key[j + e]);
  }
  }
  // the victim a following single-token step would take
  if (full) {
    __syncthreads();
    const int victim = select_victim_block<NT>(var_key, mas_key, B, a.pol.scope_size(a.scope, B), sel_sh, best_sh);
    if (tid == 0) a.next_slot[u] = victim;
  } else if (tid == 0) {
    a.next_slot[u] = -1;
  }
}

}  // namespace

// ROCO_BLOCK_SINGLE=0 keeps block_prepare in single-token steps (tests run both).
static bool single_step_off() {
  const char* e = getenv("ROCO_BLOCK_SINGLE");
  return e != nullptr && e[0] == '0';
}

template <int DT, int D>
void launch_block_tail(const BlockArgs& a, hipStream_t s) {
  ProfScope ps(kProfBlockFinish, s);
  const size_t key_lds = key_lds_bytes(a.B);
  // (if the limit is refused, the launch fails and is reported)
  if (a.heads > 1 || a.queries > 32) {
    (void)allow_key_lds(reinterpret_cast<const void*>(block_finish<DT, D, true>), key_lds);
    hipLaunchKernelGGL((block_finish<DT, D, true>), dim3(a.units), dim3(kFinThreads), key_lds, s, a);
  } else {
    (void)allow_key_lds(reinterpret_cast<const void*>(block_finish<DT, D, false>), key_lds);
    hipLaunchKernelGGL((block_finish<DT, D, false>), dim3(a.units), dim3(kFinThreads), key_lds, s, a);
  }
}

template <int DT, int D, int QMAX>
hipError_t launch_block_shared_q(const BlockArgs& a, hipStream_t s) {
  const size_t lds = SharedTile<D>::lds_bytes(QMAX);  // 37 to 114 KiB: the limit is set on every call
  const void* fn = reinterpret_cast<const void*>(block_attend_shared<DT, D, QMAX>);
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL((block_attend_shared<DT, D, QMAX>), dim3(a.splits, a.units), dim3(256), lds, s, a);
  return hipSuccess;
}

template <int DT, int D>
hipError_t launch_block_shared(const BlockArgs& a, hipStream_t s) {
  {
    ProfScope ps(kProfBlockAttend, s);
    const hipError_t e = a.queries <= 8    ? launch_block_shared_q<DT, D, 8>(a, s)
                         : a.queries <= 16 ? launch_block_shared_q<DT, D, 16>(a, s)
                         : a.queries <= 32 ? launch_block_shared_q<DT, D, 32>(a, s)
                                           : launch_block_shared_q<DT, D, kMaxBlock>(a, s);
    if (e != hipSuccess) return e;
  }
  launch_block_tail<DT, D>(a, s);
  return hipSuccess;
}

// dtype / head_dim other than bf16 / 128 take the vector-ALU attention
hipError_t launch_block(int dtype, int head_dim, const BlockArgs& args, hipStream_t s) {
  BlockArgs a = args;
  // A single-token step on the matrix-core path needs no block_prepare.
  a.single = (a.block == 1 && dtype == kBF16 && head_dim == 128 && !single_step_off()) ? 1 : 0;
  const size_t key_lds = key_lds_bytes(a.B);
  if (!allow_key_lds(reinterpret_cast<const void*>(block_prepare<512>), key_lds) ||
      !allow_key_lds(reinterpret_cast<const void*>(block_prepare<kPrepThreads>), key_lds))
    return hipErrorInvalidValue;
  constexpr size_t kAttLds = 2 * static_cast<size_t>(kTileBytes + kTileBytesV);  // 74 KiB: above the default dynamic limit
  const bool mfma_path = dtype == kBF16 && head_dim == 128;
  if (mfma_path) {  // set on every call: cheap, and right on whichever device is current
    const void* fn = a.qrows > kQ ? reinterpret_cast<const void*>(block_attend<2>) : reinterpret_cast<const void*>(block_attend<1>);
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kAttLds)) != hipSuccess)
      return hipErrorInvalidValue;
  }
  if (!a.single) {
    ProfScope ps(kProfBlockPrepare, s);
    // Two 1024-thread workgroups do not run side by side on a compute unit here (measured: the second half of 512
    // units starts when the first has finished); with more units than compute units 512 threads are faster.
    if (a.units > 256) hipLaunchKernelGGL(block_prepare<512>, dim3(a.units), dim3(512), key_lds, s, a);
    else hipLaunchKernelGGL(block_prepare<kPrepThreads>, dim3(a.units), dim3(kPrepThreads), key_lds, s, a);
  }
  if (mfma_path) {
    {
      ProfScope ps(kProfBlockAttend, s);
      if (a.qrows > kQ) hipLaunchKernelGGL(block_attend<2>, dim3(a.splits, a.units), dim3(kAttThreads), kAttLds, s, a);
      else hipLaunchKernelGGL(block_attend<1>, dim3(a.splits, a.units), dim3(kAttThreads), kAttLds, s, a);
    }
    launch_block_tail<kBF16, 128>(a, s);
  } else {
    hipError_t e = hipErrorInvalidValue;
    if (dtype == kBF16 && head_dim == 64) e = launch_block_shared<kBF16, 64>(a, s);
    else if (dtype == kF32 && head_dim == 64) e = launch_block_shared<kF32, 64>(a, s);
    else if (dtype == kF32 && head_dim == 128) e = launch_block_shared<kF32, 128>(a, s);
    if (e != hipSuccess) return e;
  }
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  return hipSuccess;
}

}  // namespace roco
