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
// (fp32, head_dim 64): grid (query rows, units), one workgroup streams all slots of the unit for one query row
// on the vector ALUs, exactly like a decode step does, with the slots that hold later tokens of the block masked
// out.  K and V are read once per query row, so this path has the semantics of the step but not its bandwidth
// saving.  Produces what block_attend produces with a single split.
template <int DT, int D>
__global__ __launch_bounds__(256) void block_attend_simple(BlockArgs a) {
  using G = RowGeom<DT, D>;
  constexpr int U = 4, WAVES = 4;
  constexpr int PASS = WAVES * U * G::R;
  __shared__ float sm_m[WAVES], sm_l[WAVES];
  __shared__ float sm_acc[WAVES][D];
  const int u = blockIdx.y, r = blockIdx.x;  // r: query row = (token, head)
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int c = lane % G::LPR;
  const int B = a.B;
  const int n = a.n_used[u];
  const int ti = r / a.heads;
  float qf[G::EPL];
  unpack16<DT>(load16(static_cast<const char*>(a.q) + (static_cast<size_t>(u) * a.queries + r) * G::ROW_BYTES + c * 16), qf);
#pragma unroll
  for (int e = 0; e < G::EPL; ++e) qf[e] *= a.scale_log2;
  const char* Kb = static_cast<const char*>(a.K) + static_cast<size_t>(u) * B * G::ROW_BYTES;
  const char* Vb = static_cast<const char*>(a.V) + static_cast<size_t>(u) * B * G::ROW_BYTES;
  const int32_t* bidx = a.blk_idx + static_cast<size_t>(u) * B;
  const int32_t* pos = a.pos + static_cast<size_t>(u) * B;
  float* z = a.z + (static_cast<size_t>(u) * a.qrows + r) * B;
  const int qp = a.qpos0[u] + ti;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  auto bias = [&](int row, int row_pos) -> float {
    if (bidx[row] > ti) return -INFINITY;  // a later token of the block
    const int dlt = qp - row_pos;
    return (w > 0 && dlt >= 0 && dlt < w) ? rb : 0.0f;
  };
  auto fix = [](int, uint4&, int) {};
  FlashState<G::EPL> st;
  st.reset();
  const int passes = (n + PASS - 1) / PASS;
  stream_attend<DT, D, U, true, false>(qf, Kb, Vb, 0, n, passes, 0, PASS, wave * (U * G::R), bias, pos, z, -1, fix, fix, st);
  merge_groups_in_wave<DT, D>(st);
  if (lane < G::LPR) {
    if (lane == 0) { sm_m[wave] = st.m; sm_l[wave] = st.l; }
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) sm_acc[wave][lane * G::EPL + e] = st.acc[e];
  }
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < WAVES; ++s) M = fmaxf(M, sm_m[s]);
  const size_t pidx = static_cast<size_t>(u) * a.qrows + r;  // one split
  if (tid < D) {
    float o = 0.0f, l = 0.0f;
#pragma unroll
    for (int s = 0; s < WAVES; ++s) {
      const float wgt = (sm_m[s] > -INFINITY) ? fast_exp2(sm_m[s] - M) : 0.0f;
      l += sm_l[s] * wgt;
      o += sm_acc[s][tid] * wgt;
    }
    a.part_o[pidx * D + tid] = o;
    if (tid == 0) { a.part_m[pidx] = M; a.part_l[pidx] = l; }
  }
}

// ------------------------------------------------------------------------------------------------
// One workgroup per unit: it walks all slots of the unit two per thread and sweep, keeps the ranking keys in LDS and
// chooses the next victim itself.  (Spreading the update over slot chunks and selecting in a launch of its own
// measured slower for every number of query rows: the extra launch costs more than the longer sweep.)
template <int DT, int D>
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
  for (int t = 0; t < a.block; ++t) {
    float mean[2] = {0.0f, 0.0f};  // sum over the token's query heads of p
    for (int h = 0; h < heads; ++h) {
      const int q = t * heads + h;
      const float2 zz = *reinterpret_cast<const float2*>(z + static_cast<size_t>(q) * B + j);
      const float M = Mq[q], inv = invq[q];
      mean[0] += fast_exp2(zz.x - M) * inv;
      mean[1] += fast_exp2(zz.y - M) * inv;
    }
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      if (j + e < n && biv[e] <= t) {  // older tokens have index -1: attended by every row
        const float p = mean[e] * inv_heads;  // group-wise averaged probability (exact for one head)
        s1[e] += p;
        s2[e] = a.pol.second_statistic(s2[e], p, static_cast<float>(n - a.block + t + 1));  // what row t attended
        sc[e] += 1.0f;
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
  (void)allow_key_lds(reinterpret_cast<const void*>(block_finish<DT, D>), key_lds);  // if refused, the launch fails and is reported
  hipLaunchKernelGGL((block_finish<DT, D>), dim3(a.units), dim3(kFinThreads), key_lds, s, a);
}

template <int DT, int D>
void launch_block_simple(const BlockArgs& a, hipStream_t s) {
  {
    ProfScope ps(kProfBlockAttend, s);
    hipLaunchKernelGGL((block_attend_simple<DT, D>), dim3(a.queries, a.units), dim3(256), 0, s, a);
  }
  launch_block_tail<DT, D>(a, s);
}

// dtype / head_dim other than bf16 / 128 take the vector-ALU attention (a.splits must then be 1)
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
  } else if (dtype == kBF16 && head_dim == 64) {
    launch_block_simple<kBF16, 64>(a, s);
  } else if (dtype == kF32 && head_dim == 64) {
    launch_block_simple<kF32, 64>(a, s);
  } else if (dtype == kF32 && head_dim == 128) {
    launch_block_simple<kF32, 128>(a, s);
  } else {
    return hipErrorInvalidValue;
  }
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  return hipSuccess;
}

}  // namespace roco
