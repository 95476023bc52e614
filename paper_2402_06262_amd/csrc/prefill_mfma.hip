// Prefill attention statistics on the gfx950 matrix cores: bf16 storage, head_dim 128.
//
// Two passes over the causal score matrix (a column statistic needs the final normaliser of every row it
// sums over), neither of which stores the L x L matrix:
//   pass 1  prefill_rows_mfma    : row normalisers -- base-2 log-sum-exp of every query row (section 2.1 eq. 1)
//   pass 2  prefill_columns_mfma : Acc[j] = sum_i P[i,j], Acc2[j] = sum_i P[i,j]^2 in fp32 (section 4.3)
//
// Both passes have the same shape.  A workgroup owns 256 rows of one operand (queries in pass 1, keys in
// pass 2), two groups of 32 per wave, held in registers as B operands of v_mfma_f32_32x32x16_bf16; the other
// operand is streamed through LDS in tiles of 64 rows (A operand, each fragment feeding two instructions).
// The 32x32 result tile then has the *owned* row in the
// lane (column = lane % 32) and the streamed rows in the 16 accumulator registers, so the reduction the pass
// needs (over keys in pass 1, over queries in pass 2) runs down the registers of a lane: no cross-lane traffic
// per tile, no atomics, a fixed summation order.
//
// Operand layout of the 32x32x16 instruction, as used here: lane l supplies row (l % 32) and the 8
// consecutive k-elements starting at 8 * (l / 32) of each 16-wide k-step, for A and for B alike; register r
// of the result belongs to A-row 8 * (r / 4) + 4 * (l / 32) + (r % 4) and B-row (l % 32).
#include <cstdlib>

#include "kernels.hpp"
#include "mfma.hpp"
#include "profile.hpp"
#include "stream.hpp"
#include "tile_ring.hpp"

namespace roco {
namespace {

using namespace mfma;

// A workgroup of WAVES waves owns 64*WAVES rows.  The more rows a workgroup owns, the fewer times the other
// operand is streamed from L2 / Infinity Cache (the bytes per flop of that stream are 1 / (2 * owned rows)).
template <int WAVES> struct Shape {
  static constexpr int kThreads = WAVES * kWave;
  static constexpr int kOwn = 64 * WAVES;                  // two groups of 32 per wave
  static constexpr int kChunks = kTile * 16 / kThreads;    // 16-byte chunks of a 64 x 256 B tile per thread
  static constexpr int kRowsPerSweep = kThreads / 16;
};

template <int WAVES> struct Staged {
  uint4 w[Shape<WAVES>::kChunks];  // this thread's bytes of a 64 x 256 B tile
};

// Thread t copies the chunks (row = t / 16 + sweep * threads / 16, column chunk t % 16) of the tile.
template <int WAVES>
__device__ __forceinline__ void tile_load(Staged<WAVES>& s, const char* base, int row0, int last_row) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < Shape<WAVES>::kChunks; ++i) {
    int row = row0 + (t >> 4) + Shape<WAVES>::kRowsPerSweep * i;
    row = row < last_row ? row : last_row;  // clamp: rows past the end are masked by the caller
    s.w[i] = load16(base + static_cast<size_t>(row) * kRowBytes + (t & 15) * 16);
  }
}
template <int WAVES, int ROW = kLdsRow>
__device__ __forceinline__ void tile_store(const Staged<WAVES>& s, char* lds) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < Shape<WAVES>::kChunks; ++i)
    *reinterpret_cast<uint4*>(lds + ((t >> 4) + Shape<WAVES>::kRowsPerSweep * i) * ROW + (t & 15) * 16) = s.w[i];
}

// Two 32x32 score tiles: streamed rows [sub*32, sub*32+32) of the LDS tile against the wave's two groups of
// 32 owned rows.  Every A fragment read from LDS feeds two matrix instructions (halves the LDS traffic per flop
// and gives the matrix pipe two independent accumulator chains).
__device__ __forceinline__ void score_tiles(const char* lds, int sub, const uint4* own0, const uint4* own1,
                                            bool do0, bool do1, f32x16& acc0, f32x16& acc1) {
  const int lane = threadIdx.x & (kWave - 1);
  const char* p = lds + (sub * 32 + (lane & 31)) * kLdsRow + (lane >> 5) * 16;
  const f32x16 zero = {0};  // the first instruction of a chain takes the constant as its C operand
  auto frag = [&](int kk) { return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p + kk * 32)); };
  auto mm = [](bf16x8 x, const uint4& y, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, __builtin_bit_cast(bf16x8, y), c, 0, 0, 0);
  };
  if (do0 && do1) {
    bf16x8 a = frag(0);
    acc0 = mm(a, own0[0], zero);
    acc1 = mm(a, own1[0], zero);
#pragma unroll
    for (int kk = 1; kk < kKSteps; ++kk) {
      a = frag(kk);
      acc0 = mm(a, own0[kk], acc0);
      acc1 = mm(a, own1[kk], acc1);
    }
  } else if (do0) {
    acc0 = mm(frag(0), own0[0], zero);
#pragma unroll
    for (int kk = 1; kk < kKSteps; ++kk) acc0 = mm(frag(kk), own0[kk], acc0);
  } else if (do1) {
    acc1 = mm(frag(0), own1[0], zero);
#pragma unroll
    for (int kk = 1; kk < kKSteps; ++kk) acc1 = mm(frag(kk), own1[kk], acc1);
  }
}

__device__ __forceinline__ void load_owned(uint4* own, const char* base, int row, int last_row) {
  const int lane = threadIdx.x & (kWave - 1);
  row = row < last_row ? row : last_row;
#pragma unroll
  for (int kk = 0; kk < kKSteps; ++kk)
    own[kk] = load16(base + static_cast<size_t>(row) * kRowBytes + kk * 32 + (lane >> 5) * 16);
}

// Workgroup -> (unit, block-pair) mapping.  The hardware hands consecutive workgroup ids to the 8 accelerator
// dies in turn and each die has its own L2, so the workgroups of one unit (which all stream the same K or Q
// tiles, at about the same time) are given ids that are congruent modulo 8: they land on one die and all but
// the first fetch of a tile hit its L2.  The grid is one-dimensional over ceil(units/8)*8 x pairs ids.
__device__ __forceinline__ bool locate(int units, int pairs, int& unit, int& pair) {
  const int lin = blockIdx.x;
  const int die = lin & 7, seq = lin >> 3;
  unit = (seq / pairs) * 8 + die;
  pair = seq % pairs;
  return unit < units;
}
// The same for (unit, query head) pairs, u = unit * group + head: the heads of a unit stream the same keys (and
// values), so they all go to the die unit % 8.  The grid covers ceil(units / 8) * 8 * group * pairs ids.
__device__ __forceinline__ bool locate_heads(int units, int group, int pairs, int& u, int& pair) {
  int v;  // virtual index: die v % 8, and on a die the heads of one unit before the next unit's
  if (!locate(((units + 7) / 8) * 8 * group, pairs, v, pair)) return false;
  const int unit = (v / (8 * group)) * 8 + (v & 7), head = (v >> 3) % group;
  u = unit * group + head;
  return unit < units;
}

// Online log-sum-exp update of one lane with the 16 scores of a tile.
//   INTERIOR: every key of the tile is visible to every query of the group and none is inside a recency window:
//             3 vector instructions per score (multiply-add, exponential, add) plus 8 for the maximum.
// l = sum 2^(t - m) is a floating-point number, so m need not be the running maximum: any reference that keeps the
// terms from overflowing gives the same sum to rounding.  The terms of a tile are first taken against the reference
// as it stands (3 instructions per score and nothing else: `sum`); only if some lane's share comes out above 2^64
// -- the first tile, whose reference is -inf, and a row whose scores later rise by more than 64 powers of two --
// is the tile redone with the reference raised to its maximum.
__device__ __forceinline__ void lazy_finish(float sum, const f32x16& s, float sc, float& m, float& l) {
  if (__builtin_amdgcn_ballot_w64(!(sum <= 0x1p64f)) == 0) {
    l += sum;
  } else {
    const float m_new = fmaxf(m, max16(s) * sc);
    const float neg_new = -m_new;
    float t0 = 0.0f, t1 = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      t0 += fast_exp2(fmaf(s[r], sc, neg_new));
      t1 += fast_exp2(fmaf(s[r + 1], sc, neg_new));
    }
    l = fmaf(l, fast_exp2(m - m_new), t0 + t1);
    m = m_new;
  }
}

template <bool INTERIOR>
__device__ __forceinline__ void lse_update(const f32x16& s, float sc, int kb, int half, int qi, int w, float rb,
                                           float& m, float& l) {
  if (INTERIOR) {
    const float neg = -m;
    float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      sum0 += fast_exp2(fmaf(s[r], sc, neg));
      sum1 += fast_exp2(fmaf(s[r + 1], sc, neg));
    }
    lazy_finish(sum0 + sum1, s, sc, m, l);
  } else {
    float tv[16];
    float mb = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = kb + 8 * (r >> 2) + 4 * half + (r & 3);
      float x = s[r] * sc;
      if (w > 0 && qi - key < w) x += rb;
      if (key > qi) x = -INFINITY;
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

// ------------------------------------------------------------------------------------------------
// pass 1: lse[i] = log2 sum_{j<=i} 2^(t_ij),  t_ij = scale*log2(e) * q_i.k_j + bias
//
// A workgroup owns 256 queries: wave w the groups of 32 that start at 32 w and at 32 (7 - w) of the block, so that
// the work under the causal diagonal is the same for every wave.  The key tiles come through a TileRing
// (tile_ring.hpp), requested two tiles ahead.  The keys below the block's first query form a rectangle in which
// nothing is masked and every wave does the same work: those tiles run software-pipelined (fill_and_consume: the
// matrix instructions of one half-tile interleaved with the exponentials of the half-tile before it, four
// accumulators).  The tiles that touch the diagonal or a recency window take the plain form, masks and all.
template <int S> struct StageTag { static constexpr int value = S; };

__global__ __launch_bounds__(256, 2) void prefill_rows_mfma(PrefillArgs a) {
  constexpr int kOwn = Shape<4>::kOwn;
  constexpr int NS = 4;  // ring stages: a tile is requested three tiles of work ahead of its use
  __shared__ __attribute__((aligned(1024))) char ring[NS * kRingTileBytes];
  int u, id;  // u counts (unit, query head) pairs: with grouped-query attention a unit has a.group heads
  if (!locate_heads(a.units, a.group, a.pairs * a.ksplit, u, id)) return;
  const int seg = id % a.ksplit, pair_id = id / a.ksplit;  // which share of the keys, which blocks of queries
  float* const lse_out = seg == 0 ? a.lse : a.acc;  // second share: see merge_key_shares (group = 1 only)
  const int uk = u / a.group;  // the unit: its keys and its length
  const int len = a.len[uk];
  const int lane = threadIdx.x & (kWave - 1);
  const int half = lane >> 5;
  TileRing tr;
  tr.init();
  const int wave = tr.wave;
  const uint32_t ring_addr = lds_address(ring);
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Qb = static_cast<const char*>(a.Q) + ubase * kRowBytes;
  const char* Kb = static_cast<const char*>(a.K) + static_cast<size_t>(uk) * a.L_max * kRowBytes;
  const v4i32 kbuf = make_buffer(Kb, static_cast<uint32_t>(len) * kRowBytes);  // keys past the end read as zeros
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const int n_blocks = (len + kOwn - 1) / kOwn;
  if (a.paired ? 2 * pair_id > n_blocks - 1 : pair_id >= n_blocks) return;  // nothing left for this id

  // Two schedules.  Paired: a workgroup takes one long and one short block (n-1-p and p), so that all of them do
  // the same amount of work whatever their position under the causal diagonal.  Unpaired: one block each.
  for (int pass = 0; pass < 2; ++pass) {
    int blk;
    if (a.paired) {
      // The long block first: the workgroups of a unit start together, on one die, and all of them then walk the keys
      // from row 0 at the same pace, so a key tile is fetched from memory once and found in that die's L2 by the others.
      blk = pass == 0 ? n_blocks - 1 - pair_id : pair_id;
      if (pass == 1 && blk == n_blocks - 1 - pair_id) break;  // the middle block of an odd number has no partner
    } else {
      if (pass == 1) break;
      blk = n_blocks - 1 - pair_id;  // the longest streams start first
    }
    const int q0 = blk * kOwn;
    const int qg0 = q0 + 32 * wave, qg1 = q0 + 32 * (7 - wave);  // first query of this wave's two groups (qg0 < qg1)
    const int qi0 = qg0 + (lane & 31), qi1 = qg1 + (lane & 31);
    const int last_key = min(len, q0 + kOwn) - 1;  // keys 0..last_key are visible to some query of the block
    const int n_tiles = last_key / kTile + 1;
    int t_lo = 0, t_hi = n_tiles - 1;  // this workgroup's share of the key tiles (possibly none)
    if (a.ksplit > 1) {
      const int per = (n_tiles + a.ksplit - 1) / a.ksplit;
      t_lo = seg * per;
      t_hi = min(t_hi, t_lo + per - 1);
    }
    // tiles [t_lo, t_rect) lie wholly below the block's first query and outside every recency window
    const int t_rect = min(t_hi + 1, max(t_lo, (q0 + 1 - w) >= 0 ? (q0 + 1 - w) / kTile : 0));
    __syncthreads();  // the previous block has finished with the ring
    if (t_lo <= t_hi) tr.request(kbuf, ring_addr, t_lo, 0);
    if (t_lo + 1 <= t_hi) tr.request(kbuf, ring_addr, t_lo + 1, 1);
    if (t_lo + 2 <= t_hi) tr.request(kbuf, ring_addr, t_lo + 2, 2);
    uint4 own0[kKSteps], own1[kKSteps];
    load_owned(own0, Qb, qi0, len - 1);
    load_owned(own1, Qb, qi1, len - 1);
    // The owned rows must have arrived before the loop: a wait for them inside it would also wait for the tiles
    // requested last, which are meant to stay in flight.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    float m0 = -INFINITY, l0 = 0.0f, m1 = -INFINITY, l1 = 0.0f;

    auto next_tile = [&](int t, int stage) {  // tile t has landed in `stage`; tile t + 3 is requested
      if (t + 2 <= t_hi) wait_loads<8>();  // tiles t + 1 and t + 2 may still be on their way
      else if (t + 1 <= t_hi) wait_loads<4>();
      else wait_loads<0>();
      __syncthreads();  // every wave's share of tile t is in LDS, and everybody has issued its last read of tile t - 1
      if (t + 3 <= t_hi) tr.request(kbuf, ring_addr, t + 3, (stage + 3) % NS);
    };

    // ---- the rectangle: software-pipelined.  A* hold the scores of a tile's first 32 keys, B* of its last 32.
    f32x16 A0, A1, B0, B1;
    bool pending = false;  // B* hold scores that have not been summed yet
    auto consume_into = [&](const f32x16& y0, const f32x16& y1, float& a0, float& b0, float& a1, float& b1) {
      const float n0 = -m0, n1 = -m1;
      return [&, n0, n1](int kk, int g) {
        if (g == 0) {
          a0 += fast_exp2(fmaf(y0[2 * kk], sc, n0));
          b0 += fast_exp2(fmaf(y0[2 * kk + 1], sc, n0));
        } else {
          a1 += fast_exp2(fmaf(y1[2 * kk], sc, n1));
          b1 += fast_exp2(fmaf(y1[2 * kk + 1], sc, n1));
        }
      };
    };
    auto rect_tile = [&](auto stage, int t) {
      constexpr int S = decltype(stage)::value;
      next_tile(t, S);
      const char* p = ring + S * kRingTileBytes;
      float a0 = 0.0f, b0 = 0.0f, a1 = 0.0f, b1 = 0.0f;
      auto pin = [&]() { asm volatile("" : "+v"(a0), "+v"(b0), "+v"(a1), "+v"(b1)); };
      if (pending) {
        fill_and_consume<true>(p, tr.frag, own0, own1, A0, A1, consume_into(B0, B1, a0, b0, a1, b1), pin);
        lazy_finish(a0 + b0, B0, sc, m0, l0);
        lazy_finish(a1 + b1, B1, sc, m1, l1);
      } else {
        fill_and_consume<false>(p, tr.frag, own0, own1, A0, A1, [](int, int) {}, pin);
      }
      a0 = b0 = a1 = b1 = 0.0f;
      fill_and_consume<true>(p + 32 * kRowBytes, tr.frag, own0, own1, B0, B1, consume_into(A0, A1, a0, b0, a1, b1), pin);
      lazy_finish(a0 + b0, A0, sc, m0, l0);
      lazy_finish(a1 + b1, A1, sc, m1, l1);
      pending = true;
    };
    int t = t_lo;
    for (; t + 3 < t_rect; t += 4) {
      rect_tile(StageTag<0>{}, t);
      rect_tile(StageTag<1>{}, t + 1);
      rect_tile(StageTag<2>{}, t + 2);
      rect_tile(StageTag<3>{}, t + 3);
    }
    int stage = 0;  // ring stage of tile t
    if (t < t_rect) { rect_tile(StageTag<0>{}, t); ++t; stage = 1; }
    if (t < t_rect) { rect_tile(StageTag<1>{}, t); ++t; stage = 2; }
    if (t < t_rect) { rect_tile(StageTag<2>{}, t); ++t; stage = 3; }
    if (pending) {  // drain
      float a0 = 0.0f, b0 = 0.0f, a1 = 0.0f, b1 = 0.0f;
      auto c = consume_into(B0, B1, a0, b0, a1, b1);
#pragma unroll
      for (int kk = 0; kk < kKSteps; ++kk) { c(kk, 0); c(kk, 1); }
      lazy_finish(a0 + b0, B0, sc, m0, l0);
      lazy_finish(a1 + b1, B1, sc, m1, l1);
    }

    // ---- the tiles that touch the diagonal (or a recency window): masks decided per wave and group
    if (w == 0 && t_hi - t < NS && t <= t_hi) {
      // No window and at most four tiles left (the block's own 256 keys): they all fit in the ring, so the waves
      // need not meet after every tile.  Per tile the work is uneven (the early group of a wave has run out of
      // visible keys while its late group still has some), over the whole triangle it is even: nine half-tiles per
      // wave.  Tiles t .. t + 2 were requested by the rectangle (or the prologue); the fourth is requested here and
      // waited for once, after the first tile's work.  Half-tiles that only the late group still sees are taken
      // two at a time, so that there are always two accumulator chains.
      const int t0 = t, stage0 = stage;
      wait_loads<0>();
      __syncthreads();  // tiles t0 .. t0 + 2 are in LDS; everybody has issued its last read of tile t0 - 1
      if (t0 + 3 <= t_hi) tr.request(kbuf, ring_addr, t0 + 3, (stage0 + 3) % NS);
      const int n_sub = 2 * (t_hi - t0 + 1);
      auto sub_ptr = [&](int sg) {
        const int st = (stage0 + (sg >> 1)) % NS;
        return ring + st * kRingTileBytes + (sg & 1) * (32 * kRowBytes);
      };
      auto update0 = [&](const f32x16& s0, int kb) {
        if (kb + 31 <= qg0) lse_update<true>(s0, sc, kb, half, qi0, w, rb, m0, l0);
        else lse_update<false>(s0, sc, kb, half, qi0, w, rb, m0, l0);
      };
      auto update1 = [&](const f32x16& s1, int kb) {
        if (kb + 31 <= qg1) lse_update<true>(s1, sc, kb, half, qi1, w, rb, m1, l1);
        else lse_update<false>(s1, sc, kb, half, qi1, w, rb, m1, l1);
      };
      auto run = [&](int sg, int sg_end) {  // half-tiles [sg, sg_end) of the triangle
        while (sg < sg_end) {
          const int kb = t0 * kTile + 32 * sg;
          if (kb > qg1 + 31) break;  // wholly above the diagonal for both groups (qg0 < qg1), and so is the rest
          f32x16 s0, s1;
          if (kb <= qg0 + 31) {  // both groups: one fragment, two chains
            score_tiles_ring(sub_ptr(sg), tr.frag, own0, own1, true, true, s0, s1);
            update0(s0, kb);
            update1(s1, kb);
            sg += 1;
          } else if (sg + 1 < sg_end && kb + 32 <= qg1 + 31) {  // the late group alone, two half-tiles at once
            score_two_subs_ring(sub_ptr(sg), sub_ptr(sg + 1), tr.frag, own1, s0, s1);
            update1(s0, kb);
            update1(s1, kb + 32);
            sg += 2;
          } else {
            score_tiles_ring(sub_ptr(sg), tr.frag, own0, own1, false, true, s0, s1);
            update1(s1, kb);
            sg += 1;
          }
        }
      };
      run(0, min(2, n_sub));
      if (n_sub > 6) {
        wait_loads<0>();
        __syncthreads();  // the fourth tile is in LDS
      }
      run(2, n_sub);
      t = t_hi + 1;
    }
    for (; t <= t_hi; ++t) {
      next_tile(t, stage);
      const char* p = ring + stage * kRingTileBytes;
      stage = stage == NS - 1 ? 0 : stage + 1;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int kb = t * kTile + sub * 32;
        const bool do0 = kb <= qg0 + 31, do1 = kb <= qg1 + 31;  // not wholly above the diagonal
        if (!do1) continue;
        f32x16 s0, s1;
        score_tiles_ring(p + sub * (32 * kRowBytes), tr.frag, own0, own1, do0, do1, s0, s1);
        if (do0) {
          if (kb + 31 + w <= qg0) lse_update<true>(s0, sc, kb, half, qi0, w, rb, m0, l0);
          else lse_update<false>(s0, sc, kb, half, qi0, w, rb, m0, l0);
        }
        if (kb + 31 + w <= qg1) lse_update<true>(s1, sc, kb, half, qi1, w, rb, m1, l1);
        else lse_update<false>(s1, sc, kb, half, qi1, w, rb, m1, l1);
      }
    }
    // the two lane halves hold different keys of the same query
    {
      const float mo = __shfl_xor(m0, 32, kWave), lo = __shfl_xor(l0, 32, kWave);
      const float mn = fmaxf(m0, mo);
      const float tot = (m0 > -INFINITY ? l0 * fast_exp2(m0 - mn) : 0.0f) + (mo > -INFINITY ? lo * fast_exp2(mo - mn) : 0.0f);
      if (half == 0 && qi0 < len) lse_out[ubase + qi0] = mn + log2f(tot);  // -inf for a share without keys
    }
    {
      const float mo = __shfl_xor(m1, 32, kWave), lo = __shfl_xor(l1, 32, kWave);
      const float mn = fmaxf(m1, mo);
      const float tot = (m1 > -INFINITY ? l1 * fast_exp2(m1 - mn) : 0.0f) + (mo > -INFINITY ? lo * fast_exp2(mo - mn) : 0.0f);
      if (half == 0 && qi1 < len) lse_out[ubase + qi1] = mn + log2f(tot);
    }
  }
}

// Column-statistics update of one lane (one key) with the 16 scores of a tile (16 queries).  COUNT: the second
// statistic is the number of queries that gave the key more than their row's average, p * (i + 1) > 1 (section
// 4.1, quantised score), instead of the sum of squares.
template <bool INTERIOR, bool COUNT>
__device__ __forceinline__ void column_update(const f32x16& s, const float* lse_tile, const float* rinv_tile, float sc,
                                              int ib, int half, int kj, int len, int w, float rb, float& s1, float& s2) {
  float a1 = 0.0f, a2 = 0.0f, b1 = 0.0f, b2 = 0.0f;
#pragma unroll
  for (int g4 = 0; g4 < 4; ++g4) {
    const float4 ls = *reinterpret_cast<const float4*>(lse_tile + 8 * g4 + 4 * half);
    const float lv[4] = {ls.x, ls.y, ls.z, ls.w};
    float rv[4] = {0.0f, 0.0f, 0.0f, 0.0f};  // COUNT: 1 / (tokens the query attended), staged with the normalisers
    if (COUNT) {
      const float4 rs = *reinterpret_cast<const float4*>(rinv_tile + 8 * g4 + 4 * half);
      rv[0] = rs.x; rv[1] = rs.y; rv[2] = rs.z; rv[3] = rs.w;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x = fmaf(s[4 * g4 + e], sc, -lv[e]);
      float p;
      if (INTERIOR) {
        p = fast_exp2(x);
      } else {
        const int qi = ib + 8 * g4 + 4 * half + e;
        if (w > 0 && qi - kj < w) x += rb;
        p = fast_exp2(x);
        if (qi < kj || qi >= len) p = 0.0f;
      }
      float second;
      if (COUNT) {
        second = p > rv[e] ? 1.0f : 0.0f;  // p * (i + 1) > 1
      } else {
        second = p * p;
      }
      if (e & 1) { b1 += p; b2 = COUNT ? b2 + second : fmaf(p, p, b2); }
      else       { a1 += p; a2 = COUNT ? a2 + second : fmaf(p, p, a2); }
    }
  }
  s1 += a1 + b1;
  s2 += a2 + b2;
}

// ------------------------------------------------------------------------------------------------
// pass 2: Acc[j] = sum_{i>=j} 2^(t_ij - lse_i),  Acc2[j] = sum_{i>=j} (same)^2
//
// A workgroup owns 256 keys (wave w the groups of 32 that start at 32 w and 32 (7 - w) of the block) and walks the
// query tiles from the end of the prompt DOWN to its own keys: every workgroup of a unit then starts at the same
// tile and moves at the same pace, so a query tile is fetched from memory once and found in the die's L2 by the
// others (a sum does not care about the order of its terms).  The tiles come through a TileRing; the row
// normalisers of a tile's 64 queries ride along with it, every wave loading them into a copy of its own (one more
// load per wave and tile; four stages, because a tile's normalisers are still needed one tile later by the
// pipelined form).  Queries that lie past all of the block's keys and outside every recency window form a
// rectangle in which nothing is masked: software-pipelined as in the row pass; the ragged end of the prompt and
// the tiles on the diagonal take the plain form.
template <bool COUNT>
__global__ __launch_bounds__(256, 2) void prefill_columns_mfma(PrefillArgs a) {
  constexpr int kOwn = Shape<4>::kOwn;
  constexpr int NS = 4;          // ring stages: a tile is requested three tiles of work ahead of its use
  constexpr int kLseStages = 8;  // the normalisers of a tile are still read while the tile after it is worked on
  __shared__ __attribute__((aligned(1024))) char ring[NS * kRingTileBytes];
  __shared__ __attribute__((aligned(256))) float lse_s[kLseStages][4][kTile];  // [stage][wave][query of the tile]
  __shared__ __attribute__((aligned(16))) float rinv_s[COUNT ? kLseStages : 1][COUNT ? kTile : 4];  // 1 / (i + 1)
  int u, id;
  if (!locate(a.units, a.pairs * a.qsplit, u, id)) return;
  const int seg = id % a.qsplit, pair_id = id / a.qsplit;  // which share of the queries, which blocks of keys
  float* const out1 = seg == 0 ? a.acc : reinterpret_cast<float*>(a.var_key);    // second share: see sum_query_shares
  float* const out2 = seg == 0 ? a.acc2 : reinterpret_cast<float*>(a.mas_key);
  const int len = a.len[u];
  const int lane = threadIdx.x & (kWave - 1);
  const int half = lane >> 5;
  TileRing tr;
  tr.init();
  const int wave = tr.wave;
  const uint32_t ring_addr = lds_address(ring);
  const uint32_t lse_addr = lds_address(&lse_s[0][wave][0]);
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Qb = static_cast<const char*>(a.Q) + ubase * kRowBytes;
  const char* Kb = static_cast<const char*>(a.K) + ubase * kRowBytes;
  const v4i32 qbuf = make_buffer(Qb, static_cast<uint32_t>(len) * kRowBytes);  // queries past the end read as zeros
  const v4i32 lbuf = make_buffer(a.lse + ubase, static_cast<uint32_t>(len) * 4u);
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const int n_blocks = (len + kOwn - 1) / kOwn;
  if (a.paired ? 2 * pair_id > n_blocks - 1 : pair_id >= n_blocks) return;  // nothing left for this id

  for (int pass = 0; pass < 2; ++pass) {  // one long and one short block of keys per workgroup, the long one first
    int blk;
    if (a.paired) {
      blk = pass == 0 ? pair_id : n_blocks - 1 - pair_id;
      if (blk < pair_id || (pass == 1 && blk == pair_id)) break;
    } else {
      if (pass == 1) break;
      blk = pair_id;  // the longest streams start first: key block 0 is attended by every query
    }
    const int j0 = blk * kOwn;
    const int kg0 = j0 + 32 * wave, kg1 = j0 + 32 * (7 - wave);  // first key of this wave's two groups (kg0 < kg1)
    const int kj0 = kg0 + (lane & 31), kj1 = kg1 + (lane & 31);  // this lane's two keys
    int t_first = j0 / kTile;  // first query tile with a query >= j0
    int t_last = (len - 1) / kTile;
    if (a.qsplit > 1) {  // this workgroup's share of those tiles (possibly none)
      const int per = (t_last - t_first + a.qsplit) / a.qsplit;
      t_first += seg * per;
      t_last = min(t_last, t_first + per - 1);
    }
    const int n = t_last - t_first + 1;  // the i-th tile of the walk is t_last - i
    // tiles from t_rect_lo on lie past every key of the block and outside every recency window
    const int t_rect_lo = (j0 + kOwn - 1 + w + kTile - 1) / kTile;
    auto request = [&](int i) {  // five loads per wave
      const int t = t_last - i;
      tr.request(qbuf, ring_addr, t, i % NS);
      load4_to_lds(lbuf, lse_addr + (i % kLseStages) * (4 * kTile * 4), lane * 4, __builtin_amdgcn_readfirstlane(t * kTile * 4));
    };
    __syncthreads();  // the previous block has finished with the ring
    if (0 < n) request(0);
    if (1 < n) request(1);
    if (2 < n) request(2);
    uint4 own0[kKSteps], own1[kKSteps];
    load_owned(own0, Kb, kj0, len - 1);
    load_owned(own1, Kb, kj1, len - 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the owned rows are in before the loop (see prefill_rows_mfma)
    float s1a = 0.0f, s2a = 0.0f, s1b = 0.0f, s2b = 0.0f;
    // second chain of each sum in the rectangle (odd scores of a register pair); folded into the sums after it
    float t1a = 0.0f, t2a = 0.0f, t1b = 0.0f, t2b = 0.0f;

    auto put_rinv = [&](int i) {
      if (COUNT && threadIdx.x < kTile)
        rinv_s[COUNT ? i % kLseStages : 0][threadIdx.x] =
            1.0f / static_cast<float>((t_last - i) * kTile + static_cast<int>(threadIdx.x) + 1);
    };
    auto next_tile = [&](int i) {  // the i-th tile has landed; the (i + 3)-th is requested
      put_rinv(i);
      if (i + 2 < n) wait_loads<10>();  // the next two tiles may still be on their way
      else if (i + 1 < n) wait_loads<5>();
      else wait_loads<0>();
      __syncthreads();
      if (i + 3 < n) request(i + 3);
    };
    auto plain_tile = [&](int i) {
      const int t = t_last - i;
      next_tile(i);
      const char* p = ring + (i % NS) * kRingTileBytes;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int ib = t * kTile + sub * 32;
        const bool do0 = ib + 31 >= kg0, do1 = ib + 31 >= kg1;  // some query of the half-tile reaches the keys
        if (!do0) continue;
        f32x16 c0, c1;
        score_tiles_ring(p + sub * (32 * kRowBytes), tr.frag, own0, own1, do0, do1, c0, c1);
        const bool whole = ib + 31 < len;  // no ragged end
        const float* lt = &lse_s[i % kLseStages][wave][sub * 32];
        const float* rt = &rinv_s[COUNT ? i % kLseStages : 0][COUNT ? sub * 32 : 0];
        if (whole && ib >= kg0 + 31 + w) column_update<true, COUNT>(c0, lt, rt, sc, ib, half, kj0, len, w, rb, s1a, s2a);
        else column_update<false, COUNT>(c0, lt, rt, sc, ib, half, kj0, len, w, rb, s1a, s2a);
        if (do1) {
          if (whole && ib >= kg1 + 31 + w) column_update<true, COUNT>(c1, lt, rt, sc, ib, half, kj1, len, w, rb, s1b, s2b);
          else column_update<false, COUNT>(c1, lt, rt, sc, ib, half, kj1, len, w, rb, s1b, s2b);
        }
      }
    };

    int i = 0;
    while (i < n && (t_last - i) * kTile + kTile - 1 >= len) plain_tile(i++);  // the ragged end of the prompt

    // ---- the rectangle: software-pipelined.  A* hold the scores of a tile's first 32 queries, B* of its last 32.
    f32x16 A0, A1, B0, B1;
    bool pending = false;   // B* hold scores that have not been added yet ...
    int pending_i = 0;      // ... of the tile with this index of the walk
    // one step: (x0, x1) are filled from the half-tile at p while (y0, y1), the scores of half `ysub` of walk index
    // `yi`, are turned into probabilities and added to the lane's two keys
    auto step = [&](auto consume_tag, const char* p, f32x16& x0, f32x16& x1, const f32x16& y0, const f32x16& y1, int yi,
                    int ysub) {
      constexpr bool CONSUME = decltype(consume_tag)::value != 0;
      float4 lv[4], rv[4];
      if (CONSUME) {
        const float* lt = &lse_s[yi % kLseStages][wave][ysub * 32 + 4 * half];
        const float* rt = &rinv_s[COUNT ? yi % kLseStages : 0][COUNT ? ysub * 32 + 4 * half : 0];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          lv[g4] = *reinterpret_cast<const float4*>(lt + 8 * g4);
          if (COUNT) rv[g4] = *reinterpret_cast<const float4*>(rt + 8 * g4);
        }
      }
      auto comp = [](const float4& v, int e) { return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w; };
      auto one = [&](float s, float lse_q, float rinv_q, float& sum1, float& sum2) {
        const float pr = fast_exp2(fmaf(s, sc, -lse_q));
        sum1 += pr;
        if (COUNT) sum2 += pr > rinv_q ? 1.0f : 0.0f;  // p * (i + 1) > 1
        else sum2 = fmaf(pr, pr, sum2);
      };
      // The probabilities go straight into the block's running sums, two chains per sum: nothing is zeroed or folded
      // per step (that cost one vector instruction per matrix instruction).
      auto consume = [&](int kk, int g) {
        const int r = 2 * kk;  // scores r and r + 1: queries 8 (r / 4) + 4 half + r % 4 (+ 1) of the half-tile
        const float la = comp(lv[r >> 2], r & 3), lb = comp(lv[r >> 2], (r & 3) + 1);
        const float ra = COUNT ? comp(rv[r >> 2], r & 3) : 0.0f, rbq = COUNT ? comp(rv[r >> 2], (r & 3) + 1) : 0.0f;
        if (g == 0) { one(y0[r], la, ra, s1a, s2a); one(y0[r + 1], lb, rbq, t1a, t2a); }
        else        { one(y1[r], la, ra, s1b, s2b); one(y1[r + 1], lb, rbq, t1b, t2b); }
      };
      auto pin = [&]() {
        asm volatile("" : "+v"(s1a), "+v"(s2a), "+v"(t1a), "+v"(t2a), "+v"(s1b), "+v"(s2b), "+v"(t1b), "+v"(t2b));
      };
      fill_and_consume<CONSUME>(p, tr.frag, own0, own1, x0, x1, consume, pin);
    };
    auto rect_tile = [&](auto stage, int ii) {
      constexpr int S = decltype(stage)::value;
      next_tile(ii);
      const char* p = ring + S * kRingTileBytes;
      if (pending) step(StageTag<1>{}, p, A0, A1, B0, B1, pending_i, 1);
      else step(StageTag<0>{}, p, A0, A1, B0, B1, 0, 0);
      step(StageTag<1>{}, p + 32 * kRowBytes, B0, B1, A0, A1, ii, 0);
      pending = true;
      pending_i = ii;
    };
    auto is_rect = [&](int ii) { return ii < n && t_last - ii >= t_rect_lo; };
    for (int stage = i % NS;;) {  // the ring stage of a tile follows from its index; the code wants it static
      if (stage == 0) { if (!is_rect(i)) break; rect_tile(StageTag<0>{}, i++); stage = 1; }
      if (stage == 1) { if (!is_rect(i)) break; rect_tile(StageTag<1>{}, i++); stage = 2; }
      if (stage == 2) { if (!is_rect(i)) break; rect_tile(StageTag<2>{}, i++); stage = 3; }
      if (stage == 3) { if (!is_rect(i)) break; rect_tile(StageTag<3>{}, i++); stage = 0; }
    }
    s1a += t1a; s2a += t2a;
    s1b += t1b; s2b += t2b;
    if (pending) {  // drain
      const float* lt = &lse_s[pending_i % kLseStages][wave][32];
      const float* rt = &rinv_s[COUNT ? pending_i % kLseStages : 0][COUNT ? 32 : 0];
      const int ib = (t_last - pending_i) * kTile + 32;
      column_update<true, COUNT>(B0, lt, rt, sc, ib, half, kj0, len, w, rb, s1a, s2a);
      column_update<true, COUNT>(B1, lt, rt, sc, ib, half, kj1, len, w, rb, s1b, s2b);
    }
    // ---- the tiles on the diagonal (or inside a recency window)
    if (!COUNT && w == 0 && i < n && n - i <= NS) {  // (the counting variant has no registers to spare for it)
      // No window and at most four tiles left (the queries at the block's own 256 positions): they all fit in the
      // ring, so the waves need not meet after every tile; see the same stretch of prefill_rows_mfma.  Half-tiles
      // are taken from the highest query position down; those that only the early group of keys still reaches are
      // taken two at a time.  The walk's tiles i .. i + 2 have been requested; the fourth is requested here and
      // waited for once, after the first tile's work.
      const int i0 = i;
      put_rinv(i0);
      if (i0 + 1 < n) put_rinv(i0 + 1);
      if (i0 + 2 < n) put_rinv(i0 + 2);
      wait_loads<0>();
      __syncthreads();  // tiles i0 .. i0 + 2 are in LDS; everybody is done with the stage the fourth tile takes
      if (i0 + 3 < n) {
        request(i0 + 3);
        put_rinv(i0 + 3);
      }
      const int n_half = 2 * (n - i0);
      const int ib_top = (t_last - i0) * kTile + 32;  // half-tile h holds the queries from ib_top - 32 h on
      auto tile_ptr = [&](int h) { return ring + ((i0 + (h >> 1)) % NS) * kRingTileBytes + (1 - (h & 1)) * (32 * kRowBytes); };
      auto update = [&](const f32x16& c, int h, int kg, int kj, float& s1, float& s2) {
        const int ib = ib_top - 32 * h;
        const int st = (i0 + (h >> 1)) % kLseStages, off = (1 - (h & 1)) * 32;
        const float* lt = &lse_s[st][wave][off];
        const float* rt = &rinv_s[COUNT ? st : 0][COUNT ? off : 0];
        if (ib + 31 < len && ib >= kg + 31) column_update<true, COUNT>(c, lt, rt, sc, ib, half, kj, len, w, rb, s1, s2);
        else column_update<false, COUNT>(c, lt, rt, sc, ib, half, kj, len, w, rb, s1, s2);
      };
      auto run = [&](int h, int h_end) {
        while (h < h_end) {
          const int ib = ib_top - 32 * h;
          if (ib + 31 < kg0) break;  // no query of this half-tile, or of any later one, reaches the wave's keys
          f32x16 c0, c1;
          if (ib + 31 >= kg1) {  // both groups: one fragment, two chains
            score_tiles_ring(tile_ptr(h), tr.frag, own0, own1, true, true, c0, c1);
            update(c0, h, kg0, kj0, s1a, s2a);
            update(c1, h, kg1, kj1, s1b, s2b);
            h += 1;
          } else if (h + 1 < h_end && ib - 1 >= kg0) {  // the early group alone, two half-tiles at once
            score_two_subs_ring(tile_ptr(h), tile_ptr(h + 1), tr.frag, own0, c0, c1);
            update(c0, h, kg0, kj0, s1a, s2a);
            update(c1, h + 1, kg0, kj0, s1a, s2a);
            h += 2;
          } else {
            score_tiles_ring(tile_ptr(h), tr.frag, own0, own1, true, false, c0, c1);
            update(c0, h, kg0, kj0, s1a, s2a);
            h += 1;
          }
        }
      };
      run(0, min(2, n_half));
      if (n_half > 6) {
        wait_loads<0>();
        __syncthreads();  // the fourth tile is in LDS
      }
      run(2, n_half);
      i = n;
    }
    while (i < n) plain_tile(i++);

    s1a += __shfl_xor(s1a, 32, kWave);
    s2a += __shfl_xor(s2a, 32, kWave);
    s1b += __shfl_xor(s1b, 32, kWave);
    s2b += __shfl_xor(s2b, 32, kWave);
    if (half == 0 && kj0 < len) { out1[ubase + kj0] = s1a; out2[ubase + kj0] = s2a; }
    if (half == 0 && kj1 < len) { out1[ubase + kj1] = s1b; out2[ubase + kj1] = s2b; }
  }
}

// ------------------------------------------------------------------------------------------------
// pass 2 for grouped-query attention (section 5.3): the unit's keys are shared by g query heads and the statistics
// are taken on the head-mean probability, Acc[j] = sum_i Pbar[i,j], Acc2[j] = sum_i Pbar[i,j]^2 with
// Pbar = mean_h P_h.  Same shape as prefill_columns_mfma, but the streamed tile holds one block of 32 queries for
// two heads (rows 0-31: head 2k, rows 32-63: head 2k+1), so that the sum over the heads of a probability stays in
// the lane's registers between tiles; after the last pair of heads it is scaled, added and squared.
template <int WAVES>
__device__ __forceinline__ void tile_load_two(Staged<WAVES>& s, const char* base0, const char* base1, int row0,
                                              int last_row) {
  const int t = threadIdx.x;
  constexpr int kHalf = Shape<WAVES>::kChunks / 2;
#pragma unroll
  for (int i = 0; i < Shape<WAVES>::kChunks; ++i) {
    int row = row0 + (t >> 4) + Shape<WAVES>::kRowsPerSweep * (i % kHalf);
    row = row < last_row ? row : last_row;  // rows past the end are masked by the caller
    s.w[i] = load16((i < kHalf ? base0 : base1) + static_cast<size_t>(row) * kRowBytes + (t & 15) * 16);
  }
}

// The 16 probabilities of a tile (one key, 16 queries of one head) added into `pb` (cleared before the first head).
template <bool INTERIOR>
__device__ __forceinline__ void column_probs(const f32x16& s, const float* lse_tile, float sc, int ib, int half,
                                             int kj, int len, int w, float rb, f32x16& pb) {
  if (!INTERIOR) {
    // The masks of this (rare) path depend only on values known before the branch that leads here; the compiler
    // would compute all of them ahead of that branch, on every tile.  An opaque copy of the block index keeps them here.
    asm volatile("" : "+s"(ib));
  }
#pragma unroll
  for (int g4 = 0; g4 < 4; ++g4) {
    const float4 ls = *reinterpret_cast<const float4*>(lse_tile + 8 * g4 + 4 * half);
    const float lv[4] = {ls.x, ls.y, ls.z, ls.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x = fmaf(s[4 * g4 + e], sc, -lv[e]);
      float p;
      if (INTERIOR) {
        p = fast_exp2(x);
      } else {
        const int qi = ib + 8 * g4 + 4 * half + e;
        if (w > 0 && qi - kj < w) x += rb;
        p = fast_exp2(x);
        if (qi < kj || qi >= len) p = 0.0f;
      }
      pb[4 * g4 + e] += p;
    }
  }
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void prefill_columns_gqa_mfma(PrefillArgs a) {
  constexpr int kOwn = Shape<WAVES>::kOwn;
  static_assert(Shape<WAVES>::kChunks % 2 == 0, "half a staged tile per head");
  __shared__ __attribute__((aligned(16))) char lds[2][kTile * kLdsRow];
  __shared__ __attribute__((aligned(16))) float lse_s[2][kTile];
  int u, id;
  if (!locate(a.units, a.pairs * a.qsplit, u, id)) return;
  const int seg = id % a.qsplit, pair_id = id / a.qsplit;  // which share of the queries, which blocks of keys
  float* const out1 = seg == 0 ? a.acc : reinterpret_cast<float*>(a.var_key);    // second share: see sum_query_shares
  float* const out2 = seg == 0 ? a.acc2 : reinterpret_cast<float*>(a.mas_key);
  const int G = a.group, HP = (G + 1) / 2;  // head pairs per block of 32 queries
  const float inv_heads = 1.0f / static_cast<float>(G);
  const int len = a.len[u];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int half = lane >> 5;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Kb = static_cast<const char*>(a.K) + ubase * kRowBytes;
  auto q_of = [&](int h) { return static_cast<const char*>(a.Q) + (static_cast<size_t>(u) * G + h) * a.L_max * kRowBytes; };
  auto lse_of = [&](int h) { return a.lse + (static_cast<size_t>(u) * G + h) * a.L_max; };
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const int n_blocks = (len + kOwn - 1) / kOwn;
  if (a.paired ? 2 * pair_id > n_blocks - 1 : pair_id >= n_blocks) return;  // nothing left for this id

  for (int pass = 0; pass < 2; ++pass) {  // one long and one short block of keys per workgroup
    int blk;
    if (a.paired) {
      blk = pass == 0 ? pair_id : n_blocks - 1 - pair_id;
      if (blk < pair_id || (pass == 1 && blk == pair_id)) break;
    } else {
      if (pass == 1) break;
      blk = pair_id;  // the longest streams start first
    }
    const int j0 = blk * kOwn;
    const int kw0 = j0 + 64 * wave;
    const int kj0 = kw0 + (lane & 31), kj1 = kj0 + 32;  // this lane's two keys
    uint4 own0[kKSteps], own1[kKSteps];
    load_owned(own0, Kb, kj0, len - 1);
    load_owned(own1, Kb, kj1, len - 1);
    float s1a = 0.0f, s2a = 0.0f, s1b = 0.0f, s2b = 0.0f;
    f32x16 pb0 = {0}, pb1 = {0};  // sums over the heads, for this lane's two keys

    int r_first = j0 / 32;         // first block of 32 queries with a query >= j0
    int r_last = (len - 1) / 32;
    if (a.qsplit > 1) {  // this workgroup's share of those blocks (possibly none)
      const int per = (r_last - r_first + a.qsplit) / a.qsplit;
      r_first += seg * per;
      r_last = min(r_last, r_first + per - 1);
    }
    const int n_it = max(0, r_last - r_first + 1) * HP;
    Staged<WAVES> stA;
    float lseA = 0.0f;
    auto fetch = [&](Staged<WAVES>& st, float& lse_st, int it) {
      const int r = r_first + it / HP, hp = it % HP;
      const int h0 = 2 * hp, h1 = min(2 * hp + 1, G - 1);  // an odd group repeats its last head; that half is skipped
      tile_load_two<WAVES>(st, q_of(h0), q_of(h1), r * 32, len - 1);
      if (threadIdx.x < kTile) {
        const int t = threadIdx.x;
        lse_st = lse_of(t < 32 ? h0 : h1)[min(r * 32 + (t & 31), len - 1)];
      }
    };
    if (n_it > 0) fetch(stA, lseA, 0);
    __syncthreads();  // the previous pass has finished with the LDS buffers
    for (int it = 0; it < n_it; ++it) {
      const int b = it & 1;
      tile_store(stA, lds[b]);
      if (threadIdx.x < kTile) lse_s[b][threadIdx.x] = lseA;
      __syncthreads();
      if (it + 1 < n_it) fetch(stA, lseA, it + 1);
      const int r = r_first + it / HP, hp = it % HP;
      const int ib = r * 32;
      const bool do0 = ib + 31 >= kw0, do1 = ib + 31 >= kw0 + 32;  // some query of the block reaches the keys
      if (!do0) continue;  // wave-uniform, and the same for every head of the block
      const bool whole = ib + 31 < len;  // no ragged end
      if (hp == 0) {  // a new block of queries: the sums over the heads start from zero
        pb0 = f32x16{0};
        pb1 = f32x16{0};
      }
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int h = 2 * hp + sub;
        if (h >= G) break;
        f32x16 c0, c1;
        score_tiles(lds[b], sub, own0, own1, do0, do1, c0, c1);
        const float* lt = &lse_s[b][sub * 32];
        if (whole && ib >= kw0 + 31 + w) column_probs<true>(c0, lt, sc, ib, half, kj0, len, w, rb, pb0);
        else column_probs<false>(c0, lt, sc, ib, half, kj0, len, w, rb, pb0);
        if (do1) {
          if (whole && ib >= kw0 + 63 + w) column_probs<true>(c1, lt, sc, ib, half, kj1, len, w, rb, pb1);
          else column_probs<false>(c1, lt, sc, ib, half, kj1, len, w, rb, pb1);
        }
      }
      if (hp == HP - 1) {  // every head of this block of queries has been added
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = pb0[e] * inv_heads;
          s1a += p;
          s2a = a.pol.second_statistic(s2a, p, static_cast<float>(ib + 8 * (e >> 2) + 4 * half + (e & 3) + 1));
        }
        if (do1) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const float p = pb1[e] * inv_heads;
            s1b += p;
            s2b = a.pol.second_statistic(s2b, p, static_cast<float>(ib + 8 * (e >> 2) + 4 * half + (e & 3) + 1));
          }
        }
      }
    }
    s1a += __shfl_xor(s1a, 32, kWave);
    s2a += __shfl_xor(s2a, 32, kWave);
    s1b += __shfl_xor(s1b, 32, kWave);
    s2b += __shfl_xor(s2b, 32, kWave);
    if (half == 0 && kj0 < len) { out1[ubase + kj0] = s1a; out2[ubase + kj0] = s2a; }
    if (half == 0 && kj1 < len) { out1[ubase + kj1] = s1b; out2[ubase + kj1] = s2b; }
  }
}

// ------------------------------------------------------------------------------------------------
// pass 2 for grouped-query attention when the number of heads divides 16 (2, 4, 8, 16): the streamed tile holds
// 64 / G query positions for all G heads, its rows ordered so that the G heads of a query land in G consecutive
// accumulator registers of a lane (register r of lane half hf holds row 8 * (r / 4) + 4 * hf + r % 4 of a 32-row
// sub-tile; that row is given to query hf * 16 / G + r / G of the sub-tile, head r % G).  The sum over the heads is
// then a sum down a few registers of one result tile: nothing is carried from tile to tile, and the kernel keeps the
// register budget -- three waves per SIMD -- of the ungrouped column pass.
template <int G> struct GroupedRows {
  static constexpr int kPerHalf = 16 / G;      // queries per lane half in a 32-row sub-tile
  static constexpr int kPerSub = 32 / G;       // query positions per sub-tile
  static constexpr int kPerTile = 64 / G;      // query positions per 64-row tile
  // LDS row of a tile -> local query position and head
  __device__ static void locate(int row, int& ql, int& h) {
    const int sub = row >> 5, rr = row & 31;
    const int hf = (rr >> 2) & 1, r = 4 * (rr >> 3) + (rr & 3);
    ql = sub * kPerSub + hf * kPerHalf + r / G;
    h = r % G;
  }
};

template <bool INTERIOR, int G>
__device__ __forceinline__ void column_update_grouped(const f32x16& s, const float* lse_tile, float sc, int ib, int half,
                                                      int kj, int len, int w, float rb, const Policy& pol,
                                                      float& s1, float& s2) {
  if (!INTERIOR) asm volatile("" : "+s"(ib));  // keeps this path's masks out of the code before the branch (see column_probs)
  constexpr int kPerHalf = GroupedRows<G>::kPerHalf;
  float p[16];
#pragma unroll
  for (int g4 = 0; g4 < 4; ++g4) {
    const float4 ls = *reinterpret_cast<const float4*>(lse_tile + 8 * g4 + 4 * half);
    const float lv[4] = {ls.x, ls.y, ls.z, ls.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int r = 4 * g4 + e;
      float x = fmaf(s[r], sc, -lv[e]);
      if (INTERIOR) {
        p[r] = fast_exp2(x);
      } else {
        const int qi = ib + half * kPerHalf + r / G;
        if (w > 0 && qi - kj < w) x += rb;
        p[r] = (qi < kj || qi >= len) ? 0.0f : fast_exp2(x);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < kPerHalf; ++q) {
    float sum = p[q * G];
#pragma unroll
    for (int h = 1; h < G; ++h) sum += p[q * G + h];
    const float pbar = sum * (1.0f / static_cast<float>(G));
    s1 += pbar;
    s2 = pol.second_statistic(s2, pbar, static_cast<float>(ib + half * kPerHalf + q + 1));
  }
}

template <int WAVES, int G>
__global__ __launch_bounds__(WAVES * kWave) void prefill_columns_gqa_pow2_mfma(PrefillArgs a) {
  using GR = GroupedRows<G>;
  constexpr int kOwn = Shape<WAVES>::kOwn;
  constexpr int QT = GR::kPerTile, QS = GR::kPerSub;
  __shared__ __attribute__((aligned(16))) char lds[2][kTile * kLdsRow];
  __shared__ __attribute__((aligned(16))) float lse_s[2][kTile];
  int u, id;
  if (!locate(a.units, a.pairs * a.qsplit, u, id)) return;
  const int seg = id % a.qsplit, pair_id = id / a.qsplit;  // which share of the queries, which blocks of keys
  float* const out1 = seg == 0 ? a.acc : reinterpret_cast<float*>(a.var_key);    // second share: see sum_query_shares
  float* const out2 = seg == 0 ? a.acc2 : reinterpret_cast<float*>(a.mas_key);
  const int len = a.len[u];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int half = lane >> 5;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Kb = static_cast<const char*>(a.K) + ubase * kRowBytes;
  const char* Qu = static_cast<const char*>(a.Q) + static_cast<size_t>(u) * G * a.L_max * kRowBytes;  // [G][L_max][d]
  const float* lse_u = a.lse + static_cast<size_t>(u) * G * a.L_max;
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const int n_blocks = (len + kOwn - 1) / kOwn;
  if (a.paired ? 2 * pair_id > n_blocks - 1 : pair_id >= n_blocks) return;  // nothing left for this id
  // this thread's rows of a staged tile: local query position and head, fixed for the whole kernel
  int row_q[Shape<WAVES>::kChunks], row_h[Shape<WAVES>::kChunks];
#pragma unroll
  for (int i = 0; i < Shape<WAVES>::kChunks; ++i)
    GR::locate((threadIdx.x >> 4) + Shape<WAVES>::kRowsPerSweep * i, row_q[i], row_h[i]);
  int lse_q = 0, lse_h = 0;
  if (threadIdx.x < kTile) GR::locate(threadIdx.x, lse_q, lse_h);

  for (int pass = 0; pass < 2; ++pass) {  // one long and one short block of keys per workgroup
    int blk;
    if (a.paired) {
      blk = pass == 0 ? pair_id : n_blocks - 1 - pair_id;
      if (blk < pair_id || (pass == 1 && blk == pair_id)) break;
    } else {
      if (pass == 1) break;
      blk = pair_id;  // the longest streams start first
    }
    const int j0 = blk * kOwn;
    const int kw0 = j0 + 64 * wave;
    const int kj0 = kw0 + (lane & 31), kj1 = kj0 + 32;  // this lane's two keys
    uint4 own0[kKSteps], own1[kKSteps];
    load_owned(own0, Kb, kj0, len - 1);
    load_owned(own1, Kb, kj1, len - 1);
    float s1a = 0.0f, s2a = 0.0f, s1b = 0.0f, s2b = 0.0f;

    int t_first = j0 / QT;  // first tile with a query >= j0
    int t_last = (len - 1) / QT;
    if (a.qsplit > 1) {  // this workgroup's share of those tiles (possibly none)
      const int per = (t_last - t_first + a.qsplit) / a.qsplit;
      t_first += seg * per;
      t_last = min(t_last, t_first + per - 1);
    }
    Staged<WAVES> stA;
    float lseA = 0.0f;
    auto fetch = [&](Staged<WAVES>& st, float& lse_st, int t) {
#pragma unroll
      for (int i = 0; i < Shape<WAVES>::kChunks; ++i) {
        const int qpos = min(t * QT + row_q[i], len - 1);  // positions past the end are masked by the update
        st.w[i] = load16(Qu + (static_cast<size_t>(row_h[i]) * a.L_max + qpos) * kRowBytes + (threadIdx.x & 15) * 16);
      }
      if (threadIdx.x < kTile) lse_st = lse_u[static_cast<size_t>(lse_h) * a.L_max + min(t * QT + lse_q, len - 1)];
    };
    if (t_first <= t_last) fetch(stA, lseA, t_first);
    __syncthreads();  // the previous pass has finished with the LDS buffers
    for (int t = t_first; t <= t_last; ++t) {
      const int b = (t - t_first) & 1;
      tile_store(stA, lds[b]);
      if (threadIdx.x < kTile) lse_s[b][threadIdx.x] = lseA;
      __syncthreads();
      if (t + 1 <= t_last) fetch(stA, lseA, t + 1);
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int ib = t * QT + sub * QS;  // first query position of the sub-tile; its last one is ib + QS - 1
        const bool do0 = ib + QS - 1 >= kw0, do1 = ib + QS - 1 >= kw0 + 32;  // some query reaches the keys
        if (!do0) continue;
        f32x16 c0, c1;
        score_tiles(lds[b], sub, own0, own1, do0, do1, c0, c1);
        const bool whole = ib + QS - 1 < len;  // no ragged end
        const float* lt = &lse_s[b][sub * 32];
        if (whole && ib >= kw0 + 31 + w) column_update_grouped<true, G>(c0, lt, sc, ib, half, kj0, len, w, rb, a.pol, s1a, s2a);
        else column_update_grouped<false, G>(c0, lt, sc, ib, half, kj0, len, w, rb, a.pol, s1a, s2a);
        if (do1) {
          if (whole && ib >= kw0 + 63 + w) column_update_grouped<true, G>(c1, lt, sc, ib, half, kj1, len, w, rb, a.pol, s1b, s2b);
          else column_update_grouped<false, G>(c1, lt, sc, ib, half, kj1, len, w, rb, a.pol, s1b, s2b);
        }
      }
    }
    s1a += __shfl_xor(s1a, 32, kWave);
    s2a += __shfl_xor(s2a, 32, kWave);
    s1b += __shfl_xor(s1b, 32, kWave);
    s2b += __shfl_xor(s2b, 32, kWave);
    if (half == 0 && kj0 < len) { out1[ubase + kj0] = s1a; out2[ubase + kj0] = s2a; }
    if (half == 0 && kj1 < len) { out1[ubase + kj1] = s1b; out2[ubase + kj1] = s2b; }
  }
}

// The grouped column pass on the tile ring, for G = 2, 4, 8, 16 heads and the sum-of-squares second statistic: the
// shape of prefill_columns_mfma (keys owned in groups w and 7 - w, query tiles walked downwards through a four-stage
// ring filled by loads that go straight to LDS, the rectangle software-pipelined on four accumulators) with the tile
// composition of prefill_columns_gqa_pow2_mfma (64 / G query positions for all G heads, the heads of a position in G
// consecutive accumulator registers of a lane).  Which (head, position) a tile row holds is a constant of the lane
// that loads it, so the gather over the G query arrays costs nothing: it is the lane's buffer offset.  In the
// rectangle the head sum of a position is carried over the G / 2 slices of the pipelined step that hold its heads.
// The tiles near the diagonal and the ragged end of the prompt take the plain form, one barrier per tile.
template <int G>
__global__ __launch_bounds__(256, 2) void prefill_columns_gqa_ring(PrefillArgs a) {
  using GR = GroupedRows<G>;
  constexpr int kOwn = Shape<4>::kOwn;
  constexpr int QT = GR::kPerTile, QS = GR::kPerSub;
  constexpr int NS = 4;          // ring stages
  constexpr int kLseStages = 8;  // see prefill_columns_mfma
  static_assert(G == 2 || G == 4 || G == 8 || G == 16, "the heads of a position fill whole pairs of registers");
  __shared__ __attribute__((aligned(1024))) char ring[NS * kRingTileBytes];
  __shared__ __attribute__((aligned(256))) float lse_s[kLseStages][4][kTile];  // [stage][wave][row of the tile]
  int u, id;
  if (!locate(a.units, a.pairs * a.qsplit, u, id)) return;
  const int seg = id % a.qsplit, pair_id = id / a.qsplit;
  float* const out1 = seg == 0 ? a.acc : reinterpret_cast<float*>(a.var_key);    // second share: see sum_query_shares
  float* const out2 = seg == 0 ? a.acc2 : reinterpret_cast<float*>(a.mas_key);
  const int len = a.len[u];
  const int lane = threadIdx.x & (kWave - 1);
  const int half = lane >> 5;
  TileRing tr;
  tr.init();
  const int wave = tr.wave;
  const uint32_t ring_addr = lds_address(ring);
  const uint32_t lse_addr = lds_address(&lse_s[0][wave][0]);
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Kb = static_cast<const char*>(a.K) + ubase * kRowBytes;
  const char* Qu = static_cast<const char*>(a.Q) + static_cast<size_t>(u) * G * a.L_max * kRowBytes;  // [G][L_max][d]
  // (the launcher checks that G * L_max rows fit a 32-bit byte offset; rows past a head's prompt are masked below)
  const v4i32 qbuf = make_buffer(Qu, static_cast<uint32_t>(G) * static_cast<uint32_t>(a.L_max) * kRowBytes);
  const v4i32 lbuf = make_buffer(a.lse + static_cast<size_t>(u) * G * a.L_max,
                                 static_cast<uint32_t>(G) * static_cast<uint32_t>(a.L_max) * 4u);
  // this lane's four rows of a tile and its row of the normalisers: head and local position are fixed
  int qoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 16 * wave + 4 * i + (lane >> 4);
    int ql, h;
    GR::locate(r, ql, h);
    qoff[i] = (h * a.L_max + ql) * kRowBytes + (((lane & 15) ^ (r & 15)) << 4);
  }
  int loff;
  {
    int ql, h;
    GR::locate(lane, ql, h);
    loff = (h * a.L_max + ql) * 4;
  }
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;
  const int n_blocks = (len + kOwn - 1) / kOwn;
  if (a.paired ? 2 * pair_id > n_blocks - 1 : pair_id >= n_blocks) return;  // nothing left for this id

  for (int pass = 0; pass < 2; ++pass) {  // one long and one short block of keys per workgroup, the long one first
    int blk;
    if (a.paired) {
      blk = pass == 0 ? pair_id : n_blocks - 1 - pair_id;
      if (blk < pair_id || (pass == 1 && blk == pair_id)) break;
    } else {
      if (pass == 1) break;
      blk = pair_id;
    }
    const int j0 = blk * kOwn;
    const int kg0 = j0 + 32 * wave, kg1 = j0 + 32 * (7 - wave);  // first key of this wave's two groups (kg0 < kg1)
    const int kj0 = kg0 + (lane & 31), kj1 = kg1 + (lane & 31);
    int t_first = j0 / QT;  // first tile with a query position >= j0
    int t_last = (len - 1) / QT;
    if (a.qsplit > 1) {
      const int per = (t_last - t_first + a.qsplit) / a.qsplit;
      t_first += seg * per;
      t_last = min(t_last, t_first + per - 1);
    }
    const int n = t_last - t_first + 1;  // the i-th tile of the walk is t_last - i
    // tiles from t_rect_lo on lie past every key of the block and outside every recency window
    const int t_rect_lo = (j0 + kOwn - 1 + w + QT - 1) / QT;
    auto request = [&](int i) {  // five loads per wave
      const int t = t_last - i;
      const uint32_t dst = ring_addr + (i % NS) * kRingTileBytes + wave * 4096;
      const int soff = __builtin_amdgcn_readfirstlane(t * QT * kRowBytes);
#pragma unroll
      for (int k = 0; k < 4; ++k) load16_to_lds(qbuf, dst + k * 1024, qoff[k], soff);
      load4_to_lds(lbuf, lse_addr + (i % kLseStages) * (4 * kTile * 4), loff, __builtin_amdgcn_readfirstlane(t * QT * 4));
    };
    __syncthreads();  // the previous block has finished with the ring
    if (0 < n) request(0);
    if (1 < n) request(1);
    if (2 < n) request(2);
    uint4 own0[kKSteps], own1[kKSteps];
    load_owned(own0, Kb, kj0, len - 1);
    load_owned(own1, Kb, kj1, len - 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the owned rows are in before the loop
    float s1a = 0.0f, s2a = 0.0f, s1b = 0.0f, s2b = 0.0f;
    float ha = 0.0f, hc = 0.0f;  // rectangle: head sum of the position under way, per key group

    auto next_tile = [&](int i) {  // the i-th tile has landed; the (i + 3)-th is requested
      if (i + 2 < n) wait_loads<10>();
      else if (i + 1 < n) wait_loads<5>();
      else wait_loads<0>();
      __syncthreads();
      if (i + 3 < n) request(i + 3);
    };
    auto plain_tile = [&](int i) {
      const int t = t_last - i;
      next_tile(i);
      const char* p = ring + (i % NS) * kRingTileBytes;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int ib = t * QT + sub * QS;  // first query position of the sub-tile; its last one is ib + QS - 1
        const bool do0 = ib + QS - 1 >= kg0, do1 = ib + QS - 1 >= kg1;  // some query reaches the keys
        if (!do0) continue;
        f32x16 c0, c1;
        score_tiles_ring(p + sub * (32 * kRowBytes), tr.frag, own0, own1, do0, do1, c0, c1);
        const bool whole = ib + QS - 1 < len;  // no ragged end
        const float* lt = &lse_s[i % kLseStages][wave][sub * 32];
        if (whole && ib >= kg0 + 31 + w) column_update_grouped<true, G>(c0, lt, sc, ib, half, kj0, len, w, rb, a.pol, s1a, s2a);
        else column_update_grouped<false, G>(c0, lt, sc, ib, half, kj0, len, w, rb, a.pol, s1a, s2a);
        if (do1) {
          if (whole && ib >= kg1 + 31 + w) column_update_grouped<true, G>(c1, lt, sc, ib, half, kj1, len, w, rb, a.pol, s1b, s2b);
          else column_update_grouped<false, G>(c1, lt, sc, ib, half, kj1, len, w, rb, a.pol, s1b, s2b);
        }
      }
    };

    int i = 0;
    while (i < n && (t_last - i) * QT + QT - 1 >= len) plain_tile(i++);  // the ragged end of the prompt

    // ---- the rectangle: software-pipelined.  A* hold the scores of a tile's first 32 rows, B* of its last 32.
    f32x16 A0, A1, B0, B1;
    bool pending = false;
    int pending_i = 0;
    constexpr float kInvG = 1.0f / static_cast<float>(G);
    auto step = [&](auto consume_tag, const char* p, f32x16& x0, f32x16& x1, const f32x16& y0, const f32x16& y1, int yi,
                    int ysub) {
      constexpr bool CONSUME = decltype(consume_tag)::value != 0;
      float4 lv[4];
      if (CONSUME) {
        const float* lt = &lse_s[yi % kLseStages][wave][ysub * 32 + 4 * half];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) lv[g4] = *reinterpret_cast<const float4*>(lt + 8 * g4);
      }
      // The head-means go straight into the block's running sums: nothing is zeroed or folded per step.
      auto comp = [](const float4& v, int e) { return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w; };
      auto consume = [&](int kk, int g) {
        const int r = 2 * kk;  // registers r and r + 1: two heads of one position (G consecutive registers each)
        const f32x16& y = g == 0 ? y0 : y1;
        float& hs = g == 0 ? ha : hc;
        float& sum1 = g == 0 ? s1a : s1b;
        float& sum2 = g == 0 ? s2a : s2b;
        const float pa = fast_exp2(fmaf(y[r], sc, -comp(lv[r >> 2], r & 3)));
        const float pb = fast_exp2(fmaf(y[r + 1], sc, -comp(lv[r >> 2], (r & 3) + 1)));
        if (r % G == 0) hs = pa + pb;
        else hs += pa + pb;
        if ((r + 2) % G == 0) {  // the position's last two heads
          const float pbar = hs * kInvG;
          sum1 += pbar;
          sum2 = fmaf(pbar, pbar, sum2);
        }
      };
      auto pin = [&]() { asm volatile("" : "+v"(s1a), "+v"(s2a), "+v"(s1b), "+v"(s2b), "+v"(ha), "+v"(hc)); };
      fill_and_consume<CONSUME>(p, tr.frag, own0, own1, x0, x1, consume, pin);
    };
    auto rect_tile = [&](auto stage, int ii) {
      constexpr int S = decltype(stage)::value;
      next_tile(ii);
      const char* p = ring + S * kRingTileBytes;
      if (pending) step(StageTag<1>{}, p, A0, A1, B0, B1, pending_i, 1);
      else step(StageTag<0>{}, p, A0, A1, B0, B1, 0, 0);
      step(StageTag<1>{}, p + 32 * kRowBytes, B0, B1, A0, A1, ii, 0);
      pending = true;
      pending_i = ii;
    };
    auto is_rect = [&](int ii) { return ii < n && t_last - ii >= t_rect_lo; };
    for (int stage = i % NS;;) {
      if (stage == 0) { if (!is_rect(i)) break; rect_tile(StageTag<0>{}, i++); stage = 1; }
      if (stage == 1) { if (!is_rect(i)) break; rect_tile(StageTag<1>{}, i++); stage = 2; }
      if (stage == 2) { if (!is_rect(i)) break; rect_tile(StageTag<2>{}, i++); stage = 3; }
      if (stage == 3) { if (!is_rect(i)) break; rect_tile(StageTag<3>{}, i++); stage = 0; }
    }
    if (pending) {  // drain: the last 32 rows of the last rectangle tile
      const float* lt = &lse_s[pending_i % kLseStages][wave][32];
      const int ib = (t_last - pending_i) * QT + QS;
      column_update_grouped<true, G>(B0, lt, sc, ib, half, kj0, len, w, rb, a.pol, s1a, s2a);
      column_update_grouped<true, G>(B1, lt, sc, ib, half, kj1, len, w, rb, a.pol, s1b, s2b);
    }
    // ---- the tiles near the diagonal (or inside a recency window)
    while (i < n) plain_tile(i++);

    s1a += __shfl_xor(s1a, 32, kWave);
    s2a += __shfl_xor(s2a, 32, kWave);
    s1b += __shfl_xor(s1b, 32, kWave);
    s2b += __shfl_xor(s2b, 32, kWave);
    if (half == 0 && kj0 < len) { out1[ubase + kj0] = s1a; out2[ubase + kj0] = s2a; }
    if (half == 0 && kj1 < len) { out1[ubase + kj1] = s1b; out2[ubase + kj1] = s2b; }
  }
}

// Row pass with few units: the keys of every block of queries are shared by two workgroups (PrefillArgs::ksplit = 2);
// the second one leaves its log-sum-exp in the plane the column pass will overwrite later, and this kernel merges
// the two: log2(2^a + 2^b).
__global__ __launch_bounds__(256) void merge_key_shares(PrefillArgs a) {
  const int u = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= a.len[u]) return;
  const size_t at = static_cast<size_t>(u) * a.L_max + i;
  const float x = a.lse[at], y = a.acc[at];
  const float top = fmaxf(x, y);
  if (top > -INFINITY) a.lse[at] = top + log2f(fast_exp2(x - top) + fast_exp2(y - top));
}

// With few units the queries of every block of keys are shared by two workgroups (PrefillArgs::qsplit = 2), so that
// the chip has enough of them; the second one leaves its sums in the planes that the selection will later use for
// its ranking keys, and this kernel adds them to the first one's: a fixed order, the same bits every run.
__global__ __launch_bounds__(256) void sum_query_shares(PrefillArgs a) {
  const int u = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= a.len[u]) return;
  const size_t i = static_cast<size_t>(u) * a.L_max + j;
  a.acc[i] += reinterpret_cast<const float*>(a.var_key)[i];
  a.acc2[i] += reinterpret_cast<const float*>(a.mas_key)[i];
}

// ------------------------------------------------------------------------------------------------
// pass 1 with the attention output:  O_i = sum_j P[i,j] v_j  next to lse[i]            (section 2.1, eq. 1)
//
// Same orientation as prefill_rows_mfma (score tile = K . Q^T, the query in the lane), one group of 32 queries
// per wave.  The probabilities of a 32-key half-tile, rounded to bf16, are already laid out as a B operand
// (column = query = lane, the tile's keys down the registers), so O^T = V^T . P^T needs V^T as the A operand:
// row = head dimension, 8 keys per lane.  V sits row-major in LDS like K; the gfx950 LDS transpose read hands
// each lane of a 16-lane group one column of a 4-row x 16-column block, i.e. 4 consecutive keys of one head
// dimension, and two such reads make the A fragment.  (Checked on the device: with lane i of a group pointing
// at row i/4, column 4*(i%4) of the block, lane i receives rows 0..3 of column i.)  The k-slot order of both
// operands follows the accumulator layout of the score tile: slots 0-3 are keys 4h..4h+3 and slots 4-7 are keys
// 8+4h..8+4h+3 of a 16-key step, h = lane / 32.

template <int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void prefill_rows_out_mfma(PrefillArgs a) {
  constexpr int kOwnQ = 32 * WAVES;  // one group of 32 queries per wave
  extern __shared__ __attribute__((aligned(16))) char lds_dyn[];  // K[2] then V[2] tiles
  int u, blk_id;
  if (!locate_heads(a.units, a.group, a.pairs, u, blk_id)) return;  // u counts (unit, query head) pairs
  const int uk = u / a.group;  // the unit: its keys, values and length
  const int len = a.len[uk];
  const int n_blocks = (len + kOwnQ - 1) / kOwnQ;
  if (blk_id >= n_blocks) return;
  const int blk = n_blocks - 1 - blk_id;  // long rows first
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int half = lane >> 5;
  const size_t ubase = static_cast<size_t>(u) * a.L_max;
  const char* Qb = static_cast<const char*>(a.Q) + ubase * kRowBytes;
  const char* Kb = static_cast<const char*>(a.K) + static_cast<size_t>(uk) * a.L_max * kRowBytes;
  const char* Vb = static_cast<const char*>(a.V) + static_cast<size_t>(uk) * a.L_max * kRowBytes;
  const float sc = a.scale_log2;
  const int w = a.recency_window;
  const float rb = a.recency_bias_log2;

  const int q0 = blk * kOwnQ;
  const int qw0 = q0 + 32 * wave;
  const int qi = qw0 + (lane & 31);
  uint4 own[kKSteps];
  load_owned(own, Qb, qi, len - 1);
  float m = -INFINITY, l = 0.0f;
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) o[db] = f32x16{0};

  const int tr_off = transposed_fragment_offset();

  const int last_key = min(len, q0 + kOwnQ) - 1;
  const int n_tiles = last_key / kTile + 1;
  Staged<WAVES> stK, stV;
  tile_load(stK, Kb, 0, len - 1);
  tile_load(stV, Vb, 0, len - 1);
  for (int t = 0; t < n_tiles; ++t) {
    char* const tileK = lds_dyn + (t & 1) * kTileBytes;
    char* const tileV = lds_dyn + 2 * kTileBytes + (t & 1) * kTileBytesV;
    tile_store(stK, tileK);
    tile_store<WAVES, kLdsRowV>(stV, tileV);
    __syncthreads();
    if (t + 1 < n_tiles) {
      tile_load(stK, Kb, (t + 1) * kTile, len - 1);
      tile_load(stV, Vb, (t + 1) * kTile, len - 1);
    }
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = t * kTile + sub * 32;
      if (kb > qw0 + 31) continue;  // wholly above the diagonal for every query of this wave
      // ---- scores of 32 keys x 32 queries
      f32x16 sacc;
      {
        const char* p = tileK + (sub * 32 + (lane & 31)) * kLdsRow + half * 16;
        const f32x16 zero = {0};
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p)), __builtin_bit_cast(bf16x8, own[0]), zero, 0, 0, 0);
#pragma unroll
        for (int kk = 1; kk < kKSteps; ++kk)
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p + kk * 32)),
              __builtin_bit_cast(bf16x8, own[kk]), sacc, 0, 0, 0);
      }
      // ---- probabilities against the reference m, as a B operand (bf16), and their sum
      const bool interior = kb + 31 + w <= qw0;  // wholly visible and wholly outside the recency window
      bf16x8 pfrag[2];
      float sum = 0.0f;
      bool done = false;
      if (interior) {
        // The reference need not be the running maximum (see lse_update): the terms are taken against it as it
        // stands, and only a half-tile whose sum leaves the safe range -- the first one, whose reference is -inf,
        // and scores that rise by more than 16 powers of two later on -- takes the path below that raises it.  (The
        // bound is kept low here because the probabilities multiply V: the unnormalised output stays within 2^16 * n
        // times the largest |v|.)
        const float neg = -m;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pv = fast_exp2(fmaf(sacc[r], sc, neg));
          sum += pv;
          pfrag[r >> 3][r & 7] = static_cast<__bf16>(pv);
        }
        done = __builtin_amdgcn_ballot_w64(!(sum <= 0x1p16f)) == 0;
      }
      if (!done) {
        float tv[16];
        float mb = -INFINITY;
        if (interior) {
#pragma unroll
          for (int r = 0; r < 16; ++r) tv[r] = sacc[r] * sc;
          mb = max16(sacc) * sc;
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kb + 8 * (r >> 2) + 4 * half + (r & 3);
            float x = sacc[r] * sc;
            if (w > 0 && qi - key < w) x += rb;
            if (key > qi) x = -INFINITY;
            tv[r] = x;
            mb = fmaxf(mb, x);
          }
        }
        // the two lane halves feed one matrix product, so they must share the reference
        mb = fmaxf(mb, __shfl_xor(mb, 32, kWave));
        const float m_new = fmaxf(m, mb);  // finite: the first half-tile holds key 0, which every query sees
        if (__any(m_new > m)) {
          const float alpha = fast_exp2(m - m_new);  // 0 when m is still -inf
          l *= alpha;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        }
        m = m_new;
        sum = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pv = fast_exp2(tv[r] - m_new);
          sum += pv;
          pfrag[r >> 3][r & 7] = static_cast<__bf16>(pv);
        }
      }
      l += sum;
      // ---- O^T += V^T . P^T : two 16-key steps x four blocks of 32 head dimensions
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const char* vt = tileV + (sub * 32 + ks * 16) * kLdsRowV + tr_off;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const uint2 lo = lds_read_transposed(vt + db * 64);                // keys 4h .. 4h+3 of the step
          const uint2 hi = lds_read_transposed(vt + 8 * kLdsRowV + db * 64);  // keys 8+4h .. 8+4h+3
          const uint4 afrag = make_uint4(lo.x, lo.y, hi.x, hi.y);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, afrag), pfrag[ks], o[db], 0, 0, 0);
        }
      }
    }
  }
  // each lane half summed different keys of the same query
  l += __shfl_xor(l, 32, kWave);
  if (qi < len) {
    if (half == 0) a.lse[ubase + qi] = m + log2f(l);
    const float inv = 1.0f / l;
    uint16_t* orow = static_cast<uint16_t*>(a.O) + (ubase + qi) * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int d0 = db * 32 + 8 * g4 + 4 * half;
        uint2 pk;
        pk.x = f32_to_bf16(o[db][4 * g4 + 0] * inv) | (static_cast<uint32_t>(f32_to_bf16(o[db][4 * g4 + 1] * inv)) << 16);
        pk.y = f32_to_bf16(o[db][4 * g4 + 2] * inv) | (static_cast<uint32_t>(f32_to_bf16(o[db][4 * g4 + 3] * inv)) << 16);
        *reinterpret_cast<uint2*>(orow + d0) = pk;
      }
  }
}

// Benchmark aid: the matrix instruction of the passes above on register operands, four independent accumulator
// chains per wave, nothing else.  The checksum keeps the chains alive.  RANDOM = false: one operand pair holding a few
// small values (few bits toggle between instructions); RANDOM = true: eight operand pairs of pseudo-random values in
// (-2, 2), the bit activity of real activations -- the matrix units then draw more power and the clock gives way.
template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_probe(int iters, float* sink) {
  constexpr int NP = RANDOM ? 8 : 1;
  const int lane = threadIdx.x & (kWave - 1);
  bf16x8 x[NP], y[NP];
#pragma unroll
  for (int j = 0; j < NP; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (RANDOM) {
        uint32_t h = threadIdx.x * 64u + j * 8u + e + blockIdx.x * 7919u;
        h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
        x[j][e] = static_cast<__bf16>((static_cast<int>(h & 0xffffu) - 32768) * (1.0f / 16384.0f));
        y[j][e] = static_cast<__bf16>((static_cast<int>(h >> 16) - 32768) * (1.0f / 16384.0f));
      } else {
        x[j][e] = static_cast<__bf16>(0.00390625f * static_cast<float>(1 + ((lane + e) & 3)));
        y[j][e] = static_cast<__bf16>(0.0078125f * static_cast<float>(1 + ((lane ^ e) & 1)));
      }
    }
  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) acc[c] = f32x16{0};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[c % NP], y[(2 * c) % NP], acc[c], 0, 0, 0);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y[(c + 4) % NP], x[(2 * c + 1) % NP], acc[c], 0, 0, 0);
  }
  float sum = 0.0f;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[c][r];
  sink[static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x] = sum;
}

// Benchmark aid: the steady state of the two passes' software-pipelined form and nothing around it.  A workgroup
// fills one LDS tile with pseudo-random values itself, then every wave runs `tiles` times the four steps of a
// tile (32 matrix instructions, their 16 fragment reads, and the pass's vector work on the 2048 scores of the two
// half-tiles before: PASS 1 = multiply-add, exponential, add per score; PASS 2 = one more multiply-add and the
// row normalisers read from LDS) -- no global loads, no barriers, no masks.  What this reaches is the ceiling of
// the passes' instruction mix on the machine at hand, its clock under that load included.
template <int PASS>
__global__ __launch_bounds__(256, 2) void prefill_mix_probe(int tiles, float* sink) {
  __shared__ __attribute__((aligned(1024))) char tile[kRingTileBytes];
  __shared__ __attribute__((aligned(16))) float lse_s[kTile];
  const int lane = threadIdx.x & (kWave - 1), half = lane >> 5;
  auto rnd = [&](uint32_t i) {
    uint32_t h = i * 0x9e3779b9u + blockIdx.x * 7919u;
    h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
    return h;
  };
  for (int i = threadIdx.x; i < kRingTileBytes / 4; i += 256) {  // two bf16 values in (-2, 2) per word
    const uint32_t h = rnd(i);
    const float lo = (static_cast<int>(h & 0xffffu) - 32768) * (1.0f / 16384.0f);
    const float hi = (static_cast<int>(h >> 16) - 32768) * (1.0f / 16384.0f);
    reinterpret_cast<uint32_t*>(tile)[i] = f32_to_bf16(lo) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
  }
  if (threadIdx.x < kTile) lse_s[threadIdx.x] = 40.0f + 0.01f * threadIdx.x;
  uint4 own0[kKSteps], own1[kKSteps];
#pragma unroll
  for (int kk = 0; kk < kKSteps; ++kk) {
    own0[kk] = make_uint4(rnd(threadIdx.x * 64 + kk * 8) & 0xbfffbfffu, rnd(threadIdx.x * 64 + kk * 8 + 1) & 0xbfffbfffu,
                          rnd(threadIdx.x * 64 + kk * 8 + 2) & 0xbfffbfffu, rnd(threadIdx.x * 64 + kk * 8 + 3) & 0xbfffbfffu);
    own1[kk] = make_uint4(rnd(threadIdx.x * 64 + kk * 8 + 4) & 0xbfffbfffu, rnd(threadIdx.x * 64 + kk * 8 + 5) & 0xbfffbfffu,
                          rnd(threadIdx.x * 64 + kk * 8 + 6) & 0xbfffbfffu, rnd(threadIdx.x * 64 + kk * 8 + 7) & 0xbfffbfffu);
  }  // (exponent bit 14 cleared: magnitudes below 2)
  TileRing tr;
  tr.init();
  __syncthreads();
  const float sc = 0.1275f;
  float l0 = 0.0f, l1 = 0.0f, q0 = 0.0f, q1 = 0.0f;
  float lb0 = 0.0f, lb1 = 0.0f, qb0 = 0.0f, qb1 = 0.0f;  // column pass: the second chain of each running sum
  f32x16 A0, A1, B0 = {0}, B1 = {0};
  auto step = [&](auto consume_tag, const char* p, f32x16& x0, f32x16& x1, const f32x16& y0, const f32x16& y1, int ysub) {
    constexpr bool CONSUME = decltype(consume_tag)::value != 0;
    float a0 = 0.0f, b0 = 0.0f, a1 = 0.0f, b1 = 0.0f;  // row pass: the sums of this step, checked before they count
    float4 lv[4];
    if (PASS == 2 && CONSUME) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) lv[g4] = *reinterpret_cast<const float4*>(&lse_s[ysub * 32 + 8 * g4 + 4 * half]);
    }
    auto comp = [](const float4& v, int e) { return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w; };
    auto consume = [&](int kk, int g) {
      const int r = 2 * kk;
      const f32x16& y = g == 0 ? y0 : y1;
      if (PASS == 1) {
        float& sa = g == 0 ? a0 : a1; float& sb = g == 0 ? b0 : b1;
        sa += fast_exp2(fmaf(y[r], sc, -40.0f));
        sb += fast_exp2(fmaf(y[r + 1], sc, -40.0f));
      } else {  // the column pass adds to the block's running sums
        float& sa = g == 0 ? l0 : l1; float& sb = g == 0 ? lb0 : lb1; float& ta = g == 0 ? q0 : q1; float& tb = g == 0 ? qb0 : qb1;
        const float pa = fast_exp2(fmaf(y[r], sc, -comp(lv[r >> 2], r & 3)));
        const float pb = fast_exp2(fmaf(y[r + 1], sc, -comp(lv[r >> 2], (r & 3) + 1)));
        sa += pa; ta = fmaf(pa, pa, ta);
        sb += pb; tb = fmaf(pb, pb, tb);
      }
    };
    auto pin = [&]() {
      if (PASS == 1) asm volatile("" : "+v"(a0), "+v"(b0), "+v"(a1), "+v"(b1));
      else asm volatile("" : "+v"(l0), "+v"(lb0), "+v"(l1), "+v"(lb1), "+v"(q0), "+v"(qb0), "+v"(q1), "+v"(qb1));
    };
    fill_and_consume<CONSUME>(p, tr.frag, own0, own1, x0, x1, consume, pin);
    if (CONSUME && PASS == 1) {  // the row pass checks every tile's sum against its safe range
      if (__builtin_amdgcn_ballot_w64(!(a0 + b0 <= 0x1p64f)) == 0) l0 += a0 + b0;
      if (__builtin_amdgcn_ballot_w64(!(a1 + b1 <= 0x1p64f)) == 0) l1 += a1 + b1;
    }
  };
  step(StageTag<0>{}, tile, A0, A1, B0, B1, 0);
  for (int t = 0; t < tiles; ++t) {
    asm volatile("" : "+v"(own0[0].x), "+v"(own1[0].x));  // not loop-invariant as far as the compiler can tell
    step(StageTag<1>{}, tile + 32 * kRowBytes, B0, B1, A0, A1, 0);
    step(StageTag<1>{}, tile, A0, A1, B0, B1, 1);
  }
  float sum = l0 + l1 + q0 + q1 + lb0 + lb1 + qb0 + qb1;
#pragma unroll
  for (int r = 0; r < 16; ++r) sum += A0[r] + A1[r];
  sink[static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x] = sum;
}

// Two workgroups per block of keys when one would leave the chip short of workgroups (fewer than four per compute
// unit); ROCO_PREFILL_QSPLIT = 1 or 2 overrides.
int columns_query_shares(const PrefillArgs& a, int pairs) {
  const char* e = getenv("ROCO_PREFILL_QSPLIT");
  if (e != nullptr && (e[0] == '1' || e[0] == '2')) return e[0] - '0';
  return static_cast<long long>(a.units) * pairs < 1024 ? 2 : 1;
}

// Grouped column pass: the in-register head sum when the number of heads divides 16, else the general kernel.
template <int WAVES>
void launch_columns_grouped(const PrefillArgs& b, dim3 grid, hipStream_t s) {
  const dim3 block(WAVES * kWave);
  // The ring-fed kernel where it applies: sum-of-squares second statistic, a power-of-two group, and all of a unit's
  // query rows inside a 32-bit byte offset.  ROCO_PREFILL_GQA_RING=0 keeps the register-staged kernels (tests run both).
  const char* e = getenv("ROCO_PREFILL_GQA_RING");
  const bool ring_ok = !(e != nullptr && e[0] == '0') && !b.pol.counts_above_average() &&
                       static_cast<long long>(b.group) * b.L_max * kRowBytes < (1ll << 31);
  if (ring_ok) {
    switch (b.group) {
      case 2: hipLaunchKernelGGL((prefill_columns_gqa_ring<2>), grid, block, 0, s, b); return;
      case 4: hipLaunchKernelGGL((prefill_columns_gqa_ring<4>), grid, block, 0, s, b); return;
      case 8: hipLaunchKernelGGL((prefill_columns_gqa_ring<8>), grid, block, 0, s, b); return;
      case 16: hipLaunchKernelGGL((prefill_columns_gqa_ring<16>), grid, block, 0, s, b); return;
      default: break;
    }
  }
  switch (b.group) {
    case 2: hipLaunchKernelGGL((prefill_columns_gqa_pow2_mfma<WAVES, 2>), grid, block, 0, s, b); break;
    case 4: hipLaunchKernelGGL((prefill_columns_gqa_pow2_mfma<WAVES, 4>), grid, block, 0, s, b); break;
    case 8: hipLaunchKernelGGL((prefill_columns_gqa_pow2_mfma<WAVES, 8>), grid, block, 0, s, b); break;
    case 16: hipLaunchKernelGGL((prefill_columns_gqa_pow2_mfma<WAVES, 16>), grid, block, 0, s, b); break;
    default: hipLaunchKernelGGL(prefill_columns_gqa_mfma<WAVES>, grid, block, 0, s, b); break;
  }
}

template <int WAVES>
hipError_t launch_t(const PrefillArgs& a, hipStream_t s) {
  constexpr int kOwn = Shape<WAVES>::kOwn;
  const int n_blocks = (a.L_max + kOwn - 1) / kOwn;
  PrefillArgs b = a;
  b.paired = a.paired >= 0 ? a.paired : 1;  // pairing measured faster than lock-step single blocks
  b.pairs = b.paired ? (n_blocks + 1) / 2 : n_blocks;  // ids per unit
  b.qsplit = columns_query_shares(a, b.pairs);
  b.ksplit = a.group == 1 ? b.qsplit : 1;  // the second share's plane has no room for several heads
  const dim3 grid(static_cast<unsigned>((a.units + 7) / 8 * 8 * b.pairs * b.qsplit));
  const dim3 rows_grid(static_cast<unsigned>((a.units + 7) / 8 * 8 * a.group * b.pairs * b.ksplit));  // one id set per query head
  if (!a.skip_rows) {
    ProfScope ps(kProfPrefillRows, s);
    hipLaunchKernelGGL(prefill_rows_mfma, rows_grid, dim3(WAVES * kWave), 0, s, b);
    if (b.ksplit > 1)
      hipLaunchKernelGGL(merge_key_shares, dim3((a.L_max + 255) / 256, a.units), dim3(256), 0, s, b);
  }
  {
    ProfScope ps(kProfPrefillColumns, s);
    if (a.group != 1) launch_columns_grouped<WAVES>(b, grid, s);
    else if (a.pol.counts_above_average())
      hipLaunchKernelGGL(prefill_columns_mfma<true>, grid, dim3(WAVES * kWave), 0, s, b);
    else hipLaunchKernelGGL(prefill_columns_mfma<false>, grid, dim3(WAVES * kWave), 0, s, b);
    if (b.qsplit > 1)
      hipLaunchKernelGGL(sum_query_shares, dim3((a.L_max + 255) / 256, a.units), dim3(256), 0, s, b);
  }
  return hipGetLastError();
}

// Rows pass that also writes O, followed by the ordinary columns pass.
hipError_t launch_with_output(const PrefillArgs& a, hipStream_t s) {
  constexpr int WAVES = 4;
  constexpr int kOwnQ = 32 * WAVES;
  constexpr size_t kLds = 2 * static_cast<size_t>(kTileBytes + kTileBytesV);  // 74 KiB: above the default dynamic limit
  // set on every call: cheap, and right on whichever device is current
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_rows_out_mfma<WAVES>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kLds)) != hipSuccess)
    return hipErrorInvalidValue;
  PrefillArgs b = a;
  b.paired = 0;
  b.pairs = (a.L_max + kOwnQ - 1) / kOwnQ;  // workgroup ids per unit
  {
    ProfScope ps(kProfPrefillRows, s);
    hipLaunchKernelGGL(prefill_rows_out_mfma<WAVES>,
                       dim3(static_cast<unsigned>((a.units + 7) / 8 * 8 * a.group * b.pairs)), dim3(WAVES * kWave), kLds,
                       s, b);
  }
  constexpr int kOwn = Shape<4>::kOwn;
  const int n_blocks = (a.L_max + kOwn - 1) / kOwn;
  PrefillArgs c = a;
  c.paired = 1;
  c.pairs = (n_blocks + 1) / 2;
  c.qsplit = columns_query_shares(a, c.pairs);
  {
    ProfScope ps(kProfPrefillColumns, s);
    const dim3 cgrid(static_cast<unsigned>((a.units + 7) / 8 * 8 * c.pairs * c.qsplit));
    if (a.group != 1) launch_columns_grouped<4>(c, cgrid, s);
    else if (a.pol.counts_above_average()) hipLaunchKernelGGL(prefill_columns_mfma<true>, cgrid, dim3(4 * kWave), 0, s, c);
    else hipLaunchKernelGGL(prefill_columns_mfma<false>, cgrid, dim3(4 * kWave), 0, s, c);
    if (c.qsplit > 1)
      hipLaunchKernelGGL(sum_query_shares, dim3((a.L_max + 255) / 256, a.units), dim3(256), 0, s, c);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_mfma_probe(int workgroups, int iters, int mode, float* sink, hipStream_t s) {
  ProfScope ps(kProfMfmaProbe, s);
  const dim3 grid(static_cast<unsigned>(workgroups));
  switch (mode) {
    case 0: hipLaunchKernelGGL(mfma_probe<false>, grid, dim3(256), 0, s, iters, sink); break;
    case 1: hipLaunchKernelGGL(mfma_probe<true>, grid, dim3(256), 0, s, iters, sink); break;
    case 2: hipLaunchKernelGGL(prefill_mix_probe<1>, grid, dim3(256), 0, s, iters, sink); break;
    case 3: hipLaunchKernelGGL(prefill_mix_probe<2>, grid, dim3(256), 0, s, iters, sink); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_prefill_attention_mfma(const PrefillArgs& a, hipStream_t s) {
  if (a.O != nullptr) return launch_with_output(a, s);
  // 256 owned rows per workgroup (512 halved the streamed traffic but left one workgroup per compute unit, all of
  // whose waves wait at the same barriers: measured slower on the serving workload).
  return launch_t<4>(a, s);
}

}  // namespace roco
