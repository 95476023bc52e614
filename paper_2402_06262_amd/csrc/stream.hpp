// Streaming dot-product / online-softmax loops on the plain vector ALUs.
//
// A row of K, V or Q (D elements) is spread over LPR = D / (elements per 16 bytes) adjacent lanes, so one
// wave-wide 128-bit load covers R = 64 / LPR consecutive rows (1 KiB of contiguous memory) and every lane
// group runs its own independent online-softmax stream; streams are merged once at the end.  This is the
// HBM-bound shape of the decode step (section 5.3 "Overhead": decoding is I/O-bounded).
#pragma once
#include "common.hpp"

namespace roco {

template <int DT, int D> struct RowGeom {
  static constexpr int EPL = Elem<DT>::per16;  // elements per lane
  static constexpr int LPR = D / EPL;          // lanes per row
  static constexpr int R = kWave / LPR;        // rows per wave-wide load
  static constexpr int ROW_BYTES = D * (16 / EPL);
  static_assert(LPR >= 1 && LPR <= kWave && (LPR & (LPR - 1)) == 0, "row must tile a wave");
};

// Online-softmax state of one lane group, in base-2 logits: sum_j 2^(t_j - m) and sum_j 2^(t_j - m) v_j.
template <int EPL> struct FlashState {
  float m, l, acc[EPL];
  __device__ __forceinline__ void reset() {
    m = -INFINITY; l = 0.0f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.0f;
  }
};

// 2^x on the hardware exponential unit, without the library's denormal-range rescaling: arguments here are
// differences to a running maximum (<= 0), and results below the normal range may flush to zero.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Attend the rows of [row_begin, row_end) that belong to this wave.  The range is cut into `passes` blocks
// of `pass_rows` rows; inside a block this wave owns rows wave_off + u*R + g (u < U).  Blocks are visited in
// rotated order starting at block `rot` (softmax does not care about order).
//
// HBM latency under load is several microseconds, so what bounds the bandwidth of a streaming kernel is the
// number of bytes it keeps in flight, and load results can only wait in registers.  The loop is therefore
// software-pipelined at the level of the two operand streams: as soon as the K registers of a block have
// been turned into scores they are reloaded with the next block's K rows, and likewise for V after the
// accumulation, so every lane has between U and 2U 128-bit loads outstanding at all times with only 2U load
// registers.  There is no control flow around the loads (the last block is peeled off), which lets the
// compiler wait for each load individually, in issue order.
//
// qf holds this lane's slice of the query already multiplied by scale*log2(e).
//   STREAMING   loads K / V with the non-temporal hint: right when the whole cache is far larger than the chip's
//               last-level cache (the rows would only displace the statistics), wrong when it fits and the next
//               step would find it there;
//   bias(row, x) is added to the base-2 logit (only evaluated when HAS_BIAS); x = aux[row] if aux is not null (the
//               row's position, say), loaded with the row's K so that it has arrived when the score is formed: a load
//               inside bias() would have to wait for every load issued before it, the next block's rows included;
//   zptr        if not null, receives every base-2 logit once: zptr[row];
//   special_row a row that must not take the branch-free path (the slot being overwritten), or -1;
//   fix_k(row, kw, c) / fix_v(row, vw, c) may replace the loaded 16 bytes of that row.
template <int DT, int D, int U, bool HAS_BIAS, bool STREAMING, class BiasFn, class FixK, class FixV>
__device__ __forceinline__ void stream_attend(const float* qf, const char* Kbase, const char* Vbase,
                                              int row_begin, int row_end, int passes, int rot, int pass_rows,
                                              int wave_off, BiasFn bias, const int32_t* aux, float* zptr, int special_row,
                                              FixK fix_k, FixV fix_v, FlashState<RowGeom<DT, D>::EPL>& st) {
  using G = RowGeom<DT, D>;
  const int lane = threadIdx.x & (kWave - 1);
  const int g = lane / G::LPR, c = lane % G::LPR;

  auto issue = [&](int blk, const char* base_ptr, uint4* w) {
    const int base = row_begin + blk * pass_rows + wave_off;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * G::R + g;
      const size_t off = static_cast<size_t>(row < row_end ? row : row_begin) * G::ROW_BYTES + c * 16;
      w[u] = STREAMING ? load16_streaming(base_ptr + off) : load16(base_ptr + off);
    }
  };
  int aw[U];
#pragma unroll
  for (int u = 0; u < U; ++u) aw[u] = 0;
  auto issue_aux = [&](int blk) {
    if (HAS_BIAS && aux != nullptr) {
      const int base = row_begin + blk * pass_rows + wave_off;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + u * G::R + g;
        aw[u] = aux[row < row_end ? row : row_begin];
      }
    }
  };
  auto is_plain = [&](int base) {
    return base + U * G::R <= row_end && (special_row < base || special_row >= base + U * G::R);
  };

  // K registers -> U base-2 logits of this lane group (t) and their maximum (mb)
  auto scores = [&](int blk, uint4* kw, float* t, float& mb) {
    const int base = row_begin + blk * pass_rows + wave_off;
    mb = -INFINITY;
    if (is_plain(base)) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float kf[G::EPL];
        unpack16<DT>(kw[u], kf);
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) dot = fmaf(qf[e], kf[e], dot);
        t[u] = group_sum<G::LPR>(dot);
        if (HAS_BIAS) t[u] += bias(base + u * G::R + g, aw[u]);
        mb = fmaxf(mb, t[u]);
      }
      if (zptr != nullptr) {  // lane c of a group stores the logit of the group's c-th row: one store per block
        float tz = t[0];
#pragma unroll
        for (int u = 1; u < U; ++u) tz = (c == u) ? t[u] : tz;
        if (c < U) zptr[base + c * G::R + g] = tz;
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + u * G::R + g;
        fix_k(row, kw[u], c);
        float kf[G::EPL];
        unpack16<DT>(kw[u], kf);
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) dot = fmaf(qf[e], kf[e], dot);
        dot = group_sum<G::LPR>(dot);
        if (row < row_end) {
          t[u] = HAS_BIAS ? dot + bias(row, aw[u]) : dot;
          if (c == 0 && zptr != nullptr) zptr[row] = t[u];
        } else {
          t[u] = -INFINITY;
        }
        mb = fmaxf(mb, t[u]);
      }
    }
  };

  // V registers + logits -> online-softmax state
  auto accumulate = [&](int blk, uint4* vw, const float* t, float mb) {
    const int base = row_begin + blk * pass_rows + wave_off;
    if (!is_plain(base)) {
      // Rows past the end were loaded from row_begin only to keep the address in range.  Their weight is 2^-inf = 0,
      // but row_begin may be the very slot this step fills for the first time, whose bytes in the caller's buffer
      // are arbitrary (0 x NaN is NaN): such rows contribute zeros, whatever was loaded.
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + u * G::R + g;
        fix_v(row, vw[u], c);
        if (row >= row_end) vw[u] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    const float m_new = fmaxf(st.m, mb);
    if (m_new > -INFINITY) {  // false only while this group has seen no valid row at all
      const float alpha = fast_exp2(st.m - m_new);
      st.l *= alpha;
#pragma unroll
      for (int e = 0; e < G::EPL; ++e) st.acc[e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = fast_exp2(t[u] - m_new);
        float vf[G::EPL];
        unpack16<DT>(vw[u], vf);
        st.l += p;
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e]);
      }
      st.m = m_new;
    }
  };

  if (passes <= 0) return;
  uint4 kw[U], vw[U];
  float t[U];
  float mb;
  int blk = rot;
  issue_aux(blk);
  issue(blk, Kbase, kw);
  issue(blk, Vbase, vw);
  for (int it = 0; it + 1 < passes; ++it) {
    const int nb = (blk + 1 == passes) ? 0 : blk + 1;
    scores(blk, kw, t, mb);
    issue_aux(nb);
    issue(nb, Kbase, kw);
    accumulate(blk, vw, t, mb);
    issue(nb, Vbase, vw);
    blk = nb;
  }
  scores(blk, kw, t, mb);
  accumulate(blk, vw, t, mb);
}

// Merge the R lane-group streams of a wave into group 0's lanes (all lanes end with the merged state).
template <int DT, int D>
__device__ __forceinline__ void merge_groups_in_wave(FlashState<RowGeom<DT, D>::EPL>& st) {
  using G = RowGeom<DT, D>;
#pragma unroll
  for (int mask = G::LPR; mask < kWave; mask <<= 1) {
    const float m_o = __shfl_xor(st.m, mask, kWave);
    const float l_o = __shfl_xor(st.l, mask, kWave);
    const float m_new = fmaxf(st.m, m_o);
    const float a = (st.m > -INFINITY) ? fast_exp2(st.m - m_new) : 0.0f;
    const float b = (m_o > -INFINITY) ? fast_exp2(m_o - m_new) : 0.0f;
    st.l = st.l * a + l_o * b;
#pragma unroll
    for (int e = 0; e < G::EPL; ++e) {
      const float acc_o = __shfl_xor(st.acc[e], mask, kWave);
      st.acc[e] = st.acc[e] * a + acc_o * b;
    }
    st.m = m_new;
  }
}

}  // namespace roco
