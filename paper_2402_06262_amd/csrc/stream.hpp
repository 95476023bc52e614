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

// Attend the rows of [row_begin, row_end) that belong to this wave.  The range is cut into `passes` blocks
// of `pass_rows` rows; inside a block this wave owns rows wave_off + u*R + g (u < U).  Blocks are visited in
// rotated order starting at block `rot` (softmax does not care about order): workgroups that start at the
// same time then begin at different offsets inside their ranges instead of marching over the same HBM
// channels in lock step.  qf holds this lane's slice of the query already multiplied by scale*log2(e).
// bias(row) is added to the base-2 logit; zstore(row, t) receives every logit once (from the first lane of
// the row's group); fix(row, kw, vw, c) may replace the loaded 16 bytes of a row (the slot being overwritten).
template <int DT, int D, int U, class BiasFn, class ZStore, class FixFn>
__device__ __forceinline__ void stream_attend(const float* qf, const char* Kbase, const char* Vbase,
                                              int row_begin, int row_end, int passes, int rot, int pass_rows,
                                              int wave_off, BiasFn bias, ZStore zstore, FixFn fix,
                                              FlashState<RowGeom<DT, D>::EPL>& st) {
  using G = RowGeom<DT, D>;
  const int lane = threadIdx.x & (kWave - 1);
  const int g = lane / G::LPR, c = lane % G::LPR;
  int blk = rot;
  for (int it = 0; it < passes; ++it) {
    const int base = row_begin + blk * pass_rows + wave_off;
    blk = (blk + 1 == passes) ? 0 : blk + 1;
    uint4 kw[U], vw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * G::R + g;
      const bool ok = row < row_end;
      const size_t off = static_cast<size_t>(ok ? row : row_begin) * G::ROW_BYTES + c * 16;
      kw[u] = load16(Kbase + off);
      vw[u] = load16(Vbase + off);
    }
    float t[U];
    float mb = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * G::R + g;
      fix(row, kw[u], vw[u], c);
      float kf[G::EPL];
      unpack16<DT>(kw[u], kf);
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < G::EPL; ++e) dot = fmaf(qf[e], kf[e], dot);
      dot = group_sum<G::LPR>(dot);
      if (row < row_end) {
        t[u] = dot + bias(row);
        if (c == 0) zstore(row, t[u]);
      } else {
        t[u] = -INFINITY;
      }
      mb = fmaxf(mb, t[u]);
    }
    const float m_new = fmaxf(st.m, mb);
    if (m_new > -INFINITY) {  // false only while this group has seen no valid row at all
      const float alpha = exp2f(st.m - m_new);
      st.l *= alpha;
#pragma unroll
      for (int e = 0; e < G::EPL; ++e) st.acc[e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = exp2f(t[u] - m_new);
        float vf[G::EPL];
        unpack16<DT>(vw[u], vf);
        st.l += p;
#pragma unroll
        for (int e = 0; e < G::EPL; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e]);
      }
      st.m = m_new;
    }
  }
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
    const float a = (st.m > -INFINITY) ? exp2f(st.m - m_new) : 0.0f;
    const float b = (m_o > -INFINITY) ? exp2f(m_o - m_new) : 0.0f;
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
