// Pieces shared by the matrix-core kernels (bf16 storage, head_dim 128, v_mfma_f32_32x32x16_bf16).
//
// Operand layout of the 32x32x16 instruction, as used here: lane l supplies row (l % 32) and the 8 consecutive
// k-elements starting at 8 * (l / 32) of each 16-wide k-step, for A and for B alike; register r of the result
// belongs to A-row 8 * (r / 4) + 4 * (l / 32) + (r % 4) and B-row (l % 32).
#pragma once
#include "common.hpp"

namespace roco {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;

constexpr int D = 128;
constexpr int kTile = 64;                // rows of K, V or Q per LDS tile
constexpr int kRowBytes = D * 2;         // 256
constexpr int kLdsRow = kRowBytes + 16;  // padded: 16 lanes x 16 B then hit distinct bank groups
constexpr int kKSteps = D / 16;          // 8 matrix instructions per 32x32 tile
constexpr int kTileBytes = kTile * kLdsRow;
// V tiles that are read with the LDS transpose read take rows of 320 bytes: a 16-lane group of that read touches 4
// consecutive rows x 32 bytes, and with 80-dword rows the 32 lanes served together fall on 64 distinct banks (with
// the 272-byte rows of the K tiles, whose 128-bit row reads need that stride, half of the LDS cycles of those reads
// were bank conflicts).
constexpr int kLdsRowV = kRowBytes + 64;
constexpr int kTileBytesV = kTile * kLdsRowV;

__device__ __forceinline__ float max16(const f32x16& s) {
  float a = fmaxf(fmaxf(s[0], s[1]), s[2]);  // the compiler folds these into three-operand maxima
  a = fmaxf(fmaxf(a, s[3]), s[4]);
  a = fmaxf(fmaxf(a, s[5]), s[6]);
  a = fmaxf(fmaxf(a, s[7]), s[8]);
  a = fmaxf(fmaxf(a, s[9]), s[10]);
  a = fmaxf(fmaxf(a, s[11]), s[12]);
  a = fmaxf(fmaxf(a, s[13]), s[14]);
  return fmaxf(a, s[15]);
}

// gfx950 LDS transpose read: within a group of 16 lanes, lane i points at 4 consecutive 16-bit elements and
// receives element (i % 4) of the data addressed by lanes i / 4, 4 + i / 4, 8 + i / 4 and 12 + i / 4.  With lane i
// of a group pointing at row i / 4, column 4 * (i % 4) of a 4-row x 16-column block, lane i therefore receives
// rows 0..3 of column i (checked on the device).  The pointer must address LDS.
__device__ __forceinline__ uint2 lds_read_transposed(const char* p) {
  const v4i16 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(p));
  return __builtin_bit_cast(uint2, v);
}

// Per-lane byte offset of the transpose reads that build a V^T fragment (A operand: row = head dimension, 8 keys
// per lane) from a row-major V tile: 16-lane group g = lane / 16 reads columns 16 * (g % 2) .. +15 of a
// 32-column block and key rows 4 * (g / 2) .. +3; a second read 8 rows further down completes the 8 k-slots
// (slots 0-3 = keys 4h..4h+3, slots 4-7 = keys 8+4h..8+4h+3 of a 16-key step, h = lane / 32: the order in which
// the accumulator of a score tile holds its keys).
__device__ __forceinline__ int transposed_fragment_offset() {
  const int lane = threadIdx.x & (kWave - 1);
  const int i16 = lane & 15, grp = lane >> 4;
  return ((grp >> 1) * 4 + (i16 >> 2)) * kLdsRowV + ((grp & 1) * 16 + (i16 & 3) * 4) * 2;
}

}  // namespace mfma
}  // namespace roco
