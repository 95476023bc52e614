// A ring of LDS tiles filled by loads that go from global memory straight into LDS (gfx950: 128 bits per lane), for
// the kernels that stream one operand of a matrix product past register-resident rows of the other.
//
// A tile is 64 rows of 256 bytes, stored unpadded.  One wave-wide load writes 1 KiB of LDS, lane i's 16 bytes at
// base + 16 i, so a wave fills four consecutive rows per instruction and the four waves of a workgroup fill a tile
// with four instructions each.  Which 16-byte chunk of its row a lane fetches is free, and that freedom replaces
// the padding: chunk c of row r is stored in slot c ^ (r & 15), so that the 128-bit fragment reads of the matrix
// instruction (16 consecutive rows, same chunk) fall on 16 distinct bank groups.  (Checked on the device: the
// placement of the lanes' bytes, and rows beyond the buffer's size coming back as zeros.)
//
// Nothing passes through registers, no address arithmetic is left on the vector ALU (a lane's offset inside a tile
// is fixed; the tile's offset is a scalar operand), and because no registers hold data in flight the ring can be
// three tiles deep: a tile is requested two tiles of work ahead of its use.
//
// The compiler does not know that these loads write LDS.  The kernel therefore orders them by hand: wait_loads<N>()
// until at most N of the wave's loads are outstanding, then a barrier, before any wave reads the tile.
#pragma once
#include "mfma.hpp"

namespace roco {
namespace mfma {

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"

typedef int v4i32 __attribute__((ext_vector_type(4)));

constexpr int kRingStages = 3;
constexpr int kRingTileBytes = kTile * kRowBytes;  // 16 KiB
constexpr int kRingBytes = kRingStages * kRingTileBytes;

// Raw buffer descriptor over `bytes` bytes at `base`: loads beyond it return zeros instead of faulting.
__device__ __forceinline__ v4i32 make_buffer(const void* base, uint32_t bytes) {
  const uint64_t b = reinterpret_cast<uint64_t>(base);
  v4i32 r;
  r.x = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(b)));
  r.y = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(b >> 32) & 0xffffu));
  r.z = __builtin_amdgcn_readfirstlane(static_cast<int>(bytes));
  r.w = 0x00020000;  // raw buffer, 32-bit data format
  return r;
}

// Wave-wide load, 16 bytes per lane: lane i's bytes from buffer offset voffset + soffset go to LDS address
// lds_addr + 16 i.  lds_addr and soffset are wave-uniform.
__device__ __forceinline__ void load16_to_lds(v4i32 rsrc, uint32_t lds_addr, int voffset, int soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory", "m0");
}
// The same with 4 bytes per lane: lane i's word goes to lds_addr + 4 i.
__device__ __forceinline__ void load4_to_lds(v4i32 rsrc, uint32_t lds_addr, int voffset, int soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory", "m0");
}
// Wait until at most N of this wave's loads are outstanding (loads complete in issue order).
template <int N> __device__ __forceinline__ void wait_loads() {
  static_assert(N >= 0 && N < 64, "six-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)p));
}

// Per-lane constants of a 256-thread workgroup streaming 64 x 256 B tiles through the ring.
struct TileRing {
  int voff[4];  // byte offset inside a tile of the four chunks this lane fetches
  int frag[8];  // byte offset inside a 32-row half-tile of this lane's fragment of each 16-wide k-step
  int wave;     // wave-uniform

  __device__ __forceinline__ void init() {
    const int lane = threadIdx.x & (kWave - 1);
    wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 16 * wave + 4 * i + (lane >> 4);
      voff[i] = r * kRowBytes + (((lane & 15) ^ (r & 15)) << 4);
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      frag[kk] = (lane & 31) * kRowBytes + (((2 * kk + (lane >> 5)) ^ (lane & 15)) << 4);
  }
  // Request tile `tile` (rows 64 tile ..) of the buffer into ring stage `stage`: four loads per wave.
  __device__ __forceinline__ void request(v4i32 rsrc, uint32_t ring_addr, int tile, int stage) const {
    const uint32_t dst = ring_addr + stage * kRingTileBytes + wave * 4096;
    const int soff = __builtin_amdgcn_readfirstlane(tile * kRingTileBytes);
#pragma unroll
    for (int i = 0; i < 4; ++i) load16_to_lds(rsrc, dst + i * 1024, voff[i], soff);
  }
};

// Two 32x32 score tiles: the 32 streamed rows of the half-tile at `p` (a ring stage plus 0 or 32 rows) against the
// wave's two groups of 32 owned rows (each fragment read from LDS feeds two matrix instructions).
__device__ __forceinline__ void score_tiles_ring(const char* p, const int* frag, const uint4* own0, const uint4* own1,
                                                 bool do0, bool do1, f32x16& acc0, f32x16& acc1) {
  const f32x16 zero = {0};
  auto fr = [&](int kk) { return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p + frag[kk])); };
  auto mm = [](bf16x8 x, const uint4& y, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, __builtin_bit_cast(bf16x8, y), c, 0, 0, 0);
  };
  if (do0 && do1) {
    bf16x8 a = fr(0);
    acc0 = mm(a, own0[0], zero);
    acc1 = mm(a, own1[0], zero);
#pragma unroll
    for (int kk = 1; kk < kKSteps; ++kk) {
      a = fr(kk);
      acc0 = mm(a, own0[kk], acc0);
      acc1 = mm(a, own1[kk], acc1);
    }
  } else if (do0) {
    acc0 = mm(fr(0), own0[0], zero);
#pragma unroll
    for (int kk = 1; kk < kKSteps; ++kk) acc0 = mm(fr(kk), own0[kk], acc0);
  } else if (do1) {
    acc1 = mm(fr(0), own1[0], zero);
#pragma unroll
    for (int kk = 1; kk < kKSteps; ++kk) acc1 = mm(fr(kk), own1[kk], acc1);
  }
}

// Two 32x32 score tiles of one group of owned rows against two different half-tiles (two independent accumulator
// chains, as above, for the stretch of the diagonal where only one of a wave's groups still has keys to see).
__device__ __forceinline__ void score_two_subs_ring(const char* pa, const char* pb, const int* frag, const uint4* own,
                                                    f32x16& acc_a, f32x16& acc_b) {
  const f32x16 zero = {0};
  auto mm = [](bf16x8 x, const uint4& y, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, __builtin_bit_cast(bf16x8, y), c, 0, 0, 0);
  };
#pragma unroll
  for (int kk = 0; kk < kKSteps; ++kk) {
    const bf16x8 fa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(pa + frag[kk]));
    const bf16x8 fb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(pb + frag[kk]));
    acc_a = mm(fa, own[kk], kk == 0 ? zero : acc_a);
    acc_b = mm(fb, own[kk], kk == 0 ? zero : acc_b);
  }
}

// The software-pipelined form of the above for tiles where nothing is masked: the 16 matrix instructions that fill
// (x0, x1) from the half-tile at `p` are issued one at a time, and after each of them comes one slice of the vector
// work that consumes the two score tiles (y0, y1) filled one step earlier -- consume(kk, g) handles scores 2 kk and
// 2 kk + 1 of group g.  A wave issues in order, so only vector instructions that sit between two matrix
// instructions in program order run while the matrix pipe works; scheduling fences keep the order written here.
// Two accumulator chains are filled at a time: a single chain of dependent matrix instructions runs at half rate.
// pin() must name the consumer's running results in an empty volatile asm: without a use inside this block the
// compiler sinks the whole vector chain to wherever its result is first needed, behind the last matrix instruction.
template <bool CONSUME, class ConsumeFn, class PinFn>
__device__ __forceinline__ void fill_and_consume(const char* p, const int* frag, const uint4* own0, const uint4* own1,
                                                 f32x16& x0, f32x16& x1, ConsumeFn consume, PinFn pin) {
  const f32x16 zero = {0};
  auto rd = [&](int kk) { return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p + frag[kk])); };
  auto mm = [](bf16x8 x, const uint4& y, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, __builtin_bit_cast(bf16x8, y), c, 0, 0, 0);
  };
  bf16x8 f[kKSteps];
  f[0] = rd(0);
  f[1] = rd(1);
  f[2] = rd(2);
#pragma unroll
  for (int kk = 0; kk < kKSteps; ++kk) {
    if (kk + 3 < kKSteps) f[kk + 3] = rd(kk + 3);  // fragments are requested three slices ahead of their use
    __builtin_amdgcn_sched_barrier(0);
    if (CONSUME) consume(kk, 0);
    __builtin_amdgcn_sched_barrier(0);
    x0 = mm(f[kk], own0[kk], kk == 0 ? zero : x0);
    __builtin_amdgcn_sched_barrier(0);
    if (CONSUME) consume(kk, 1);
    __builtin_amdgcn_sched_barrier(0);
    x1 = mm(f[kk], own1[kk], kk == 0 ? zero : x1);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (CONSUME) pin();
}

#pragma clang diagnostic pop

}  // namespace mfma
}  // namespace roco
