// Building blocks of the bf16 MFMA kernels (gfx950 only): vector types, the
// swizzled LDS tile layout, MFMA operand fragment loads and small wave-level
// helpers.
//
// MFMA v_mfma_f32_32x32x16_bf16 operand layout (lane l, g = l / 32):
//   A (32 x 16):  row  l % 32, contraction elements 8g .. 8g+7
//   B (16 x 32):  col  l % 32, contraction elements 8g .. 8g+7
//   C (32 x 32):  col  l % 32, register v holds row 8*(v/4) + 4g + (v%4)
// Only the pairing of A and B contraction slots matters, so an accumulator tile can
// be fed back as a B operand without any cross-lane movement when the other operand
// is loaded with the matching row permutation: B slot e of k-step t (16 rows) takes
// accumulator register 8t + e, i.e. row 16t + 8*(e/4) + 4g + (e%4).
//
// LDS tiles hold 128 bf16 (256 bytes) per row, unpadded, with the sixteen 16-byte
// chunks of a row XOR-permuted by a function of the row.  The permutation makes both
// access patterns bank-conflict free: row-major 16-byte reads by 16 consecutive rows
// and transposing ds_read_b64_tr_b16 reads of 4 consecutive rows x 64 bytes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define S2_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int kRowBytes = 256;          // one tile row: 128 bf16
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// Byte offset of 16-byte chunk `chunk` (0..15) of row `row` inside a tile.
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * kRowBytes + ((chunk ^ swz(row)) << 4);
}

// Per-lane byte offsets of the two kinds of operand fragments inside a tile, computed
// once per kernel.  Because the swizzle depends on (row mod 16) only, a fragment of a
// row block that starts at a multiple of 16 rows is the same offset plus a constant,
// which the compiler folds into the LDS instruction's immediate offset.
struct LaneOffsets {
  int rm[8];      // row-major fragment k: elements [16k + 8g, +8) of row (l % 32)
  int tr[4][2];   // transposed fragment, column block cb: rows 4g + L/4 and that + 8
};

__device__ __forceinline__ void init_lane_offsets(LaneOffsets& o, int lane) {
  const int l32 = lane & 31, g32 = lane >> 5;
#pragma unroll
  for (int k = 0; k < 8; ++k) o.rm[k] = tile_off(l32, 2 * k + g32);
  const int L = lane & 15, half = lane & 16;
  const int row = 4 * g32 + (L >> 2);
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) {
    const int col = 32 * cb + half + 4 * (L & 3);
    const int chunk = col >> 3, within = (col & 7) * 2;
    o.tr[cb][0] = row * kRowBytes + ((chunk ^ swz(row)) << 4) + within;
    o.tr[cb][1] = (row + 8) * kRowBytes + ((chunk ^ swz(row + 8)) << 4) + within;
  }
}

// Row-major operand fragment k (elements [16k + 8g, +8)) of row ROW0 + (l % 32);
// ROW0 must be a multiple of 16.
template <int ROW0>
__device__ __forceinline__ bf16x8 frag_rm(const char* tile, const LaneOffsets& o, int k) {
  static_assert(ROW0 % 16 == 0, "row block must start at a multiple of 16 rows");
  return *reinterpret_cast<const bf16x8*>(tile + o.rm[k] + ROW0 * kRowBytes);
}

// Transposed operand fragment: the operand row index runs along the tile's columns
// (32 columns starting at 32*cb) and the contraction index along the 16 tile rows
// starting at KROW0 (a multiple of 16), in the accumulator-feedback order described
// above.  Two transposing 64-bit LDS reads: within each block of 16 lanes, lane L
// points at 4 elements of tile row (L / 4) and receives one column of the 4 rows.
template <int KROW0>
__device__ __forceinline__ bf16x8 frag_tr(const char* tile, const LaneOffsets& o, int cb) {
  static_assert(KROW0 % 16 == 0, "row block must start at a multiple of 16 rows");
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
      S2_LDS(bf16x4, tile + o.tr[cb][0] + KROW0 * kRowBytes));
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
      S2_LDS(bf16x4, tile + o.tr[cb][1] + KROW0 * kRowBytes));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Rows narrower than the 128-element tile (head dimension 64): the kernels built for partial
// tiles have a second instantiation (DH = 64) that stages only the first eight 16-byte chunks
// of every tile row, loads only the first four register fragments of a row, runs its products
// over d = 0 .. 63 and stores the first half of the output tiles; the upper half of the LDS
// rows is never read.

// Direct global -> LDS copy of 16 bytes per lane (global_load_lds_dwordx4): lane i of
// the wave fetches the 16 bytes at its own global address `g`, and they land at LDS byte
// address lds_base + 16*i, where lds_base must be wave-uniform.  Issued as inline
// assembly so that the compiler does not fence unrelated LDS reads behind it; the
// caller waits with s_waitcnt vmcnt(0) and a barrier before the data is read.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(g) : "memory", "m0");
}

// Scalar-base form: the global address is a wave-uniform 64-bit base plus a per-lane
// unsigned 32-bit byte offset, so that a kernel that streams tiles keeps one offset
// register per lane and does the per-tile address arithmetic on the scalar unit.
__device__ __forceinline__ uint64_t uni64(uint64_t u) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ void dma16s(uint64_t base, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(lane_off), "s"(base) : "memory", "m0");
}

__device__ __forceinline__ void dma4s(uint64_t base, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(lane_off), "s"(base) : "memory", "m0");
}

// Same with 4 bytes per lane (global_load_lds_dword): lane i lands at lds_base + 4*i.
__device__ __forceinline__ void dma4(const void* g, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(g) : "memory", "m0");
}

// Marks a wave-uniform value that was computed with vector instructions (integer division has
// no scalar form) so that it lives in a scalar register and loops/branches on it are scalar.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)S2_LDS(const char, p));
}

__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Value of the same register in lane (l ^ 32).
__device__ __forceinline__ float other_half(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // lanes < 32 receive the partner in r[1], lanes >= 32 in r[0]
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

__device__ __forceinline__ float max_halves(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float sum_halves(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3,
                                        float a4, float a5, float a6, float a7) {
  bf16x8 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
  return r;
}

__device__ __forceinline__ bf16x4 pack4(float a0, float a1, float a2, float a3) {
  bf16x4 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  return r;
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Scheduling hint for the region since the last sched_barrier: N times
// {1 MFMA, up to DS LDS reads, up to VA VALU/transcendental instructions}, so that the
// vector work of one block is issued in the shadow of another block's matrix work.
template <int N, int DS, int VA>
__device__ __forceinline__ void interleave_mfma() {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (DS > 0) __builtin_amdgcn_sched_group_barrier(0x100, DS, 0);
    if (VA > 0) __builtin_amdgcn_sched_group_barrier(0x402, VA, 0);
  }
}

// Two-part variant: the first N1 MFMAs each take up to DS1 LDS reads behind them (the
// operand loads of the following phase go out early), the remaining N2 MFMAs each take
// up to VA2 VALU/transcendental instructions.
template <int N1, int DS1, int N2, int VA2>
__device__ __forceinline__ void interleave_mfma2() {
#pragma unroll
  for (int i = 0; i < N1; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, DS1, 0);
  }
#pragma unroll
  for (int i = 0; i < N2; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (VA2 > 0) __builtin_amdgcn_sched_group_barrier(0x402, VA2, 0);
  }
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// Transposes a wave's 32 x 128 accumulator block (rows lane-indexed, columns
// register-indexed) through its private 8 KB LDS region.
__device__ __forceinline__ void acc_to_lds(char* region, const f32x16 (&acc)[4], float mul, int l32, int g32) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
      const bf16x4 pk = pack4(acc[db][4 * vv] * mul, acc[db][4 * vv + 1] * mul,
                              acc[db][4 * vv + 2] * mul, acc[db][4 * vv + 3] * mul);
      *reinterpret_cast<bf16x4*>(region + tile_off(l32, 4 * db + vv) + 8 * g32) = pk;
    }
}

}  // namespace s2
