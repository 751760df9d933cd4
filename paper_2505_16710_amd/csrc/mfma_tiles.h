// Device-side building blocks for the bf16 matrix-core kernels (gfx950, wave64, head_dim 128).
//
// Operand layouts of v_mfma_f32_32x32x16_bf16 (D = A[32x16] * B[16x32] + C), lane l, g = l / 32:
//   A: row  l % 32, contraction slots 8g .. 8g+7
//   B: col  l % 32, contraction slots 8g .. 8g+7
//   C: col  l % 32, register r holds row 8*(r/4) + 4g + r%4
// so a C tile can be fed back as an A or B operand over 16 contraction steps by taking
// registers 8t .. 8t+7: slot s then stands for index 16t + 8*(s/4) + 4g + s%4 of the
// contracted dimension.  The other operand must present the same slot -> index map; when it
// comes from a row-major LDS tile whose ROWS are contracted, the LDS transpose read
// (ds_read_b64_tr_b16: lane i of a 16-lane group receives element i%4 of the 8 bytes
// addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4) delivers exactly that.
//
// LDS tiles are row-major, 256 bytes per row (128 bf16), with the sixteen 16-byte chunks of a
// row XOR-swizzled by a function of the row number so that both access patterns are free of
// bank conflicts: 16 lanes reading the same chunk of 16 consecutive rows, and the transpose
// read's 4 rows x 64 bytes per half-wave.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace seco {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define SECO_LDS __attribute__((address_space(3)))
typedef SECO_LDS char lds_char;

constexpr int kHeadDim = 128;
constexpr int kRowBytes = kHeadDim * 2;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// byte offset of 16-byte chunk `chunk` (0..15) of row `row` inside a tile
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * kRowBytes + ((chunk ^ swz(row)) << 4); }

// 8 consecutive head_dim elements of one row (operand whose contraction runs along head_dim)
__device__ __forceinline__ bf16x8 lds_row8(lds_char* tile, int row, int chunk) {
  return *reinterpret_cast<SECO_LDS bf16x8*>(tile + tile_off(row, chunk));
}

__device__ __forceinline__ void lds_store16(lds_char* tile, int row, int chunk, bf16x8 v) {
  *reinterpret_cast<SECO_LDS bf16x8*>(tile + tile_off(row, chunk)) = v;
}

// Operand whose contraction runs along the tile's ROWS: for head_dim column 32*db + lane%32,
// slots s = 0..7 hold rows row0 + 8*(s/4) + 4*(lane/32) + s%4.
__device__ __forceinline__ bf16x8 lds_tr8(lds_char* tile, int row0, int db, int lane) {
  const int ii = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const int row = row0 + 4 * g + (ii >> 2);
  const int chunk = 4 * db + 2 * half + ((ii & 3) >> 1);
  const int sub = (ii & 1) << 3;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<SECO_LDS s16x4*>(tile + tile_off(row, chunk) + sub));
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      reinterpret_cast<SECO_LDS s16x4*>(tile + tile_off(row + 8, chunk) + sub));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// The same two reads with the lane-dependent part of the address taken out of the loop.  tile_off(row0 + r, chunk)
// = row0 * kRowBytes + tile_off(r, chunk) whenever row0 is a multiple of 16 (the swizzle looks at the low four row
// bits only), so a kernel can compute these offsets once; an access in its main loop is then
// tile base + per-lane offset (one add per tile and offset) + a compile-time constant folded into the instruction.
struct TrOff { int lo, hi; };     // rows r and r + 8 of lds_tr8
__device__ __forceinline__ int row8_lane_off(int l32, int chunk) { return tile_off(l32, chunk); }
__device__ __forceinline__ TrOff tr8_lane_off(int db, int lane) {
  const int ii = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const int row = 4 * g + (ii >> 2);
  const int chunk = 4 * db + 2 * half + ((ii & 3) >> 1);
  const int sub = (ii & 1) << 3;
  return {tile_off(row, chunk) + sub, tile_off(row + 8, chunk) + sub};
}
__device__ __forceinline__ bf16x8 lds_row8_at(lds_char* tile_plus_off, int row0) {   // row0: multiple of 32
  return *reinterpret_cast<SECO_LDS bf16x8*>(tile_plus_off + row0 * kRowBytes);
}
__device__ __forceinline__ bf16x8 lds_tr8_at(lds_char* tile, TrOff off, int row0) {   // row0: multiple of 16
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<SECO_LDS s16x4*>(tile + off.lo + row0 * kRowBytes));
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<SECO_LDS s16x4*>(tile + off.hi + row0 * kRowBytes));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// registers 8t .. 8t+7 of a C tile, rounded to bf16 (pairwise, one v_cvt_pk_bf16_f32 per pair),
// as an operand over 16 contraction steps
__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int t) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x2 v = {x[8 * t + 2 * i], x[8 * t + 2 * i + 1]};
    r[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
  return __builtin_bit_cast(bf16x8, r);
}

// Asynchronous copy of four 256-byte rows (rows r .. r+3 of a swizzled tile, r wavefront-uniform)
// from global memory straight into LDS with global_load_lds_dwordx4: lane i's 16 bytes land at
// dst + 16*i, so the swizzle is applied by choosing which 16-byte chunk of its source row the
// lane fetches.  `row_ptr` is this lane's source row (lane / 16 selects the row), already
// clamped by the caller.  The copy is tracked by vmcnt only: the issuing wavefront must call
// dma_wait_all() before the barrier that publishes the tile.  (Issued as inline assembly on
// purpose: with the compiler builtin every later LDS read in the loop is made to wait for the
// copy, because the destination cannot be told apart from the tiles being read.)
__device__ __forceinline__ void dma4rows(lds_char* dst_tile, int r, const __bf16* row_ptr, int lane) {
  const int row = r + (lane >> 4);
  const int chunk = (lane & 15) ^ swz(row);
  const uint32_t m = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(dst_tile + r * kRowBytes));
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(row_ptr + chunk * 8), "s"(m) : "memory", "m0");
}
// Same copy with the address split into a wavefront-uniform 64-bit base (held in scalar registers) and a per-lane
// 32-bit byte offset that does not change from tile to tile: no vector arithmetic per copy.  `lds_dst` must be
// wavefront-uniform and already in a scalar register (e.g. derived from __builtin_amdgcn_readfirstlane).
__device__ __forceinline__ void dma16_sbase(const void* base_uniform, uint32_t lane_off_bytes, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off_bytes), "s"(base_uniform), "s"(lds_dst) : "memory", "m0");
}
// per-lane byte offset of the 16-byte chunk this lane fetches when rows r .. r+3 (r % 4 == 0) of a tile whose
// source rows are `row_stride_bytes` apart are copied by one dma16_sbase
__device__ __forceinline__ uint32_t dma_lane_offset(int r, int64_t row_stride_bytes, int lane) {
  const int row = r + (lane >> 4);
  return (uint32_t)(row * row_stride_bytes) + (uint32_t)((((lane & 15) ^ swz(row))) << 4);
}
__device__ __forceinline__ void dma_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Make the compiler wait, here, for the load that produces `v`.  Used on operand fragments that are
// loaded once before a loop: otherwise the first use inside the loop carries a conservative vmcnt wait
// on every iteration, which would also wait for the asynchronous tile copies issued in the loop.
__device__ __forceinline__ void settle(const bf16x8& v) { asm volatile("" : : "v"(v)); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// XCD-aware work mapping: consecutive workgroup ids go round-robin over the 8 XCDs, each
// with its own L2.  Giving XCD x the contiguous item range [x * per_xcd, (x+1) * per_xcd)
// keeps the workgroups that stream one KV head on one L2.
__device__ __forceinline__ int xcd_item(int block, int total_items) {
  const int per_xcd = (total_items + 7) >> 3;
  const int item = (block & 7) * per_xcd + (block >> 3);
  return item < total_items ? item : -1;
}
inline int xcd_grid(int total_items) { return ((total_items + 7) / 8) * 8; }

}  // namespace seco
