// Tile helpers shared by the two backward kernels of libsegattn (segattn_bwd_dq.hip,
// segattn_bwd_mfma.hip): the swizzled [32 x D] LDS tile and the MFMA operand reads from it.
#pragma once
#include "segattn_work.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

constexpr int kBwdStep = 32;
constexpr float kLog2e = 1.4426950408889634f;

// A [32 x D] bf16 tile in LDS: dense rows, the 16-byte chunks of a row XOR-swizzled with a
// function of the row chosen so that both access patterns are free of bank conflicts: the row
// reads (16 lanes = 16 consecutive rows at one logical chunk) and the transposing reads (16
// lanes = 4 consecutive rows x 32 contiguous bytes).
template <int D>
struct BwdTile {
  static constexpr int kRowBytes = 2 * D;
  static constexpr int kBytes = kBwdStep * kRowBytes;
  static constexpr int kChunks = D / 8;                 // 16-byte chunks per row
  static constexpr int kLoads = kBwdStep * kChunks / 256;  // chunks per thread per tile
  __device__ static constexpr int swz(int row) {
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    const int a = row >> 1;  // 128-byte rows: two rows share a 64-bank line
    return ((a & 1) << 2) | (((a >> 2) & 1) << 1) | ((a >> 1) & 1);
  }
  // byte offset of logical chunk `chunk` of row `row`
  __device__ static constexpr int at(int row, int chunk) { return row * kRowBytes + ((chunk ^ swz(row)) << 4); }
};

// acc += A . B
__device__ inline void mma_acc(f32x16 &acc, const bf16x8 a, const bf16x8 b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}

// Move four dwords into accumulation registers; the result is used as an MFMA operand only.
__device__ inline bf16x8 park(const uint4 v) {
  int a0, a1, a2, a3;
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a0) : "v"(v.x));
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a1) : "v"(v.y));
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a2) : "v"(v.z));
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a3) : "v"(v.w));
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const i32x4 q4 = {a0, a1, a2, a3};
  return __builtin_bit_cast(bf16x8, q4);
}

// A operand of a transposed product from a row-major [32 x D] tile: for the 32-column block nb
// and the 16-row half h2, k-slot e of half-wave hi is tile row 16 h2 + 8 (e/4) + 4 hi + e%4 (the
// accumulator layout of the score tile) and the lane's operand row is tile column 32 nb + lane%32.
template <int D>
__device__ inline bf16x8 read_transposed(const unsigned char *tile, int lane, int nb, int h2) {
  using T = BwdTile<D>;
  const int hi = lane >> 5, i16 = lane & 15, g16 = (lane >> 4) & 1;
  const int row = 4 * hi + (i16 >> 2) + 16 * h2;
  const int chunk = 4 * nb + 2 * g16 + ((i16 & 3) >> 1), half = 8 * (i16 & 1);
  const LDS_AS s16x4 *p0 = (const LDS_AS s16x4 *)(tile + T::at(row, chunk) + half);
  const LDS_AS s16x4 *p1 = (const LDS_AS s16x4 *)(tile + T::at(row + 8, chunk) + half);
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)p0);
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)p1);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

// A operand of a row product: tile row lane%32, elements 16 kc + 8 (lane/32) .. +7
template <int D>
__device__ inline bf16x8 read_row(const unsigned char *tile, int lane, int kc) {
  using T = BwdTile<D>;
  return *(const bf16x8 *)(tile + T::at(lane & 31, 2 * kc + (lane >> 5)));
}

}  // namespace segattn
