// gfx950 matrix-core helpers for the bf16 / head_dim-128 kernels.
//
// v_mfma_f32_32x32x16_bf16 computes D[32x32] += A[32x16] * B[16x32] per 64-lane wave.
// Operand layout (lane = 32*g + i, g in {0,1}):
//   A: lane holds row i, eight consecutive k's of half g        (8 bf16)
//   B: lane holds column i, the same eight k's                   (8 bf16)
//   D: lane holds column i; element v (0..15) is row 8*(v/4) + 4*g + v%4
// Only the pairing of A's and B's k slots matters for the product, so both operands are always
// gathered with one and the same slot -> k map.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;

constexpr int kHeadDim = 128;
constexpr int kTileKeys = 64;   // keys (or state rows) per LDS tile
constexpr int kKStride = 136;   // elements per K-tile row in LDS (272 B: 16-byte aligned, padded)
constexpr int kVtStride = 68;   // elements per V^T-tile row in LDS (136 B)

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// row of D held in element v by lane half g
__device__ __forceinline__ int mfma_row(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

union Frag8 {
  bf16x8 v;
  uint4 q;
  uint2 d[2];
  uint32_t w[4];
};

// Stage a 64 x 128 bf16 tile (row-major in global memory, `stride` elements between rows) in
// registers: thread t takes rows 16*p + t/16 (p = 0..3), columns 8*(t%16) .. +7.  Rows at or
// beyond `rows_valid` repeat the last valid row (they are masked by the caller).
__device__ __forceinline__ void tile_rows_load(const uint16_t *base, int64_t stride, int rows_valid,
                                               int tid, uint4 (&r)[4]) {
  const int c8 = (tid & 15) * 8;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int row = 16 * p + (tid >> 4);
    row = row < rows_valid ? row : rows_valid - 1;
    r[p] = *reinterpret_cast<const uint4 *>(base + (int64_t)row * stride + c8);
  }
}

__device__ __forceinline__ void tile_rows_to_lds(uint16_t *lds, int tid, const uint4 (&r)[4]) {
  const int c8 = (tid & 15) * 8;
#pragma unroll
  for (int p = 0; p < 4; ++p)
    *reinterpret_cast<uint4 *>(lds + (16 * p + (tid >> 4)) * kKStride + c8) = r[p];
}

// A-operand fragment of a row-major LDS tile: row = 32*blk + lane%32, k = 16*ks + 8*(lane/32) ..
__device__ __forceinline__ bf16x8 tile_rows_frag(const uint16_t *lds, int blk, int ks, int lane) {
  Frag8 f;
  f.q = *reinterpret_cast<const uint4 *>(lds + (32 * blk + (lane & 31)) * kKStride + 16 * ks +
                                         8 * (lane >> 5));
  return f.v;
}

}  // namespace kvm
