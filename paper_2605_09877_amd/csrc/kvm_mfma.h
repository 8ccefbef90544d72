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

#include "kvm_device.h"

namespace kvm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kHeadDim = 128;
constexpr int kTileKeys = 64;   // keys (or state rows) per LDS tile
constexpr int kKStride = 136;   // elements per K-tile row in LDS (272 B: 16-byte aligned, padded)
constexpr int kVtStride = 68;   // elements per V^T-tile row in LDS (136 B)

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// row of D held in element v by lane half g
__device__ __forceinline__ int mfma_row(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

// Exchange between lanes i and i + 32 on the vector ALU (v_permlane32_swap; no LDS round trip):
// of the two results one is the lane's own value and the other its partner's, so a commutative
// combination of both is the combination of own and partner for every lane.
__device__ __forceinline__ float xhalf_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
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

// ---------------------------------------------------------------------------------------------
// Swizzled 64 x 128 bf16 tiles filled by direct global -> LDS loads (no register staging).
//
// global_load_lds with 16 bytes per lane writes lane i's chunk to lds_base + 16*i, so one wave
// instruction fills 1 KiB = four unpadded 256-byte rows.  Which global chunk a lane fetches is
// free, so a row's sixteen 16-byte chunks are stored permuted: chunk q of row r sits in slot
// q ^ swz(r).  Rows are 256 B apart (a multiple of the bank cycle), the permutation is what keeps
// the fragment reads below conflict-free.
//   K tiles (read with ds_read_b128, lanes walk rows):        swz(r) = r & 15
//   V tiles (read with ds_read_b64_tr_b16, 4 rows x 32 B):    swz(r) = 2 * (r & 3)
typedef short v4i16 __attribute__((ext_vector_type(4)));
#define KVM_LDS_V4(p) ((__attribute__((address_space(3))) v4i16 *)(p))
#define KVM_LDS_VOID(p) ((__attribute__((address_space(3))) void *)(p))

constexpr int kTileElems = kTileKeys * kHeadDim;  // 8192 bf16 = 16 KiB

// Per-lane byte offsets of a lane's 16-byte chunk within its row, for the four loads a wave
// issues per tile (the chunk permutation depends on the row, see above).
struct DmaLane {
  uint32_t rl;       // row of the lane within a 4-row block
  uint32_t kcol[4];  // K layout, loads n = 0..3
  uint32_t vcol;     // V layout, same for all four loads
};
__device__ __forceinline__ DmaLane dma_lane(int lane) {
  DmaLane d;
  const int rl = lane >> 4, c16 = lane & 15;
  d.rl = (uint32_t)rl;
#pragma unroll
  for (int n = 0; n < 4; ++n) d.kcol[n] = (uint32_t)(16 * (c16 ^ (4 * n + rl)));
  d.vcol = (uint32_t)(16 * (c16 ^ (2 * rl)));
  return d;
}

// One 16-byte-per-lane direct load: lane i's chunk from sbase + voff lands at lds_addr + 16*i.
// Written as an instruction sequence of its own rather than through the compiler's builtin: the
// compiler cannot see that such a load into one tile buffer leaves the other buffer alone, and
// puts a full wait for it in front of the next LDS read, which would undo the prefetch.  The
// kernels wait themselves (s_waitcnt vmcnt(0) ahead of the barrier that publishes a tile).
__device__ __forceinline__ void dma16(const char *sbase, uint32_t voff, uint32_t lds_addr) {
  // Both are wave-uniform by construction; say so where the compiler cannot prove it.  The
  // builtin returns a signed int: each half goes through uint32_t, or a low half with its top
  // bit set would be sign-extended over the high half and the load would go astray.
  lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
  const uint64_t sb = (uint64_t)sbase;
  const uint32_t sb_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)sb);
  const uint32_t sb_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(sb >> 32));
  sbase = (const char *)(((uint64_t)sb_hi << 32) | (uint64_t)sb_lo);
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(sbase), "s"(lds_addr)
      : "memory", "m0");
}
// Four such loads from one scalar base into four consecutive 1-KiB pieces of LDS: M0 is written
// once, load n carries the immediate 1024 * n, which the hardware adds to the LDS address and to
// the global address alike.  One instruction sequence, so nothing can come between the write of
// M0 and the loads that depend on it.
__device__ __forceinline__ void dma16x4(const char *sbase, uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3,
                                        uint32_t lds_addr) {
  lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
  const uint64_t sb = (uint64_t)sbase;
  const uint32_t sb_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)sb);
  const uint32_t sb_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(sb >> 32));
  sbase = (const char *)(((uint64_t)sb_hi << 32) | (uint64_t)sb_lo);
  asm volatile(
      "s_mov_b32 m0, %5\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %4\n\t"
      "global_load_lds_dwordx4 %1, %4 offset:1024\n\t"
      "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
      "global_load_lds_dwordx4 %3, %4 offset:3072"
      :
      : "v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(sbase), "s"(lds_addr)
      : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void *p) {
  return (uint32_t)(uintptr_t)KVM_LDS_VOID(p);
}

// The kNW waves of a workgroup share a tile's sixteen 1-KiB loads: wave w issues loads
// bi = (16/kNW)*w + n, each fetching rows 4*bi .. 4*bi+3; kVSwz: V layout.  `base` (bytes) and
// `stride` (bytes between rows) are wave-uniform; the per-lane part is a 32-bit byte offset, so
// each load is scalar base + vector offset.  lds_tile_addr: LDS byte address of the tile buffer.  Rows at or beyond rows_valid repeat the last valid
// row (only looked at when the tile is not full).
template <bool kVSwz, int kNW>
__device__ __forceinline__ void tile_dma(const char *base, uint32_t stride, int rows_valid,
                                         uint32_t lds_tile_addr, int wave, const DmaLane &dl) {
  constexpr int kPer = 16 / kNW;
  if (rows_valid >= kTileKeys) {
    const uint32_t lane_row = dl.rl * stride;
    if constexpr (kPer == 4) {
      // the wave's four loads share one scalar base and one write of M0; the immediate that
      // moves load n to its piece of LDS also moves its global address, so the per-lane offset
      // takes that back out (a row is at least 256 bytes: 4 * n * stride >= 1024 * n)
      const int bi0 = kPer * wave;
      const uint32_t step = 4u * stride - 1024u;
      const uint32_t v0 = lane_row + (kVSwz ? dl.vcol : dl.kcol[0]);
      const uint32_t v1 = lane_row + (kVSwz ? dl.vcol : dl.kcol[1]) + step;
      const uint32_t v2 = lane_row + (kVSwz ? dl.vcol : dl.kcol[2]) + 2u * step;
      const uint32_t v3 = lane_row + (kVSwz ? dl.vcol : dl.kcol[3]) + 3u * step;
      dma16x4(base + (uint32_t)(4 * bi0) * stride, v0, v1, v2, v3, lds_tile_addr + (uint32_t)bi0 * 1024u);
    } else {
#pragma unroll
      for (int n = 0; n < kPer; ++n) {
        const int bi = kPer * wave + n;
        // the K chunk permutation depends on bi % 4: 2*(wave%2) + n for eight waves (a
        // wave-uniform choice between two precomputed values)
        const uint32_t kcol = (wave & 1) ? dl.kcol[2 + n] : dl.kcol[n];
        dma16(base + (uint32_t)(4 * bi) * stride, lane_row + (kVSwz ? dl.vcol : kcol),
              lds_tile_addr + (uint32_t)bi * 1024u);
      }
    }
  } else {
#pragma unroll
    for (int n = 0; n < kPer; ++n) {
      const int bi = kPer * wave + n;
      const uint32_t kcol = kPer == 4 ? dl.kcol[n] : ((wave & 1) ? dl.kcol[2 + n] : dl.kcol[n]);
      int r = 4 * bi + (int)dl.rl;
      r = r < rows_valid ? r : rows_valid - 1;
      dma16(base, (uint32_t)r * stride + (kVSwz ? dl.vcol : kcol), lds_tile_addr + (uint32_t)bi * 1024u);
    }
  }
}

// Per-lane LDS element offsets of the K fragments (one per 16-channel step; the row block adds
// a constant): row = lane%32 (+32*blk), chunk (2*ks + lane/32) ^ (row & 15).
__device__ __forceinline__ void ktile_offsets(int lane, uint32_t (&off)[8]) {
  const int l32 = lane & 31;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) off[ks] = (uint32_t)(l32 * kHeadDim + 8 * ((2 * ks + (lane >> 5)) ^ (l32 & 15)));
}
__device__ __forceinline__ bf16x8 ktile_frag(const uint16_t *lds_tile, const uint32_t (&off)[8], int blk, int ks) {
  Frag8 f;
  f.q = *reinterpret_cast<const uint4 *>(lds_tile + off[ks] + 32 * blk * kHeadDim);
  return f.v;
}

// A-operand fragment of V^T from a swizzled row-major V tile, through the transposing LDS read:
// lane gets channel 32*dblk + lane%32 and keys 16*ks + 4*g + {0..3}, 16*ks + 8 + 4*g + {0..3}
// (g = lane/32) -- the key order in which a lane holds P^T after the first product.
// ds_read_b64_tr_b16: within 16 lanes, result element t of lane i = element i%4 of the 8 bytes
// addressed by lane 4*t + i/4.  So lane j addresses key row K0 + j/4, channels dbase + 4*(j%4).
// The per-lane part of the address depends on dblk only through its low bit (it meets the row
// swizzle in one bit), so two offsets cover all sixteen fragments; the rest are constants.
__device__ __forceinline__ void vtile_offsets(int lane, uint32_t (&off)[2]) {
  const int j = lane & 15, t = j >> 2, c = j & 3;
  const int g = lane >> 5, half = (lane >> 4) & 1;
#pragma unroll
  for (int odd = 0; odd < 2; ++odd) {
    const int q = 4 * odd + 2 * half + (c >> 1);
    off[odd] = (uint32_t)((4 * g + t) * kHeadDim + 8 * (q ^ (2 * t)) + 4 * (c & 1));
  }
}
__device__ __forceinline__ bf16x8 vtile_frag(const uint16_t *lds_tile, const uint32_t (&off)[2], int dblk, int ks) {
  const uint16_t *p = lds_tile + off[dblk & 1] + 16 * ks * kHeadDim + 64 * (dblk >> 1);
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(KVM_LDS_V4(p));
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(KVM_LDS_V4(p + 8 * kHeadDim));
  Frag8 f;
  f.d[0] = __builtin_bit_cast(uint2, lo);
  f.d[1] = __builtin_bit_cast(uint2, hi);
  return f.v;
}

}  // namespace kvm
