// Device-side helpers: I/O element types, bf16 conversion, 64-lane wavefront reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvm {

constexpr int kWave = 64;

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits) {
  return __uint_as_float(bits << 16);
}

// Round to nearest, ties to even.  Inputs here are finite.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Two floats to a pair of bf16 (round to nearest even) with the hardware conversion.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

template <typename T>
struct Io;
template <>
struct Io<float> {
  static constexpr int kVec = 4;  // elements per 16-byte access
  __device__ static __forceinline__ float load(const float *p) { return *p; }
  __device__ static __forceinline__ void store(float *p, float v) { *p = v; }
  // the value a double becomes when it is materialised in this dtype
  __device__ static __forceinline__ float round_from(double v) { return (float)v; }
};
template <>
struct Io<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load(const bf16_t *p) { return bf16_bits_to_float(p->bits); }
  __device__ static __forceinline__ void store(bf16_t *p, float v) { p->bits = float_to_bf16_bits(v); }
  __device__ static __forceinline__ float round_from(double v) {
    return bf16_bits_to_float(float_to_bf16_bits((float)v));
  }
};

// 16 bytes of consecutive elements as floats (4 fp32 or 8 bf16); p is 16-byte aligned.
template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
  static constexpr int kN = 4;
  __device__ static __forceinline__ void load(const float *p, float (&f)[4]) {
    const float4 x = *reinterpret_cast<const float4 *>(p);
    f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w;
  }
  __device__ static __forceinline__ void store(float *p, const float (&f)[4]) {
    *reinterpret_cast<float4 *>(p) = make_float4(f[0], f[1], f[2], f[3]);
  }
};
template <>
struct Vec16<bf16_t> {
  static constexpr int kN = 8;
  __device__ static __forceinline__ void load(const bf16_t *p, float (&f)[8]) {
    const uint4 x = *reinterpret_cast<const uint4 *>(p);
    const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(wds[i] << 16);
      f[2 * i + 1] = __uint_as_float(wds[i] & 0xffff0000u);
    }
  }
  __device__ static __forceinline__ void store(bf16_t *p, const float (&f)[8]) {
    uint32_t wds[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) wds[i] = pack_bf16(f[2 * i], f[2 * i + 1]);
    *reinterpret_cast<uint4 *>(p) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
  }
};

// The floats of 16 bytes already in registers (4 fp32 or 8 bf16).
template <typename T>
__device__ __forceinline__ void unpack16(const uint4 &x, float (&f)[Vec16<T>::kN]);
template <>
__device__ __forceinline__ void unpack16<float>(const uint4 &x, float (&f)[4]) {
  f[0] = __uint_as_float(x.x); f[1] = __uint_as_float(x.y); f[2] = __uint_as_float(x.z); f[3] = __uint_as_float(x.w);
}
template <>
__device__ __forceinline__ void unpack16<bf16_t>(const uint4 &x, float (&f)[8]) {
  const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(wds[i] << 16);
    f[2 * i + 1] = __uint_as_float(wds[i] & 0xffff0000u);
  }
}

// All-reduce sums on the vector ALU, without the LDS crossbar: four DPP steps inside a row of 16
// lanes (partners lane^1, lane^2, then the mirror images within 8 and within 16 lanes, which pair
// up the partial sums just as well), then the row exchanges v_permlane16_swap and
// v_permlane32_swap.  A swap of a register with itself returns the lane's own value and its
// partner's; their sum is the same number, added in the same order, in both lanes, so every lane
// of a group ends with the identical result.
template <int kCtrl>
__device__ __forceinline__ float dpp_get(float x) {
  return __uint_as_float(__builtin_amdgcn_mov_dpp(__float_as_uint(x), kCtrl, 0xF, 0xF, true));
}
template <int kCtrl>
__device__ __forceinline__ double dpp_get(double x) {
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  const uint32_t lo = __builtin_amdgcn_mov_dpp((uint32_t)b, kCtrl, 0xF, 0xF, true);
  const uint32_t hi = __builtin_amdgcn_mov_dpp((uint32_t)(b >> 32), kCtrl, 0xF, 0xF, true);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
template <bool k32>
__device__ __forceinline__ float swap_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = k32 ? __builtin_amdgcn_permlane32_swap(u, u, false, false)
                     : __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
template <bool k32>
__device__ __forceinline__ double swap_sum(double x) {
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  const uint32_t lo = (uint32_t)b, hi = (uint32_t)(b >> 32);
  const auto l = k32 ? __builtin_amdgcn_permlane32_swap(lo, lo, false, false)
                     : __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
  const auto h = k32 ? __builtin_amdgcn_permlane32_swap(hi, hi, false, false)
                     : __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
  return __longlong_as_double((long long)(((uint64_t)h[0] << 32) | l[0])) +
         __longlong_as_double((long long)(((uint64_t)h[1] << 32) | l[1]));
}

// Sum over aligned groups of kLanes adjacent lanes (8, 16, 32 or 64), in every lane of the group.
template <int kLanes, typename V>
__device__ __forceinline__ V group_sum(V x) {
  static_assert(kLanes == 8 || kLanes == 16 || kLanes == 32 || kLanes == 64, "group size");
  x += dpp_get<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_get<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_get<0x141>(x);  // row_half_mirror
  if (kLanes >= 16) x += dpp_get<0x140>(x);  // row_mirror
  if (kLanes >= 32) x = swap_sum<false>(x);
  if (kLanes >= 64) x = swap_sum<true>(x);
  return x;
}

template <typename V>
__device__ __forceinline__ V wave_sum(V x) {
  return group_sum<64>(x);
}

template <typename V>
__device__ __forceinline__ V wave_max(V x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    V y = __shfl_xor(x, o, kWave);
    x = y > x ? y : x;
  }
  return x;
}

}  // namespace kvm
