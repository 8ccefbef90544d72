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

template <typename V>
__device__ __forceinline__ V wave_sum(V x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
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
