// Measured peaks of the GPU the library runs on, for rooflines: a bf16 matrix-core microkernel
// that touches registers only, and a streaming copy.  Measurement aids, not part of the method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kvm.h"
#include "kvm_mfma.h"

namespace kvm {
namespace {

__global__ __launch_bounds__(256, 2) void mfma_peak_kernel(int iters, float *sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)(threadIdx.x % 7);
    b[i] = (__bf16)(float)(threadIdx.x % 5);
  }
  f32x16 c0 = {0.f}, c1 = {0.f}, c2 = {0.f}, c3 = {0.f};
  for (int it = 0; it < iters; ++it) {  // four independent accumulation chains per wave
    c0 = mfma32(a, b, c0);
    c1 = mfma32(a, b, c1);
    c2 = mfma32(a, b, c2);
    c3 = mfma32(a, b, c3);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 12345.678f) sink[0] = s;  // keeps the loop alive; never true
}

__global__ __launch_bounds__(256) void copy_peak_kernel(const uint4 *src, uint4 *dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

constexpr int kInFlight = 8;
// Read-only stream: what a kernel that reads far more than it writes (the decode attention) can
// be held against.  Eight 16-byte loads of a thread are in flight together (a grid stride apart,
// so every load instruction of a wave covers 1 KiB of consecutive bytes); the loaded words are
// folded together and the store never happens.
__global__ __launch_bounds__(256) void read_peak_kernel(const uint4 *src, size_t n, uint32_t *sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t acc = 0;
  for (size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x; i0 < n; i0 += stride * kInFlight) {
    uint4 x[kInFlight];
#pragma unroll
    for (int q = 0; q < kInFlight; ++q) x[q] = i0 + q * stride < n ? src[i0 + q * stride] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int q = 0; q < kInFlight; ++q) acc ^= x[q].x ^ x[q].y ^ x[q].z ^ x[q].w;
  }
  if (acc == 0x9e3779b9u && n == 1) sink[0] = acc;  // keeps the loads alive; not taken for the sizes measured
}

int timed(hipStream_t st, hipEvent_t a, hipEvent_t b, float *ms) {
  if (hipEventRecord(b, st) != hipSuccess || hipEventSynchronize(b) != hipSuccess) return KVM_ERR_HIP;
  return hipEventElapsedTime(ms, a, b) == hipSuccess ? KVM_OK : KVM_ERR_HIP;
}

}  // namespace
}  // namespace kvm

extern "C" int kvm_measure_mfma_bf16_peak(int iters, void *scratch, double *tflops, void *stream_) {
  if (iters <= 0 || !scratch || !tflops) return KVM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream_;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return KVM_ERR_HIP;
  const int wgs = 2048;
  hipLaunchKernelGGL(kvm::mfma_peak_kernel, dim3(wgs), dim3(256), 0, st, 64, (float *)scratch);  // warm-up
  int rc = hipEventRecord(a, st) == hipSuccess ? KVM_OK : KVM_ERR_HIP;
  hipLaunchKernelGGL(kvm::mfma_peak_kernel, dim3(wgs), dim3(256), 0, st, iters, (float *)scratch);
  float ms = 0.f;
  if (rc == KVM_OK) rc = kvm::timed(st, a, b, &ms);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (rc != KVM_OK) return rc;
  *tflops = (double)wgs * 4 * iters * 4 * 2.0 * 32 * 32 * 16 / (ms * 1e-3) * 1e-12;
  return KVM_OK;
}

extern "C" int kvm_measure_copy_peak(const void *src, void *dst, size_t bytes, double *gbs, void *stream_) {
  if (!src || !dst || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15) || !gbs)
    return KVM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream_;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return KVM_ERR_HIP;
  const size_t n = bytes / 16;
  const unsigned wgs = 32768;
  hipLaunchKernelGGL(kvm::copy_peak_kernel, dim3(wgs), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, n);
  int rc = hipEventRecord(a, st) == hipSuccess ? KVM_OK : KVM_ERR_HIP;
  const int reps = 5;
  for (int i = 0; i < reps; ++i)
    hipLaunchKernelGGL(kvm::copy_peak_kernel, dim3(wgs), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, n);
  float ms = 0.f;
  if (rc == KVM_OK) rc = kvm::timed(st, a, b, &ms);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (rc != KVM_OK) return rc;
  *gbs = 2.0 * (double)bytes * reps / (ms * 1e-3) * 1e-9;
  return KVM_OK;
}

extern "C" int kvm_measure_read_peak(const void *src, size_t bytes, void *scratch, double *gbs, void *stream_) {
  if (!src || !scratch || bytes < 32 || (bytes & 15) || ((uintptr_t)src & 15) || !gbs) return KVM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream_;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return KVM_ERR_HIP;
  const size_t n = bytes / 16;
  const unsigned wgs = 8192;
  hipLaunchKernelGGL(kvm::read_peak_kernel, dim3(wgs), dim3(256), 0, st, (const uint4 *)src, n, (uint32_t *)scratch);
  int rc = hipEventRecord(a, st) == hipSuccess ? KVM_OK : KVM_ERR_HIP;
  const int reps = 5;
  for (int i = 0; i < reps; ++i)
    hipLaunchKernelGGL(kvm::read_peak_kernel, dim3(wgs), dim3(256), 0, st, (const uint4 *)src, n, (uint32_t *)scratch);
  float ms = 0.f;
  if (rc == KVM_OK) rc = kvm::timed(st, a, b, &ms);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (rc != KVM_OK) return rc;
  *gbs = (double)bytes * reps / (ms * 1e-3) * 1e-9;
  return KVM_OK;
}
