// Two small measurement kernels: what this GPU attains on a dense bf16 MFMA stream that never
// leaves the registers, and on a plain device-to-device copy.  The benchmark reports kernel
// rates against these attained figures as well as against the published peaks.
#include "kvp_internal.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kProbeThreads = 512;      // eight waves: two per SIMD, as in the attention kernel
constexpr int kChains = 4;              // independent accumulators per wave
constexpr int kMfmaPerIter = 16;

__global__ void __launch_bounds__(kProbeThreads)
probe_mfma_kernel(float* out, int iters) {
  const int lane = threadIdx.x & 63;
  // operands of ordinary magnitude (the matrix pipe draws more power on real data than on zeros)
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.01f * (float)((lane * 7 + i * 3) % 61 - 30));
    b[i] = (__bf16)(0.02f * (float)((lane * 5 + i * 11) % 53 - 26));
  }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kMfmaPerIter; ++m)
      acc[m % kChains] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m % kChains], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[c][r];
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

__global__ void __launch_bounds__(256)
probe_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace kvp

extern "C" {

int kvp_probe_mfma(void* device_out, size_t out_bytes, int32_t workgroups, int32_t iters, void* stream,
                   double* flops) {
  using namespace kvp;
  if (!device_out || workgroups < 1 || iters < 1 || !flops) return KVP_EINVAL;
  if (out_bytes < (size_t)workgroups * kProbeThreads * sizeof(float)) return KVP_ENOMEM;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<float*>(device_out), iters);
  if (hipGetLastError() != hipSuccess) return KVP_EDEVICE;
  // one 32x32x16 product is 2 * 32 * 32 * 16 flops, one per wave and instruction
  *flops = 2.0 * 32 * 32 * 16 * kMfmaPerIter * (double)iters * (kProbeThreads / 64) * (double)workgroups;
  return KVP_OK;
}

int kvp_probe_copy(void* device_dst, const void* device_src, size_t bytes, int32_t workgroups, void* stream) {
  using namespace kvp;
  if (!device_dst || !device_src || workgroups < 1 || bytes % 16 != 0 || bytes == 0) return KVP_EINVAL;
  if (reinterpret_cast<uintptr_t>(device_dst) % 16 || reinterpret_cast<uintptr_t>(device_src) % 16) return KVP_EINVAL;
  hipLaunchKernelGGL(probe_copy_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint4*>(device_dst), static_cast<const uint4*>(device_src), bytes / 16);
  return hipGetLastError() == hipSuccess ? KVP_OK : KVP_EDEVICE;
}

}  // extern "C"
