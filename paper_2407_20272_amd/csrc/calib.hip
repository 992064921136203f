// Measurement helpers (not part of the decode path): kernels of known traffic / known arithmetic against which the
// chip's attainable rates are measured on the box a benchmark runs on.
#include "ee_common.h"

namespace ee {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Plain streaming read: every wavefront owns one contiguous piece of the buffer and walks it 1 KiB per load
// instruction with 16 loads (16 KiB) in flight: the access pattern of the weight streams.  Nothing is written
// (the guard below is practically never true; it keeps the loads alive).
__global__ __launch_bounds__(256) void read_kernel(const u32x4* p, size_t n, u32x4* sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const size_t nwaves = (size_t)gridDim.x * (blockDim.x >> 6);
  const size_t per = n / nwaves / 64 * 64;   // 16-byte words per wavefront, whole 1 KiB rows
  const u32x4* q = p + wave * per + lane;
  u32x4 acc = {0, 0, 0, 0};
  size_t i = 0;
  for (; i + 16 * 64 <= per; i += 16 * 64) {
    u32x4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load(q + i + u * 64);
#pragma unroll
    for (int u = 0; u < 16; ++u) acc ^= v[u];
  }
  for (; i + 64 <= per; i += 64) acc ^= q[i];
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 1u) sink[0] = acc;
}

// Back-to-back 32x32x16 bf16 MFMAs on registers, four independent accumulators per wavefront, no memory traffic.
__global__ __launch_bounds__(256) void mfma_kernel(float* sink, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (bf16_t)(threadIdx.x * 0.001f + i);
    b[i] = (bf16_t)(i * 0.5f);
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.0f;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 1.2345f) sink[threadIdx.x] = s;   // never true for these operands; keeps the loop alive
}

}  // namespace
}  // namespace ee

using namespace ee;

extern "C" {

int ee_calibration_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream) {
  if (!src || !sink) EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_read: NULL pointer");
  if ((reinterpret_cast<uintptr_t>(src) & 15) || workgroups < 1 || bytes < (size_t)workgroups * 4 * 1024)
    EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_read: src must be 16-byte aligned, bytes at least 4 KiB per workgroup");
  hipLaunchKernelGGL(read_kernel, dim3(workgroups), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<const u32x4*>(src), bytes / 16, reinterpret_cast<u32x4*>(sink));
  EE_HIP(hipGetLastError());
  return EE_OK;
}

int ee_calibration_mfma(int32_t workgroups, int32_t iterations, float* sink, void* stream) {
  if (!sink || workgroups < 1 || iterations < 1) EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_mfma: bad argument");
  hipLaunchKernelGGL(mfma_kernel, dim3(workgroups), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), sink, iterations);
  EE_HIP(hipGetLastError());
  return EE_OK;
}

}  // extern "C"
