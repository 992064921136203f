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

// What one compute unit takes in when half of what it asks for comes from beyond its L2: every wavefront alternates
// 1 KiB loads from a stream of its own (read once, from HBM) with 1 KiB loads from a small buffer that every workgroup
// walks alike (its lines are in L2 after the first reader: the activation operand of a projection), D loads in flight
// per wavefront, two register sets so that the next D / 2 are requested before the current ones are consumed.
template <int D>
__global__ __launch_bounds__(256) void intake_kernel(const u32x4* own, size_t words_per_wave, const u32x4* common,
                                                     size_t common_mask, u32x4* sink, int pairs) {
  constexpr int H = D / 2;            // loads per register set: H / 2 from each source
  const int lane = threadIdx.x & 63, wave_in_wg = threadIdx.x >> 6;
  // pairs: workgroups whose ids differ by 8 (same XCD, same L2) read the same stream, as the two row blocks of a
  // column block of the ring projection kernel do: every byte of it then leaves HBM once and L2 twice
  const size_t piece = pairs ? (size_t)(blockIdx.x >> 4) * 8 + (blockIdx.x & 7) : blockIdx.x;
  const size_t wave = piece * 4 + wave_in_wg;
  const u32x4* q = own + wave * words_per_wave + lane;
  u32x4 a[H], b[H], acc = {0, 0, 0, 0};
  size_t c = (size_t)wave_in_wg * 64;   // the four wavefronts of a workgroup walk consecutive KiB of the common buffer
  auto issue = [&](u32x4 (&v)[H], size_t i) {
#pragma unroll
    for (int u = 0; u < H / 2; ++u) v[u] = __builtin_nontemporal_load(q + i + (size_t)u * 64);
#pragma unroll
    for (int u = 0; u < H / 2; ++u) {
      v[H / 2 + u] = common[((c + (size_t)u * 256) & common_mask) + lane];
    }
    c += (size_t)(H / 2) * 256;
  };
  auto eat = [&](const u32x4 (&v)[H]) {
#pragma unroll
    for (int u = 0; u < H; ++u) acc ^= v[u];
  };
  const size_t step = (size_t)(H / 2) * 64;
  const size_t n = words_per_wave / step;      // whole steps only
  if (n >= 2) {
    issue(a, 0);
    size_t i = 1;
    for (; i + 1 < n; i += 2) {
      issue(b, i * step);
      eat(a);
      issue(a, (i + 1) * step);
      eat(b);
    }
    eat(a);
  }
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 1u) sink[0] = acc;
}

// The inner loop of a 128 x 128 wavefront tile with nothing around it: per contraction step 16 MFMAs on 4 x 4
// accumulators and, if READS, the 4 + 4 operand fragments of the next step read from LDS (1 KiB each, the
// fragment order of the projection kernels) while the current step is multiplied.  Four wavefronts per
// workgroup, 96 KiB of LDS so that one workgroup runs per compute unit.  No global memory traffic in the loop.
template <bool READS>
__global__ __launch_bounds__(256) void mfma_tile_kernel(float* sink, int iters) {
  extern __shared__ u32x4 frag_lds[];   // 64 KiB are read: four stages of 16 fragments
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 64 * 1024 / 16; i += blockDim.x)
    frag_lds[i] = u32x4{0x3c003c00u + (unsigned)i, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  __syncthreads();
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;
  u32x4 fa[2][4], fb[2][4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    fa[0][a] = fa[1][a] = frag_lds[a * 64 + lane];
    fb[0][a] = fb[1][a] = frag_lds[(8 + a) * 64 + lane];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (READS) {
        const u32x4* st = frag_lds + (size_t)(((it * 2 + u) & 3) * 16) * 64 + lane;
#pragma unroll
        for (int a = 0; a < 4; ++a) fa[(u + 1) & 1][a] = st[((wave & 1) * 4 + a) * 64];
#pragma unroll
        for (int b = 0; b < 4; ++b) fb[(u + 1) & 1][b] = st[(8 + (wave >> 1) * 4 + b) * 64];
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[u & 1][a]),
                                                              __builtin_bit_cast(bf16x8, fb[u & 1][b]), acc[a][b], 0, 0, 0);
    }
  }
  float r = 0.0f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) r += acc[a][b][0] + acc[a][b][15];
  if (r == 1.2345f) sink[threadIdx.x] = r;   // practically never true; keeps the loop alive
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

int ee_calibration_intake(const void* own, size_t own_bytes, const void* common, size_t common_bytes, int32_t workgroups,
                          int32_t loads_in_flight, int32_t pairs, void* sink, void* stream) {
  if (!own || !common || !sink) EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_intake: NULL pointer");
  if (((reinterpret_cast<uintptr_t>(own) | reinterpret_cast<uintptr_t>(common)) & 15) || workgroups < 1 ||
      common_bytes < (64u << 10) || (common_bytes & (common_bytes - 1)) || own_bytes < (size_t)workgroups * 4 * (128u << 10) ||
      (pairs && (workgroups & 15)))
    EE_FAIL(EE_ERR_INVALID_ARG,
            "ee_calibration_intake: 16-byte aligned buffers, a power of two >= 64 KiB of common bytes, >= 128 KiB of own bytes per "
            "wavefront, a multiple of 16 workgroups with pairs");
  const size_t pieces = pairs ? (size_t)workgroups / 2 : (size_t)workgroups;
  const size_t words_per_wave = own_bytes / 16 / (pieces * 4) / 64 * 64;
  const size_t mask = common_bytes / 16 - 1 - 63;   // index of a 1 KiB row start: the low six bits come from the lane
  auto st = reinterpret_cast<hipStream_t>(stream);
  auto o = reinterpret_cast<const u32x4*>(own);
  auto cm = reinterpret_cast<const u32x4*>(common);
  auto sk = reinterpret_cast<u32x4*>(sink);
  switch (loads_in_flight) {
    case 8: hipLaunchKernelGGL(intake_kernel<8>, dim3(workgroups), dim3(256), 0, st, o, words_per_wave, cm, mask, sk, pairs); break;
    case 16: hipLaunchKernelGGL(intake_kernel<16>, dim3(workgroups), dim3(256), 0, st, o, words_per_wave, cm, mask, sk, pairs); break;
    case 32: hipLaunchKernelGGL(intake_kernel<32>, dim3(workgroups), dim3(256), 0, st, o, words_per_wave, cm, mask, sk, pairs); break;
    case 48: hipLaunchKernelGGL(intake_kernel<48>, dim3(workgroups), dim3(256), 0, st, o, words_per_wave, cm, mask, sk, pairs); break;
    default: EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_intake: loads_in_flight must be 8, 16, 32 or 48");
  }
  EE_HIP(hipGetLastError());
  return EE_OK;
}

int ee_calibration_mfma_tile(int32_t workgroups, int32_t steps, int32_t lds_fragment_reads, float* sink, void* stream) {
  if (!sink || workgroups < 1 || steps < 2 || (steps & 1) || (lds_fragment_reads != 0 && lds_fragment_reads != 8))
    EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_mfma_tile: steps must be even and >= 2, lds_fragment_reads 0 or 8");
  const size_t lds = 96 * 1024;
  auto st = reinterpret_cast<hipStream_t>(stream);
  if (lds_fragment_reads) {
    EE_HIP(hipFuncSetAttribute((const void*)mfma_tile_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(mfma_tile_kernel<true>, dim3(workgroups), dim3(256), lds, st, sink, steps / 2);
  } else {
    EE_HIP(hipFuncSetAttribute((const void*)mfma_tile_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(mfma_tile_kernel<false>, dim3(workgroups), dim3(256), lds, st, sink, steps / 2);
  }
  EE_HIP(hipGetLastError());
  return EE_OK;
}

}  // extern "C"
