// One-time reordering of a plain bf16 weight matrix into the tile order the MFMA projections stream.
#include "ee_common.h"

namespace ee {
namespace {

// One thread per 16-byte group: packed[((nt * k_steps + ks) * 64 + lane) * 8 + j] =
//   w[row(nt, lane % 32)][ks * 16 + (lane / 32) * 8 + j]
__global__ void pack_weight_kernel(const bf16_t* w, int n_in, int pair_stride, size_t n_groups, bf16_t* packed) {
  const size_t gidx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gidx >= n_groups) return;
  const int k_steps = n_in >> 4;
  const int lane = (int)(gidx & 63);
  const size_t tile = gidx >> 6;
  const int ks = (int)(tile % k_steps);
  const int nt = (int)(tile / k_steps);
  const int r = lane & 31;
  const int row = packed_row_lo(nt, r & 15, pair_stride) + (r >> 4) * pair_stride;
  const bf16_t* src = w + (size_t)row * n_in + ks * 16 + (lane >> 5) * 8;
  *reinterpret_cast<uint4*>(packed + gidx * 8) = *reinterpret_cast<const uint4*>(src);
}

}  // namespace

void launch_pack_weight(const bf16_t* w, int n_out, int n_in, int pair_stride, bf16_t* packed, hipStream_t st) {
  const size_t n_groups = (size_t)n_out * n_in / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n_groups + 255) / 256)), dim3(256), 0, st, w, n_in, pair_stride,
                     n_groups, packed);
}

}  // namespace ee
