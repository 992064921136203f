// fp32 projections (plain row-major weights): the small reference-shaped workload runs entirely in float.
// One wavefront computes one pair of output rows for every batch row: lanes stride over the contraction
// and a butterfly adds the 64 partial sums.  Not a throughput kernel; the bf16 path is.
#include <type_traits>

#include "ee_common.h"
#include "ee_epilogue.h"

namespace ee {
namespace {

constexpr int MC = 4;  // batch rows per pass

template <class Epi>
__global__ __launch_bounds__(256) void gemm_simple_kernel(SimpleShape g, Epi e, Pred pred) {
  if (pred_skip(pred)) return;
  const int lane = threadIdx.x & 63;
  const int pair = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pair >= g.n_rows / 2) return;
  const int s = g.pair_stride;
  const int f_lo = g.row_begin + (pair / s) * 2 * s + pair % s;
  const int f_hi = f_lo + s;
  const float* w_lo = g.w + (size_t)f_lo * g.K;
  const float* w_hi = g.w + (size_t)f_hi * g.K;
  for (int m0 = 0; m0 < g.M; m0 += MC) {
    float lo[MC], hi[MC];
#pragma unroll
    for (int i = 0; i < MC; ++i) lo[i] = hi[i] = 0.0f;
    for (int k = lane; k < g.K; k += 64) {
      const float a = w_lo[k], b = w_hi[k];
#pragma unroll
      for (int i = 0; i < MC; ++i) {
        const float x = m0 + i < g.M ? g.x[(size_t)(m0 + i) * g.K + k] : 0.0f;
        lo[i] = fmaf(a, x, lo[i]);
        hi[i] = fmaf(b, x, hi[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < MC; ++i)
#pragma unroll
      for (int x = 1; x < 64; x <<= 1) {
        lo[i] += __shfl_xor(lo[i], x);
        hi[i] += __shfl_xor(hi[i], x);
      }
    if (lane == 0) {
#pragma unroll
      for (int i = 0; i < MC; ++i) {
        const int m = m0 + i;
        if (m >= g.M) break;
        if constexpr (std::is_same<Epi, QkvEpi>::value) {
          epi_qkv<float>(e, m, f_lo, lo[i], hi[i]);
        } else if constexpr (std::is_same<Epi, AccEpi>::value) {
          epi_acc(e, m, f_lo, lo[i]);
          epi_acc(e, m, f_hi, hi[i]);
        } else if constexpr (std::is_same<Epi, GateUpEpi>::value) {
          epi_gateup<float>(e, m, f_lo, lo[i], hi[i]);
        } else {
          e.logits[(size_t)m * e.vocab + f_lo] = lo[i];
          e.logits[(size_t)m * e.vocab + f_hi] = hi[i];
        }
      }
    }
  }
}

template <class Epi>
void launch(const SimpleShape& g, const Epi& e, Pred pred, hipStream_t st) {
  const int pairs = g.n_rows / 2;
  hipLaunchKernelGGL((gemm_simple_kernel<Epi>), dim3((pairs + 3) / 4), dim3(256), 0, st, g, e, pred);
}

}  // namespace

void launch_simple_qkv(const SimpleShape& g, const QkvEpi& e, Pred pred, hipStream_t st) { launch(g, e, pred, st); }
void launch_simple_acc(const SimpleShape& g, const AccEpi& e, Pred pred, hipStream_t st) { launch(g, e, pred, st); }
void launch_simple_gateup(const SimpleShape& g, const GateUpEpi& e, Pred pred, hipStream_t st) { launch(g, e, pred, st); }
void launch_simple_lm(const SimpleShape& g, const LmEpi& e, Pred pred, hipStream_t st) { launch(g, e, pred, st); }

}  // namespace ee
