// Exit decision of one layer (Section 3.1), shared by the stand-alone combine kernel and by the QKV projection
// launch that carries the previous layer's decision along.
#pragma once

#include "ee_common.h"
#include "ee_epilogue.h"

namespace ee {

// Section 3.1 status rule for one sequence: an accepted sequence stays accepted (and is not re-checked);
// otherwise the confidence (or the forced exit layer) decides; the last acceptance of the batch raises `done`.
__device__ inline void decide_row(const IterState& s, int m, int B, int layer, float conf, float threshold,
                                  const int32_t* forced_exit_layer, float* conf_out) {
  if (ctl_load(s.status + m) != 0) {
    if (conf_out) conf_out[m] = __builtin_nanf("");
    return;
  }
  if (conf_out) conf_out[m] = conf;
  const bool accepted = forced_exit_layer ? (layer >= forced_exit_layer[m]) : (conf > threshold);
  if (!accepted) return;
  ctl_store(s.status + m, 1);
  ctl_store(s.exit_layer + m, layer);
  const int before = __hip_atomic_fetch_add(s.n_exited, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (before + 1 == B) {
    ctl_store(s.batch_exit_layer, layer);
    ctl_store(s.done, 1);
  }
}

// One workgroup of 256 threads merges the per-tile softmax statistics of row m into the confidence and applies
// the status rule.  red: 256 float4 of LDS.  layer == 0: final token selection only.
__device__ inline void combine_row(const CombineArgs& a, int m, float4* red) {
  if (a.left && ctl_load(a.left + m) != 0) return;   // left at an earlier layer: its token and exit layer stand
  HeadStat s = stat_empty();
  for (int i = threadIdx.x; i < a.n_parts; i += blockDim.x)
    s = stat_merge(s, stat_unpack(a.partials[(size_t)m * a.n_parts + i]), a.scale);
  red[threadIdx.x] = stat_pack(s);
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w)
      red[threadIdx.x] = stat_pack(stat_merge(stat_unpack(red[threadIdx.x]), stat_unpack(red[threadIdx.x + w]), a.scale));
    __syncthreads();
  }
  if (threadIdx.x != 0) return;
  s = stat_unpack(red[0]);
  if (a.argmax_out) a.argmax_out[m] = s.idx;
  if (a.layer == 0) return;
  float conf = 1.0f / s.sum;                                          // largest softmax probability
  if (a.conf_mode == 1) conf = (1.0f - expf(a.scale * (s.z2 - s.zmax))) / s.sum;  // top-1 minus top-2
  decide_row(a.s, m, a.B, a.layer, conf, a.threshold, a.forced_exit_layer, a.conf_out);
}

// Confidence of row m from one dot product (hidden states similarity, dedicated classifier) and the status rule.
__device__ inline void decide_from_dot(const DecideArgs& a, int m) {
  float conf;
  if (a.conf_mode == 2) {
    conf = a.dots[m] / (sqrtf(a.sq_a[m]) * sqrtf(a.sq_b[m]));
  } else {
    conf = 1.0f / (1.0f + expf(-(a.dots[m] * rsqrtf(a.sq_b[m] / (float)a.d + a.eps) + a.bias[0])));
  }
  decide_row(a.s, m, a.B, a.layer, conf, a.threshold, a.forced_exit_layer, a.conf_out);
}

}  // namespace ee
