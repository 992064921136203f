// Small kernels of the decode step: state reset, embedding gather, normalisation, exit-head decision.
#include "ee_common.h"
#include "ee_epilogue.h"
#include "ee_decide.h"

namespace ee {
namespace {

// ---------------------------------------------------------------------------------------------------
// Status <- False for every sequence (Algorithm 1, initialisation), counters, scratch that must start at 0.
// ---------------------------------------------------------------------------------------------------
__global__ void iter_init_kernel(IterState s, int B, int n_layers, float* conf_out, float* zero_buf, size_t zero_count) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = t; i < (size_t)B; i += stride) {
    s.status[i] = 0;
    s.exit_layer[i] = n_layers;
  }
  if (t == 0) {
    *s.n_exited = 0;
    *s.done = 0;
    *s.batch_exit_layer = n_layers;
  }
  if (conf_out)
    for (size_t i = t; i < (size_t)B * n_layers; i += stride) conf_out[i] = __builtin_nanf("");
  for (size_t i = t; i < zero_count; i += stride) zero_buf[i] = 0.0f;
}

// hidden_states <- Embed(input_tokens): one row gather per sequence; padding rows of the last tile are zero.
// A token id outside 0..vocab-1 reads row 0 (the result is unspecified, the access stays inside the table).
__global__ void embed_bf16_kernel(const bf16_t* E, const int32_t* tokens, float* hT, int B, int Mpad, int d, int vocab) {
  const int k = blockIdx.x * blockDim.y + threadIdx.y;
  const int m = blockIdx.y * 32 + threadIdx.x;
  if (k >= d || m >= Mpad) return;
  float v = 0.0f;
  if (m < B) {
    const int tok = tokens[m];
    v = (float)E[(size_t)((unsigned)tok < (unsigned)vocab ? tok : 0) * d + k];
  }
  hT[ht_index(m, k, Mpad)] = v;
}
__global__ void embed_f32_kernel(const float* E, const int32_t* tokens, float* h, int B, int d, int vocab) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = blockIdx.y;
  const int tok = tokens[m];
  if (k < d) h[(size_t)m * d + k] = E[(size_t)((unsigned)tok < (unsigned)vocab ? tok : 0) * d + k];
}

__global__ void hidden_to_ht_kernel(const float* plain, float* hT, int B, int Mpad, int d) {
  const int k = blockIdx.x * blockDim.y + threadIdx.y;
  const int m = blockIdx.y * 32 + threadIdx.x;
  if (k >= d || m >= Mpad) return;
  hT[ht_index(m, k, Mpad)] = m < B ? plain[(size_t)m * d + k] : 0.0f;
}
__global__ void ht_to_hidden_kernel(const float* hT, float* plain, int B, int Mpad, int d) {
  const int k = blockIdx.x * blockDim.y + threadIdx.y;
  const int m = blockIdx.y * 32 + threadIdx.x;
  if (k >= d || m >= B) return;
  plain[(size_t)m * d + k] = hT[ht_index(m, k, Mpad)];
}
// (cos, sin) of pos_m * theta^(-2j/dh) for every sequence m and channel pair j, angles formed in double.
__global__ void rope_table_kernel(const int32_t* context_lens, float2* table, int B, int head_dim, float theta) {
  const int half = head_dim >> 1;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * half) return;
  const int m = idx / half, j = idx - m * half;
  const double ang = (double)context_lens[m] * exp2(-2.0 * (double)j / (double)head_dim * log2((double)theta));
  double sn, cs;
  sincos(ang, &sn, &cs);
  table[idx] = make_float2((float)cs, (float)sn);
}
__global__ void copy_f32_kernel(const float* src, float* dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------------
// bf16 path, RMSNorm in two small steps.
//   rowsq_kernel : rowsq[m] += sum_k h[m][k]^2 (grid = Mpad/32 workgroups of 1024 threads).
//   prep_x_kernel: x = bf16(h * rsqrt(rowsq/d + eps) * gain) written in operand-tile order.
//     A workgroup covers one 32-row batch tile x 64 channels: thread (m = t%32, c = t/32) owns 8 channels.
//     grid = (d/64, Mpad/32, slabs); slab z uses gains.g[z] and writes slab z of xT (KV filling: one per layer;
//     after a layer with an exit head: the head's operand and the next layer's attention operand in one launch).
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void rowsq_kernel(const float* hT, float* rowsq, int Mpad, int d, Pred pred) {
  // One workgroup per 32-row batch tile walks every channel and sums in a fixed order, so the result does not
  // depend on how workgroups are scheduled (it runs once per call, not once per layer).
  if (pred_skip(pred)) return;
  const int ml = threadIdx.x & 31, cl = threadIdx.x >> 5;
  const int m = blockIdx.x * 32 + ml;
  float ss = 0.0f;
  for (int k = cl; k < d; k += 32) {
    const float h = hT[ht_index(m, k, Mpad)];
    ss = fmaf(h, h, ss);
  }
  __shared__ float part[32][32];
  part[cl][ml] = ss;
  __syncthreads();
  if (cl == 0) {
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 32; ++j) s += part[j][ml];
    rowsq[m] += s;
  }
}

__global__ __launch_bounds__(256) void prep_x_kernel(const float* hT, GainTable gains, const bf16_t* gain0, bf16_t* xT,
                                                     size_t slab_elems, const float* rowsq, size_t rowsq_layer_stride,
                                                     const int32_t* slot_ptr, float eps, const int32_t* fill_from,
                                                     int fill_from_stride, int B, int Mpad, int d, RowDot rd,
                                                     RowMap rm, Pred pred) {
  if (pred_skip(pred)) return;
  const int z = blockIdx.z;
  const int ml = threadIdx.x & 31, cl = threadIdx.x >> 5;
  const int m = blockIdx.y * 32 + ml;
  // slab 0 of a launch with a row map is compacted: position m holds batch row perm[m], zeros from *n_active on
  // (never combined with the second job below)
  const bool compacted = rm.perm != nullptr && z == 0;
  const int n_valid = compacted ? rm.n_active[0] : Mpad;
  if ((int)blockIdx.y * 32 >= n_valid) return;
  const bool valid = m < n_valid;
  const int row = (compacted && valid) ? rm.perm[m] : m;
  if (fill_from) {
    // KV filling: slab z is layer z+1; skip slabs no sequence needs
    const int layer = z + 1;
    if (fill_from_stride == 0) {
      if (!(fill_from[0] < layer)) return;
    } else {
      __shared__ int any_row;
      if (threadIdx.x == 0) any_row = 0;
      __syncthreads();
      int need = 0;
      for (int r = threadIdx.x; r < B; r += blockDim.x) need |= fill_from[r] < layer;
      if (need) any_row = 1;
      __syncthreads();
      if (!any_row) return;
    }
  }
  const bf16_t* gain = gains.g[z] ? reinterpret_cast<const bf16_t*>(gains.g[z]) : gain0;
  const int c = blockIdx.x * 8 + cl;  // 8-channel chunk
  const int k0 = c * 8;
  // Hidden state of the batch exit layer L (KV filling and the final token inside a decode iteration): its sums
  // were left by the down projection of layer L in slot 2L of the per-iteration table; *slot_ptr = L
  if (rowsq_layer_stride) rowsq += (size_t)slot_ptr[0] * rowsq_layer_stride;
  const float rq = rowsq[row];
  float hv[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) hv[i] = valid ? hT[ht_index(row, k0 + i, Mpad)] : 0.0f;
  const bf16x8 gv = *reinterpret_cast<const bf16x8*>(gain + k0);
  const float r = valid ? rsqrtf(rq / (float)d + eps) : 0.0f;
  bf16x8 out;
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = (bf16_t)(hv[i] * r * (float)gv[i]);
  *reinterpret_cast<bf16x8*>(xT + (size_t)z * slab_elems + xt_index(m, k0, d)) = out;
  if (z != 0) return;
  // second job (uniform over the launch): dot product of every row with the previous hidden state or a weight
  // row, and the snapshot that becomes the next layer's "previous hidden state"
  if (rd.dots) {
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float o = rd.per_row ? rd.other[ht_index(m, k0 + i, Mpad)] : rd.other[k0 + i];
      acc = fmaf(hv[i], o, acc);
    }
    __shared__ float part[8][32];
    part[cl][ml] = acc;
    __syncthreads();
    if (cl == 0) {
      float t = 0.0f;
#pragma unroll
      for (int j = 0; j < 8; ++j) t += part[j][ml];
      unsafeAtomicAdd(rd.dots + m, t);
    }
  }
  if (rd.snapshot) {
#pragma unroll
    for (int i = 0; i < 8; ++i) rd.snapshot[ht_index(m, k0 + i, Mpad)] = hv[i];
  }
}

// fp32 path: the three sums a one-dot-product confidence measure needs, one workgroup per row.
__global__ __launch_bounds__(256) void measure_f32_kernel(const float* h, float* other, int per_row, float* out, int B,
                                                          int d, Pred pred) {
  if (pred_skip(pred)) return;
  const int m = blockIdx.x;
  const float* hp = h + (size_t)m * d;
  float* op = per_row ? other + (size_t)m * d : other;
  float dot = 0.0f, so = 0.0f, sh = 0.0f;
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    const float a = hp[k], b = op[k];
    dot = fmaf(a, b, dot);
    so = fmaf(b, b, so);
    sh = fmaf(a, a, sh);
    if (per_row) op[k] = a;   // this hidden state is the next layer's previous one
  }
  __shared__ float red[3][256];
  red[0][threadIdx.x] = dot;
  red[1][threadIdx.x] = so;
  red[2][threadIdx.x] = sh;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s)
      for (int j = 0; j < 3; ++j) red[j][threadIdx.x] += red[j][threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x < 3) out[(size_t)threadIdx.x * B + m] = red[threadIdx.x][0];
}

// fp32 path: plain RMSNorm, one workgroup per row.
__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float* h, const float* gain, float* x, int d, float eps,
                                                          Pred pred) {
  if (pred_skip(pred)) return;
  const int m = blockIdx.x;
  const float* hp = h + (size_t)m * d;
  float ss = 0.0f;
  for (int k = threadIdx.x; k < d; k += blockDim.x) ss = fmaf(hp[k], hp[k], ss);
  __shared__ float red[256];
  red[threadIdx.x] = ss;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  const float r = 1.0f / sqrtf(red[0] / (float)d + eps);
  for (int k = threadIdx.x; k < d; k += blockDim.x) x[(size_t)m * d + k] = hp[k] * r * gain[k];
}

// fp32 path: softmax statistics of one row of materialised logits -> one partial record.
__global__ __launch_bounds__(256) void head_stats_f32_kernel(const float* logits, float4* partials, int vocab, float scale,
                                                             Pred pred) {
  if (pred_skip(pred)) return;
  const int m = blockIdx.x;
  HeadStat s = stat_empty();
  for (int v = threadIdx.x; v < vocab; v += blockDim.x) s = stat_push(s, logits[(size_t)m * vocab + v], v, scale);
  __shared__ float4 red[256];
  red[threadIdx.x] = stat_pack(s);
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w)
      red[threadIdx.x] = stat_pack(stat_merge(stat_unpack(red[threadIdx.x]), stat_unpack(red[threadIdx.x + w]), scale));
    __syncthreads();
  }
  if (threadIdx.x == 0) partials[m] = red[0];
}

// ---------------------------------------------------------------------------------------------------
// Exit decision of one layer (Section 3.1): merge the per-tile statistics of every row into the confidence,
// apply the sticky status rule, count accepted sequences and raise the all-exited flag.  One workgroup per row.
// layer == 0: final token selection only.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a, Pred pred) {
  if (pred_skip(pred)) return;
  __shared__ float4 red[256];
  combine_row(a, blockIdx.x, red);
}

// Row map of the sequences that are still active, in batch order (one workgroup walks the batch 256 rows at a
// time); rows that have left get their sums of squares carried into the next layer's two slots.
__global__ __launch_bounds__(256) void compact_kernel(const int32_t* status, int B, RowMap rm, float* rowsq_table,
                                                      int slot, int Mpad, Pred pred) {
  if (pred_skip(pred)) return;
  __shared__ int wave_total[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int base = 0;
  for (int m0 = 0; m0 < B; m0 += 256) {
    const int m = m0 + (int)threadIdx.x;
    const bool in = m < B;
    const bool active = in && ctl_load(status + m) == 0;
    const unsigned long long bal = __ballot(active);
    if (lane == 0) wave_total[wave] = __popcll(bal);
    __syncthreads();
    int off = base + __popcll(bal & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) off += wave_total[w];
    if (active) {
      rm.perm[off] = m;
      rm.cpos[m] = off;
    } else if (in) {
      rm.cpos[m] = -1;
      if (rowsq_table) {
        const float v = rowsq_table[(size_t)slot * Mpad + m];
        rowsq_table[(size_t)(slot + 1) * Mpad + m] = v;
        rowsq_table[(size_t)(slot + 2) * Mpad + m] = v;
      }
    }
    base += wave_total[0] + wave_total[1] + wave_total[2] + wave_total[3];
    __syncthreads();
  }
  if (threadIdx.x == 0) rm.n_active[0] = base;
}

// One thread per row: confidence from one dot product (hidden states similarity, dedicated classifier).
__global__ __launch_bounds__(256) void decide_kernel(DecideArgs a, Pred pred) {
  if (pred_skip(pred)) return;
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= a.B) return;
  decide_from_dot(a, m);
}

}  // namespace

void launch_iter_init(const IterState& s, int B, int n_layers, float* conf_out, float* zero_buf, size_t zero_count,
                      hipStream_t st) {
  size_t work = (size_t)B * n_layers;
  if (zero_count > work) work = zero_count;
  int blocks = (int)((work + 255) / 256);
  if (blocks < 1) blocks = 1;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(iter_init_kernel, dim3(blocks), dim3(256), 0, st, s, B, n_layers, conf_out, zero_buf, zero_count);
}
void launch_embed_bf16(const bf16_t* E, const int32_t* tokens, float* hT, int B, int Mpad, int d, int vocab, hipStream_t st) {
  hipLaunchKernelGGL(embed_bf16_kernel, dim3((d + 7) / 8, Mpad / 32), dim3(32, 8), 0, st, E, tokens, hT, B, Mpad, d, vocab);
}
void launch_embed_f32(const float* E, const int32_t* tokens, float* h, int B, int d, int vocab, hipStream_t st) {
  hipLaunchKernelGGL(embed_f32_kernel, dim3((d + 255) / 256, B), dim3(256), 0, st, E, tokens, h, B, d, vocab);
}
void launch_hidden_to_ht(const float* plain, float* hT, int B, int Mpad, int d, hipStream_t st) {
  hipLaunchKernelGGL(hidden_to_ht_kernel, dim3((d + 7) / 8, Mpad / 32), dim3(32, 8), 0, st, plain, hT, B, Mpad, d);
}
void launch_ht_to_hidden(const float* hT, float* plain, int B, int Mpad, int d, hipStream_t st) {
  hipLaunchKernelGGL(ht_to_hidden_kernel, dim3((d + 7) / 8, Mpad / 32), dim3(32, 8), 0, st, hT, plain, B, Mpad, d);
}
void launch_rope_table(const int32_t* context_lens, float2* table, int B, int head_dim, float theta, hipStream_t st) {
  if (theta <= 0.0f || B == 0) return;
  const int n = B * (head_dim / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, context_lens, table, B, head_dim, theta);
}
void launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t st) {
  int blocks = (int)((n + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks), dim3(256), 0, st, src, dst, n);
}
void launch_rowsq(const float* hT, float* rowsq, int Mpad, int d, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(rowsq_kernel, dim3(Mpad / 32), dim3(1024), 0, st, hT, rowsq, Mpad, d, pred);
}
void launch_prep_x(const float* hT, const bf16_t* gain, bf16_t* xT, const float* rowsq, float eps, int Mpad, int d,
                   Pred pred, hipStream_t st) {
  GainTable none{};
  hipLaunchKernelGGL(prep_x_kernel, dim3(d / 64, Mpad / 32, 1), dim3(256), 0, st, hT, none, gain, xT, (size_t)0, rowsq, (size_t)0,
                     (const int32_t*)nullptr, eps, (const int32_t*)nullptr, 0, 0, Mpad, d, RowDot{}, RowMap{}, pred);
}
void launch_prep_x_dot(const float* hT, const bf16_t* gain, bf16_t* xT, const float* rowsq, const int32_t* slot_ptr,
                       size_t slot_stride, float eps, int Mpad, int d, const RowDot& rd, Pred pred, hipStream_t st) {
  GainTable none{};
  hipLaunchKernelGGL(prep_x_kernel, dim3(d / 64, Mpad / 32, 1), dim3(256), 0, st, hT, none, gain, xT, (size_t)0, rowsq,
                     slot_ptr ? slot_stride : (size_t)0, slot_ptr, eps, (const int32_t*)nullptr, 0, 0, Mpad, d, rd, RowMap{}, pred);
}
void launch_prep_x_pair(const float* hT, const bf16_t* gain_a, const bf16_t* gain_b, bf16_t* xT_pair, const float* rowsq,
                        float eps, int Mpad, int d, Pred pred, hipStream_t st) {
  GainTable two{};
  two.g[0] = gain_a;
  two.g[1] = gain_b;
  hipLaunchKernelGGL(prep_x_kernel, dim3(d / 64, Mpad / 32, 2), dim3(256), 0, st, hT, two, (const bf16_t*)nullptr, xT_pair,
                     (size_t)Mpad * d, rowsq, (size_t)0, (const int32_t*)nullptr, eps, (const int32_t*)nullptr, 0, 0, Mpad, d,
                     RowDot{}, RowMap{}, pred);
}
void launch_prep_x_compact(const float* hT, const bf16_t* gain_a, const bf16_t* gain_b, bf16_t* xT, const float* rowsq,
                           const RowMap& rm, float eps, int Mpad, int d, Pred pred, hipStream_t st) {
  GainTable two{};
  two.g[0] = gain_a;
  two.g[1] = gain_b;
  hipLaunchKernelGGL(prep_x_kernel, dim3(d / 64, Mpad / 32, gain_b ? 2 : 1), dim3(256), 0, st, hT, two, (const bf16_t*)nullptr,
                     xT, (size_t)Mpad * d, rowsq, (size_t)0, (const int32_t*)nullptr, eps, (const int32_t*)nullptr, 0, 0, Mpad,
                     d, RowDot{}, rm, pred);
}
void launch_compact(const int32_t* status, int B, const RowMap& rm, float* rowsq_table, int slot, int Mpad, Pred pred,
                    hipStream_t st) {
  hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(256), 0, st, status, B, rm, rowsq_table, slot, Mpad, pred);
}
void launch_prep_x_layers(const float* hT, const GainTable& gains, int n_layers, bf16_t* xT_slabs, const float* rowsq,
                          size_t rowsq_layer_stride, const int32_t* slot_ptr, float eps, const int32_t* fill_from,
                          int fill_from_stride, int B, int Mpad, int d, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(prep_x_kernel, dim3(d / 64, Mpad / 32, n_layers), dim3(256), 0, st, hT, gains,
                     (const bf16_t*)nullptr, xT_slabs, (size_t)Mpad * d, rowsq, rowsq_layer_stride, slot_ptr, eps, fill_from,
                     fill_from_stride, B, Mpad, d, RowDot{}, RowMap{}, pred);
}
void launch_rmsnorm_f32(const float* h, const float* gain, float* x, int B, int d, float eps, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3(B), dim3(256), 0, st, h, gain, x, d, eps, pred);
}
void launch_head_stats_f32(const float* logits, float4* partials, int B, int vocab, float scale, Pred pred,
                           hipStream_t st) {
  hipLaunchKernelGGL(head_stats_f32_kernel, dim3(B), dim3(256), 0, st, logits, partials, vocab, scale, pred);
}
void launch_measure_f32(const float* h, float* other, int per_row, float* out, int B, int d, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(measure_f32_kernel, dim3(B), dim3(256), 0, st, h, other, per_row, out, B, d, pred);
}
void launch_decide(const DecideArgs& a, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(decide_kernel, dim3((a.B + 255) / 256), dim3(256), 0, st, a, pred);
}
void launch_combine(const CombineArgs& a, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(combine_kernel, dim3(a.B), dim3(256), 0, st, a, pred);
}

}  // namespace ee
