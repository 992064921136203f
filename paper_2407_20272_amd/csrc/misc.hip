// Small kernels of the decode step: state reset, embedding gather, normalisation, exit-head decision.
#include "ee_common.h"
#include "ee_epilogue.h"
#include "ee_decide.h"

namespace ee {
namespace {

// ---------------------------------------------------------------------------------------------------
// Status <- False for every sequence (Algorithm 1, initialisation), counters.
// ---------------------------------------------------------------------------------------------------
__global__ void iter_init_kernel(IterState s, int B, int n_layers, float* conf_out) {
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
}

// hidden_states <- Embed(input_tokens): one row gather per sequence; padding rows of the last tile are zero.
// A token id outside 0..vocab-1 reads row 0 (the result is unspecified, the access stays inside the table).
__global__ __launch_bounds__(256) void embed_bf16_kernel(const bf16_t* E, const int32_t* tokens, float* h, int B, int d, int vocab) {
  const int m = blockIdx.x;
  const bf16_t* row = nullptr;
  if (m < B) {
    const int tok = tokens[m];
    row = E + (size_t)((unsigned)tok < (unsigned)vocab ? tok : 0) * d;
  }
  for (int k = threadIdx.x; k < d; k += blockDim.x) h[(size_t)m * d + k] = row ? (float)row[k] : 0.0f;
}
__global__ void embed_f32_kernel(const float* E, const int32_t* tokens, float* h, int B, int d, int vocab) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = blockIdx.y;
  const int tok = tokens[m];
  if (k < d) h[(size_t)m * d + k] = E[(size_t)((unsigned)tok < (unsigned)vocab ? tok : 0) * d + k];
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
// bf16 path: residual update + RMSNorm, one workgroup per batch row.
//   The projection before (output or down projection) left S partial results of the row, one per contraction
//   slice; they are summed in slice order and added to the residual row (nothing is added for a sequence that has
//   left, or when S == 0).  The row's sum of squares is reduced in a fixed order (lanes, then wavefronts), so the
//   whole update is reproducible bit for bit.  Then x = bf16(h * rsqrt(sumsq/d + eps) * gain) is written in
//   operand-tile order for up to two gains (after a layer with an exit head: the head's operand and the next
//   layer's).
// ---------------------------------------------------------------------------------------------------
constexpr int NORM_THREADS = 512;
constexpr int NORM_CHUNKS = 2;    // thread t owns channels [c * 4096 + 8t, +8), c = 0..1: d <= 8192

__device__ inline float block_sum(float v, float* red /* [NORM_THREADS / 64] of LDS */) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.0f;
#pragma unroll
  for (int w = 0; w < NORM_THREADS / 64; ++w) t += red[w];
  __syncthreads();
  return t;
}

__device__ inline void load8(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ inline void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ inline void zero_x_row(bf16_t* x, int m, int d) {
  for (int k0 = threadIdx.x * 8; k0 < d; k0 += NORM_THREADS * 8) {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (bf16_t)0.0f;
    *reinterpret_cast<bf16x8*>(x + xt_index(m, k0, d)) = z;
  }
}
// The gains are fetched before the row's sum of squares is reduced, so that the loads overlap the reduction instead of
// following it.
__device__ inline void load_gain(const bf16_t* gain, int d, bf16x8 (&gv)[NORM_CHUNKS]) {
#pragma unroll
  for (int c = 0; c < NORM_CHUNKS; ++c) {
    const int k0 = (c * NORM_THREADS + threadIdx.x) * 8;
    if (k0 < d) gv[c] = *reinterpret_cast<const bf16x8*>(gain + k0);
  }
}
__device__ inline void write_x_row(bf16_t* x, int row, int d, const float (&v)[NORM_CHUNKS][8], float r,
                                   const bf16x8 (&gv)[NORM_CHUNKS]) {
#pragma unroll
  for (int c = 0; c < NORM_CHUNKS; ++c) {
    const int k0 = (c * NORM_THREADS + threadIdx.x) * 8;
    if (k0 < d) {
      bf16x8 out;
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] = (bf16_t)(v[c][i] * r * (float)gv[c][i]);
      *reinterpret_cast<bf16x8*>(x + xt_index(row, k0, d)) = out;
    }
  }
}

// S: number of partial results to add (0 = none), a template parameter so that all of a thread's loads are in
// flight together; they are then added in slice order.
template <int S>
__global__ __launch_bounds__(NORM_THREADS) void finish_norm_kernel(NormArgs a, Pred pred) {
  if (pred_skip(pred)) return;
  __shared__ float red[NORM_THREADS / 64];
  const int m = blockIdx.x;
  const int d = a.d;
  // rows that hold no sequence: padding rows of an in-place operand, positions behind the active rows of a
  // compacted one
  const int n_act = a.rm.perm ? a.rm.n_active[0] : a.B;
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (a.x[j] && m >= (a.compacted[j] ? n_act : a.B)) zero_x_row(a.x[j], m, d);
  if (m >= a.B) return;
  const int pos = a.rm.perm ? a.rm.cpos[m] : m;   // row of the partial results; -1 for a sequence that has left
  const bool frozen = pos < 0 || (a.skip && ctl_load(a.skip + m) != 0);
  const bool add = S > 0 && !frozen;
  float v[NORM_CHUNKS][8];
  float ss = 0.0f, dot = 0.0f;
  bf16x8 gv[2][NORM_CHUNKS];
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (a.x[j]) load_gain(a.gain[j], d, gv[j]);
#pragma unroll
  for (int c = 0; c < NORM_CHUNKS; ++c) {
    const int k0 = (c * NORM_THREADS + threadIdx.x) * 8;
    if (k0 < d) {
      load8(a.h_in + (size_t)m * d + k0, v[c]);
      if (add) {
        float part[S > 0 ? S : 1][8];
#pragma unroll
        for (int s = 0; s < S; ++s) load8(a.y + ((size_t)s * a.Mpad + pos) * d + k0, part[s]);
#pragma unroll
        for (int s = 1; s < S; ++s)
#pragma unroll
          for (int i = 0; i < 8; ++i) part[0][i] += part[s][i];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[c][i] += part[0][i];
        store8(a.h_out + (size_t)m * d + k0, v[c]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) ss = fmaf(v[c][i], v[c][i], ss);
      if (a.rd.dots) {
        float o[8];
        load8(a.rd.other + (a.rd.per_row ? (size_t)m * d : (size_t)0) + k0, o);
#pragma unroll
        for (int i = 0; i < 8; ++i) dot = fmaf(v[c][i], o[i], dot);
      }
      if (a.rd.snapshot) store8(a.rd.snapshot + (size_t)m * d + k0, v[c]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[c][i] = 0.0f;
    }
  }
  ss = block_sum(ss, red);
  if (a.rd.dots) {
    dot = block_sum(dot, red);
    if (threadIdx.x == 0) a.rd.dots[m] = dot;
  }
  if (a.rowsq_out && threadIdx.x == 0) a.rowsq_out[m] = ss;
  const float r = rsqrtf(ss / (float)d + a.eps);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    if (!a.x[j]) continue;
    const int row = a.compacted[j] ? pos : m;
    if (row >= 0) write_x_row(a.x[j], row, d, v, r, gv[j]);
  }
}

// KV filling: grid (Mpad, n_layers); workgroup (m, l-1) normalises row m with layer l's attention gain into slab
// l-1.  Same arithmetic, thread for thread, as finish_norm_kernel, so that what is filled for a layer equals bit
// for bit the operand that layer's own pass would have built from the same hidden state.
__global__ __launch_bounds__(NORM_THREADS) void fill_prep_kernel(const float* h, GainTable gains, bf16_t* x_slabs,
                                                                 size_t slab_elems, float eps, const int32_t* fill_from,
                                                                 int fill_from_stride, int B, int d, Pred pred) {
  if (pred_skip(pred)) return;
  __shared__ float red[NORM_THREADS / 64];
  const int m = blockIdx.x, layer = blockIdx.y + 1;
  bf16_t* x = x_slabs + (size_t)blockIdx.y * slab_elems;
  if (fill_from_stride == 0) {
    if (!(ctl_load(fill_from) < layer)) return;     // Algorithm 1: one batch exit layer for everybody
  } else if (m < B && !(fill_from[m] < layer)) {
    return;                                          // this row's K/V of this layer exist already: its operand row is never used
  }
  if (m >= B) {
    zero_x_row(x, m, d);
    return;
  }
  float v[NORM_CHUNKS][8];
  float ss = 0.0f;
  bf16x8 gv[NORM_CHUNKS];
  load_gain(reinterpret_cast<const bf16_t*>(gains.g[blockIdx.y]), d, gv);
#pragma unroll
  for (int c = 0; c < NORM_CHUNKS; ++c) {
    const int k0 = (c * NORM_THREADS + threadIdx.x) * 8;
    if (k0 < d) {
      load8(h + (size_t)m * d + k0, v[c]);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss = fmaf(v[c][i], v[c][i], ss);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[c][i] = 0.0f;
    }
  }
  ss = block_sum(ss, red);
  write_x_row(x, m, d, v, rsqrtf(ss / (float)d + eps), gv);
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
// time).
__global__ __launch_bounds__(256) void compact_kernel(const int32_t* status, int B, RowMap rm, Pred pred) {
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

void launch_iter_init(const IterState& s, int B, int n_layers, float* conf_out, hipStream_t st) {
  size_t work = (size_t)B * n_layers;
  int blocks = (int)((work + 255) / 256);
  if (blocks < 1) blocks = 1;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(iter_init_kernel, dim3(blocks), dim3(256), 0, st, s, B, n_layers, conf_out);
}
void launch_embed_bf16(const bf16_t* E, const int32_t* tokens, float* h, int B, int Mpad, int d, int vocab, hipStream_t st) {
  hipLaunchKernelGGL(embed_bf16_kernel, dim3(Mpad), dim3(256), 0, st, E, tokens, h, B, d, vocab);
}
void launch_embed_f32(const float* E, const int32_t* tokens, float* h, int B, int d, int vocab, hipStream_t st) {
  hipLaunchKernelGGL(embed_f32_kernel, dim3((d + 255) / 256, B), dim3(256), 0, st, E, tokens, h, B, d, vocab);
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
void launch_finish_norm(const NormArgs& a, Pred pred, hipStream_t st) {
  const dim3 grid(a.Mpad), block(NORM_THREADS);
  switch (a.S) {
    case 0: hipLaunchKernelGGL(finish_norm_kernel<0>, grid, block, 0, st, a, pred); break;
    case 1: hipLaunchKernelGGL(finish_norm_kernel<1>, grid, block, 0, st, a, pred); break;
    case 2: hipLaunchKernelGGL(finish_norm_kernel<2>, grid, block, 0, st, a, pred); break;
    case 3: hipLaunchKernelGGL(finish_norm_kernel<3>, grid, block, 0, st, a, pred); break;
    case 4: hipLaunchKernelGGL(finish_norm_kernel<4>, grid, block, 0, st, a, pred); break;
    case 5: hipLaunchKernelGGL(finish_norm_kernel<5>, grid, block, 0, st, a, pred); break;
    case 6: hipLaunchKernelGGL(finish_norm_kernel<6>, grid, block, 0, st, a, pred); break;
    case 7: hipLaunchKernelGGL(finish_norm_kernel<7>, grid, block, 0, st, a, pred); break;
    default: hipLaunchKernelGGL(finish_norm_kernel<8>, grid, block, 0, st, a, pred); break;   // the planner never asks for more
  }
}
void launch_fill_prep(const float* h, const GainTable& gains, int n_layers, bf16_t* x_slabs, float eps,
                      const int32_t* fill_from, int fill_from_stride, int B, int Mpad, int d, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(fill_prep_kernel, dim3(Mpad, n_layers), dim3(NORM_THREADS), 0, st, h, gains, x_slabs, (size_t)Mpad * d, eps,
                     fill_from, fill_from_stride, B, d, pred);
}
void launch_compact(const int32_t* status, int B, const RowMap& rm, Pred pred, hipStream_t st) {
  hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(256), 0, st, status, B, rm, pred);
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
