// Device-side epilogues shared by the MFMA (bf16) and the plain (fp32) projection kernels.
// Each takes one batch row m and one pair of output rows (f_lo, f_hi) with their finished dot products.
#pragma once

#include "ee_common.h"

namespace ee {

// The control words of an iteration (status, exit layers, the count of accepted sequences, the all-exited flag and
// the batch exit layer) are written by the workgroups that take an exit decision and read by workgroups of other
// compute units, sometimes of the same launch: every access is a relaxed device-scope atomic.
__device__ inline int32_t ctl_load(const int32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ inline void ctl_store(int32_t* p, int32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__device__ inline float row_rinv(const float* rowsq, int m, int d, float eps) {
  return rowsq ? rsqrtf(rowsq[m] / (float)d + eps) : 1.0f;
}

__device__ inline void store_elem(float* p, float v) { *p = v; }
__device__ inline void store_elem(bf16_t* p, float v) { *p = (bf16_t)v; }

// Rotary embedding (split-half pairing: channel j with j + dh/2, angle = pos * theta^(-2j/dh)) and the write of
// this position's K/V into the paged cache; q goes to a dense buffer.  The (cos, sin) pairs come from a table
// that rope_table_kernel fills once per call from angles formed in double (long contexts would lose the fraction
// of the angle to float rounding of the frequency).
template <class T>
__device__ inline void epi_qkv(const QkvEpi& e, int m, int f_lo, float lo, float hi) {
  if (e.fill_from && !(e.fill_from[(size_t)m * e.fill_from_stride] < e.layer)) return;
  const float r = row_rinv(e.rowsq, m, e.d_model, e.eps);
  lo *= r;
  hi *= r;
  const int d = e.d_model, dh = e.head_dim, half = dh >> 1;
  const int which = f_lo / d;  // 0 q, 1 k, 2 v
  const int within = f_lo - which * d;
  const int head = within / dh;
  const int j = within - head * dh;  // < dh/2
  const int p = e.context_lens[m];
  if (which < 2 && e.rope_theta > 0.0f) {
    const float2 cs = e.rope[(size_t)m * half + j];   // (cos, sin) of pos * theta^(-2j/dh), tabulated once per iteration
    const float c = cs.x, s = cs.y;
    const float a = lo * c - hi * s;
    const float b = hi * c + lo * s;
    lo = a;
    hi = b;
  }
  if (which == 0) {
    if (e.q) {
      float* q = e.q + (size_t)m * d + head * dh + j;
      q[0] = lo;
      q[half] = hi;
    }
    return;
  }
  const bool p_ok = (unsigned)p < (unsigned)(e.max_blocks * 16);
  const int blk = e.block_tables[(size_t)(e.row_table ? safe_row(e.row_table[m], e.table_rows) : m) * e.max_blocks + (p_ok ? p >> 4 : 0)];
  if (!p_ok || (unsigned)blk >= (unsigned)e.num_blocks) return;   // never outside the pools
  const size_t at = (((size_t)blk * e.n_heads + head) * 16 + (p & 15)) * dh + j;
  T* pool = reinterpret_cast<T*>(which == 1 ? e.k_pool : e.v_pool);
  store_elem(pool + at, lo);
  store_elem(pool + at + half, hi);
}

// The same for four consecutive channels f_lo0..f_lo0+3 (f_lo0 a multiple of 4) of batch row m and their four
// rotary partners, bf16 cache: one look-up of the slot, 8-byte stores into the cache, 16-byte stores into q.
__device__ inline void epi_qkv4(const QkvEpi& e, int m, int f_lo0, float (&lo)[4], float (&hi)[4]) {
  if (e.fill_from && !(e.fill_from[(size_t)m * e.fill_from_stride] < e.layer)) return;
  const float r = row_rinv(e.rowsq, m, e.d_model, e.eps);
  const int d = e.d_model, dh = e.head_dim, half = dh >> 1;
  const int which = f_lo0 / d;  // 0 q, 1 k, 2 v
  const int within = f_lo0 - which * d;
  const int head = within / dh;
  const int j = within - head * dh;  // < dh/2, a multiple of 4
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    lo[i] *= r;
    hi[i] *= r;
  }
  if (which < 2 && e.rope_theta > 0.0f) {
    const float4 c01 = *reinterpret_cast<const float4*>(e.rope + (size_t)m * half + j);       // (cos, sin) x 2
    const float4 c23 = *reinterpret_cast<const float4*>(e.rope + (size_t)m * half + j + 2);
    const float cs[4] = {c01.x, c01.z, c23.x, c23.z}, sn[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float a = lo[i] * cs[i] - hi[i] * sn[i];
      const float b = hi[i] * cs[i] + lo[i] * sn[i];
      lo[i] = a;
      hi[i] = b;
    }
  }
  if (which == 0) {
    if (e.q) {
      float* q = e.q + (size_t)m * d + head * dh + j;
      *reinterpret_cast<float4*>(q) = make_float4(lo[0], lo[1], lo[2], lo[3]);
      *reinterpret_cast<float4*>(q + half) = make_float4(hi[0], hi[1], hi[2], hi[3]);
    }
    return;
  }
  const int p = e.context_lens[m];
  const bool p_ok = (unsigned)p < (unsigned)(e.max_blocks * 16);
  const int blk = e.block_tables[(size_t)(e.row_table ? safe_row(e.row_table[m], e.table_rows) : m) * e.max_blocks + (p_ok ? p >> 4 : 0)];
  if (!p_ok || (unsigned)blk >= (unsigned)e.num_blocks) return;   // never outside the pools
  const size_t at = (((size_t)blk * e.n_heads + head) * 16 + (p & 15)) * dh + j;
  bf16_t* pool = reinterpret_cast<bf16_t*>(which == 1 ? e.k_pool : e.v_pool);
  typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
  *reinterpret_cast<bf16x4*>(pool + at) = bf16x4{(bf16_t)lo[0], (bf16_t)lo[1], (bf16_t)lo[2], (bf16_t)lo[3]};
  *reinterpret_cast<bf16x4*>(pool + at + half) = bf16x4{(bf16_t)hi[0], (bf16_t)hi[1], (bf16_t)hi[2], (bf16_t)hi[3]};
}

__device__ inline void epi_acc(const AccEpi& e, int m, int f, float v) {
  if (e.skip && ctl_load(e.skip + m) != 0) return;
  e.h[(size_t)m * e.n_out + f] += v;   // fp32 path: every element of the residual stream has one contributor per launch
}

// SwiGLU product; f_lo is the gate row f, f_hi the up row f + d_ffn.
template <class T>
__device__ inline void epi_gateup(const GateUpEpi& e, int m, int f, float gate, float up) {
  const float r = row_rinv(e.rowsq, m, e.d_model, e.eps);
  gate *= r;
  up *= r;
  const float a = gate / (1.0f + expf(-gate)) * up;
  if constexpr (sizeof(T) == 2) {
    reinterpret_cast<bf16_t*>(e.act)[xt_index(m, f, e.d_ffn)] = (bf16_t)a;
  } else {
    reinterpret_cast<float*>(e.act)[(size_t)m * e.d_ffn + f] = a;
  }
}

// SwiGLU products of four consecutive features f0..f0+3 (f0 a multiple of 4), bf16 operand-tile order: one 8-byte store.
__device__ inline void epi_gateup4(const GateUpEpi& e, int m, int f0, const float (&gate)[4], const float (&up)[4]) {
  const float r = row_rinv(e.rowsq, m, e.d_model, e.eps);
  typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float g = gate[i] * r, u = up[i] * r;
    out[i] = (bf16_t)(g / (1.0f + expf(-g)) * u);
  }
  *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(e.act) + xt_index(m, f0, e.d_ffn)) = out;
}

// Running softmax statistics of one row: largest and second largest (unscaled) logit, index of the largest
// (lowest index on ties) and sum of exp(scale * (z - max)).
struct HeadStat {
  float zmax, sum, z2;
  int idx;
};
// exp of a non-positive argument for the softmax sums: the hardware's base-2 exponential (relative error about 1e-7;
// the library routine costs several times the instructions, and an exit head evaluates one per logit and row)
__device__ inline float stat_exp(float x) { return __expf(x); }
__device__ inline HeadStat stat_empty() { return {-INFINITY, 0.0f, -INFINITY, 0x7fffffff}; }
__device__ inline HeadStat stat_merge(const HeadStat& a, const HeadStat& b, float scale) {
  HeadStat o;
  if (a.zmax > b.zmax || (a.zmax == b.zmax && a.idx < b.idx)) {
    o.zmax = a.zmax;
    o.idx = a.idx;
    o.z2 = fmaxf(a.z2, b.zmax);
  } else {
    o.zmax = b.zmax;
    o.idx = b.idx;
    o.z2 = fmaxf(b.z2, a.zmax);
  }
  const float wa = a.sum > 0.0f ? a.sum * stat_exp(scale * (a.zmax - o.zmax)) : 0.0f;
  const float wb = b.sum > 0.0f ? b.sum * stat_exp(scale * (b.zmax - o.zmax)) : 0.0f;
  o.sum = wa + wb;
  return o;
}
__device__ inline HeadStat stat_push(const HeadStat& a, float z, int idx, float scale) {
  HeadStat b = {z, 1.0f, -INFINITY, idx};
  return stat_merge(a, b, scale);
}
// Statistics of 32 logits of one row that sit four each in eight neighbouring lanes (lane & 7 = which four):
// two short passes (largest with its index, then the sum of exponentials and the runner-up) instead of 32
// dependent pushes.  z[i] has vocabulary index idx0 + i.  Every one of the eight lanes returns the result.
__device__ inline HeadStat stat_of_8x4(const float (&z)[4], int idx0, float scale) {
  float best = z[0];
  int bi = idx0;
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (z[i] > best) {   // strict: the lowest index wins among equals
      best = z[i];
      bi = idx0 + i;
    }
#pragma unroll
  for (int x = 1; x < 8; x <<= 1) {
    const float ob = __shfl_xor(best, x);
    const int oi = __shfl_xor(bi, x);
    if (ob > best || (ob == best && oi < bi)) {
      best = ob;
      bi = oi;
    }
  }
  float sum = 0.0f, z2 = -INFINITY;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sum += stat_exp(scale * (z[i] - best));
    if (idx0 + i != bi) z2 = fmaxf(z2, z[i]);
  }
#pragma unroll
  for (int x = 1; x < 8; x <<= 1) {
    sum += __shfl_xor(sum, x);
    z2 = fmaxf(z2, __shfl_xor(z2, x));
  }
  return {best, sum, z2, bi};
}

// Statistics of N logits held by one thread (z[i] has vocabulary index idx[i], ascending): largest first, then
// the exponentials, which are independent of each other.
template <int N>
__device__ inline HeadStat stat_of(const float (&z)[N], const int (&idx)[N], float scale) {
  float best = z[0];
  int bi = idx[0];
#pragma unroll
  for (int i = 1; i < N; ++i)
    if (z[i] > best) {
      best = z[i];
      bi = idx[i];
    }
  float sum = 0.0f, z2 = -INFINITY;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    sum += stat_exp(scale * (z[i] - best));
    if (idx[i] != bi) z2 = fmaxf(z2, z[i]);
  }
  return {best, sum, z2, bi};
}

__device__ inline float4 stat_pack(const HeadStat& s) { return make_float4(s.zmax, s.sum, s.z2, __int_as_float(s.idx)); }
__device__ inline HeadStat stat_unpack(const float4& v) { return {v.x, v.y, v.z, __float_as_int(v.w)}; }

__device__ inline bool pred_skip(const Pred& p) { return p.flag && ((ctl_load(p.flag) != 0) != (p.run_when != 0)); }

}  // namespace ee
