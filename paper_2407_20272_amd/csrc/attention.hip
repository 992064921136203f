// Single-query attention over the paged KV cache (the attention inside one layer of the decode step).
//
// Bandwidth-bound: every cached K and V value of the sequence is read once (about one flop per byte), so the
// kernel is organised around the reads.  One workgroup owns one (sequence, head); its four wavefronts take the
// sequence's 16-token blocks round-robin.  A block of one head is 16 tokens x head_dim values of consecutive
// memory (4 KiB for bf16 x 128), which a wavefront fetches with 16-byte loads per lane, every load instruction
// covering 1 KiB of consecutive bytes; the next block's K and V are in flight while the current one is reduced.
// Lanes that share a token add their partial dot products with a butterfly; every group of lanes keeps its own
// running softmax (max, sum, weighted V) over the tokens it sees, and the groups, then the wavefronts, are merged
// once at the end.  No score is ever written to memory.
#include <type_traits>

#include "ee_common.h"
#include "ee_epilogue.h"

namespace ee {
namespace {

constexpr int NW = 4;
constexpr float NEG_BIG = -1.0e30f;

template <class T>
struct Elems;
template <>
struct Elems<float> {
  static constexpr int N = 4;
  __device__ static void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
  }
};
template <>
struct Elems<bf16_t> {
  static constexpr int N = 8;
  __device__ static void unpack(const uint4& v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16);
    f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16);
    f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
};

// Sum over the LPT lanes that share a token; every lane of the group ends up with the total.
// Within a 16-lane row the butterfly runs on the DPP cross-lane network (quad permutes, half-row and row
// mirrors); only a 32-lane group needs one LDS-crossbar shuffle on top.
template <int LPT>
__device__ inline float group_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  if constexpr (LPT >= 16)
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  if constexpr (LPT >= 32) v += __shfl_xor(v, 16);
  return v;
}

// 16 bytes of the cache, read once per iteration and never again: a streaming (non-temporal) load, which leaves
// the caches to the data that is reused.
template <class T>
__device__ inline uint4 load_stream(const T* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Sixteen bytes of zeros (never written; not const, so that it lives in the same address space as the cache).
// A lane whose token lies after the sequence's last position reads its V values from here instead of from the
// cache: what an earlier owner of the block, or nobody, left in those slots is weighted with zero, and 0 * NaN
// would still be NaN.  The choice is made on the ADDRESS; the load itself stays unconditional.
__device__ uint4 k_zero16;

constexpr int TABLE_LDS_MAX = kAttnMaxBlocks;   // block-table entries staged in LDS

template <class T, int DH, bool OUT_XT, bool SPLIT>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a, Pred pred) {
  constexpr int EPL = Elems<T>::N;         // values per 16-byte lane load
  constexpr int LPT = DH / EPL;            // lanes per token
  constexpr int TPL = 64 / LPT;            // tokens per wavefront load
  constexpr int LPB = 16 / TPL;            // loads per 16-token block
  static_assert(LPT >= 8 && LPT <= 32, "unsupported head_dim for this element type");

  const int head = blockIdx.x, b = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane % LPT;              // which EPL-wide slice of the head this lane holds
  const int grp = lane / LPT;              // which token of a load this lane sees
  const int32_t* table = a.block_tables + (size_t)(a.row_table ? safe_row(a.row_table[b], a.B) : b) * a.max_blocks;

  extern __shared__ int32_t tbl[];
  if (pred_skip(pred)) return;
  // Everything the first K/V load needs is requested before any of it is waited for: the context length, the
  // start of the block-table row (its width is known without the length) and q: one memory round trip, not
  // three in a row.
  const int t0 = (int)threadIdx.x < a.max_blocks ? safe_block(table[threadIdx.x], a.num_blocks) : 0;
  const int len = a.context_lens[b];
  const int left = a.skip ? __hip_atomic_load(a.skip + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
  const int out_row = a.out_pos ? a.out_pos[b] : b;
  float q[EPL];
  {
    const float* qp = a.q + ((size_t)b * a.n_heads + head) * DH + sub * EPL;
#pragma unroll
    for (int i = 0; i < EPL; ++i) q[i] = qp[i];
  }
  if (left != 0) return;   // the sequence has left at an earlier layer: nothing to attend, nothing read
  // positions 0..p inclusive, never beyond the block table's width
  const int n_ctx = min(len + 1, a.max_blocks * 16);
  const int n_blocks = (n_ctx + 15) >> 4;

  // The sequence's block table goes to LDS once (max_blocks entries of dynamic LDS).  The block loop must not
  // read it from memory: the wait for such a read would also wait for every K/V load issued before it.
  if ((int)threadIdx.x < a.max_blocks) tbl[threadIdx.x] = t0;
  for (int i = threadIdx.x + blockDim.x; i < n_blocks; i += blockDim.x) tbl[i] = safe_block(table[i], a.num_blocks);

  // q slice, pre-scaled so that exp2 can be used: softmax(x) = 2^(x*log2 e)
  {
    const float sc = 1.4426950408889634f / sqrtf((float)DH);
#pragma unroll
    for (int i = 0; i < EPL; ++i) q[i] *= sc;
  }
  __syncthreads();

  float m_run = NEG_BIG, l_run = 0.0f, o[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) o[i] = 0.0f;

  const size_t head_off = (size_t)head * 16 * DH;             // elements, inside a block
  const size_t block_elems = (size_t)a.n_heads * 16 * DH;
  const T* kbase = reinterpret_cast<const T*>(a.k_pool) + head_off + (size_t)grp * DH + sub * EPL;
  const T* vbase = reinterpret_cast<const T*>(a.v_pool) + head_off + (size_t)grp * DH + sub * EPL;

  struct Blk {
    uint4 k[LPB], v[LPB];
  };
  const T* zero_src = reinterpret_cast<const T*>(&k_zero16);
  auto fetch = [&](Blk& x, int lb) {
    const int phys = tbl[lb];
    const size_t off = (size_t)phys * block_elems;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      x.k[i] = load_stream(kbase + off + (size_t)i * TPL * DH);
      x.v[i] = load_stream(lb * 16 + i * TPL + grp < n_ctx ? vbase + off + (size_t)i * TPL * DH : zero_src);
    }
  };
  auto consume = [&](const Blk& x, int lb) {
    float s[LPB];
    float m_new = m_run;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      float kf[EPL];
      Elems<T>::unpack(x.k[i], kf);
      float d = 0.0f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(q[e], kf[e], d);
      d = group_sum<LPT>(d);
      const int tok = lb * 16 + i * TPL + grp;
      s[i] = tok < n_ctx ? d : NEG_BIG;
      m_new = fmaxf(m_new, s[i]);
    }
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    l_run *= alpha;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] *= alpha;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      const int tok = lb * 16 + i * TPL + grp;
      const float p = tok < n_ctx ? __builtin_amdgcn_exp2f(s[i] - m_new) : 0.0f;
      l_run += p;
      float vf[EPL];
      Elems<T>::unpack(x.v[i], vf);
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] = fmaf(p, vf[e], o[e]);
    }
    m_run = m_new;
  };

  // Two blocks of this wavefront in flight at any time.  The steady loop has no conditional load: a load under
  // a condition makes the compiler wait for every outstanding load where the paths join, which would drain
  // the stream once per block; the scheduling fences keep each block's loads together ahead of the arithmetic.
  // SPLIT: this workgroup is part blockIdx.z of gridDim.z and walks a contiguous range of the sequence's blocks
  // (possibly empty: a short sequence in a wide table); otherwise all of them.
  int lb_begin = 0, lb_end = n_blocks;
  if constexpr (SPLIT) {
    const int per = (n_blocks + (int)gridDim.z - 1) / (int)gridDim.z;
    lb_begin = min(n_blocks, (int)blockIdx.z * per);
    lb_end = min(n_blocks, lb_begin + per);
  }
  Blk A, B;
  int lb = lb_begin + wave;
  if (lb < lb_end) fetch(A, lb);
  if (lb + NW < lb_end) fetch(B, lb + NW);
  for (; lb + 3 * NW < lb_end; lb += 2 * NW) {
    consume(A, lb);
    __builtin_amdgcn_sched_barrier(0);
    fetch(A, lb + 2 * NW);
    __builtin_amdgcn_sched_barrier(0);
    consume(B, lb + NW);
    __builtin_amdgcn_sched_barrier(0);
    fetch(B, lb + 3 * NW);
    __builtin_amdgcn_sched_barrier(0);
  }
  // at most three blocks left: lb (in A), lb + NW (in B), lb + 2 NW (not fetched yet)
  if (lb < lb_end) {
    consume(A, lb);
    const bool third = lb + 2 * NW < lb_end;
    if (third) fetch(A, lb + 2 * NW);
    if (lb + NW < lb_end) consume(B, lb + NW);
    if (third) consume(A, lb + 2 * NW);
  }

  // merge the TPL lane groups of the wavefront
#pragma unroll
  for (int x = LPT; x < 64; x <<= 1) {
    const float m_o = __shfl_xor(m_run, x);
    const float l_o = __shfl_xor(l_run, x);
    const float m_new = fmaxf(m_run, m_o);
    const float wa = __builtin_amdgcn_exp2f(m_run - m_new), wb = __builtin_amdgcn_exp2f(m_o - m_new);
    l_run = l_run * wa + l_o * wb;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float o_o = __shfl_xor(o[e], x);
      o[e] = o[e] * wa + o_o * wb;
    }
    m_run = m_new;
  }

  // merge the wavefronts
  __shared__ float sm[NW], sl[NW], so[NW][DH];
  if (grp == 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) so[wave][sub * EPL + e] = o[e];
    if (sub == 0) {
      sm[wave] = m_run;
      sl[wave] = l_run;
    }
  }
  __syncthreads();
  if (threadIdx.x < DH) {
    float M = sm[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm[w]);
    float L = 0.0f, acc = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(sm[w] - M);
      L += sl[w] * wgt;
      acc += so[w][threadIdx.x] * wgt;
    }
    if constexpr (SPLIT) {
      // this part's running maximum, sum and unnormalised output; the merge launch takes it from here
      float* ws = a.split_ws + (((size_t)b * a.n_heads + head) * gridDim.z + blockIdx.z) * (DH + 2);
      if (threadIdx.x == 0) {
        ws[0] = M;
        ws[1] = L;
      }
      ws[2 + threadIdx.x] = acc;
    } else {
      const float r = acc / L;
      const int col = head * DH + threadIdx.x;
      if constexpr (OUT_XT) {
        reinterpret_cast<bf16_t*>(a.out)[xt_index(out_row, col, a.n_heads * DH)] = (bf16_t)r;
      } else {
        reinterpret_cast<float*>(a.out)[(size_t)out_row * a.n_heads * DH + col] = r;
      }
    }
  }
}

// Second launch of the split form: one workgroup of DH threads per (sequence, head) adds the parts in part order.
template <int DH, bool OUT_XT>
__global__ __launch_bounds__(DH) void attn_merge_kernel(AttnArgs a, Pred pred) {
  if (pred_skip(pred)) return;
  const int head = blockIdx.x, b = blockIdx.y;
  const int left = a.skip ? __hip_atomic_load(a.skip + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
  if (left != 0) return;
  const int out_row = a.out_pos ? a.out_pos[b] : b;
  const float* ws = a.split_ws + ((size_t)b * a.n_heads + head) * a.split_parts * (DH + 2);
  float M = NEG_BIG;
  for (int s = 0; s < a.split_parts; ++s) M = fmaxf(M, ws[(size_t)s * (DH + 2)]);
  float L = 0.0f, acc = 0.0f;
  for (int s = 0; s < a.split_parts; ++s) {
    const float* p = ws + (size_t)s * (DH + 2);
    const float wgt = __builtin_amdgcn_exp2f(p[0] - M);   // an empty part has the maximum -1e30: weight 0
    L += p[1] * wgt;
    acc += p[2 + threadIdx.x] * wgt;
  }
  const float r = acc / L;
  const int col = head * DH + threadIdx.x;
  if constexpr (OUT_XT) {
    reinterpret_cast<bf16_t*>(a.out)[xt_index(out_row, col, a.n_heads * DH)] = (bf16_t)r;
  } else {
    reinterpret_cast<float*>(a.out)[(size_t)out_row * a.n_heads * DH + col] = r;
  }
}

// ---------------------------------------------------------------------------------------------------------
// Several batch rows of ONE sequence per workgroup (a chunk of a prompt pushed through the decode step: rows
// that share a block table).  A workgroup owns R consecutive batch rows of one head; rows of the same sequence
// form a run, and the run's K/V blocks are streamed once and multiplied against every row of the run, each row
// masking the positions after its own.  A workgroup whose rows span several sequences walks its runs one after
// the other.  Per row the arithmetic is that of the single-row kernel above; only the K/V traffic is shared.
// ---------------------------------------------------------------------------------------------------------
template <class T, int DH, int R, bool OUT_XT>
__global__ __launch_bounds__(256) void attn_rows_kernel(AttnArgs a, Pred pred) {
  constexpr int EPL = Elems<T>::N;
  constexpr int LPT = DH / EPL;
  constexpr int TPL = 64 / LPT;
  constexpr int LPB = 16 / TPL;
  extern __shared__ int32_t tbl[];
  if (pred_skip(pred)) return;

  const int head = blockIdx.x, row0 = blockIdx.y * R;
  const int nrows = min(R, a.B - row0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane % LPT, grp = lane / LPT;

  int seq[R], npos[R];
  float q[R][EPL], m_run[R], l_run[R], o[R][EPL];
  const float sc = 1.4426950408889634f / sqrtf((float)DH);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bool valid = r < nrows;
    seq[r] = valid ? safe_row(a.row_table[row0 + r], a.B) : -1;
    npos[r] = valid ? min(a.context_lens[row0 + r] + 1, a.max_blocks * 16) : 0;
    const float* qp = a.q + ((size_t)(valid ? row0 + r : row0) * a.n_heads + head) * DH + sub * EPL;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      q[r][i] = qp[i] * sc;
      o[r][i] = 0.0f;
    }
    m_run[r] = NEG_BIG;
    l_run[r] = 0.0f;
  }

  const size_t head_off = (size_t)head * 16 * DH;
  const size_t block_elems = (size_t)a.n_heads * 16 * DH;
  const T* kbase = reinterpret_cast<const T*>(a.k_pool) + head_off + (size_t)grp * DH + sub * EPL;
  const T* vbase = reinterpret_cast<const T*>(a.v_pool) + head_off + (size_t)grp * DH + sub * EPL;
  struct Blk {
    uint4 k[LPB], v[LPB];
  };

  int r_begin = 0;
  while (r_begin < nrows) {
    // the run: rows r_begin .. r_end-1 of one sequence (uniform over the workgroup)
    int r_end = r_begin + 1, run_ctx = 0, run_seq = -1;
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (r == r_begin) run_seq = seq[r];
#pragma unroll
    for (int r = 1; r < R; ++r)
      if (r == r_end && r < nrows && seq[r] == run_seq) ++r_end;
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (r >= r_begin && r < r_end) run_ctx = max(run_ctx, npos[r]);
    const int n_blocks = (run_ctx + 15) >> 4;
    const int32_t* table = a.block_tables + (size_t)run_seq * a.max_blocks;
    __syncthreads();   // the previous run's table is no longer read
    for (int i = threadIdx.x; i < n_blocks; i += blockDim.x) tbl[i] = safe_block(table[i], a.num_blocks);
    __syncthreads();

    const T* zero_src = reinterpret_cast<const T*>(&k_zero16);
    auto fetch = [&](Blk& x, int lb) {
      const size_t off = (size_t)tbl[lb] * block_elems;
#pragma unroll
      for (int i = 0; i < LPB; ++i) {
        x.k[i] = load_stream(kbase + off + (size_t)i * TPL * DH);
        x.v[i] = load_stream(lb * 16 + i * TPL + grp < run_ctx ? vbase + off + (size_t)i * TPL * DH : zero_src);
      }
    };
    auto consume = [&](const Blk& x, int lb) {
      float kf[LPB][EPL], vf[LPB][EPL];
#pragma unroll
      for (int i = 0; i < LPB; ++i) {
        Elems<T>::unpack(x.k[i], kf[i]);
        Elems<T>::unpack(x.v[i], vf[i]);
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (r < r_begin || r >= r_end) continue;   // uniform: rows of other runs keep their state
        float s[LPB];
        float m_new = m_run[r];
#pragma unroll
        for (int i = 0; i < LPB; ++i) {
          float d = 0.0f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) d = fmaf(q[r][e], kf[i][e], d);
          d = group_sum<LPT>(d);
          const int tok = lb * 16 + i * TPL + grp;
          s[i] = tok < npos[r] ? d : NEG_BIG;
          m_new = fmaxf(m_new, s[i]);
        }
        const float alpha = __builtin_amdgcn_exp2f(m_run[r] - m_new);
        l_run[r] *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[r][e] *= alpha;
#pragma unroll
        for (int i = 0; i < LPB; ++i) {
          const int tok = lb * 16 + i * TPL + grp;
          const float p = tok < npos[r] ? __builtin_amdgcn_exp2f(s[i] - m_new) : 0.0f;
          l_run[r] += p;
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[r][e] = fmaf(p, vf[i][e], o[r][e]);
        }
        m_run[r] = m_new;
      }
    };

    // one block in flight behind the one being multiplied (the multiplies of R rows hide the load)
    Blk A, B;
    int lb = wave;
    if (lb < n_blocks) fetch(A, lb);
    for (; lb + NW < n_blocks; lb += 2 * NW) {
      fetch(B, lb + NW);
      consume(A, lb);
      if (lb + 2 * NW < n_blocks) fetch(A, lb + 2 * NW);
      consume(B, lb + NW);
    }
    if (lb < n_blocks) consume(A, lb);
    r_begin = r_end;
  }

  // merge the lane groups of each wavefront, then the wavefronts, row by row
  __shared__ float sm[NW][R], sl[NW][R], so[NW][R][DH];
#pragma unroll
  for (int r = 0; r < R; ++r) {
#pragma unroll
    for (int x = LPT; x < 64; x <<= 1) {
      const float m_o = __shfl_xor(m_run[r], x);
      const float l_o = __shfl_xor(l_run[r], x);
      const float m_new = fmaxf(m_run[r], m_o);
      const float wa = __builtin_amdgcn_exp2f(m_run[r] - m_new), wb = __builtin_amdgcn_exp2f(m_o - m_new);
      l_run[r] = l_run[r] * wa + l_o * wb;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float o_o = __shfl_xor(o[r][e], x);
        o[r][e] = o[r][e] * wa + o_o * wb;
      }
      m_run[r] = m_new;
    }
    if (grp == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) so[wave][r][sub * EPL + e] = o[r][e];
      if (sub == 0) {
        sm[wave][r] = m_run[r];
        sl[wave][r] = l_run[r];
      }
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < nrows * DH; t += blockDim.x) {
    const int r = t / DH, c = t - r * DH;
    float M = sm[0][r];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm[w][r]);
    float L = 0.0f, acc = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(sm[w][r] - M);
      L += sl[w][r] * wgt;
      acc += so[w][r][c] * wgt;
    }
    const float res = acc / L;
    const int col = head * DH + c;
    if constexpr (OUT_XT) {
      reinterpret_cast<bf16_t*>(a.out)[xt_index(row0 + r, col, a.n_heads * DH)] = (bf16_t)res;
    } else {
      reinterpret_cast<float*>(a.out)[(size_t)(row0 + r) * a.n_heads * DH + col] = res;
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Sixteen batch rows of a prompt chunk per workgroup on the matrix cores (bf16 cache).  A workgroup owns 16
// consecutive batch rows of one head; rows of one sequence form a run whose K/V blocks are streamed ONCE, 32
// tokens per wavefront step, and multiplied against all 16 rows with v_mfma_f32_16x16x32_bf16:
//   scores^T [token][row] = K [token][dh] . q^T [dh][row]      (K straight from the cache as the A operand)
//   out^T    [dh][row]   += V^T [dh][token] . p^T [token][row]  (V transposed through a per-wavefront LDS tile)
// With the transposed products a lane holds everything of ONE row (row = lane % 16): its 8 scores of the step,
// its running maximum and its slice of the output, so the online softmax needs two shuffles per step and the
// probabilities go from the score registers into the next product without leaving the lane (the contraction
// slots of the second product are simply numbered in the order the first one delivers the tokens).
// q and the probabilities stay float in effect: each is split into a bf16 head and a bf16 remainder and
// multiplied twice.  Rows outside the current run, and positions after a row's own, are masked.
// ---------------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int CHUNK_ROWS = 16;
constexpr int VPITCH = 34;   // bf16 per transposed V row in LDS: 32 tokens + 2 (keeps the 8 writes of a lane group on separate banks)

template <int DH, bool OUT_XT>
__global__ __launch_bounds__(256) void attn_chunk_kernel(AttnArgs a, Pred pred) {
  constexpr int CH = DH / 32;   // 32-channel contraction steps of q . K
  constexpr int DT = DH / 16;   // 16-channel tiles of the output
  constexpr int VS_BYTES = NW * DH * VPITCH * 2;
  constexpr int SO_BYTES = NW * CHUNK_ROWS * DH * 4;
  extern __shared__ int32_t tbl[];
  __shared__ __align__(16) unsigned char smem[VS_BYTES > SO_BYTES ? VS_BYTES : SO_BYTES];
  __shared__ int s_seq[CHUNK_ROWS], s_npos[CHUNK_ROWS];
  __shared__ float sm[NW][CHUNK_ROWS], sl[NW][CHUNK_ROWS];
  if (pred_skip(pred)) return;

  const int head = blockIdx.x, row0 = blockIdx.y * CHUNK_ROWS;
  const int nrows = min(CHUNK_ROWS, a.B - row0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i16 = lane & 15, g = lane >> 4;
  const int my_row = row0 + i16;
  const bool row_ok = i16 < nrows;
  const int my_seq = row_ok ? safe_row(a.row_table[my_row], a.B) : -1;
  const int my_npos = row_ok ? min(a.context_lens[my_row] + 1, a.max_blocks * 16) : 0;
  if (threadIdx.x < CHUNK_ROWS) {
    s_seq[i16] = my_seq;
    s_npos[i16] = my_npos;
  }

  // q of this lane's row, channels c*32 + g*8 .. +8 of every contraction step, scaled, as bf16 head + remainder
  const float sc = 1.4426950408889634f / sqrtf((float)DH);
  bf16x8_t qh[CH], ql[CH];
  {
    const float* qp = a.q + ((size_t)(row_ok ? my_row : row0) * a.n_heads + head) * DH + g * 8;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const float4 lo = *reinterpret_cast<const float4*>(qp + c * 32);
      const float4 hi = *reinterpret_cast<const float4*>(qp + c * 32 + 4);
      const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = row_ok ? v[e] * sc : 0.0f;
        const __bf16 h = (__bf16)x;
        qh[c][e] = h;
        ql[c][e] = (__bf16)(x - (float)h);
      }
    }
  }

  float m_run = NEG_BIG, l_run = 0.0f;
  f32x4_t o[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d) o[d] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

  const size_t block_elems = (size_t)a.n_heads * 16 * DH;
  const size_t lane_off = (size_t)head * 16 * DH + (size_t)i16 * DH + g * 8;   // token i16 of a block, channels g*8..
  const bf16_t* kbase = reinterpret_cast<const bf16_t*>(a.k_pool) + lane_off;
  const bf16_t* vbase = reinterpret_cast<const bf16_t*>(a.v_pool) + lane_off;
  __bf16 (*vw)[VPITCH] = reinterpret_cast<__bf16 (*)[VPITCH]>(smem + (size_t)wave * DH * VPITCH * 2);

  __syncthreads();
  int r_begin = 0;
  while (r_begin < nrows) {
    // the run: rows r_begin .. r_end-1 of one sequence (uniform over the workgroup)
    const int run_seq = __builtin_amdgcn_readfirstlane(s_seq[r_begin]);
    int r_end = r_begin + 1;
    while (r_end < nrows && __builtin_amdgcn_readfirstlane(s_seq[r_end]) == run_seq) ++r_end;
    int run_ctx = 0;
    for (int r = r_begin; r < r_end; ++r) run_ctx = max(run_ctx, __builtin_amdgcn_readfirstlane(s_npos[r]));
    const int n_blocks = (run_ctx + 15) >> 4;
    const int n_steps = (n_blocks + 1) >> 1;
    const int32_t* table = a.block_tables + (size_t)run_seq * a.max_blocks;
    __syncthreads();   // the previous run's table is no longer read
    for (int x = threadIdx.x; x < n_blocks; x += blockDim.x) tbl[x] = safe_block(table[x], a.num_blocks);
    __syncthreads();
    const int npos_eff = (i16 >= r_begin && i16 < r_end) ? my_npos : 0;

    for (int s = wave; s < n_steps; s += NW) {
      // two 16-token blocks; an odd block count reads the last block twice (its second copy is masked)
      const int lb1 = min(2 * s + 1, n_blocks - 1);
      const size_t off[2] = {(size_t)__builtin_amdgcn_readfirstlane(tbl[2 * s]) * block_elems,
                             (size_t)__builtin_amdgcn_readfirstlane(tbl[lb1]) * block_elems};
      u32x4_t kt[2][CH], vt[2][CH];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          kt[t][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(kbase + off[t] + c * 32));
          // positions from the run's end on (also the second copy of a repeated last block) come from the zeros
          vt[t][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(
              s * 32 + t * 16 + i16 < run_ctx ? vbase + off[t] + c * 32 : reinterpret_cast<const bf16_t*>(&k_zero16)));
        }
      // scores^T of the 32 tokens: lane (i16, g) gets tokens 4g..4g+3 of each block for row i16
      f32x4_t st[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        st[t] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const bf16x8_t kk = __builtin_bit_cast(bf16x8_t, kt[t][c]);
          st[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, qh[c], st[t], 0, 0, 0);
          st[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, ql[c], st[t], 0, 0, 0);
        }
      }
      float sv[8];
      float mx = m_run;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int tok = s * 32 + t * 16 + 4 * g + r;
          sv[t * 4 + r] = tok < npos_eff ? st[t][r] : NEG_BIG;
          mx = fmaxf(mx, sv[t * 4 + r]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float alpha = __builtin_amdgcn_exp2f(m_run - mx);
      m_run = mx;
      l_run *= alpha;
#pragma unroll
      for (int d = 0; d < DT; ++d) o[d] *= alpha;
      bf16x8_t ph, pl;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int tok = s * 32 + t * 16 + 4 * g + r;
          const float p = tok < npos_eff ? __builtin_amdgcn_exp2f(sv[t * 4 + r] - mx) : 0.0f;
          l_run += p;
          const __bf16 h = (__bf16)p;
          ph[t * 4 + r] = h;
          pl[t * 4 + r] = (__bf16)(p - (float)h);
        }
      // V of the 32 tokens, transposed into this wavefront's LDS tile: vw[channel][token]
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const bf16x8_t vv = __builtin_bit_cast(bf16x8_t, vt[t][c]);
#pragma unroll
          for (int e = 0; e < 8; ++e) vw[c * 32 + g * 8 + e][t * 16 + i16] = vv[e];
        }
      // out^T += V^T . p^T; contraction slot e of lane group g is token 4g+e of the first block (e < 4) or
      // token 4g+e-4 of the second: the order in which ph / pl hold the probabilities
#pragma unroll
      for (int d = 0; d < DT; ++d) {
        const __bf16* rowp = &vw[16 * d + i16][0];
        bf16x8_t va;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          va[e] = rowp[4 * g + e];
          va[4 + e] = rowp[16 + 4 * g + e];
        }
        o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, ph, o[d], 0, 0, 0);
        o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pl, o[d], 0, 0, 0);
      }
    }
    r_begin = r_end;
  }

  // the four lane groups of a row hold partial sums of the same maximum; then merge the wavefronts row by row
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();   // every wavefront is done with its V tile: the space now holds the partial outputs
  float (*so)[CHUNK_ROWS][DH] = reinterpret_cast<float (*)[CHUNK_ROWS][DH]>(smem);
#pragma unroll
  for (int d = 0; d < DT; ++d)
    *reinterpret_cast<float4*>(&so[wave][i16][16 * d + 4 * g]) = make_float4(o[d][0], o[d][1], o[d][2], o[d][3]);
  if (g == 0) {
    sm[wave][i16] = m_run;
    sl[wave][i16] = l_run;
  }
  __syncthreads();
  // one thread per (row, 8 consecutive channels): 16-byte (bf16 operand order) or 2 x 16-byte (float) stores
  {
    constexpr int G8 = DH / 8;
    const int r = threadIdx.x / G8, c0 = (threadIdx.x % G8) * 8;
    if (r < nrows) {
      float M = sm[0][r];
#pragma unroll
      for (int w = 1; w < NW; ++w) M = fmaxf(M, sm[w][r]);
      float L = 0.0f, acc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float wgt = __builtin_amdgcn_exp2f(sm[w][r] - M);
        L += sl[w][r] * wgt;
        const float4 lo = *reinterpret_cast<const float4*>(&so[w][r][c0]);
        const float4 hi = *reinterpret_cast<const float4*>(&so[w][r][c0 + 4]);
        const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v[e] * wgt;
      }
      const float inv = 1.0f / L;
      const int col = head * DH + c0;
      if constexpr (OUT_XT) {
        bf16x8_t o8;
#pragma unroll
        for (int e = 0; e < 8; ++e) o8[e] = (__bf16)(acc[e] * inv);
        *reinterpret_cast<bf16x8_t*>(reinterpret_cast<bf16_t*>(a.out) + xt_index(row0 + r, col, a.n_heads * DH)) = o8;
      } else {
        float* op = reinterpret_cast<float*>(a.out) + (size_t)(row0 + r) * a.n_heads * DH + col;
        *reinterpret_cast<float4*>(op) = make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
        *reinterpret_cast<float4*>(op + 4) = make_float4(acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv);
      }
    }
  }
}

// Four rows per workgroup measured best at the 7B shape (eight: 300 registers, one wavefront per SIMD, slower).
constexpr int ROWS_PER_GROUP = 4;

template <class T, int DH>
void launch_t(const AttnArgs& a, Pred pred, hipStream_t st) {
  dim3 block(256);
  const size_t lds = (size_t)a.max_blocks * sizeof(int32_t);
  if (a.row_table) {   // rows share sequences: stream every sequence's K/V once per group of rows
    if constexpr (std::is_same<T, bf16_t>::value) {
      dim3 grid16(a.n_heads, (a.B + CHUNK_ROWS - 1) / CHUNK_ROWS);
      if (a.out_xt)
        hipLaunchKernelGGL((attn_chunk_kernel<DH, true>), grid16, block, lds, st, a, pred);
      else
        hipLaunchKernelGGL((attn_chunk_kernel<DH, false>), grid16, block, lds, st, a, pred);
      return;
    }
    dim3 grid(a.n_heads, (a.B + ROWS_PER_GROUP - 1) / ROWS_PER_GROUP);
    if (a.out_xt)
      hipLaunchKernelGGL((attn_rows_kernel<T, DH, ROWS_PER_GROUP, true>), grid, block, lds, st, a, pred);
    else
      hipLaunchKernelGGL((attn_rows_kernel<T, DH, ROWS_PER_GROUP, false>), grid, block, lds, st, a, pred);
    return;
  }
  if (a.split_ws && a.split_parts > 1) {
    // the output form only matters to the merge launch; the parts always leave as floats
    dim3 grid(a.n_heads, a.B, a.split_parts);
    hipLaunchKernelGGL((attn_decode_kernel<T, DH, false, true>), grid, block, lds, st, a, pred);
    dim3 gridm(a.n_heads, a.B);
    if (a.out_xt)
      hipLaunchKernelGGL((attn_merge_kernel<DH, true>), gridm, dim3(DH), 0, st, a, pred);
    else
      hipLaunchKernelGGL((attn_merge_kernel<DH, false>), gridm, dim3(DH), 0, st, a, pred);
    return;
  }
  dim3 grid(a.n_heads, a.B);
  if (a.out_xt)
    hipLaunchKernelGGL((attn_decode_kernel<T, DH, true, false>), grid, block, lds, st, a, pred);
  else
    hipLaunchKernelGGL((attn_decode_kernel<T, DH, false, false>), grid, block, lds, st, a, pred);
}

}  // namespace

// One workgroup per (sequence, head) keeps the chip busy from about 256 pairs on.  With at most 64, up to eight
// workgroups share a pair so that about 256 run, as long as every part still has eight blocks (128 positions) of the
// table's width to walk: below that, and at 128 pairs (measured: 28.6 against 29.0 us at 4 x 2048 positions), the second
// launch costs what the idle compute units would have gained.  Measured at the 7B shape, one sequence: 16384
// positions 147 -> 52 us per layer, 4096 positions 41 -> 21 us.
int attn_split_parts(int B, int n_heads, int max_blocks) {
  const long pairs = (long)B * n_heads;
  if (pairs <= 0 || pairs > kAttnSplitMaxPairs) return 1;
  int parts = (int)(256 / pairs);
  if (parts > kAttnMaxSplit) parts = kAttnMaxSplit;
  if (parts > max_blocks / 8) parts = max_blocks / 8;
  return parts < 2 ? 1 : parts;
}

int launch_attention(const AttnArgs& a, int dtype, Pred pred, hipStream_t st) {
  if (a.B == 0) return EE_OK;
  if (a.split_parts > 1 && a.row_table) EE_FAIL(EE_ERR_UNSUPPORTED, "attention: split_parts does not go with row_table");
  if (a.split_parts > kAttnMaxSplit) EE_FAIL(EE_ERR_UNSUPPORTED, "attention: split_parts %d above %d", a.split_parts, kAttnMaxSplit);
  if (a.max_blocks < 1 || a.max_blocks > TABLE_LDS_MAX)
    EE_FAIL(EE_ERR_UNSUPPORTED, "attention: max_blocks %d outside 1..%d", a.max_blocks, TABLE_LDS_MAX);
  if (a.out_pos && a.row_table) EE_FAIL(EE_ERR_UNSUPPORTED, "attention: out_pos does not go with row_table");
  if (dtype == EE_FP32) {
    if (a.head_dim == 64) launch_t<float, 64>(a, pred, st);
    else if (a.head_dim == 128) launch_t<float, 128>(a, pred, st);
    else EE_FAIL(EE_ERR_UNSUPPORTED, "attention: head_dim %d not supported for fp32 (64 or 128)", a.head_dim);
  } else {
    if (a.head_dim == 64) launch_t<bf16_t, 64>(a, pred, st);
    else if (a.head_dim == 128) launch_t<bf16_t, 128>(a, pred, st);
    else EE_FAIL(EE_ERR_UNSUPPORTED, "attention: head_dim %d not supported for bf16 (64 or 128)", a.head_dim);
  }
  return EE_OK;
}

}  // namespace ee
