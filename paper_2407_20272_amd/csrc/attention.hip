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

template <class T, int DH, bool OUT_XT>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a, Pred pred) {
  if (pred_skip(pred)) return;
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
  const int n_ctx = a.context_lens[b] + 1; // positions 0..p inclusive
  const int n_blocks = (n_ctx + 15) >> 4;
  const int32_t* table = a.block_tables + (size_t)b * a.max_blocks;

  // q slice, pre-scaled so that exp2 can be used: softmax(x) = 2^(x*log2 e)
  float q[EPL];
  {
    const float sc = 1.4426950408889634f / sqrtf((float)DH);
    const float* qp = a.q + ((size_t)b * a.n_heads + head) * DH + sub * EPL;
#pragma unroll
    for (int i = 0; i < EPL; ++i) q[i] = qp[i] * sc;
  }

  float m_run = NEG_BIG, l_run = 0.0f, o[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) o[i] = 0.0f;

  const size_t head_off = (size_t)head * 16 * DH;             // elements, inside a block
  const size_t block_elems = (size_t)a.n_heads * 16 * DH;
  const T* kbase = reinterpret_cast<const T*>(a.k_pool) + head_off + (size_t)grp * DH + sub * EPL;
  const T* vbase = reinterpret_cast<const T*>(a.v_pool) + head_off + (size_t)grp * DH + sub * EPL;

  uint4 kc[LPB], vc[LPB], kn[LPB], vn[LPB];
  int lb = wave;
  if (lb < n_blocks) {
    const size_t off = (size_t)table[lb] * block_elems;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      kc[i] = *reinterpret_cast<const uint4*>(kbase + off + (size_t)i * TPL * DH);
      vc[i] = *reinterpret_cast<const uint4*>(vbase + off + (size_t)i * TPL * DH);
    }
  }
  for (; lb < n_blocks; lb += NW) {
    const int nxt = lb + NW;
    if (nxt < n_blocks) {
      const size_t off = (size_t)table[nxt] * block_elems;
#pragma unroll
      for (int i = 0; i < LPB; ++i) {
        kn[i] = *reinterpret_cast<const uint4*>(kbase + off + (size_t)i * TPL * DH);
        vn[i] = *reinterpret_cast<const uint4*>(vbase + off + (size_t)i * TPL * DH);
      }
    }
    // scores of this lane group's LPB tokens of the block
    float s[LPB];
    float m_new = m_run;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      float kf[EPL];
      Elems<T>::unpack(kc[i], kf);
      float d = 0.0f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(q[e], kf[e], d);
#pragma unroll
      for (int x = 1; x < LPT; x <<= 1) d += __shfl_xor(d, x);
      const int tok = lb * 16 + i * TPL + grp;
      s[i] = tok < n_ctx ? d : NEG_BIG;
      m_new = fmaxf(m_new, s[i]);
    }
    const float alpha = exp2f(m_run - m_new);
    l_run *= alpha;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] *= alpha;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      const int tok = lb * 16 + i * TPL + grp;
      const float p = tok < n_ctx ? exp2f(s[i] - m_new) : 0.0f;
      l_run += p;
      float vf[EPL];
      Elems<T>::unpack(vc[i], vf);
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] = fmaf(p, vf[e], o[e]);
    }
    m_run = m_new;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      kc[i] = kn[i];
      vc[i] = vn[i];
    }
  }

  // merge the TPL lane groups of the wavefront
#pragma unroll
  for (int x = LPT; x < 64; x <<= 1) {
    const float m_o = __shfl_xor(m_run, x);
    const float l_o = __shfl_xor(l_run, x);
    const float m_new = fmaxf(m_run, m_o);
    const float wa = exp2f(m_run - m_new), wb = exp2f(m_o - m_new);
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
      const float wgt = exp2f(sm[w] - M);
      L += sl[w] * wgt;
      acc += so[w][threadIdx.x] * wgt;
    }
    const float r = acc / L;
    const int col = head * DH + threadIdx.x;
    if constexpr (OUT_XT) {
      reinterpret_cast<bf16_t*>(a.out)[xt_index(b, col, a.n_heads * DH)] = (bf16_t)r;
    } else {
      reinterpret_cast<float*>(a.out)[(size_t)b * a.n_heads * DH + col] = r;
    }
  }
}

template <class T, int DH>
void launch_t(const AttnArgs& a, Pred pred, hipStream_t st) {
  dim3 grid(a.n_heads, a.B), block(256);
  if (a.out_xt)
    hipLaunchKernelGGL((attn_decode_kernel<T, DH, true>), grid, block, 0, st, a, pred);
  else
    hipLaunchKernelGGL((attn_decode_kernel<T, DH, false>), grid, block, 0, st, a, pred);
}

}  // namespace

int launch_attention(const AttnArgs& a, int dtype, Pred pred, hipStream_t st) {
  if (a.B == 0) return EE_OK;
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
