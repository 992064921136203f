// bf16 projections of the decode step on the matrix cores (v_mfma_f32_32x32x16_bf16).  Three kernels, by batch size:
//
//   gemm_mfma_kernel   one or two 32-row batch tiles, few output tiles (QKV, output projection): a weight streamer.
//                      Every weight byte is fetched from HBM exactly once, straight into registers (1 KiB of
//                      consecutive bytes per wavefront load thanks to the packed tile order), the small activation
//                      operand comes out of L2.  A workgroup of four wavefronts owns one 32-row output tile and splits
//                      the contraction four ways; the partial tiles meet in LDS.
//   gemm_tiled_kernel  everything else up to 384 rows, and the projections with few output tiles beyond: the four
//                      wavefronts own different output tiles over the same contraction range and share the activation
//                      operand through LDS; 128-row chunks.
//   gemm_ring_kernel   LM head and gate/up at 385-512 rows, where the matrix cores are what counts: 256 x 256 blocks.
//
// The epilogues (rotary + paged cache write, partial results of the residual updates, SwiGLU, exit-head softmax
// statistics) run on the finished sums, from LDS in the first kernel and from registers in the other two.
//
// The second operand is bf16 in operand-tile order: the attention output, the SwiGLU product, or the normalised
// hidden state written by finish_norm_kernel.  (Building the normalised operand on the fly from the float residual
// stream inside the loop was tried and measured slower: twice the L2 traffic per weight byte plus the conversion
// arithmetic cost more than the normalisation launch they replaced.)
#include <type_traits>

#include "ee_common.h"
#include "ee_epilogue.h"
#include "ee_decide.h"

namespace ee {
namespace {

constexpr int NW = 4;  // wavefronts per workgroup
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct FillCtl {  // KV filling: one grid.z slice per layer
  FillLayers layers;
  const bf16_t* x_slabs;
  size_t x_slab_elems;
  size_t pool_layer_bytes;
};

struct Lds {
  float red[NW][16][64];
  float zt[32][33];
  float part[8][32];
  int flag;
};

// KV filling: should this workgroup (layer slice `layer`) return at once?  Uniform over the workgroup.  With one
// fill-from layer for the whole batch (Algorithm 1) the predicate word and that layer are fetched together: the
// workgroup waits for one memory round trip, not three, before its first weight load.
__device__ inline bool fill_skip(const Pred& pred, const QkvEpi& e, int M, int layer, int& lds_flag) {
  if (e.fill_from_stride == 0) {
    const int32_t from = ctl_load(e.fill_from);
    const int32_t flag = pred.flag ? ctl_load(pred.flag) : 0;
    if (pred.flag && ((flag != 0) != (pred.run_when != 0))) return true;
    return !(from < layer);
  }
  if (pred_skip(pred)) return true;
  if (threadIdx.x == 0) lds_flag = 0;
  __syncthreads();
  int need = 0;
  for (int m = threadIdx.x; m < M; m += blockDim.x) need |= e.fill_from[m] < layer;
  if (need) lds_flag = 1;
  __syncthreads();
  const bool any = lds_flag != 0;
  __syncthreads();
  return !any;
}

// Meets the four wavefronts' partial 32x32 tiles in LDS and runs the epilogue on the finished sums.
// Thread t owns result rows r16(a) and r16(a)+16 for a = 2*(t/64), 2*(t/64)+1 in column t%32 (+32*(t%64/32) picks
// the upper row group): the two rows that an epilogue needs together always sit in the same thread.
template <class Epi>
__device__ inline void tile_finish(const f32x16& acc, int nt, int mt_global, const GemmShape& g, const Epi& e, Lds& s,
                                   int wave, int lane, int row_half = -1) {
  __syncthreads();
#pragma unroll
  for (int a = 0; a < 16; ++a) s.red[wave][a][lane] = acc[a];
  __syncthreads();
  const int l2 = threadIdx.x & 63, qq = threadIdx.x >> 6;
  const int m = mt_global * 32 + (l2 & 31);
  float vlo[2], vhi[2];
  int r16[2];
#pragma unroll
  for (int ai = 0; ai < 2; ++ai) {
    const int a = 2 * qq + ai;
    vlo[ai] = s.red[0][a][l2] + s.red[1][a][l2] + s.red[2][a][l2] + s.red[3][a][l2];
    vhi[ai] = s.red[0][a + 8][l2] + s.red[1][a + 8][l2] + s.red[2][a + 8][l2] + s.red[3][a + 8][l2];
    r16[ai] = (a >> 2) * 8 + (l2 >> 5) * 4 + (a & 3);
  }
  if constexpr (std::is_same<Epi, LmEpi>::value) {
    const float r = m < g.M ? row_rinv(e.rowsq, m, e.d_model, e.eps) : 0.0f;
#pragma unroll
    for (int ai = 0; ai < 2; ++ai) {
      s.zt[r16[ai]][l2 & 31] = vlo[ai] * r;
      s.zt[r16[ai] + 16][l2 & 31] = vhi[ai] * r;
    }
    __syncthreads();
    {   // eight neighbouring lanes share one batch row: four logits each
      const int ml = threadIdx.x >> 3, part = threadIdx.x & 7;
      float z[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) z[i] = s.zt[part * 4 + i][ml];
      const HeadStat st = stat_of_8x4(z, nt * 32 + part * 4, e.scale);
      const int mm = mt_global * 32 + ml;
      if (part == 0 && mm < g.M) e.partials[(size_t)mm * e.n_parts + (nt - g.tile_begin)] = stat_pack(st);
    }
  } else if constexpr (std::is_same<Epi, AccEpi>::value) {
    // This workgroup summed one slice of the contraction (blockIdx.y): the tile goes to that slice of the partial
    // results with plain stores, transposed through LDS so that a batch row's 32 channels leave as whole 16-byte
    // pieces.  The normalisation launch that follows sums the slices in slice order: no atomics, no dependence on
    // which workgroup finishes first.  (Plain row order of the packed matrix: tile row r is channel nt*32 + r.)
#pragma unroll
    for (int ai = 0; ai < 2; ++ai) {
      s.zt[r16[ai]][l2 & 31] = vlo[ai];
      s.zt[r16[ai] + 16][l2 & 31] = vhi[ai];
    }
    __syncthreads();
    {
      const int mr = threadIdx.x >> 3, c0 = (threadIdx.x & 7) * 4;
      const int mm = mt_global * 32 + mr;
      if (mm < g.M) {
        const float4 v = make_float4(s.zt[c0][mr], s.zt[c0 + 1][mr], s.zt[c0 + 2][mr], s.zt[c0 + 3][mr]);
        *reinterpret_cast<float4*>(e.h + ((size_t)blockIdx.y * e.Mpad + mm) * e.n_out + nt * 32 + c0) = v;
      }
    }
  } else {
    if constexpr (std::is_same<Epi, QkvEpi>::value) {
      // The tile holds, for each of its 32 batch rows, 16 consecutive channels of one head and their 16 rotary
      // partners (half a head further on).  Rotate in registers, stage the tile in LDS, then write whole 16-channel
      // runs (one 16-byte store per thread) instead of single elements scattered over the cache blocks.
      const int d = e.d_model, dh = e.head_dim, hdim = dh >> 1;
      const int f0 = packed_row_lo(nt, 0, g.pair_stride);   // first channel of the tile (uniform)
      const int which = f0 / d;                              // 0 q, 1 k, 2 v
      const int head = (f0 - which * d) / dh;
      const int j0 = f0 - which * d - head * dh;             // < dh/2, a multiple of 16
      const int mcol = l2 & 31;
#pragma unroll
      for (int ai = 0; ai < 2; ++ai) {
        float lo = vlo[ai], hi = vhi[ai];
        if (m < g.M) {
          const float r = row_rinv(e.rowsq, m, e.d_model, e.eps);
          lo *= r;
          hi *= r;
          if (which < 2 && e.rope_theta > 0.0f) {
            const float2 cs = e.rope[(size_t)m * hdim + j0 + r16[ai]];
            const float a = lo * cs.x - hi * cs.y;
            const float b = hi * cs.x + lo * cs.y;
            lo = a;
            hi = b;
          }
        }
        s.zt[r16[ai]][mcol] = lo;
        s.zt[16 + r16[ai]][mcol] = hi;
      }
      __syncthreads();
      if (which == 0) {
        if (e.q) {   // thread -> (row, run, quarter of the run): four floats
          const int mr = threadIdx.x >> 3, part = threadIdx.x & 7, run = part >> 2, c0 = run * 16 + (part & 3) * 4;
          const int mm = mt_global * 32 + mr;
          if (mm < g.M && !(e.fill_from && !(e.fill_from[(size_t)mm * e.fill_from_stride] < e.layer))) {
            float4 v = make_float4(s.zt[c0][mr], s.zt[c0 + 1][mr], s.zt[c0 + 2][mr], s.zt[c0 + 3][mr]);
            *reinterpret_cast<float4*>(e.q + (size_t)mm * d + head * dh + j0 + run * hdim + (part & 3) * 4) = v;
          }
        }
      } else if (threadIdx.x < 128) {   // thread -> (row, run, half of the run): eight bf16
        const int mr = threadIdx.x >> 2, part = threadIdx.x & 3, run = part >> 1, c0 = run * 16 + (part & 1) * 8;
        const int mm = mt_global * 32 + mr;
        // a workgroup that computed one half of the tile's rows (row_half) holds one of the two runs only
        if (mm < g.M && (row_half < 0 || run == row_half) &&
            !(e.fill_from && !(e.fill_from[(size_t)mm * e.fill_from_stride] < e.layer))) {
          const int p = e.context_lens[mm];
          const bool p_ok = (unsigned)p < (unsigned)(e.max_blocks * 16);
          const int blk = e.block_tables[(size_t)(e.row_table ? safe_row(e.row_table[mm], e.table_rows) : mm) * e.max_blocks + (p_ok ? p >> 4 : 0)];
          const size_t at = (((size_t)blk * e.n_heads + head) * 16 + (p & 15)) * dh + j0 + run * hdim + (part & 1) * 8;
          bf16x8 v;
#pragma unroll
          for (int i = 0; i < 8; ++i) v[i] = (bf16_t)s.zt[c0 + i][mr];
          bf16_t* pool = reinterpret_cast<bf16_t*>(which == 1 ? e.k_pool : e.v_pool);
          if (p_ok && (unsigned)blk < (unsigned)e.num_blocks) *reinterpret_cast<bf16x8*>(pool + at) = v;
        }
      }
    } else {
      if (m < g.M) {
#pragma unroll
        for (int ai = 0; ai < 2; ++ai) {
          const int f_lo = packed_row_lo(nt, r16[ai], g.pair_stride);
          epi_gateup<bf16_t>(e, m, f_lo, vlo[ai], vhi[ai]);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Main loop 1: bf16 operand tiles on both sides
// ---------------------------------------------------------------------------------------------------------
template <int MT, int U>
struct Frag {
  u32x4 w[U];
  u32x4 x[MT][U];
};

template <int MT, int U>
__device__ inline void frag_load(Frag<MT, U>& f, const u32x4* __restrict__ wp, const u32x4* __restrict__ xp,
                                 size_t x_tile_stride, int ks) {
#pragma unroll
  for (int u = 0; u < U; ++u) f.w[u] = __builtin_nontemporal_load(wp + (size_t)(ks + u) * 64);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int u = 0; u < U; ++u) f.x[mt][u] = xp[mt * x_tile_stride + (size_t)(ks + u) * 64];
}

// Last, partial group: steps past ks1 re-read the last valid weight tile against a zero activation tile.
template <int MT, int U>
__device__ inline void frag_load_tail(Frag<MT, U>& f, const u32x4* __restrict__ wp, const u32x4* __restrict__ xp,
                                      size_t x_tile_stride, int ks, int ks1) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const bool ok = ks + u < ks1;
    const int kk = ok ? ks + u : ks1 - 1;
    f.w[u] = __builtin_nontemporal_load(wp + (size_t)kk * 64);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      u32x4 v = xp[mt * x_tile_stride + (size_t)kk * 64];
      f.x[mt][u] = ok ? v : u32x4{0, 0, 0, 0};
    }
  }
}

template <int MT, int U>
__device__ inline void frag_mma(const Frag<MT, U>& f, f32x16 (&acc)[MT]) {
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.w[u]),
                                                        __builtin_bit_cast(bf16x8, f.x[mt][u]), acc[mt], 0, 0, 0);
}

template <int MT, int U, class Epi, bool FILL>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmShape g, Epi e, Pred pred, FillCtl fc, CombineJob cj) {
  __shared__ Lds s;

  int bx = blockIdx.x;
  if constexpr (std::is_same<Epi, QkvEpi>::value && !FILL) {
    // Leading workgroups: the exit decision of the previous layer, one row each.  That layer ran if the batch
    // has not left, or left at that very layer or later (the words may already show a sibling's update of this
    // launch; `done` set at an earlier layer comes with a smaller batch exit layer, both visible since an earlier
    // launch).  The projection's own workgroups apply the SAME rule instead of the live flag, so every workgroup of
    // the launch takes the same branch whatever the interleaving: the projection of the layer after the batch exit
    // layer always runs (what it caches is what KV filling caches there anyway), and a tile that two workgroups
    // share is never left half done.
    if (cj.n_wg) {
      const IterState& cs = cj.kind == 1 ? cj.a.s : cj.d.s;
      const int decided_layer = cj.kind == 1 ? cj.a.layer : cj.d.layer;
      const bool ran = ctl_load(cs.done) == 0 || ctl_load(cs.batch_exit_layer) >= decided_layer;
      if (bx < cj.n_wg) {
        if (cj.kind == 1) {
          if (bx < cj.a.B && ran) combine_row(cj.a, bx, reinterpret_cast<float4*>(&s.red[0][0][0]));
        } else if (bx == 0 && ran) {
          for (int m = threadIdx.x; m < cj.d.B; m += blockDim.x) decide_from_dot(cj.d, m);
        }
        return;
      }
      if (!ran) return;
      bx -= cj.n_wg;
    } else if (pred_skip(pred)) {
      return;
    }
  } else if constexpr (!FILL) {
    if (pred_skip(pred)) return;
  }
  if constexpr (FILL) {
    const int layer = (int)gridDim.z - (int)blockIdx.z;   // deepest layer first: the slices that have work start first
    if (fill_skip(pred, e, g.M, layer, s.flag)) return;
    g.w = fc.layers.w_qkv[layer - 1];
    g.x = fc.x_slabs + (size_t)(layer - 1) * fc.x_slab_elems;
    e.layer = layer;
    e.k_pool = reinterpret_cast<char*>(e.k_pool) + (size_t)(layer - 1) * fc.pool_layer_bytes;
    e.v_pool = reinterpret_cast<char*>(e.v_pool) + (size_t)(layer - 1) * fc.pool_layer_bytes;
  }

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // Tiles that two workgroups share come first in the grid (two consecutive block indices per tile): each computes
  // 16 of the tile's 32 output rows, i.e. one of its two 16-channel runs, over the whole contraction, from the half
  // of every weight tile that holds those rows (two 256-byte pieces of each kilobyte).  Both halves are complete
  // results: the workgroups share nothing and never meet.  With 384 tiles on 256 compute units this turns two rounds
  // of workgroups into one and a half.  Only tiles without a rotation may be split (V: the host sees to that).
  const bool half_tile = bx < 2 * g.split_tiles;
  int tl = half_tile ? bx >> 1 : bx - 2 * g.split_tiles;   // tile within its class (halved / whole)
  int rhalf = bx & 1;
  if constexpr (std::is_same<Epi, QkvEpi>::value) {
    // Four consecutive tiles hold the 128 channels of one head (or two heads of 64): each writes 32-byte runs of
    // the same cache lines of the paged cache (64-byte runs of q).  Workgroup ids congruent modulo 8 run on the
    // same XCD behind the same L2, so the four tiles of a head get ids 8 apart: their partial lines meet in that
    // L2 before they go to memory.  Only whole groups are rearranged (32 whole tiles = 8 heads x 4 tiles; 64 half
    // tiles = 8 heads x 4 tiles x 2 halves, both halves of a tile on one XCD as well).
    if (half_tile) {
      if (bx < ((2 * g.split_tiles) & ~63)) {
        const int q = (bx >> 3) & 7;
        tl = (((bx >> 6) << 3) + (bx & 7)) * 4 + (q >> 1);
        rhalf = q & 1;
      }
    } else if (tl < ((g.n_tiles - g.split_tiles) & ~31)) {
      tl = (tl & ~31) + ((tl & 7) << 2) + ((tl >> 3) & 3);
    }
  }
  const int nt = half_tile ? g.tile_begin + g.n_tiles - g.split_tiles + tl : g.tile_begin + tl;
  const int k_steps = g.K >> 4;
  const int chunks = gridDim.y * NW;
  const int c = blockIdx.y * NW + wave;
  const int ks0 = (int)((long)k_steps * c / chunks);
  const int ks1 = (int)((long)k_steps * (c + 1) / chunks);
  const int m_tiles = (g.M + 31) >> 5;
  const size_t x_tile_stride = (size_t)k_steps * 64;

  // Lane l of a weight tile holds row l % 32.  In a halved tile the lanes of the other 16 rows fetch what their
  // partner lanes fetch (the same bytes, no further memory traffic): their result rows are duplicates, never written.
  const int wlane = half_tile ? ((lane & ~16) | (rhalf << 4)) : lane;
  const u32x4* wp = reinterpret_cast<const u32x4*>(g.w) + (size_t)nt * k_steps * 64 + wlane;

  for (int mt0 = 0; mt0 < m_tiles; mt0 += MT) {
    const u32x4* xp = reinterpret_cast<const u32x4*>(g.x) + (size_t)mt0 * x_tile_stride + lane;
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][i] = 0.0f;

    // double-buffered stream over this wavefront's share of the contraction
    Frag<MT, U> A, B;
    const int n = (ks1 - ks0) / U;
    int k = ks0;
    if (n > 0) frag_load(A, wp, xp, x_tile_stride, k);
    int i = 0;
    // (An unconditional steady-state loop with counted waits that keeps a whole group in flight behind the one
    // being multiplied was measured too: no faster in the decode step, so the simpler loop stays.)
    for (; i + 2 <= n; i += 2) {
      frag_load(B, wp, xp, x_tile_stride, k + U);
      frag_mma(A, acc);
      if (i + 2 < n) frag_load(A, wp, xp, x_tile_stride, k + 2 * U);
      frag_mma(B, acc);
      k += 2 * U;
    }
    if (i < n) {
      frag_mma(A, acc);
      k += U;
    }
    if (k < ks1) {
      frag_load_tail(A, wp, xp, x_tile_stride, k, ks1);
      frag_mma(A, acc);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) tile_finish(acc[mt], nt, mt0 + mt, g, e, s, wave, lane, half_tile ? rhalf : -1);
  }
}

// ---------------------------------------------------------------------------------------------------------
// Main loop 2 (from three 32-row batch tiles on; LM head, gate/up and down projection always): the four
// wavefronts of a workgroup own four different 32-row
// output tiles over the SAME contraction range, so the activation operand is fetched from L2 once per
// workgroup, staged in LDS and read by all four; weights still go straight from HBM to registers, each byte
// once per batch chunk of MT*32 rows.  Groups of UT contraction steps: while group g is multiplied, the loads
// of groups g+1 and g+2 are in flight (three rotating weight register sets, two activation register sets that
// drain into two LDS stages).  Every wavefront finishes its own tiles, so the epilogue runs from registers.
// ---------------------------------------------------------------------------------------------------------
constexpr int UT = 4;
__device__ u32x4 k_zero_tile[64];   // one operand tile of zeros, never written (activation rows past the contraction range; not const: it must live in the same address space as the operands)

// Epilogue of one finished 32 x 32 result tile held in a wavefront's registers (tiled and ring kernels): accumulator a
// (< 8) of a lane is result row r16 = (a/4)*8 + (lane/32)*4 + a%4 of column lane%32, accumulator a+8 is row r16+16 (its
// partner row in the packed order).  nt: packed weight tile, mtile: 32-row batch tile, M_eff: valid rows, ksl: the
// contraction slice this workgroup summed (accumulate projections).
template <class Epi>
__device__ inline void finish_from_registers(const f32x16& acc, int nt, int mtile, int M_eff, int ksl, const GemmShape& g,
                                             const Epi& e, int lane) {
  const int half = lane >> 5, ml = lane & 31;
  const int m = mtile * 32 + ml;
  if constexpr (std::is_same<Epi, LmEpi>::value) {
    // this lane's 16 logits of the row in ascending vocabulary order: rows r16(a), a = 0..7, then r16(a)+16
    float z[16];
    int zi[16];
    const float rs = m < M_eff ? row_rinv(e.rowsq, e.perm ? e.perm[m] : m, e.d_model, e.eps) : 0.0f;
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      const int r16 = (a >> 2) * 8 + half * 4 + (a & 3);
      z[a] = acc[a] * rs;
      zi[a] = nt * 32 + r16;
      z[a + 8] = acc[a + 8] * rs;
      zi[a + 8] = nt * 32 + r16 + 16;
    }
    HeadStat st = stat_of<16>(z, zi, e.scale);
    HeadStat o;
    o.zmax = __shfl_xor(st.zmax, 32);
    o.sum = __shfl_xor(st.sum, 32);
    o.z2 = __shfl_xor(st.z2, 32);
    o.idx = __shfl_xor(st.idx, 32);
    st = stat_merge(st, o, e.scale);
    if (half == 0 && m < M_eff) {
      const int row = e.perm ? e.perm[m] : m;
      e.partials[(size_t)row * e.n_parts + (nt - g.tile_begin)] = stat_pack(st);
    }
  } else if constexpr (std::is_same<Epi, AccEpi>::value) {
    // this workgroup's contraction slice (ksl) of the partial results, plain 16-byte stores: a lane holds, for its
    // batch row, two runs of four consecutive channels and the two runs 16 channels further on
    if (m < M_eff) {
      float* row = e.h + ((size_t)ksl * e.Mpad + m) * e.n_out + nt * 32 + half * 4;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        *reinterpret_cast<float4*>(row + q * 8) = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
        *reinterpret_cast<float4*>(row + q * 8 + 16) =
            make_float4(acc[4 * q + 8], acc[4 * q + 9], acc[4 * q + 10], acc[4 * q + 11]);
      }
    }
  } else {
    if (m < M_eff) {
      // this lane holds two runs of four consecutive output rows (and their partners 16 rows on) of its batch row
#pragma unroll
      for (int run = 0; run < 2; ++run) {
        const int f_lo0 = packed_row_lo(nt, run * 8 + half * 4, g.pair_stride);
        float lo[4], hi[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          lo[i] = acc[run * 4 + i];
          hi[i] = acc[run * 4 + i + 8];
        }
        if constexpr (std::is_same<Epi, QkvEpi>::value) {
          epi_qkv4(e, m, f_lo0, lo, hi);
        } else {
          epi_gateup4(e, m, f_lo0, lo, hi);
        }
      }
    }
  }
}

template <int MT>
struct TiledLds {
  u32x4 b[2][UT][MT][64];
  int flag;
};

template <int MT, int NTW, class Epi, bool FILL>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmShape g, Epi e, Pred pred, FillCtl fc) {
  __shared__ TiledLds<MT> s;
  constexpr int XR = UT * MT / NW;   // activation tiles each wavefront stages per group
  static_assert(UT * MT % NW == 0, "stage must split evenly over the wavefronts");

  if constexpr (!FILL) {
    if (pred_skip(pred)) return;
  } else {
    const int layer = (int)gridDim.z - (int)blockIdx.z;   // deepest layer first: the slices that have work start first
    if (fill_skip(pred, e, g.M, layer, s.flag)) return;
    g.w = fc.layers.w_qkv[layer - 1];
    g.x = fc.x_slabs + (size_t)(layer - 1) * fc.x_slab_elems;
    e.layer = layer;
    e.k_pool = reinterpret_cast<char*>(e.k_pool) + (size_t)(layer - 1) * fc.pool_layer_bytes;
    e.v_pool = reinterpret_cast<char*>(e.v_pool) + (size_t)(layer - 1) * fc.pool_layer_bytes;
  }

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m_tiles = (g.M + 31) >> 5;
  const int chunks = (m_tiles + MT - 1) / MT;   // the last chunk may be short: its missing tiles re-read its last
                                                // valid one, and their rows are never written
  // One-dimensional grid.  Workgroup ids that are congruent modulo 8 run on the same XCD and share its L2, so
  // the workgroups that stream the SAME weight tiles (the batch chunks and contraction slices of one tile group)
  // get consecutive ids of one residue class: they start together on one XCD, and all but the first read of a
  // weight tile hit that L2 instead of going out to memory once per chunk.
  const int ny = g.grid_y;                      // chunks * contraction slices
  const int ksplit = ny / chunks;
  const int slot = (int)blockIdx.x >> 3;
  int bx, by;
  if (g.n_rows_dev) {
    // compacted operand: most chunks may have nothing to do, and their workgroups return at once; chunk-major
    // order keeps those behind the chunks that work instead of in between them
    const int groups8 = (int)gridDim.x / (8 * ny);
    by = slot / groups8;
    bx = (slot % groups8) * 8 + ((int)blockIdx.x & 7);
  } else {
    bx = (slot / ny) * 8 + ((int)blockIdx.x & 7);
    by = slot % ny;
  }
  // Which output tiles this workgroup owns.  Even split: four per workgroup.  Uneven split (g.even_wgs > 0, one
  // chunk, no contraction slices): the tiles are dealt out over exactly g.even_wgs workgroups, n_tiles / even_wgs
  // or one more each, and a wavefront beyond its workgroup's count owns none: it still stages its share of the
  // activation operand, but streams no weights.  A compute unit sustains only so many bytes per second from beyond
  // its L2, so the launch is as fast as its most loaded compute unit: 688 tiles as 172 x 4 keep a third of the chip
  // idle while 172 units stream four tiles each; as 176 x 3 + 80 x 2 nobody streams more than three.
  int my_tiles = NW, tile0 = bx * NW * NTW;
  if (g.even_wgs > 0) {
    if (bx >= g.even_wgs) return;
    const int base = g.n_tiles / g.even_wgs, rem = g.n_tiles % g.even_wgs;
    my_tiles = base + (bx < rem ? 1 : 0);
    tile0 = bx * base + min(bx, rem);
  } else if (tile0 >= g.n_tiles) {
    return;                                     // the group count is padded to a multiple of 8
  }
  const bool active = wave < my_tiles;
  const int chunk = by / ksplit, ksl = by % ksplit;
  // compacted operand: only the first *n_rows_dev rows hold sequences that are still active
  const int M_eff = g.n_rows_dev ? g.n_rows_dev[0] : g.M;
  if (chunk * MT * 32 >= M_eff) return;
  // this wavefront's NTW consecutive output tiles (a wavefront without tiles points at the workgroup's first: never loaded)
  const int nt0 = g.tile_begin + tile0 + (active ? wave : 0) * NTW;
  const int k_steps = g.K >> 4;
  const int ks0 = (int)((long)k_steps * ksl / ksplit);
  const int ks1 = (int)((long)k_steps * (ksl + 1) / ksplit);
  const size_t x_tile_stride = (size_t)k_steps * 64;
  const size_t w_tile_stride = (size_t)k_steps * 64;
  const u32x4* wp = reinterpret_cast<const u32x4*>(g.w) + (size_t)nt0 * k_steps * 64 + lane;
  const u32x4* xp = reinterpret_cast<const u32x4*>(g.x) + (size_t)(chunk * MT) * x_tile_stride + lane;
  const int mt_last = min(MT, m_tiles - chunk * MT) - 1;   // last batch tile of this chunk that exists

  f32x16 acc[NTW][MT];
#pragma unroll
  for (int t = 0; t < NTW; ++t)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[t][mt][i] = 0.0f;

  // Everything in the loop is unconditional (a conditional load would force the compiler to wait for every
  // outstanding load where the branches meet): the group count is rounded up to the rotation period and
  // groups past the end load a clamped weight tile against zero activations.
  const int n = (ks1 - ks0 + UT - 1) / UT;
  // The main loop exists twice, chosen once per wavefront: with and without a weight stream.  Both take the same
  // barriers.
  auto main_loop = [&](auto streams_c) {
    constexpr bool STREAMS = decltype(streams_c)::value;
    u32x4 W[4][NTW][UT], X[2][XR];
    auto gload = [&](int grp, u32x4 (&wr)[NTW][UT], u32x4 (&xr)[XR]) {
      const int kbase = ks0 + grp * UT;
      if constexpr (STREAMS) {
#pragma unroll
        for (int u = 0; u < UT; ++u) {
          const int kk = kbase + u < ks1 ? kbase + u : ks1 - 1;
#pragma unroll
          for (int t = 0; t < NTW; ++t) wr[t][u] = __builtin_nontemporal_load(wp + t * w_tile_stride + (size_t)kk * 64);
        }
      }
#pragma unroll
      for (int j = 0; j < XR; ++j) {
        const int t = wave + NW * j, u = t / MT, mt = t % MT;
        // past the end: a tile of zeros, chosen by address (a select on the loaded value would sit right behind
        // the load and make the wavefront wait for everything it has in flight)
        const bool ok = kbase + u < ks1;
        const u32x4* src = ok ? xp + min(mt, mt_last) * x_tile_stride + (size_t)(kbase + u) * 64 : k_zero_tile + lane;
        xr[j] = *src;
      }
    };
    // One group: drain its activation registers into LDS stage XS, start the loads of group grp+2 into the
    // registers just freed and an idle weight set, multiply group grp.
    auto step = [&](int grp, const u32x4 (&wcur)[NTW][UT], u32x4 (&wnext2)[NTW][UT], u32x4 (&xs)[XR], int XS) {
      // keeps the LDS stores below from being hoisted into the previous group, ahead of its loads: there they would
      // wait for loads that were only just issued
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < XR; ++j) {
        const int t = wave + NW * j;
        s.b[XS][t / MT][t % MT][lane] = xs[j];
      }
      __syncthreads();
      gload(grp + 2, wnext2, xs);
      if constexpr (STREAMS) {
        // the LDS reads of contraction step u+1 are issued before the multiplies of step u
        u32x4 bf[2][MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) bf[0][mt] = s.b[XS][0][mt][lane];
#pragma unroll
        for (int u = 0; u < UT; ++u) {
          if (u + 1 < UT) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) bf[(u + 1) & 1][mt] = s.b[XS][u + 1][mt][lane];
          }
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < NTW; ++t)
              acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wcur[t][u]),
                                                                   __builtin_bit_cast(bf16x8, bf[u & 1][mt]), acc[t][mt], 0, 0, 0);
        }
        if constexpr (MT >= 4) {
          // Order of the group, spelled out for the scheduler: the first step's fragments, then one fragment read
          // of the next step behind every NTW multiplies, the last step's multiplies.  Left alone it issues each
          // read right in front of the multiplies that use it and the matrix cores wait out every LDS round trip.
          __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);
#pragma unroll
          for (int i = 0; i < (UT - 1) * MT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, NTW, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, MT * NTW, 0);
        }
      }
    };

    gload(0, W[0], X[0]);
    gload(1, W[1], X[1]);
    for (int gi = 0; gi < n; gi += 4) {
      step(gi, W[0], W[2], X[0], 0);
      step(gi + 1, W[1], W[3], X[1], 1);
      step(gi + 2, W[2], W[0], X[0], 0);
      step(gi + 3, W[3], W[1], X[1], 1);
    }
    __syncthreads();
  };
  if (active) {
    main_loop(std::true_type{});
  } else {
    main_loop(std::false_type{});
    return;       // nothing to finish; the epilogues below take no workgroup barrier
  }

  // every wavefront finishes its own tiles from registers
#pragma unroll
  for (int t = 0; t < NTW; ++t)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) finish_from_registers(acc[t][mt], nt0 + t, chunk * MT + mt, M_eff, ksl, g, e, lane);
}

// ---------------------------------------------------------------------------------------------------------
// Main loop 3 (LM head and gate/up at 385 to 512 rows, where the matrix cores are what counts): one workgroup owns a
// 256-row x 256-column block of the result (eight batch tiles x eight weight tiles).  Wavefront w owns two weight
// tiles (64 columns) against all eight batch tiles, 16 accumulator tiles = all 256 accumulation registers:
//   * its weight fragments come straight from HBM into registers, RING_D contraction steps ahead (nobody else in
//     the workgroup needs them, so they never touch LDS);
//   * the activation fragments of a step (8 KiB, needed by all four wavefronts) land in a ring of RING_D + 1 LDS
//     slots through direct-to-LDS loads, two tiles per wavefront, just as far ahead: a wavefront's loads complete
//     in order, so a fragment from L2 queued behind a weight tile from HBM is ready no sooner than that tile and must
//     have been asked for as early;
//   * one bare barrier per contraction step (a fence would wait for every load in flight): at step s every
//     wavefront has waited for its own two tiles of step s+1, and the slot of step s-1, whose fragments everybody
//     has multiplied, takes step s+RING_D.
// Per compute unit and step: 16 KiB from memory, 8 KiB written to and 32 KiB read from LDS, 64 MFMAs.  Every weight
// byte leaves HBM once: the two row blocks of a column block run on one XCD and meet in its L2.
// ---------------------------------------------------------------------------------------------------------
constexpr int RING_D = 15;
constexpr int RING_LDS_BYTES = (RING_D + 1) * 8 * 1024;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;
template <int N>
__device__ inline void wait_loads_but() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

template <class Epi>
__global__ __launch_bounds__(256) void gemm_ring_kernel(GemmShape g, Epi e, Pred pred) {
  extern __shared__ u32x4 ring[];   // [RING_D + 1][8 batch tiles][64 lanes]
  if (pred_skip(pred)) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m_tiles = (g.M + 31) >> 5;
  const int row_blocks = (m_tiles + 7) >> 3, col_blocks = g.n_tiles >> 3;
  // ids congruent modulo 8 share an XCD: the row blocks of one column block get consecutive ids of one class
  const int xcd = (int)blockIdx.x & 7, j = (int)blockIdx.x >> 3;
  const int bm = j % row_blocks, bn = (j / row_blocks) * 8 + xcd;
  if (bn >= col_blocks) return;
  const int M_eff = g.M;            // (compacted operands stay with the tiled kernel, which skips empty 128-row chunks)
  const int k_steps = g.K >> 4;     // a multiple of RING_D + 1 (the host checks)
  const int nt0 = g.tile_begin + bn * 8 + wave * 2;
  const u32x4* wsrc[2];
  const u32x4* xsrc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    wsrc[i] = reinterpret_cast<const u32x4*>(g.w) + (size_t)(nt0 + i) * k_steps * 64 + lane;
    xsrc[i] = reinterpret_cast<const u32x4*>(g.x) + (size_t)min(bm * 8 + wave * 2 + i, m_tiles - 1) * k_steps * 64 + lane;
  }
  // Exactly four loads per wavefront and step, in this order; steps past the end repeat the last one (never used).
  auto issue = [&](int s, u32x4 (&wr)[2], int slot) {
    const int ss = s < k_steps ? s : k_steps - 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) wr[i] = __builtin_nontemporal_load(wsrc[i] + (size_t)ss * 64);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      __builtin_amdgcn_global_load_lds((global_void_ptr)(xsrc[i] + (size_t)ss * 64),
                                       (lds_void_ptr)(ring + ((size_t)slot * 8 + wave * 2 + i) * 64), 16, 0, 0);
  };
  auto read_x = [&](u32x4 (&f)[8], int slot) {
    const u32x4* sp = ring + (size_t)slot * 8 * 64 + lane;
#pragma unroll
    for (int b = 0; b < 8; ++b) f[b] = sp[b * 64];
  };
  f32x16 acc[2][8];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

  u32x4 wr[RING_D + 1][2];
  u32x4 f[2][8];
#pragma unroll
  for (int q = 0; q < RING_D; ++q) {
    issue(q, wr[q], q);
    asm volatile("" ::: "memory");      // the counted waits rely on the loads of a step staying together, in step order
  }
  wait_loads_but<(RING_D - 1) * 4>();   // step 0 has landed; the loop's own waits take it from there
  __builtin_amdgcn_s_barrier();
  read_x(f[0], 0);
  // q = s % (RING_D + 1): step s lives in register set / ring slot q
  auto step = [&](int s, const u32x4 (&wcur)[2], u32x4 (&wnew)[2], const u32x4 (&fcur)[8], u32x4 (&fnext)[8], int q) {
    // loads issued after this wavefront's activation tiles of step s+1: the RING_D - 2 steps s-13 .. s-1
    wait_loads_but<(RING_D - 2) * 4>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    issue(s + RING_D, wnew, (q + RING_D) % (RING_D + 1));
    read_x(fnext, (q + 1) % (RING_D + 1));
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
      for (int a = 0; a < 2; ++a)
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wcur[a]),
                                                            __builtin_bit_cast(bf16x8, fcur[b]), acc[a][b], 0, 0, 0);
    // the multiplies start at once; one load, then one fragment read, goes out behind each of the first twelve
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    __builtin_amdgcn_sched_barrier(0);
  };
  static_assert(RING_D == 15, "the loop below is unrolled for sixteen register sets");
  for (int s = 0; s < k_steps; s += 16) {
#define EE_RING_STEP(i) step(s + i, wr[i], wr[(i + 15) % 16], f[i & 1], f[(i + 1) & 1], i)
    EE_RING_STEP(0); EE_RING_STEP(1); EE_RING_STEP(2); EE_RING_STEP(3);
    EE_RING_STEP(4); EE_RING_STEP(5); EE_RING_STEP(6); EE_RING_STEP(7);
    EE_RING_STEP(8); EE_RING_STEP(9); EE_RING_STEP(10); EE_RING_STEP(11);
    EE_RING_STEP(12); EE_RING_STEP(13); EE_RING_STEP(14); EE_RING_STEP(15);
#undef EE_RING_STEP
  }
  wait_loads_but<0>();   // the repeated loads past the end still target LDS and registers
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b)
      if (bm * 8 + b < m_tiles) finish_from_registers(acc[a][b], nt0 + a, bm * 8 + b, M_eff, 0, g, e, lane);
}

// Which shapes the ring kernel serves: 385 to 512 rows (two row blocks, the second at least half full: below that the
// tiled kernel's 128-row chunks waste less; above, the workgroups no longer fit the chip in one round), whole blocks
// of eight weight tiles, a contraction of whole groups of sixteen steps.
bool ring_serves(int M, int n_tiles, int K) {
  return M > 384 && M <= 512 && n_tiles % 8 == 0 && (K >> 4) % (RING_D + 1) == 0 && (K & 15) == 0;
}

// Batch tiles per pass of the streaming kernel / per chunk of the tiled kernel.
int pick_mt(int M, int cap) {
  const int m_tiles = (M + 31) / 32;
  for (int mt = cap; mt > 1; mt >>= 1)
    if (m_tiles % mt == 0) return mt;
  return 1;
}

// From three batch tiles on, the tiled kernel (128-row chunks, the last one padded) beats re-streaming the weights
// once per pass of the streaming kernel.
bool tiled(int M, int n_tiles) { return (M + 31) / 32 >= 3 && n_tiles % NW == 0; }

// Which kernel an accumulate projection (output or down projection) of M rows onto n_tiles packed tiles over a
// contraction of K runs in, and how many contraction slices it writes.  Every slice is one more partial result for
// the normalisation launch to read, so the count stays as small as filling the chip allows.
struct AccPlan {
  int kind;     // 0: streaming kernel, 1: tiled kernel with 128-row chunks, 2: tiled kernel, one chunk of one or two tiles
  int ksplit;
};
AccPlan acc_plan(int M, int n_tiles, int K) {
  const int m_tiles = (M + 31) / 32, k_steps = K / 16;
  AccPlan p{0, 1};
  if (tiled(M, n_tiles)) {
    const int chunks = (m_tiles + 3) / 4, groups = n_tiles / NW;
    // one workgroup per compute unit (measured at 96-512 rows: better than two), slices of at least 64 steps
    p.kind = 1;
    p.ksplit = 256 / (groups * chunks);
  } else if (m_tiles <= 2 && n_tiles % NW == 0 && k_steps >= 512) {
    p.kind = 2;
    p.ksplit = 256 / (n_tiles / NW);
  } else {
    // streaming kernel (its four wavefronts already split the slice four ways): enough workgroups for every
    // compute unit, no more
    p.ksplit = (256 + n_tiles - 1) / n_tiles;
  }
  if (p.ksplit > k_steps / 64) p.ksplit = k_steps / 64;
  if (p.ksplit > 8) p.ksplit = 8;   // the normalisation launch adds at most eight partial results
  if (p.ksplit < 1) p.ksplit = 1;
  return p;
}

// The ring kernel needs 128 KiB of dynamic LDS: asked for once per process (the attribute belongs to the function,
// not to a launch), at the first launch that wants it or by gemm_bf16_prepare().
template <class Epi>
bool ring_allowed() {
  static int ok = -1;
  if (ok < 0)
    ok = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_kernel<Epi>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             RING_LDS_BYTES) == hipSuccess;
  return ok > 0;
}

template <class Epi, bool FILL>
void launch(const GemmShape& g, const Epi& e, Pred pred, const FillCtl& fc, int nz, hipStream_t st,
            const CombineJob& cj = CombineJob{}) {
  dim3 block(256);
  const int m_tiles = (g.M + 31) / 32;
  constexpr bool ACC = std::is_same<Epi, AccEpi>::value;
  const AccPlan ap = ACC ? acc_plan(g.M, g.n_tiles, g.K) : AccPlan{0, 1};
  // Batch chunks of 4 tiles (128 rows) measured faster than 8 at batch 256 and 512: twice the workgroups, each
  // with half the accumulators, keeps more loads in flight; the second chunk's weight reads mostly hit the caches.
  if (tiled(g.M, g.n_tiles)) {
    // tiled kernel: the workgroup's output tiles share the activation operand through LDS
    const int chunks = (m_tiles + 3) / 4;
    // One output tile per wavefront, except for the LM head (below).
    const int groups = g.n_tiles / NW;
    const int ksplit = ap.ksplit;
    if constexpr (std::is_same<Epi, QkvEpi>::value && !FILL) {
      // Few output tiles and one 128-row chunk leave most compute units idle (QKV at 7B width: 96 workgroups):
      // 64-row chunks double the workgroups as long as they all still start at once (measured at 128 rows:
      // 61 -> 45 us; with more workgroups than compute units the second weight pass costs more than it gains).
      const int chunks2 = (m_tiles + 1) / 2;
      if (!g.n_rows_dev && groups * chunks < 128 && groups * chunks2 <= 256) {
        GemmShape g2 = g;
        g2.grid_y = chunks2;
        dim3 grid2((groups + 7) / 8 * 8 * chunks2, 1, nz);
        hipLaunchKernelGGL((gemm_tiled_kernel<2, 1, Epi, FILL>), grid2, block, 0, st, g2, e, pred, fc);
        return;
      }
    }
    if constexpr (!FILL && (std::is_same<Epi, LmEpi>::value || std::is_same<Epi, GateUpEpi>::value)) {
      // if the runtime refused the ring its 128 KiB of dynamic LDS, the tiled kernel below serves the shape
      if (ring_allowed<Epi>() && !g.n_rows_dev && ring_serves(g.M, g.n_tiles, g.K)) {
        const int row_blocks = (m_tiles + 7) / 8, col_blocks = g.n_tiles / 8;
        dim3 gridr((col_blocks + 7) / 8 * 8 * row_blocks, 1, 1);
        hipLaunchKernelGGL((gemm_ring_kernel<Epi>), gridr, block, RING_LDS_BYTES, st, g, e, pred);
        return;
      }
    }
    GemmShape g4 = g;
    g4.grid_y = chunks * ksplit;
    if constexpr (!FILL && std::is_same<Epi, LmEpi>::value) {
      // LM head: two output tiles per wavefront (each LDS operand read feeds two MFMAs, half the workgroups):
      // 161 -> 153 us at 512 rows.  The same arrangement is slower for gate/up (119 -> 135 us) and is not used there.
      // (from two 128-row chunks on: with one chunk it would halve the workgroups below the compute units; for the same
      // reason not with a compacted operand, where often only the first chunk holds rows)
      if (g.n_tiles % (2 * NW) == 0 && chunks >= 2 && !g.n_rows_dev) {
        const int groups2 = g.n_tiles / (2 * NW);
        dim3 grid2((groups2 + 7) / 8 * 8 * chunks * ksplit, 1, nz);
        hipLaunchKernelGGL((gemm_tiled_kernel<4, 2, Epi, FILL>), grid2, block, 0, st, g4, e, pred, fc);
        return;
      }
    }
    dim3 grid((groups + 7) / 8 * 8 * chunks * ksplit, 1, nz);
    hipLaunchKernelGGL((gemm_tiled_kernel<4, 1, Epi, FILL>), grid, block, 0, st, g4, e, pred, fc);
    return;
  }
  // One or two batch tiles: the tiled kernel still wins where enough output tiles keep the chip busy with four
  // tiles per workgroup (its four wavefronts share every activation tile through LDS, a quarter of the L2 reads
  // of the streaming kernel): LM head, gate/up and the down projection (measured at 32 rows: 47.0 -> 44.0,
  // 34.6 -> 33.2, 21.8 -> 20.8 us; at 64 rows: 62.8 -> 43.5, 44.4 -> 38.3, 27.5 -> 25.4).  QKV and the output
  // projection have too few tiles for that and stay with the streaming kernel.
  // KV filling takes the same route: one launch covers many layers, so there are always enough workgroups, and the
  // four tiles of a workgroup are the 128 channels of one head, whose cache lines then leave from one L2.
  if constexpr (FILL || !std::is_same<Epi, QkvEpi>::value) {
    const bool small_tiled = ACC ? ap.kind == 2 : (m_tiles <= 2 && g.n_tiles % NW == 0 && g.split_tiles == 0);
    if (small_tiled) {
      const int groups = g.n_tiles / NW;
      GemmShape gs = g;
      gs.grid_y = ap.ksplit;   // one chunk
      dim3 grid1((groups + 7) / 8 * 8 * ap.ksplit, 1, nz);
      // Fewer groups of four than compute units, more tiles than compute units: deal the tiles out over all 256
      // units instead (two to four each), so that no unit streams more than its share.
      if (!ACC && !FILL && groups < 256 && g.n_tiles > 256) {
        gs.even_wgs = 256;
        grid1 = dim3(256, 1, nz);
      }
      if (m_tiles == 1)
        hipLaunchKernelGGL((gemm_tiled_kernel<1, 1, Epi, FILL>), grid1, block, 0, st, gs, e, pred, fc);
      else
        hipLaunchKernelGGL((gemm_tiled_kernel<2, 1, Epi, FILL>), grid1, block, 0, st, gs, e, pred, fc);
      return;
    }
  }
  // split tiles take two workgroups each (one batch tile only); the workgroups of a combine job come first
  dim3 grid(g.n_tiles + g.split_tiles + cj.n_wg, ACC ? ap.ksplit : 1, nz);
  switch (pick_mt(g.M, 4)) {
    case 4:
      hipLaunchKernelGGL((gemm_mfma_kernel<4, 2, Epi, FILL>), grid, block, 0, st, g, e, pred, fc, cj);
      break;
    case 2:
      hipLaunchKernelGGL((gemm_mfma_kernel<2, 4, Epi, FILL>), grid, block, 0, st, g, e, pred, fc, cj);
      break;
    default:
      hipLaunchKernelGGL((gemm_mfma_kernel<1, 8, Epi, FILL>), grid, block, 0, st, g, e, pred, fc, cj);
  }
}

}  // namespace

bool gemm_bf16_is_tiled(int M, int n_tiles) { return tiled(M, n_tiles); }

void gemm_bf16_prepare() {
  ring_allowed<LmEpi>();
  ring_allowed<GateUpEpi>();
}

int gemm_acc_slices(int M, int n_tiles, int K) { return acc_plan(M, n_tiles, K).ksplit; }

bool gemm_qkv_carries_combine(int M) { return (M + 31) / 32 <= 2; }   // the streaming kernel serves these batches

void launch_gemm_qkv_bf16(const GemmShape& g, const QkvEpi& e, Pred pred, hipStream_t st, const CombineArgs* with_combine,
                          const DecideArgs* with_decide) {
  FillCtl fc{};
  CombineJob cj{};
  if (with_combine) {
    cj.a = *with_combine;
    cj.kind = 1;
    cj.n_wg = (with_combine->B + 7) / 8 * 8;   // a multiple of 8: the tiles keep their XCDs
  } else if (with_decide) {
    cj.d = *with_decide;
    cj.kind = 2;
    cj.n_wg = 8;
  }
  launch<QkvEpi, false>(g, e, pred, fc, 1, st, cj);
}
void launch_gemm_acc_bf16(const GemmShape& g, const AccEpi& e, Pred pred, hipStream_t st) {
  FillCtl fc{};
  launch<AccEpi, false>(g, e, pred, fc, 1, st);
}
void launch_gemm_gateup_bf16(const GemmShape& g, const GateUpEpi& e, Pred pred, hipStream_t st) {
  FillCtl fc{};
  launch<GateUpEpi, false>(g, e, pred, fc, 1, st);
}
void launch_gemm_lm_bf16(const GemmShape& g, const LmEpi& e, Pred pred, hipStream_t st) {
  FillCtl fc{};
  launch<LmEpi, false>(g, e, pred, fc, 1, st);
}
void launch_gemm_kvfill_bf16(const FillLayers& fl, int n_layers, const bf16_t* x_slabs, size_t x_slab_elems,
                             size_t pool_layer_elems, const GemmShape& g, const QkvEpi& e, Pred pred, hipStream_t st) {
  FillCtl fc{};
  fc.layers = fl;
  fc.x_slabs = x_slabs;
  fc.x_slab_elems = x_slab_elems;
  fc.pool_layer_bytes = pool_layer_elems * sizeof(bf16_t);
  launch<QkvEpi, true>(g, e, pred, fc, n_layers, st);
}

}  // namespace ee
