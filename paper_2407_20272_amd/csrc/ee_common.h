// Shared declarations of the early-exit decode library: types, memory layouts, launch interfaces.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ee_decode.h"

namespace ee {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------------------------
// Error reporting (host)
// ---------------------------------------------------------------------------------------------------
void set_error(const char* fmt, ...);
#define EE_FAIL(code, ...)      \
  do {                          \
    ee::set_error(__VA_ARGS__); \
    return (code);              \
  } while (0)
#define EE_HIP(expr)                                                                        \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) EE_FAIL(EE_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// ---------------------------------------------------------------------------------------------------
// Layouts of the bf16 path.
//
// XT ("operand tiles"): a [rows m][cols k] bf16 activation matrix stored in the order in which the
//   32x32x16 MFMA wants its second operand: [m/32][k/16][lane][8] with lane = (m%32) + 32*((k%16)/8) and
//   element k%8, so a wavefront fetches one 32x16 operand tile as 1 KiB of consecutive bytes.
// The fp32 residual stream is plain row-major [Mpad][d].  The output and down projections do not add into it:
//   each contraction slice writes its partial result to a slice of its own ([slices][Mpad][d], plain stores), and
//   the normalisation kernel that follows sums the slices in slice order, adds them to the residual row and
//   normalises it.  No float atomics anywhere, so the bf16 path is reproducible bit for bit.
// ---------------------------------------------------------------------------------------------------
__host__ __device__ inline size_t xt_index(int m, int k, int K) {
  return ((size_t)(m >> 5) * (size_t)(K >> 4) + (size_t)(k >> 4)) * 512 + (size_t)((((k >> 3) & 1) << 5) + (m & 31)) * 8 +
         (size_t)(k & 7);
}
__host__ __device__ inline int round_up(int x, int to) { return (x + to - 1) / to * to; }

// Packed weight row order: packed tile `nt`, row r (0..31) holds plain output row
//   f_lo(nt, r%16) + (r/16) * pair_stride,   f_lo = (nt / tpb) * 2*pair_stride + 16*(nt % tpb) + r%16,  tpb = pair_stride/16.
// pair_stride 16 is the identity order.
__host__ __device__ inline int packed_row_lo(int nt, int r16, int pair_stride) {
  const int tpb = pair_stride >> 4;
  return (nt / tpb) * 2 * pair_stride + ((nt % tpb) << 4) + r16;
}

// ---------------------------------------------------------------------------------------------------
// Per-iteration device state
// ---------------------------------------------------------------------------------------------------
struct IterState {
  int32_t* status;            // [B] sticky exit status
  int32_t* exit_layer;        // [B]
  int32_t* n_exited;          // [1]
  int32_t* done;              // [1] 1 once every sequence of the batch is accepted
  int32_t* batch_exit_layer;  // [1] output_layer of Algorithm 1
};

// Compaction of the rows that are still active (per-sequence exit at batch sizes the tiled projection kernel
// serves): position p < *n_active of a compacted operand holds batch row perm[p]; cpos is the inverse map.
// The map is rebuilt after every exit check and is constant inside a layer.
struct RowMap {
  int32_t* perm;      // [Mpad]; nullptr = no compaction (every row, in place)
  int32_t* cpos;      // [Mpad] batch row -> position, -1 for a sequence that has left
  int32_t* n_active;  // [1]
};

// Epilogue parameter blocks ---------------------------------------------------------------------------
struct QkvEpi {                 // rotary embedding + paged cache write (+ q output)
  float* q;                     // [M][d] fp32 or nullptr (KV filling)
  void* k_pool;                 // layer base of the pools ([num_blocks][H][16][dh])
  void* v_pool;
  const int32_t* context_lens;  // [M]
  const int32_t* block_tables;  // [M][max_blocks]
  const int32_t* row_table;     // nullptr, or [M]: row m uses row row_table[m] of block_tables
  const int32_t* fill_from;     // nullptr, or [M]: only rows with fill_from[m] < layer are written (KV filling)
  int fill_from_stride;         // 1 = per row, 0 = one value for the whole batch
  int layer;
  int max_blocks, n_heads, head_dim, d_model;
  float rope_theta;
  const float2* rope;           // [M][dh/2] (cos, sin) of the rotary angles at context_lens[m] (rope_theta > 0)
  const float* rowsq;           // nullptr, or [M] sum of squares of the hidden row: value *= rsqrt(rowsq/d + eps)
  float eps;
  int num_blocks;               // blocks per layer of the pools: a slot whose block id or position is out of range is not written
  int table_rows;               // rows of block_tables (the batch size): a row_table entry outside 0..table_rows-1 is read as 0
};
struct AccEpi {                 // residual update
  float* h;                     // fp32 path: the residual stream [M][n_out], added to in place (one contributor per element).
                                // bf16 path: partial results [slices][Mpad][n_out]; slice s receives the sum over the
                                // s-th part of the contraction (operand row m -> row m: compacted operands stay compacted)
  int Mpad;                     // row count of a slice (bf16 path) or 0 (fp32 path)
  int n_out;
  const int32_t* skip;          // fp32 path: nullptr, or [M]: rows with skip[m] != 0 keep their hidden state
};
struct GateUpEpi {              // act = silu(gate) * up
  void* act;                    // XT bf16 [Mpad][f] (bf16 path) or plain float [M][f]
  int d_ffn;
  const float* rowsq;
  float eps;
  int d_model;
};
struct LmEpi {                  // per-tile softmax statistics of the scaled logits
  float4* partials;             // [M][n_parts]: {max logit (unscaled), sum exp(scale*(z - max)), 2nd max, arg max as int bits}
  float* logits;                // fp32 path: [M][vocab] raw logits; bf16 path: nullptr
  int n_parts;
  int vocab;
  float scale;                  // logit_scale * layer
  const float* rowsq;
  float eps;
  int d_model;
  const int32_t* perm;          // nullptr, or [M]: operand row m is batch row perm[m] (compacted operand, tiled kernel only)
};

// ---------------------------------------------------------------------------------------------------
// Launchers (each enqueues on `st`).  A launch carries a predicate on a device word: its kernels return at once
// unless (*flag != 0) == run_when.  The layer loop runs while the all-exited flag is 0, KV filling once it is 1.
// ---------------------------------------------------------------------------------------------------
struct Pred {
  const int32_t* flag;  // nullptr = always run
  int run_when;         // run when (*flag != 0) == run_when
};

// misc.hip
void launch_iter_init(const IterState& s, int B, int n_layers, float* conf_out, hipStream_t st);
void launch_embed_bf16(const bf16_t* E, const int32_t* tokens, float* h, int B, int Mpad, int d, int vocab, hipStream_t st);
void launch_embed_f32(const float* E, const int32_t* tokens, float* h, int B, int d, int vocab, hipStream_t st);
void launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t st);
void launch_rope_table(const int32_t* context_lens, float2* table, int B, int head_dim, float theta, hipStream_t st);
struct GainTable {
  const void* g[EE_MAX_LAYERS];
};
// Optional second job of a normalisation launch (confidence measures that need no LM head, Section 2.1):
// dots[m] = sum_k h[m][k] * other, where other is the previous hidden state (per_row: [Mpad][d], the similarity
// measure) or one weight row shared by all rows ([d], the dedicated classifier); snapshot, if set, receives h
// (it may be the buffer `other` points to: every element is read before it is written, by the same thread).
struct RowDot {
  const float* other;
  float* snapshot;
  float* dots;      // [Mpad]
  int per_row;
};
// Rebuilds the row map from the status words (active rows keep their order).
void launch_compact(const int32_t* status, int B, const RowMap& rm, Pred pred, hipStream_t st);
// Residual update + RMSNorm of the bf16 path, one workgroup per batch row:
//   h[m] += y[0][p] + y[1][p] + .. (slice order; p = m, or cpos[m] with a row map; not for rows that have left),
//   rowsq_out[m] = sum_k h[m][k]^2, and for each gain j: x[j] row = bf16(h * rsqrt(rowsq/d + eps) * gain[j]) in
//   operand-tile order (at row m, or at position cpos[m] of a compacted operand, which is zero from *n_active on).
struct NormArgs {
  const float* h_in;      // [rows][d]
  float* h_out;           // nullptr (nothing to add) or the same buffer
  const float* y;         // [S][Mpad][d]
  int S;
  const int32_t* skip;    // nullptr, or [B] status words: rows with skip[m] != 0 have left and keep their hidden state
  RowMap rm;              // perm == nullptr: no compaction
  const bf16_t* gain[2];
  bf16_t* x[2];           // nullptr = unused
  int compacted[2];
  float* rowsq_out;       // nullptr or [Mpad]
  RowDot rd;
  float eps;
  int B, Mpad, d;
};
void launch_finish_norm(const NormArgs& a, Pred pred, hipStream_t st);
// KV filling: x slab of layer l = bf16(RMSNorm(h; gains.g[l-1])) for every layer some row needs (fill_from < l).
void launch_fill_prep(const float* h, const GainTable& gains, int n_layers, bf16_t* x_slabs, float eps,
                      const int32_t* fill_from, int fill_from_stride, int B, int Mpad, int d, Pred pred, hipStream_t st);
void launch_rmsnorm_f32(const float* h, const float* gain, float* x, int B, int d, float eps, Pred pred, hipStream_t st);
// fp32 path: out[0][m] = h[m] . other, out[1][m] = |other|^2, out[2][m] = |h[m]|^2 (out is [3][B]); other is
// the previous hidden state [B][d] (per_row) or one row [d]; with per_row, h is then copied over other.
void launch_measure_f32(const float* h, float* other, int per_row, float* out, int B, int d, Pred pred, hipStream_t st);
void launch_head_stats_f32(const float* logits, float4* partials, int B, int vocab, float scale, Pred pred,
                           hipStream_t st);
struct CombineArgs {
  const float4* partials;
  int n_parts;
  int B;
  int layer;           // 1-based; 0 = final token selection (no status update)
  float scale;         // logit_scale * layer
  float threshold;
  int conf_mode;
  const int32_t* forced_exit_layer;
  IterState s;
  int32_t* argmax_out;  // [B] or nullptr
  float* conf_out;      // [B] or nullptr
  const int32_t* left;  // nullptr, or [B]: rows with left[m] != 0 are not touched (per-sequence exit: token and state stay)
};
void launch_combine(const CombineArgs& a, Pred pred, hipStream_t st);
// Exit decision from a measure that is one dot product per row (conf_mode 2: cosine of consecutive hidden
// states = dots / sqrt(sq_a * sq_b); conf_mode 3: logistic function of dots * rsqrt(sq_b / d + eps) + bias[0],
// the classifier's unit applied to the hidden state at unit root mean square).
struct DecideArgs {
  const float* dots;   // [B]
  const float* sq_a;   // [B] squared norms (conf_mode 2)
  const float* sq_b;
  const float* bias;   // device, this layer's bias (conf_mode 3)
  int d;               // width of the hidden state
  float eps;
  int B;
  int layer;
  float threshold;
  int conf_mode;
  const int32_t* forced_exit_layer;
  IterState s;
  float* conf_out;
};
void launch_decide(const DecideArgs& a, Pred pred, hipStream_t st);
// The exit decision of layer i may ride along with the QKV projection launch of layer i+1 instead of taking a
// launch of its own (see launch_gemm_qkv_bf16): n_wg leading workgroups of that launch (a multiple of 8) take it.
// kind 1: softmax-response measures, workgroup m < a.B runs combine_row for batch row m.
// kind 2: one-dot-product measures, workgroup 0 runs decide_from_dot for every row.  n_wg == 0: none.
struct CombineJob {
  CombineArgs a;
  DecideArgs d;
  int kind;
  int n_wg;
};

// pack.hip
void launch_pack_weight(const bf16_t* w, int n_out, int n_in, int pair_stride, bf16_t* packed, hipStream_t st);

// gemm_mfma.hip (bf16 path).  w: packed; x: XT [Mpad][K].  tiles [tile_begin, tile_begin + n_tiles).
struct GemmShape {
  const void* w;
  const void* x;
  int K;            // contraction length
  int M;            // valid rows
  int tile_begin;   // first packed 32-row tile
  int n_tiles;      // tiles to compute
  int pair_stride;  // row order of the packed matrix
  int unused_;      // (kept so that aggregate initialisers stay positional)
  // QKV projection with one batch tile: the last split_tiles tiles (tiles without a rotation: V) are each computed
  // by two workgroups, 16 of the 32 output rows each, dispatched first; see gemm_mfma.hip.  0 = off.
  int split_tiles;
  // Tiled kernel only: nullptr, or the device-side number of valid operand rows (<= M).  Row chunks beyond it
  // return at once, rows beyond it are not written.
  const int32_t* n_rows_dev;
  int grid_y;   // set by the launcher (tiled kernel): batch chunks x contraction slices per group of output tiles
  int even_wgs; // set by the launcher (tiled kernel): > 0 = the tiles are dealt out evenly over this many workgroups
};
// Whether a projection of M rows onto n_tiles packed tiles runs in the tiled kernel (the one that takes
// n_rows_dev and the epilogues' perm).
bool gemm_bf16_is_tiled(int M, int n_tiles);
// One-time host-side set-up of the projection kernels (function attributes) that the first launch would otherwise do.
void gemm_bf16_prepare();
// with_combine != nullptr (only where gemm_qkv_carries_combine(M) holds): the launch also takes the exit decision
// of the previous layer.  The projection then runs SPECULATIVELY when that decision ends the iteration (its
// predicate word may or may not show the new value yet): what it caches for its layer is what KV filling
// (Section 3.2) caches there anyway, and KV filling runs afterwards over every layer above the batch exit layer.
void launch_gemm_qkv_bf16(const GemmShape& g, const QkvEpi& e, Pred pred, hipStream_t st,
                          const CombineArgs* with_combine = nullptr, const DecideArgs* with_decide = nullptr);
bool gemm_qkv_carries_combine(int M);
// Contraction slices the accumulate launch of this shape writes (the launch below uses exactly this many).
int gemm_acc_slices(int M, int n_tiles, int K);
void launch_gemm_acc_bf16(const GemmShape& g, const AccEpi& e, Pred pred, hipStream_t st);
void launch_gemm_gateup_bf16(const GemmShape& g, const GateUpEpi& e, Pred pred, hipStream_t st);
void launch_gemm_lm_bf16(const GemmShape& g, const LmEpi& e, Pred pred, hipStream_t st);
// KV filling over layers first..n in one launch: per-layer weights / x slabs / pools.
struct FillLayers {
  const void* w_qkv[EE_MAX_LAYERS];
};
void launch_gemm_kvfill_bf16(const FillLayers& fl, int n_layers, const bf16_t* x_slabs, size_t x_slab_elems,
                             size_t pool_layer_elems, const GemmShape& g, const QkvEpi& e, Pred pred, hipStream_t st);

// gemm_simple.hip (fp32 path).  w: plain [n_out][K]; x: plain [M][K].
struct SimpleShape {
  const float* w;
  const float* x;
  int K, M;
  int row_begin;    // first output row
  int n_rows;       // output rows to compute (even)
  int pair_stride;  // rows (f, f + pair_stride) are computed together
};
void launch_simple_qkv(const SimpleShape& g, const QkvEpi& e, Pred pred, hipStream_t st);
void launch_simple_acc(const SimpleShape& g, const AccEpi& e, Pred pred, hipStream_t st);
void launch_simple_gateup(const SimpleShape& g, const GateUpEpi& e, Pred pred, hipStream_t st);
void launch_simple_lm(const SimpleShape& g, const LmEpi& e, Pred pred, hipStream_t st);

// attention.hip
// Block ids and positions come from device memory the caller filled in; the kernels never let them reach outside
// the pools or the block table (the result for such a sequence is unspecified, the access is not).
__host__ __device__ inline int safe_block(int blk, int num_blocks) { return (unsigned)blk < (unsigned)num_blocks ? blk : 0; }
__host__ __device__ inline int safe_row(int row, int n_rows) { return (unsigned)row < (unsigned)n_rows ? row : 0; }

// Block-table entries per sequence that the attention kernels stage in LDS (contexts up to 262144 tokens).  The
// entry points check ee_batch.max_blocks against it before anything is enqueued.
constexpr int kAttnMaxBlocks = 16384;

struct AttnArgs {
  const float* q;               // [B][H*dh] fp32, rotary applied
  const void* k_pool;           // layer base
  const void* v_pool;
  const int32_t* context_lens;  // attends positions 0..context_lens[b] inclusive
  const int32_t* block_tables;
  int max_blocks, B, n_heads, head_dim;
  void* out;                    // fp32 plain [B][H*dh], or XT bf16 [Mpad][H*dh]
  int out_xt;                   // 1: XT bf16
  const int32_t* skip;          // nullptr, or [B]: sequences with skip[b] != 0 are not attended (they have left)
  const int32_t* row_table;     // nullptr, or [B]: row b uses row row_table[b] of block_tables
  const int32_t* out_pos;       // nullptr, or [B]: the result of sequence b goes to row out_pos[b] of out (compacted operand)
  int num_blocks;               // blocks per layer of the pools: a block id outside 0..num_blocks-1 is read as block 0
  // Few (sequence, head) pairs and long contexts: split_parts > 1 workgroups share one pair, each over a contiguous
  // range of the sequence's blocks; their partial results (running maximum, sum and unnormalised output:
  // head_dim + 2 floats each) meet in split_ws [B][H][split_parts][head_dim + 2] and a second launch merges them in
  // part order.  1 (or split_ws == nullptr) = one workgroup per pair.  Not with row_table.
  float* split_ws;
  int split_parts;
};
int launch_attention(const AttnArgs& a, int dtype, Pred pred, hipStream_t st);
// How many workgroups should share one (sequence, head) pair for this batch, and the floats of split_ws that takes.
int attn_split_parts(int B, int n_heads, int max_blocks);
inline size_t attn_split_floats(int B, int n_heads, int head_dim, int parts) {
  return parts > 1 ? (size_t)B * n_heads * parts * (head_dim + 2) : 0;
}
constexpr int kAttnMaxSplit = 8;
constexpr int kAttnSplitMaxPairs = 64;   // (sequence, head) pairs up to which the split form is used

}  // namespace ee
