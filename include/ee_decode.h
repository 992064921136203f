/*
 * ee_decode.h -- C ABI of the early-exit decode step for MI355X (gfx950).
 *
 * One call of ee_decode_iteration is one iteration of the paper's Algorithm 1
 * ("Iteration-level Batch Inference for Early-exit LLMs"): one new token for every
 * sequence of a batch, with the per-sequence sticky exit status of Section 3.1, the
 * whole-batch break at output_layer, and the KV-cache filling of Section 3.2.  The
 * other entry points expose the steps of that iteration one by one.
 *
 * Conventions
 *   - "dev" pointers are DEVICE pointers owned by the caller; the library borrows
 *     them for the duration of the enqueued work and never frees them.  "host"
 *     pointers are read before the call returns.
 *   - Every call only ENQUEUES work on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and returns without synchronising.  Outputs are
 *     valid once the caller has synchronised the stream.  No call allocates or
 *     frees device memory; scratch space comes in through `workspace`.
 *   - Layers are 1-based in every argument and output, as in Algorithm 1.
 *   - Return value: EE_OK, or a negative error code.  Arguments are validated on
 *     the host before anything is launched; on error nothing has been enqueued.
 *     ee_last_error() returns a thread-local message for the last failing call.
 *     Data errors that only the device can see (a block id outside 0..num_blocks-1,
 *     a position outside the block table, a row_table entry outside 0..B-1, a token
 *     id outside 0..vocab-1) are the
 *     caller's contract: the result for such a sequence is unspecified.  The kernels
 *     keep such an access inside the caller's buffers all the same (the id is read as
 *     0, the cache write is dropped), so bad data cannot fault the device.
 *   - dtype EE_FP32: weights, activations and KV cache are float; matrices are plain
 *     row-major [out_features][in_features].
 *     dtype EE_BF16: weights, embedding, gains and KV cache are bfloat16; matrices
 *     are in the MFMA tile order written by ee_pack_weight.  The residual stream,
 *     q, softmax statistics, logits and confidences are float in both cases.
 */
#ifndef EE_DECODE_H
#define EE_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EE_OK 0
#define EE_ERR_INVALID_ARG (-1)  /* null pointer, non-positive size, bad enum          */
#define EE_ERR_SHAPE (-2)        /* sizes inconsistent with each other                 */
#define EE_ERR_UNSUPPORTED (-3)  /* a shape or mode this build has no kernel for       */
#define EE_ERR_WORKSPACE (-4)    /* workspace too small or misaligned                  */
#define EE_ERR_HIP (-5)          /* a HIP call failed (message in ee_last_error)       */

#define EE_FP32 0
#define EE_BF16 1

/* Row orders understood by ee_pack_weight. */
#define EE_PACK_PLAIN 0    /* w_o, w_down, w_lm                                           */
#define EE_PACK_QKV 1      /* w_qkv : rotary partners (j, j + head_dim/2) share a tile    */
#define EE_PACK_GATE_UP 2  /* w_gate_up : gate row f and up row f share a tile            */

#define EE_MAX_LAYERS 64

typedef struct ee_model_desc {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab; /* d_model == n_heads * head_dim */
  int32_t dtype;       /* EE_FP32 | EE_BF16                                                        */
  float rms_eps;       /* RMSNorm epsilon                                                          */
  float rope_theta;    /* rotary base; <= 0 disables the rotary embedding                         */
  int32_t exit_every;  /* exit head after layers i with i % exit_every == 0 and i < n_layers       */
  float logit_scale;   /* s: exit-head logits at layer i are multiplied by s * i                   */
  int32_t conf_mode;   /* confidence measure of the paper's Section 2.1.
                          0: largest softmax probability of the exit head;
                          1: top-1 minus top-2 probability (softmax response as the paper writes it);
                          2: hidden states similarity, cos(h_{i-1}, h_i) of the hidden states before and
                             after layer i (h_0 = the embedding), on the float residual stream;
                          3: dedicated classifier, 1 / (1 + exp(-(w_cls[i] . x_i + b_cls[i]))) with
                             x_i = h_i / sqrt(mean(h_i^2) + rms_eps), the hidden state at unit root mean square.
                          2 and 3 touch no LM head inside the layer loop (logit_scale is unused); the
                          tokens then come from one LM-head pass over the hidden state at output_layer */
} ee_model_desc;

/* Weights of one decoder layer (all dev).  Plain shapes: g_attn,g_ffn [d]; w_qkv [3d][d] (q rows, then
 * k rows, then v rows); w_o [d][d]; w_gate_up [2f][d] (gate rows, then up rows); w_down [d][f].
 * For EE_BF16 the matrices are the ee_pack_weight images of those plain matrices. */
typedef struct ee_layer_weights {
  const void *g_attn, *w_qkv, *w_o, *g_ffn, *w_gate_up, *w_down;
} ee_layer_weights;

typedef struct ee_model {
  ee_model_desc desc;
  const void* embed;              /* dev [vocab][d], plain row-major in the model dtype            */
  const void* g_final;            /* dev [d]; final RMSNorm gain, shared by every exit head        */
  const void* w_lm;               /* dev [vocab][d]; LM head (packed PLAIN for EE_BF16), shared by
                                     every exit head and by the final token selection              */
  const ee_layer_weights* layers; /* host array [n_layers]                                         */
  const float* w_cls;             /* dev [n_layers][d] float, row i-1 = classifier of layer i; may be
                                     NULL unless conf_mode == 3                                     */
  const float* b_cls;             /* dev [n_layers] float, its biases; may be NULL unless conf_mode == 3 */
} ee_model;

/* Paged KV cache (the block-virtualised cache the paper inherits, Section 2.2 / 3.2).
 * k_pool and v_pool: dev [n_layers][num_blocks][n_heads][block_size][head_dim] in the model dtype.
 * block_size must be 16.  Position p of sequence b lives in block block_tables[b][p / 16] at offset p % 16.
 * Slots that hold no position of a sequence (the rest of its last block, blocks nobody owns) may contain
 * anything, NaN included: the attention kernels never let them reach a result. */
typedef struct ee_kv_cache {
  void* k_pool;
  void* v_pool;
  int32_t num_blocks, block_size;
} ee_kv_cache;

/* One batch of sequences, one token each.  The block allocator is the caller's: the library only
 * dereferences block_tables, and writes position context_lens[b] of sequence b (whose block must exist). */
typedef struct ee_batch {
  int32_t batch;               /* B >= 0; B == 0 is a no-op that still returns EE_OK                     */
  const int32_t* tokens;       /* dev [B]: token each sequence consumes this iteration                   */
  const int32_t* context_lens; /* dev [B]: p_b = positions already cached; the new K/V go to position p_b */
  const int32_t* block_tables; /* dev [B][max_blocks]: physical block of each logical block (with row_table:
                                  one row per sequence, at least max(row_table) + 1 rows)                */
  int32_t max_blocks;          /* row pitch of block_tables                                              */
  int32_t max_context;         /* host-side upper bound of context_lens[b] + 1 (sizes the attention grid) */
  const int32_t* row_table;    /* dev [B] or NULL.  NULL: row b of the batch uses row b of block_tables.  Else
                                  row b uses row row_table[b]: several rows may then share one sequence's block
                                  table at consecutive positions p, p+1, .. (a chunk of a prompt pushed through
                                  in one call: every row caches its K/V before any row attends, and row b
                                  attends positions 0..context_lens[b], so the chunk is causal).  Only with
                                  EE_EXIT_NONE, and with ee_paged_attention_decode.                          */
} ee_batch;

const char* ee_last_error(void);

/* Number of bytes ee_pack_weight writes for an [n_out][n_in] matrix (EE_BF16 only). */
size_t ee_packed_weight_bytes(int32_t n_out, int32_t n_in);

/* Reorders a plain bf16 matrix w [n_out][n_in] (dev) into the tile order the MFMA kernels stream:
 * tiles of 32 output rows x 16 input columns, stored [row_tile][col_tile][lane 0..63][8 values], so that a
 * wavefront fetches one operand tile as 1 KiB of consecutive bytes.  `order` (EE_PACK_*) says which output
 * rows share a tile; pair_stride is head_dim/2 for EE_PACK_QKV, d_ffn for EE_PACK_GATE_UP, ignored for PLAIN.
 * n_out must be a multiple of 32, n_in of 16, pair_stride of 16.  A set-up step, not part of the decode step. */
int ee_pack_weight(const void* w /*dev*/, int32_t n_out, int32_t n_in, int32_t order, int32_t pair_stride,
                   void* packed /*dev*/, void* stream);

/* Scratch bytes the calls below need for batches up to max_batch and contexts up to max_context.
 * The workspace must be 256-byte aligned.  Its contents need no initialisation and are dead between calls. */
size_t ee_workspace_bytes(const ee_model_desc* desc, int32_t max_batch, int32_t max_context);

/* One decode iteration: Algorithm 1 of the paper.
 *   embed the batch's tokens; for layer i = 1..n run the layer over the whole batch (caching this position's
 *   K/V of layer i), evaluate the exit head on every sequence whose status is still false, OR the result into
 *   the status (sticky), and stop at the first layer where every status is true (output_layer); fill K/V of
 *   this position for layers output_layer+1..n from the hidden state at output_layer (Section 3.2); pick the
 *   greedy token of every sequence from that hidden state.
 * The layer loop is enqueued once: a device-side flag makes the kernels of the layers after output_layer
 * return at once, so there is no host round trip inside the iteration.
 *   thresholds        host [n_layers]: lambda_i; accepted means confidence > lambda_i (strict).
 *   forced_exit_layer dev [B] or NULL: synthetic confidence injection; the decision of sequence b at layer i
 *                     becomes (i >= forced_exit_layer[b]) while the exit-head arithmetic still runs.
 *   use_exit_heads    EE_EXIT_NONE (0): full-layer baseline, no exit check is made, output_layer = n.
 *                     EE_EXIT_BATCH (1): Algorithm 1 as above.
 *                     EE_EXIT_PER_SEQUENCE (2): an extension of Algorithm 1 in which each sequence leaves on its
 *                     own: once its status is true, later layers neither attend for it nor change its hidden
 *                     state; the loop still ends at the first layer after which every status is true
 *                     (output_layer = the largest exit layer); K/V of all layers above a sequence's OWN exit
 *                     layer are filled from its own exit hidden state (Section 3.2 applied per sequence), and
 *                     its token comes from that state.
 *   out_tokens        dev [B] int32: greedy token (lowest index on ties).
 *   out_exit_layer    dev [B] int32: first layer whose check accepted the sequence, n_layers if none.
 *   out_batch_exit_layer dev [1] int32: output_layer.
 *   out_conf          dev [n_layers][B] float or NULL: confidence evaluated at each layer; NaN where no check
 *                     was made (no head, sequence already accepted, layer not run).
 *   out_hidden        dev [B][d] float or NULL: hidden state at output_layer (what the tokens come from). */
#define EE_EXIT_NONE 0
#define EE_EXIT_BATCH 1
#define EE_EXIT_PER_SEQUENCE 2
int ee_decode_iteration(const ee_model* model, const ee_kv_cache* cache, const ee_batch* batch,
                        const float* thresholds, const int32_t* forced_exit_layer, int32_t use_exit_heads,
                        int32_t* out_tokens, int32_t* out_exit_layer, int32_t* out_batch_exit_layer,
                        float* out_conf, float* out_hidden, void* workspace, size_t workspace_bytes, void* stream);

/* The exit check of one layer (Section 3.1 status rule with the softmax-response confidence of Section 2.1;
 * conf_mode 0 or 1 only: EE_ERR_UNSUPPORTED for the measures without an exit head, which need the layer loop):
 * z = (logit_scale * layer) * (RMSNorm(hidden; g_final) . W_lm^T); confidence per conf_mode; a sequence whose
 * status is 0 and whose confidence exceeds `threshold` gets status 1 and exit_layer = layer; statuses never
 * revert.  n_exited counts the sequences with status 1; done_flag is set to 1 (and batch_exit_layer to `layer`)
 * when it reaches `batch`, and is left alone otherwise.
 *   hidden dev [B][d] float.  status, exit_layer dev [B] int32 in/out.  n_exited, done_flag, batch_exit_layer
 *   dev [1] int32 in/out.  argmax dev [B] int32 or NULL (arg max of the logits, every row).  conf dev [B] float
 *   or NULL (NaN for rows whose status was already 1).  forced_exit_layer as above. */
int ee_exit_check(const ee_model* model, int32_t layer, const float* hidden, int32_t batch, float threshold,
                  const int32_t* forced_exit_layer, int32_t* status, int32_t* exit_layer, int32_t* n_exited,
                  int32_t* done_flag, int32_t* batch_exit_layer, int32_t* argmax, float* conf, void* workspace,
                  size_t workspace_bytes, void* stream);

/* The same exit check for callers that cannot allocate device memory or hand over a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, semantics and
 * results as ee_exit_check without the workspace: the scratch memory is a static device array of
 * EE_NOALLOC_SCRATCH_BYTES inside the library (each GPU the library runs on holds its own copy until the process
 * ends).  The call allocates and frees nothing.  A shape and batch that need more scratch than the array holds
 * (ee_exit_check_noalloc_bytes says how much: roughly batch * (vocab / 2 + 2 * d_model) bytes for EE_BF16, batch *
 * 4 * (vocab + d_model) for EE_FP32) are refused with EE_ERR_WORKSPACE before anything is enqueued.
 * Every call on one GPU uses that GPU's one array: calls that overlap on a GPU (two streams, two threads) race;
 * calls on one stream are ordered and each clears what it needs to start at zero.
 * ee_noalloc_init resolves the array's device address for the current device (one host-side query, no
 * allocation) and sets the function attributes of the projection kernels; both are otherwise done by the first
 * call that needs them, so call it beforehand if that first call would fall inside a graph capture. */
#define EE_NOALLOC_SCRATCH_BYTES (8u << 20)
int ee_noalloc_init(void);
size_t ee_exit_check_noalloc_bytes(const ee_model_desc* desc, int32_t batch);
int ee_exit_check_noalloc(const ee_model* model, int32_t layer, const float* hidden, int32_t batch, float threshold,
                          const int32_t* forced_exit_layer, int32_t* status, int32_t* exit_layer, int32_t* n_exited,
                          int32_t* done_flag, int32_t* batch_exit_layer, int32_t* argmax, float* conf, void* stream);

/* KV-cache filling (Algorithm 1's second loop, Section 3.2): for every sequence b and every layer
 * i > fill_from_layer[b], K = RoPE(RMSNorm(hidden_b; g_attn_i) . Wk_i^T, p_b), V = RMSNorm(..) . Wv_i^T, written to
 * position p_b = context_lens[b] of layer i.  The paper's rule passes the same output_layer for every b.
 *   hidden dev [B][d] float; fill_from_layer dev [B] int32.  batch->tokens is not read. */
int ee_kv_fill(const ee_model* model, const ee_kv_cache* cache, const ee_batch* batch, const float* hidden,
               const int32_t* fill_from_layer, void* workspace, size_t workspace_bytes, void* stream);

/* Single-query attention over the paged cache of one layer (the attention inside Algorithm 1's M(i, ...)):
 * out[b][h] = softmax_j(q[b][h] . K[b][j][h] / sqrt(head_dim)) . V[b][j][h], j = 0..context_lens[b] INCLUSIVE: the new
 * token's K/V must already be in the cache.   q dev [B][H][dh] float, rotary embedding applied.
 * out dev [B][H][dh] float.  batch->tokens is not read.
 * workspace (dev, 16-byte aligned) may be NULL.  With B * H <= 64 and a block table at least 16 blocks wide, a
 * workspace of at least B * H * 8 * (head_dim + 2) * 4 bytes lets up to eight workgroups share one (sequence, head)
 * pair, each over a contiguous part of the context, merged in a fixed order by a second launch (single-stream decoding
 * over a long context would otherwise keep only B * H compute units busy); a smaller or missing one is not an error,
 * the call then runs one workgroup per pair.  ee_decode_iteration does the same out of its own workspace. */
int ee_paged_attention_decode(const ee_model_desc* desc, const ee_kv_cache* cache, int32_t layer, const float* q,
                              const ee_batch* batch, float* out, void* workspace, size_t workspace_bytes,
                              void* stream);

/* ---- Measurement helpers (not part of the decode path) ------------------------------------------------------
 * While enabled, every later ee_* call brackets each kernel it enqueues with a pair of HIP events on the call's
 * stream (the events add a few microseconds per kernel, so throughput is timed with profiling off).
 * ee_profile_read waits for the recorded events and returns, for up to max_records kernels in launch order,
 * the kernel class (EE_K_*), the 1-based layer it belongs to (0 = none) and its duration in milliseconds;
 * the records are then discarded.  Returns the number of records written, or a negative error code. */
#define EE_K_NORM 0     /* sum of squares + normalised projection input                         */
#define EE_K_QKV 1      /* QKV projection + rotary + cache write                                */
#define EE_K_ATTN 2     /* paged decode attention                                               */
#define EE_K_OPROJ 3    /* output projection + residual                                         */
#define EE_K_GATEUP 4   /* gate/up projection + SwiGLU                                          */
#define EE_K_DOWN 5     /* down projection + residual                                           */
#define EE_K_HEAD 6     /* exit head / LM head projection with softmax statistics               */
#define EE_K_COMBINE 7  /* exit decision                                                        */
#define EE_K_KVFILL 8   /* KV filling projection                                                */
#define EE_K_OTHER 9    /* state reset, embedding, copies                                       */
#define EE_K_CLASSES 10
/* Plain device copy of n_floats floats (dev to dev) with the library's own copy kernel: a kernel of known traffic
 * (4 * n_floats bytes read, as many written) against which hardware byte counters are calibrated. */
int ee_calibration_copy(const float* src, float* dst, size_t n_floats, void* stream);
/* Attainable-rate probes of the chip the benchmark runs on (what the fractions of the published peaks are set beside).
 * ee_calibration_read: a plain streaming read of `bytes` bytes (dev, 16-byte aligned) by `workgroups` workgroups of four
 *   wavefronts, each wavefront walking one contiguous piece with 16 KiB in flight; `sink` (dev, 16 bytes) is written only
 *   if the exclusive-or of a wavefront's words equals one fixed pattern.  Traffic: `bytes` read, nothing written.
 * ee_calibration_mfma: `workgroups` x 4 wavefronts each issue 4 * iterations 32x32x16 bf16 matrix instructions on
 *   registers (2 * 32 * 32 * 16 flop each), no memory traffic; `sink` (dev, 1 KiB) is never written.
 * ee_calibration_mfma_tile: the inner loop of a 128 x 128 wavefront tile alone: `workgroups` x 4 wavefronts (96 KiB of LDS
 *   each: one workgroup per compute unit) run `steps` (even, >= 2) contraction steps of 16 such instructions on 4 x 4
 *   accumulators; with `lds_fragment_reads` = 8 every step also reads the next step's 4 + 4 operand fragments (1 KiB
 *   each) from LDS, with 0 it reads none.  No global memory traffic in the loop; `sink` (dev, 1 KiB) is never written.
 *   Errors: EE_ERR_INVALID_ARG for a NULL sink, an odd or too small step count, another number of reads.
 * ee_calibration_intake: what a compute unit takes in when half of its loads come from beyond its L2: `workgroups` x 4
 *   wavefronts each read a piece of `own` (dev, own_bytes, read once: from HBM) in 1 KiB loads, alternating with 1 KiB
 *   loads from `common` (dev, a power of two >= 64 KiB of bytes that every workgroup walks alike, so its lines are in
 *   L2 after the first reader), `loads_in_flight` (8, 16, 32 or 48) per wavefront.  pairs = 0: every workgroup has a
 *   piece of `own` to itself; each workgroup takes in own_bytes / workgroups from `own` and as much from `common`.
 *   pairs = 1 (workgroups a multiple of 16): workgroups whose ids differ by 8 (one XCD, one L2) read the same piece, so
 *   every byte of `own` leaves HBM once and L2 twice: each takes in 2 * own_bytes / workgroups from `own` and as much from
 *   `common`.  `sink` (dev, 16 bytes) is practically never written. */
int ee_calibration_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream);
int ee_calibration_mfma(int32_t workgroups, int32_t iterations, float* sink, void* stream);
int ee_calibration_mfma_tile(int32_t workgroups, int32_t steps, int32_t lds_fragment_reads, float* sink, void* stream);
int ee_calibration_intake(const void* own, size_t own_bytes, const void* common, size_t common_bytes, int32_t workgroups,
                          int32_t loads_in_flight, int32_t pairs, void* sink, void* stream);
int ee_profile_enable(int32_t on);
int ee_profile_read(int32_t* kernel_class /*host*/, int32_t* layer /*host*/, float* ms /*host*/, int32_t max_records);

#ifdef __cplusplus
}
#endif
#endif /* EE_DECODE_H */
