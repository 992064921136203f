// C ABI of the early-exit decode step: argument validation, workspace carving, kernel sequencing.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "ee_common.h"

// Scratch of ee_exit_check_noalloc (see noalloc_scratch below).
static __device__ __align__(256) unsigned char scratch[EE_NOALLOC_SCRATCH_BYTES];

namespace ee {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

namespace {

// ---- optional per-kernel timing with HIP events --------------------------------------------------------
struct ProfRecord {
  int cls, layer;
  hipEvent_t start, stop;
};
struct Profiler {
  bool on = false;
  std::vector<ProfRecord> used;
  std::vector<hipEvent_t> spare;
  hipEvent_t get() {
    if (!spare.empty()) {
      hipEvent_t e = spare.back();
      spare.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Profiler g_prof;
std::mutex g_prof_mutex;

// Brackets the launches made inside its scope with one event pair.
struct ProfScope {
  hipStream_t st;
  hipEvent_t stop = nullptr;
  ProfScope(int cls, int layer, hipStream_t s) : st(s) {
    if (!g_prof.on) return;
    std::lock_guard<std::mutex> lk(g_prof_mutex);
    hipEvent_t a = g_prof.get(), b = g_prof.get();
    if (!a || !b) return;
    g_prof.used.push_back({cls, layer, a, b});
    (void)hipEventRecord(a, st);
    stop = b;
  }
  ~ProfScope() {
    if (stop) (void)hipEventRecord(stop, st);
  }
};

struct Carver {
  char* base;
  size_t off;
  template <class T>
  T* take(size_t count) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct Workspace {
  // shared
  int32_t *status, *n_exited, *done, *scratch_exit_layer, *scratch_L;
  float* q;           // [B][d]
  float* attn_split;  // [B][H][8][head_dim + 2] partial attention results, only for batches of at most 64 (sequence, head) pairs
  float2* rope;       // [B][head_dim/2] (cos, sin) of this iteration's rotary angles
  float4* partials;   // bf16: [Mpad][vocab/32]; fp32: [B]
  float* h;           // residual stream: bf16 [Mpad][d], fp32 [B][d]
  // bf16 path
  float* y;           // [slices][Mpad][d] partial results of the output / down projection
  bf16_t* xH;         // [Mpad][d] exit-head operand, directly followed by
  bf16_t* xT;         // [Mpad][d] layer operand
  bf16_t* aoT;        // [Mpad][d]
  bf16_t* actT;       // [Mpad][f]
  float* rowsq;       // [2n + 2][Mpad]: sum of squares of the residual rows after the embedding / each update
  bf16_t* fill_x;     // [n][Mpad][d]
  float* dots;        // [n][Mpad] per-layer row dot products of the head-less confidence measures
  float* hprev;       // bf16: [Mpad][d], fp32: [B][d]: hidden state before the current layer (similarity measure)
  float* msr;         // fp32: [3][B] sums of the head-less confidence measures
  RowMap rowmap;      // bf16: [Mpad] + [Mpad] + [1] row map of the sequences still active (per-sequence exit)
  // fp32 path
  float *x, *ao, *act, *logits;
  size_t bytes;
};

// Contraction slices of the two accumulate projections of a layer (what the launches will write).
int acc_slices_max(const ee_model_desc& D, int B) {
  const int a = gemm_acc_slices(B, D.d_model / 32, D.d_model), b = gemm_acc_slices(B, D.d_model / 32, D.d_ffn);
  return a > b ? a : b;
}

Workspace carve(const ee_model_desc& D, int B, void* base) {
  Workspace w{};
  Carver c{reinterpret_cast<char*>(base), 0};
  const int Bp = B < 1 ? 1 : B;
  const int Mpad = round_up(Bp, 32);
  const size_t d = D.d_model, f = D.d_ffn, V = D.vocab, n = D.n_layers;
  w.status = c.take<int32_t>(Bp);
  w.n_exited = c.take<int32_t>(1);
  w.done = c.take<int32_t>(1);
  w.scratch_exit_layer = c.take<int32_t>(Bp);
  w.scratch_L = c.take<int32_t>(1);
  w.q = c.take<float>(Bp * d);
  {   // room for the largest batch that splits its attention, so that a workspace sized for B rows serves any fewer
    const long pairs = (long)Bp * D.n_heads < kAttnSplitMaxPairs ? (long)Bp * D.n_heads : kAttnSplitMaxPairs;
    w.attn_split = c.take<float>((size_t)pairs * kAttnMaxSplit * (D.head_dim + 2));
  }
  w.rope = c.take<float2>((size_t)Bp * (D.head_dim / 2));
  if (D.dtype == EE_BF16) {
    w.partials = c.take<float4>((size_t)Mpad * (V / 32));
    w.h = c.take<float>(d * Mpad);
    w.y = c.take<float>((size_t)acc_slices_max(D, Bp) * d * Mpad);
    w.xH = c.take<bf16_t>(2 * d * Mpad);
    w.xT = w.xH ? w.xH + d * Mpad : nullptr;
    w.aoT = c.take<bf16_t>(d * Mpad);
    w.actT = c.take<bf16_t>(f * Mpad);
    w.rowsq = c.take<float>((2 * n + 2) * Mpad);
    w.dots = c.take<float>(n * Mpad);
    w.fill_x = c.take<bf16_t>(n * Mpad * d);
    w.hprev = c.take<float>(d * Mpad);
    w.rowmap.perm = c.take<int32_t>(Mpad);
    w.rowmap.cpos = c.take<int32_t>(Mpad);
    w.rowmap.n_active = c.take<int32_t>(1);
  } else {
    w.partials = c.take<float4>(Bp);
    w.h = c.take<float>(Bp * d);
    w.x = c.take<float>(Bp * d);
    w.ao = c.take<float>(Bp * d);
    w.act = c.take<float>(Bp * f);
    w.logits = c.take<float>(Bp * V);
    w.hprev = c.take<float>(Bp * d);
    w.msr = c.take<float>(3 * Bp);
  }
  w.bytes = (c.off + 255) & ~(size_t)255;
  return w;
}

// The part of the workspace the stand-alone exit check touches, carved on its own: the allocation-free entry
// point fits it into the library's static scratch array instead of a caller's workspace.
Workspace carve_exit_check(const ee_model_desc& D, int B, void* base) {
  Workspace w{};
  Carver c{reinterpret_cast<char*>(base), 0};
  const int Bp = B < 1 ? 1 : B;
  const int Mpad = round_up(Bp, 32);
  const size_t d = D.d_model, V = D.vocab;
  w.status = c.take<int32_t>(Bp);
  w.n_exited = c.take<int32_t>(1);
  w.done = c.take<int32_t>(1);
  w.scratch_exit_layer = c.take<int32_t>(Bp);
  w.scratch_L = c.take<int32_t>(1);
  if (D.dtype == EE_BF16) {
    w.partials = c.take<float4>((size_t)Mpad * (V / 32));
    w.xH = c.take<bf16_t>(d * Mpad);
  } else {
    w.partials = c.take<float4>(Bp);
    w.x = c.take<float>(Bp * d);
    w.logits = c.take<float>(Bp * V);
  }
  w.bytes = (c.off + 255) & ~(size_t)255;
  return w;
}

int check_desc(const ee_model_desc* D) {
  if (!D) EE_FAIL(EE_ERR_INVALID_ARG, "model description is NULL");
  if (D->n_layers < 1 || D->d_model < 1 || D->n_heads < 1 || D->head_dim < 1 || D->d_ffn < 1 || D->vocab < 1)
    EE_FAIL(EE_ERR_INVALID_ARG, "model sizes must be positive");
  if (D->n_layers > EE_MAX_LAYERS) EE_FAIL(EE_ERR_UNSUPPORTED, "n_layers %d exceeds %d", D->n_layers, EE_MAX_LAYERS);
  if (D->dtype != EE_FP32 && D->dtype != EE_BF16) EE_FAIL(EE_ERR_INVALID_ARG, "dtype must be EE_FP32 or EE_BF16");
  if (D->d_model != D->n_heads * D->head_dim)
    EE_FAIL(EE_ERR_SHAPE, "d_model %d != n_heads %d * head_dim %d", D->d_model, D->n_heads, D->head_dim);
  if (D->head_dim != 64 && D->head_dim != 128) EE_FAIL(EE_ERR_UNSUPPORTED, "head_dim %d: only 64 and 128", D->head_dim);
  if (D->exit_every < 1) EE_FAIL(EE_ERR_INVALID_ARG, "exit_every must be >= 1");
  if (D->conf_mode < 0 || D->conf_mode > 3) EE_FAIL(EE_ERR_INVALID_ARG, "conf_mode must be 0, 1, 2 or 3");
  if (!(D->logit_scale >= 0.0f)) EE_FAIL(EE_ERR_INVALID_ARG, "logit_scale must be >= 0");
  if (!(D->rms_eps >= 0.0f)) EE_FAIL(EE_ERR_INVALID_ARG, "rms_eps must be >= 0");
  if (D->vocab % 2) EE_FAIL(EE_ERR_UNSUPPORTED, "vocab must be even");
  if (D->dtype == EE_BF16) {
    if (D->d_model % 64 || D->d_ffn % 16 || D->vocab % 32)
      EE_FAIL(EE_ERR_UNSUPPORTED, "bf16 path needs d_model %% 64 == 0, d_ffn %% 16 == 0, vocab %% 32 == 0");
    if (D->d_model > 8192) EE_FAIL(EE_ERR_UNSUPPORTED, "bf16 path: d_model %d exceeds 8192", D->d_model);
  }
  return EE_OK;
}

int check_model(const ee_model* M) {
  if (!M) EE_FAIL(EE_ERR_INVALID_ARG, "model is NULL");
  int rc = check_desc(&M->desc);
  if (rc) return rc;
  if (!M->embed || !M->g_final || !M->w_lm || !M->layers) EE_FAIL(EE_ERR_INVALID_ARG, "model has a NULL weight pointer");
  for (int i = 0; i < M->desc.n_layers; ++i) {
    const ee_layer_weights& L = M->layers[i];
    if (!L.g_attn || !L.w_qkv || !L.w_o || !L.g_ffn || !L.w_gate_up || !L.w_down)
      EE_FAIL(EE_ERR_INVALID_ARG, "layer %d has a NULL weight pointer", i + 1);
  }
  return EE_OK;
}

int check_cache(const ee_kv_cache* C) {
  if (!C || !C->k_pool || !C->v_pool) EE_FAIL(EE_ERR_INVALID_ARG, "KV cache or one of its pools is NULL");
  if (C->block_size != 16) EE_FAIL(EE_ERR_UNSUPPORTED, "block_size %d: only 16", C->block_size);
  if (C->num_blocks < 1) EE_FAIL(EE_ERR_INVALID_ARG, "num_blocks must be positive");
  return EE_OK;
}

int check_batch(const ee_batch* Bt, bool need_tokens, bool attends = true) {
  if (!Bt) EE_FAIL(EE_ERR_INVALID_ARG, "batch is NULL");
  if (Bt->batch < 0) EE_FAIL(EE_ERR_INVALID_ARG, "batch size %d is negative", Bt->batch);
  if (Bt->batch == 0) return EE_OK;
  if ((need_tokens && !Bt->tokens) || !Bt->context_lens || !Bt->block_tables)
    EE_FAIL(EE_ERR_INVALID_ARG, "batch has a NULL pointer");
  if (Bt->max_blocks < 1) EE_FAIL(EE_ERR_INVALID_ARG, "max_blocks must be positive");
  if (attends && Bt->max_blocks > kAttnMaxBlocks)
    EE_FAIL(EE_ERR_UNSUPPORTED, "attention: max_blocks %d outside 1..%d", Bt->max_blocks, kAttnMaxBlocks);
  if (Bt->max_context < 1 || Bt->max_context > Bt->max_blocks * 16)
    EE_FAIL(EE_ERR_SHAPE, "max_context %d does not fit max_blocks %d * 16", Bt->max_context, Bt->max_blocks);
  return EE_OK;
}

int check_workspace(const ee_model_desc& D, int B, void* ws, size_t ws_bytes) {
  if (!ws) EE_FAIL(EE_ERR_WORKSPACE, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(ws) & 255) EE_FAIL(EE_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  const size_t need = carve(D, B, nullptr).bytes;
  if (ws_bytes < need) EE_FAIL(EE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
  return EE_OK;
}

bool has_head(const ee_model_desc& D, int i) { return i < D.n_layers && i % D.exit_every == 0; }

// Row compaction needs every projection that takes a compacted operand to run in the tiled kernel, and pays
// from two 128-row chunks on (a chunk is what the kernel can skip).
bool bf16_compactable(const ee_model_desc& D, int B) {
  return D.dtype == EE_BF16 && B > 128 && gemm_bf16_is_tiled(B, D.d_model / 32) && gemm_bf16_is_tiled(B, 2 * D.d_ffn / 32) &&
         gemm_bf16_is_tiled(B, D.vocab / 32);
}

size_t pool_layer_elems(const ee_model_desc& D, const ee_kv_cache& C) {
  return (size_t)C.num_blocks * D.n_heads * 16 * D.head_dim;
}
size_t elem_bytes(const ee_model_desc& D) { return D.dtype == EE_BF16 ? 2 : 4; }

QkvEpi make_qkv_epi(const ee_model_desc& D, const ee_kv_cache& C, const ee_batch& Bt, const Workspace& w, int layer,
                    float* q) {
  QkvEpi e{};
  e.q = q;
  e.rope = w.rope;
  const size_t lb = pool_layer_elems(D, C) * elem_bytes(D) * (size_t)(layer - 1);
  e.k_pool = reinterpret_cast<char*>(C.k_pool) + lb;
  e.v_pool = reinterpret_cast<char*>(C.v_pool) + lb;
  e.context_lens = Bt.context_lens;
  e.block_tables = Bt.block_tables;
  e.row_table = Bt.row_table;
  e.fill_from = nullptr;
  e.fill_from_stride = 0;
  e.layer = layer;
  e.max_blocks = Bt.max_blocks;
  e.n_heads = D.n_heads;
  e.head_dim = D.head_dim;
  e.d_model = D.d_model;
  e.rope_theta = D.rope_theta;
  e.rowsq = nullptr;
  e.eps = D.rms_eps;
  e.num_blocks = C.num_blocks;
  e.table_rows = Bt.batch;
  return e;
}

// --- exit head: statistics of (scale * logits) for every row of the hidden state ------------------------
// The normalised operand is already in w.xH (written by the normalisation launch before).
void enqueue_head_bf16(const ee_model& M, const Workspace& w, int B, float scale, int layer, const RowMap& rm, Pred pred,
                       hipStream_t st) {
  const ee_model_desc& D = M.desc;
  GemmShape g{M.w_lm, w.xH, D.d_model, B, 0, D.vocab / 32, 16, 1};
  g.n_rows_dev = rm.n_active;   // compacted operand (prepared by the caller through the same map)
  LmEpi e{w.partials, nullptr, D.vocab / 32, D.vocab, scale, nullptr, D.rms_eps, D.d_model, rm.perm};
  ProfScope ps(EE_K_HEAD, layer, st);
  launch_gemm_lm_bf16(g, e, pred, st);
}
// RMSNorm of hidden rows h [B][d] (nothing added) with one gain into x.
NormArgs plain_norm(const ee_model_desc& D, const float* h, const void* gain, bf16_t* x, int B) {
  NormArgs a{};
  a.h_in = h;
  a.gain[0] = reinterpret_cast<const bf16_t*>(gain);
  a.x[0] = x;
  a.eps = D.rms_eps;
  a.B = B;
  a.Mpad = round_up(B, 32);
  a.d = D.d_model;
  return a;
}
void enqueue_head_f32(const ee_model& M, const Workspace& w, const float* h, int B, float scale, int layer, Pred pred,
                      hipStream_t st) {
  const ee_model_desc& D = M.desc;
  ProfScope ps(EE_K_HEAD, layer, st);
  launch_rmsnorm_f32(h, reinterpret_cast<const float*>(M.g_final), w.x, B, D.d_model, D.rms_eps, pred, st);
  SimpleShape g{reinterpret_cast<const float*>(M.w_lm), w.x, D.d_model, B, 0, D.vocab, 1};
  LmEpi e{w.partials, w.logits, 1, D.vocab, scale, nullptr, D.rms_eps, D.d_model};
  launch_simple_lm(g, e, pred, st);
  launch_head_stats_f32(w.logits, w.partials, B, D.vocab, scale, pred, st);
}

// --- KV filling for layers above fill_from ----------------------------------------------------------------
// h: hidden rows [B][d] (inside an iteration: the residual stream, final at the batch exit layer).
void enqueue_fill_bf16(const ee_model& M, const ee_kv_cache& C, const ee_batch& Bt, const Workspace& w, const float* h,
                       int Mpad, const int32_t* fill_from, int stride, Pred pred, hipStream_t st) {
  const ee_model_desc& D = M.desc;
  GainTable gt{};
  FillLayers fl{};
  for (int i = 0; i < D.n_layers; ++i) {
    gt.g[i] = M.layers[i].g_attn;
    fl.w_qkv[i] = M.layers[i].w_qkv;
  }
  ProfScope ps(EE_K_KVFILL, 0, st);
  launch_fill_prep(h, gt, D.n_layers, w.fill_x, D.rms_eps, fill_from, stride, Bt.batch, Mpad, D.d_model, pred, st);
  GemmShape g{nullptr, nullptr, D.d_model, Bt.batch, D.d_model / 32, 2 * D.d_model / 32, D.head_dim / 2, 1};
  QkvEpi e = make_qkv_epi(D, C, Bt, w, 1, nullptr);
  e.fill_from = fill_from;
  e.fill_from_stride = stride;
  launch_gemm_kvfill_bf16(fl, D.n_layers, w.fill_x, (size_t)Mpad * D.d_model, pool_layer_elems(D, C), g, e, pred, st);
}
void enqueue_fill_f32(const ee_model& M, const ee_kv_cache& C, const ee_batch& Bt, const Workspace& w, const float* h,
                      const int32_t* fill_from, int stride, Pred pred, hipStream_t st) {
  const ee_model_desc& D = M.desc;
  ProfScope ps(EE_K_KVFILL, 0, st);
  for (int i = 1; i <= D.n_layers; ++i) {
    const ee_layer_weights& L = M.layers[i - 1];
    launch_rmsnorm_f32(h, reinterpret_cast<const float*>(L.g_attn), w.x, Bt.batch, D.d_model, D.rms_eps, pred, st);
    SimpleShape g{reinterpret_cast<const float*>(L.w_qkv), w.x, D.d_model, Bt.batch, D.d_model, 2 * D.d_model,
                  D.head_dim / 2};
    QkvEpi e = make_qkv_epi(D, C, Bt, w, i, nullptr);
    e.fill_from = fill_from;
    e.fill_from_stride = stride;
    launch_simple_qkv(g, e, pred, st);
  }
}

// --- stand-alone exit check: validation and launch sequence shared by the two entry points -----------------
int check_exit_check_args(const ee_model* model, int32_t layer, const float* hidden, int32_t batch, const int32_t* status,
                          const int32_t* exit_layer, const int32_t* n_exited, const int32_t* done_flag,
                          const int32_t* batch_exit_layer) {
  int rc;
  if ((rc = check_model(model))) return rc;
  const ee_model_desc& D = model->desc;
  if (batch < 0) EE_FAIL(EE_ERR_INVALID_ARG, "batch size %d is negative", batch);
  if (batch == 0) return EE_OK;
  if (layer < 1 || layer > D.n_layers) EE_FAIL(EE_ERR_INVALID_ARG, "layer %d outside 1..%d", layer, D.n_layers);
  if (D.conf_mode >= 2)
    EE_FAIL(EE_ERR_UNSUPPORTED, "ee_exit_check: conf_mode %d has no exit head; it only runs inside ee_decode_iteration",
            D.conf_mode);
  if (!hidden || !status || !exit_layer || !n_exited || !done_flag || !batch_exit_layer)
    EE_FAIL(EE_ERR_INVALID_ARG, "ee_exit_check: NULL pointer");
  return EE_OK;
}

int enqueue_exit_check(const ee_model& M, int32_t layer, const float* hidden, int32_t batch, float threshold,
                       const int32_t* forced_exit_layer, int32_t* status, int32_t* exit_layer, int32_t* n_exited,
                       int32_t* done_flag, int32_t* batch_exit_layer, int32_t* argmax, float* conf, const Workspace& w,
                       hipStream_t st) {
  const ee_model_desc& D = M.desc;
  const Pred always{nullptr, 0};
  const float scale = D.logit_scale * (float)layer;
  if (D.dtype == EE_BF16) {
    launch_finish_norm(plain_norm(D, hidden, M.g_final, w.xH, batch), always, st);
    enqueue_head_bf16(M, w, batch, scale, layer, RowMap{}, always, st);
  } else {
    enqueue_head_f32(M, w, hidden, batch, scale, layer, always, st);
  }
  IterState s{status, exit_layer, n_exited, done_flag, batch_exit_layer};
  CombineArgs ca{w.partials, D.dtype == EE_BF16 ? D.vocab / 32 : 1, batch, layer, scale, threshold, D.conf_mode,
                 forced_exit_layer, s, argmax, conf};
  launch_combine(ca, always, st);
  EE_HIP(hipGetLastError());
  return EE_OK;
}

// --- scratch of the allocation-free entry point ---------------------------------------------------------------
// A file-scope device array: every GPU the library runs on holds its own copy at its own address until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address that kernels, fills
// and copies take is the one resolved below, once per device, with that device current.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int noalloc_scratch(void** out) {
  int dev = -1;
  EE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) EE_FAIL(EE_ERR_UNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    EE_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255)) EE_FAIL(EE_ERR_HIP, "static scratch array has no usable device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return EE_OK;
}

}  // namespace
}  // namespace ee

using namespace ee;

extern "C" {

const char* ee_last_error(void) { return g_error; }

int ee_calibration_copy(const float* src, float* dst, size_t n_floats, void* stream) {
  if (!src || !dst) EE_FAIL(EE_ERR_INVALID_ARG, "ee_calibration_copy: NULL pointer");
  launch_copy_f32(src, dst, n_floats, reinterpret_cast<hipStream_t>(stream));
  EE_HIP(hipGetLastError());
  return EE_OK;
}

int ee_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lk(g_prof_mutex);
  g_prof.on = on != 0;
  return EE_OK;
}

int ee_profile_read(int32_t* kernel_class, int32_t* layer, float* ms, int32_t max_records) {
  if (!kernel_class || !layer || !ms || max_records < 0) EE_FAIL(EE_ERR_INVALID_ARG, "ee_profile_read: bad argument");
  std::lock_guard<std::mutex> lk(g_prof_mutex);
  int n = 0;
  for (ProfRecord& r : g_prof.used) {
    EE_HIP(hipEventSynchronize(r.stop));
    float t = 0.0f;
    EE_HIP(hipEventElapsedTime(&t, r.start, r.stop));
    if (n < max_records) {
      kernel_class[n] = r.cls;
      layer[n] = r.layer;
      ms[n] = t;
      ++n;
    }
    g_prof.spare.push_back(r.start);
    g_prof.spare.push_back(r.stop);
  }
  g_prof.used.clear();
  return n;
}

size_t ee_packed_weight_bytes(int32_t n_out, int32_t n_in) {
  if (n_out <= 0 || n_in <= 0) return 0;
  return (size_t)n_out * (size_t)n_in * sizeof(bf16_t);
}

int ee_pack_weight(const void* w, int32_t n_out, int32_t n_in, int32_t order, int32_t pair_stride, void* packed,
                   void* stream) {
  if (!w || !packed) EE_FAIL(EE_ERR_INVALID_ARG, "ee_pack_weight: NULL pointer");
  if (n_out <= 0 || n_in <= 0 || n_out % 32 || n_in % 16)
    EE_FAIL(EE_ERR_SHAPE, "ee_pack_weight: n_out %d must be a positive multiple of 32, n_in %d of 16", n_out, n_in);
  int s = 16;
  if (order == EE_PACK_QKV || order == EE_PACK_GATE_UP) {
    s = pair_stride;
    if (s < 16 || s % 16 || n_out % (2 * s))
      EE_FAIL(EE_ERR_SHAPE, "ee_pack_weight: pair_stride %d must be a multiple of 16 and 2*pair_stride divide n_out %d", s,
              n_out);
  } else if (order != EE_PACK_PLAIN) {
    EE_FAIL(EE_ERR_INVALID_ARG, "ee_pack_weight: unknown order %d", order);
  }
  launch_pack_weight(reinterpret_cast<const bf16_t*>(w), n_out, n_in, s, reinterpret_cast<bf16_t*>(packed),
                     reinterpret_cast<hipStream_t>(stream));
  EE_HIP(hipGetLastError());
  return EE_OK;
}

size_t ee_workspace_bytes(const ee_model_desc* desc, int32_t max_batch, int32_t max_context) {
  (void)max_context;
  if (check_desc(desc) != EE_OK || max_batch < 0) return 0;
  return carve(*desc, max_batch, nullptr).bytes;
}

int ee_decode_iteration(const ee_model* model, const ee_kv_cache* cache, const ee_batch* batch, const float* thresholds,
                        const int32_t* forced_exit_layer, int32_t use_exit_heads, int32_t* out_tokens,
                        int32_t* out_exit_layer, int32_t* out_batch_exit_layer, float* out_conf, float* out_hidden,
                        void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_model(model)) || (rc = check_cache(cache)) || (rc = check_batch(batch, true))) return rc;
  const ee_model_desc& D = model->desc;
  const int B = batch->batch;
  if (B == 0) return EE_OK;
  if (use_exit_heads && !thresholds) EE_FAIL(EE_ERR_INVALID_ARG, "thresholds is NULL");
  if (!out_tokens || !out_exit_layer || !out_batch_exit_layer) EE_FAIL(EE_ERR_INVALID_ARG, "an output pointer is NULL");
  if ((rc = check_workspace(D, B, workspace, workspace_bytes))) return rc;
  // Confidence measures that need no LM head (Section 2.1): 2 = similarity of consecutive hidden states,
  // 3 = dedicated classifier.  Both are one dot product per row, taken while the next operand is prepared.
  if (batch->row_table && use_exit_heads != EE_EXIT_NONE)
    EE_FAIL(EE_ERR_INVALID_ARG, "row_table (several rows per sequence) only goes with EE_EXIT_NONE");
  if (use_exit_heads < 0 || use_exit_heads > EE_EXIT_PER_SEQUENCE)
    EE_FAIL(EE_ERR_INVALID_ARG, "use_exit_heads must be EE_EXIT_NONE, EE_EXIT_BATCH or EE_EXIT_PER_SEQUENCE");
  const bool dotmode = use_exit_heads && D.conf_mode >= 2;
  const bool simmode = use_exit_heads && D.conf_mode == 2;
  if (use_exit_heads && D.conf_mode == 3 && (!model->w_cls || !model->b_cls))
    EE_FAIL(EE_ERR_INVALID_ARG, "conf_mode 3 needs the classifier weights w_cls and b_cls");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const Workspace w = carve(D, B, workspace);
  const int Mpad = round_up(B, 32);
  const int n = D.n_layers, d = D.d_model, f = D.d_ffn;
  const bool bf = D.dtype == EE_BF16;
  IterState s{w.status, out_exit_layer, w.n_exited, w.done, out_batch_exit_layer};
  // Per-sequence exit (an extension of Algorithm 1): a sequence whose status is set has left.  Layers still run
  // over the whole batch, but for such a sequence they attend nothing and leave its hidden state as it is, so at
  // the end every sequence's column of the residual stream is its own exit hidden state.  The QKV projection of a
  // later layer i still caches K/V for it: its operand row is RMSNorm(own exit hidden state; layer i's gain), so
  // what it caches IS the KV filling of layer i for that sequence (Section 3.2) and only the layers above the
  // batch exit layer are left to the filling launch, as in Algorithm 1.
  const int32_t* left = use_exit_heads == EE_EXIT_PER_SEQUENCE ? w.status : nullptr;
  // At batch sizes where the projections run in the tiled kernel (whose cost grows with the rows), the layers'
  // operands are compacted as well: attention writes the result of an active sequence to its position in the row
  // map, the output, FFN and exit-head projections run over the first n_active rows only and scatter into the
  // residual columns.  The QKV projection keeps all rows in place (it does the KV filling of those that left).
  const bool compact = left && bf16_compactable(D, B);
  const RowMap rmap = compact ? w.rowmap : RowMap{};
  const Pred run_layers{w.done, 0};  // kernels of the layer loop: only while the batch has not left
  const Pred run_fill{w.done, 1};    // KV filling: only after it has
  const Pred always{nullptr, 0};

  // Algorithm 1, initialisation.  rowsq slot 0: after the embedding; slot 2i-1: after layer i's attention
  // update; slot 2i: after layer i.
  auto rs = [&](int slot) { return w.rowsq + (size_t)slot * Mpad; };
  {
    ProfScope ps(EE_K_OTHER, 0, st);
    launch_iter_init(s, B, n, out_conf, st);
    launch_rope_table(batch->context_lens, w.rope, B, D.head_dim, D.rope_theta, st);
    if (bf) {
      launch_embed_bf16(reinterpret_cast<const bf16_t*>(model->embed), batch->tokens, w.h, B, Mpad, d, D.vocab, st);
      if (compact) launch_compact(w.status, B, rmap, always, st);   // nobody has left: identity
    } else {
      launch_embed_f32(reinterpret_cast<const float*>(model->embed), batch->tokens, w.h, B, d, D.vocab, st);
      if (simmode) launch_copy_f32(w.h, w.hprev, (size_t)B * d, st);   // h_0, the "previous" state of layer 1
    }
  }
  // bf16 path: the residual update of a projection and the RMSNorm that follows it are one launch (NormArgs):
  // it adds the projection's partial results (n_slices of them) to the residual rows, leaves the rows' sums of
  // squares in rowsq slot `slot` and writes the operand(s) of what comes next.
  auto norm_args = [&](int n_slices, int slot) {
    NormArgs a{};
    a.h_in = w.h;
    a.h_out = n_slices ? w.h : nullptr;
    a.y = w.y;
    a.S = n_slices;
    a.skip = compact ? nullptr : left;   // with a row map, a sequence that has left has no position in it
    a.rm = rmap;
    a.rowsq_out = rs(slot);
    a.eps = D.rms_eps;
    a.B = B;
    a.Mpad = Mpad;
    a.d = d;
    return a;
  };
  const int slices_o = bf ? gemm_acc_slices(B, d / 32, d) : 0, slices_down = bf ? gemm_acc_slices(B, d / 32, f) : 0;

  // The exit decision of layer i (softmax-response measures, bf16, batches the streaming projection kernel serves)
  // rides along with the QKV projection launch of layer i + 1: one launch less per checked layer.
  const bool carry_combine = bf && !dotmode && !compact && gemm_qkv_carries_combine(B);
  const bool carry_decide = bf && dotmode && !compact && gemm_qkv_carries_combine(B);
  CombineArgs pending{};
  DecideArgs pending_dot{};
  bool have_pending = false, have_pending_dot = false;
  // Algorithm 1, batch inference loop.  Everything is enqueued; the done flag turns later layers into no-ops.
  for (int i = 1; i <= n; ++i) {
    const ee_layer_weights& L = model->layers[i - 1];
    const size_t pool_off = pool_layer_elems(D, *cache) * elem_bytes(D) * (size_t)(i - 1);
    AttnArgs at{w.q, reinterpret_cast<char*>(cache->k_pool) + pool_off, reinterpret_cast<char*>(cache->v_pool) + pool_off,
                batch->context_lens, batch->block_tables, batch->max_blocks, B, D.n_heads, D.head_dim, nullptr, 0, left,
                batch->row_table, rmap.cpos, cache->num_blocks, nullptr, 1};
    if (!batch->row_table && (long)B * D.n_heads <= kAttnSplitMaxPairs) {   // few pairs, long contexts: several workgroups per pair
      at.split_parts = attn_split_parts(B, D.n_heads, batch->max_blocks);
      at.split_ws = at.split_parts > 1 ? w.attn_split : nullptr;
    }
    const bool head_here = use_exit_heads && has_head(D, i);
    if (bf) {
      if (i == 1) {   // operand of the first layer from the embedding (also h_0, the "previous" hidden state of layer 1)
        ProfScope ps(EE_K_NORM, i, st);
        NormArgs na = norm_args(0, 0);
        na.gain[0] = reinterpret_cast<const bf16_t*>(L.g_attn);
        na.x[0] = w.xT;
        if (simmode) na.rd = RowDot{nullptr, w.hprev, nullptr, 1};
        launch_finish_norm(na, run_layers, st);
      }
      {
        ProfScope ps(EE_K_QKV, i, st);
        GemmShape gq{L.w_qkv, w.xT, d, B, 0, 3 * d / 32, D.head_dim / 2, 1};
        // one batch tile: each V tile (the last third; no rotation) is computed as two 16-row halves
        if (Mpad == 32 && d / 16 >= 8) gq.split_tiles = d / 32;
        QkvEpi qe = make_qkv_epi(D, *cache, *batch, w, i, w.q);
        launch_gemm_qkv_bf16(gq, qe, run_layers, st, have_pending ? &pending : nullptr,
                             have_pending_dot ? &pending_dot : nullptr);
        have_pending = have_pending_dot = false;
      }
      {
        ProfScope ps(EE_K_ATTN, i, st);
        at.out = w.aoT;
        at.out_xt = 1;
        if ((rc = launch_attention(at, D.dtype, run_layers, st))) return rc;
      }
      {
        ProfScope ps(EE_K_OPROJ, i, st);
        GemmShape go{L.w_o, w.aoT, d, B, 0, d / 32, 16, 1};
        go.n_rows_dev = rmap.n_active;
        launch_gemm_acc_bf16(go, AccEpi{w.y, Mpad, d, nullptr}, run_layers, st);
      }
      {   // h += attention update; operand of the FFN (compacted with a row map)
        ProfScope ps(EE_K_NORM, i, st);
        NormArgs na = norm_args(slices_o, 2 * i - 1);
        na.gain[0] = reinterpret_cast<const bf16_t*>(L.g_ffn);
        na.x[0] = w.xT;
        na.compacted[0] = compact;
        launch_finish_norm(na, run_layers, st);
      }
      {
        ProfScope ps(EE_K_GATEUP, i, st);
        GemmShape gg{L.w_gate_up, w.xT, d, B, 0, 2 * f / 32, f, 1};
        gg.n_rows_dev = rmap.n_active;
        launch_gemm_gateup_bf16(gg, GateUpEpi{w.actT, f, nullptr, D.rms_eps, d}, run_layers, st);
      }
      {
        ProfScope ps(EE_K_DOWN, i, st);
        GemmShape gd{L.w_down, w.actT, f, B, 0, d / 32, 16, 1};
        gd.n_rows_dev = rmap.n_active;
        launch_gemm_acc_bf16(gd, AccEpi{w.y, Mpad, d, nullptr}, run_layers, st);
      }
      {
        // h += FFN update; then the operand of the next layer's attention, and of this layer's exit head (compacted
        // with a row map) in the same launch; after the last layer: the operand of the final LM-head pass.  The
        // head-less confidence measures take their dot product here as well (with h_{i-1} or the classifier's row).
        ProfScope ps(EE_K_NORM, i, st);
        NormArgs na = norm_args(slices_down, 2 * i);
        if (i < n) {
          na.gain[0] = reinterpret_cast<const bf16_t*>(model->layers[i].g_attn);
          na.x[0] = w.xT;
          if (head_here && !dotmode) {
            na.gain[1] = reinterpret_cast<const bf16_t*>(model->g_final);
            na.x[1] = w.xH;
            na.compacted[1] = compact;
          }
          if (simmode) {   // h_{i-1} . h_i where a check follows; the snapshot moves on after every layer
            float* dots = head_here ? w.dots + (size_t)(i - 1) * Mpad : nullptr;
            na.rd = RowDot{dots ? w.hprev : nullptr, w.hprev, dots, 1};
          } else if (head_here && dotmode) {
            na.rd = RowDot{model->w_cls + (size_t)(i - 1) * d, nullptr, w.dots + (size_t)(i - 1) * Mpad, 0};
          }
        } else {
          na.gain[0] = reinterpret_cast<const bf16_t*>(model->g_final);
          na.x[0] = w.xH;
        }
        launch_finish_norm(na, run_layers, st);
      }
    } else {
      {
        ProfScope ps(EE_K_QKV, i, st);
        launch_rmsnorm_f32(w.h, reinterpret_cast<const float*>(L.g_attn), w.x, B, d, D.rms_eps, run_layers, st);
        SimpleShape gq{reinterpret_cast<const float*>(L.w_qkv), w.x, d, B, 0, 3 * d, D.head_dim / 2};
        QkvEpi qe = make_qkv_epi(D, *cache, *batch, w, i, w.q);
        launch_simple_qkv(gq, qe, run_layers, st);
      }
      {
        ProfScope ps(EE_K_ATTN, i, st);
        at.out = w.ao;
        at.out_xt = 0;
        if ((rc = launch_attention(at, D.dtype, run_layers, st))) return rc;
      }
      {
        ProfScope ps(EE_K_OPROJ, i, st);
        SimpleShape go{reinterpret_cast<const float*>(L.w_o), w.ao, d, B, 0, d, 1};
        launch_simple_acc(go, AccEpi{w.h, 0, d, left}, run_layers, st);
      }
      {
        ProfScope ps(EE_K_GATEUP, i, st);
        launch_rmsnorm_f32(w.h, reinterpret_cast<const float*>(L.g_ffn), w.x, B, d, D.rms_eps, run_layers, st);
        SimpleShape gg{reinterpret_cast<const float*>(L.w_gate_up), w.x, d, B, 0, 2 * f, f};
        launch_simple_gateup(gg, GateUpEpi{w.act, f, nullptr, D.rms_eps, d}, run_layers, st);
      }
      {
        ProfScope ps(EE_K_DOWN, i, st);
        SimpleShape gd{reinterpret_cast<const float*>(L.w_down), w.act, f, B, 0, d, 1};
        launch_simple_acc(gd, AccEpi{w.h, 0, d, left}, run_layers, st);
      }
    }
    if (!bf && simmode && !head_here && i < n) launch_copy_f32(w.h, w.hprev, (size_t)B * d, st);
    if (head_here && dotmode) {
      DecideArgs da{};
      if (bf) {
        da.dots = w.dots + (size_t)(i - 1) * Mpad;
        da.sq_a = rs(2 * i - 2);
        da.sq_b = rs(2 * i);
      } else {
        ProfScope ps(EE_K_HEAD, i, st);
        float* other = simmode ? w.hprev : const_cast<float*>(model->w_cls) + (size_t)(i - 1) * d;
        launch_measure_f32(w.h, other, simmode ? 1 : 0, w.msr, B, d, run_layers, st);
        da.dots = w.msr;
        da.sq_a = w.msr + B;
        da.sq_b = w.msr + 2 * (size_t)B;
      }
      da.bias = D.conf_mode == 3 ? model->b_cls + (i - 1) : nullptr;
      da.d = d;
      da.eps = D.rms_eps;
      da.B = B;
      da.layer = i;
      da.threshold = thresholds[i - 1];
      da.conf_mode = D.conf_mode;
      da.forced_exit_layer = forced_exit_layer;
      da.s = s;
      da.conf_out = out_conf ? out_conf + (size_t)(i - 1) * B : nullptr;
      if (carry_decide) {   // decided inside the next layer's QKV projection launch
        pending_dot = da;
        have_pending_dot = true;
      } else {
        ProfScope ps(EE_K_COMBINE, i, st);
        launch_decide(da, run_layers, st);
      }
      if (compact) launch_compact(w.status, B, rmap, run_layers, st);
    } else if (head_here) {
      const float scale = D.logit_scale * (float)i;
      if (bf)
        enqueue_head_bf16(*model, w, B, scale, i, rmap, run_layers, st);
      else
        enqueue_head_f32(*model, w, w.h, B, scale, i, run_layers, st);
      CombineArgs ca{w.partials, bf ? D.vocab / 32 : 1, B, i, scale, thresholds[i - 1], D.conf_mode, forced_exit_layer, s,
                     out_tokens, out_conf ? out_conf + (size_t)(i - 1) * B : nullptr, left};
      if (carry_combine) {   // decided inside the next layer's QKV projection launch (i < n: there is one)
        pending = ca;
        have_pending = true;
      } else {
        ProfScope ps(EE_K_COMBINE, i, st);
        launch_combine(ca, run_layers, st);
      }
      if (compact) launch_compact(w.status, B, rmap, run_layers, st);
    }
  }

  // Algorithm 1, KV cache filling for layers output_layer+1..n (runs only if the batch left early).  With
  // per-sequence exit the layers between a sequence's own exit layer and output_layer were filled by those
  // layers' own QKV projections (see above); every column of the residual stream is that sequence's exit state.
  if (use_exit_heads) {
    if (bf)
      enqueue_fill_bf16(*model, *cache, *batch, w, w.h, Mpad, out_batch_exit_layer, 0, run_fill, st);
    else
      enqueue_fill_f32(*model, *cache, *batch, w, w.h, out_batch_exit_layer, 0, run_fill, st);
  }

  // With a head-less confidence measure no exit head has produced a token: the LM head then always runs, on the
  // hidden state at output_layer (still in place: later layers were skipped).  Otherwise it runs only when the loop
  // reached the last layer, whose normalisation launch has left the head's operand in place.
  {
    const Pred final_pred = dotmode ? always : run_layers;
    if (bf && dotmode) {
      {
        ProfScope ps(EE_K_NORM, n, st);
        launch_finish_norm(plain_norm(D, w.h, model->g_final, w.xH, B), always, st);
      }
      enqueue_head_bf16(*model, w, B, 0.0f, n, RowMap{}, always, st);
    } else if (bf) {
      enqueue_head_bf16(*model, w, B, 0.0f, n, RowMap{}, run_layers, st);
    } else {
      enqueue_head_f32(*model, w, w.h, B, 0.0f, n, final_pred, st);
    }
    CombineArgs ca{w.partials, bf ? D.vocab / 32 : 1, B, 0, 0.0f, 0.0f, 0, nullptr, s, out_tokens, nullptr};
    ProfScope ps(EE_K_COMBINE, n, st);
    launch_combine(ca, final_pred, st);
  }
  if (out_hidden) launch_copy_f32(w.h, out_hidden, (size_t)B * d, st);
  (void)always;
  EE_HIP(hipGetLastError());
  return EE_OK;
}

int ee_exit_check(const ee_model* model, int32_t layer, const float* hidden, int32_t batch, float threshold,
                  const int32_t* forced_exit_layer, int32_t* status, int32_t* exit_layer, int32_t* n_exited,
                  int32_t* done_flag, int32_t* batch_exit_layer, int32_t* argmax, float* conf, void* workspace,
                  size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_exit_check_args(model, layer, hidden, batch, status, exit_layer, n_exited, done_flag, batch_exit_layer)))
    return rc;
  if (batch == 0) return EE_OK;
  if ((rc = check_workspace(model->desc, batch, workspace, workspace_bytes))) return rc;
  return enqueue_exit_check(*model, layer, hidden, batch, threshold, forced_exit_layer, status, exit_layer, n_exited,
                            done_flag, batch_exit_layer, argmax, conf, carve(model->desc, batch, workspace),
                            reinterpret_cast<hipStream_t>(stream));
}

size_t ee_exit_check_noalloc_bytes(const ee_model_desc* desc, int32_t batch) {
  if (check_desc(desc) != EE_OK || batch < 0) return 0;
  return carve_exit_check(*desc, batch, nullptr).bytes;
}

int ee_noalloc_init(void) {
  void* p = nullptr;
  gemm_bf16_prepare();
  return noalloc_scratch(&p);
}

int ee_exit_check_noalloc(const ee_model* model, int32_t layer, const float* hidden, int32_t batch, float threshold,
                          const int32_t* forced_exit_layer, int32_t* status, int32_t* exit_layer, int32_t* n_exited,
                          int32_t* done_flag, int32_t* batch_exit_layer, int32_t* argmax, float* conf, void* stream) {
  int rc;
  if ((rc = check_exit_check_args(model, layer, hidden, batch, status, exit_layer, n_exited, done_flag, batch_exit_layer)))
    return rc;
  if (batch == 0) return EE_OK;
  const size_t need = carve_exit_check(model->desc, batch, nullptr).bytes;
  if (need > (size_t)EE_NOALLOC_SCRATCH_BYTES)
    EE_FAIL(EE_ERR_WORKSPACE, "ee_exit_check_noalloc: this shape and batch need %zu bytes of scratch, the static array holds %zu",
            need, (size_t)EE_NOALLOC_SCRATCH_BYTES);
  void* base = nullptr;
  if ((rc = noalloc_scratch(&base))) return rc;
  return enqueue_exit_check(*model, layer, hidden, batch, threshold, forced_exit_layer, status, exit_layer, n_exited,
                            done_flag, batch_exit_layer, argmax, conf, carve_exit_check(model->desc, batch, base),
                            reinterpret_cast<hipStream_t>(stream));
}

int ee_kv_fill(const ee_model* model, const ee_kv_cache* cache, const ee_batch* batch, const float* hidden,
               const int32_t* fill_from_layer, void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_model(model)) || (rc = check_cache(cache)) || (rc = check_batch(batch, false, false))) return rc;
  const ee_model_desc& D = model->desc;
  const int B = batch->batch;
  if (B == 0) return EE_OK;
  if (!hidden || !fill_from_layer) EE_FAIL(EE_ERR_INVALID_ARG, "ee_kv_fill: NULL pointer");
  if ((rc = check_workspace(D, B, workspace, workspace_bytes))) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const Workspace w = carve(D, B, workspace);
  const int Mpad = round_up(B, 32);
  const Pred always{nullptr, 0};
  launch_rope_table(batch->context_lens, w.rope, B, D.head_dim, D.rope_theta, st);
  if (D.dtype == EE_BF16)
    enqueue_fill_bf16(*model, *cache, *batch, w, hidden, Mpad, fill_from_layer, 1, always, st);
  else
    enqueue_fill_f32(*model, *cache, *batch, w, hidden, fill_from_layer, 1, always, st);
  EE_HIP(hipGetLastError());
  return EE_OK;
}

int ee_paged_attention_decode(const ee_model_desc* desc, const ee_kv_cache* cache, int32_t layer, const float* q,
                              const ee_batch* batch, float* out, void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_desc(desc)) || (rc = check_cache(cache)) || (rc = check_batch(batch, false))) return rc;
  if (batch->batch == 0) return EE_OK;
  if (layer < 1 || layer > desc->n_layers) EE_FAIL(EE_ERR_INVALID_ARG, "layer %d outside 1..%d", layer, desc->n_layers);
  if (!q || !out) EE_FAIL(EE_ERR_INVALID_ARG, "ee_paged_attention_decode: NULL pointer");
  const size_t off = pool_layer_elems(*desc, *cache) * elem_bytes(*desc) * (size_t)(layer - 1);
  AttnArgs at{q, reinterpret_cast<char*>(cache->k_pool) + off, reinterpret_cast<char*>(cache->v_pool) + off,
              batch->context_lens, batch->block_tables, batch->max_blocks, batch->batch, desc->n_heads, desc->head_dim,
              out, 0, nullptr, batch->row_table, nullptr, cache->num_blocks, nullptr, 1};
  if (workspace && !batch->row_table) {   // a workspace lets few (sequence, head) pairs share their contexts among workgroups
    const int parts = attn_split_parts(batch->batch, desc->n_heads, batch->max_blocks);
    if (parts > 1 && (reinterpret_cast<uintptr_t>(workspace) & 15) == 0 &&
        workspace_bytes >= attn_split_floats(batch->batch, desc->n_heads, desc->head_dim, parts) * sizeof(float)) {
      at.split_parts = parts;
      at.split_ws = reinterpret_cast<float*>(workspace);
    }
  }
  const Pred always{nullptr, 0};
  if ((rc = launch_attention(at, desc->dtype, always, reinterpret_cast<hipStream_t>(stream)))) return rc;
  EE_HIP(hipGetLastError());
  return EE_OK;
}

}  // extern "C"
