// Host runtime and C ABI of libaxonn_stage: the stage handle (flat parameter / gradient
// buffers, activation stash slots, backward workspace), the per-layer forward and backward
// launch sequences, the message-driven scheduler of Alg. 2 and the bucketed offloaded Adam
// pipeline of Sec. 5.2.  No kernels live here; see gemm.hip, attention.hip, elementwise.hip.
#include "../../include/axonn_stage.h"
#include "common.h"
#include "host_logic.h"

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <functional>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

using namespace axonn;

namespace {

thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return fail(e_ == hipErrorOutOfMemory ? AXONN_ENOMEM : AXONN_EHIP, "%s failed: %s", \
                  #expr, hipGetErrorString(e_));                                          \
  } while (0)

#define AX_TRY(expr)       \
  do {                     \
    int r_ = (expr);       \
    if (r_ != AXONN_OK) return r_; \
  } while (0)


// ---- optional per-launch timing: event pairs around every kernel launch, by category ----
enum ProfCat { PC_GEMM_FWD, PC_GEMM_DGRAD, PC_GEMM_WGRAD, PC_ATTN_FWD, PC_ATTN_BWD, PC_LN_FWD,
               PC_LN_BWD, PC_GRAD_CONVERT, PC_ADAM, PC_COPY_IN, PC_EMBED, PC_XENT, PC_COUNT };
const char* const kProfNames[PC_COUNT] = {
    "gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attention_fwd", "attention_bwd", "layernorm_fwd",
    "layernorm_bwd", "grad_convert", "adam", "copy_in", "embedding", "cross_entropy"};
struct ProfRec { int cat; hipEvent_t a, b; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_pool;

hipEvent_t prof_event() {
  if (!g_prof_pool.empty()) { hipEvent_t e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
struct ProfScope {
  hipStream_t s; hipEvent_t a = nullptr, b = nullptr; int cat;
  ProfScope(int cat_, hipStream_t s_) : s(s_), cat(cat_) {
    if (!g_prof_on) return;
    a = prof_event(); b = prof_event();
    if (a && b) (void)hipEventRecord(a, s);
  }
  ~ProfScope() {
    if (!a || !b) return;
    (void)hipEventRecord(b, s);
    g_prof_recs.push_back(ProfRec{cat, a, b});
  }
};

constexpr int kTensorsPerLayer = 12;
const char* const kTensorNames[kTensorsPerLayer] = {
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2"};
enum { P_LN1G, P_LN1B, P_WQKV, P_BQKV, P_WO, P_BO, P_LN2G, P_LN2B, P_WFC1, P_BFC1, P_WFC2, P_BFC2 };

struct TensorInfo {
  std::string name;
  uint64_t offset;
  int rank;
  int64_t dims[4];
  uint64_t numel;
};

struct LayerStash {
  // forward activations kept for the backward pass
  elem_t *x, *u, *qkv, *o, *y, *w, *pre, *g;   // pre: GeLU'(w W1 + b1), the derivative at the pre-activation
  elem_t* u_lo;   // only with qkv_input_split: the part of LayerNorm-1's output that bf16 rounding dropped
  float *stats1, *stats2, *lse;
  // output gradients of the four linear maps, written by the backward pass and kept until the
  // weight gradients of a group of microbatches are formed in one contraction
  elem_t *dz, *dpre, *dy_mid, *dqkv;
};

using host::SLOT_AWAIT_WGRAD;
using host::SLOT_FREE;
using host::SLOT_LIVE;

struct Slot {
  int state = SLOT_FREE;
  int mb_id = -1;          // valid while SLOT_LIVE (forward issued, backward not yet)
  char* base = nullptr;
  std::vector<LayerStash> layers;
  // fwd_done: forward finished; dgrad_done: backward's activation-gradient chain finished;
  // released: the weight-gradient contraction that read the slot finished (slot reusable)
  hipEvent_t fwd_done = nullptr, dgrad_done = nullptr, released = nullptr;
  bool released_recorded = false;
  const int32_t* tokens = nullptr;   // first stage: the microbatch's token ids, needed again by Backward
  elem_t* head_y = nullptr;          // last stage: the stage output the head consumes
};

struct PendingMsg {
  axonn_msg m;
};

// With activation checkpointing (Sec. 5.1) a slot keeps only the inputs of layers 0, ac, 2ac, ...; every
// other activation lives in a set like this one, shared by all microbatches: a forward pass runs its layers
// through a one-layer set, a backward pass regenerates a segment of ac layers into an ac-layer set.
struct ActSet {
  char* base = nullptr;
  std::vector<LayerStash> layers;
  elem_t* x2 = nullptr;             // forward sets: second buffer for the layer inputs that are not kept
  hipEvent_t chain_done = nullptr;  // the backward chain through the set has finished (stream of the chain)
  hipEvent_t released = nullptr;    // the last work that reads or writes the set has finished
  bool released_recorded = false;
};

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

}  // namespace

struct axonn_offload_adam {
  int device = 0;
  uint64_t n = 0, bucket = 0;
  elem_t* p16 = nullptr;
  const elem_t* g16 = nullptr;
  float *h_theta = nullptr, *h_m = nullptr, *h_v = nullptr;
  static constexpr int kSets = 3;  // one being filled, one being updated, one being drained
  float* d_buf[kSets][3] = {};
  hipStream_t s_h2d = nullptr, s_k = nullptr, s_d2h = nullptr;
  hipEvent_t ev_start = nullptr, ev_h2d[kSets] = {}, ev_k[kSets] = {}, ev_d2h[kSets] = {};
  bool d2h_recorded[kSets] = {};
  uint64_t device_bytes = 0;
};

// First-stage extras (Alg. 2, i = 0): token and position tables in one flat bf16 buffer [wte | wpe].
struct axonn_embed {
  int device = 0, vocab = 0, h = 0, s = 0, b = 0;
  uint64_t n_params = 0;
  elem_t *params = nullptr, *grads = nullptr;
  int bwd_count = 0;   // backward passes since zero_grad
};

// Last-stage extras (Alg. 2, i = G_inter - 1): final LayerNorm, LM head, loss.  Flat bf16 buffer
// [lnf_g | lnf_b | w_head[h, V]].
struct axonn_head {
  int device = 0, vocab = 0, h = 0, T = 0, M = 0;
  float eps = 1e-5f;
  float loss_scale = 1.0f;   // multiplies dloss/dlogits (Sec. 2, mixed precision), not the reported loss
  uint64_t n_params = 0;
  elem_t *params = nullptr, *grads = nullptr;
  char* ws_base = nullptr;
  uint64_t ws_bytes = 0;
  elem_t *a = nullptr, *logits = nullptr, *da = nullptr;
  float *stats = nullptr, *token_loss = nullptr, *red_ws = nullptr;
  int count = 0;       // microbatches since zero_grad
};

struct axonn_stage {
  axonn_stage_config cfg;
  int T = 0, h = 0, f = 0, d = 0;
  uint64_t n_params = 0;
  std::vector<TensorInfo> tensors;
  elem_t* params = nullptr;
  elem_t* grads = nullptr;
  float* grads32 = nullptr;
  uint64_t* nonfinite_ws = nullptr;   // counters of launch_count_nonfinite, allocated on first use
  std::vector<Slot> slots;
  uint64_t slot_bytes = 0;
  // backward workspace
  char* ws_base = nullptr;
  uint64_t ws_bytes = 0;
  elem_t *dw = nullptr, *dattn = nullptr, *du = nullptr;
  float *delta = nullptr, *red_ws = nullptr, *wgrad_red_ws = nullptr;
  // activation checkpointing: shared activation sets (empty when cfg.ckpt_stride == 0)
  std::vector<ActSet> fwd_sets, regen_sets;
  unsigned fwd_set_rr = 0, regen_rr = 0;
  uint64_t act_set_bytes = 0;
  // state
  int in_flight = 0;
  int bwd_count = 0;  // backwards since the last zero_grad
  hipEvent_t last_bwd = nullptr, last_wgrad = nullptr, fork_ev = nullptr;
  bool last_bwd_recorded = false, last_wgrad_recorded = false;
  int wgrad_flushes = 0;              // weight-gradient contractions since the last zero_grad
  // per layer, for the last microbatch of a batch: chain_layer[l] = its backward chain has passed layer l;
  // grads_final[l] = every gradient of layer l is final in the bf16 buffer (the overlapped optimizer step
  // starts on a layer's parameters from there)
  std::vector<hipEvent_t> chain_layer, grads_final;
  bool grads_final_recorded = false;
  hipStream_t wgrad_stream = nullptr; // message-driven mode: weight gradients overlap other work
  hipEvent_t wgrad_tail = nullptr;
  // message-driven mode
  std::deque<PendingMsg> inbox;
  std::vector<hipStream_t> streams;
  std::vector<hipEvent_t> stream_tail;
  int fwd_rr = 0;
  int fwd_issued = 0, bwd_issued = 0;  // within the current batch (run mode)
  double message_wait_s = 120.0;       // limit of each wait of the blocking receive loop
  std::vector<int32_t> dispatch_log;
  axonn_offload_adam* opt = nullptr;
  // the two ends of the pipeline, when this stage is the first and / or the last one (borrowed handles)
  axonn_embed* embed = nullptr;
  axonn_head* head = nullptr;
  elem_t *embed_dx = nullptr, *head_dx = nullptr, *head_y_base = nullptr;
};

namespace {

elem_t* param_ptr(axonn_stage* st, int layer, int which) {
  return st->params + st->tensors[layer * kTensorsPerLayer + which].offset;
}
void* grad_ptr(axonn_stage* st, int layer, int which) {
  const uint64_t off = st->tensors[layer * kTensorsPerLayer + which].offset;
  return st->cfg.grad_accum_fp32 ? (void*)(st->grads32 + off) : (void*)(st->grads + off);
}

int check_launch(hipError_t e, const char* what) {
  if (e != hipSuccess) return fail(AXONN_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return AXONN_OK;
}

// Set while axonn_stage_run enqueues work on several streams: the GEMMs then share the chip with the
// kernels of the other streams.
static thread_local int t_concurrent = 0;

int gemm(bool a_kc, bool b_kc, int epi, int M, int N, int K, const void* A, int64_t lda,
         const void* B, int64_t ldb, void* C, int64_t ldc, const void* bias, const void* res,
         int64_t ld_res, void* aux, int64_t ld_aux, int accumulate, hipStream_t s) {
  GemmArgs g;
  memset(&g, 0, sizeof g);
  g.A_seg[0] = (const elem_t*)A; g.B_seg[0] = (const elem_t*)B; g.C = C; g.n_seg = 1;
  g.bias = (const elem_t*)bias; g.res = (const elem_t*)res; g.aux = (elem_t*)aux;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.ld_res = ld_res; g.ld_aux = ld_aux;
  g.M = M; g.N = N; g.K = K; g.accumulate = accumulate; g.tiles_m = g.tiles_n = 0;
  g.concurrent = t_concurrent;
  ProfScope ps(a_kc ? (b_kc ? PC_GEMM_DGRAD : PC_GEMM_FWD) : PC_GEMM_WGRAD, s);
  return check_launch(launch_gemm(a_kc, b_kc, epi, g, s), "gemm");
}


int ln_fwd(int64_t T, int64_t h, const void* x, const void* g, const void* b, float eps, void* out,
           void* out_lo, float* stats, hipStream_t s) {
  ProfScope ps(PC_LN_FWD, s);
  return check_launch(launch_layernorm_fwd(T, h, x, g, b, eps, out, out_lo, stats, s), "layernorm_fwd");
}
// The LayerNorm parameter gradients and the bias gradients (column sums) go straight into the
// gradient accumulators: stored if acc == 0, added otherwise.
int ln_bwd(axonn_stage* st, int layer, int which_g, int which_b, int64_t T, int64_t h, const void* dout,
           const void* x, const float* stats, const void* g, const void* res, void* dx, int acc, hipStream_t s) {
  ProfScope ps(PC_LN_BWD, s);
  return check_launch(launch_layernorm_bwd(T, h, dout, x, stats, g, res, dx, grad_ptr(st, layer, which_g),
                                           grad_ptr(st, layer, which_b), acc ? 2 : 1,
                                           st->cfg.grad_accum_fp32 != 0, st->red_ws, s), "layernorm_bwd");
}
int attn_fwd(int b, int sq, int a, int d, const void* qkv, void* o, float* lse, hipStream_t s) {
  ProfScope ps(PC_ATTN_FWD, s);
  return check_launch(launch_attention_fwd(b, sq, a, d, qkv, o, lse, s), "attention_fwd");
}
int attn_bwd(int b, int sq, int a, int d, const void* qkv, const void* o, const float* lse, const void* dout,
             void* dqkv, float* delta, hipStream_t s) {
  ProfScope ps(PC_ATTN_BWD, s);
  return check_launch(launch_attention_bwd(b, sq, a, d, qkv, o, lse, dout, dqkv, delta, s), "attention_bwd");
}
int adam(uint64_t n, float* th, float* m, float* v, const void* g16, void* p16, double lr, double b1, double b2,
         double eps, double wd, int64_t step, double gs, hipStream_t s) {
  ProfScope ps(PC_ADAM, s);
  return check_launch(launch_adam(n, th, m, v, g16, p16, lr, b1, b2, eps, wd, step, gs, s), "adam");
}

// ------------------------------------------------------------------- forward of a layer
// Runs layer l on a.x, filling the activations of `a`; z receives the layer's output (null: the last
// contraction is left out, for a regenerated layer whose output nobody reads).
int forward_layer(axonn_stage* st, int l, const LayerStash& a, elem_t* z, hipStream_t s) {
  const int T = st->T, h = st->h, f = st->f;
  AX_TRY(ln_fwd(T, h, a.x, param_ptr(st, l, P_LN1G), param_ptr(st, l, P_LN1B), st->cfg.ln_eps, a.u, a.u_lo,
                a.stats1, s));
  if (a.u_lo) {
    // [q|k|v] = (u_hi + u_lo) W + b as one contraction of length 2h: segment 0 pairs u_hi with W, segment 1 pairs
    // u_lo with the same W.  qkv_input_split == 2: for the q and k thirds only (the logits are what amplifies the
    // rounding of u); v = u_hi W_v + b_v as usual.
    const int n_split = st->cfg.qkv_input_split == 2 ? 2 * h : 3 * h;
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.A_seg[0] = a.u; g.A_seg[1] = a.u_lo;
    g.B_seg[0] = g.B_seg[1] = param_ptr(st, l, P_WQKV);
    g.n_seg = 2; g.C = a.qkv; g.bias = param_ptr(st, l, P_BQKV);
    g.lda = h; g.ldb = 3 * h; g.ldc = 3 * h; g.M = T; g.N = n_split; g.K = h;
    g.concurrent = t_concurrent;
    {
      ProfScope ps(PC_GEMM_FWD, s);
      AX_TRY(check_launch(launch_gemm(true, false, EPI_BIAS, g, s), "gemm (split input)"));
    }
    if (n_split < 3 * h)
      AX_TRY(gemm(true, false, EPI_BIAS, T, h, h, a.u, h, param_ptr(st, l, P_WQKV) + 2 * h, 3 * h, a.qkv + 2 * h, 3 * h,
                  param_ptr(st, l, P_BQKV) + 2 * h, nullptr, 0, nullptr, 0, 0, s));
  } else {
    AX_TRY(gemm(true, false, EPI_BIAS, T, 3 * h, h, a.u, h, param_ptr(st, l, P_WQKV), 3 * h, a.qkv, 3 * h,
                param_ptr(st, l, P_BQKV), nullptr, 0, nullptr, 0, 0, s));
  }
  AX_TRY(attn_fwd(st->cfg.microbatch_size, st->cfg.seq_len, st->cfg.n_heads, st->d, a.qkv, a.o, a.lse, s));
  AX_TRY(gemm(true, false, EPI_BIAS_RES, T, h, h, a.o, h, param_ptr(st, l, P_WO), h, a.y, h,
              param_ptr(st, l, P_BO), a.x, h, nullptr, 0, 0, s));
  AX_TRY(ln_fwd(T, h, a.y, param_ptr(st, l, P_LN2G), param_ptr(st, l, P_LN2B), st->cfg.ln_eps, a.w, nullptr,
                a.stats2, s));
  AX_TRY(gemm(true, false, EPI_BIAS_GELU, T, f, h, a.w, h, param_ptr(st, l, P_WFC1), f, a.g, f,
              param_ptr(st, l, P_BFC1), nullptr, 0, a.pre, f, 0, s));
  if (z)
    AX_TRY(gemm(true, false, EPI_BIAS_RES, T, h, f, a.g, f, param_ptr(st, l, P_WFC2), h, z, h,
                param_ptr(st, l, P_BFC2), a.y, h, nullptr, 0, 0, s));
  return AXONN_OK;
}

int forward_layers(axonn_stage* st, Slot& slot, void* y_out, hipStream_t s) {
  const int L = st->cfg.n_layers;
  for (int l = 0; l < L; ++l)
    AX_TRY(forward_layer(st, l, slot.layers[l], (l + 1 < L) ? slot.layers[l + 1].x : (elem_t*)y_out, s));
  return AXONN_OK;
}

// Forward pass that keeps only the inputs of layers 0, ac, 2ac, ... in the slot (Sec. 5.1); all other
// activations go through a shared one-layer set and are overwritten by the next layer.
int forward_layers_ckpt(axonn_stage* st, Slot& slot, void* y_out, hipStream_t s) {
  const int L = st->cfg.n_layers, ac = st->cfg.ckpt_stride;
  ActSet& F = st->fwd_sets[st->fwd_set_rr++ % st->fwd_sets.size()];
  if (F.released_recorded) HIP_TRY(hipStreamWaitEvent(s, F.released, 0));
  elem_t* const xb[2] = {F.layers[0].x, F.x2};
  for (int l = 0; l < L; ++l) {
    LayerStash a = F.layers[0];
    a.x = (l % ac == 0) ? slot.layers[l].x : xb[l & 1];
    elem_t* z = (l + 1 == L) ? (elem_t*)y_out : ((l + 1) % ac == 0) ? slot.layers[l + 1].x : xb[(l + 1) & 1];
    AX_TRY(forward_layer(st, l, a, z, s));
  }
  HIP_TRY(hipEventRecord(F.released, s));
  F.released_recorded = true;
  return AXONN_OK;
}

// ------------------------------------------------------------------ backward of a layer
// Given dL/d(output) in a.dz, writes dL/d(input) to d_out, the output gradients of the four linear maps
// to a.dpre, a.dy_mid, a.dqkv (a.dz is the fourth) and adds the LayerNorm gradients.  The bias gradients, column
// sums of those four, are left to the weight-gradient pass, which reads the same four matrices.
int backward_layer(axonn_stage* st, int l, const LayerStash& a, elem_t* d_out, int acc, hipStream_t s) {
  const int T = st->T, h = st->h, f = st->f;
  const elem_t* d_in = a.dz;
  // z = y + g W2 + b2
  AX_TRY(gemm(true, true, EPI_DGELU, T, f, h, d_in, h, param_ptr(st, l, P_WFC2), h, a.dpre, f,
              nullptr, nullptr, 0, a.pre, f, 0, s));
  // pre = w W1 + b1
  AX_TRY(gemm(true, true, EPI_BIAS, T, h, f, a.dpre, f, param_ptr(st, l, P_WFC1), f, st->dw, h,
              nullptr, nullptr, 0, nullptr, 0, 0, s));
  // w = LN2(y); residual: dy = d_in + dLN2
  AX_TRY(ln_bwd(st, l, P_LN2G, P_LN2B, T, h, st->dw, a.y, a.stats2, param_ptr(st, l, P_LN2G), d_in, a.dy_mid,
                acc, s));
  // y = x + o Wo + bo
  AX_TRY(gemm(true, true, EPI_BIAS, T, h, h, a.dy_mid, h, param_ptr(st, l, P_WO), h, st->dattn, h,
              nullptr, nullptr, 0, nullptr, 0, 0, s));
  // attention
  AX_TRY(attn_bwd(st->cfg.microbatch_size, st->cfg.seq_len, st->cfg.n_heads, st->d, a.qkv, a.o, a.lse, st->dattn,
                  a.dqkv, st->delta, s));
  // qkv = u Wqkv + b
  AX_TRY(gemm(true, true, EPI_BIAS, T, h, 3 * h, a.dqkv, 3 * h, param_ptr(st, l, P_WQKV), 3 * h, st->du, h,
              nullptr, nullptr, 0, nullptr, 0, 0, s));
  // u = LN1(x); residual: dx = dy + dLN1
  AX_TRY(ln_bwd(st, l, P_LN1G, P_LN1B, T, h, st->du, a.x, a.stats1, param_ptr(st, l, P_LN1G), a.dy_mid, d_out,
                acc, s));
  return AXONN_OK;
}

int backward_layers(axonn_stage* st, Slot& slot, const void* dy_in, void* dx_out, int acc, bool last,
                    hipStream_t s) {
  const int T = st->T, h = st->h, L = st->cfg.n_layers;
  // the upstream gradient is copied into the stash: it is an operand of the deferred weight
  // gradient and the caller may recycle its receive buffer
  {
    ProfScope ps(PC_COPY_IN, s);
    HIP_TRY(hipMemcpyAsync(slot.layers[L - 1].dz, dy_in, (uint64_t)T * h * sizeof(elem_t), hipMemcpyDeviceToDevice, s));
  }
  for (int l = L - 1; l >= 0; --l) {
    AX_TRY(backward_layer(st, l, slot.layers[l], (l == 0) ? (elem_t*)dx_out : slot.layers[l - 1].dz, acc, s));
    if (last) HIP_TRY(hipEventRecord(st->chain_layer[l], s));
  }
  return AXONN_OK;
}

// Weight gradients of every slot that has finished its backward chain, summed over those
// microbatches inside one contraction per weight (the token index of all of them is the
// contraction index): dW = sum_mb x_mb^T dy_mb.  Runs on `s` after the chains it reads and after
// the previous such pass (they update the same accumulators), then releases the slots.
int gemm_seg(int epi, int M, int N, int K, const elem_t* const* A, int64_t lda, const elem_t* const* B,
             int64_t ldb, int n_seg, void* C, int64_t ldc, void* colsum, float* colsum_ws, int accumulate,
             hipStream_t s) {
  GemmArgs g;
  memset(&g, 0, sizeof g);
  for (int i = 0; i < n_seg; ++i) { g.A_seg[i] = A[i]; g.B_seg[i] = B[i]; }
  g.n_seg = n_seg; g.C = C; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.M = M; g.N = N; g.K = K; g.accumulate = accumulate;
  g.colsum = colsum; g.colsum_ws = colsum_ws;
  g.concurrent = t_concurrent;
  ProfScope ps(PC_GEMM_WGRAD, s);
  return check_launch(launch_gemm(false, false, epi, g, s), "gemm (weight gradient)");
}

// dW += sum_i in_i^T dout_i for the four weights of layer l over n activation records, and with each the bias
// gradient db += sum_i (column sums of dout_i), formed by the same launch
int wgrad_layer(axonn_stage* st, int l, const LayerStash* const* rec, int n, int acc, hipStream_t s) {
  const int T = st->T, h = st->h, f = st->f;
  const int epi = st->cfg.grad_accum_fp32 ? EPI_ACC_F32 : EPI_ACC_BF16;
  float* const cws = st->wgrad_red_ws;
  const elem_t *A[kMaxKSegments], *B[kMaxKSegments];
  for (int i = 0; i < n; ++i) { A[i] = rec[i]->g; B[i] = rec[i]->dz; }
  AX_TRY(gemm_seg(epi, f, h, T, A, f, B, h, n, grad_ptr(st, l, P_WFC2), h, grad_ptr(st, l, P_BFC2), cws, acc, s));
  for (int i = 0; i < n; ++i) { A[i] = rec[i]->w; B[i] = rec[i]->dpre; }
  AX_TRY(gemm_seg(epi, h, f, T, A, h, B, f, n, grad_ptr(st, l, P_WFC1), f, grad_ptr(st, l, P_BFC1), cws, acc, s));
  for (int i = 0; i < n; ++i) { A[i] = rec[i]->o; B[i] = rec[i]->dy_mid; }
  AX_TRY(gemm_seg(epi, h, h, T, A, h, B, h, n, grad_ptr(st, l, P_WO), h, grad_ptr(st, l, P_BO), cws, acc, s));
  for (int i = 0; i < n; ++i) { A[i] = rec[i]->u; B[i] = rec[i]->dqkv; }
  AX_TRY(gemm_seg(epi, h, 3 * h, T, A, h, B, 3 * h, n, grad_ptr(st, l, P_WQKV), 3 * h, grad_ptr(st, l, P_BQKV), cws,
                  acc, s));
  return AXONN_OK;
}

// Rounds layer l's fp32 gradient accumulators into the bf16 gradient buffer (fp32 accumulation only) and
// marks the layer's gradients final on `s`.
int finish_layer_grads(axonn_stage* st, int l, hipStream_t s) {
  if (st->cfg.grad_accum_fp32) {
    const uint64_t lo = st->tensors[l * kTensorsPerLayer].offset;
    const uint64_t hi = (l + 1 < st->cfg.n_layers) ? st->tensors[(l + 1) * kTensorsPerLayer].offset : st->n_params;
    ProfScope ps(PC_GRAD_CONVERT, s);
    AX_TRY(check_launch(launch_f32_to_elem(hi - lo, st->grads32 + lo, st->grads + lo, s), "f32_to_bf16"));
  }
  HIP_TRY(hipEventRecord(st->grads_final[l], s));
  return AXONN_OK;
}

// Weight gradients of every slot that has finished its backward chain (see above).  `last_slot` is the
// slot of the batch's last microbatch when this is the batch's final pass (else null): the pass then
// follows that microbatch's chain layer by layer from the last layer down, and finishes each layer's
// gradients as soon as its contractions are queued.
int flush_wgrad(axonn_stage* st, hipStream_t s, Slot* last_slot = nullptr) {
  std::vector<Slot*> ready;
  for (Slot& sl : st->slots)
    if (sl.state == SLOT_AWAIT_WGRAD) ready.push_back(&sl);
  if (ready.empty()) return AXONN_OK;
  const int L = st->cfg.n_layers;
  for (Slot* sl : ready)
    if (sl != last_slot) HIP_TRY(hipStreamWaitEvent(s, sl->dgrad_done, 0));
  if (st->last_wgrad_recorded) HIP_TRY(hipStreamWaitEvent(s, st->last_wgrad, 0));
  for (int i = 0; i < L; ++i) {
    const int l = last_slot ? L - 1 - i : i;
    if (last_slot) HIP_TRY(hipStreamWaitEvent(s, st->chain_layer[l], 0));
    for (size_t first = 0; first < ready.size(); first += kMaxKSegments) {
      const int n = (int)std::min<size_t>(kMaxKSegments, ready.size() - first);
      const int acc = (st->wgrad_flushes > 0 || first > 0) ? 1 : 0;
      const LayerStash* rec[kMaxKSegments];
      for (int k = 0; k < n; ++k) rec[k] = &ready[first + k]->layers[l];
      AX_TRY(wgrad_layer(st, l, rec, n, acc, s));
    }
    if (last_slot) AX_TRY(finish_layer_grads(st, l, s));
  }
  st->wgrad_flushes++;
  if (last_slot) st->grads_final_recorded = true;
  HIP_TRY(hipEventRecord(st->last_wgrad, s));
  st->last_wgrad_recorded = true;
  for (Slot* sl : ready) {
    HIP_TRY(hipEventRecord(sl->released, s));
    sl->released_recorded = true;
  }
  host::release_awaiting(st->slots);
  return AXONN_OK;
}

// Backward pass from kept layer inputs (Sec. 5.1).  Segment by segment from the last: the segment's ac
// layers are run forward again from the kept input into a shared activation set (the output of the
// segment's last layer is not needed and not formed), the gradient chain runs back through them on `s`,
// and their weight gradients follow at once on `ws`, since the set is about to be reused.  Three sets
// rotate: while `ws` still reads one, the chain regenerates into the next and leaves the gradient that
// crosses the segment boundary in the one after.  `last`: this is the batch's last microbatch.
int backward_layers_ckpt(axonn_stage* st, Slot& slot, const void* dy_in, void* dx_out, int acc, bool last,
                         hipStream_t s, hipStream_t ws) {
  const int T = st->T, h = st->h, L = st->cfg.n_layers, ac = st->cfg.ckpt_stride;
  const size_t n_sets = st->regen_sets.size();
  for (int seg = L / ac - 1; seg >= 0; --seg) {
    ActSet& R = st->regen_sets[st->regen_rr % n_sets];
    ActSet& Rnext = st->regen_sets[(st->regen_rr + 1) % n_sets];
    st->regen_rr++;
    if (R.released_recorded) HIP_TRY(hipStreamWaitEvent(s, R.released, 0));
    if (seg > 0 && Rnext.released_recorded) HIP_TRY(hipStreamWaitEvent(s, Rnext.released, 0));
    if (seg == L / ac - 1) {
      // the upstream gradient is an operand of the weight gradient, which may outlive the caller's buffer
      ProfScope ps(PC_COPY_IN, s);
      HIP_TRY(hipMemcpyAsync(R.layers[ac - 1].dz, dy_in, (uint64_t)T * h * sizeof(elem_t), hipMemcpyDeviceToDevice, s));
    }
    std::vector<LayerStash> rec(R.layers.begin(), R.layers.begin() + ac);
    rec[0].x = slot.layers[seg * ac].x;
    for (int i = 0; i < ac; ++i)
      AX_TRY(forward_layer(st, seg * ac + i, rec[i], (i + 1 < ac) ? rec[i + 1].x : nullptr, s));
    for (int i = ac - 1; i >= 0; --i) {
      elem_t* d_out = (i > 0) ? rec[i - 1].dz : (seg == 0) ? (elem_t*)dx_out : Rnext.layers[ac - 1].dz;
      AX_TRY(backward_layer(st, seg * ac + i, rec[i], d_out, acc, s));
    }
    HIP_TRY(hipEventRecord(R.chain_done, s));
    if (ws != s) HIP_TRY(hipStreamWaitEvent(ws, R.chain_done, 0));
    if (st->last_wgrad_recorded) HIP_TRY(hipStreamWaitEvent(ws, st->last_wgrad, 0));
    for (int i = 0; i < ac; ++i) {
      const LayerStash* one[1] = {&rec[i]};
      AX_TRY(wgrad_layer(st, seg * ac + i, one, 1, acc, ws));
    }
    // last microbatch of the batch: the segment's gradients are final (the chain has passed its layers)
    if (last)
      for (int i = ac - 1; i >= 0; --i) AX_TRY(finish_layer_grads(st, seg * ac + i, ws));
    HIP_TRY(hipEventRecord(st->last_wgrad, ws));
    st->last_wgrad_recorded = true;
    HIP_TRY(hipEventRecord(R.released, ws));
    R.released_recorded = true;
  }
  return AXONN_OK;
}

int slots_in_state(const axonn_stage* st, int state) { return host::count_state(st->slots, state); }

Slot* find_live(axonn_stage* st, int mb_id) {
  const int i = host::find_live(st->slots, mb_id);
  return i >= 0 ? &st->slots[i] : nullptr;
}

// `ws` is the stream weight-gradient passes go to (the caller's stream in direct mode).
int embed_forward(axonn_embed* e, const int32_t* tokens, void* x, hipStream_t s);

// `x` holds [b,s,h] bf16 activations, or, on a stage with an embedding attached, [b,s] int32 token ids.
int do_forward(axonn_stage* st, int mb_id, const void* x, void* y, hipStream_t s, hipStream_t ws) {
  int si = -1;
  int adm = host::admit_forward(st->slots, mb_id, st->in_flight, st->cfg.pipeline_limit, &si);
  if (adm == host::FWD_NEEDS_FLUSH) {
    // every slot not in flight is waiting for its weight gradients: form them now
    AX_TRY(flush_wgrad(st, ws));
    adm = host::admit_forward(st->slots, mb_id, st->in_flight, st->cfg.pipeline_limit, &si);
  }
  switch (adm) {
    case host::FWD_OK: break;
    case host::FWD_NEGATIVE_ID: return fail(AXONN_EINVAL, "forward: negative microbatch id %d", mb_id);
    case host::FWD_ALREADY_LIVE: return fail(AXONN_ESTATE, "forward: microbatch %d is already in flight", mb_id);
    case host::FWD_PIPELINE_FULL:
      return fail(AXONN_ESTATE, "forward: pipeline_limit (%d) microbatches already in flight", st->cfg.pipeline_limit);
    default: return fail(AXONN_ESTATE, "forward: no free stash slot");
  }
  Slot* slot = &st->slots[si];
  // the weight-gradient pass that read the slot's previous contents must have finished
  if (slot->released_recorded) HIP_TRY(hipStreamWaitEvent(s, slot->released, 0));
  const uint64_t bytes = (uint64_t)st->T * st->h * sizeof(elem_t);
  if (st->head) y = slot->head_y;   // the last stage's output goes to its own head, not onwards
  if (st->embed) {
    slot->tokens = (const int32_t*)x;
    AX_TRY(embed_forward(st->embed, slot->tokens, slot->layers[0].x, s));
  } else {
    ProfScope ps(PC_COPY_IN, s);
    HIP_TRY(hipMemcpyAsync(slot->layers[0].x, x, bytes, hipMemcpyDeviceToDevice, s));
  }
  if (st->cfg.ckpt_stride > 0) AX_TRY(forward_layers_ckpt(st, *slot, y, s));
  else AX_TRY(forward_layers(st, *slot, y, s));
  HIP_TRY(hipEventRecord(slot->fwd_done, s));
  host::commit_forward(st->slots, si, mb_id, &st->in_flight);
  return AXONN_OK;
}

int do_backward(axonn_stage* st, int mb_id, const void* dy, void* dx, hipStream_t s, hipStream_t ws) {
  const int si = host::admit_backward(st->slots, mb_id);
  if (si < 0) return fail(AXONN_ESTATE, "backward: microbatch %d has no forward in flight", mb_id);
  Slot* slot = &st->slots[si];
  HIP_TRY(hipStreamWaitEvent(s, slot->fwd_done, 0));
  // backward chains share the workspace and the bias / LayerNorm accumulators: keep them in order
  if (st->last_bwd_recorded) HIP_TRY(hipStreamWaitEvent(s, st->last_bwd, 0));
  const int acc = st->bwd_count > 0 ? 1 : 0;
  const bool ckpt = st->cfg.ckpt_stride > 0;
  const bool last = st->bwd_count + 1 == st->cfg.n_microbatches;
  if (ckpt) AX_TRY(backward_layers_ckpt(st, *slot, dy, dx, acc, last, s, ws));
  else AX_TRY(backward_layers(st, *slot, dy, dx, acc, last, s));
  st->bwd_count++;
  HIP_TRY(hipEventRecord(slot->dgrad_done, s));
  HIP_TRY(hipEventRecord(st->last_bwd, s));
  st->last_bwd_recorded = true;
  host::commit_backward(st->slots, si, ckpt, &st->in_flight);
  if (ckpt) {
    // the weight gradients are already queued and read the shared sets: the slot (kept inputs only) is
    // free as soon as the chain on `s` is through
    HIP_TRY(hipEventRecord(slot->released, s));
    slot->released_recorded = true;
    if (last) st->grads_final_recorded = true;
  } else {
    switch (host::wgrad_action(last, st->cfg.wgrad_group, slots_in_state(st, SLOT_AWAIT_WGRAD))) {
      case host::WGRAD_FLUSH_FINAL: AX_TRY(flush_wgrad(st, ws, slot)); break;
      case host::WGRAD_FLUSH: AX_TRY(flush_wgrad(st, ws)); break;
      default: break;
    }
  }
  return AXONN_OK;
}

int embed_backward(axonn_embed* e, const int32_t* tokens, const void* dx, hipStream_t s);

// Backward(msg), followed on the first stage by the embedding's backward pass.
int backward_msg(axonn_stage* st, int mb_id, const void* dy, void* dx, hipStream_t s, hipStream_t ws) {
  if (!st->embed) return do_backward(st, mb_id, dy, dx, s, ws);
  Slot* slot = (mb_id >= 0) ? find_live(st, mb_id) : nullptr;
  const int32_t* tokens = slot ? slot->tokens : nullptr;
  AX_TRY(do_backward(st, mb_id, dy, st->embed_dx, s, ws));
  AX_TRY(embed_backward(st->embed, tokens, st->embed_dx, s));
  // the next backward chain overwrites embed_dx: it must follow the embedding's pass as well
  HIP_TRY(hipEventRecord(st->last_bwd, s));
  return AXONN_OK;
}

int head_forward_backward(axonn_head* hd, const void* x, const int32_t* targets, float* loss, void* dx,
                          hipStream_t s);

int ensure_streams(axonn_stage* st, int n) {
  while ((int)st->streams.size() < n) {
    hipStream_t s;
    hipEvent_t e;
    HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    st->streams.push_back(s);
    st->stream_tail.push_back(e);
  }
  return AXONN_OK;
}

void destroy_adam(axonn_offload_adam* o) {
  if (!o) return;
  (void)hipSetDevice(o->device);
  if (o->s_h2d) (void)hipStreamSynchronize(o->s_h2d);
  if (o->s_k) (void)hipStreamSynchronize(o->s_k);
  if (o->s_d2h) (void)hipStreamSynchronize(o->s_d2h);
  for (int i = 0; i < axonn_offload_adam::kSets; ++i) {
    for (int j = 0; j < 3; ++j)
      if (o->d_buf[i][j]) (void)hipFree(o->d_buf[i][j]);
    if (o->ev_h2d[i]) (void)hipEventDestroy(o->ev_h2d[i]);
    if (o->ev_k[i]) (void)hipEventDestroy(o->ev_k[i]);
    if (o->ev_d2h[i]) (void)hipEventDestroy(o->ev_d2h[i]);
  }
  if (o->ev_start) (void)hipEventDestroy(o->ev_start);
  if (o->s_h2d) (void)hipStreamDestroy(o->s_h2d);
  if (o->s_k) (void)hipStreamDestroy(o->s_k);
  if (o->s_d2h) (void)hipStreamDestroy(o->s_d2h);
  delete o;
}

void destroy_stage(axonn_stage* st) {
  if (!st) return;
  (void)hipSetDevice(st->cfg.device);
  (void)hipDeviceSynchronize();
  destroy_adam(st->opt);
  for (Slot& s : st->slots) {
    if (s.base) (void)hipFree(s.base);
    if (s.fwd_done) (void)hipEventDestroy(s.fwd_done);
    if (s.dgrad_done) (void)hipEventDestroy(s.dgrad_done);
    if (s.released) (void)hipEventDestroy(s.released);
  }
  for (hipStream_t s : st->streams) (void)hipStreamDestroy(s);
  for (hipEvent_t e : st->stream_tail) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->chain_layer) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->grads_final) if (e) (void)hipEventDestroy(e);
  if (st->last_bwd) (void)hipEventDestroy(st->last_bwd);
  if (st->fork_ev) (void)hipEventDestroy(st->fork_ev);
  if (st->last_wgrad) (void)hipEventDestroy(st->last_wgrad);
  if (st->wgrad_tail) (void)hipEventDestroy(st->wgrad_tail);
  if (st->wgrad_stream) (void)hipStreamDestroy(st->wgrad_stream);
  for (std::vector<ActSet>* sets : {&st->fwd_sets, &st->regen_sets})
    for (ActSet& a : *sets) {
      if (a.base) (void)hipFree(a.base);
      if (a.chain_done) (void)hipEventDestroy(a.chain_done);
      if (a.released) (void)hipEventDestroy(a.released);
    }
  if (st->embed_dx) (void)hipFree(st->embed_dx);
  if (st->head_dx) (void)hipFree(st->head_dx);
  if (st->head_y_base) (void)hipFree(st->head_y_base);
  if (st->ws_base) (void)hipFree(st->ws_base);
  if (st->params) (void)hipFree(st->params);
  if (st->grads) (void)hipFree(st->grads);
  if (st->grads32) (void)hipFree(st->grads32);
  if (st->nonfinite_ws) (void)hipFree(st->nonfinite_ws);
  delete st;
}

int validate_config(const axonn_stage_config* c) {
  if (c->n_layers < 1 || c->hidden < 1 || c->n_heads < 1 || c->ffn_hidden < 1 || c->seq_len < 1 ||
      c->microbatch_size < 1 || c->n_microbatches < 1)
    return fail(AXONN_EINVAL, "stage config: sizes must be positive");
  if (c->pipeline_limit < 1 || c->pipeline_limit > c->n_microbatches)
    return fail(AXONN_EINVAL, "stage config: pipeline_limit must be in 1..n_microbatches");
  if (c->hidden % c->n_heads != 0) return fail(AXONN_EINVAL, "stage config: hidden %% n_heads != 0");
  if (!(c->ln_eps > 0.f)) return fail(AXONN_EINVAL, "stage config: ln_eps must be positive");
  if (c->device < 0) return fail(AXONN_EINVAL, "stage config: negative device ordinal");
  if (c->wgrad_group < 0) return fail(AXONN_EINVAL, "stage config: negative wgrad_group");
  if (c->qkv_input_split < 0 || c->qkv_input_split > 2)
    return fail(AXONN_EINVAL, "config: qkv_input_split must be 0, 1 or 2 (got %d)", c->qkv_input_split);
  if (c->ckpt_stride < 0 || (c->ckpt_stride > 0 && c->n_layers % c->ckpt_stride != 0))
    return fail(AXONN_EINVAL, "stage config: ckpt_stride (%d) must be 0 or a factor of n_layers (%d)",
                c->ckpt_stride, c->n_layers);
  const int d = c->hidden / c->n_heads;
  if (d % 4 || d > 192)
    return fail(AXONN_EUNSUPPORTED, "head dim %d unsupported: it must be a multiple of 4, at most 192", d);
  if (c->hidden % 8 || c->ffn_hidden % 8)
    return fail(AXONN_EUNSUPPORTED, "hidden and ffn_hidden must be multiples of 8 (16-byte rows)");
  if (((int64_t)c->seq_len * c->microbatch_size) % 8)
    return fail(AXONN_EUNSUPPORTED, "microbatch_size*seq_len must be a multiple of 8");
  if (c->hidden > 16384) return fail(AXONN_EUNSUPPORTED, "hidden > 16384 unsupported by the LayerNorm kernel");
  if ((int64_t)c->seq_len * c->microbatch_size > (1 << 24))
    return fail(AXONN_EUNSUPPORTED, "more than 2^24 tokens per microbatch unsupported");
  return AXONN_OK;
}

// ------------------------------------------------------------------ the pipeline's two ends
int embed_forward(axonn_embed* e, const int32_t* tokens, void* x, hipStream_t s) {
  ProfScope ps(PC_EMBED, s);
  return check_launch(launch_embed_fwd(e->b * e->s, e->h, e->s, e->vocab, tokens, e->params,
                                       e->params + (uint64_t)e->vocab * e->h, x, s), "embed_fwd");
}

int embed_backward(axonn_embed* e, const int32_t* tokens, const void* dx, hipStream_t s) {
  elem_t* dwte = e->grads;
  elem_t* dwpe = e->grads + (uint64_t)e->vocab * e->h;
  const int acc = e->bwd_count > 0 ? 1 : 0;
  ProfScope ps(PC_EMBED, s);
  // the table kernel touches only the rows whose ids occur: the first pass of a batch clears the table
  if (!acc) AX_TRY(check_launch(launch_fill_elem((uint64_t)e->vocab * e->h, dwte, 0.0f, s), "fill"));
  AX_TRY(check_launch(launch_embed_bwd(e->b, e->s, e->h, e->vocab, tokens, dx, dwte, dwpe, acc, s), "embed_bwd"));
  e->bwd_count++;
  return AXONN_OK;
}

// Forward of the last-stage extras followed at once by Backward(1) (Alg. 2): a = LN(x), logits = a W,
// loss and dL/dlogits in place, dW += a^T dlogits, da = dlogits W^T, dx = LN'(da).
int head_forward_backward(axonn_head* hd, const void* x, const int32_t* targets, float* loss, void* dx,
                          hipStream_t s) {
  const int T = hd->T, h = hd->h, V = hd->vocab;
  elem_t* g = hd->params;
  elem_t* bt = hd->params + h;
  elem_t* W = hd->params + 2 * (uint64_t)h;
  const int acc = hd->count > 0 ? 1 : 0;
  AX_TRY(ln_fwd(T, h, x, g, bt, hd->eps, hd->a, nullptr, hd->stats, s));
  AX_TRY(gemm(true, false, EPI_BIAS, T, V, h, hd->a, h, W, V, hd->logits, V, nullptr, nullptr, 0, nullptr, 0, 0, s));
  {
    ProfScope ps(PC_XENT, s);
    AX_TRY(check_launch(launch_xent(T, V, hd->logits, targets, hd->M, hd->loss_scale, hd->token_loss, loss, s), "cross_entropy"));
  }
  {
    const elem_t* A[1] = {hd->a};
    const elem_t* B[1] = {hd->logits};
    AX_TRY(gemm_seg(EPI_ACC_BF16, h, V, T, A, h, B, V, 1, hd->grads + 2 * (uint64_t)h, V, nullptr, nullptr, acc, s));
  }
  AX_TRY(gemm(true, true, EPI_BIAS, T, h, V, hd->logits, V, W, V, hd->da, h, nullptr, nullptr, 0, nullptr, 0, 0, s));
  {
    ProfScope ps(PC_LN_BWD, s);
    AX_TRY(check_launch(launch_layernorm_bwd(T, h, hd->da, x, hd->stats, g, nullptr, dx, hd->grads, hd->grads + h,
                                             acc ? 2 : 1, false, hd->red_ws, s), "layernorm_bwd (head)"));
  }
  hd->count++;
  return AXONN_OK;
}

}  // namespace

// ======================================================================== C ABI
extern "C" {

const char* axonn_last_error(void) { return g_last_error.c_str(); }

int axonn_pinned_alloc(void** host_out, uint64_t bytes) {
  if (!host_out || bytes == 0) return fail(AXONN_EINVAL, "pinned_alloc: null output or zero size");
  HIP_TRY(hipHostMalloc(host_out, bytes, hipHostMallocDefault));
  return AXONN_OK;
}
int axonn_pinned_free(void* host) {
  if (!host) return fail(AXONN_EINVAL, "pinned_free: null pointer");
  HIP_TRY(hipHostFree(host));
  return AXONN_OK;
}

int axonn_stage_create(const axonn_stage_config* cfg, axonn_stage_t** out) {
  if (!cfg || !out) return fail(AXONN_EINVAL, "stage_create: null argument");
  *out = nullptr;
  AX_TRY(validate_config(cfg));
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (cfg->device >= ndev) return fail(AXONN_EINVAL, "stage_create: device %d of %d", cfg->device, ndev);
  HIP_TRY(hipSetDevice(cfg->device));
  axonn_stage* st = new (std::nothrow) axonn_stage();
  if (!st) return fail(AXONN_ENOMEM, "stage_create: host allocation failed");
  st->cfg = *cfg;
  st->h = cfg->hidden; st->f = cfg->ffn_hidden; st->d = cfg->hidden / cfg->n_heads;
  st->T = cfg->seq_len * cfg->microbatch_size;
  const int64_t h = st->h, f = st->f, T = st->T;
  // flat parameter table
  uint64_t off = 0;
  for (int l = 0; l < cfg->n_layers; ++l) {
    const int64_t shp[kTensorsPerLayer][2] = {{h, 0}, {h, 0}, {h, 3 * h}, {3 * h, 0}, {h, h}, {h, 0},
                                             {h, 0}, {h, 0}, {h, f}, {f, 0}, {f, h}, {h, 0}};
    for (int t = 0; t < kTensorsPerLayer; ++t) {
      TensorInfo ti;
      ti.name = "layer" + std::to_string(l) + "." + kTensorNames[t];
      ti.offset = off;
      ti.rank = shp[t][1] ? 2 : 1;
      ti.dims[0] = shp[t][0]; ti.dims[1] = shp[t][1] ? shp[t][1] : 1; ti.dims[2] = ti.dims[3] = 1;
      ti.numel = (uint64_t)shp[t][0] * (shp[t][1] ? shp[t][1] : 1);
      off += ti.numel;
      st->tensors.push_back(ti);
    }
  }
  st->n_params = off;

  auto bail = [&](int code) { destroy_stage(st); return code; };
#define CREATE_TRY(expr)                                                                         \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess)                                                                        \
      return bail(fail(e_ == hipErrorOutOfMemory ? AXONN_ENOMEM : AXONN_EHIP, "%s failed: %s",   \
                       #expr, hipGetErrorString(e_)));                                           \
  } while (0)

  CREATE_TRY(hipMalloc((void**)&st->params, st->n_params * sizeof(elem_t)));
  CREATE_TRY(hipMalloc((void**)&st->grads, st->n_params * sizeof(elem_t)));
  CREATE_TRY(hipMemset(st->params, 0, st->n_params * sizeof(elem_t)));
  CREATE_TRY(hipMemset(st->grads, 0, st->n_params * sizeof(elem_t)));
  if (cfg->grad_accum_fp32) {
    CREATE_TRY(hipMalloc((void**)&st->grads32, st->n_params * sizeof(float)));
    CREATE_TRY(hipMemset(st->grads32, 0, st->n_params * sizeof(float)));
  }
  for (int l = 0; l < cfg->n_layers; ++l) {
    CREATE_TRY(launch_fill_elem(h, param_ptr(st, l, P_LN1G), 1.0f, nullptr));
    CREATE_TRY(launch_fill_elem(h, param_ptr(st, l, P_LN2G), 1.0f, nullptr));
  }

  // activation stash: per layer x,u,o,y,w [T,h], qkv [T,3h], pre (GeLU' of the pre-activation),g [T,f],
  // stats [T,2]x2, lse [b,a,s]
  // plus the output gradients kept for the deferred weight gradients: dz,dy_mid [T,h], dpre [T,f], dqkv [T,3h]
  const uint64_t e_th = align_up((uint64_t)T * h * 2, 256), e_t3h = align_up((uint64_t)T * 3 * h * 2, 256),
                 e_tf = align_up((uint64_t)T * f * 2, 256), e_st = align_up((uint64_t)T * 2 * 4, 256),
                 e_lse = align_up((uint64_t)cfg->microbatch_size * cfg->n_heads * cfg->seq_len * 4, 256);
  const uint64_t per_layer = (cfg->qkv_input_split ? 8 : 7) * e_th + 2 * e_t3h + 3 * e_tf + 2 * e_st + e_lse;
  // carves one layer's record out of p
  auto carve = [&](char*& p, LayerStash& a) {
    a.x = (elem_t*)p; p += e_th;  a.u = (elem_t*)p; p += e_th;  a.o = (elem_t*)p; p += e_th;
    a.y = (elem_t*)p; p += e_th;  a.w = (elem_t*)p; p += e_th;  a.qkv = (elem_t*)p; p += e_t3h;
    a.pre = (elem_t*)p; p += e_tf; a.g = (elem_t*)p; p += e_tf;
    a.stats1 = (float*)p; p += e_st; a.stats2 = (float*)p; p += e_st; a.lse = (float*)p; p += e_lse;
    a.dz = (elem_t*)p; p += e_th; a.dy_mid = (elem_t*)p; p += e_th;
    a.dpre = (elem_t*)p; p += e_tf; a.dqkv = (elem_t*)p; p += e_t3h;
    a.u_lo = nullptr;
    if (cfg->qkv_input_split) { a.u_lo = (elem_t*)p; p += e_th; }
  };
  const int ac = cfg->ckpt_stride;
  st->slot_bytes = ac > 0 ? (uint64_t)(cfg->n_layers / ac) * e_th : per_layer * cfg->n_layers;
  st->slots.resize(cfg->pipeline_limit);
  for (Slot& s : st->slots) {
    CREATE_TRY(hipMalloc((void**)&s.base, st->slot_bytes));
    CREATE_TRY(hipEventCreateWithFlags(&s.fwd_done, hipEventDisableTiming));
    CREATE_TRY(hipEventCreateWithFlags(&s.dgrad_done, hipEventDisableTiming));
    CREATE_TRY(hipEventCreateWithFlags(&s.released, hipEventDisableTiming));
    s.layers.resize(cfg->n_layers);
    char* p = s.base;
    for (int l = 0; l < cfg->n_layers; ++l) {
      LayerStash& a = s.layers[l];
      if (ac > 0) {
        // only the inputs of layers 0, ac, 2ac, ... are kept (Sec. 5.1)
        memset(&a, 0, sizeof a);
        if (l % ac == 0) { a.x = (elem_t*)p; p += e_th; }
      } else {
        carve(p, a);
      }
    }
  }
  if (ac > 0) {
    // shared activation sets: two one-layer sets for forward passes (one more buffer each for the layer
    // inputs that are not kept), three ac-layer sets for regeneration in backward passes
    auto make_set = [&](ActSet& a, int n_layers, bool second_x) -> hipError_t {
      const uint64_t bytes = (uint64_t)n_layers * per_layer + (second_x ? e_th : 0);
      hipError_t e = hipMalloc((void**)&a.base, bytes);
      if (e != hipSuccess) return e;
      st->act_set_bytes += bytes;
      if ((e = hipEventCreateWithFlags(&a.chain_done, hipEventDisableTiming)) != hipSuccess) return e;
      if ((e = hipEventCreateWithFlags(&a.released, hipEventDisableTiming)) != hipSuccess) return e;
      a.layers.resize(n_layers);
      char* p = a.base;
      for (LayerStash& l : a.layers) carve(p, l);
      if (second_x) { a.x2 = (elem_t*)p; p += e_th; }
      return hipSuccess;
    };
    st->fwd_sets.resize(2);
    st->regen_sets.resize(3);
    for (ActSet& a : st->fwd_sets) CREATE_TRY(make_set(a, 1, true));
    for (ActSet& a : st->regen_sets) CREATE_TRY(make_set(a, ac, false));
  }
  // backward workspace
  const int64_t wide = std::max<int64_t>(f, 3 * h);
  // partial column sums: of the LayerNorm parameter gradients (gradient chain), and of the bias gradients where
  // a weight-gradient kernel does not form them itself (weight-gradient stream): one area each
  const uint64_t e_red = align_up((uint64_t)2 * ((T + 63) / 64) * h * 4, 256);
  const uint64_t e_wred = align_up((uint64_t)2 * ((T + 63) / 64) * wide * 4, 256);
  st->ws_bytes = 3 * e_th + e_lse + e_red + e_wred;
  CREATE_TRY(hipMalloc((void**)&st->ws_base, st->ws_bytes));
  {
    char* p = st->ws_base;
    st->dw = (elem_t*)p; p += e_th; st->dattn = (elem_t*)p; p += e_th; st->du = (elem_t*)p; p += e_th;
    st->delta = (float*)p; p += e_lse; st->red_ws = (float*)p; p += e_red;
    st->wgrad_red_ws = (float*)p; p += e_wred;
  }
  CREATE_TRY(hipEventCreateWithFlags(&st->last_bwd, hipEventDisableTiming));
  CREATE_TRY(hipEventCreateWithFlags(&st->last_wgrad, hipEventDisableTiming));
  CREATE_TRY(hipEventCreateWithFlags(&st->wgrad_tail, hipEventDisableTiming));
  CREATE_TRY(hipEventCreateWithFlags(&st->fork_ev, hipEventDisableTiming));
  st->chain_layer.assign(cfg->n_layers, nullptr);
  st->grads_final.assign(cfg->n_layers, nullptr);
  for (int l = 0; l < cfg->n_layers; ++l) {
    CREATE_TRY(hipEventCreateWithFlags(&st->chain_layer[l], hipEventDisableTiming));
    CREATE_TRY(hipEventCreateWithFlags(&st->grads_final[l], hipEventDisableTiming));
  }
  CREATE_TRY(hipDeviceSynchronize());
#undef CREATE_TRY
  *out = st;
  return AXONN_OK;
}

int axonn_stage_destroy(axonn_stage_t* st) {
  if (!st) return fail(AXONN_EINVAL, "stage_destroy: null handle");
  destroy_stage(st);
  return AXONN_OK;
}

int axonn_stage_param_count(const axonn_stage_t* st, uint64_t* n) {
  if (!st || !n) return fail(AXONN_EINVAL, "param_count: null argument");
  *n = st->n_params;
  return AXONN_OK;
}
int axonn_stage_num_tensors(const axonn_stage_t* st, int32_t* n) {
  if (!st || !n) return fail(AXONN_EINVAL, "num_tensors: null argument");
  *n = (int32_t)st->tensors.size();
  return AXONN_OK;
}
int axonn_stage_param_layout(const axonn_stage_t* st, int32_t idx, const char** name, uint64_t* offset,
                             int32_t* rank, int64_t dims[4]) {
  if (!st) return fail(AXONN_EINVAL, "param_layout: null handle");
  if (idx < 0 || idx >= (int32_t)st->tensors.size()) return fail(AXONN_EINVAL, "param_layout: index %d out of range", idx);
  const TensorInfo& t = st->tensors[idx];
  if (name) *name = t.name.c_str();
  if (offset) *offset = t.offset;
  if (rank) *rank = t.rank;
  if (dims) memcpy(dims, t.dims, sizeof t.dims);
  return AXONN_OK;
}
int axonn_stage_params(axonn_stage_t* st, void** p) {
  if (!st || !p) return fail(AXONN_EINVAL, "stage_params: null argument");
  *p = st->params;
  return AXONN_OK;
}
int axonn_stage_grads(axonn_stage_t* st, void** p) {
  if (!st || !p) return fail(AXONN_EINVAL, "stage_grads: null argument");
  *p = st->grads;
  return AXONN_OK;
}
int axonn_stage_zero_grad(axonn_stage_t* st, void* hip_stream) {
  if (!st) return fail(AXONN_EINVAL, "zero_grad: null handle");
  if (st->in_flight) return fail(AXONN_ESTATE, "zero_grad: %d microbatches in flight", st->in_flight);
  HIP_TRY(hipSetDevice(st->cfg.device));
  hipStream_t s = (hipStream_t)hip_stream;
  if (st->last_bwd_recorded) HIP_TRY(hipStreamWaitEvent(s, st->last_bwd, 0));
  if (st->last_wgrad_recorded) HIP_TRY(hipStreamWaitEvent(s, st->last_wgrad, 0));
  // no memory is touched: the first backward / weight-gradient pass of a batch overwrites the
  // accumulators.  Microbatches whose weight gradients were still pending are dropped.
  host::release_awaiting(st->slots);
  st->bwd_count = 0;
  st->wgrad_flushes = 0;
  st->grads_final_recorded = false;
  if (st->embed) st->embed->bwd_count = 0;
  if (st->head) st->head->count = 0;
  st->fwd_issued = st->bwd_issued = 0;
  st->dispatch_log.clear();
  return AXONN_OK;
}
int axonn_stage_device_bytes(const axonn_stage_t* st, uint64_t bytes[6]) {
  if (!st || !bytes) return fail(AXONN_EINVAL, "device_bytes: null argument");
  bytes[0] = st->n_params * 2;
  bytes[1] = st->n_params * 2;
  bytes[2] = st->grads32 ? st->n_params * 4 : 0;
  bytes[3] = st->slot_bytes * st->slots.size();
  bytes[4] = st->ws_bytes + st->act_set_bytes;
  bytes[5] = st->opt ? st->opt->device_bytes : 0;
  return AXONN_OK;
}

int axonn_stage_forward(axonn_stage_t* st, int32_t mb_id, const void* x, void* y, void* hip_stream) {
  if (!st || !x || !y) return fail(AXONN_EINVAL, "forward: null argument");
  if (st->embed || st->head)
    return fail(AXONN_ESTATE, "forward: a stage with the pipeline's ends attached runs in message-driven mode");
  HIP_TRY(hipSetDevice(st->cfg.device));
  return do_forward(st, mb_id, x, y, (hipStream_t)hip_stream, (hipStream_t)hip_stream);
}
int axonn_stage_backward(axonn_stage_t* st, int32_t mb_id, const void* dy, void* dx, void* hip_stream) {
  if (!st || !dy || !dx) return fail(AXONN_EINVAL, "backward: null argument");
  if (st->embed || st->head)
    return fail(AXONN_ESTATE, "backward: a stage with the pipeline's ends attached runs in message-driven mode");
  HIP_TRY(hipSetDevice(st->cfg.device));
  return do_backward(st, mb_id, dy, dx, (hipStream_t)hip_stream, (hipStream_t)hip_stream);
}

int axonn_stage_post(axonn_stage_t* st, const axonn_msg* msg) {
  if (!st || !msg) return fail(AXONN_EINVAL, "post: null argument");
  if (msg->kind != 0 && msg->kind != 1) return fail(AXONN_EINVAL, "post: kind must be 0 (forward) or 1 (backward)");
  if (!msg->payload_dev) return fail(AXONN_EINVAL, "post: null payload");
  // a result nobody receives may be left out: the input gradient of a stage that starts with the embedding
  const bool result_unused = st->embed && (msg->kind == 1 || st->head);
  if (!msg->result_dev && !result_unused) return fail(AXONN_EINVAL, "post: null result buffer");
  if (st->head && msg->kind == 1)
    return fail(AXONN_ESTATE, "post: the last stage starts Backward itself after each Forward (Alg. 2); it takes "
                "no messages from a next stage");
  if (st->head && msg->kind == 0 && (!msg->targets_dev || !msg->loss_dev))
    return fail(AXONN_EINVAL, "post: a forward message to the last stage needs targets_dev and loss_dev");
  if (msg->mb_id < 0) return fail(AXONN_EINVAL, "post: negative microbatch id");
  const auto posted = [st](size_t i) { return std::make_pair((int)st->inbox[i].m.kind, (int)st->inbox[i].m.mb_id); };
  switch (host::check_post(msg->kind, msg->mb_id, st->inbox.size(), posted,
                           msg->kind == 0 ? st->fwd_issued : st->bwd_issued, st->cfg.n_microbatches)) {
    case host::POST_DUPLICATE: return fail(AXONN_ESTATE, "post: duplicate message for microbatch %d", msg->mb_id);
    case host::POST_SURPLUS:
      return fail(AXONN_ESTATE, "post: more than n_microbatches (%d) messages of kind %d in this batch",
                  st->cfg.n_microbatches, msg->kind);
    default: break;
  }
  st->inbox.push_back(PendingMsg{*msg});
  return AXONN_OK;
}

}  // extern "C"

namespace {
// The receive loop of Alg. 2.  blocking: until the batch's last message is dispatched (waiting for posted
// messages to arrive; an error if none can ever be scheduled).  Otherwise: dispatches what is ready now and
// returns, so that one host thread can serve several stages in turn.
int run_loop(axonn_stage* st, int n_streams, void* hip_stream, bool blocking, int32_t* n_dispatched) {
  if (n_dispatched) *n_dispatched = 0;
  HIP_TRY(hipSetDevice(st->cfg.device));
  AX_TRY(ensure_streams(st, n_streams));
  // the library streams start after everything already queued on the caller's stream
  HIP_TRY(hipEventRecord(st->fork_ev, (hipStream_t)hip_stream));
  for (int i = 0; i < n_streams; ++i) HIP_TRY(hipStreamWaitEvent(st->streams[i], st->fork_ev, 0));
  // weight-gradient passes get a stream of their own when there is more than one, so that they
  // overlap the next microbatches' work
  hipStream_t ws = st->streams[0];
  struct ConcurrentScope {
    explicit ConcurrentScope(int v) { t_concurrent = v; }
    ~ConcurrentScope() { t_concurrent = 0; }
  } concurrent_scope(n_streams > 1 ? 1 : 0);
  if (n_streams > 1) {
    if (!st->wgrad_stream) HIP_TRY(hipStreamCreateWithFlags(&st->wgrad_stream, hipStreamNonBlocking));
    ws = st->wgrad_stream;
    HIP_TRY(hipStreamWaitEvent(ws, st->fork_ev, 0));
  }
  const int M = st->cfg.n_microbatches;
  const auto t0 = std::chrono::steady_clock::now();
  const auto now_s = [t0] { return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count(); };
  host::WaitClock wait(st->message_wait_s);
  hipError_t query_error = hipSuccess;
  const auto posted = [st](size_t i) { return std::make_pair((int)st->inbox[i].m.kind, (int)st->inbox[i].m.mb_id); };
  const auto arrived = [st, &query_error](size_t i) {
    void* ev = st->inbox[i].m.ready_event;
    if (!ev) return 1;
    const hipError_t q = hipEventQuery((hipEvent_t)ev);
    if (q == hipSuccess) return 1;
    if (q == hipErrorNotReady) return 0;
    query_error = q;
    return -1;
  };
  while (st->fwd_issued < M || st->bwd_issued < M) {
    // first posted message that has arrived and is admissible
    bool any_admissible = false;
    int err = 0;
    const int chosen = host::choose_message(st->inbox.size(), posted, arrived, st->slots, st->in_flight,
                                            st->cfg.pipeline_limit, &any_admissible, &err);
    if (err) return fail(AXONN_EHIP, "run: hipEventQuery failed: %s", hipGetErrorString(query_error));
    if (chosen < 0) {
      if (!blocking) break;
      if (!any_admissible)
        return fail(AXONN_ESTATE,
                    "run: %d forward and %d backward messages still expected but none of the %zu posted "
                    "messages can be scheduled", M - st->fwd_issued, M - st->bwd_issued, st->inbox.size());
      // Every wait has its own limit (a long batch with a slow but live producer is no error).  On expiry nothing
      // is lost: the posted messages stay posted, what was dispatched stays enqueued, and the caller may call run
      // again, or synchronize and start over with zero_grad.
      if (wait.expired(now_s()))
        return fail(AXONN_ESTATE, "run: waited %.0f s for a posted message to arrive (axonn_stage_set_message_wait "
                    "changes the limit); the batch can be resumed with another run", st->message_wait_s);
      std::this_thread::yield();
      continue;
    }
    wait.dispatched();
    const axonn_msg m = st->inbox[chosen].m;
    st->inbox.erase(st->inbox.begin() + chosen);
    const int si = host::stream_index(m.kind, n_streams, &st->fwd_rr);
    hipStream_t s = st->streams[si];
    if (m.ready_event) HIP_TRY(hipStreamWaitEvent(s, (hipEvent_t)m.ready_event, 0));
    if (m.kind == 0) {
      AX_TRY(do_forward(st, m.mb_id, m.payload_dev, m.result_dev, s, ws));
      st->fwd_issued++;
      st->dispatch_log.push_back(m.mb_id * 2);
      if (st->head) {
        // last stage (Alg. 2): the loss follows the forward pass and Backward(1) starts at once, on the
        // stream of the backward chains
        Slot* slot = find_live(st, m.mb_id);
        hipStream_t bs = st->streams[0];
        HIP_TRY(hipStreamWaitEvent(bs, slot->fwd_done, 0));
        if (st->last_bwd_recorded) HIP_TRY(hipStreamWaitEvent(bs, st->last_bwd, 0));   // head_dx is shared
        AX_TRY(head_forward_backward(st->head, slot->head_y, (const int32_t*)m.targets_dev, (float*)m.loss_dev,
                                     st->head_dx, bs));
        AX_TRY(backward_msg(st, m.mb_id, st->head_dx, m.result_dev, bs, ws));
        st->bwd_issued++;
        st->dispatch_log.push_back(m.mb_id * 2 + 1);
        s = bs;
      }
    } else {
      AX_TRY(backward_msg(st, m.mb_id, m.payload_dev, m.result_dev, s, ws));
      st->bwd_issued++;
      st->dispatch_log.push_back(m.mb_id * 2 + 1);
    }
    // the result buffer is complete once this fires: what a neighbouring stage's message waits for
    if (m.done_event) HIP_TRY(hipEventRecord((hipEvent_t)m.done_event, s));
    if (n_dispatched) ++*n_dispatched;
  }
  return AXONN_OK;
}
}  // namespace

extern "C" {
int axonn_stage_run(axonn_stage_t* st, int32_t n_streams, void* hip_stream) {
  if (!st) return fail(AXONN_EINVAL, "run: null handle");
  if (n_streams < 1 || n_streams > 8) return fail(AXONN_EINVAL, "run: n_streams must be in 1..8");
  return run_loop(st, n_streams, hip_stream, true, nullptr);
}

int axonn_stage_poll(axonn_stage_t* st, int32_t n_streams, void* hip_stream, int32_t* n_dispatched,
                     int32_t* n_remaining) {
  if (!st) return fail(AXONN_EINVAL, "poll: null handle");
  if (n_streams < 1 || n_streams > 8) return fail(AXONN_EINVAL, "poll: n_streams must be in 1..8");
  const int rc = run_loop(st, n_streams, hip_stream, false, n_dispatched);
  if (n_remaining) *n_remaining = 2 * st->cfg.n_microbatches - st->fwd_issued - st->bwd_issued;
  return rc;
}

int axonn_stage_set_message_wait(axonn_stage_t* st, double seconds) {
  if (!st) return fail(AXONN_EINVAL, "set_message_wait: null handle");
  if (!(seconds > 0.0)) return fail(AXONN_EINVAL, "set_message_wait: the limit must be positive");
  st->message_wait_s = seconds;
  return AXONN_OK;
}

int axonn_stage_join(axonn_stage_t* st, void* user_stream) {
  if (!st) return fail(AXONN_EINVAL, "join: null handle");
  HIP_TRY(hipSetDevice(st->cfg.device));
  for (size_t i = 0; i < st->streams.size(); ++i) {
    HIP_TRY(hipEventRecord(st->stream_tail[i], st->streams[i]));
    HIP_TRY(hipStreamWaitEvent((hipStream_t)user_stream, st->stream_tail[i], 0));
  }
  if (st->wgrad_stream) {
    HIP_TRY(hipEventRecord(st->wgrad_tail, st->wgrad_stream));
    HIP_TRY(hipStreamWaitEvent((hipStream_t)user_stream, st->wgrad_tail, 0));
  }
  return AXONN_OK;
}

int axonn_stage_synchronize(axonn_stage_t* st) {
  if (!st) return fail(AXONN_EINVAL, "synchronize: null handle");
  HIP_TRY(hipSetDevice(st->cfg.device));
  HIP_TRY(hipDeviceSynchronize());
  return AXONN_OK;
}

int axonn_stage_dispatch_log(const axonn_stage_t* st, int32_t* out, int32_t capacity, int32_t* n_written) {
  if (!st || !n_written || (capacity > 0 && !out)) return fail(AXONN_EINVAL, "dispatch_log: null argument");
  int n = 0;
  for (; n < capacity && n < (int)st->dispatch_log.size(); ++n) out[n] = st->dispatch_log[n];
  *n_written = n;
  return AXONN_OK;
}

// ----------------------------------------------------------------- offloaded Adam
int axonn_offload_adam_create(int32_t device, uint64_t n, uint64_t bucket_elems, void* param16_dev,
                              const void* grad16_dev, float* host_master, float* host_m, float* host_v,
                              axonn_offload_adam_t** out) {
  if (!out) return fail(AXONN_EINVAL, "adam_create: null output");
  *out = nullptr;
  if (!param16_dev || !grad16_dev || !host_master || !host_m || !host_v)
    return fail(AXONN_EINVAL, "adam_create: null buffer");
  if (n == 0) return fail(AXONN_EINVAL, "adam_create: n == 0");
  if (bucket_elems == 0 || bucket_elems % 8) return fail(AXONN_EINVAL, "adam_create: bucket_elems must be a positive multiple of 8");
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (device < 0 || device >= ndev) return fail(AXONN_EINVAL, "adam_create: device %d of %d", device, ndev);
  HIP_TRY(hipSetDevice(device));
  axonn_offload_adam* o = new (std::nothrow) axonn_offload_adam();
  if (!o) return fail(AXONN_ENOMEM, "adam_create: host allocation failed");
  o->device = device; o->n = n; o->bucket = std::min<uint64_t>(bucket_elems, align_up(n, 8));
  o->p16 = (elem_t*)param16_dev; o->g16 = (const elem_t*)grad16_dev;
  o->h_theta = host_master; o->h_m = host_m; o->h_v = host_v;
#define ADAM_TRY(expr)                                                                           \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) {                                                                      \
      destroy_adam(o);                                                                           \
      return fail(e_ == hipErrorOutOfMemory ? AXONN_ENOMEM : AXONN_EHIP, "%s failed: %s", #expr, \
                  hipGetErrorString(e_));                                                        \
    }                                                                                            \
  } while (0)
  for (int i = 0; i < axonn_offload_adam::kSets; ++i) {
    for (int j = 0; j < 3; ++j) {
      ADAM_TRY(hipMalloc((void**)&o->d_buf[i][j], o->bucket * sizeof(float)));
      o->device_bytes += o->bucket * sizeof(float);
    }
    ADAM_TRY(hipEventCreateWithFlags(&o->ev_h2d[i], hipEventDisableTiming));
    ADAM_TRY(hipEventCreateWithFlags(&o->ev_k[i], hipEventDisableTiming));
    ADAM_TRY(hipEventCreateWithFlags(&o->ev_d2h[i], hipEventDisableTiming));
  }
  ADAM_TRY(hipEventCreateWithFlags(&o->ev_start, hipEventDisableTiming));
  ADAM_TRY(hipStreamCreateWithFlags(&o->s_h2d, hipStreamNonBlocking));
  ADAM_TRY(hipStreamCreateWithFlags(&o->s_k, hipStreamNonBlocking));
  ADAM_TRY(hipStreamCreateWithFlags(&o->s_d2h, hipStreamNonBlocking));
#undef ADAM_TRY
  *out = o;
  return AXONN_OK;
}

int axonn_offload_adam_destroy(axonn_offload_adam_t* opt) {
  if (!opt) return fail(AXONN_EINVAL, "adam_destroy: null handle");
  destroy_adam(opt);
  return AXONN_OK;
}

int axonn_offload_adam_device_bytes(const axonn_offload_adam_t* opt, uint64_t* bytes) {
  if (!opt || !bytes) return fail(AXONN_EINVAL, "adam_device_bytes: null argument");
  *bytes = opt->device_bytes;
  return AXONN_OK;
}

namespace {
int fetch_bucket(axonn_offload_adam* o, int set, uint64_t off, size_t bytes, hipStream_t s) {
  // the set must have been drained by the bucket that used it last
  if (o->d2h_recorded[set]) HIP_TRY(hipStreamWaitEvent(s, o->ev_d2h[set], 0));
  HIP_TRY(hipMemcpyAsync(o->d_buf[set][0], o->h_theta + off, bytes, hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(o->d_buf[set][1], o->h_m + off, bytes, hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(o->d_buf[set][2], o->h_v + off, bytes, hipMemcpyHostToDevice, s));
  HIP_TRY(hipEventRecord(o->ev_h2d[set], s));
  return AXONN_OK;
}

// One pass over all buckets.  Without `gate`: in ascending order, after everything queued on the caller's
// stream.  With `gate`: in descending order and in chunks of chunk_buckets buckets; the updates of a chunk
// start once gate(lo, hi) (elements [lo, hi) of the chunk) has fired, while the fetches of the fp32 state
// do not wait for gradients at all.  `early` (or null): a stream that has nothing left to do but the work
// already queued on it; the first fetches (one per buffer set) go there instead of the fetch stream, whose
// commands may share a hardware queue with busy streams and would then start behind all their queued work.
int adam_pass_body(axonn_offload_adam* o, double lr, double beta1, double beta2, double eps, double weight_decay,
                   int64_t step, double grad_scale, hipStream_t user, int chunk_buckets,
                   const std::function<hipEvent_t(uint64_t, uint64_t)>* gate, hipStream_t early,
                   uint64_t* buckets_queued) {
  constexpr int S = axonn_offload_adam::kSets;
  // everything already queued on the caller's stream comes first
  HIP_TRY(hipEventRecord(o->ev_start, user));
  HIP_TRY(hipStreamWaitEvent(o->s_h2d, o->ev_start, 0));
  HIP_TRY(hipStreamWaitEvent(o->s_k, o->ev_start, 0));
  HIP_TRY(hipStreamWaitEvent(o->s_d2h, o->ev_start, 0));
  // the early fetches deliberately do not wait for the caller's stream: an event recorded there can sit in a
  // hardware queue behind the whole batch; they are ordered after the previous pass by the sets' drain events
  const uint64_t nb = host::bucket_count(o->n, o->bucket);
  for (uint64_t i = 0; i < nb; ++i) {
    const host::BucketPlan bp = host::bucket_plan(o->n, o->bucket, S, i, gate != nullptr);
    const int set = bp.set;
    const uint64_t off = bp.offset, cnt = bp.count;
    const size_t bytes = cnt * sizeof(float);
    AX_TRY(fetch_bucket(o, set, off, bytes, (early && i < (uint64_t)S) ? early : o->s_h2d));
    // update
    if (gate && i % (uint64_t)chunk_buckets == 0) {
      // the chunk: the next chunk_buckets buckets in processing order, i.e. downwards from this one
      uint64_t lo = 0, hi = 0;
      host::chunk_span(o->n, o->bucket, (uint64_t)chunk_buckets, i, &lo, &hi);
      HIP_TRY(hipStreamWaitEvent(o->s_k, (*gate)(lo, hi), 0));
    }
    HIP_TRY(hipStreamWaitEvent(o->s_k, o->ev_h2d[set], 0));
    AX_TRY(adam(cnt, o->d_buf[set][0], o->d_buf[set][1], o->d_buf[set][2], o->g16 + off, o->p16 + off, lr, beta1,
                beta2, eps, weight_decay, step, grad_scale, o->s_k));
    HIP_TRY(hipEventRecord(o->ev_k[set], o->s_k));
    // offload
    HIP_TRY(hipStreamWaitEvent(o->s_d2h, o->ev_k[set], 0));
    HIP_TRY(hipMemcpyAsync(o->h_theta + off, o->d_buf[set][0], bytes, hipMemcpyDeviceToHost, o->s_d2h));
    HIP_TRY(hipMemcpyAsync(o->h_m + off, o->d_buf[set][1], bytes, hipMemcpyDeviceToHost, o->s_d2h));
    HIP_TRY(hipMemcpyAsync(o->h_v + off, o->d_buf[set][2], bytes, hipMemcpyDeviceToHost, o->s_d2h));
    HIP_TRY(hipEventRecord(o->ev_d2h[set], o->s_d2h));
    o->d2h_recorded[set] = true;
    ++*buckets_queued;
  }
  // the caller's stream continues after the last bucket is back in host memory
  const int last = (int)((nb - 1) % S);
  HIP_TRY(hipStreamWaitEvent(user, o->ev_d2h[last], 0));
  HIP_TRY(hipStreamWaitEvent(user, o->ev_k[last], 0));
  // The call returns when the host copies are complete.  Without this, a caller that runs ahead and queues its
  // next batch behind the pending pass fills the hardware queues that the pass's copies share: measured on the 12B
  // stage, the pass then takes 500 ms instead of 323, and single batches behind it run 10 % slower.
  HIP_TRY(hipStreamSynchronize(user));
  return AXONN_OK;
}

int adam_pass(axonn_offload_adam* o, double lr, double beta1, double beta2, double eps, double weight_decay,
              int64_t step, double grad_scale, hipStream_t user, int chunk_buckets,
              const std::function<hipEvent_t(uint64_t, uint64_t)>* gate, hipStream_t early) {
  if (step < 1) return fail(AXONN_EINVAL, "adam_step: step must be >= 1 (got %lld)", (long long)step);
  if (!(beta1 >= 0. && beta1 < 1.) || !(beta2 >= 0. && beta2 < 1.))
    return fail(AXONN_EINVAL, "adam_step: betas must be in [0,1)");
  HIP_TRY(hipSetDevice(o->device));
  uint64_t queued = 0;
  const int rc = adam_pass_body(o, lr, beta1, beta2, eps, weight_decay, step, grad_scale, user, chunk_buckets, gate,
                                early, &queued);
  if (rc != AXONN_OK) {
    // An error in the middle of the pass: whatever was queued may still be copying into the caller's host arrays
    // or writing parameters.  Wait for it, so that nothing is in flight when the error reaches the caller; the
    // buffer sets are then all drained.  The buckets queued before the error have been updated, the rest not.
    const std::string first = g_last_error;
    (void)hipStreamSynchronize(o->s_h2d);
    (void)hipStreamSynchronize(o->s_k);
    (void)hipStreamSynchronize(o->s_d2h);
    if (early) (void)hipStreamSynchronize(early);
    for (bool& r : o->d2h_recorded) r = false;
    return fail(rc, "%s (optimizer pass stopped after %llu of %llu buckets in %s order; those are updated in host "
                "memory and in the 16-bit parameters, the others are untouched)", first.c_str(),
                (unsigned long long)queued, (unsigned long long)host::bucket_count(o->n, o->bucket),
                gate ? "descending" : "ascending");
  }
  return AXONN_OK;
}
}  // namespace

int axonn_offload_adam_step(axonn_offload_adam_t* o, double lr, double beta1, double beta2, double eps,
                            double weight_decay, int64_t step, double grad_scale, void* hip_stream) {
  if (!o) return fail(AXONN_EINVAL, "adam_step: null handle");
  return adam_pass(o, lr, beta1, beta2, eps, weight_decay, step, grad_scale, (hipStream_t)hip_stream, 1, nullptr,
                   nullptr);
}

int axonn_stage_optimizer_attach(axonn_stage_t* st, float* host_master, float* host_m, float* host_v,
                                 uint64_t n, uint64_t bucket_elems) {
  if (!st) return fail(AXONN_EINVAL, "optimizer_attach: null handle");
  if (n != st->n_params) return fail(AXONN_EINVAL, "optimizer_attach: n (%llu) != param_count (%llu)",
                                     (unsigned long long)n, (unsigned long long)st->n_params);
  if (st->opt) { destroy_adam(st->opt); st->opt = nullptr; }
  return axonn_offload_adam_create(st->cfg.device, n, bucket_elems, st->params, st->grads, host_master,
                                   host_m, host_v, &st->opt);
}

int axonn_stage_optimizer_step(axonn_stage_t* st, double lr, double beta1, double beta2, double eps,
                               double weight_decay, int64_t step, double grad_scale, void* hip_stream) {
  if (!st) return fail(AXONN_EINVAL, "optimizer_step: null handle");
  if (!st->opt) return fail(AXONN_ESTATE, "optimizer_step: no optimizer attached");
  if (st->in_flight) return fail(AXONN_ESTATE, "optimizer_step: %d microbatches in flight", st->in_flight);
  HIP_TRY(hipSetDevice(st->cfg.device));
  hipStream_t user = (hipStream_t)hip_stream;
  if (st->last_bwd_recorded) HIP_TRY(hipStreamWaitEvent(user, st->last_bwd, 0));
  if (st->last_wgrad_recorded) HIP_TRY(hipStreamWaitEvent(user, st->last_wgrad, 0));
  if (slots_in_state(st, SLOT_AWAIT_WGRAD))
    return fail(AXONN_ESTATE, "optimizer_step: %d microbatches still await their weight gradients (fewer than "
                "n_microbatches backwards since zero_grad)", slots_in_state(st, SLOT_AWAIT_WGRAD));
  return axonn_offload_adam_step(st->opt, lr, beta1, beta2, eps, weight_decay, step, grad_scale, hip_stream);
}


int axonn_stage_optimizer_step_overlapped(axonn_stage_t* st, double lr, double beta1, double beta2, double eps,
                                          double weight_decay, int64_t step, double grad_scale,
                                          int32_t chunk_buckets, void* hip_stream) {
  if (!st) return fail(AXONN_EINVAL, "optimizer_step_overlapped: null handle");
  if (!st->opt) return fail(AXONN_ESTATE, "optimizer_step_overlapped: no optimizer attached");
  if (chunk_buckets < 1) return fail(AXONN_EINVAL, "optimizer_step_overlapped: chunk_buckets must be >= 1");
  if (st->in_flight) return fail(AXONN_ESTATE, "optimizer_step_overlapped: %d microbatches in flight", st->in_flight);
  if (!st->grads_final_recorded)
    return fail(AXONN_ESTATE, "optimizer_step_overlapped: the batch is not complete (%d of %d backwards since "
                "zero_grad)", st->bwd_count, st->cfg.n_microbatches);
  HIP_TRY(hipSetDevice(st->cfg.device));
  const int L = st->cfg.n_layers;
  // gradients become final from the last layer down: a chunk may start once the lowest layer it touches is
  std::vector<uint64_t> layer_begin(L);
  for (int l = 0; l < L; ++l) layer_begin[l] = st->tensors[l * kTensorsPerLayer].offset;
  const std::function<hipEvent_t(uint64_t, uint64_t)> gate = [st, &layer_begin, L](uint64_t lo, uint64_t) {
    return st->grads_final[host::lowest_layer(layer_begin.data(), L, lo)];
  };
  // message-driven mode with forward streams: the first of them has no more work in this batch
  hipStream_t early = st->streams.size() > 1 ? st->streams[1] : nullptr;
  return adam_pass(st->opt, lr, beta1, beta2, eps, weight_decay, step, grad_scale, (hipStream_t)hip_stream,
                   chunk_buckets, &gate, early);
}

// ------------------------------------------------------------- loss scaling (Sec. 2, mixed precision)
int32_t axonn_element_type(void) { return AXONN_ELEM_TYPE_ID; }

int axonn_count_nonfinite(const void* x_dev, uint64_t n, uint64_t* workspace_dev, void* hip_stream) {
  if (!x_dev || !workspace_dev) return fail(AXONN_EINVAL, "count_nonfinite: null argument");
  return check_launch(launch_count_nonfinite(n, x_dev, workspace_dev, (hipStream_t)hip_stream), "count_nonfinite");
}

// Orders `user` behind the batch's gradients, as the optimizer entry points do.
static int wait_for_gradients(axonn_stage_t* st, hipStream_t user, const char* who) {
  if (st->in_flight) return fail(AXONN_ESTATE, "%s: %d microbatches in flight", who, st->in_flight);
  if (st->last_bwd_recorded) HIP_TRY(hipStreamWaitEvent(user, st->last_bwd, 0));
  if (st->last_wgrad_recorded) HIP_TRY(hipStreamWaitEvent(user, st->last_wgrad, 0));
  if (slots_in_state(st, SLOT_AWAIT_WGRAD))
    return fail(AXONN_ESTATE, "%s: %d microbatches still await their weight gradients (fewer than "
                "n_microbatches backwards since zero_grad)", who, slots_in_state(st, SLOT_AWAIT_WGRAD));
  return AXONN_OK;
}

int axonn_stage_count_nonfinite_grads(axonn_stage_t* st, void* hip_stream, uint64_t* count_host) {
  if (!st || !count_host) return fail(AXONN_EINVAL, "count_nonfinite_grads: null argument");
  HIP_TRY(hipSetDevice(st->cfg.device));
  hipStream_t user = (hipStream_t)hip_stream;
  AX_TRY(wait_for_gradients(st, user, "count_nonfinite_grads"));
  if (!st->nonfinite_ws) HIP_TRY(hipMalloc((void**)&st->nonfinite_ws, kNonfiniteWsCounters * sizeof(uint64_t)));
  AX_TRY(check_launch(launch_count_nonfinite(st->n_params, st->grads, st->nonfinite_ws, user), "count_nonfinite"));
  HIP_TRY(hipMemcpyAsync(count_host, st->nonfinite_ws + (kNonfiniteWsCounters - 1), sizeof(uint64_t),
                         hipMemcpyDeviceToHost, user));
  HIP_TRY(hipStreamSynchronize(user));
  return AXONN_OK;
}

int axonn_stage_optimizer_step_scaled(axonn_stage_t* st, double lr, double beta1, double beta2, double eps,
                                      double weight_decay, int64_t step, double grad_scale,
                                      axonn_loss_scaler* scaler, uint64_t other_nonfinite, void* hip_stream,
                                      int32_t* skipped) {
  if (!st || !scaler || !skipped) return fail(AXONN_EINVAL, "optimizer_step_scaled: null argument");
  if (!st->opt) return fail(AXONN_ESTATE, "optimizer_step_scaled: no optimizer attached");
  if (!(scaler->scale > 0.f) || !(scaler->growth >= 1.f) || !(scaler->backoff > 0.f && scaler->backoff <= 1.f) ||
      scaler->growth_interval < 1 || scaler->good_steps < 0)
    return fail(AXONN_EINVAL, "optimizer_step_scaled: scaler needs scale > 0, growth >= 1, 0 < backoff <= 1, "
                "growth_interval >= 1, good_steps >= 0");
  uint64_t bad = 0;
  AX_TRY(axonn_stage_count_nonfinite_grads(st, hip_stream, &bad));
  if (bad + other_nonfinite != 0) {          // overflow somewhere: drop the batch, lower the scale
    scaler->scale *= scaler->backoff;
    scaler->good_steps = 0;
    *skipped = 1;
    return AXONN_OK;
  }
  *skipped = 0;
  AX_TRY(axonn_stage_optimizer_step(st, lr, beta1, beta2, eps, weight_decay, step, grad_scale / scaler->scale,
                                    hip_stream));
  if (++scaler->good_steps >= scaler->growth_interval) {
    scaler->scale *= scaler->growth;
    scaler->good_steps = 0;
  }
  return AXONN_OK;
}

int axonn_head_set_loss_scale(axonn_head_t* hd, float loss_scale) {
  if (!hd) return fail(AXONN_EINVAL, "head_set_loss_scale: null handle");
  if (!(loss_scale > 0.f) || loss_scale > 3.0e38f) return fail(AXONN_EINVAL, "head_set_loss_scale: scale must be positive and finite");
  hd->loss_scale = loss_scale;
  return AXONN_OK;
}

// ------------------------------------------------------------- first / last stage extras
int axonn_embed_create(int32_t device, int32_t vocab, int32_t hidden, int32_t seq_len, int32_t microbatch_size,
                       axonn_embed_t** out) {
  if (!out) return fail(AXONN_EINVAL, "embed_create: null argument");
  *out = nullptr;
  if (device < 0 || vocab < 1 || hidden < 8 || seq_len < 1 || microbatch_size < 1)
    return fail(AXONN_EINVAL, "embed_create: sizes must be positive");
  if (hidden % 8) return fail(AXONN_EUNSUPPORTED, "embed_create: hidden must be a multiple of 8 (16-byte rows)");
  HIP_TRY(hipSetDevice(device));
  axonn_embed* e = new (std::nothrow) axonn_embed();
  if (!e) return fail(AXONN_ENOMEM, "embed_create: host allocation failed");
  e->device = device; e->vocab = vocab; e->h = hidden; e->s = seq_len; e->b = microbatch_size;
  e->n_params = ((uint64_t)vocab + seq_len) * hidden;
  hipError_t err = hipMalloc((void**)&e->params, e->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = hipMalloc((void**)&e->grads, e->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = hipMemset(e->params, 0, e->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = hipMemset(e->grads, 0, e->n_params * sizeof(elem_t));
  if (err != hipSuccess) {
    if (e->params) (void)hipFree(e->params);
    if (e->grads) (void)hipFree(e->grads);
    delete e;
    return fail(err == hipErrorOutOfMemory ? AXONN_ENOMEM : AXONN_EHIP, "embed_create: %s", hipGetErrorString(err));
  }
  *out = e;
  return AXONN_OK;
}
int axonn_embed_destroy(axonn_embed_t* e) {
  if (!e) return fail(AXONN_EINVAL, "embed_destroy: null handle");
  (void)hipSetDevice(e->device);
  (void)hipDeviceSynchronize();
  (void)hipFree(e->params);
  (void)hipFree(e->grads);
  delete e;
  return AXONN_OK;
}
int axonn_embed_buffers(axonn_embed_t* e, void** params_dev_bf16, void** grads_dev_bf16, uint64_t* n_elements) {
  if (!e) return fail(AXONN_EINVAL, "embed_buffers: null handle");
  if (params_dev_bf16) *params_dev_bf16 = e->params;
  if (grads_dev_bf16) *grads_dev_bf16 = e->grads;
  if (n_elements) *n_elements = e->n_params;
  return AXONN_OK;
}
int axonn_embed_zero_grad(axonn_embed_t* e) {
  if (!e) return fail(AXONN_EINVAL, "embed_zero_grad: null handle");
  e->bwd_count = 0;
  return AXONN_OK;
}
int axonn_embed_forward(axonn_embed_t* e, const int32_t* tokens_dev, void* x_dev_bf16, void* hip_stream) {
  if (!e || !tokens_dev || !x_dev_bf16) return fail(AXONN_EINVAL, "embed_forward: null argument");
  HIP_TRY(hipSetDevice(e->device));
  return embed_forward(e, tokens_dev, x_dev_bf16, (hipStream_t)hip_stream);
}
int axonn_embed_backward(axonn_embed_t* e, const int32_t* tokens_dev, const void* dx_dev_bf16, void* hip_stream) {
  if (!e || !tokens_dev || !dx_dev_bf16) return fail(AXONN_EINVAL, "embed_backward: null argument");
  HIP_TRY(hipSetDevice(e->device));
  return embed_backward(e, tokens_dev, dx_dev_bf16, (hipStream_t)hip_stream);
}

int axonn_head_create(int32_t device, int32_t vocab, int32_t hidden, int32_t tokens_per_microbatch,
                      int32_t n_microbatches, float ln_eps, axonn_head_t** out) {
  if (!out) return fail(AXONN_EINVAL, "head_create: null argument");
  *out = nullptr;
  if (device < 0 || vocab < 1 || hidden < 8 || tokens_per_microbatch < 1 || n_microbatches < 1 || !(ln_eps > 0.f))
    return fail(AXONN_EINVAL, "head_create: sizes and ln_eps must be positive");
  if (hidden % 8 || vocab % 8 || tokens_per_microbatch % 8)
    return fail(AXONN_EUNSUPPORTED, "head_create: hidden, vocab and tokens_per_microbatch must be multiples of 8");
  if (hidden > 16384) return fail(AXONN_EUNSUPPORTED, "head_create: hidden > 16384 unsupported by the LayerNorm kernel");
  if ((int64_t)tokens_per_microbatch > (1 << 24)) return fail(AXONN_EUNSUPPORTED, "head_create: too many tokens");
  HIP_TRY(hipSetDevice(device));
  axonn_head* hd = new (std::nothrow) axonn_head();
  if (!hd) return fail(AXONN_ENOMEM, "head_create: host allocation failed");
  hd->device = device; hd->vocab = vocab; hd->h = hidden; hd->T = tokens_per_microbatch; hd->M = n_microbatches;
  hd->eps = ln_eps;
  const uint64_t T = hd->T, h = hd->h, V = hd->vocab;
  hd->n_params = 2 * h + h * V;
  const uint64_t e_th = align_up(T * h * 2, 256), e_tv = align_up(T * V * 2, 256), e_st = align_up(T * 2 * 4, 256),
                 e_tl = align_up(T * 4, 256), e_red = align_up(2 * ((T + 63) / 64) * h * 4, 256);
  hd->ws_bytes = 2 * e_th + e_tv + e_st + e_tl + e_red;
  hipError_t err = hipMalloc((void**)&hd->params, hd->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = hipMalloc((void**)&hd->grads, hd->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = hipMalloc((void**)&hd->ws_base, hd->ws_bytes);
  if (err == hipSuccess) err = hipMemset(hd->params, 0, hd->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = hipMemset(hd->grads, 0, hd->n_params * sizeof(elem_t));
  if (err == hipSuccess) err = launch_fill_elem(h, hd->params, 1.0f, nullptr);   // LayerNorm gain 1
  if (err == hipSuccess) err = hipDeviceSynchronize();
  if (err != hipSuccess) {
    if (hd->params) (void)hipFree(hd->params);
    if (hd->grads) (void)hipFree(hd->grads);
    if (hd->ws_base) (void)hipFree(hd->ws_base);
    delete hd;
    return fail(err == hipErrorOutOfMemory ? AXONN_ENOMEM : AXONN_EHIP, "head_create: %s", hipGetErrorString(err));
  }
  char* p = hd->ws_base;
  hd->a = (elem_t*)p; p += e_th; hd->da = (elem_t*)p; p += e_th; hd->logits = (elem_t*)p; p += e_tv;
  hd->stats = (float*)p; p += e_st; hd->token_loss = (float*)p; p += e_tl; hd->red_ws = (float*)p; p += e_red;
  *out = hd;
  return AXONN_OK;
}
int axonn_head_destroy(axonn_head_t* hd) {
  if (!hd) return fail(AXONN_EINVAL, "head_destroy: null handle");
  (void)hipSetDevice(hd->device);
  (void)hipDeviceSynchronize();
  (void)hipFree(hd->params);
  (void)hipFree(hd->grads);
  (void)hipFree(hd->ws_base);
  delete hd;
  return AXONN_OK;
}
int axonn_head_buffers(axonn_head_t* hd, void** params_dev_bf16, void** grads_dev_bf16, uint64_t* n_elements) {
  if (!hd) return fail(AXONN_EINVAL, "head_buffers: null handle");
  if (params_dev_bf16) *params_dev_bf16 = hd->params;
  if (grads_dev_bf16) *grads_dev_bf16 = hd->grads;
  if (n_elements) *n_elements = hd->n_params;
  return AXONN_OK;
}
int axonn_head_zero_grad(axonn_head_t* hd) {
  if (!hd) return fail(AXONN_EINVAL, "head_zero_grad: null handle");
  hd->count = 0;
  return AXONN_OK;
}
int axonn_head_forward_backward(axonn_head_t* hd, const void* x_dev_bf16, const int32_t* targets_dev,
                                float* loss_dev, void* dx_dev_bf16, void* hip_stream) {
  if (!hd || !x_dev_bf16 || !targets_dev || !loss_dev || !dx_dev_bf16)
    return fail(AXONN_EINVAL, "head_forward_backward: null argument");
  HIP_TRY(hipSetDevice(hd->device));
  return head_forward_backward(hd, x_dev_bf16, targets_dev, loss_dev, dx_dev_bf16, (hipStream_t)hip_stream);
}

int axonn_stage_attach_ends(axonn_stage_t* st, axonn_embed_t* embed, axonn_head_t* head) {
  if (!st) return fail(AXONN_EINVAL, "attach_ends: null handle");
  if (st->in_flight || !st->inbox.empty()) return fail(AXONN_ESTATE, "attach_ends: work in flight");
  if (embed && (embed->h != st->h || embed->s != st->cfg.seq_len || embed->b != st->cfg.microbatch_size ||
                embed->device != st->cfg.device))
    return fail(AXONN_EINVAL, "attach_ends: the embedding's hidden size, sequence length, microbatch size or device "
                "differ from the stage's");
  if (head && (head->h != st->h || head->T != st->T || head->M != st->cfg.n_microbatches ||
               head->device != st->cfg.device))
    return fail(AXONN_EINVAL, "attach_ends: the head's hidden size, tokens per microbatch, microbatch count or "
                "device differ from the stage's");
  HIP_TRY(hipSetDevice(st->cfg.device));
  HIP_TRY(hipDeviceSynchronize());
  const uint64_t e_th = align_up((uint64_t)st->T * st->h * 2, 256);
  if (embed && !st->embed_dx) HIP_TRY(hipMalloc((void**)&st->embed_dx, e_th));
  if (head && !st->head_dx) {
    HIP_TRY(hipMalloc((void**)&st->head_dx, e_th));
    HIP_TRY(hipMalloc((void**)&st->head_y_base, e_th * st->slots.size()));
    for (size_t i = 0; i < st->slots.size(); ++i) st->slots[i].head_y = (elem_t*)((char*)st->head_y_base + i * e_th);
  }
  st->embed = embed;
  st->head = head;
  return AXONN_OK;
}

// ----------------------------------------------------------------- tuning and test hooks
int axonn_tuning(int32_t knob, int64_t value) {
  if (!set_gemm_tuning(knob, value))
    return fail(AXONN_EINVAL, "tuning: unknown knob %d or value %lld out of range", (int)knob, (long long)value);
  return AXONN_OK;
}

// ----------------------------------------------------------------- launch timing
int axonn_profile_enable(int32_t on) {
  g_prof_on = on != 0;
  return AXONN_OK;
}
int axonn_profile_num_categories(int32_t* n) {
  if (!n) return fail(AXONN_EINVAL, "profile_num_categories: null argument");
  *n = PC_COUNT;
  return AXONN_OK;
}
int axonn_profile_category_name(int32_t idx, const char** name) {
  if (!name || idx < 0 || idx >= PC_COUNT) return fail(AXONN_EINVAL, "profile_category_name: bad argument");
  *name = kProfNames[idx];
  return AXONN_OK;
}
int axonn_profile_collect(double* total_ms, int64_t* launches, int32_t n_categories) {
  if (!total_ms || !launches || n_categories < PC_COUNT)
    return fail(AXONN_EINVAL, "profile_collect: need arrays of at least %d entries", (int)PC_COUNT);
  for (int i = 0; i < n_categories; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  int rc = AXONN_OK;
  for (ProfRec& r : g_prof_recs) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess && rc == AXONN_OK)
      rc = fail(AXONN_EHIP, "profile_collect: %s", hipGetErrorString(e));
    if (e == hipSuccess) { total_ms[r.cat] += ms; launches[r.cat]++; }
    g_prof_pool.push_back(r.a);
    g_prof_pool.push_back(r.b);
  }
  g_prof_recs.clear();
  return rc;
}

// Bare copy rates of the host link with the calls the optimizer pipeline makes (hipMemcpyAsync between pinned host
// memory and device memory, one stream per direction): the denominator of the optimizer step's link fraction.
int axonn_host_link_probe(int32_t device, uint64_t bytes, int32_t reps, double gbps_out[3]) {
  if (!gbps_out || bytes == 0 || reps < 1) return fail(AXONN_EINVAL, "host_link_probe: bad argument");
  HIP_TRY(hipSetDevice(device));
  void *h_in = nullptr, *h_out = nullptr, *d_in = nullptr, *d_out = nullptr;
  hipStream_t s_in = nullptr, s_out = nullptr;
  hipEvent_t e[4] = {};
  int rc = AXONN_OK;
  auto run = [&]() -> int {
    HIP_TRY(hipHostMalloc(&h_in, bytes, hipHostMallocDefault));
    HIP_TRY(hipHostMalloc(&h_out, bytes, hipHostMallocDefault));
    HIP_TRY(hipMalloc(&d_in, bytes));
    HIP_TRY(hipMalloc(&d_out, bytes));
    memset(h_in, 1, bytes);
    memset(h_out, 2, bytes);
    HIP_TRY(hipMemset(d_out, 3, bytes));
    HIP_TRY(hipStreamCreateWithFlags(&s_in, hipStreamNonBlocking));
    HIP_TRY(hipStreamCreateWithFlags(&s_out, hipStreamNonBlocking));
    for (auto& ev : e) HIP_TRY(hipEventCreate(&ev));
    for (int mode = -1; mode < 3; ++mode) {          // -1: warm-up of both directions; 0: in; 1: out; 2: both
      const bool in = mode != 1, out = mode != 0;
      HIP_TRY(hipDeviceSynchronize());
      if (in) HIP_TRY(hipEventRecord(e[0], s_in));
      if (out) HIP_TRY(hipEventRecord(e[2], s_out));
      for (int r = 0; r < reps; ++r) {
        if (in) HIP_TRY(hipMemcpyAsync(d_in, h_in, bytes, hipMemcpyHostToDevice, s_in));
        if (out) HIP_TRY(hipMemcpyAsync(h_out, d_out, bytes, hipMemcpyDeviceToHost, s_out));
      }
      if (in) HIP_TRY(hipEventRecord(e[1], s_in));
      if (out) HIP_TRY(hipEventRecord(e[3], s_out));
      HIP_TRY(hipDeviceSynchronize());
      float ms_in = 0.f, ms_out = 0.f;
      if (in) HIP_TRY(hipEventElapsedTime(&ms_in, e[0], e[1]));
      if (out) HIP_TRY(hipEventElapsedTime(&ms_out, e[2], e[3]));
      const double total = (double)bytes * reps / 1e9;
      if (mode == 0) gbps_out[0] = total / (ms_in * 1e-3);
      if (mode == 1) gbps_out[1] = total / (ms_out * 1e-3);
      if (mode == 2) gbps_out[2] = total / (std::max(ms_in, ms_out) * 1e-3);     // per direction, both running
    }
    return AXONN_OK;
  };
  rc = run();
  for (auto& ev : e) if (ev) (void)hipEventDestroy(ev);
  if (s_in) (void)hipStreamDestroy(s_in);
  if (s_out) (void)hipStreamDestroy(s_out);
  if (d_in) (void)hipFree(d_in);
  if (d_out) (void)hipFree(d_out);
  if (h_in) (void)hipHostFree(h_in);
  if (h_out) (void)hipHostFree(h_out);
  return rc;
}

// -------------------------------------------------------------- single operations
int axonn_gemm_bf16(int32_t a_kcontig, int32_t b_kcontig, int32_t epilogue, int64_t M, int64_t N, int64_t K,
                    const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                    const void* bias, const void* res, int64_t ld_res, void* aux, int64_t ld_aux,
                    int32_t accumulate, void* hip_stream) {
  if (!A || !B || !C) return fail(AXONN_EINVAL, "gemm: null operand");
  if (M < 1 || N < 1 || K < 1) return fail(AXONN_EINVAL, "gemm: non-positive size");
  if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24)) return fail(AXONN_EUNSUPPORTED, "gemm: dimension above 2^24");
  if ((M | N | K | lda | ldb | ldc) % 8) return fail(AXONN_EUNSUPPORTED, "gemm: M, N, K and leading dimensions must be multiples of 8");
  if (epilogue < 0 || epilogue > 5) return fail(AXONN_EINVAL, "gemm: unknown epilogue %d", epilogue);
  const bool akc = a_kcontig != 0, bkc = b_kcontig != 0;
  const bool fwd = akc && !bkc, dgrad = akc && bkc, wgrad = !akc && !bkc;
  const bool ok = (fwd && epilogue <= 2) || (dgrad && (epilogue == 0 || epilogue == 3)) ||
                  (wgrad && (epilogue == 4 || epilogue == 5));
  if (!ok) return fail(AXONN_EUNSUPPORTED, "gemm: epilogue %d is not built for layout (a_kcontig=%d, b_kcontig=%d)",
                       epilogue, (int)akc, (int)bkc);
  if (lda < (akc ? K : M) || ldb < (bkc ? K : N) || ldc < N) return fail(AXONN_EINVAL, "gemm: leading dimension too small");
  if (epilogue == 1 && (!res || ld_res < N || ld_res % 8)) return fail(AXONN_EINVAL, "gemm: epilogue 1 needs res with ld_res >= N, multiple of 8");
  if ((epilogue == 2 || epilogue == 3) && (!aux || ld_aux < N || ld_aux % 8)) return fail(AXONN_EINVAL, "gemm: epilogue %d needs aux with ld_aux >= N, multiple of 8", epilogue);
  return gemm(akc, bkc, epilogue, (int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, bias, res, ld_res, aux, ld_aux,
              accumulate, (hipStream_t)hip_stream);
}

int axonn_gemm_wgrad_colsum(int32_t epilogue, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                            const void* B, int64_t ldb, void* C, int64_t ldc, void* colsum, float* workspace,
                            int32_t accumulate, void* hip_stream) {
  if (!A || !B || !C || !colsum || !workspace) return fail(AXONN_EINVAL, "gemm_wgrad_colsum: null argument");
  if (M < 1 || N < 1 || K < 1) return fail(AXONN_EINVAL, "gemm_wgrad_colsum: non-positive size");
  if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24))
    return fail(AXONN_EUNSUPPORTED, "gemm_wgrad_colsum: dimension above 2^24");
  if ((M | N | K | lda | ldb | ldc) % 8)
    return fail(AXONN_EUNSUPPORTED, "gemm_wgrad_colsum: M, N, K and leading dimensions must be multiples of 8");
  if (epilogue != 4 && epilogue != 5) return fail(AXONN_EINVAL, "gemm_wgrad_colsum: epilogue must be 4 or 5 (got %d)", epilogue);
  if (lda < M || ldb < N || ldc < N) return fail(AXONN_EINVAL, "gemm_wgrad_colsum: leading dimension too small");
  const elem_t* a1[1] = {(const elem_t*)A};
  const elem_t* b1[1] = {(const elem_t*)B};
  return gemm_seg(epilogue, (int)M, (int)N, (int)K, a1, lda, b1, ldb, 1, C, ldc, colsum, workspace, accumulate,
                  (hipStream_t)hip_stream);
}

int axonn_layernorm_fwd(int64_t T, int64_t h, const void* x, const void* gamma, const void* beta, float eps,
                        void* out, float* stats, void* hip_stream) {
  if (!x || !gamma || !beta || !out || !stats) return fail(AXONN_EINVAL, "layernorm_fwd: null argument");
  if (T < 1 || h < 1) return fail(AXONN_EINVAL, "layernorm_fwd: non-positive size");
  if (h % 8 || h > 16384) return fail(AXONN_EUNSUPPORTED, "layernorm_fwd: h must be a multiple of 8 and <= 16384");
  return check_launch(launch_layernorm_fwd(T, h, x, gamma, beta, eps, out, nullptr, stats, (hipStream_t)hip_stream), "layernorm_fwd");
}

int axonn_layernorm_bwd(int64_t T, int64_t h, const void* dout, const void* x, const float* stats,
                        const void* gamma, const void* res_grad, void* dx, float* dgamma, float* dbeta,
                        float* workspace, void* hip_stream) {
  if (!dout || !x || !stats || !gamma || !dx || !dgamma || !dbeta || !workspace)
    return fail(AXONN_EINVAL, "layernorm_bwd: null argument");
  if (T < 1 || h < 1) return fail(AXONN_EINVAL, "layernorm_bwd: non-positive size");
  if (h % 8 || h > 16384) return fail(AXONN_EUNSUPPORTED, "layernorm_bwd: h must be a multiple of 8 and <= 16384");
  return check_launch(launch_layernorm_bwd(T, h, dout, x, stats, gamma, res_grad, dx, dgamma, dbeta, 0, true,
                                           workspace, (hipStream_t)hip_stream), "layernorm_bwd");
}

}  // extern "C"

// Scratch of axonn_layernorm_bwd_noalloc: the column partial sums that axonn_layernorm_bwd takes as its
// workspace argument, in device memory that exists from the moment the library is loaded.  Every GPU
// holds its own copy of the array at its own address, so the address is looked up once per device, with
// that device current; host code uses that address, never the array's name.
namespace {
constexpr uint64_t kNoallocScratchFloats = AXONN_LAYERNORM_BWD_NOALLOC_MAX_FLOATS;
static __device__ __align__(256) float scratch[kNoallocScratchFloats];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int noalloc_scratch(float** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices)
    return fail(AXONN_EUNSUPPORTED, "layernorm_bwd_noalloc: device ordinal %d above %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(AXONN_EHIP, "layernorm_bwd_noalloc: the scratch array has no address on device %d", dev);
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return AXONN_OK;
}
}  // namespace

extern "C" {

int axonn_layernorm_bwd_noalloc(int64_t T, int64_t h, const void* dout, const void* x, const float* stats,
                                const void* gamma, const void* res_grad, void* dx, float* dgamma, float* dbeta,
                                void* hip_stream) {
  if (!dout || !x || !stats || !gamma || !dx || !dgamma || !dbeta)
    return fail(AXONN_EINVAL, "layernorm_bwd_noalloc: null argument");
  if (T < 1 || h < 1) return fail(AXONN_EINVAL, "layernorm_bwd_noalloc: non-positive size");
  if (h % 8 || h > 16384)
    return fail(AXONN_EUNSUPPORTED, "layernorm_bwd_noalloc: h must be a multiple of 8 and <= 16384");
  const uint64_t need = 2 * (((uint64_t)T + 63) / 64) * (uint64_t)h;
  if (need > kNoallocScratchFloats)
    return fail(AXONN_EUNSUPPORTED, "layernorm_bwd_noalloc: 2*ceil(T/64)*h = %llu floats of scratch needed, the "
                "built-in buffer holds %llu (use axonn_layernorm_bwd with a workspace of your own)",
                (unsigned long long)need, (unsigned long long)kNoallocScratchFloats);
  float* ws = nullptr;
  AX_TRY(noalloc_scratch(&ws));
  // every partial sum the final reduction reads is written by this call's own first launch: nothing to clear
  return check_launch(launch_layernorm_bwd(T, h, dout, x, stats, gamma, res_grad, dx, dgamma, dbeta, 0, true, ws,
                                           (hipStream_t)hip_stream), "layernorm_bwd");
}

int axonn_colsum(int64_t T, int64_t N, const void* y, int64_t ldy, float* out, float* workspace, void* hip_stream) {
  if (!y || !out || !workspace) return fail(AXONN_EINVAL, "colsum: null argument");
  if (T < 1 || N < 1) return fail(AXONN_EINVAL, "colsum: non-positive size");
  if (N % 8 || ldy % 8 || ldy < N) return fail(AXONN_EUNSUPPORTED, "colsum: N and ldy must be multiples of 8, ldy >= N");
  return check_launch(launch_colsum(T, N, y, ldy, out, 0, true, workspace, (hipStream_t)hip_stream), "colsum");
}

int axonn_attention_fwd(int32_t b, int32_t s, int32_t n_heads, int32_t head_dim, const void* qkv, void* o,
                        float* lse, void* hip_stream) {
  if (!qkv || !o || !lse) return fail(AXONN_EINVAL, "attention_fwd: null argument");
  if (b < 1 || s < 1 || n_heads < 1) return fail(AXONN_EINVAL, "attention_fwd: non-positive size");
  if (head_dim < 4 || head_dim % 4 || head_dim > 192 || ((int64_t)n_heads * head_dim) % 8)
    return fail(AXONN_EUNSUPPORTED, "attention_fwd: head dim must be a multiple of 4, at most 192, and n_heads * "
                "head_dim a multiple of 8");
  if ((int64_t)b * n_heads > 65535) return fail(AXONN_EUNSUPPORTED, "attention_fwd: b*n_heads > 65535");
  return check_launch(launch_attention_fwd(b, s, n_heads, head_dim, qkv, o, lse, (hipStream_t)hip_stream), "attention_fwd");
}

int axonn_attention_bwd(int32_t b, int32_t s, int32_t n_heads, int32_t head_dim, const void* qkv, const void* o,
                        const float* lse, const void* dout, void* dqkv, float* delta_ws, void* hip_stream) {
  if (!qkv || !o || !lse || !dout || !dqkv || !delta_ws) return fail(AXONN_EINVAL, "attention_bwd: null argument");
  if (b < 1 || s < 1 || n_heads < 1) return fail(AXONN_EINVAL, "attention_bwd: non-positive size");
  if (head_dim < 4 || head_dim % 4 || head_dim > 192 || ((int64_t)n_heads * head_dim) % 8)
    return fail(AXONN_EUNSUPPORTED, "attention_bwd: head dim must be a multiple of 4, at most 192, and n_heads * "
                "head_dim a multiple of 8");
  if ((int64_t)b * n_heads > 65535) return fail(AXONN_EUNSUPPORTED, "attention_bwd: b*n_heads > 65535");
  return check_launch(launch_attention_bwd(b, s, n_heads, head_dim, qkv, o, lse, dout, dqkv, delta_ws,
                                           (hipStream_t)hip_stream), "attention_bwd");
}

int axonn_adam_bucket(uint64_t n, float* theta, float* m, float* v, const void* grad16, void* param16, double lr,
                      double beta1, double beta2, double eps, double weight_decay, int64_t step, double grad_scale,
                      void* hip_stream) {
  if (!theta || !m || !v || !grad16 || !param16) return fail(AXONN_EINVAL, "adam_bucket: null argument");
  if (n == 0) return fail(AXONN_EINVAL, "adam_bucket: n == 0");
  if (step < 1) return fail(AXONN_EINVAL, "adam_bucket: step must be >= 1");
  if (!(beta1 >= 0. && beta1 < 1.) || !(beta2 >= 0. && beta2 < 1.))
    return fail(AXONN_EINVAL, "adam_bucket: betas must be in [0,1)");
  return check_launch(launch_adam(n, theta, m, v, grad16, param16, lr, beta1, beta2, eps, weight_decay, step,
                                  grad_scale, (hipStream_t)hip_stream), "adam");
}

}  // extern "C"
