/*
 * axonn_stage.h -- C ABI of libaxonn_stage.so (MI355X / gfx950 only).
 *
 * The per-GPU hot path of AxoNN (arXiv 2110.13005): one pipeline stage ("nn_shard",
 * Sec. 3.1 / Alg. 1) of pre-LayerNorm GPT transformer layers whose Forward(msg) /
 * Backward(msg) are driven by received messages (Alg. 2), followed by the stage's
 * mixed-precision Adam step whose fp32 master weights and moments live in host memory
 * and are streamed through HBM in buckets (Sec. 5.2).
 *
 * Conventions
 *  - Every function returns 0 (AXONN_OK) or a negative axonn_status; nothing throws or
 *    aborts.  axonn_last_error() gives a thread-local, library-owned message.
 *  - "dev" pointers are HIP device pointers, "host" pointers are host memory.  bf16 means
 *    bfloat16 bit patterns (uint16_t storage).  hip_stream arguments are hipStream_t
 *    passed as void* (NULL = the null stream).
 *  - All tensors are dense row-major.  Activations are [b, s, h] = [T, h] with T = b*s.
 *    Weights are [in, out].  Per (batch, head) attention operands are column slices of the
 *    packed qkv tensor [T, 3h]: columns [0,h) = Q, [h,2h) = K, [2h,3h) = V, head j owning
 *    columns j*d..(j+1)*d-1 of each third.
 *  - Unless stated otherwise a call only enqueues work on the given stream and returns;
 *    the caller keeps every buffer alive until that stream work has completed.
 *  - A handle may be used from one host thread at a time.
 */
#ifndef AXONN_STAGE_H
#define AXONN_STAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AXONN_OK = 0,
  AXONN_EINVAL = -1,       /* bad argument: null pointer, non-positive size, ...      */
  AXONN_ESTATE = -2,       /* call not allowed in the handle's current state           */
  AXONN_ENOMEM = -3,       /* device or host allocation failed                         */
  AXONN_EHIP = -4,         /* a HIP runtime call failed (message has the HIP error)    */
  AXONN_EUNSUPPORTED = -5  /* shape outside what the kernels support (message says why)*/
} axonn_status;

const char* axonn_last_error(void);

/* Pinned host memory (hipHostMalloc / hipHostFree) for the optimizer's master state. */
int axonn_pinned_alloc(void** host_out, uint64_t bytes);
int axonn_pinned_free(void* host);

/* ------------------------------------------------------------------------------------
 * Stage handle (Sec. 3.1: a contiguous subset of layers owned by one GPU).
 * ---------------------------------------------------------------------------------- */
typedef struct axonn_stage axonn_stage_t;

typedef struct {
  int32_t n_layers;        /* transformer layers in this stage                         */
  int32_t hidden;          /* h; multiple of 8                                         */
  int32_t n_heads;         /* a; head dim d = h / a: a multiple of 4, at most 192
                              (64 and 128 have kernels of their own; other sizes, such
                              as the 188 of the paper's Table 1, run on the next of 64 /
                              128 / 192 with the columns beyond d masked)              */
  int32_t ffn_hidden;      /* MLP width (4h in every benchmark shape); multiple of 8   */
  int32_t seq_len;         /* s                                                        */
  int32_t microbatch_size; /* b (Sec. 3.3: user-defined microbatch size); b*s % 8 == 0 */
  int32_t n_microbatches;  /* M: microbatches per batch                                */
  int32_t pipeline_limit;  /* max microbatches in flight (Sec. 3.3); 1..M              */
  float ln_eps;            /* LayerNorm epsilon (inside the root, biased variance)     */
  int32_t device;          /* HIP device ordinal                                       */
  int32_t grad_accum_fp32; /* 1: accumulate weight gradients over microbatches in an
                              fp32 shadow buffer, rounded once to bf16 after the M-th
                              backward; 0: accumulate directly in the bf16 gradient
                              buffer (the paper's 4*phi device footprint, Sec. 5.2)    */
  int32_t wgrad_group;     /* weight gradients are formed for groups of microbatches in
                              one contraction over all their tokens, not per microbatch:
                              a group is closed once this many backwards are pending
                              (0: only when a stash slot is needed or the batch ends)  */
  int32_t qkv_input_split; /* 1: the QKV projection consumes LayerNorm-1's output as the
                              sum of two bf16 numbers (value and rounding remainder) in
                              one contraction of length 2h, so that the bf16 rounding of
                              the LayerNorm output does not reach the attention logits
                              (for shapes with large logits, e.g. h = 10240 with N(0,0.02)
                              weights: without it the worst weight gradient of that shape is
                              3.4e-2 off the fp64 result, with it 2.6e-2; costs one more
                              QKV-sized GEMM per layer forward).  2: the same for the Q and K
                              thirds only, V from the rounded output as usual (two thirds of
                              the extra cost)                                              */
  int32_t ckpt_stride;     /* activation checkpointing (Sec. 5.1): 0 keeps every activation of
                              a microbatch in flight; ac > 0 (a factor of n_layers) keeps only
                              the inputs of layers 0, ac, 2ac, ... and Backward regenerates
                              each segment of ac layers from its kept input before it
                              differentiates it.  Weight gradients are then formed per
                              microbatch and segment, right after the segment's backward
                              chain (wgrad_group is ignored): the regenerated activations
                              live in shared buffers that the next segment overwrites      */
} axonn_stage_config;

/* Allocates bf16 parameters and gradients (flat buffers), pipeline_limit activation
 * stash slots (forward activations plus the output gradients of the linear maps, which
 * stay until the slot's weight gradients have been formed; with ckpt_stride = ac only
 * n_layers / ac kept layer inputs per slot, plus five shared activation buffers: two of
 * one layer for forward passes, three of ac layers for regeneration, cf. Eq. 1) and the
 * backward workspace on cfg->device.  Parameters are zero except
 * LayerNorm gains = 1; gradients are zero.  Synchronous. */
int axonn_stage_create(const axonn_stage_config* cfg, axonn_stage_t** out);
/* Waits for all work of the stage, then frees everything it owns.  Synchronous. */
int axonn_stage_destroy(axonn_stage_t* st);

/* Flat parameter layout.  The stage holds 12 tensors per layer, in this order:
 * ln1_g[h] ln1_b[h] w_qkv[h,3h] b_qkv[3h] w_o[h,h] b_o[h] ln2_g[h] ln2_b[h]
 * w_fc1[h,f] b_fc1[f] w_fc2[f,h] b_fc2[h]; tensor idx = layer*12 + position.
 * name is "layer<l>.<tensor>", library-owned.  offset is in elements. */
int axonn_stage_param_count(const axonn_stage_t* st, uint64_t* n_elements);
int axonn_stage_num_tensors(const axonn_stage_t* st, int32_t* n_tensors);
int axonn_stage_param_layout(const axonn_stage_t* st, int32_t idx, const char** name,
                             uint64_t* offset, int32_t* rank, int64_t dims[4]);
/* Borrowed device pointers to the flat bf16 buffers (param_count elements each). */
int axonn_stage_params(axonn_stage_t* st, void** dev_bf16);
int axonn_stage_grads(axonn_stage_t* st, void** dev_bf16);
/* Starts a new batch: the next backward overwrites the gradient accumulators instead of
 * adding to them (so no memory is cleared), and the per-batch microbatch count restarts.
 * Until that backward the gradient buffer still holds the previous batch's gradients. */
int axonn_stage_zero_grad(axonn_stage_t* st, void* hip_stream);
/* Device bytes the stage holds, by category (Sec. 5.2 accounting): [0] bf16 params,
 * [1] bf16 grads, [2] fp32 grad shadow (0 unless grad_accum_fp32), [3] activation stash,
 * [4] backward workspace (with ckpt_stride: including the shared activation buffers),
 * [5] optimizer bucket buffers (0 until attached). */
int axonn_stage_device_bytes(const axonn_stage_t* st, uint64_t bytes[6]);

/* Forward(msg) of Alg. 2: runs the stage's layers on microbatch mb_id.
 * x_dev_bf16 [b,s,h] is read (and copied into the stash, so the caller may recycle its
 * receive buffer once the stream work is done); y_dev_bf16 [b,s,h] is written.
 * AXONN_ESTATE if mb_id is already in flight or pipeline_limit microbatches are. */
int axonn_stage_forward(axonn_stage_t* st, int32_t mb_id, const void* x_dev_bf16,
                        void* y_dev_bf16, void* hip_stream);
/* Backward(msg) of Alg. 2: given dL/dy for microbatch mb_id, writes dL/dx to
 * dx_dev_bf16 [b,s,h] (dy is copied, so the caller may recycle its receive buffer), adds
 * the bias and LayerNorm gradients into the accumulators and leaves the microbatch's
 * weight gradients pending (see wgrad_group); the microbatch no longer counts as in
 * flight.  AXONN_ESTATE if mb_id has no forward in flight.  After the n_microbatches-th
 * backward since the last zero_grad all pending weight gradients are formed and the bf16
 * gradient buffer is final on that stream; before that its contents are unspecified. */
int axonn_stage_backward(axonn_stage_t* st, int32_t mb_id, const void* dy_dev_bf16,
                         void* dx_dev_bf16, void* hip_stream);

/* Message-driven mode (steady-state loop of Alg. 2).  A message is what a neighbouring
 * pipeline stage would send: kind 0 comes from the previous stage (activations, triggers
 * Forward), kind 1 from the next stage (gradients w.r.t. this stage's output, triggers
 * Backward).  payload_dev is the [b,s,h] bf16 receive buffer, result_dev the [b,s,h]
 * bf16 buffer to send onwards; ready_event (hipEvent_t or NULL) is signalled when the
 * payload has arrived.  post() never blocks (a pre-posted receive, Sec. 4.1). */
typedef struct {
  int32_t kind;
  int32_t mb_id;
  const void* payload_dev;
  void* result_dev;
  void* ready_event;
  const void* targets_dev; /* last stage only (axonn_stage_attach_ends): int32 [b,s] target ids  */
  void* loss_dev;          /* last stage only: one float, the microbatch's pre-divided loss      */
  void* done_event;        /* hipEvent_t or NULL: recorded when the message's work is enqueued, it
                              fires once result_dev is complete -- the "Send(output)" of Alg. 2:
                              the neighbour's message for this microbatch takes it as ready_event */
} axonn_msg;
int axonn_stage_post(axonn_stage_t* st, const axonn_msg* msg);
/* Consumes posted messages until n_microbatches forwards and n_microbatches backwards
 * have been enqueued: repeatedly takes the first posted message whose payload has
 * arrived (event query) and that is admissible (forward: a stash slot is free; backward:
 * its forward was issued) and launches Forward or Backward for it.  Forwards go round
 * robin over n_streams-1 library streams, backwards to their own stream (n_streams = 1:
 * one stream for both); they start after everything already queued on hip_stream (use
 * axonn_stage_join to make hip_stream wait for them in turn).  Returns AXONN_ESTATE if messages remain but none can ever
 * become admissible.  Work is only enqueued; see axonn_stage_synchronize. */
int axonn_stage_run(axonn_stage_t* st, int32_t n_streams, void* hip_stream);
/* The same loop without blocking: dispatches the posted messages that are admissible and have
 * arrived right now and returns; n_dispatched (may be NULL) receives their number, n_remaining
 * (may be NULL) the number of messages the batch still expects.  One host thread can serve
 * several stages of a pipeline in turn with it, posting to a stage's neighbours what its
 * dispatch log shows as done (with the message's done_event as their ready_event). */
int axonn_stage_poll(axonn_stage_t* st, int32_t n_streams, void* hip_stream,
                     int32_t* n_dispatched, int32_t* n_remaining);
/* Limit, in seconds, of each wait of axonn_stage_run for the next message to arrive (default 120): counted from
 * the moment the loop finds nothing it can dispatch until it dispatches again, not from the start of the call.
 * When it expires, run returns AXONN_ESTATE; nothing is lost: posted messages stay posted, dispatched work stays
 * enqueued, and another axonn_stage_run resumes the batch (or synchronize and start over with zero_grad). */
int axonn_stage_set_message_wait(axonn_stage_t* st, double seconds);
/* Makes user_stream wait for everything the library streams have been given so far. */
int axonn_stage_join(axonn_stage_t* st, void* user_stream);
/* Blocks the host until all enqueued work of the stage is complete. */
int axonn_stage_synchronize(axonn_stage_t* st);
/* Order in which run() dispatched messages: entries are mb_id*2 + kind. */
int axonn_stage_dispatch_log(const axonn_stage_t* st, int32_t* out, int32_t capacity,
                             int32_t* n_written);

/* ------------------------------------------------------------------------------------
 * Offloaded, bucketed Adam (Sec. 5.2): only theta16 and grad16 live on the GPU; the fp32
 * master weights theta and the two Adam moments live in pinned host memory.  One step
 * fetches bucket after bucket (bucket_elems parameters) into reusable device buffers,
 * updates it and writes it back; H2D copy, update kernel and D2H copy of consecutive
 * buckets overlap on three streams.
 * Per element (Sec. 2.1 mixed precision; Kingma & Ba; decoupled decay):
 *   g = grad_scale * float(grad16);  m = b1*m + (1-b1)*g;  v = b2*v + (1-b2)*g*g
 *   theta -= lr * ( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + weight_decay*theta )
 *   theta16 = bf16_rne(theta)
 * Hyper-parameters are doubles: 1-b1, 1-b2 and the bias corrections are formed in double
 * on the host and rounded once to the kernel's float constants.
 * ---------------------------------------------------------------------------------- */
typedef struct axonn_offload_adam axonn_offload_adam_t;
/* n parameters; param16_dev / grad16_dev are caller-owned device bf16 arrays of n
 * elements; host_master / host_m / host_v are caller-owned PINNED host fp32 arrays of n
 * elements.  Allocates 3 sets of 3 fp32 device buffers of min(bucket_elems, n) elements.
 * bucket_elems must be a positive multiple of 8. */
int axonn_offload_adam_create(int32_t device, uint64_t n, uint64_t bucket_elems,
                              void* param16_dev, const void* grad16_dev,
                              float* host_master, float* host_m, float* host_v,
                              axonn_offload_adam_t** out);
int axonn_offload_adam_destroy(axonn_offload_adam_t* opt);
/* One full step (all buckets).  The work starts after everything already in hip_stream;
 * the call returns when the step is complete and the host arrays hold the new state (it
 * synchronizes hip_stream): a caller that ran ahead and queued its next batch behind a
 * pending step would fill the hardware queues that the step's copies share, which slows
 * the step by half.  step t >= 1.  If a HIP call fails in the middle of the step, the step's streams are drained
 * before the error is returned (nothing is in flight any more); the buckets processed up to then are updated, the
 * others untouched, and the message says how many. */
int axonn_offload_adam_step(axonn_offload_adam_t* opt, double lr, double beta1, double beta2,
                            double eps, double weight_decay, int64_t step, double grad_scale,
                            void* hip_stream);
int axonn_offload_adam_device_bytes(const axonn_offload_adam_t* opt, uint64_t* bytes);

/* The same, bound to a stage's own parameter and gradient buffers ("run the optimizer",
 * Alg. 1).  n must equal the stage's param_count.  step returns AXONN_ESTATE while
 * microbatches are in flight. */
int axonn_stage_optimizer_attach(axonn_stage_t* st, float* host_master, float* host_m,
                                 float* host_v, uint64_t n, uint64_t bucket_elems);
int axonn_stage_optimizer_step(axonn_stage_t* st, double lr, double beta1, double beta2,
                               double eps, double weight_decay, int64_t step,
                               double grad_scale, void* hip_stream);
/* The same step, started while the tail of the batch's backward work is still running (the
 * one-GPU counterpart of Sec. 5.3, where a chunk of k buckets enters the optimizer as soon
 * as its gradients have arrived).  Gradients become final layer by layer from the last
 * layer down while the batch's last microbatch passes through Backward; the buckets are
 * processed from the highest offset down in chunks of chunk_buckets (the paper's k), a
 * chunk's updates starting when the lowest layer it touches is final; the fetches of the
 * fp32 state do not wait for gradients at all (after a message-driven run with forward
 * streams the first ones are queued on a forward stream, which is idle once the batch's
 * forwards are through, so that they run during the backward work; those fetches are
 * ordered after the previous step, not after hip_stream: the host state must be in place
 * when the call is made).  Call it after the batch's last message has
 * been dispatched (axonn_stage_run has returned, or the n_microbatches-th
 * axonn_stage_backward) -- no axonn_stage_join is needed in between; AXONN_ESTATE before
 * that.  The call returns when the step is complete, which implies the batch is.
 * Results are identical to axonn_stage_optimizer_step's. */
int axonn_stage_optimizer_step_overlapped(axonn_stage_t* st, double lr, double beta1,
                                          double beta2, double eps, double weight_decay,
                                          int64_t step, double grad_scale,
                                          int32_t chunk_buckets, void* hip_stream);

/* ------------------------------------------------------------------------------------
 * Element type and loss scaling (Sec. 2, "Mixed precision": forward and backward run in half
 * precision; to keep small gradients from underflowing, the loss is multiplied by a scaling
 * factor, and the optimizer converts the half precision gradients to full precision and
 * descales them).  The library is built twice from the same sources: libaxonn_stage.so
 * computes with bfloat16 as its 16-bit element type, libaxonn_stage_fp16.so with IEEE half
 * precision (the paper's arithmetic).  Every "bf16" in the names and comments of this
 * header means "the 16-bit element type of the library at hand".  bfloat16 has fp32's range
 * and needs no loss scale; with half precision the scale matters.  The paper does not say how
 * the factor is chosen; the scaler here is the usual dynamic one (Micikevicius et al. 2018,
 * Sec. 3.2): a batch whose gradients contain an infinity or a NaN is dropped and the scale
 * multiplied by `backoff`; after `growth_interval` good batches in a row it is multiplied
 * by `growth`.
 * ---------------------------------------------------------------------------------- */

/* 0: bfloat16, 1: IEEE half precision. */
int32_t axonn_element_type(void);

typedef struct axonn_loss_scaler {
  float scale;              /* current loss scale S > 0 (the caller's initial value)       */
  float growth;             /* >= 1, e.g. 2                                                 */
  float backoff;            /* in (0, 1], e.g. 0.5                                          */
  int32_t growth_interval;  /* good batches in a row before the scale grows, >= 1           */
  int32_t good_steps;       /* good batches since the last change of the scale (state)      */
} axonn_loss_scaler;

/* Number of elements of x_dev[0..n) (device, 16-bit elements) that are infinite or NaN.
 * workspace_dev: 1025 64-bit counters of device memory, all overwritten; the count is left
 * in workspace_dev[1024].  Enqueued on hip_stream; no atomics, same result every run. */
int axonn_count_nonfinite(const void* x_dev, uint64_t n, uint64_t* workspace_dev,
                          void* hip_stream);

/* The same over the stage's gradient buffer, after the batch's gradients are final (the
 * ordering and state rules of axonn_stage_optimizer_step); *count_host (host) is valid on
 * return: the call synchronizes hip_stream. */
int axonn_stage_count_nonfinite_grads(axonn_stage_t* st, void* hip_stream,
                                      uint64_t* count_host);

/* Optimizer step under a dynamic loss scale.  The gradients of the batch were computed from a
 * loss multiplied by scaler->scale (the upstream gradients that reached this stage carried
 * it; a last stage sets it with axonn_head_set_loss_scale).  If the stage's gradients, or
 * those the caller checked elsewhere (other_nonfinite: the sum of the counts of the other
 * buffers that take part in the decision, 0 if none), contain a non-finite value: nothing
 * is updated, scaler->scale *= backoff, good_steps = 0, *skipped = 1.  Otherwise
 * axonn_stage_optimizer_step runs with grad_scale / scaler->scale, *skipped = 0, and after
 * growth_interval such steps in a row scaler->scale *= growth.  Synchronizes hip_stream once
 * (the decision is taken on the host).  AXONN_EINVAL for a scaler outside the ranges above. */
int axonn_stage_optimizer_step_scaled(axonn_stage_t* st, double lr, double beta1, double beta2,
                                      double eps, double weight_decay, int64_t step,
                                      double grad_scale, axonn_loss_scaler* scaler,
                                      uint64_t other_nonfinite, void* hip_stream,
                                      int32_t* skipped);

/* ------------------------------------------------------------------------------------
 * The two ends of the pipeline (the special cases of Alg. 2).  The first stage (i = 0)
 * turns a microbatch of token ids into activations: x[b,i,:] = wte[token[b,i],:] + wpe[i,:].
 * The last stage (i = G_inter - 1) applies a final LayerNorm and the LM head, computes the
 * token-mean cross-entropy divided by the number of microbatches of the batch (Sec. 4.2:
 * the loss is pre-divided, so that gradients summed over microbatches are those of the
 * batch mean) and starts Backward(1) at once.  The paper prints no equations for them;
 * these are the GPT ones, with a head matrix of its own ([h, V]; tying it to the token
 * table needs a collective between the first and the last GPU).  Vocabulary 51200 in the
 * paper's runs (Sec. 6.1); the head is the V/16lh term of Eq. 3.
 * Both objects own flat bf16 parameter and gradient buffers (embedding: wte[V,h] then
 * wpe[s,h]; head: lnf_g[h], lnf_b[h], w_head[h,V]; parameters start at zero, LayerNorm gain
 * at one) that axonn_offload_adam_create can be pointed at.  Gradients accumulate in bf16
 * over the calls since the last zero_grad (the first call overwrites).  Ids outside
 * [0, vocab) are clamped into range.  All calls enqueue on hip_stream.
 * ---------------------------------------------------------------------------------- */
typedef struct axonn_embed axonn_embed_t;
typedef struct axonn_head axonn_head_t;
/* hidden % 8 == 0. */
int axonn_embed_create(int32_t device, int32_t vocab, int32_t hidden, int32_t seq_len,
                       int32_t microbatch_size, axonn_embed_t** out);
int axonn_embed_destroy(axonn_embed_t* e);
/* Borrowed device pointers and the element count (vocab + seq_len) * hidden; any may be NULL. */
int axonn_embed_buffers(axonn_embed_t* e, void** params_dev_bf16, void** grads_dev_bf16,
                        uint64_t* n_elements);
int axonn_embed_zero_grad(axonn_embed_t* e);
/* tokens_dev: int32 [b,s] on the device; x_dev_bf16: [b,s,h] written. */
int axonn_embed_forward(axonn_embed_t* e, const int32_t* tokens_dev, void* x_dev_bf16,
                        void* hip_stream);
/* Adds the microbatch's table gradients: every use of a row adds its dx row (summed in
 * fp32 in token order, one writer per row: reproducible); dwpe[i,:] += sum_b dx[b,i,:]. */
int axonn_embed_backward(axonn_embed_t* e, const int32_t* tokens_dev, const void* dx_dev_bf16,
                         void* hip_stream);
/* hidden, vocab and tokens_per_microbatch (= b*s) multiples of 8.  Holds a [b*s, vocab]
 * bf16 logit buffer. */
int axonn_head_create(int32_t device, int32_t vocab, int32_t hidden,
                      int32_t tokens_per_microbatch, int32_t n_microbatches, float ln_eps,
                      axonn_head_t** out);
int axonn_head_destroy(axonn_head_t* hd);
int axonn_head_buffers(axonn_head_t* hd, void** params_dev_bf16, void** grads_dev_bf16,
                       uint64_t* n_elements);
int axonn_head_zero_grad(axonn_head_t* hd);
/* Forward, loss and Backward(1) of one microbatch: x_dev_bf16 [b,s,h] is the last layer's
 * output, targets_dev int32 [b,s]; loss_dev receives one float (mean token loss / number
 * of microbatches), dx_dev_bf16 [b,s,h] the gradient to run the stage's Backward on; the
 * head's gradients are accumulated. */
int axonn_head_forward_backward(axonn_head_t* hd, const void* x_dev_bf16,
                                const int32_t* targets_dev, float* loss_dev,
                                void* dx_dev_bf16, void* hip_stream);

/* Loss scale S of the last stage (default 1): dloss/dlogits, and with it every gradient of
 * the backward pass, is multiplied by S; the loss written to loss_dev is not.  Positive and
 * finite, else AXONN_EINVAL.  Takes effect from the next axonn_head_forward_backward. */
int axonn_head_set_loss_scale(axonn_head_t* head, float loss_scale);
/* Makes a stage the first and / or the last one of the pipeline (either handle may be NULL;
 * the handles stay the caller's).  In message-driven mode a forward message to a first
 * stage then carries int32 token ids [b,s] as payload (the buffer must stay valid until the
 * microbatch's backward has run) and its backward messages may leave result_dev NULL; a
 * forward message to a last stage carries targets_dev and loss_dev, is followed at once by
 * the loss and Backward, and result_dev receives the input gradient to send back; a last
 * stage accepts no backward messages.  axonn_stage_zero_grad also restarts the ends'
 * accumulation.  With ends attached axonn_stage_forward / _backward return AXONN_ESTATE.
 * Sizes must match the stage's (AXONN_EINVAL otherwise). */
int axonn_stage_attach_ends(axonn_stage_t* st, axonn_embed_t* embed, axonn_head_t* head);

/* ------------------------------------------------------------------------------------
 * Single operations of the layer (the kernels Forward/Backward are built from), exposed
 * so that each can be checked against the oracle on its own.  All pointers are device
 * pointers; all calls enqueue on hip_stream.
 * ---------------------------------------------------------------------------------- */

/* C[M,N] = epilogue( sum_k A(m,k) * B(n,k) ), bf16 operands, fp32 accumulation (MFMA).
 * a_kcontig: A(m,k) = A[m*lda + k], else A[k*lda + m]; b_kcontig likewise for B(n,k).
 * So a forward linear map y = x W is (a_kcontig=1, b_kcontig=0), its input gradient
 * dx = dy W^T is (1,1) and its weight gradient dW = x^T dy is (0,0).
 * M, N, K, lda, ldb, ldc (and ld_aux, ld_res) must be multiples of 8.
 * epilogue:
 *   0  C = bf16(acc + bias[n])                      bias may be NULL (treated as 0)
 *   1  C = bf16(acc + bias[n] + res[m,n])
 *   2  z = acc + bias[n];  C = bf16(GeLU(z));  aux = bf16(GeLU'(z))  (exact erf GeLU; the derivative is
 *      stored instead of z, from the unrounded z, so that the backward epilogue is a multiplication)
 *   3  C = bf16(acc * aux[m,n])                      aux = the derivative stored by epilogue 2
 *   4  C_f32 = (accumulate ? C_f32 : 0) + acc        C is float32
 *   5  C = bf16((accumulate ? float(C) : 0) + acc)
 */
int axonn_gemm_bf16(int32_t a_kcontig, int32_t b_kcontig, int32_t epilogue,
                    int64_t M, int64_t N, int64_t K,
                    const void* A, int64_t lda, const void* B, int64_t ldb,
                    void* C, int64_t ldc, const void* bias,
                    const void* res, int64_t ld_res, void* aux, int64_t ld_aux,
                    int32_t accumulate, void* hip_stream);

/* Weight gradient and bias gradient of a linear map in one call (Sec. 2: both are sums over the
 * tokens of the microbatches, of x^T dy and of dy): axonn_gemm_bf16 with (a_kcontig, b_kcontig) =
 * (0, 0) and epilogue 4 or 5, so C[M,N] (+)= sum_k A[k*lda + m] * B[k*ldb + n], and beside it
 *   colsum[n] = (accumulate ? colsum[n] : 0) + sum_k B[k*ldb + n],   n < N,
 * in C's element type (float32 for epilogue 4, bf16 for 5; sums in fp32, one rounding).  Problems of
 * at least 128 tiles of 256 x 256 form the sums inside the GEMM kernel, from the tiles of B it
 * multiplies (B is read once); smaller ones run axonn_colsum's kernels behind the GEMM.
 * workspace_f32: ceil(K/64)*N floats, needed either way.  Sizes as for axonn_gemm_bf16. */
int axonn_gemm_wgrad_colsum(int32_t epilogue, int64_t M, int64_t N, int64_t K,
                            const void* A, int64_t lda, const void* B, int64_t ldb,
                            void* C, int64_t ldc, void* colsum, float* workspace_f32,
                            int32_t accumulate, void* hip_stream);

/* Per-row LayerNorm over h (multiple of 8, <= 16384): out = g*(x-mean)*rstd + b, biased
 * variance, rstd = 1/sqrt(var+eps).  stats[T,2] float32 = (mean, rstd). */
int axonn_layernorm_fwd(int64_t T, int64_t h, const void* x_bf16, const void* gamma_bf16,
                        const void* beta_bf16, float eps, void* out_bf16, float* stats,
                        void* hip_stream);
/* dx = (res_grad ? res_grad : 0) + dLN(dout; x, stats, gamma);
 * dgamma_f32[h], dbeta_f32[h] are OVERWRITTEN with this call's column sums
 * sum_t dout*xhat and sum_t dout.  workspace_f32 needs 2*ceil(T/64)*h floats. */
int axonn_layernorm_bwd(int64_t T, int64_t h, const void* dout_bf16, const void* x_bf16,
                        const float* stats, const void* gamma_bf16, const void* res_grad_bf16,
                        void* dx_bf16, float* dgamma_f32, float* dbeta_f32,
                        float* workspace_f32, void* hip_stream);
/* axonn_layernorm_bwd for callers that cannot allocate device memory and have no workspace to
 * hand over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same kernels, same results, but the column partial sums go to a buffer that is part of the
 * library's own device image (AXONN_LAYERNORM_BWD_NOALLOC_MAX_FLOATS floats = 8 MiB, held on every
 * GPU the library runs on until the process ends).  The call allocates and frees nothing; its
 * first call on a device looks the buffer's address up.  AXONN_EUNSUPPORTED if
 * 2*ceil(T/64)*h exceeds the buffer (e.g. T = 4096 rows at h = 16384 still fit).  The device that
 * is current at the call is the one used.  All calls on one GPU share the one buffer: calls that
 * may overlap on the same GPU (different streams, different host threads) race; keep them on one
 * stream or order them with events.  Nothing needs clearing between calls. */
#define AXONN_LAYERNORM_BWD_NOALLOC_MAX_FLOATS (2u * 64u * 16384u)
int axonn_layernorm_bwd_noalloc(int64_t T, int64_t h, const void* dout_bf16, const void* x_bf16,
                                const float* stats, const void* gamma_bf16,
                                const void* res_grad_bf16, void* dx_bf16, float* dgamma_f32,
                                float* dbeta_f32, void* hip_stream);
/* out_f32[N] = sum_t y[t, n] over T rows (bias gradient).  workspace: ceil(T/64)*N floats. */
int axonn_colsum(int64_t T, int64_t N, const void* y_bf16, int64_t ldy, float* out_f32,
                 float* workspace_f32, void* hip_stream);

/* Causal self-attention over the packed qkv [b*s, 3h] (layout above); head dim a multiple
 * of 4, at most 192; h = n_heads * head_dim a multiple of 8.
 * o [b*s, h] bf16;  lse [b, a, s] float32 = log sum_j<=i exp(q_i.k_j / sqrt(d)). */
int axonn_attention_fwd(int32_t b, int32_t s, int32_t n_heads, int32_t head_dim,
                        const void* qkv_bf16, void* o_bf16, float* lse, void* hip_stream);
/* dqkv [b*s, 3h] bf16 from do [b*s, h]; delta_ws: b*a*s floats of scratch. */
int axonn_attention_bwd(int32_t b, int32_t s, int32_t n_heads, int32_t head_dim,
                        const void* qkv_bf16, const void* o_bf16, const float* lse,
                        const void* do_bf16, void* dqkv_bf16, float* delta_ws,
                        void* hip_stream);

/* Adam update of n elements resident on the device (one bucket's kernel, formula above).
 * theta/m/v float32 are updated in place; grad16 is read; param16 is written. */
int axonn_adam_bucket(uint64_t n, float* theta, float* m, float* v, const void* grad16,
                      void* param16, double lr, double beta1, double beta2, double eps,
                      double weight_decay, int64_t step, double grad_scale, void* hip_stream);

/* ------------------------------------------------------------------------------------
 * Launch timing (measurement aid, off by default).  While enabled, every kernel launch the
 * library makes is bracketed by a pair of HIP events on the stream it is launched on;
 * collect() waits for them, adds up elapsed milliseconds and launch counts per category
 * and clears the records.  Categories (num_categories of them, names by index): the three
 * GEMM layouts (the bias gradients come with the weight-gradient launches), attention
 * forward / backward, LayerNorm forward / backward (the backward with the reduction of its
 * gain and shift gradients), gradient conversion, Adam, input copy, embedding,
 * cross-entropy.  Process-wide, not thread-safe.  Intervals of kernels that overlap on different streams are each counted
 * in full.
 * ---------------------------------------------------------------------------------- */
int axonn_profile_enable(int32_t on);
int axonn_profile_num_categories(int32_t* n);
int axonn_profile_category_name(int32_t idx, const char** name);
int axonn_profile_collect(double* total_ms, int64_t* launches, int32_t n_categories);

/* Tuning and test hooks of the GEMM launcher; process-wide, not needed in normal use.  value -1 restores the
 * built-in rule.  AXONN_EINVAL for an unknown knob or a value out of range.
 *   AXONN_TUNE_GEMM_COPY_MASK      which problem classes take the large-problem kernel whose tiles are copied
 *                                  into LDS by the memory pipeline (instead of the register-staged one), as a bit
 *                                  mask: 1 input gradients, 2 forward, 4 weight gradients with a 16-bit result,
 *                                  8 weight gradients with an fp32 result (built-in: 7); it applies where K is a
 *                                  multiple of 64
 *   AXONN_TUNE_GEMM_BIG_MIN_TILES  number of 256 x 256 tiles from which the large-problem kernels are used
 *                                  (built-in: 128)
 *   AXONN_TUNE_GEMM_TILE_N         block width of the large-problem kernels: 160, 192 or 256 (0 or -1: chosen per
 *                                  problem) */
typedef enum {
  AXONN_TUNE_GEMM_COPY_MASK = 0,
  AXONN_TUNE_GEMM_BIG_MIN_TILES = 1,
  AXONN_TUNE_GEMM_TILE_N = 2
} axonn_tuning_knob;
int axonn_tuning(int32_t knob, int64_t value);

/* Bare copy rates of the host link (measurement aid): `reps` copies of `bytes` between pinned host memory and
 * device memory with hipMemcpyAsync, as the optimizer pipeline issues them.  gbps_out[0]: host to device alone,
 * [1]: device to host alone, [2]: per direction with both running at once (10^9 bytes per second).  Allocates and
 * frees its own buffers; synchronizes the device. */
int axonn_host_link_probe(int32_t device, uint64_t bytes, int32_t reps, double gbps_out[3]);

#ifdef __cplusplus
}
#endif
#endif /* AXONN_STAGE_H */
