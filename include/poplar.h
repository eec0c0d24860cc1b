/*
 * poplar.h - C ABI of libpoplar: one rank's ZeRO training step on one MI355X
 * (gfx950), the per-stage step-time profile and the host-side batch allocator
 * of "Poplar: Efficient Scaling of Distributed DNN Training on Heterogeneous
 * GPU Clusters" (arXiv 2408.12596).
 *
 * General rules
 *  - Every function returns a poplar_status (0 = POPLAR_OK).  On failure
 *    poplar_last_error() gives a thread-local message.  No exception crosses
 *    this boundary.
 *  - "device" pointers are HIP device memory owned by the caller; the library
 *    never frees or keeps them beyond the call, except the ones handed over
 *    with poplar_bind_state (kept until rebinding or poplar_destroy).
 *    "host" pointers are ordinary host memory.
 *  - Device work is enqueued on the stream given to poplar_create and is
 *    asynchronous unless stated otherwise; the caller synchronises.
 *  - Matrices are row-major.  Every Linear weight is stored [out, in]
 *    (y = x W^T + b).  "lowp" is the compute dtype of the context
 *    (POPLAR_F32: float, POPLAR_BF16: bfloat16); gradients and optimizer state
 *    are always float.
 *  - Shape preconditions (checked, POPLAR_ERR_INVALID otherwise): hidden and
 *    ffn multiples of 8, hidden = n_head * head_dim with head_dim 64 or 128
 *    for POPLAR_BF16 (any even head_dim for POPLAR_F32), batch >= 1.
 *
 * Flat parameter order (the paper fixes none; Appendix "Details about ZeRO"
 * only says that the model states are split across ranks):
 *   GPT   layer: g1 b1 Wqkv[3H,H] bqkv Wo[H,H] bo g2 b2 W1[F,H] bm1 W2[H,F] bm2
 *         model: wte[V,H] wpe[S,H] layer0..L-1 gf bf        (LM head tied to wte)
 *   Llama layer: g1 Wqkv[3H,H] Wo[H,H] g2 Wg[F,H] Wu[F,H] Wd[H,F]
 *         model: wte[V,H] layer0..L-1 gf Whead[V,H]
 *   Wqkv rows: all q, all k, all v; head h owns rows h*d..(h+1)*d of each third.
 */
#ifndef POPLAR_H
#define POPLAR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  POPLAR_OK = 0,
  POPLAR_ERR_INVALID = -1,       /* bad argument or shape */
  POPLAR_ERR_OOM = -2,           /* emulated memory cap (or workspace) exceeded; nothing was launched */
  POPLAR_ERR_HIP = -3,           /* a HIP runtime call failed */
  POPLAR_ERR_UNIMPLEMENTED = -4
} poplar_status;

enum { POPLAR_ARCH_GPT = 0, POPLAR_ARCH_LLAMA = 1 };
enum { POPLAR_F32 = 0, POPLAR_BF16 = 1 };

/* Tensor ids for poplar_param_offset.  Layer tensors need 0 <= layer < n_layer;
 * model tensors (WTE..WHEAD) ignore `layer`. */
enum {
  POPLAR_T_G1 = 0, POPLAR_T_B1, POPLAR_T_WQKV, POPLAR_T_BQKV, POPLAR_T_WO, POPLAR_T_BO,
  POPLAR_T_G2, POPLAR_T_B2, POPLAR_T_W1, POPLAR_T_BM1, POPLAR_T_W2, POPLAR_T_BM2, /* GPT: W1/W2; Llama: W1 = Wg|Wu as [2F,H], W2 = Wd */
  POPLAR_T_WTE = 100, POPLAR_T_WPE, POPLAR_T_GF, POPLAR_T_BF, POPLAR_T_WHEAD
};

typedef struct poplar_model_cfg {
  int32_t arch;        /* POPLAR_ARCH_* */
  int32_t n_layer;     /* L */
  int32_t hidden;      /* H */
  int32_t n_head;      /* nh; head_dim d = H / nh */
  int32_t ffn;         /* F */
  int32_t seq;         /* S: every sample has exactly S tokens */
  int32_t vocab;       /* V */
  int32_t dtype;       /* POPLAR_F32 or POPLAR_BF16: compute dtype */
  int32_t world;       /* N: simulated ZeRO world size */
  int32_t rank;        /* r in [0, N) */
  int32_t zero_stage;  /* 0..3, default stage of the context */
  int32_t causal;      /* 1: causal mask (decoder) */
  int64_t cap_bytes;   /* emulated device memory in bytes, 0 = no cap */
  int32_t checkpoint;  /* 1: whole steps keep one activation stash instead of L and run every layer's forward pass
                          again inside the backward pass (a memory-for-compute knob next to the ZeRO stage: Section
                          "Heterogeneity Aware" only asks for the largest batch that fits) */
  int32_t deterministic; /* 1: every sum is taken in a fixed order, so that a step repeated on the same inputs gives the
                          same bits: the embedding-matrix gradient is summed token by token in sequence order instead
                          of with float atomics, and no GEMM splits its contraction over atomics (splits into halves
                          with a separate sum are kept).  Slower for small batches; off by default */
} poplar_model_cfg;

typedef struct poplar_ctx poplar_ctx;

/* Thread-local text of the last error on this thread ("" if none). host. */
const char* poplar_last_error(void);

/* Create a context.  `hip_stream` is a hipStream_t (NULL = default stream);
 * all device work of this context goes there.  The context owns only small
 * host state and a few hipEvents.  Fails with POPLAR_ERR_INVALID on shapes
 * outside the preconditions above. */
int poplar_create(const poplar_model_cfg* cfg, void* hip_stream, poplar_ctx** out);
int poplar_destroy(poplar_ctx* ctx);

/* ---- layout and shard arithmetic (host only, integers) ------------------- */

/* Elements in one layer block / in the whole model, in the flat order above. */
int poplar_layer_param_count(const poplar_model_cfg* cfg, int64_t* count);
int poplar_model_param_count(const poplar_model_cfg* cfg, int64_t* count);

/* Offset (in elements, from the start of the whole flat vector) and shape of
 * one tensor.  1-D tensors report cols = 1.  Tensors the architecture lacks
 * give POPLAR_ERR_INVALID. */
int poplar_param_offset(const poplar_model_cfg* cfg, int32_t layer, int32_t tensor_id,
                        int64_t* offset, int64_t* rows, int64_t* cols);

/* ZeRO partition of a flat vector of P elements over N ranks (Appendix
 * "Details about ZeRO": model states are split across all GPUs).  Contiguous
 * shards of len = ceil(P/N); rank r owns [off, off+len), of which `valid`
 * elements lie inside [0, P) and the rest is zero padding. */
int poplar_shard_range(int64_t P, int32_t N, int32_t r, int64_t* off, int64_t* len, int64_t* valid);

/* ---- one decoder layer (Algorithm 1's model.step is built from these) ---- */

/* Bytes of the activation stash one layer keeps between forward and backward
 * at local batch B, and of the scratch workspace poplar_layer_fwd/bwd need. */
int poplar_layer_saved_bytes(const poplar_model_cfg* cfg, int32_t B, int64_t* bytes);
int poplar_layer_workspace_bytes(const poplar_model_cfg* cfg, int32_t B, int64_t* bytes);

/* Forward of one pre-norm decoder layer at local batch B:
 *   GPT  : a = LN(x); qkv = a Wqkv^T + bqkv; o = causal softmax(q k^T / sqrt d) v;
 *          x1 = x + o Wo^T + bo; m = LN(x1); out = x1 + GeLU_tanh(m W1^T + bm1) W2^T + bm2
 *   Llama: RMSNorm, no biases, RoPE(base 10000) on q and k, SwiGLU MLP.
 * x_in, x_out: device lowp [B*S, H] (may not alias).  params: device lowp, the
 * layer's block in flat order.  saved: device, poplar_layer_saved_bytes bytes,
 * written here and read by poplar_layer_bwd.  workspace: device scratch of at
 * least poplar_layer_workspace_bytes (POPLAR_ERR_OOM if smaller). */
int poplar_layer_fwd(poplar_ctx* ctx, int32_t B, const void* x_in, const void* params,
                     void* x_out, void* saved, void* workspace, int64_t workspace_bytes);

/* Backward of the same layer.  dy: device lowp [B*S, H] (gradient of x_out);
 * dx: device lowp [B*S, H] (gradient of x_in; may alias dy).  grads: device
 * float, the layer's block in flat order; accumulate = 0 overwrites it,
 * 1 adds to it (gradient accumulation over micro-steps). */
int poplar_layer_bwd(poplar_ctx* ctx, int32_t B, const void* x_in, const void* dy, const void* params,
                     const void* saved, void* dx, float* grads, int32_t accumulate,
                     void* workspace, int64_t workspace_bytes);

/* poplar_layer_bwd for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments and results as poplar_layer_bwd without the
 * workspace pair: the scratch the pass needs (poplar_layer_workspace_bytes)
 * lives in an array inside the library's code object, poplar_static_scratch_bytes
 * (64 MiB) on every GPU the library runs on, held until the process ends.  A
 * batch whose scratch does not fit is refused with POPLAR_ERR_INVALID before
 * anything is launched (GPT-2-small's layer fits at local batch 1).  The call
 * allocates nothing, on the device or through any library.  All calls on one GPU
 * share that GPU's array: calls that overlap there (two streams, two threads)
 * race; calls in stream order on one stream do not.  Nothing needs clearing
 * between calls: every part of the scratch is written before it is read. */
int poplar_layer_bwd_static(poplar_ctx* ctx, int32_t B, const void* x_in, const void* dy, const void* params,
                            const void* saved, void* dx, float* grads, int32_t accumulate);
int poplar_static_scratch_bytes(int64_t* bytes);

/* The projection GEMM the layer is built from, on its own (lowp inputs, float
 * accumulation): the three operand layouts of a Linear layer y = x W^T,
 *   POPLAR_GEMM_NT  C[M,N] = A[M,K] B[N,K]^T      (forward)
 *   POPLAR_GEMM_NN  C[M,N] = A[M,K] B[K,N]        (input gradient dx = dy W)
 *   POPLAR_GEMM_TN  C[M,N] = A[K,M]^T B[K,N]      (weight gradient dW = dy^T x)
 * A, B: device lowp, row-major with strides lda, ldb (elements).  C: device,
 * lowp, or float when c_float = 1 (then C = A.B + beta C, beta 0 or 1).
 * POPLAR_BF16 needs 16-byte aligned pointers, strides that are multiples of 8
 * and at least the contiguous dimension rounded up to 8 (the padding of the
 * reduction dimension must hold zeros). */
enum { POPLAR_GEMM_NT = 0, POPLAR_GEMM_NN = 1, POPLAR_GEMM_TN = 2 };
int poplar_gemm(poplar_ctx* ctx, int32_t layout, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_float, float beta);

/* ---- embedding, head and loss --------------------------------------------- */

/* x[b,s,:] = wte[tok[b,s],:] (+ wpe[s,:] for GPT).  tokens: device int32 [B,S]
 * with ids in [0,V); an id outside that range embeds as a zero row and
 * receives no gradient (the table is never indexed with it).  wpe may be
 * NULL for Llama. */
int poplar_embed_fwd(poplar_ctx* ctx, int32_t B, const int32_t* tokens, const void* wte, const void* wpe, void* x);

/* dwte[tok[b,s],:] += dx[b,s,:] (float atomics, summation order not fixed; in sequence order when the context
 * was created with cfg.deterministic = 1),
 * dwpe[s,:] (+)= sum_b dx[b,s,:].  With accumulate = 0 dwpe is overwritten but
 * dwte is still added to (the tied LM head wrote it first); zero it yourself
 * when there is no tied head. */
int poplar_embed_bwd(poplar_ctx* ctx, int32_t B, const int32_t* tokens, const void* dx,
                     float* dwte, float* dwpe, int32_t accumulate);

int poplar_head_workspace_bytes(const poplar_model_cfg* cfg, int32_t B, int64_t* bytes);

/* Final norm, LM head, cross-entropy and their backward in one call:
 *   hf = Norm(x; gf[,bf]); logits = hf Whead^T;
 *   loss = loss_scale * sum_t CE(logits_t, targets_t)   (device float scalar, overwritten)
 *   dx = d loss / d x; d_gf, d_bf, d_whead (+)= parameter gradients (float).
 * loss_scale is explicit because ranks with unequal local batches must all use
 * 1 / (global tokens) for the summed gradient to be the global mean (the paper
 * keeps the global batch fixed and the local batch dynamic, Section "Offline
 * Analyzing of Configuration").  targets: device int32 [B*S], each in [0, V), or
 * negative for a position that is not predicted (a masked-language-model
 * batch scores only its masked positions): such a position adds nothing to
 * the loss and its gradient is zero.  A value of V or more is treated the
 * same way (no memory outside the row is read). */
int poplar_head_loss_fwd_bwd(poplar_ctx* ctx, int32_t B, const void* x, const int32_t* targets,
                             const void* gf, const void* bf, const void* whead, float loss_scale,
                             float* loss, void* dx, float* d_gf, float* d_bf, float* d_whead,
                             int32_t accumulate, void* workspace, int64_t workspace_bytes);

/* ---- sharded optimizer and the single-rank share of the collectives ------- */

/* Adam on one ZeRO shard (Appendix "Details about ZeRO", stage 1: each rank
 * updates only its partition of the optimizer states).  For i in [0, len):
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 *   p -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
 * in IEEE float, in place on p32, m, v (device float [len]); g: device float
 * [len]; p_lowp: device lowp [len] or NULL, receives the rounded new p
 * (round-to-nearest-even).  step_t counts from 1.  No weight decay. */
int poplar_adam_shard(poplar_ctx* ctx, float* p32, float* m, float* v, const float* g, void* p_lowp,
                      int64_t len, int32_t step_t, float lr, float b1, float b2, float eps);

/* ZeRO-2: this rank's own term of the gradient reduce-scatter.  g_unit holds
 * the full gradient of flat range [unit_lo, unit_hi) (device float); the part
 * that falls inside this rank's shard [shard_off, shard_off+shard_len) is added
 * into gshard (device float [shard_len]).  Peers' terms and the wire are not
 * part of a one-GPU build. */
int poplar_zero2_reduce_local(poplar_ctx* ctx, float* gshard, const float* g_unit,
                              int64_t unit_lo, int64_t unit_hi, int64_t shard_off, int64_t shard_len);

/* ZeRO-3: materialise flat range [lo, hi) of the lowp parameters before a
 * layer runs: elements inside this rank's shard come from own_shard (device
 * lowp [shard_len]), all others from peers (device lowp, indexed by flat
 * position; stands in for what the all-gather would deliver).  out: device lowp
 * [hi-lo]. */
int poplar_zero3_gather_local(poplar_ctx* ctx, void* out, const void* own_shard, const void* peers,
                              int64_t lo, int64_t hi, int64_t shard_off, int64_t shard_len);

/* ---- whole step, profile and search ---------------------------------------- */

/* Device buffers of one rank's training state, bound to a context for
 * poplar_profile_step / poplar_search_mbs.  All stay owned by the caller.
 * `len` below is the shard length of the stage that runs: ceil(P / world) at
 * stages 1-3, but P at stage 0, where every rank keeps the whole optimizer
 * (Appendix "Details about ZeRO": stage 0 duplicates all model states).  The
 * three *_len fields say how many elements the caller really allocated; a
 * step at a stage that needs more is refused with POPLAR_ERR_INVALID before
 * anything is launched. */
typedef struct poplar_state {
  void*    params;       /* lowp [P]: full compute copy (stages 0-2); at stage 3 it plays the peers' stand-in */
  void*    own_shard;    /* lowp [len]: stage 3 only, this rank's parameter shard (else NULL) */
  float*   master;       /* float [len]: master parameters of the shard */
  float*   m;            /* float [len] */
  float*   v;            /* float [len] */
  float*   grads;        /* stage 0/1: float [P]; stage 2/3: float [len] shard buffer */
  int64_t  master_len;   /* elements in each of master, m, v (>= 1) */
  int64_t  grads_len;    /* elements in grads (>= 1) */
  int64_t  own_len;      /* elements in own_shard (0 when it is NULL) */
  const int32_t* tokens; /* int32 [max_batch, S+1]; inputs [:, :S], targets [:, 1:] */
  int32_t  max_batch;
  void*    workspace;    /* activations, logits, staging: poplar_step_workspace_bytes (may be NULL, with 0 bytes, when
                            memory hooks supply the workspace of every step) */
  int64_t  workspace_bytes;
  float*   loss;         /* device float scalar */
  int32_t  adam_t;       /* step counter passed to Adam */
  float    lr, beta1, beta2, eps;
  const int32_t* targets; /* NULL: next-token targets tokens[:, 1:].  Else int32 [max_batch, S] targets of their own
                             (negative = position not predicted), e.g. the masked positions of a bidirectional model */
} poplar_state;

int poplar_bind_state(poplar_ctx* ctx, const poplar_state* st);

/* Workspace bytes a whole step needs at (stage, B), and the bytes a real rank
 * would hold at that point (model states of the stage + activations +
 * staging), which is what the emulated cap is compared with.  Both are affine
 * in B (Section "Heterogeneity Aware": memory is linear in the batch size). */
int poplar_step_workspace_bytes(const poplar_model_cfg* cfg, int32_t stage, int32_t B, int64_t* bytes);
/* Workspace bytes of the forward pass alone: what Algorithm 1's memory probe at batch 1 allocates through the
 * memory hooks (always below poplar_step_workspace_bytes of the same stage and batch). */
int poplar_step_forward_bytes(const poplar_model_cfg* cfg, int32_t stage, int32_t B, int64_t* bytes);
int poplar_step_accounted_bytes(const poplar_model_cfg* cfg, int32_t stage, int32_t B, int32_t forward_only, int64_t* bytes);

typedef struct poplar_profile {
  int32_t stage, batch;
  double t_fwd, t_bwd;          /* seconds, including the stand-ins below */
  double t_gather_fwd;          /* stage 3: parameter gather stand-in inside forward */
  double t_gather_bwd;          /* stage 3: same inside backward */
  double t_reduce_bwd;          /* stage 2/3: local gradient reduce inside backward */
  double t_adam;                /* optimizer on the shard */
  double t_consumed;            /* TimeConsumedDuringStep of the stage */
  int64_t accounted_bytes;      /* poplar_step_accounted_bytes(stage, batch) */
  double flops;                 /* algorithmic flop of forward + backward */
  float loss;
  /* filled only after poplar_set_kernel_timing: every selected GEMM / attention
   * launch of the step carries two events on the context's stream */
  double t_gemm, gemm_flops;    /* summed launch durations (s) and algorithmic flop 2*M*N*K of the GEMM launches */
  double t_attn, attn_flops;    /* same for the attention kernels: 2 S^2 H fwd, 5 S^2 H bwd per sample (causal) */
  int32_t n_gemm, n_attn;       /* launches counted */
  int64_t measured_bytes;       /* with memory hooks: what bytes_now() returned while the step's workspace was held; else 0 */
  int32_t n_gemm_kernels;       /* GEMM kernels inside the n_gemm timed spans (a grouped launch whose partial last round is cut
                                   off, or a product cut along N, is one span and two kernels) */
  int64_t reduce_elems;         /* stage 2/3: gradient elements the local reduces of the step added into the shard buffer (12 bytes
                                   of memory traffic each).  More than the shard's length where a tied embedding matrix lies in the
                                   shard: its head term and its embedding term are reduced one after the other. */
} poplar_profile;

/* What the current HIP device reports: compute units, the peak engine clock in
 * kHz, bytes of device memory.  Measurement reads the matrix-core peak off
 * these (4096 bf16 flop per clock per compute unit) next to the published
 * figure.  Any pointer may be NULL. */
int poplar_device_info(int32_t* compute_units, int32_t* clock_khz, int64_t* memory_bytes);

/* Kernel-level timing inside poplar_profile_step (off by default).  The paper
 * records wall time per step because no single operation explains it (Section
 * "Time Consumed Estimation"); this switch adds the per-kernel view needed to
 * place the GEMM and attention kernels against the matrix-core roofline. */
/* on: 0 none, 1 the GEMM launches, 2 the attention launches, 3 both (each timed
 * launch costs a few microseconds of step time); anything else ERR_INVALID. */
int poplar_set_kernel_timing(poplar_ctx* ctx, int32_t on);

/* How many runs stand behind one profile sample of poplar_profile_step and of
 * the searches: `warmup` untimed runs first, then `repeats` timed ones, of which
 * the run with the median TimeConsumedDuringStep is reported (the lower middle
 * one for an even count).  The default, 0 and 1, is the single run of Algorithm
 * 1; Appendix "Relationship Between Compute Capability and Batch Size" notes
 * that single runs fluctuate.  Every run is a real training step: the optimizer
 * state and the parameters advance once per run (adam_t stays as bound).
 * 0 <= warmup <= 64, 1 <= repeats <= 65. */
int poplar_set_sampling(poplar_ctx* ctx, int32_t warmup, int32_t repeats);

/* Memory by measurement instead of by accounting.  Algorithm 1 reads the
 * allocator before and after a forward pass and reacts to an out-of-memory
 * event; with these hooks the library does the same against the caller's
 * allocator.  While hooks are set, every step (poplar_profile_step,
 * poplar_accum_step, each step of the searches) asks `alloc` for its workspace
 * of poplar_step_workspace_bytes(stage, batch) bytes, runs in it and hands it
 * back through `release` after the stream has been synchronised; the bound
 * workspace and cfg.cap_bytes are not consulted.  alloc returning NULL is the
 * out-of-memory event: the call returns POPLAR_ERR_OOM with nothing launched
 * and the training state untouched (the searches take it as "this batch does
 * not fit").  poplar_search_mbs estimates the maximum from bytes_now() before
 * the forward workspace of one sample is allocated and while it is held, and
 * from bytes_total().  All four are called on the calling thread, between
 * launches; `user` is passed back untouched.  hooks = NULL removes them. */
typedef struct poplar_mem_hooks {
  void*   user;
  void*   (*alloc)(void* user, int64_t bytes);      /* device memory, 256-byte aligned, or NULL */
  void    (*release)(void* user, void* ptr);
  int64_t (*bytes_now)(void* user);                 /* bytes the allocator holds right now (CurrentMemoryAlloced) */
  int64_t (*bytes_total)(void* user);               /* bytes it may hold at most (TotalMemory) */
} poplar_mem_hooks;
int poplar_set_mem_hooks(poplar_ctx* ctx, const poplar_mem_hooks* hooks);

/* model.step(local_batch) of Algorithm 1 at a ZeRO stage, timed:
 * embedding, L layers, head and loss, backward, (stage 2/3) local gradient
 * reduce per unit, (stage 3) parameter gather per layer in both passes, Adam
 * on the shard.  Synchronises the stream.  t_consumed follows Section "Time
 * Consumed Estimation": stage 0/1 t_fwd + t_bwd; stage 2 t_fwd + t_bwd -
 * t_reduce_bwd; stage 3 additionally minus both gathers (the three are sums
 * of the stand-in kernels' own durations, start to end, taken by events that
 * ride on their launches; a unit that does not meet the shard launches
 * nothing and adds nothing).  Returns
 * POPLAR_ERR_OOM, with nothing launched and the state untouched, when the
 * accounted bytes exceed cfg.cap_bytes (the "find OOM error" of Algorithm 1)
 * or the bound workspace is too small. */
int poplar_profile_step(poplar_ctx* ctx, int32_t stage, int32_t local_batch, poplar_profile* out);

/* One optimizer step over an uneven run of micro-batches (Section "Optimal
 * Batch Size Searching": a device that was given gmbs samples runs gas - 1
 * micro-steps at its micro-batch size and a last one at lbs, Algorithm 2's
 * outputs): micro-step k runs forward and backward on micro_batch[k] samples,
 * the rows of the bound token buffer that follow those of micro-steps 0..k-1,
 * with the loss weighted 1 / (loss_batch * seq) per token, and adds its
 * gradients to those of the micro-steps before it (stage 0/1 in the flat
 * gradient buffer, stage 2/3 in the shard buffer through the local reduce);
 * Adam then runs once on the shard.  The result equals one step on the whole
 * run when loss_batch is the sum of micro_batch (up to rounding order).
 * micro_batch: host array of n_micro entries, each >= 1, their sum at most the
 * bound max_batch.  out: sums of the micro-steps' times, flops and losses;
 * batch = the sum; accounted_bytes = the largest micro-step's.  Errors as
 * poplar_profile_step, checked for every micro-batch before anything runs. */
int poplar_accum_step(poplar_ctx* ctx, int32_t stage, int32_t n_micro, const int32_t* micro_batch, int32_t loss_batch,
                      poplar_profile* out);

/* Algorithm 1 for this device: estimate mbs from the memory of one forward
 * pass at batch 1, run steps at 1, 2, 4, ... and then bisect to the largest
 * batch that fits.  samples: host array of max_samples entries, filled in call
 * order with the successful steps; *n_samples their count; *mbs = 0 means
 * batch 1 does not fit at this stage.  Each sample is a real step (see
 * poplar_set_sampling): the bound optimizer state and parameters advance by
 * one update per run, as they do when the paper's profiler calls model.step. */
int poplar_search_mbs(poplar_ctx* ctx, int32_t stage, int32_t* mbs,
                      poplar_profile* samples, int32_t max_samples, int32_t* n_samples);

/* Section "Heterogeneity Aware": when not even one sample fits at a ZeRO stage,
 * the search moves to the next stage, which holds less model state per device.
 * Runs poplar_search_mbs at first_stage, first_stage + 1, ... 3 and stops at the
 * first stage whose mbs is positive: *stage is that stage (-1 if none fits),
 * *mbs and the samples are that stage's.  The bound state must serve every
 * stage tried (gradient buffer of P floats; master, m and v of P floats when
 * first_stage is 0; own_shard for stage 3): a stage the state is too small for
 * ends the search with POPLAR_ERR_INVALID before anything of it runs. */
int poplar_search_stage(poplar_ctx* ctx, int32_t first_stage, int32_t* stage, int32_t* mbs,
                        poplar_profile* samples, int32_t max_samples, int32_t* n_samples);

/* ---- offline analysis (host only, double precision, deterministic) --------- */

typedef struct poplar_curve {
  int32_t n_pts;          /* >= 1 */
  const int32_t* batch;   /* host [n_pts], each in [1, ...] */
  const double* time;     /* host [n_pts], TimeConsumedDuringStep at that batch, > 0 */
  int32_t mbs;            /* largest batch the device can run (0 = none) */
} poplar_curve;

/* Communication one device does at a ZeRO stage, and its time on a link of
 * bytes_per_second per device (Appendix "Analysis of Experiments": a collective
 * over P elements moves P elements to each of the d devices, which gives the
 * 24 d h^2 of a feed-forward block at stage 3; Appendix "Details about ZeRO"
 * for which collectives each stage runs).  Per micro-step: stage 2 the
 * gradient reduce-scatter, stage 3 two parameter all-gathers and the
 * reduce-scatter.  Per optimizer step: stage 0 the gradient all-reduce (twice
 * P), stage 1 that and the parameter all-gather, stage 2 the parameter
 * all-gather.  A world of one moves nothing.  t_micro is the
 * time_communication Algorithm 2 adds to every accumulation step at stages 2
 * and 3.  Host only; any output pointer may be NULL. */
int poplar_comm_model(int64_t P, int32_t world, int32_t stage, double param_bytes, double grad_bytes, double bytes_per_second,
                      double* micro_bytes, double* step_bytes, double* total_micro_elements, double* t_micro, double* t_step);

/* Speed curve of one device (Section "Optimal Batch Size Searching"): speed
 * points batch/time, samples at equal batch averaged, natural cubic spline
 * (Appendix "Cubic Spline Interpolation") read at b = 1..mbs, clamped to the
 * end knots outside the sampled range and floored at 1e-9 of the largest knot.
 * speed: host [mbs+1], speed[0] = 0. */
int poplar_speed_curve(const poplar_curve* curve, double* speed);

typedef struct poplar_alloc {
  int32_t* gmbs;   /* host [n_dev]: samples per iteration for each device; sums to gbs */
  int32_t* b;      /* host [n_dev]: micro-batch */
  int32_t* gas;    /* host [n_dev]: accumulation steps (stage 2/3: same on every device) */
  int32_t* lbs;    /* host [n_dev]: batch of the last accumulation step */
  double T;        /* predicted iteration time: Eq. (1) with t_i = gmbs_i / speed_i for stage 0/1, wall time for 2/3 */
  double t;        /* stage 2/3: chosen per-micro-step time; stage 0/1: time_optimal */
  double T_steps;  /* stage 0/1: Eq. (1) with t_i read off device i's own curve for the steps it will run,
                      (gas_i - 1) time_i(b_i) + time_i(lbs_i), time_i(b) = b / speed_i(b): never below T, and above
                      it where lbs_i sits on the slow part of the curve.  Stage 2/3: equal to T */
} poplar_alloc;

/* Algorithm 2.  Stage 0/1: speed_i = max of the curve, time_optimal = gbs /
 * sum speed, gmbs_i = floor(time_optimal speed_i), each remaining sample to
 * argmin (gmbs_i + 1) / speed_i (lowest index on ties); micro-batch = largest
 * batch with speed >= peak_frac * max, capped by gmbs_i; gas_i = ceil(gmbs_i /
 * b_i); lbs_i = gmbs_i - (gas_i - 1) b_i.  Stage 2/3: for every distinct value
 * t of the (running-max) step-time curves, b_i = largest batch with time_i <= t,
 * gas = ceil(gbs / sum b_i), wall = (t + time_communication) gas; first strict
 * minimum wins; the last step's gbs - (gas-1) sum b_i samples go one at a time
 * to the device whose time after taking it is smallest.  Output arrays are
 * caller-allocated.  POPLAR_ERR_INVALID if no device can run one sample. */
int poplar_allocate(int32_t stage, int32_t n_dev, const poplar_curve* curves, int64_t gbs,
                    double time_communication, double peak_frac, poplar_alloc* out);

#ifdef __cplusplus
}
#endif
#endif /* POPLAR_H */
