// Entry points for one decoder layer, the embedding, the head + loss, the
// sharded optimizer and the single-rank share of the ZeRO collectives.
// Host orchestration only: every arithmetic step is a kernel launch.
#include "layer_plan.h"
#include <mutex>

int gemm(hipStream_t s, int dtype, const GemmArgs& a) {
  if (dtype == POPLAR_BF16) {
    // the direct-to-LDS kernel takes every shape inside its preconditions, the register-staged one the rest (K tails)
    const int r = gemm_bf16_dtl(s, a);
    return r == POPLAR_ERR_UNIMPLEMENTED ? gemm_bf16_mfma(s, a) : r;
  }
  return gemm_simple(s, dtype, a);
}

// Launch wrappers that, inside a profiled step with kernel timing on, time each GEMM / attention launch and
// note its algorithmic flop count.  The tuned kernels take the two events with the launch itself
// (hipExtLaunchKernelGGL: the events receive the kernel's own start and end, nothing is put between kernels);
// launches that go to another kernel are bracketed by two recorded events instead.
struct LaunchTimer {
  poplar_ctx* ctx;
  bool on;
  TimedLaunch tl;
  int64_t launched0 = 0;
  // hands out the two events, unrecorded
  int begin(int kind, double flops) {
    on = ((ctx->kernel_timing >> kind) & 1) && ctx->in_step;
    tl.a = nullptr; tl.b = nullptr;
    if (!on) return POPLAR_OK;
    tl.kind = kind; tl.flops = flops;
    launched0 = poplar_gemm_kernel_launches;
    POPLAR_TRY(ctx_take(ctx, &tl.a));
    return ctx_take(ctx, &tl.b);
  }
  int record_start() { return on ? (hipEventRecord(tl.a, ctx->stream) == hipSuccess ? POPLAR_OK : poplar_fail(POPLAR_ERR_HIP, "hipEventRecord")) : POPLAR_OK; }
  int record_stop() { return on ? (hipEventRecord(tl.b, ctx->stream) == hipSuccess ? POPLAR_OK : poplar_fail(POPLAR_ERR_HIP, "hipEventRecord")) : POPLAR_OK; }
  int done() {
    if (on) {
      tl.kernels = (int)(poplar_gemm_kernel_launches - launched0);
      ctx->launches.push_back(tl);
    }
    return POPLAR_OK;
  }
};
static int gemm(poplar_ctx* ctx, const GemmArgs& a0) {
  GemmArgs a = a0;
  a.no_atomics = ctx->cfg.deterministic;
  LaunchTimer t{ctx};
  POPLAR_TRY(t.begin(KIND_GEMM, 2.0 * (double)a.M * (double)a.N * (double)a.K));
  if (ctx->cfg.dtype == POPLAR_BF16) {
    GemmArgs b = a;
    b.ev_start = t.tl.a; b.ev_stop = t.tl.b;
    const int r = gemm_bf16_dtl(ctx->stream, b);
    if (r == POPLAR_OK) return t.done();
    if (r != POPLAR_ERR_UNIMPLEMENTED) return r;
  }
  if (a.a_rowsum) return poplar_fail(POPLAR_ERR_UNIMPLEMENTED, "row sums are produced by the direct-to-LDS GEMM only");
  POPLAR_TRY(t.record_start());
  POPLAR_TRY(ctx->cfg.dtype == POPLAR_BF16 ? gemm_bf16_mfma(ctx->stream, a) : gemm_simple(ctx->stream, ctx->cfg.dtype, a));
  POPLAR_TRY(t.record_stop());
  return t.done();
}

// Several independent GEMMs: one grouped launch where the direct-to-LDS kernel takes the group (the weight
// gradients of a layer: too few tiles each to fill the chip, enough together), one launch each otherwise.
static int gemm_group(poplar_ctx* ctx, const GemmArgs* a, int n) {
  if (ctx->cfg.dtype == POPLAR_BF16 && n > 1 && n <= 4) {
    double flops = 0.0;
    for (int i = 0; i < n; ++i) flops += 2.0 * (double)a[i].M * (double)a[i].N * (double)a[i].K;
    LaunchTimer t{ctx};
    POPLAR_TRY(t.begin(KIND_GEMM, flops));
    GemmArgs b[4];
    for (int i = 0; i < n; ++i) { b[i] = a[i]; b[i].no_atomics = ctx->cfg.deterministic; }
    b[0].ev_start = t.tl.a; b[0].ev_stop = t.tl.b;
    const int r = gemm_bf16_dtl_group(ctx->stream, b, n);
    if (r == POPLAR_OK) return t.done();
    if (r != POPLAR_ERR_UNIMPLEMENTED) return r;
    // nothing was launched: the two events handed out are simply not used
  }
  for (int i = 0; i < n; ++i) POPLAR_TRY(gemm(ctx, a[i]));
  return POPLAR_OK;
}

// algorithmic attention flop: 2 S^2 H forward and 5 S^2 H backward per sample under a causal mask, twice that without
static double attn_flops(const poplar_model_cfg& c, int B, double per_pair) {
  return per_pair * (c.causal ? 1.0 : 2.0) * (double)B * (double)c.seq * (double)c.seq * (double)c.hidden;
}
static int attn_fwd(poplar_ctx* ctx, int B, const void* qkv, void* o, float* lse) {
  const poplar_model_cfg& c = ctx->cfg;
  hipStream_t s = ctx->stream;
  const int d = c.hidden / c.n_head;
  LaunchTimer t{ctx};
  POPLAR_TRY(t.begin(KIND_ATTN, attn_flops(c, B, 2.0)));
  if (c.dtype == POPLAR_BF16) {
    POPLAR_TRY(attn_fwd_flash(s, B, c.seq, c.n_head, d, c.causal, qkv, o, lse, t.tl.a, t.tl.b));
    return t.done();
  }
  POPLAR_TRY(t.record_start());
  POPLAR_TRY(attn_fwd_simple(s, c.dtype, B, c.seq, c.n_head, d, c.causal, qkv, o, lse));
  POPLAR_TRY(t.record_stop());
  return t.done();
}
static int attn_bwd(poplar_ctx* ctx, int B, const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv,
                    float* delta) {
  const poplar_model_cfg& c = ctx->cfg;
  hipStream_t s = ctx->stream;
  const int d = c.hidden / c.n_head;
  LaunchTimer t{ctx};
  POPLAR_TRY(t.begin(KIND_ATTN, attn_flops(c, B, 5.0)));
  if (c.dtype == POPLAR_BF16) {
    POPLAR_TRY(attn_bwd_flash(s, B, c.seq, c.n_head, d, c.causal, qkv, o, dout, lse, dqkv, delta, t.tl.a, t.tl.b));
    return t.done();
  }
  POPLAR_TRY(t.record_start());
  POPLAR_TRY(attn_bwd_simple(s, c.dtype, B, c.seq, c.n_head, d, c.causal, qkv, o, dout, lse, dqkv, delta));
  POPLAR_TRY(t.record_stop());
  return t.done();
}

static GemmArgs gemm_args(int layout, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb,
                          void* C, int64_t ldc) {
  GemmArgs g;
  g.layout = layout; g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.c_float = 0; g.beta = 0.f; g.bias = nullptr; g.residual = nullptr; g.act = ACT_NONE; g.aux = nullptr; g.ldaux = 0;
  g.a_k_pad_zero = 0; g.ev_start = nullptr; g.ev_stop = nullptr; g.a_rowsum = nullptr; g.a_rowsum_accumulate = 0;
  return g;
}

SavedPlan saved_plan(const poplar_model_cfg& c, int B) {
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, F = c.ffn, es = elt_size(c.dtype);
  const int64_t hw = c.arch == POPLAR_ARCH_LLAMA ? 2 * F : F;
  SavedPlan p;
  int64_t at = 0;
  auto take = [&](int64_t bytes) { int64_t r = at; at += round_up(bytes, 256); return r; };
  p.stats1 = take(T * 2 * 4);
  p.a = take(T * H * es);
  p.qkv = take(T * 3 * H * es);
  p.o = take(T * H * es);
  p.lse = take((int64_t)B * c.n_head * c.seq * 4);
  p.x1 = take(T * H * es);
  p.stats2 = take(T * 2 * 4);
  p.m = take(T * H * es);
  p.h = take(T * hw * es);
  p.g = take(T * F * es);
  p.bytes = at;
  return p;
}

// The layer's backward pass keeps the partial sums of both norms and of the bias gradients until one
// reduction at its end finishes them all: two norm regions, then one for the grouped column sums.
static int64_t norm_scratch_floats(const poplar_model_cfg& c) { return (int64_t)768 * 2 * c.hidden; }   // <= 768 blocks x 2 x H
static int64_t colsum_scratch_floats(const poplar_model_cfg& c) {
  // chunks <= 2048 / strips + 1 and columns <= strips * 512: chunks x columns <= 2048 * 512 + columns
  return (int64_t)2048 * 512 + 5 * (int64_t)c.hidden + c.ffn;
}

int64_t scratch_floats(const poplar_model_cfg& c) {
  // norm backward: <= 768 blocks x 2 x H; column sums: <= (2048/strips + 1) chunks x N
  const int64_t H = c.hidden, F = c.ffn;
  const int64_t maxN = std::max<int64_t>(3 * H, 2 * F);
  const int64_t a = 768 * 2 * H;
  const int64_t b = 2048 * 64 * 8 + 2 * maxN;
  return std::max(a, b);
}

BwdPlan bwd_plan(const poplar_model_cfg& c, int B) {
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, F = c.ffn, es = elt_size(c.dtype);
  const bool llama = c.arch == POPLAR_ARCH_LLAMA;
  BwdPlan p;
  int64_t at = 0;
  auto take = [&](int64_t bytes) { int64_t r = at; at += round_up(bytes, 256); return r; };
  p.dh = take(T * (llama ? 2 * F : F) * es);
  p.dg = llama ? take(T * F * es) : -1;
  p.dm = take(T * H * es);
  p.dx1 = take(T * H * es);
  p.dob = take(T * H * es);
  p.dqkv = take(T * 3 * H * es);
  p.da = take(T * H * es);
  p.delta = take((int64_t)B * c.n_head * c.seq * 4);
  p.scratch = take((2 * norm_scratch_floats(c) + colsum_scratch_floats(c)) * 4);
  // bf16: room for the second half of each weight-gradient GEMM's sums (and of the bias gradient that rides on it)
  // when its contraction over the tokens is cut in two; in the order of the GEMMs: W2, W1 (or Wg | Wu), Wo, Wqkv
  const int64_t hw = llama ? 2 * F : F;
  const int64_t rows[4] = {H, hw, H, 3 * H}, cols[4] = {F, H, H, H};
  const int64_t before = at;
  for (int i = 0; i < 4; ++i) p.kpart[i] = c.dtype == POPLAR_BF16 ? take((rows[i] * cols[i] + rows[i]) * 4) : -1;
  p.kpart_bytes = at - before;
  p.bytes = at;
  return p;
}

extern "C" int poplar_layer_saved_bytes(const poplar_model_cfg* cfg, int32_t B, int64_t* bytes) {
  POPLAR_TRY(validate_cfg(cfg));
  if (B < 1 || !bytes) return poplar_fail(POPLAR_ERR_INVALID, "batch must be >= 1 and bytes non-null");
  *bytes = saved_plan(*cfg, B).bytes;
  return POPLAR_OK;
}

extern "C" int poplar_layer_workspace_bytes(const poplar_model_cfg* cfg, int32_t B, int64_t* bytes) {
  POPLAR_TRY(validate_cfg(cfg));
  if (B < 1 || !bytes) return poplar_fail(POPLAR_ERR_INVALID, "batch must be >= 1 and bytes non-null");
  *bytes = bwd_plan(*cfg, B).bytes;
  return POPLAR_OK;
}

static inline const char* at(const void* base, int64_t elems, int64_t es) { return (const char*)base + elems * es; }

int layer_fwd_impl(poplar_ctx* ctx, int B, const void* x_in, const void* params, void* x_out, void* saved) {
  const poplar_model_cfg& c = ctx->cfg;
  hipStream_t s = ctx->stream;
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, F = c.ffn, es = elt_size(c.dtype);
  const bool llama = c.arch == POPLAR_ARCH_LLAMA;
  const LayerOffsets lo = layer_offsets(c);
  const SavedPlan sp = saved_plan(c, B);
  char* sv = (char*)saved;
  auto P = [&](int64_t off) -> const void* { return off < 0 ? nullptr : at(params, off, es); };
  float* stats1 = (float*)(sv + sp.stats1);
  float* stats2 = (float*)(sv + sp.stats2);
  float* lse = (float*)(sv + sp.lse);
  void *a = sv + sp.a, *qkv = sv + sp.qkv, *o = sv + sp.o, *x1 = sv + sp.x1, *m = sv + sp.m, *h = sv + sp.h, *g = sv + sp.g;

  POPLAR_TRY(layernorm_fwd(s, c.dtype, T, (int)H, x_in, P(lo.g1), P(lo.b1), a, stats1, llama));
  GemmArgs ga = gemm_args(GEMM_NT, T, 3 * H, H, a, H, P(lo.wqkv), H, qkv, 3 * H);
  ga.bias = P(lo.bqkv);
  POPLAR_TRY(gemm(ctx, ga));
  if (llama) POPLAR_TRY(rope_inplace(s, c.dtype, B, c.seq, c.n_head, (int)(H / c.n_head), qkv, 3 * H, 1.0f));
  POPLAR_TRY(attn_fwd(ctx, B, qkv, o, lse));
  ga = gemm_args(GEMM_NT, T, H, H, o, H, P(lo.wo), H, x1, H);
  ga.bias = P(lo.bo); ga.residual = x_in;
  POPLAR_TRY(gemm(ctx, ga));
  POPLAR_TRY(layernorm_fwd(s, c.dtype, T, (int)H, x1, P(lo.g2), P(lo.b2), m, stats2, llama));
  if (llama) {
    ga = gemm_args(GEMM_NT, T, 2 * F, H, m, H, P(lo.w1), H, h, 2 * F);
    POPLAR_TRY(gemm(ctx, ga));
    POPLAR_TRY(swiglu_fwd(s, c.dtype, T, (int)F, h, g));
  } else {
    ga = gemm_args(GEMM_NT, T, F, H, m, H, P(lo.w1), H, g, F);
    ga.bias = P(lo.bm1); ga.act = ACT_GELU; ga.aux = h; ga.ldaux = F;
    POPLAR_TRY(gemm(ctx, ga));
  }
  ga = gemm_args(GEMM_NT, T, H, F, g, F, P(lo.w2), F, x_out, H);
  ga.bias = P(lo.bm2); ga.residual = x1;
  POPLAR_TRY(gemm(ctx, ga));
  return POPLAR_OK;
}

int layer_bwd_impl(poplar_ctx* ctx, int B, const void* x_in, const void* dy, const void* params, const void* saved, void* dx,
                   float* grads, int accumulate, void* workspace) {
  const poplar_model_cfg& c = ctx->cfg;
  hipStream_t s = ctx->stream;
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, F = c.ffn, es = elt_size(c.dtype);
  const bool llama = c.arch == POPLAR_ARCH_LLAMA;
  const int64_t hw = llama ? 2 * F : F;
  const LayerOffsets lo = layer_offsets(c);
  const SavedPlan sp = saved_plan(c, B);
  const BwdPlan bp = bwd_plan(c, B);
  const char* sv = (const char*)saved;
  char* ws = (char*)workspace;
  auto P = [&](int64_t off) -> const void* { return off < 0 ? nullptr : at(params, off, es); };
  auto G = [&](int64_t off) -> float* { return off < 0 ? nullptr : grads + off; };
  const float* stats1 = (const float*)(sv + sp.stats1);
  const float* stats2 = (const float*)(sv + sp.stats2);
  const float* lse = (const float*)(sv + sp.lse);
  const void *a = sv + sp.a, *qkv = sv + sp.qkv, *o = sv + sp.o, *x1 = sv + sp.x1, *m = sv + sp.m, *h = sv + sp.h, *g = sv + sp.g;
  void *dh = ws + bp.dh, *dm = ws + bp.dm, *dx1 = ws + bp.dx1, *dob = ws + bp.dob, *dqkv = ws + bp.dqkv, *da = ws + bp.da;
  float* delta = (float*)(ws + bp.delta);
  const int64_t norm_n = norm_scratch_floats(c), cs_n = colsum_scratch_floats(c);
  float *scratch_n2 = (float*)(ws + bp.scratch), *scratch_n1 = scratch_n2 + norm_n, *scratch_cs = scratch_n1 + norm_n;
  const float beta = accumulate ? 1.f : 0.f;
  GemmArgs ga;
  // Bias gradients = column sums of dy, dh, dx1, dqkv, each the transposed operand of a weight-gradient GEMM:
  // the direct-to-LDS GEMM forms them on the way (one more MFMA per fragment on its first column of tiles).
  // Where that kernel does not take the problems, one column-sum launch at the end covers them, when all four
  // matrices exist; its reductions and those of the two norms' gamma / beta gradients share one more launch.
  ColsumProblem cs[COLSUM_MAX_GROUP];
  int cs_dw[COLSUM_MAX_GROUP];   // the weight-gradient GEMM each belongs to
  int ncs = 0;
  ReduceJob jobs[REDUCE_MAX_JOBS];
  int njobs = 0;
  const bool dy_is_dx = dy == dx;   // allowed by the interface: dy is then gone at the end, so what reads it cannot wait

  // MLP down projection: out = x1 + g W2^T + bm2
  if (!llama && !dy_is_dx) { cs_dw[ncs] = 0; cs[ncs++] = ColsumProblem{dy, H, H, G(lo.bm2)}; }
  // the four weight-gradient GEMMs are collected and run as one group at the end: their operands (dy, dh,
  // dx1, dqkv and the stashed activations) all stay valid until then
  GemmArgs dw[4];
  dw[0] = gemm_args(GEMM_TN, H, F, T, dy, H, g, F, G(lo.w2), F);
  dw[0].c_float = 1; dw[0].beta = beta;
  if (dy_is_dx) {
    if (!llama) {
      if (c.dtype == POPLAR_BF16 && gemm_bf16_dtl_accepts(&dw[0], 1)) { dw[0].a_rowsum = G(lo.bm2); dw[0].a_rowsum_accumulate = accumulate; }
      else POPLAR_TRY(colsum(s, c.dtype, T, H, dy, H, G(lo.bm2), accumulate, scratch_cs, cs_n));
    }
    POPLAR_TRY(gemm(ctx, dw[0]));
  }
  if (llama) {
    void* dg = ws + bp.dg;
    ga = gemm_args(GEMM_NN, T, F, H, dy, H, P(lo.w2), F, dg, F);
    POPLAR_TRY(gemm(ctx, ga));
    POPLAR_TRY(swiglu_bwd(s, c.dtype, T, (int)F, dg, h, dh));
  } else {
    ga = gemm_args(GEMM_NN, T, F, H, dy, H, P(lo.w2), F, dh, F);
    ga.act = ACT_GELU_BWD; ga.aux = const_cast<void*>(h); ga.ldaux = F;
    POPLAR_TRY(gemm(ctx, ga));
    cs_dw[ncs] = 1; cs[ncs++] = ColsumProblem{dh, F, F, G(lo.bm1)};
  }
  // MLP up projection
  dw[1] = gemm_args(GEMM_TN, hw, H, T, dh, hw, m, H, G(lo.w1), H);
  ga = gemm_args(GEMM_NN, T, H, hw, dh, hw, P(lo.w1), H, dm, H);
  POPLAR_TRY(gemm(ctx, ga));
  // second norm; dx1 = dy + norm_bwd(dm)
  POPLAR_TRY(layernorm_bwd_partial(s, c.dtype, T, (int)H, dm, x1, P(lo.g2), stats2, dy, dx1, G(lo.g2), G(lo.b2), scratch_n2, norm_n, llama, &jobs[njobs++]));
  // attention output projection: x1 = x + o Wo^T + bo
  if (!llama) { cs_dw[ncs] = 2; cs[ncs++] = ColsumProblem{dx1, H, H, G(lo.bo)}; }
  dw[2] = gemm_args(GEMM_TN, H, H, T, dx1, H, o, H, G(lo.wo), H);
  ga = gemm_args(GEMM_NN, T, H, H, dx1, H, P(lo.wo), H, dob, H);
  POPLAR_TRY(gemm(ctx, ga));
  // attention
  POPLAR_TRY(attn_bwd(ctx, B, qkv, o, dob, lse, dqkv, delta));
  if (llama) POPLAR_TRY(rope_inplace(s, c.dtype, B, c.seq, c.n_head, (int)(H / c.n_head), dqkv, 3 * H, -1.0f));
  // QKV projection
  if (!llama) { cs_dw[ncs] = 3; cs[ncs++] = ColsumProblem{dqkv, 3 * H, 3 * H, G(lo.bqkv)}; }
  dw[3] = gemm_args(GEMM_TN, 3 * H, H, T, dqkv, 3 * H, a, H, G(lo.wqkv), H);
  ga = gemm_args(GEMM_NN, T, H, 3 * H, dqkv, 3 * H, P(lo.wqkv), H, da, H);
  POPLAR_TRY(gemm(ctx, ga));
  // first norm; dx = dx1 + norm_bwd(da)
  POPLAR_TRY(layernorm_bwd_partial(s, c.dtype, T, (int)H, da, x_in, P(lo.g1), stats1, dx1, dx, G(lo.g1), G(lo.b1), scratch_n1, norm_n, llama, &jobs[njobs++]));
  for (int i = 1; i < 4; ++i) { dw[i].c_float = 1; dw[i].beta = beta; }
  for (int i = 0; i < 4; ++i) dw[i].k_partial = bp.kpart[i] < 0 ? nullptr : (float*)(ws + bp.kpart[i]);
  GemmArgs* grp = dy_is_dx ? dw + 1 : dw;
  const int ngrp = dy_is_dx ? 3 : 4;
  if (ncs && c.dtype == POPLAR_BF16 && gemm_bf16_dtl_accepts(grp, ngrp)) {
    for (int i = 0; i < ncs; ++i) { dw[cs_dw[i]].a_rowsum = cs[i].out; dw[cs_dw[i]].a_rowsum_accumulate = accumulate; }
    ncs = 0;
  }
  if (ncs) {
    POPLAR_TRY(colsum_partial(s, c.dtype, T, cs, ncs, scratch_cs, cs_n, jobs + njobs));
    njobs += ncs;
  }
  POPLAR_TRY(reduce_group(s, jobs, njobs, accumulate));
  return gemm_group(ctx, grp, ngrp);
}

static int check_ctx_batch(poplar_ctx* ctx, int B) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (B < 1) return poplar_fail(POPLAR_ERR_INVALID, "batch must be >= 1, got %d", B);
  if ((int64_t)B * ctx->cfg.seq > (int64_t)1 << 24) return poplar_fail(POPLAR_ERR_INVALID, "batch * seq above 2^24 tokens");
  return POPLAR_OK;
}

extern "C" int poplar_layer_fwd(poplar_ctx* ctx, int32_t B, const void* x_in, const void* params, void* x_out, void* saved,
                                void* workspace, int64_t workspace_bytes) {
  POPLAR_TRY(check_ctx_batch(ctx, B));
  if (!x_in || !params || !x_out || !saved) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (x_in == x_out) return poplar_fail(POPLAR_ERR_INVALID, "x_in and x_out may not alias");
  (void)workspace; (void)workspace_bytes;  // the forward pass keeps everything it writes in `saved`
  return layer_fwd_impl(ctx, B, x_in, params, x_out, saved);
}

extern "C" int poplar_layer_bwd(poplar_ctx* ctx, int32_t B, const void* x_in, const void* dy, const void* params, const void* saved,
                                void* dx, float* grads, int32_t accumulate, void* workspace, int64_t workspace_bytes) {
  POPLAR_TRY(check_ctx_batch(ctx, B));
  if (!x_in || !dy || !params || !saved || !dx || !grads || !workspace) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (workspace_bytes < bwd_plan(ctx->cfg, B).bytes)
    return poplar_fail(POPLAR_ERR_OOM, "layer backward workspace: have %lld bytes, need %lld", (long long)workspace_bytes, (long long)bwd_plan(ctx->cfg, B).bytes);
  return layer_bwd_impl(ctx, B, x_in, dy, params, saved, dx, grads, accumulate, workspace);
}

// ---- the same backward pass for callers that cannot allocate -----------------
// Scratch of the no-allocation entry point: one array per GPU, loaded with the code object and held until the
// process ends.  Host code never uses the array's name as an address; it asks the runtime for the device address
// once per device (below) and passes that pointer on.
#define POPLAR_STATIC_SCRATCH_BYTES (64ll << 20)
static __device__ __align__(256) unsigned char scratch[POPLAR_STATIC_SCRATCH_BYTES];

#define POPLAR_MAX_DEVICES 64
static void* scratch_ptr[POPLAR_MAX_DEVICES];   // device address of `scratch` on each GPU, null until first asked for
static std::mutex scratch_mutex;

// Device address of this GPU's copy of the scratch array (the current device's: each GPU holds its own copy at
// its own address).
static int static_scratch(void** out) {
  int dev = -1;
  POPLAR_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= POPLAR_MAX_DEVICES) return poplar_fail(POPLAR_ERR_INVALID, "device %d outside the %d the static scratch serves", dev, POPLAR_MAX_DEVICES);
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    POPLAR_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return poplar_fail(POPLAR_ERR_HIP, "hipGetSymbolAddress gave a null address for the static scratch");
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return POPLAR_OK;
}

extern "C" int poplar_layer_bwd_static(poplar_ctx* ctx, int32_t B, const void* x_in, const void* dy, const void* params,
                                       const void* saved, void* dx, float* grads, int32_t accumulate) {
  POPLAR_TRY(check_ctx_batch(ctx, B));
  if (!x_in || !dy || !params || !saved || !dx || !grads) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  const int64_t need = bwd_plan(ctx->cfg, B).bytes;
  if (need > POPLAR_STATIC_SCRATCH_BYTES)
    return poplar_fail(POPLAR_ERR_INVALID, "layer backward at batch %d needs %lld bytes of scratch, the static scratch holds %lld: use poplar_layer_bwd with a workspace",
                       B, (long long)need, (long long)POPLAR_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  POPLAR_TRY(static_scratch(&ws));
  // every region of the workspace is written by this pass before it is read (partial sums, staged gradients, the
  // second halves of a cut contraction), so what an earlier call left behind needs no clearing
  return layer_bwd_impl(ctx, B, x_in, dy, params, saved, dx, grads, accumulate, ws);
}

extern "C" int poplar_static_scratch_bytes(int64_t* bytes) {
  if (!bytes) return poplar_fail(POPLAR_ERR_INVALID, "bytes is null");
  *bytes = POPLAR_STATIC_SCRATCH_BYTES;
  return POPLAR_OK;
}

extern "C" int poplar_gemm(poplar_ctx* ctx, int32_t layout, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                           const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_float, float beta) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (layout < GEMM_NT || layout > GEMM_TN) return poplar_fail(POPLAR_ERR_INVALID, "unknown GEMM layout %d", layout);
  if (M < 0 || N < 0 || K < 0 || lda < 1 || ldb < 1 || ldc < N) return poplar_fail(POPLAR_ERR_INVALID, "bad GEMM extents");
  if (M == 0 || N == 0) return POPLAR_OK;
  if (!A || !B || !C) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (beta != 0.f && !(c_float && beta == 1.f)) return poplar_fail(POPLAR_ERR_INVALID, "beta must be 0, or 1 with a float output");
  GemmArgs ga = gemm_args(layout, M, N, K, A, lda, B, ldb, C, ldc);
  ga.c_float = c_float ? 1 : 0; ga.beta = beta;
  return gemm(ctx, ga);
}

// ---- embedding -------------------------------------------------------------
extern "C" int poplar_embed_fwd(poplar_ctx* ctx, int32_t B, const int32_t* tokens, const void* wte, const void* wpe, void* x) {
  POPLAR_TRY(check_ctx_batch(ctx, B));
  const poplar_model_cfg& c = ctx->cfg;
  if (!tokens || !wte || !x) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (c.arch == POPLAR_ARCH_GPT && !wpe) return poplar_fail(POPLAR_ERR_INVALID, "GPT needs wpe");
  return embed_fwd(ctx->stream, c.dtype, B, c.seq, c.hidden, c.vocab, tokens, c.seq, wte, c.arch == POPLAR_ARCH_GPT ? wpe : nullptr, x);
}

extern "C" int poplar_embed_bwd(poplar_ctx* ctx, int32_t B, const int32_t* tokens, const void* dx, float* dwte, float* dwpe, int32_t accumulate) {
  POPLAR_TRY(check_ctx_batch(ctx, B));
  const poplar_model_cfg& c = ctx->cfg;
  if (!tokens || !dx || !dwte) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (c.arch == POPLAR_ARCH_GPT && !dwpe) return poplar_fail(POPLAR_ERR_INVALID, "GPT needs dwpe");
  return embed_bwd(ctx->stream, c.dtype, B, c.seq, c.hidden, c.vocab, tokens, c.seq, dx, dwte, c.arch == POPLAR_ARCH_GPT ? dwpe : nullptr, accumulate,
                   c.deterministic);
}

// ---- head + loss -----------------------------------------------------------
HeadPlan head_plan(const poplar_model_cfg& c, int B) {
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, es = elt_size(c.dtype);
  HeadPlan p;
  p.ldl = round_up(c.vocab, 128);
  int64_t at = 0;
  auto take = [&](int64_t bytes) { int64_t r = at; at += round_up(bytes, 256); return r; };
  p.hf = take(T * H * es);
  p.stats = take(T * 2 * 4);
  p.logits = take(T * p.ldl * es);
  p.row_loss = take(T * 4);
  p.dhf = take(T * H * es);
  // Few rows: the input gradient of the head is a small matrix behind a contraction over the whole vocabulary,
  // too few tiles to fill the chip.  It is then formed in float, which lets the GEMM split the vocabulary
  // between blocks, and cast afterwards.  The float copy is reserved at every batch (the workspace stays
  // affine in the batch) and used only at the small ones.
  p.dhf32 = take(T * H * 4);
  p.dhf_split = c.dtype == POPLAR_BF16 && cdiv(T, 256) * cdiv(H, 256) < 128;
  p.scratch = take(scratch_floats(c) * 4);
  p.bytes = at;
  return p;
}

extern "C" int poplar_head_workspace_bytes(const poplar_model_cfg* cfg, int32_t B, int64_t* bytes) {
  POPLAR_TRY(validate_cfg(cfg));
  if (B < 1 || !bytes) return poplar_fail(POPLAR_ERR_INVALID, "batch must be >= 1 and bytes non-null");
  *bytes = head_plan(*cfg, B).bytes;
  return POPLAR_OK;
}

int head_fwd_part(poplar_ctx* ctx, int B, const void* x, const int32_t* targets, int64_t tgt_ld, const void* gf, const void* bf,
                  const void* whead, float loss_scale, float* loss, void* workspace) {
  const poplar_model_cfg& c = ctx->cfg;
  hipStream_t s = ctx->stream;
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, V = c.vocab;
  const bool llama = c.arch == POPLAR_ARCH_LLAMA;
  const HeadPlan hp = head_plan(c, B);
  char* ws = (char*)workspace;
  void *hf = ws + hp.hf, *logits = ws + hp.logits;
  float *stats = (float*)(ws + hp.stats), *row_loss = (float*)(ws + hp.row_loss);
  POPLAR_TRY(layernorm_fwd(s, c.dtype, T, (int)H, x, gf, bf, hf, stats, llama));
  GemmArgs ga = gemm_args(GEMM_NT, T, V, H, hf, H, whead, H, logits, hp.ldl);
  POPLAR_TRY(gemm(ctx, ga));
  // the gradient of the logits replaces them in place; it belongs to the
  // forward half because it is one pass over the same rows
  POPLAR_TRY(xent_fwd_bwd(s, c.dtype, T, (int)V, hp.ldl, logits, targets, tgt_ld, c.seq, loss_scale, loss, row_loss));
  return POPLAR_OK;
}

int head_bwd_part(poplar_ctx* ctx, int B, const void* x, const void* gf, const void* whead, void* dx, float* d_gf, float* d_bf,
                  float* d_whead, int accumulate, void* workspace) {
  const poplar_model_cfg& c = ctx->cfg;
  hipStream_t s = ctx->stream;
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, V = c.vocab;
  const bool llama = c.arch == POPLAR_ARCH_LLAMA;
  const HeadPlan hp = head_plan(c, B);
  char* ws = (char*)workspace;
  void *hf = ws + hp.hf, *logits = ws + hp.logits, *dhf = ws + hp.dhf;
  float *stats = (float*)(ws + hp.stats), *scratch = (float*)(ws + hp.scratch);
  GemmArgs ga = gemm_args(GEMM_TN, V, H, T, logits, hp.ldl, hf, H, d_whead, H);
  ga.c_float = 1; ga.beta = accumulate ? 1.f : 0.f;
  POPLAR_TRY(gemm(ctx, ga));
  ga = gemm_args(GEMM_NN, T, H, V, logits, hp.ldl, whead, H, dhf, H);
  ga.a_k_pad_zero = 1;   // the loss kernel zeroed columns V .. ldl of every row
  if (hp.dhf_split) {
    ga.C = ws + hp.dhf32; ga.c_float = 1;
    POPLAR_TRY(gemm(ctx, ga));
    POPLAR_TRY(cast_f32_to_lowp(s, c.dtype, (const float*)(ws + hp.dhf32), dhf, T * H));
  } else {
    POPLAR_TRY(gemm(ctx, ga));
  }
  POPLAR_TRY(layernorm_bwd(s, c.dtype, T, (int)H, dhf, x, gf, stats, nullptr, dx, d_gf, d_bf, accumulate, scratch, scratch_floats(c), llama));
  return POPLAR_OK;
}

extern "C" int poplar_head_loss_fwd_bwd(poplar_ctx* ctx, int32_t B, const void* x, const int32_t* targets, const void* gf, const void* bf,
                                        const void* whead, float loss_scale, float* loss, void* dx, float* d_gf, float* d_bf,
                                        float* d_whead, int32_t accumulate, void* workspace, int64_t workspace_bytes) {
  POPLAR_TRY(check_ctx_batch(ctx, B));
  const poplar_model_cfg& c = ctx->cfg;
  if (!x || !targets || !gf || !whead || !loss || !dx || !d_gf || !d_whead || !workspace) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (c.arch == POPLAR_ARCH_GPT && (!bf || !d_bf)) return poplar_fail(POPLAR_ERR_INVALID, "GPT needs bf and d_bf");
  if (workspace_bytes < head_plan(c, B).bytes)
    return poplar_fail(POPLAR_ERR_OOM, "head workspace: have %lld bytes, need %lld", (long long)workspace_bytes, (long long)head_plan(c, B).bytes);
  POPLAR_TRY(head_fwd_part(ctx, B, x, targets, c.seq, gf, bf, whead, loss_scale, loss, workspace));
  return head_bwd_part(ctx, B, x, gf, whead, dx, d_gf, d_bf, d_whead, accumulate, workspace);
}

// ---- optimizer and collectives' local share ---------------------------------
extern "C" int poplar_adam_shard(poplar_ctx* ctx, float* p32, float* m, float* v, const float* g, void* p_lowp, int64_t len,
                                 int32_t step_t, float lr, float b1, float b2, float eps) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (len < 0 || step_t < 1) return poplar_fail(POPLAR_ERR_INVALID, "len must be >= 0 and step_t >= 1");
  if (len > 0 && (!p32 || !m || !v || !g)) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  if (!(b1 >= 0.f && b1 < 1.f && b2 >= 0.f && b2 < 1.f)) return poplar_fail(POPLAR_ERR_INVALID, "betas must be in [0, 1)");
  return adam_shard(ctx->stream, ctx->cfg.dtype, p32, m, v, g, p_lowp, len, step_t, lr, b1, b2, eps);
}

extern "C" int poplar_zero2_reduce_local(poplar_ctx* ctx, float* gshard, const float* g_unit, int64_t unit_lo, int64_t unit_hi,
                                         int64_t shard_off, int64_t shard_len) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (unit_lo < 0 || unit_hi < unit_lo || shard_off < 0 || shard_len < 0) return poplar_fail(POPLAR_ERR_INVALID, "bad ranges");
  if (unit_hi == unit_lo || shard_len == 0) return POPLAR_OK;
  if (!gshard || !g_unit) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  return zero2_reduce_local(ctx->stream, gshard, g_unit, unit_lo, unit_hi, shard_off, shard_len);
}

extern "C" int poplar_zero3_gather_local(poplar_ctx* ctx, void* out, const void* own_shard, const void* peers, int64_t lo, int64_t hi,
                                         int64_t shard_off, int64_t shard_len) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (lo < 0 || hi < lo || shard_off < 0 || shard_len < 0) return poplar_fail(POPLAR_ERR_INVALID, "bad ranges");
  if (hi == lo) return POPLAR_OK;
  if (!out || !own_shard || !peers) return poplar_fail(POPLAR_ERR_INVALID, "null device pointer");
  return zero3_gather_local(ctx->stream, ctx->cfg.dtype, out, own_shard, peers, lo, hi, shard_off, shard_len);
}
