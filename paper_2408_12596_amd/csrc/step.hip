// One rank's whole training step at a ZeRO stage, timed the way the paper's
// online profiling needs it (Section "Time Consumed Estimation"), the memory
// accounting behind the emulated cap, and the max-batch search of Algorithm 1.
#include "layer_plan.h"
#include <math.h>
#include <string.h>

extern "C" int poplar_create(const poplar_model_cfg* cfg, void* hip_stream, poplar_ctx** out) {
  POPLAR_TRY(validate_cfg(cfg));
  if (!out) return poplar_fail(POPLAR_ERR_INVALID, "out is null");
  poplar_ctx* c = new poplar_ctx();
  c->cfg = *cfg;
  c->stream = (hipStream_t)hip_stream;
  memset(&c->st, 0, sizeof c->st);
  c->bound = false;
  c->ev_next = 0;
  c->kernel_timing = 0;
  c->in_step = false;
  c->warmup = 0;
  c->repeats = 1;
  c->have_hooks = false;
  memset(&c->hooks, 0, sizeof c->hooks);
  *out = c;
  return POPLAR_OK;
}

extern "C" int poplar_destroy(poplar_ctx* ctx) {
  if (!ctx) return POPLAR_OK;
  for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
  delete ctx;
  return POPLAR_OK;
}

extern "C" int poplar_bind_state(poplar_ctx* ctx, const poplar_state* st) {
  if (!ctx || !st) return poplar_fail(POPLAR_ERR_INVALID, "null argument");
  if (!st->params || !st->master || !st->m || !st->v || !st->grads || !st->tokens || !st->loss)
    return poplar_fail(POPLAR_ERR_INVALID, "state has a null device pointer");
  if (!st->workspace && st->workspace_bytes != 0) return poplar_fail(POPLAR_ERR_INVALID, "null workspace with a size");
  if (st->max_batch < 1 || st->workspace_bytes < 0 || st->adam_t < 1) return poplar_fail(POPLAR_ERR_INVALID, "bad max_batch / workspace_bytes / adam_t");
  if (st->master_len < 1 || st->grads_len < 1 || st->own_len < 0 || (st->own_shard != nullptr) != (st->own_len > 0))
    return poplar_fail(POPLAR_ERR_INVALID, "state needs master_len >= 1, grads_len >= 1 and own_len > 0 exactly when own_shard is given");
  ctx->st = *st;
  ctx->bound = true;
  return POPLAR_OK;
}

// ---- units of the flat vector: embeddings | layer 0..L-1 | tail ------------
struct Units {
  int64_t P, emb_hi, layer0, lc, tail_lo, max_unit, tail_count;
};
static Units units_of(const poplar_model_cfg& c) {
  ModelOffsets mo = model_offsets(c);
  Units u;
  u.P = mo.count; u.emb_hi = mo.layer0; u.layer0 = mo.layer0; u.lc = mo.layer_count;
  u.tail_lo = mo.gf; u.tail_count = mo.count - mo.gf;
  u.max_unit = std::max(std::max(u.emb_hi, u.lc), u.tail_count);
  return u;
}

static void stage_shard(const poplar_model_cfg& c, int stage, int64_t P, int64_t* off, int64_t* len, int64_t* valid) {
  // stage 0 keeps the whole optimizer on every rank (plain data parallelism)
  if (stage == 0) { *off = 0; *len = P; *valid = P; return; }
  poplar_shard_range(P, c.world, c.rank, off, len, valid);
}

struct StepPlan {
  int64_t xs, saved, saved_each, shared, dxa, dxb, staging, gather, bytes;
};
// forward_only: what a forward pass alone touches (the probe of Algorithm 1's memory estimate): residual stream,
// stashes, the head's forward half, the stage 3 gather buffer; the other offsets are -1.
static StepPlan step_plan(const poplar_model_cfg& c, int stage, int B, bool forward_only = false) {
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, es = elt_size(c.dtype);
  const Units u = units_of(c);
  StepPlan p;
  int64_t at = 0;
  auto take = [&](int64_t bytes) { int64_t r = at; at += round_up(bytes, 256); return r; };
  p.xs = take((int64_t)(c.n_layer + 1) * round_up(T * H * es, 256));
  p.saved_each = saved_plan(c, B).bytes;
  p.saved = take(p.saved_each * (c.checkpoint ? 1 : c.n_layer));
  if (forward_only) {
    p.shared = take(head_plan(c, B).dhf);   // normed input, statistics, logits, per-row loss
    p.dxa = p.dxb = p.staging = -1;
    p.gather = stage >= 3 ? take((u.max_unit + u.tail_count) * es) : -1;
    p.bytes = at;
    return p;
  }
  {
    // the head's and the layers' backward workspaces share one region; the layers' constant part (the K-split
    // buffers) is counted on both sides of the max so that the size stays affine in the batch
    const BwdPlan bw = bwd_plan(c, B);
    p.shared = take(std::max(head_plan(c, B).bytes + bw.kpart_bytes, bw.bytes));
  }
  p.dxa = take(T * H * es);
  p.dxb = take(T * H * es);
  p.staging = stage >= 2 ? take((u.max_unit + 2 * H) * 4) : -1;
  p.gather = stage >= 3 ? take((u.max_unit + u.tail_count) * es) : -1;
  p.bytes = at;
  return p;
}

static int64_t state_bytes(const poplar_model_cfg& c, int stage) {
  const Units u = units_of(c);
  const int64_t es = elt_size(c.dtype), H = c.hidden;
  int64_t off, len, valid;
  stage_shard(c, stage, u.P, &off, &len, &valid);
  const int64_t bucket = (u.max_unit + 2 * H) * 4;
  switch (stage) {
    case 0: return es * u.P + 4 * u.P + 12 * u.P;
    case 1: return es * u.P + 4 * u.P + 12 * len;
    case 2: return es * u.P + 4 * len + bucket + 12 * len;
    default: return es * len + 2 * es * u.max_unit + 4 * len + bucket + 12 * len;
  }
}

static int64_t accounted_bytes(const poplar_model_cfg& c, int stage, int B, int forward_only) {
  if (B == 0) return state_bytes(c, stage);
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, es = elt_size(c.dtype);
  const HeadPlan hp = head_plan(c, B);
  int64_t act = (int64_t)(c.n_layer + 1) * round_up(T * H * es, 256) + saved_plan(c, B).bytes * (c.checkpoint ? 1 : c.n_layer) + (int64_t)B * (c.seq + 1) * 4;
  if (forward_only) act += hp.dhf;  // hf, stats, logits, row_loss (everything before dhf)
  else {
    const BwdPlan bw = bwd_plan(c, B);
    act += std::max(hp.bytes + bw.kpart_bytes, bw.bytes) + 2 * round_up(T * H * es, 256);
  }
  return state_bytes(c, stage) + act;
}

extern "C" int poplar_step_workspace_bytes(const poplar_model_cfg* cfg, int32_t stage, int32_t B, int64_t* bytes) {
  POPLAR_TRY(validate_cfg(cfg));
  if (stage < 0 || stage > 3 || B < 1 || !bytes) return poplar_fail(POPLAR_ERR_INVALID, "bad stage / batch / null pointer");
  *bytes = step_plan(*cfg, stage, B).bytes;
  return POPLAR_OK;
}

extern "C" int poplar_step_forward_bytes(const poplar_model_cfg* cfg, int32_t stage, int32_t B, int64_t* bytes) {
  POPLAR_TRY(validate_cfg(cfg));
  if (stage < 0 || stage > 3 || B < 1 || !bytes) return poplar_fail(POPLAR_ERR_INVALID, "bad stage / batch / null pointer");
  *bytes = step_plan(*cfg, stage, B, true).bytes;
  return POPLAR_OK;
}

extern "C" int poplar_step_accounted_bytes(const poplar_model_cfg* cfg, int32_t stage, int32_t B, int32_t forward_only, int64_t* bytes) {
  POPLAR_TRY(validate_cfg(cfg));
  if (stage < 0 || stage > 3 || B < 0 || !bytes) return poplar_fail(POPLAR_ERR_INVALID, "bad stage / batch / null pointer");
  *bytes = accounted_bytes(*cfg, stage, B, forward_only);
  return POPLAR_OK;
}

static double step_flops(const poplar_model_cfg& c, int B) {
  const double S = c.seq, H = c.hidden, F = c.ffn, V = c.vocab, L = c.n_layer;
  const double mlp = c.arch == POPLAR_ARCH_LLAMA ? 3.0 : 2.0;
  const double attn = (c.causal ? 7.0 : 14.0) * S * S * H;  // fwd 2 + bwd 5 per S^2 H at half density
  return (double)B * (L * (3.0 * 2.0 * S * (4.0 * H * H + mlp * H * F) + attn) + 3.0 * 2.0 * S * H * V);
}

// ---- event pool --------------------------------------------------------------
int ctx_take(poplar_ctx* ctx, hipEvent_t* e) {
  if (ctx->ev_next == ctx->events.size()) {
    hipEvent_t ne;
    // device-scope release: a default event flushes the caches to system scope each time it is recorded,
    // which costs microseconds between kernels and evicts what the next kernel would have found in L2
    POPLAR_CHECK_HIP(hipEventCreateWithFlags(&ne, hipEventReleaseToDevice));
    ctx->events.push_back(ne);
  }
  *e = ctx->events[ctx->ev_next++];
  return POPLAR_OK;
}
// grow the pool to n events now, so that no event is created between two timed marks
static int ctx_reserve(poplar_ctx* ctx, size_t n) {
  while (ctx->events.size() < n) {
    hipEvent_t ne;
    POPLAR_CHECK_HIP(hipEventCreateWithFlags(&ne, hipEventReleaseToDevice));
    ctx->events.push_back(ne);
  }
  return POPLAR_OK;
}
int ctx_mark(poplar_ctx* ctx, hipEvent_t* e) {
  POPLAR_TRY(ctx_take(ctx, e));
  POPLAR_CHECK_HIP(hipEventRecord(*e, ctx->stream));
  return POPLAR_OK;
}
struct EventCursor {
  poplar_ctx* ctx;
  int mark(hipEvent_t* e) { return ctx_mark(ctx, e); }
};

extern "C" int poplar_device_info(int32_t* compute_units, int32_t* clock_khz, int64_t* memory_bytes) {
  int dev = 0, v = 0;
  POPLAR_CHECK_HIP(hipGetDevice(&dev));
  if (compute_units) {
    POPLAR_CHECK_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
    *compute_units = v;
  }
  if (clock_khz) {
    POPLAR_CHECK_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeClockRate, dev));
    *clock_khz = v;
  }
  if (memory_bytes) {
    size_t free_b = 0, total_b = 0;
    POPLAR_CHECK_HIP(hipMemGetInfo(&free_b, &total_b));
    *memory_bytes = (int64_t)total_b;
  }
  return POPLAR_OK;
}

extern "C" int poplar_set_kernel_timing(poplar_ctx* ctx, int32_t on) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (on < 0 || on > 3) return poplar_fail(POPLAR_ERR_INVALID, "kernel timing selector %d: 0 off, 1 GEMM, 2 attention, 3 both", on);
  ctx->kernel_timing = on;
  return POPLAR_OK;
}

struct Span { hipEvent_t a, b; };

static int span_seconds(const std::vector<Span>& v, double* out) {
  double total = 0.0;
  for (const Span& s : v) {
    float ms = 0.f;
    POPLAR_CHECK_HIP(hipEventElapsedTime(&ms, s.a, s.b));
    total += (double)ms * 1e-3;
  }
  *out = total;
  return POPLAR_OK;
}

// How one pass of run_step sits in a gradient-accumulation run: which rows of the token buffer it reads, the
// loss weight per token, whether its gradients add to what is there, whether the optimizer runs after it.
struct MicroStep { int row0; float loss_scale; int accumulate; int optimizer; };

// workspace: the bound one, or one the memory hooks handed out for this step alone
static int run_step(poplar_ctx* ctx, int stage, int B, int forward_only, poplar_profile* out, const MicroStep* mstep = nullptr,
                    void* workspace = nullptr) {
  const poplar_model_cfg& c = ctx->cfg;
  const poplar_state& st = ctx->st;
  hipStream_t s = ctx->stream;
  const bool llama = c.arch == POPLAR_ARCH_LLAMA;
  const int64_t T = (int64_t)B * c.seq, H = c.hidden, es = elt_size(c.dtype);
  const Units u = units_of(c);
  const ModelOffsets mo = model_offsets(c);
  const StepPlan sp = step_plan(c, stage, B, forward_only != 0);
  int64_t sh_off, sh_len, sh_valid;
  stage_shard(c, stage, u.P, &sh_off, &sh_len, &sh_valid);

  char* ws = (char*)(workspace ? workspace : st.workspace);
  const int64_t xstride = round_up(T * H * es, 256);
  auto X = [&](int l) -> void* { return ws + sp.xs + (int64_t)l * xstride; };
  // with checkpointing every layer uses the one stash: the forward pass leaves nothing but the layer inputs X(l)
  auto SV = [&](int l) -> void* { return ws + sp.saved + (c.checkpoint ? 0 : (int64_t)l * sp.saved_each); };
  void* shared = ws + sp.shared;
  void* dx_cur = forward_only ? nullptr : ws + sp.dxa;
  void* dx_nxt = forward_only ? nullptr : ws + sp.dxb;
  float* staging = sp.staging >= 0 ? (float*)(ws + sp.staging) : nullptr;
  float* staging_tail = staging ? staging + u.max_unit : nullptr;  // GPT: gf, bf gradients next to the tied wte bucket
  char* gbuf = sp.gather >= 0 ? ws + sp.gather : nullptr;
  const int64_t tok_ld = c.seq + 1;
  const int32_t* tokens = st.tokens + (mstep ? (int64_t)mstep->row0 * tok_ld : 0);
  // next-token targets out of the token rows, or the caller's own target rows (masked-language-model batches)
  const int32_t* targets = st.targets ? st.targets + (mstep ? (int64_t)mstep->row0 * c.seq : 0) : tokens + 1;
  const int64_t tgt_ld = st.targets ? c.seq : tok_ld;
  const float loss_scale = mstep ? mstep->loss_scale : 1.0f / (float)((double)B * c.seq);
  const int acc = mstep ? mstep->accumulate : 0;          // gradients add to those already in st.grads
  const bool optimizer = mstep ? mstep->optimizer != 0 : true;

  ctx->ev_next = 0;
  ctx->launches.clear();
  // every event of the step exists before the first mark: four step marks, two per gather and per reduce span
  // (at most two gathers and three reduces per unit), two per timed launch (at most 16 GEMM and 3 attention
  // launches per layer, 4 in the head)
  POPLAR_TRY(ctx_reserve(ctx, 8 + 2 * (size_t)(5 * (c.n_layer + 4)) + (ctx->kernel_timing ? 2 * (size_t)(20 * c.n_layer + 8) : 0)));
  ctx->in_step = true;
  struct StepScope { poplar_ctx* c; ~StepScope() { c->in_step = false; } } scope{ctx};
  EventCursor ev{ctx};
  std::vector<Span> sp_gf, sp_gb, sp_red;
  int64_t red_elems = 0;   // elements the local reduces of this step add into the shard buffer
  hipEvent_t e_start, e_mid, e_bwd_end, e_adam_end;

  // parameter access: stages 0-2 read the resident compute copy; stage 3
  // gathers flat range [lo, hi) into the staging buffer first
  auto params_at = [&](int64_t lo, int64_t hi, char* dst, std::vector<Span>& spans, const void** p) -> int {
    if (stage < 3) { *p = (const char*)st.params + lo * es; return POPLAR_OK; }
    // the span's two events ride on the launch: kernel start to kernel end, no packet between kernels
    Span sn;
    int launched = 0;
    POPLAR_TRY(ctx_take(ctx, &sn.a));
    POPLAR_TRY(ctx_take(ctx, &sn.b));
    POPLAR_TRY(zero3_gather_local(s, c.dtype, dst, st.own_shard, st.params, lo, hi, sh_off, sh_len, sn.a, sn.b, &launched));
    if (launched) spans.push_back(sn);
    *p = dst;
    return POPLAR_OK;
  };
  // gradient destination of a unit and its hand-over to the shard buffer
  auto unit_grads = [&](int64_t lo) -> float* { return stage >= 2 ? staging : st.grads + lo; };
  auto reduce_unit = [&](const float* g_unit, int64_t lo, int64_t hi) -> int {
    if (stage < 2) return POPLAR_OK;
    Span sn;
    int launched = 0;
    POPLAR_TRY(ctx_take(ctx, &sn.a));
    POPLAR_TRY(ctx_take(ctx, &sn.b));
    POPLAR_TRY(zero2_reduce_local(s, st.grads, g_unit, lo, hi, sh_off, sh_len, sn.a, sn.b, &launched));
    if (launched) {   // a unit outside the shard moves nothing: no span
      sp_red.push_back(sn);
      red_elems += std::min(hi, sh_off + sh_len) - std::max(lo, sh_off);
    }
    return POPLAR_OK;
  };

  POPLAR_TRY(ev.mark(&e_start));
  // ---------------- forward ----------------
  const void* p_emb;
  POPLAR_TRY(params_at(0, u.emb_hi, gbuf, sp_gf, &p_emb));
  POPLAR_TRY(embed_fwd(s, c.dtype, B, c.seq, (int)H, c.vocab, tokens, tok_ld, p_emb, llama ? nullptr : (const char*)p_emb + mo.wpe * es, X(0)));
  for (int l = 0; l < c.n_layer; ++l) {
    const void* p_l;
    const int64_t lo = u.layer0 + (int64_t)l * u.lc;
    POPLAR_TRY(params_at(lo, lo + u.lc, gbuf, sp_gf, &p_l));
    POPLAR_TRY(layer_fwd_impl(ctx, B, X(l), p_l, X(l + 1), SV(l)));
  }
  // head parameters: gf[, bf] and the output matrix (GPT: tied wte)
  const void *p_tail, *p_whead;
  auto head_params = [&](std::vector<Span>& spans) -> int {
    if (llama) {
      POPLAR_TRY(params_at(u.tail_lo, u.P, gbuf, spans, &p_tail));
      p_whead = (const char*)p_tail + (mo.whead - mo.gf) * es;
    } else {
      POPLAR_TRY(params_at(0, u.emb_hi, gbuf, spans, &p_whead));  // wte sits first in the embedding unit
      POPLAR_TRY(params_at(u.tail_lo, u.P, gbuf ? gbuf + u.max_unit * es : nullptr, spans, &p_tail));
    }
    return POPLAR_OK;
  };
  POPLAR_TRY(head_params(sp_gf));
  const void* p_gf = p_tail;
  const void* p_bf = llama ? nullptr : (const char*)p_tail + H * es;
  POPLAR_TRY(head_fwd_part(ctx, B, X(c.n_layer), targets, tgt_ld, p_gf, p_bf, p_whead, loss_scale, st.loss, shared));
  POPLAR_TRY(ev.mark(&e_mid));

  if (!forward_only) {
    // ---------------- backward ----------------
    if (stage >= 2 && !acc) POPLAR_TRY(fill_zero(s, st.grads, sh_len * 4));
    if (stage >= 3) POPLAR_TRY(head_params(sp_gb));
    if (llama) {
      float* gt = unit_grads(u.tail_lo);  // tail unit: gf then Whead
      POPLAR_TRY(head_bwd_part(ctx, B, X(c.n_layer), p_gf, p_whead, dx_cur, gt, nullptr, gt + (mo.whead - mo.gf), stage < 2 ? acc : 0, shared));
      POPLAR_TRY(reduce_unit(gt, u.tail_lo, u.P));
    } else {
      float* gt = stage >= 2 ? staging_tail : st.grads + u.tail_lo;
      float* ge = unit_grads(0);  // embedding unit: wte first
      POPLAR_TRY(head_bwd_part(ctx, B, X(c.n_layer), p_gf, p_whead, dx_cur, gt, gt + H, ge, stage < 2 ? acc : 0, shared));
      POPLAR_TRY(reduce_unit(gt, u.tail_lo, u.P));
      // the tied matrix's head term goes to the shard now, the embedding term at the end
      POPLAR_TRY(reduce_unit(ge, 0, (int64_t)c.vocab * H));
    }
    for (int l = c.n_layer - 1; l >= 0; --l) {
      const void* p_l;
      const int64_t lo = u.layer0 + (int64_t)l * u.lc;
      POPLAR_TRY(params_at(lo, lo + u.lc, gbuf, sp_gb, &p_l));
      float* gl = unit_grads(lo);
      // checkpointing: the layer's forward pass again, from its kept input, to refill the stash (X(l+1) is
      // rewritten with the values it already holds)
      if (c.checkpoint) POPLAR_TRY(layer_fwd_impl(ctx, B, X(l), p_l, X(l + 1), SV(l)));
      POPLAR_TRY(layer_bwd_impl(ctx, B, X(l), dx_cur, p_l, SV(l), dx_nxt, gl, stage < 2 ? acc : 0, shared));
      POPLAR_TRY(reduce_unit(gl, lo, lo + u.lc));
      std::swap(dx_cur, dx_nxt);
    }
    {
      float* ge = unit_grads(0);
      // stage 0/1 GPT: the head already wrote dwte, the embedding adds to it; everywhere else start from zero
      // (an accumulating pass at stage 0/1 adds to the earlier micro-steps' gradient instead)
      if (stage >= 2 || (llama && !acc)) POPLAR_TRY(fill_zero(s, ge, (int64_t)c.vocab * H * 4));
      POPLAR_TRY(embed_bwd(s, c.dtype, B, c.seq, (int)H, c.vocab, tokens, tok_ld, dx_cur, ge, llama ? nullptr : ge + mo.wpe, stage < 2 ? acc : 0, c.deterministic));
      POPLAR_TRY(reduce_unit(ge, 0, u.emb_hi));
    }
    POPLAR_TRY(ev.mark(&e_bwd_end));
    // ---------------- optimizer on the shard ----------------
    const float* g_adam = stage >= 2 ? st.grads : st.grads + sh_off;
    void* lowp_dst = stage >= 3 ? st.own_shard : (char*)st.params + sh_off * es;
    if (optimizer)
      POPLAR_TRY(adam_shard(s, c.dtype, st.master, st.m, st.v, g_adam, lowp_dst, sh_valid, st.adam_t, st.lr, st.beta1, st.beta2, st.eps));
    POPLAR_TRY(ev.mark(&e_adam_end));
  }
  float loss_host = 0.f;
  POPLAR_CHECK_HIP(hipMemcpyAsync(&loss_host, st.loss, sizeof(float), hipMemcpyDeviceToHost, s));
  POPLAR_CHECK_HIP(hipStreamSynchronize(s));

  memset(out, 0, sizeof *out);
  out->stage = stage; out->batch = B;
  float ms = 0.f;
  POPLAR_CHECK_HIP(hipEventElapsedTime(&ms, e_start, e_mid));
  out->t_fwd = ms * 1e-3;
  POPLAR_TRY(span_seconds(sp_gf, &out->t_gather_fwd));
  if (!forward_only) {
    POPLAR_CHECK_HIP(hipEventElapsedTime(&ms, e_mid, e_bwd_end));
    out->t_bwd = ms * 1e-3;
    POPLAR_CHECK_HIP(hipEventElapsedTime(&ms, e_bwd_end, e_adam_end));
    out->t_adam = ms * 1e-3;
    POPLAR_TRY(span_seconds(sp_gb, &out->t_gather_bwd));
    POPLAR_TRY(span_seconds(sp_red, &out->t_reduce_bwd));
    out->reduce_elems = red_elems;
  }
  out->t_consumed = out->t_fwd + out->t_bwd;
  if (stage >= 2) out->t_consumed -= out->t_reduce_bwd;
  if (stage >= 3) out->t_consumed -= out->t_gather_fwd + out->t_gather_bwd;
  out->accounted_bytes = accounted_bytes(c, stage, B, forward_only);
  out->flops = forward_only ? step_flops(c, B) / 3.0 : step_flops(c, B);
  out->loss = loss_host;
  for (const TimedLaunch& tl : ctx->launches) {
    POPLAR_CHECK_HIP(hipEventElapsedTime(&ms, tl.a, tl.b));
    if (tl.kind == KIND_GEMM) { out->t_gemm += ms * 1e-3; out->gemm_flops += tl.flops; out->n_gemm += 1; out->n_gemm_kernels += tl.kernels; }
    else { out->t_attn += ms * 1e-3; out->attn_flops += tl.flops; out->n_attn += 1; }
  }
  return POPLAR_OK;
}

static int check_step_args(poplar_ctx* ctx, int stage, int B) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (!ctx->bound) return poplar_fail(POPLAR_ERR_INVALID, "no state bound: call poplar_bind_state first");
  if (stage < 0 || stage > 3) return poplar_fail(POPLAR_ERR_INVALID, "stage %d outside 0..3", stage);
  if (B < 1) return poplar_fail(POPLAR_ERR_INVALID, "batch must be >= 1, got %d", B);
  if (stage == 3 && !ctx->st.own_shard) return poplar_fail(POPLAR_ERR_INVALID, "stage 3 needs own_shard");
  if (B > ctx->st.max_batch) return poplar_fail(POPLAR_ERR_INVALID, "batch %d above the bound token buffer (%d)", B, ctx->st.max_batch);
  // the bound buffers must hold what this stage touches: the optimizer runs over the stage's shard (all P elements
  // at stage 0), the gradients are the whole flat vector at stage 0/1 and the shard at 2/3
  const Units u = units_of(ctx->cfg);
  int64_t off, len, valid;
  stage_shard(ctx->cfg, stage, u.P, &off, &len, &valid);
  if (valid > ctx->st.master_len)
    return poplar_fail(POPLAR_ERR_INVALID, "stage %d updates %lld optimizer elements, master / m / v hold %lld", stage, (long long)valid,
                       (long long)ctx->st.master_len);
  const int64_t gneed = stage < 2 ? u.P : len;
  if (gneed > ctx->st.grads_len)
    return poplar_fail(POPLAR_ERR_INVALID, "stage %d needs a gradient buffer of %lld floats, the bound one holds %lld", stage, (long long)gneed,
                       (long long)ctx->st.grads_len);
  if (stage == 3 && valid > ctx->st.own_len)
    return poplar_fail(POPLAR_ERR_INVALID, "stage 3 writes %lld parameters to own_shard, it holds %lld", (long long)valid, (long long)ctx->st.own_len);
  return POPLAR_OK;
}

static int check_memory(poplar_ctx* ctx, int stage, int B, int forward_only) {
  if (ctx->have_hooks) return POPLAR_OK;   // the allocator behind the hooks decides
  const poplar_model_cfg& c = ctx->cfg;
  const int64_t acc = accounted_bytes(c, stage, B, forward_only);
  if (c.cap_bytes > 0 && acc > c.cap_bytes)
    return poplar_fail(POPLAR_ERR_OOM, "stage %d batch %d needs %lld bytes, cap is %lld", stage, B, (long long)acc, (long long)c.cap_bytes);
  const int64_t need = step_plan(c, stage, B).bytes;
  if (need > ctx->st.workspace_bytes)
    return poplar_fail(POPLAR_ERR_OOM, "stage %d batch %d needs a %lld byte workspace, bound one has %lld", stage, B, (long long)need,
                       (long long)ctx->st.workspace_bytes);
  return POPLAR_OK;
}

extern "C" int poplar_set_sampling(poplar_ctx* ctx, int32_t warmup, int32_t repeats) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (warmup < 0 || repeats < 1 || warmup > 64 || repeats > 65) return poplar_fail(POPLAR_ERR_INVALID, "need 0 <= warmup <= 64 and 1 <= repeats <= 65");
  ctx->warmup = warmup; ctx->repeats = repeats;
  return POPLAR_OK;
}

extern "C" int poplar_set_mem_hooks(poplar_ctx* ctx, const poplar_mem_hooks* hooks) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (!hooks) { ctx->have_hooks = false; return POPLAR_OK; }
  if (!hooks->alloc || !hooks->release || !hooks->bytes_now || !hooks->bytes_total) return poplar_fail(POPLAR_ERR_INVALID, "a memory hook is null");
  ctx->hooks = *hooks;
  ctx->have_hooks = true;
  return POPLAR_OK;
}

// A workspace for one step at (stage, B): with hooks, asked of the caller's allocator (POPLAR_ERR_OOM when it has
// none to give; nothing has been launched and the state is as it was); without, the bound one.
struct StepWorkspace {
  poplar_ctx* ctx;
  void* p = nullptr;
  bool owned = false;
  int64_t held_bytes = 0;   // what the allocator reports while the workspace is held
  int acquire(int stage, int B, bool forward_only) {
    if (!ctx->have_hooks) { p = ctx->st.workspace; return POPLAR_OK; }
    const int64_t need = step_plan(ctx->cfg, stage, B, forward_only).bytes;
    p = ctx->hooks.alloc(ctx->hooks.user, need);
    if (!p) return poplar_fail(POPLAR_ERR_OOM, "stage %d batch %d: the allocator refused a workspace of %lld bytes", stage, B, (long long)need);
    owned = true;
    held_bytes = ctx->hooks.bytes_now(ctx->hooks.user);
    return POPLAR_OK;
  }
  ~StepWorkspace() {
    if (owned) ctx->hooks.release(ctx->hooks.user, p);   // every step has synchronised the stream before it returns
  }
};

// One profile sample: `warmup` untimed runs, `repeats` timed ones, the run with the median TimeConsumedDuringStep
// (the lower of the two middle ones for an even count) is reported whole, so that its fields belong together.
static int sample_step(poplar_ctx* ctx, int stage, int B, poplar_profile* out) {
  StepWorkspace w{ctx};
  POPLAR_TRY(w.acquire(stage, B, false));
  poplar_profile tmp;
  for (int i = 0; i < ctx->warmup; ++i) POPLAR_TRY(run_step(ctx, stage, B, 0, &tmp, nullptr, w.p));
  std::vector<poplar_profile> runs((size_t)ctx->repeats);
  for (int i = 0; i < ctx->repeats; ++i) POPLAR_TRY(run_step(ctx, stage, B, 0, &runs[i], nullptr, w.p));
  std::vector<int> order((size_t)ctx->repeats);
  for (int i = 0; i < ctx->repeats; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return runs[a].t_consumed < runs[b].t_consumed; });
  *out = runs[order[(ctx->repeats - 1) / 2]];
  out->measured_bytes = w.held_bytes;
  return POPLAR_OK;
}

extern "C" int poplar_profile_step(poplar_ctx* ctx, int32_t stage, int32_t local_batch, poplar_profile* out) {
  POPLAR_TRY(check_step_args(ctx, stage, local_batch));
  if (!out) return poplar_fail(POPLAR_ERR_INVALID, "out is null");
  POPLAR_TRY(check_memory(ctx, stage, local_batch, 0));
  return sample_step(ctx, stage, local_batch, out);
}

extern "C" int poplar_accum_step(poplar_ctx* ctx, int32_t stage, int32_t n_micro, const int32_t* micro_batch, int32_t loss_batch,
                                 poplar_profile* out) {
  if (!ctx) return poplar_fail(POPLAR_ERR_INVALID, "ctx is null");
  if (n_micro < 1 || !micro_batch || !out) return poplar_fail(POPLAR_ERR_INVALID, "need n_micro >= 1, micro_batch and out");
  if (loss_batch < 1) return poplar_fail(POPLAR_ERR_INVALID, "loss_batch must be >= 1, got %d", loss_batch);
  int64_t rows = 0;
  int bmax = 0;
  for (int k = 0; k < n_micro; ++k) {
    POPLAR_TRY(check_step_args(ctx, stage, micro_batch[k]));
    POPLAR_TRY(check_memory(ctx, stage, micro_batch[k], 0));
    rows += micro_batch[k];
    bmax = std::max(bmax, (int)micro_batch[k]);
  }
  if (rows > ctx->st.max_batch)
    return poplar_fail(POPLAR_ERR_INVALID, "micro-batches sum to %lld samples, the bound token buffer holds %d", (long long)rows, ctx->st.max_batch);
  // one workspace, sized for the largest micro-batch, serves the whole run
  StepWorkspace w{ctx};
  POPLAR_TRY(w.acquire(stage, bmax, false));
  poplar_profile tot;
  memset(&tot, 0, sizeof tot);
  tot.stage = stage;
  tot.measured_bytes = w.held_bytes;
  int row0 = 0;
  for (int k = 0; k < n_micro; ++k) {
    MicroStep ms;
    ms.row0 = row0;
    ms.loss_scale = 1.0f / (float)((double)loss_batch * ctx->cfg.seq);
    ms.accumulate = k > 0;
    ms.optimizer = k == n_micro - 1;
    poplar_profile pr;
    POPLAR_TRY(run_step(ctx, stage, micro_batch[k], 0, &pr, &ms, w.p));
    row0 += micro_batch[k];
    tot.batch += pr.batch;
    tot.t_fwd += pr.t_fwd; tot.t_bwd += pr.t_bwd; tot.t_gather_fwd += pr.t_gather_fwd; tot.t_gather_bwd += pr.t_gather_bwd;
    tot.t_reduce_bwd += pr.t_reduce_bwd; tot.t_consumed += pr.t_consumed; tot.flops += pr.flops; tot.loss += pr.loss;
    tot.t_gemm += pr.t_gemm; tot.gemm_flops += pr.gemm_flops; tot.t_attn += pr.t_attn; tot.attn_flops += pr.attn_flops;
    tot.n_gemm += pr.n_gemm; tot.n_attn += pr.n_attn; tot.n_gemm_kernels += pr.n_gemm_kernels; tot.reduce_elems += pr.reduce_elems;
    if (pr.accounted_bytes > tot.accounted_bytes) tot.accounted_bytes = pr.accounted_bytes;
    if (ms.optimizer) tot.t_adam = pr.t_adam;
  }
  *out = tot;
  return POPLAR_OK;
}

extern "C" int poplar_search_mbs(poplar_ctx* ctx, int32_t stage, int32_t* mbs, poplar_profile* samples, int32_t max_samples,
                                 int32_t* n_samples) {
  POPLAR_TRY(check_step_args(ctx, stage, 1));
  if (!mbs || !samples || !n_samples || max_samples < 1) return poplar_fail(POPLAR_ERR_INVALID, "null output or no room for samples");
  const poplar_model_cfg& c = ctx->cfg;
  *mbs = 0; *n_samples = 0;
  // step 1: memory before and after one forward pass at batch 1 gives the theoretical maximum.  With memory hooks
  // both readings and the total are the allocator's; without, they are the accounted bytes and the emulated cap.
  int64_t total, bf, af;
  if (ctx->have_hooks) {
    total = ctx->hooks.bytes_total(ctx->hooks.user);
    bf = ctx->hooks.bytes_now(ctx->hooks.user);
    StepWorkspace w{ctx};
    const int rc = w.acquire(stage, 1, true);
    if (rc == POPLAR_ERR_OOM) return POPLAR_OK;   // not even the forward pass of one sample can be held: mbs = 0
    POPLAR_TRY(rc);
    poplar_profile fwd;
    POPLAR_TRY(run_step(ctx, stage, 1, 1, &fwd, nullptr, w.p));
    af = w.held_bytes;
  } else {
    total = c.cap_bytes;
    if (total == 0) {
      size_t free_b = 0, total_b = 0;
      POPLAR_CHECK_HIP(hipMemGetInfo(&free_b, &total_b));
      total = (int64_t)total_b;
    }
    bf = accounted_bytes(c, stage, 0, 1);
    poplar_profile fwd;
    const int rc = check_memory(ctx, stage, 1, 1);
    if (rc == POPLAR_ERR_OOM) return POPLAR_OK;  // not even a forward pass of one sample fits: mbs = 0
    POPLAR_TRY(rc);
    POPLAR_TRY(run_step(ctx, stage, 1, 1, &fwd));
    af = fwd.accounted_bytes;
  }
  if (af <= bf) return poplar_fail(POPLAR_ERR_INVALID, "forward pass took no memory (%lld bytes before, %lld after)", (long long)bf, (long long)af);
  int64_t est = (total - bf) / (af - bf);
  if (est > ctx->st.max_batch) est = ctx->st.max_batch;
  auto try_step = [&](int b, bool* fits) -> int {
    *fits = false;
    int r = check_memory(ctx, stage, b, 0);
    if (r == POPLAR_ERR_OOM) return POPLAR_OK;
    POPLAR_TRY(r);
    if (*n_samples >= max_samples) return poplar_fail(POPLAR_ERR_INVALID, "more than %d samples", max_samples);
    r = sample_step(ctx, stage, b, &samples[*n_samples]);
    if (r == POPLAR_ERR_OOM) return POPLAR_OK;   // the allocator behind the hooks had no room: nothing ran
    POPLAR_TRY(r);
    *n_samples += 1;
    *fits = true;
    return POPLAR_OK;
  };
  // step 2: doubling sweep; step 3: bisection between the last fit and the first failure
  int64_t lo = 0, hi = est;
  for (int64_t b = 1; b <= est; b *= 2) {
    bool fits;
    POPLAR_TRY(try_step((int)b, &fits));
    if (!fits) { hi = b - 1; break; }
    lo = b;
  }
  while (lo < hi) {
    int64_t mid = (lo + hi + 1) / 2;
    bool fits;
    POPLAR_TRY(try_step((int)mid, &fits));
    if (fits) lo = mid; else hi = mid - 1;
  }
  *mbs = (int32_t)lo;
  return POPLAR_OK;
}

extern "C" int poplar_search_stage(poplar_ctx* ctx, int32_t first_stage, int32_t* stage, int32_t* mbs, poplar_profile* samples,
                                   int32_t max_samples, int32_t* n_samples) {
  if (!ctx || !stage || !mbs || !n_samples) return poplar_fail(POPLAR_ERR_INVALID, "null argument");
  if (first_stage < 0 || first_stage > 3) return poplar_fail(POPLAR_ERR_INVALID, "first_stage %d outside 0..3", first_stage);
  *stage = -1; *mbs = 0; *n_samples = 0;
  for (int s = first_stage; s <= 3; ++s) {
    POPLAR_TRY(poplar_search_mbs(ctx, s, mbs, samples, max_samples, n_samples));
    if (*mbs > 0) { *stage = s; return POPLAR_OK; }
  }
  return POPLAR_OK;
}
