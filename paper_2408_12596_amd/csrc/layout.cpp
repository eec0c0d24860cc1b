// Error reporting, configuration checks, flat parameter layout and ZeRO shard
// arithmetic.  Host only, integers only.
#include "common.h"
#include <stdio.h>
#include <string.h>

static thread_local char g_err[512] = "";
thread_local int64_t poplar_gemm_kernel_launches = 0;

int poplar_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

extern "C" const char* poplar_last_error(void) { return g_err; }

int validate_cfg(const poplar_model_cfg* c) {
  if (!c) return poplar_fail(POPLAR_ERR_INVALID, "cfg is null");
  if (c->arch != POPLAR_ARCH_GPT && c->arch != POPLAR_ARCH_LLAMA) return poplar_fail(POPLAR_ERR_INVALID, "unknown arch %d", c->arch);
  if (c->dtype != POPLAR_F32 && c->dtype != POPLAR_BF16) return poplar_fail(POPLAR_ERR_INVALID, "unknown dtype %d", c->dtype);
  if (c->n_layer < 0 || c->hidden < 8 || c->n_head < 1 || c->ffn < 8 || c->seq < 1 || c->vocab < 1)
    return poplar_fail(POPLAR_ERR_INVALID, "non-positive model dimension");
  if (c->hidden % 8 || c->ffn % 8) return poplar_fail(POPLAR_ERR_INVALID, "hidden (%d) and ffn (%d) must be multiples of 8", c->hidden, c->ffn);
  if (c->hidden % c->n_head) return poplar_fail(POPLAR_ERR_INVALID, "hidden %d not divisible by n_head %d", c->hidden, c->n_head);
  int d = c->hidden / c->n_head;
  if (d % 2) return poplar_fail(POPLAR_ERR_INVALID, "head_dim %d must be even", d);
  if (c->dtype == POPLAR_BF16 && d != 64 && d != 128) return poplar_fail(POPLAR_ERR_INVALID, "bf16 attention needs head_dim 64 or 128, got %d", d);
  if (d > 256) return poplar_fail(POPLAR_ERR_INVALID, "head_dim %d above 256", d);
  if (c->world < 1 || c->rank < 0 || c->rank >= c->world) return poplar_fail(POPLAR_ERR_INVALID, "rank %d outside world %d", c->rank, c->world);
  if (c->zero_stage < 0 || c->zero_stage > 3) return poplar_fail(POPLAR_ERR_INVALID, "zero_stage %d outside 0..3", c->zero_stage);
  if (c->cap_bytes < 0) return poplar_fail(POPLAR_ERR_INVALID, "negative cap_bytes");
  if (c->checkpoint != 0 && c->checkpoint != 1) return poplar_fail(POPLAR_ERR_INVALID, "checkpoint must be 0 or 1, got %d", c->checkpoint);
  if (c->deterministic != 0 && c->deterministic != 1) return poplar_fail(POPLAR_ERR_INVALID, "deterministic must be 0 or 1, got %d", c->deterministic);
  return POPLAR_OK;
}

LayerOffsets layer_offsets(const poplar_model_cfg& c) {
  const int64_t H = c.hidden, F = c.ffn;
  LayerOffsets o;
  int64_t at = 0;
  auto take = [&](int64_t n) { int64_t r = at; at += n; return r; };
  if (c.arch == POPLAR_ARCH_GPT) {
    o.g1 = take(H); o.b1 = take(H);
    o.wqkv = take(3 * H * H); o.bqkv = take(3 * H);
    o.wo = take(H * H); o.bo = take(H);
    o.g2 = take(H); o.b2 = take(H);
    o.w1 = take(F * H); o.bm1 = take(F);
    o.w2 = take(H * F); o.bm2 = take(H);
  } else {
    o.g1 = take(H); o.b1 = -1;
    o.wqkv = take(3 * H * H); o.bqkv = -1;
    o.wo = take(H * H); o.bo = -1;
    o.g2 = take(H); o.b2 = -1;
    o.w1 = take(2 * F * H); o.bm1 = -1;   // Wg then Wu: one [2F, H] matrix
    o.w2 = take(H * F); o.bm2 = -1;
  }
  o.count = at;
  return o;
}

ModelOffsets model_offsets(const poplar_model_cfg& c) {
  const int64_t H = c.hidden, V = c.vocab, S = c.seq;
  ModelOffsets o;
  o.layer_count = layer_offsets(c).count;
  int64_t at = 0;
  o.wte = at; at += V * H;
  if (c.arch == POPLAR_ARCH_GPT) { o.wpe = at; at += S * H; } else o.wpe = -1;
  o.layer0 = at; at += o.layer_count * c.n_layer;
  o.gf = at; at += H;
  if (c.arch == POPLAR_ARCH_GPT) { o.bf = at; at += H; o.whead = -1; }
  else { o.bf = -1; o.whead = at; at += V * H; }
  o.count = at;
  return o;
}

extern "C" int poplar_layer_param_count(const poplar_model_cfg* cfg, int64_t* count) {
  POPLAR_TRY(validate_cfg(cfg));
  if (!count) return poplar_fail(POPLAR_ERR_INVALID, "count is null");
  *count = layer_offsets(*cfg).count;
  return POPLAR_OK;
}

extern "C" int poplar_model_param_count(const poplar_model_cfg* cfg, int64_t* count) {
  POPLAR_TRY(validate_cfg(cfg));
  if (!count) return poplar_fail(POPLAR_ERR_INVALID, "count is null");
  *count = model_offsets(*cfg).count;
  return POPLAR_OK;
}

extern "C" int poplar_param_offset(const poplar_model_cfg* cfg, int32_t layer, int32_t id,
                                   int64_t* offset, int64_t* rows, int64_t* cols) {
  POPLAR_TRY(validate_cfg(cfg));
  if (!offset || !rows || !cols) return poplar_fail(POPLAR_ERR_INVALID, "null output pointer");
  const poplar_model_cfg& c = *cfg;
  const int64_t H = c.hidden, F = c.ffn, V = c.vocab, S = c.seq;
  ModelOffsets mo = model_offsets(c);
  int64_t off = -1, r = 0, cc = 1;
  if (id >= POPLAR_T_WTE) {
    switch (id) {
      case POPLAR_T_WTE: off = mo.wte; r = V; cc = H; break;
      case POPLAR_T_WPE: off = mo.wpe; r = S; cc = H; break;
      case POPLAR_T_GF: off = mo.gf; r = H; break;
      case POPLAR_T_BF: off = mo.bf; r = H; break;
      case POPLAR_T_WHEAD: off = mo.whead; r = V; cc = H; break;
      default: return poplar_fail(POPLAR_ERR_INVALID, "unknown tensor id %d", id);
    }
    if (off < 0) return poplar_fail(POPLAR_ERR_INVALID, "tensor %d absent in this architecture", id);
  } else {
    if (layer < 0 || layer >= c.n_layer) return poplar_fail(POPLAR_ERR_INVALID, "layer %d outside 0..%d", layer, c.n_layer - 1);
    LayerOffsets lo = layer_offsets(c);
    const bool llama = c.arch == POPLAR_ARCH_LLAMA;
    switch (id) {
      case POPLAR_T_G1: off = lo.g1; r = H; break;
      case POPLAR_T_B1: off = lo.b1; r = H; break;
      case POPLAR_T_WQKV: off = lo.wqkv; r = 3 * H; cc = H; break;
      case POPLAR_T_BQKV: off = lo.bqkv; r = 3 * H; break;
      case POPLAR_T_WO: off = lo.wo; r = H; cc = H; break;
      case POPLAR_T_BO: off = lo.bo; r = H; break;
      case POPLAR_T_G2: off = lo.g2; r = H; break;
      case POPLAR_T_B2: off = lo.b2; r = H; break;
      case POPLAR_T_W1: off = lo.w1; r = llama ? 2 * F : F; cc = H; break;
      case POPLAR_T_BM1: off = lo.bm1; r = F; break;
      case POPLAR_T_W2: off = lo.w2; r = H; cc = F; break;
      case POPLAR_T_BM2: off = lo.bm2; r = H; break;
      default: return poplar_fail(POPLAR_ERR_INVALID, "unknown tensor id %d", id);
    }
    if (off < 0) return poplar_fail(POPLAR_ERR_INVALID, "tensor %d absent in this architecture", id);
    off += mo.layer0 + (int64_t)layer * lo.count;
  }
  *offset = off; *rows = r; *cols = cc;
  return POPLAR_OK;
}

extern "C" int poplar_shard_range(int64_t P, int32_t N, int32_t r, int64_t* off, int64_t* len, int64_t* valid) {
  if (P < 0 || N < 1 || r < 0 || r >= N) return poplar_fail(POPLAR_ERR_INVALID, "shard_range(P=%lld, N=%d, r=%d)", (long long)P, N, r);
  if (!off || !len || !valid) return poplar_fail(POPLAR_ERR_INVALID, "null output pointer");
  int64_t l = (P + N - 1) / N;
  int64_t o = (int64_t)r * l;
  int64_t v = P - o;
  if (v > l) v = l;
  if (v < 0) v = 0;
  *off = o; *len = l; *valid = v;
  return POPLAR_OK;
}
