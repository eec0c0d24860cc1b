// Byte plans of the per-layer activation stash and scratch areas, and the
// internal (unchecked) layer / head routines shared with the whole-step code.
#pragma once
#include "common.h"
#include <algorithm>

struct SavedPlan { int64_t stats1, a, qkv, o, lse, x1, stats2, m, h, g, bytes; };
struct BwdPlan { int64_t dh, dg, dm, dx1, dob, dqkv, da, delta, scratch, kpart[4], kpart_bytes, bytes; };   // kpart: -1 without (fp32 path); kpart_bytes: their share of bytes (no batch in it)
struct HeadPlan { int64_t ldl, hf, stats, logits, row_loss, dhf, dhf32, scratch, bytes; bool dhf_split; };

SavedPlan saved_plan(const poplar_model_cfg& c, int B);
BwdPlan bwd_plan(const poplar_model_cfg& c, int B);
HeadPlan head_plan(const poplar_model_cfg& c, int B);
int64_t scratch_floats(const poplar_model_cfg& c);

int layer_fwd_impl(poplar_ctx* ctx, int B, const void* x_in, const void* params, void* x_out, void* saved);
int layer_bwd_impl(poplar_ctx* ctx, int B, const void* x_in, const void* dy, const void* params, const void* saved, void* dx,
                   float* grads, int accumulate, void* workspace);
int head_fwd_part(poplar_ctx* ctx, int B, const void* x, const int32_t* targets, int64_t tgt_ld, const void* gf, const void* bf,
                  const void* whead, float loss_scale, float* loss, void* workspace);
int head_bwd_part(poplar_ctx* ctx, int B, const void* x, const void* gf, const void* whead, void* dx, float* d_gf, float* d_bf,
                  float* d_whead, int accumulate, void* workspace);
