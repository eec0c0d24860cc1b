// Internal declarations shared by the translation units of libpoplar.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdarg.h>
#include <vector>
#include "../../include/poplar.h"

typedef __hip_bfloat16 bf16;

int poplar_fail(int code, const char* fmt, ...);

#define POPLAR_CHECK_HIP(expr)                                                         \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess)                                                              \
      return poplar_fail(POPLAR_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));      \
  } while (0)

#define POPLAR_TRY(expr)            \
  do {                              \
    int s_ = (expr);                \
    if (s_ != POPLAR_OK) return s_; \
  } while (0)

#define POPLAR_LAUNCH_CHECK() POPLAR_CHECK_HIP(hipGetLastError())

enum LaunchKind { KIND_GEMM = 0, KIND_ATTN = 1, KIND_COUNT = 2 };
struct TimedLaunch { int kind; hipEvent_t a, b; double flops; int kernels; };
// GEMM kernels launched by this thread so far (every tile kernel of every GEMM path; not the zero fills and adds
// around them): a timed span reads it before and after to know how many kernels it covered
extern thread_local int64_t poplar_gemm_kernel_launches;

struct poplar_ctx {
  poplar_model_cfg cfg;
  hipStream_t stream;
  poplar_state st;
  bool bound;
  std::vector<hipEvent_t> events;  // pool reused by every profiled step
  size_t ev_next;                  // next unused event of the pool in the running step
  int kernel_timing;               // bit 0: time every GEMM launch with events, bit 1: every attention launch
  bool in_step;                    // a profiled step is being enqueued
  std::vector<TimedLaunch> launches;
  int warmup, repeats;             // untimed and timed runs behind one profile sample
  bool have_hooks;                 // step workspaces come from the caller's allocator
  poplar_mem_hooks hooks;
};
// record the next pooled event on the context's stream
int ctx_mark(poplar_ctx* ctx, hipEvent_t* e);
// hand out the next pooled event without recording it (a launcher records it with the kernel it brackets)
int ctx_take(poplar_ctx* ctx, hipEvent_t* e);

static inline int64_t elt_size(int dtype) { return dtype == POPLAR_BF16 ? 2 : 4; }
static inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// layout.cpp
struct LayerOffsets {  // element offsets inside one layer block; -1 = absent
  int64_t g1, b1, wqkv, bqkv, wo, bo, g2, b2, w1, bm1, w2, bm2, count;
};
LayerOffsets layer_offsets(const poplar_model_cfg& c);
struct ModelOffsets {
  int64_t wte, wpe, layer0, gf, bf, whead, count, layer_count;
};
ModelOffsets model_offsets(const poplar_model_cfg& c);
int validate_cfg(const poplar_model_cfg* cfg);

// ---- kernel launchers (each returns a poplar_status) ------------------------
// GEMM: C[M,N] = epilogue(sum_k A(m,k) * B(k,n)).
enum GemmLayout { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };
// NT: A[M,K] row-major (lda), B stored [N,K] row-major (ldb)   -> y = x W^T
// NN: A[M,K] row-major (lda), B stored [K,N] row-major (ldb)   -> dx = dy W
// TN: A stored [K,M] row-major (lda), B stored [K,N] (ldb)     -> dW = dy^T x
enum GemmAct { ACT_NONE = 0, ACT_GELU = 1, ACT_GELU_BWD = 2 };
struct GemmArgs {
  int layout;
  int64_t M, N, K;
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  void* C; int64_t ldc;
  int c_float;            // 1: C is float regardless of the input dtype
  float beta;             // C = acc + beta * C_old  (float C only; 0 or 1)
  const void* bias;       // lowp [N] or null, added per column
  const void* residual;   // lowp [M,N] (ldc) or null, added after activation
  int act;                // ACT_GELU: with h = acc + bias, aux <- gelu'(h), C <- gelu(h);  ACT_GELU_BWD: C <- acc * aux
  void* aux; int64_t ldaux;
  float* a_rowsum;        // TN only, or null: a_rowsum[m] (+)= sum_k A(k, m), the bias gradient next to a weight gradient;
  int a_rowsum_accumulate;  //   honoured by the direct-to-LDS kernel only (ask gemm_bf16_dtl_accepts first)
  // TN with a float C and nothing fused (a weight gradient), or null: room for M * ldc + M floats.  With it the
  // direct-to-LDS kernel may cut K in two: the second half's sums go here and are added to C (and to a_rowsum) afterwards.
  float* k_partial = nullptr;
  int no_atomics = 0;     // 1: the contraction is never split over float atomics (sums in a fixed order)
  int a_k_pad_zero;       // NN only: A's rows hold zeros from column K up to K rounded up to 64 (lda covers them)
  // Optional: events that receive the start and the end of the kernel itself (hipExtLaunchKernelGGL), without the
  // barrier packets a recorded event puts between kernels.  Honoured by the direct-to-LDS kernel only.
  hipEvent_t ev_start, ev_stop;
};
int gemm_simple(hipStream_t s, int dtype, const GemmArgs& a);
int gemm_bf16_mfma(hipStream_t s, const GemmArgs& a);
int gemm_bf16_dtl(hipStream_t s, const GemmArgs& a);   // POPLAR_ERR_UNIMPLEMENTED when the shape is outside its preconditions
// up to four problems of one layout and one K in a single launch (two when their K is cut in two halves); POPLAR_ERR_UNIMPLEMENTED (nothing launched) when it cannot
int gemm_bf16_dtl_group(hipStream_t s, const GemmArgs* a, int n);
bool gemm_bf16_dtl_accepts(const GemmArgs* a, int n);   // preconditions only, nothing launched
int gemm(hipStream_t s, int dtype, const GemmArgs& a);

// attention on the fused qkv activation [B*S, 3H]; o [B*S, H]; lse float [B, nh, S]
int attn_fwd_simple(hipStream_t s, int dtype, int B, int S, int nh, int d, int causal, const void* qkv, void* o, float* lse);
int attn_bwd_simple(hipStream_t s, int dtype, int B, int S, int nh, int d, int causal, const void* qkv, const void* o,
                    const void* dout, const float* lse, void* dqkv, float* delta);
// ev_start / ev_stop (optional): receive the start of the first and the end of the last kernel launched
int attn_fwd_flash(hipStream_t s, int B, int S, int nh, int d, int causal, const void* qkv, void* o, float* lse,
                   hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
int attn_bwd_flash(hipStream_t s, int B, int S, int nh, int d, int causal, const void* qkv, const void* o,
                   const void* dout, const float* lse, void* dqkv, float* delta, hipEvent_t ev_start = nullptr,
                   hipEvent_t ev_stop = nullptr);

// row-wise / elementwise kernels (elementwise.hip)
int layernorm_fwd(hipStream_t s, int dtype, int64_t T, int H, const void* x, const void* g, const void* b, void* y, float* stats, int rms);
// dx = (dres ? dres : 0) + norm_bwd(dy); partial dgamma/dbeta to `partials` (float [nblk, 2, H]); then reduced into dg/db
int layernorm_bwd(hipStream_t s, int dtype, int64_t T, int H, const void* dy, const void* x, const void* g, const float* stats,
                  const void* dres, void* dx, float* dg, float* db, int accumulate, float* partials, int64_t partials_elems, int rms);
// Deferred second pass of the two-pass column reductions: out[j] (+)= sum over nchunks rows of partials
// (row stride `stride`); columns [0, n0) go to out0, [n0, n) to out1.  n == 0: nothing to do.
struct ReduceJob { const float* partials; int nchunks; int64_t stride; float* out0; float* out1; int64_t n0, n; };
#define REDUCE_MAX_JOBS 8
int reduce_group(hipStream_t s, const ReduceJob* jobs, int n, int accumulate);   // one launch for all jobs
// as layernorm_bwd, but leaves the reduction of dgamma / dbeta to the caller (*job)
int layernorm_bwd_partial(hipStream_t s, int dtype, int64_t T, int H, const void* dy, const void* x, const void* g, const float* stats,
                          const void* dres, void* dx, float* dg, float* db, float* partials, int64_t partials_elems, int rms, ReduceJob* job);
struct ColsumProblem { const void* x; int64_t ldx, N; float* out; };
#define COLSUM_MAX_GROUP 4
// first pass of up to four column sums over matrices of T rows in one launch; jobs[i] finishes problem i
int colsum_partial(hipStream_t s, int dtype, int64_t T, const ColsumProblem* p, int n, float* partials, int64_t partials_elems,
                   ReduceJob* jobs);
int colsum(hipStream_t s, int dtype, int64_t T, int64_t N, const void* x, int64_t ldx, float* out, int accumulate,
           float* partials, int64_t partials_elems);
int swiglu_fwd(hipStream_t s, int dtype, int64_t T, int F, const void* hgu, void* g);
int swiglu_bwd(hipStream_t s, int dtype, int64_t T, int F, const void* dg, const void* hgu, void* dhgu);
int rope_inplace(hipStream_t s, int dtype, int B, int S, int nh, int d, void* qkv, int64_t ld, float sign);
int embed_fwd(hipStream_t s, int dtype, int B, int S, int H, int V, const int32_t* tok, int64_t tok_ld, const void* wte, const void* wpe, void* x);
// ordered = 1: the embedding-matrix rows are summed token by token in sequence order (no atomics)
int embed_bwd(hipStream_t s, int dtype, int B, int S, int H, int V, const int32_t* tok, int64_t tok_ld, const void* dx, float* dwte, float* dwpe, int accumulate,
              int ordered = 0);
int xent_fwd_bwd(hipStream_t s, int dtype, int64_t T, int V, int64_t ld, void* logits, const int32_t* targets, int64_t tgt_ld, int S,
                 float loss_scale, float* loss, float* row_loss);
int adam_shard(hipStream_t s, int lowp_dtype, float* p, float* m, float* v, const float* g, void* p_lowp, int64_t n,
               int step_t, float lr, float b1, float b2, float eps);
// ev_start / ev_stop: optional events carried by the launches (kernel start / kernel end); *launched: whether anything ran
int zero2_reduce_local(hipStream_t s, float* gshard, const float* g_unit, int64_t unit_lo, int64_t unit_hi, int64_t shard_off, int64_t shard_len,
                       hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, int* launched = nullptr);
int zero3_gather_local(hipStream_t s, int dtype, void* out, const void* own, const void* peers, int64_t lo, int64_t hi, int64_t shard_off, int64_t shard_len,
                       hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, int* launched = nullptr);
int fill_zero(hipStream_t s, void* p, int64_t bytes);
int fill_zero_2d(hipStream_t s, void* p, int64_t rows, int64_t cols, int64_t ld);   // rows x cols 32-bit words, row stride ld words
int cast_f32_to_lowp(hipStream_t s, int dtype, const float* in, void* out, int64_t n);
