// Plain attention kernels for the fp32 compute path (also usable with bf16
// storage).  One wavefront owns one query row (forward, dq) or one key row
// (dk, dv); scores of the row live in LDS.  No atomics: results do not depend
// on scheduling.  qkv is the fused projection output [B*S, 3H] with q | k | v
// in the three column thirds and head h in columns h*d .. (h+1)*d of each.
#include "device_utils.h"

template <typename T>
__device__ inline float dot_rows(const T* a, const T* b, int d) {
  float acc = 0.f;
  for (int c = 0; c < d; ++c) acc += to_float<T>(a[c]) * to_float<T>(b[c]);
  return acc;
}

// forward: o[i,:] = sum_j softmax_j(q_i . k_j * scale) v_j ; lse[i] = logsumexp_j
template <typename T>
__global__ void __launch_bounds__(256) attn_fwd_simple_kernel(const T* __restrict__ qkv, T* __restrict__ o, float* __restrict__ lse,
                                                               int B, int S, int nh, int d, int causal, float scale) {
  extern __shared__ float lds[];  // [4][S]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + wv;  // over B*nh*S
  if (row >= (int64_t)B * nh * S) return;
  const int i = (int)(row % S);
  const int h = (int)((row / S) % nh);
  const int64_t b = row / ((int64_t)S * nh);
  const int H = nh * d;
  const int64_t ld = 3 * (int64_t)H;
  const T* q = qkv + (b * S + i) * ld + h * d;
  const T* kbase = qkv + (b * S) * ld + H + h * d;
  const T* vbase = kbase + H;
  float* sc = lds + wv * S;
  const int jend = causal ? i + 1 : S;
  float mx = -INFINITY;
  for (int j = lane; j < jend; j += 64) {
    float s = dot_rows(q, kbase + (int64_t)j * ld, d) * scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < jend; j += 64) {
    float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  wave_lds_sync();
  for (int c = lane; c < d; c += 64) {
    float acc = 0.f;
    for (int j = 0; j < jend; ++j) acc += sc[j] * to_float<T>(vbase[(int64_t)j * ld + c]);
    o[(b * S + i) * H + h * d + c] = from_float<T>(acc / sum);
  }
  if (lane == 0) lse[(b * nh + h) * S + i] = mx + logf(sum);
}

// delta[b,h,i] = sum_c dout[i,c] * o[i,c]
template <typename T>
__global__ void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ dout, float* __restrict__ delta, int B, int S, int nh, int d) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= (int64_t)B * nh * S) return;
  const int i = (int)(row % S);
  const int h = (int)((row / S) % nh);
  const int64_t b = row / ((int64_t)S * nh);
  const int64_t base = (b * S + i) * (int64_t)(nh * d) + h * d;
  float acc = 0.f;
  for (int c = lane; c < d; c += 64) acc += to_float<T>(o[base + c]) * to_float<T>(dout[base + c]);
  acc = wave_sum(acc);
  if (lane == 0) delta[(b * nh + h) * S + i] = acc;
}

// dq_i = scale * sum_j ds_ij k_j,  ds_ij = p_ij (dout_i . v_j - delta_i)
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_dq_simple_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                                  const float* __restrict__ lse, const float* __restrict__ delta,
                                                                  T* __restrict__ dqkv, int B, int S, int nh, int d, int causal, float scale) {
  extern __shared__ float lds[];  // [4][S]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + wv;
  if (row >= (int64_t)B * nh * S) return;
  const int i = (int)(row % S);
  const int h = (int)((row / S) % nh);
  const int64_t b = row / ((int64_t)S * nh);
  const int H = nh * d;
  const int64_t ld = 3 * (int64_t)H;
  const T* q = qkv + (b * S + i) * ld + h * d;
  const T* kbase = qkv + (b * S) * ld + H + h * d;
  const T* vbase = kbase + H;
  const T* doi = dout + (b * S + i) * H + h * d;
  const float l = lse[(b * nh + h) * S + i], dl = delta[(b * nh + h) * S + i];
  float* ds = lds + wv * S;
  const int jend = causal ? i + 1 : S;
  for (int j = lane; j < jend; j += 64) {
    float p = expf(dot_rows(q, kbase + (int64_t)j * ld, d) * scale - l);
    float dp = dot_rows(doi, vbase + (int64_t)j * ld, d);
    ds[j] = p * (dp - dl);
  }
  wave_lds_sync();
  for (int c = lane; c < d; c += 64) {
    float acc = 0.f;
    for (int j = 0; j < jend; ++j) acc += ds[j] * to_float<T>(kbase[(int64_t)j * ld + c]);
    dqkv[(b * S + i) * ld + h * d + c] = from_float<T>(acc * scale);
  }
}

// dk_j = scale * sum_i ds_ij q_i,  dv_j = sum_i p_ij dout_i   (i >= j when causal)
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_dkv_simple_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                                   const float* __restrict__ lse, const float* __restrict__ delta,
                                                                   T* __restrict__ dqkv, int B, int S, int nh, int d, int causal, float scale) {
  extern __shared__ float lds[];  // [4][2][S]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + wv;
  if (row >= (int64_t)B * nh * S) return;
  const int j = (int)(row % S);
  const int h = (int)((row / S) % nh);
  const int64_t b = row / ((int64_t)S * nh);
  const int H = nh * d;
  const int64_t ld = 3 * (int64_t)H;
  const T* qbase = qkv + (b * S) * ld + h * d;
  const T* kj = qkv + (b * S + j) * ld + H + h * d;
  const T* vj = kj + H;
  const T* dobase = dout + (b * S) * H + h * d;
  float* pp = lds + wv * 2 * S;
  float* ds = pp + S;
  const int ibeg = causal ? j : 0;
  for (int i = ibeg + lane; i < S; i += 64) {
    float p = expf(dot_rows(qbase + (int64_t)i * ld, kj, d) * scale - lse[(b * nh + h) * S + i]);
    float dp = dot_rows(dobase + (int64_t)i * H, vj, d);
    pp[i] = p;
    ds[i] = p * (dp - delta[(b * nh + h) * S + i]);
  }
  wave_lds_sync();
  for (int c = lane; c < d; c += 64) {
    float ak = 0.f, av = 0.f;
    for (int i = ibeg; i < S; ++i) {
      ak += ds[i] * to_float<T>(qbase[(int64_t)i * ld + c]);
      av += pp[i] * to_float<T>(dobase[(int64_t)i * H + c]);
    }
    dqkv[(b * S + j) * ld + H + h * d + c] = from_float<T>(ak * scale);
    dqkv[(b * S + j) * ld + 2 * H + h * d + c] = from_float<T>(av);
  }
}

static int check_simple(int S) {
  if ((size_t)8 * S * sizeof(float) > 64 * 1024) return poplar_fail(POPLAR_ERR_INVALID, "fp32 attention path supports seq <= 2048, got %d", S);
  return POPLAR_OK;
}

int attn_fwd_simple(hipStream_t s, int dtype, int B, int S, int nh, int d, int causal, const void* qkv, void* o, float* lse) {
  POPLAR_TRY(check_simple(S));
  int64_t rows = (int64_t)B * nh * S;
  if (rows == 0) return POPLAR_OK;
  float scale = 1.0f / sqrtf((float)d);
  size_t lds = (size_t)4 * S * sizeof(float);
  if (dtype == POPLAR_BF16)
    hipLaunchKernelGGL(attn_fwd_simple_kernel<bf16>, dim3((unsigned)cdiv(rows, 4)), dim3(256), lds, s, (const bf16*)qkv, (bf16*)o, lse, B, S, nh, d, causal, scale);
  else
    hipLaunchKernelGGL(attn_fwd_simple_kernel<float>, dim3((unsigned)cdiv(rows, 4)), dim3(256), lds, s, (const float*)qkv, (float*)o, lse, B, S, nh, d, causal, scale);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int attn_bwd_simple(hipStream_t s, int dtype, int B, int S, int nh, int d, int causal, const void* qkv, const void* o,
                    const void* dout, const float* lse, void* dqkv, float* delta) {
  POPLAR_TRY(check_simple(S));
  int64_t rows = (int64_t)B * nh * S;
  if (rows == 0) return POPLAR_OK;
  float scale = 1.0f / sqrtf((float)d);
  dim3 grid((unsigned)cdiv(rows, 4));
  size_t lds1 = (size_t)4 * S * sizeof(float), lds2 = 2 * lds1;
  if (dtype == POPLAR_BF16) {
    hipLaunchKernelGGL(attn_delta_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)o, (const bf16*)dout, delta, B, S, nh, d);
    hipLaunchKernelGGL(attn_bwd_dq_simple_kernel<bf16>, grid, dim3(256), lds1, s, (const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, B, S, nh, d, causal, scale);
    hipLaunchKernelGGL(attn_bwd_dkv_simple_kernel<bf16>, grid, dim3(256), lds2, s, (const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, B, S, nh, d, causal, scale);
  } else {
    hipLaunchKernelGGL(attn_delta_kernel<float>, grid, dim3(256), 0, s, (const float*)o, (const float*)dout, delta, B, S, nh, d);
    hipLaunchKernelGGL(attn_bwd_dq_simple_kernel<float>, grid, dim3(256), lds1, s, (const float*)qkv, (const float*)dout, lse, delta, (float*)dqkv, B, S, nh, d, causal, scale);
    hipLaunchKernelGGL(attn_bwd_dkv_simple_kernel<float>, grid, dim3(256), lds2, s, (const float*)qkv, (const float*)dout, lse, delta, (float*)dqkv, B, S, nh, d, causal, scale);
  }
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
