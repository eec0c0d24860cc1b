// Plain LDS-tiled GEMM with float accumulation for the fp32 compute path.
// One kernel serves the three operand layouts through element strides:
//   A(m,k) = A[m*sam + k*sak],  B(k,n) = B[k*sbk + n*sbn].
// 64x64 output tile, K step 16, 256 threads, 4x4 outputs per thread.
#include "device_utils.h"

struct SimpleGemmParams {
  int64_t M, N, K;
  int64_t sam, sak, sbk, sbn, ldc, ldaux;
  int c_float, act;
  float beta;
};

template <typename T>
__global__ void __launch_bounds__(256) gemm_simple_kernel(const T* __restrict__ A, const T* __restrict__ B, void* __restrict__ Cv,
                                                           const T* __restrict__ bias, const T* __restrict__ residual,
                                                           T* __restrict__ aux, SimpleGemmParams p) {
  __shared__ float As[16][64 + 1];
  __shared__ float Bs[16][64 + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < p.K; k0 += 16) {
    for (int e = threadIdx.x; e < 64 * 16; e += 256) {
      // choose the fast index along the contiguous dimension of each operand
      int am, ak, bn, bk;
      if (p.sak == 1) { ak = e & 15; am = e >> 4; } else { am = e & 63; ak = e >> 6; }
      if (p.sbk == 1) { bk = e & 15; bn = e >> 4; } else { bn = e & 63; bk = e >> 6; }
      int64_t m = m0 + am, ka = k0 + ak, n = n0 + bn, kb = k0 + bk;
      As[ak][am] = (m < p.M && ka < p.K) ? to_float<T>(A[m * p.sam + ka * p.sak]) : 0.f;
      Bs[bk][bn] = (n < p.N && kb < p.K) ? to_float<T>(B[kb * p.sbk + n * p.sbn]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int64_t m = m0 + ty * 4 + i;
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t n = n0 + tx * 4 + j;
      if (n >= p.N) continue;
      float v = acc[i][j];
      if (bias) v += to_float<T>(bias[n]);
      if (p.act == ACT_GELU) { aux[m * p.ldaux + n] = from_float<T>(gelu_tanh_grad(v)); v = gelu_tanh(v); }
      else if (p.act == ACT_GELU_BWD) v *= to_float<T>(aux[m * p.ldaux + n]);
      if (residual) v += to_float<T>(residual[m * p.ldc + n]);
      if (p.c_float) {
        float* C = reinterpret_cast<float*>(Cv);
        C[m * p.ldc + n] = p.beta != 0.f ? v + p.beta * C[m * p.ldc + n] : v;
      } else {
        reinterpret_cast<T*>(Cv)[m * p.ldc + n] = from_float<T>(v);
      }
    }
  }
}

int gemm_simple(hipStream_t s, int dtype, const GemmArgs& a) {
  poplar_gemm_kernel_launches += 1;
  if (a.M == 0 || a.N == 0) return POPLAR_OK;
  SimpleGemmParams p;
  p.M = a.M; p.N = a.N; p.K = a.K;
  switch (a.layout) {
    case GEMM_NT: p.sam = a.lda; p.sak = 1; p.sbk = 1; p.sbn = a.ldb; break;
    case GEMM_NN: p.sam = a.lda; p.sak = 1; p.sbk = a.ldb; p.sbn = 1; break;
    case GEMM_TN: p.sam = 1; p.sak = a.lda; p.sbk = a.ldb; p.sbn = 1; break;
    default: return poplar_fail(POPLAR_ERR_INVALID, "unknown GEMM layout %d", a.layout);
  }
  p.ldc = a.ldc; p.ldaux = a.ldaux; p.c_float = a.c_float; p.act = a.act; p.beta = a.beta;
  dim3 grid((unsigned)cdiv(a.N, 64), (unsigned)cdiv(a.M, 64));
  if (dtype == POPLAR_BF16)
    hipLaunchKernelGGL(gemm_simple_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)a.A, (const bf16*)a.B, a.C, (const bf16*)a.bias,
                       (const bf16*)a.residual, (bf16*)a.aux, p);
  else
    hipLaunchKernelGGL(gemm_simple_kernel<float>, grid, dim3(256), 0, s, (const float*)a.A, (const float*)a.B, a.C, (const float*)a.bias,
                       (const float*)a.residual, (float*)a.aux, p);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
