// HBM-bound kernels of the training step: Adam on a shard, the single-rank
// share of the ZeRO-2 / ZeRO-3 collectives, LayerNorm / RMSNorm forward and
// backward, column sums (bias gradients), SwiGLU, RoPE, embedding, and the
// softmax cross-entropy.  All use 16-byte accesses per lane and 64-lane
// wavefront reductions; math is float whatever the storage type.
#include <hip/hip_ext.h>
#include "device_utils.h"
#include <algorithm>
#include <type_traits>

#define DISPATCH_DTYPE(dtype, ...)                                         \
  do {                                                                      \
    if ((dtype) == POPLAR_BF16) { typedef bf16 T; __VA_ARGS__; }            \
    else { typedef float T; __VA_ARGS__; }                                  \
  } while (0)

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
// Streaming kernels get one work item per thread up to a very large grid: measured on a 4 GB Adam update,
// 131072 blocks walking memory in block order reach 6.0 TB/s where 8192 blocks in a grid-stride loop reach 4.7.
static inline int grid_for(int64_t work_items, int block, int max_blocks = 1 << 20) {
  int64_t g = cdiv(work_items, block);
  if (g < 1) g = 1;
  if (g > max_blocks) g = max_blocks;
  return (int)g;
}

// ---------------------------------------------------------------------------
// fill
// ---------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint32_t* p, int64_t n_words) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n_words; i += stride) p[i] = 0u;
}
int fill_zero(hipStream_t s, void* p, int64_t bytes) {
  if (bytes == 0) return POPLAR_OK;
  if (bytes % 4 || ((uintptr_t)p & 3)) return poplar_fail(POPLAR_ERR_INVALID, "fill_zero needs 4-byte granularity");
  int64_t n = bytes / 4;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, (uint32_t*)p, n);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

// rows x cols 32-bit words at row stride ld (words), in one launch: blockIdx.y walks the rows
__global__ void fill_zero_2d_kernel(uint32_t* p, int64_t rows, int64_t cols, int64_t ld) {
  for (int64_t r = blockIdx.y; r < rows; r += gridDim.y)
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cols; i += (int64_t)gridDim.x * blockDim.x) p[r * ld + i] = 0u;
}
int fill_zero_2d(hipStream_t s, void* p, int64_t rows, int64_t cols, int64_t ld) {
  if (rows <= 0 || cols <= 0) return POPLAR_OK;
  if ((uintptr_t)p & 3) return poplar_fail(POPLAR_ERR_INVALID, "fill_zero_2d needs 4-byte alignment");
  if (ld < cols) return poplar_fail(POPLAR_ERR_INVALID, "fill_zero_2d: row stride below the row length");
  const dim3 grid((unsigned)std::min<int64_t>(cdiv(cols, 256), 64), (unsigned)std::min<int64_t>(rows, 16384));
  hipLaunchKernelGGL(fill_zero_2d_kernel, grid, dim3(256), 0, s, (uint32_t*)p, rows, cols, ld);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

template <typename T>
__global__ void cast_kernel(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = from_float<T>(in[i]);
}
int cast_f32_to_lowp(hipStream_t s, int dtype, const float* in, void* out, int64_t n) {
  if (n == 0) return POPLAR_OK;
  DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(cast_kernel<T>, dim3(grid_for(n, 256)), dim3(256), 0, s, in, (T*)out, n));
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

// ---------------------------------------------------------------------------
// Adam on a shard.  Per element: read g, p, m, v (16 B), write p, m, v (12 B)
// and the rounded low-precision copy (2 B for bf16).
// ---------------------------------------------------------------------------
struct AdamConst { float lr, b1, b2, eps, omb1, omb2, inv_bc1, inv_bc2; };

__device__ inline void adam_one(float g, float& p, float& m, float& v, const AdamConst& c) {
  // explicit roundings: every element sees the same operations whichever
  // kernel (vector body, scalar tail) or shard it falls in
  m = __fmaf_rn(c.b1, m, __fmul_rn(c.omb1, g));
  v = __fmaf_rn(c.b2, v, __fmul_rn(__fmul_rn(c.omb2, g), g));
  float mhat = __fmul_rn(m, c.inv_bc1);
  float vhat = __fmul_rn(v, c.inv_bc2);
  p = __fsub_rn(p, __fdiv_rn(__fmul_rn(c.lr, mhat), __fadd_rn(__fsqrt_rn(vhat), c.eps)));
}

template <typename L, bool HAS_LOWP>
__global__ void __launch_bounds__(256) adam_vec_kernel(float* __restrict__ p, float* __restrict__ m, float* __restrict__ v,
                                                        const float* __restrict__ g, L* __restrict__ lowp, int64_t n4, AdamConst c) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) {
    float4 gg = nt_load4(g, i);
    float4 pp = nt_load4(p, i);
    float4 mm = nt_load4(m, i);
    float4 vv = nt_load4(v, i);
    adam_one(gg.x, pp.x, mm.x, vv.x, c);
    adam_one(gg.y, pp.y, mm.y, vv.y, c);
    adam_one(gg.z, pp.z, mm.z, vv.z, c);
    adam_one(gg.w, pp.w, mm.w, vv.w, c);
    nt_store4(p, i, pp);
    nt_store4(m, i, mm);
    nt_store4(v, i, vv);
    if (HAS_LOWP) {
      if (sizeof(L) == 2) {
        uint2 w;
        w.x = float_to_bf16_bits(pp.x) | (float_to_bf16_bits(pp.y) << 16);
        w.y = float_to_bf16_bits(pp.z) | (float_to_bf16_bits(pp.w) << 16);
        nt_store2(reinterpret_cast<uint32_t*>(lowp), i, w);
      } else {
        nt_store4(reinterpret_cast<float*>(lowp), i, pp);
      }
    }
  }
}

template <typename L, bool HAS_LOWP>
__global__ void adam_scalar_kernel(float* __restrict__ p, float* __restrict__ m, float* __restrict__ v,
                                   const float* __restrict__ g, L* __restrict__ lowp, int64_t begin, int64_t n, AdamConst c) {
  int64_t i = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    float pp = p[i], mm = m[i], vv = v[i];
    adam_one(g[i], pp, mm, vv, c);
    p[i] = pp; m[i] = mm; v[i] = vv;
    if (HAS_LOWP) lowp[i] = from_float<L>(pp);
  }
}

template <typename L, bool HAS_LOWP>
static int adam_launch(hipStream_t s, float* p, float* m, float* v, const float* g, L* lowp, int64_t n, const AdamConst& c) {
  bool vec = aligned16(p) && aligned16(m) && aligned16(v) && aligned16(g) && (!HAS_LOWP || ((uintptr_t)lowp & 15) == 0);
  int64_t n4 = vec ? n / 4 : 0;
  if (n4 > 0) {
    hipLaunchKernelGGL((adam_vec_kernel<L, HAS_LOWP>), dim3(grid_for(n4, 256)), dim3(256), 0, s, p, m, v, g, lowp, n4, c);
    POPLAR_LAUNCH_CHECK();
  }
  if (n4 * 4 < n) {
    hipLaunchKernelGGL((adam_scalar_kernel<L, HAS_LOWP>), dim3(grid_for(n - n4 * 4, 256)), dim3(256), 0, s, p, m, v, g, lowp, n4 * 4, n, c);
    POPLAR_LAUNCH_CHECK();
  }
  return POPLAR_OK;
}

int adam_shard(hipStream_t s, int lowp_dtype, float* p, float* m, float* v, const float* g, void* p_lowp, int64_t n,
               int step_t, float lr, float b1, float b2, float eps) {
  if (n == 0) return POPLAR_OK;
  AdamConst c;
  c.lr = lr; c.b1 = b1; c.b2 = b2; c.eps = eps;
  c.omb1 = 1.0f - b1; c.omb2 = 1.0f - b2;
  c.inv_bc1 = (float)(1.0 / (1.0 - pow((double)b1, (double)step_t)));
  c.inv_bc2 = (float)(1.0 / (1.0 - pow((double)b2, (double)step_t)));
  if (!p_lowp) return adam_launch<float, false>(s, p, m, v, g, (float*)nullptr, n, c);
  if (lowp_dtype == POPLAR_BF16) return adam_launch<bf16, true>(s, p, m, v, g, (bf16*)p_lowp, n, c);
  return adam_launch<float, true>(s, p, m, v, g, (float*)p_lowp, n, c);
}

// ---------------------------------------------------------------------------
// ZeRO-2 local reduce and ZeRO-3 local gather
// ---------------------------------------------------------------------------
__global__ void axpy_vec_kernel(float* __restrict__ dst, const float* __restrict__ src, int64_t n4) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) {
    float4 a = reinterpret_cast<float4*>(dst)[i];
    float4 b = nt_load4(src, i);
    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    reinterpret_cast<float4*>(dst)[i] = a;
  }
}
__global__ void axpy_scalar_kernel(float* __restrict__ dst, const float* __restrict__ src, int64_t begin, int64_t n) {
  int64_t i = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] += src[i];
}

// ev_start / ev_stop (both or neither): events that ride on the launches themselves and receive the first kernel's
// start and the last kernel's end, so that a timed span holds the kernels and nothing else.  *launched tells the
// caller whether anything ran (an empty intersection launches nothing and leaves the events untouched).
int zero2_reduce_local(hipStream_t s, float* gshard, const float* g_unit, int64_t unit_lo, int64_t unit_hi,
                       int64_t shard_off, int64_t shard_len, hipEvent_t ev_start, hipEvent_t ev_stop, int* launched) {
  if (launched) *launched = 0;
  int64_t lo = unit_lo > shard_off ? unit_lo : shard_off;
  int64_t hi = unit_hi < shard_off + shard_len ? unit_hi : shard_off + shard_len;
  if (hi <= lo) return POPLAR_OK;
  float* dst = gshard + (lo - shard_off);
  const float* src = g_unit + (lo - unit_lo);
  int64_t n = hi - lo;
  int64_t n4 = (aligned16(dst) && aligned16(src)) ? n / 4 : 0;
  const bool tail = n4 * 4 < n;
  if (n4 > 0) {
    hipExtLaunchKernelGGL(axpy_vec_kernel, dim3(grid_for(n4, 256)), dim3(256), 0, s, ev_start, tail ? nullptr : ev_stop, 0, dst, src, n4);
    POPLAR_LAUNCH_CHECK();
  }
  if (tail) {
    hipExtLaunchKernelGGL(axpy_scalar_kernel, dim3(grid_for(n - n4 * 4, 256)), dim3(256), 0, s, n4 > 0 ? nullptr : ev_start, ev_stop, 0,
                          dst, src, n4 * 4, n);
    POPLAR_LAUNCH_CHECK();
  }
  if (launched) *launched = 1;
  return POPLAR_OK;
}

// out[i - lo] = (i in own shard) ? own[i - shard_off] : peers[i]; W = words of 16 or 2/4 bytes
template <typename W>
__global__ void gather_kernel(W* __restrict__ out, const W* __restrict__ own, const W* __restrict__ peers,
                              int64_t lo, int64_t n, int64_t own_lo, int64_t own_hi) {
  // all indices in units of W; own_lo/own_hi are the shard bounds in the same units
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int64_t f = lo + i;
    out[i] = (f >= own_lo && f < own_hi) ? own[f - own_lo] : peers[f];
  }
}

int zero3_gather_local(hipStream_t s, int dtype, void* out, const void* own, const void* peers, int64_t lo, int64_t hi,
                       int64_t shard_off, int64_t shard_len, hipEvent_t ev_start, hipEvent_t ev_stop, int* launched) {
  if (launched) *launched = 0;
  if (hi <= lo) return POPLAR_OK;
  const int64_t es = elt_size(dtype);
  const int64_t per = 16 / es;  // elements per 16-byte word
  int64_t n = hi - lo;
  bool vec = aligned16(out) && aligned16(own) && aligned16(peers) && lo % per == 0 && n % per == 0 &&
             shard_off % per == 0 && shard_len % per == 0;
  if (vec) {
    hipExtLaunchKernelGGL(gather_kernel<uint4>, dim3(grid_for(n / per, 256)), dim3(256), 0, s, ev_start, ev_stop, 0, (uint4*)out, (const uint4*)own,
                          (const uint4*)peers, lo / per, n / per, shard_off / per, (shard_off + shard_len) / per);
  } else if (es == 2) {
    hipExtLaunchKernelGGL(gather_kernel<uint16_t>, dim3(grid_for(n, 256)), dim3(256), 0, s, ev_start, ev_stop, 0, (uint16_t*)out, (const uint16_t*)own,
                          (const uint16_t*)peers, lo, n, shard_off, shard_off + shard_len);
  } else {
    hipExtLaunchKernelGGL(gather_kernel<uint32_t>, dim3(grid_for(n, 256)), dim3(256), 0, s, ev_start, ev_stop, 0, (uint32_t*)out, (const uint32_t*)own,
                          (const uint32_t*)peers, lo, n, shard_off, shard_off + shard_len);
  }
  POPLAR_LAUNCH_CHECK();
  if (launched) *launched = 1;
  return POPLAR_OK;
}

// ---------------------------------------------------------------------------
// LayerNorm / RMSNorm.  One wavefront per row, the row held in registers
// (NV 16-byte vectors per lane), so x is read from HBM once.
// stats: float [T, 2] = (mean, rstd); RMSNorm stores mean = 0.
//
// A wave walks rows wave, wave + nwaves, ... with the row after the current one already requested: two register
// sets take turns inside a loop body that handles two rows and has no branch in it (a row that does not exist is a
// descriptor of zero bytes: its loads return zeros, its stores go nowhere), every load and store goes through a row
// descriptor and is issued unconditionally (see span_rsrc), and before the loop a row's worth of stores is issued to
// nowhere, so that the loop is entered with the same operations in flight as it is re-entered with.  The waits the
// compiler then places let the next row's loads and the previous row's stores stay in flight.
// ---------------------------------------------------------------------------
template <typename T, int NV, bool RMS>
__global__ void __launch_bounds__(256) norm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ g, const T* __restrict__ b,
                                                        T* __restrict__ y, float* __restrict__ stats, int64_t rows, int H) {
  constexpr int VN = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  if (wave >= rows) return;
  const uint32_t row_bytes = (uint32_t)H * sizeof(T);
  const float inv_h = 1.0f / (float)H;
  Vec<T> gam[NV], bet[NV];
  {
    const __amdgpu_buffer_rsrc_t rg = span_rsrc(g, row_bytes), rb = span_rsrc(RMS ? g : b, row_bytes);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      span_load<T>(gam[i], rg, (uint32_t)(i * 64 + lane) * 16);
      if (!RMS) span_load<T>(bet[i], rb, (uint32_t)(i * 64 + lane) * 16);
    }
  }
  // row r if it exists, else nothing: the address stays inside the tensor either way
  auto fetch = [&](Vec<T> (&q)[NV], int64_t r) __attribute__((always_inline)) {
    const bool have = r < rows;
    const __amdgpu_buffer_rsrc_t rs = span_rsrc(x + (have ? r : 0) * H, have ? row_bytes : 0u);
    __builtin_amdgcn_sched_barrier(0);   // the loads go out here, in this order: not after the arithmetic they are meant to overlap
#pragma unroll
    for (int i = 0; i < NV; ++i) span_load<T>(q[i], rs, (uint32_t)(i * 64 + lane) * 16);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto work = [&](Vec<T> (&q)[NV], int64_t r) __attribute__((always_inline)) {
    const bool have = r < rows;
    float f[NV][VN];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      q[i].unpack(f[i]);   // lanes past the row's end hold zeros
#pragma unroll
      for (int k = 0; k < VN; ++k) sum += RMS ? f[i][k] * f[i][k] : f[i][k];
    }
    sum = wave_sum(sum);
    float mean = 0.f, var;
    if (RMS) {
      var = sum * inv_h;
    } else {
      mean = sum * inv_h;
      float sq = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const bool in = (i * 64 + lane) * VN < H;
#pragma unroll
        for (int k = 0; k < VN; ++k) { const float d = in ? f[i][k] - mean : 0.f; sq += d * d; }
      }
      var = wave_sum(sq) * inv_h;
    }
    const float rstd = 1.0f / sqrtf(var + 1e-5f);
    span_store_f2(mean, rstd, span_rsrc(stats + 2 * (have ? r : 0), have ? 8u : 0u), (uint32_t)lane * 8);
    const __amdgpu_buffer_rsrc_t ry = span_rsrc(y + (have ? r : 0) * H, have ? row_bytes : 0u);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float gg[VN], bb[VN], o[VN];
      gam[i].unpack(gg);
      if (!RMS) bet[i].unpack(bb);
#pragma unroll
      for (int k = 0; k < VN; ++k) o[k] = (f[i][k] - mean) * rstd * gg[k] + (RMS ? 0.f : bb[k]);
      Vec<T> v; v.pack(o);
      span_store<T>(v, ry, (uint32_t)(i * 64 + lane) * 16);
    }
  };
  Vec<T> qa[NV], qb[NV];
  // rows r and r + nwaves; qa holds row r on entry and row r + 2 nwaves on exit
  auto pair = [&](int64_t r) __attribute__((always_inline)) {
    fetch(qb, r + nwaves);
    work(qa, r);
    fetch(qa, r + 2 * nwaves);
    work(qb, r + nwaves);
  };
  int64_t r = wave;
  fetch(qa, r);
  {
    // as many stores as work() issues, through a descriptor of zero bytes: they go nowhere, and the loop is entered
    // with the same sequence of operations behind qa's loads as it is re-entered with
    const __amdgpu_buffer_rsrc_t none = span_rsrc(y, 0u);
    Vec<T> z; float zf[VN];
#pragma unroll
    for (int k = 0; k < VN; ++k) zf[k] = 0.f;
    z.pack(zf);
    span_store_f2(0.f, 0.f, none, 0u);
#pragma unroll
    for (int i = 0; i < NV; ++i) span_store<T>(z, none, (uint32_t)i * 16);   // distinct offsets: identical stores would be merged
    __builtin_amdgcn_sched_barrier(0);
  }
  do {
    pair(r);
    r += 2 * nwaves;
  } while (r < rows);
}

// Rows too long for two register sets (NV = 16): one row at a time.
template <typename T, int NV, bool RMS>
__global__ void __launch_bounds__(256) norm_fwd_long_kernel(const T* __restrict__ x, const T* __restrict__ g, const T* __restrict__ b,
                                                             T* __restrict__ y, float* __restrict__ stats, int64_t rows, int H) {
  constexpr int VN = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t r = wave; r < rows; r += nwaves) {
    const T* xr = x + r * H;
    float f[NV][VN];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int c = (i * 64 + lane) * VN;
      if (c < H) {
        Vec<T> v; v.load(xr + c); v.unpack(f[i]);
#pragma unroll
        for (int k = 0; k < VN; ++k) sum += RMS ? f[i][k] * f[i][k] : f[i][k];
      }
    }
    sum = wave_sum(sum);
    float mean = 0.f, var;
    if (RMS) {
      var = sum / H;
    } else {
      mean = sum / H;
      float sq = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        int c = (i * 64 + lane) * VN;
        if (c < H) {
#pragma unroll
          for (int k = 0; k < VN; ++k) { float d = f[i][k] - mean; sq += d * d; }
        }
      }
      var = wave_sum(sq) / H;
    }
    float rstd = 1.0f / sqrtf(var + 1e-5f);
    if (lane == 0) { stats[2 * r] = mean; stats[2 * r + 1] = rstd; }
    T* yr = y + r * H;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int c = (i * 64 + lane) * VN;
      if (c < H) {
        float gg[VN], bb[VN], o[VN];
        Vec<T> v; v.load(g + c); v.unpack(gg);
        if (!RMS) { v.load(b + c); v.unpack(bb); }
#pragma unroll
        for (int k = 0; k < VN; ++k) o[k] = (f[i][k] - mean) * rstd * gg[k] + (RMS ? 0.f : bb[k]);
        v.pack(o); v.store(yr + c);
      }
    }
  }
}

// Waves per CU that keep about 96 KB of rows in flight (two rows per wave), in blocks of four waves over 256 CUs,
// but never fewer than two rows per wave's walk where the rows allow it.
static int norm_fwd_blocks(int64_t rows, int64_t row_bytes) {
  int64_t per_cu = cdiv(96 * 1024, 2 * row_bytes * 4);   // blocks per CU
  if (per_cu < 1) per_cu = 1;
  if (per_cu > 6) per_cu = 6;
  int64_t blocks = per_cu * 256;
  if (blocks > cdiv(rows, 8)) blocks = cdiv(rows, 8);
  return (int)(blocks < 1 ? 1 : blocks);
}

template <typename T, bool RMS>
static int norm_fwd_launch(hipStream_t s, int64_t rows, int H, const T* x, const T* g, const T* b, T* y, float* stats) {
  constexpr int VN = Vec<T>::N;
  int need = (int)cdiv(H, 64 * VN);
  int grid = norm_fwd_blocks(rows, (int64_t)H * sizeof(T));
#define NORM_FWD_CASE(NVV) \
  hipLaunchKernelGGL((norm_fwd_kernel<T, NVV, RMS>), dim3(grid), dim3(256), 0, s, x, g, b, y, stats, rows, H)
  if (need <= 1) NORM_FWD_CASE(1);
  else if (need <= 2) NORM_FWD_CASE(2);
  else if (need <= 4) NORM_FWD_CASE(4);
  else if (need <= 8) NORM_FWD_CASE(8);
  else if (need <= 16) hipLaunchKernelGGL((norm_fwd_long_kernel<T, 16, RMS>), dim3(grid_for(rows, 4)), dim3(256), 0, s, x, g, b, y, stats, rows, H);
  else return poplar_fail(POPLAR_ERR_INVALID, "hidden %d too large for the norm kernel", H);
#undef NORM_FWD_CASE
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int layernorm_fwd(hipStream_t s, int dtype, int64_t T_, int H, const void* x, const void* g, const void* b, void* y, float* stats, int rms) {
  if (T_ == 0) return POPLAR_OK;
  DISPATCH_DTYPE(dtype, {
    if (rms) return norm_fwd_launch<T, true>(s, T_, H, (const T*)x, (const T*)g, (const T*)b, (T*)y, stats);
    return norm_fwd_launch<T, false>(s, T_, H, (const T*)x, (const T*)g, (const T*)b, (T*)y, stats);
  });
  return POPLAR_OK;
}

// Backward: dx = dres + rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)),  dxhat = dy * gamma
// (RMSNorm drops the mean(dxhat) term).  Each wave walks rows r = wave, wave + nwaves, ...
// and keeps per-column partial sums of dy*xhat (dgamma) and dy (dbeta) in
// registers; the four waves of a block are added through LDS and the block
// writes one row of `partials` [nblocks, 2, H].
// The row loop is built like the forward kernel's: rows in pairs, two register sets, every access through a row
// descriptor (a row that does not exist, and a residual gradient that is not given, are descriptors of zero bytes
// and read as zeros, which add nothing to any sum).
template <typename T, int NV, bool RMS>
__global__ void __launch_bounds__(256) norm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x, const T* __restrict__ g,
                                                        const float* __restrict__ stats, const T* __restrict__ dres,
                                                        T* __restrict__ dx, float* __restrict__ partials, int64_t rows, int H) {
  constexpr int VN = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int wv = threadIdx.x >> 6;
  const int64_t wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + wv));
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  const uint32_t row_bytes = (uint32_t)H * sizeof(T);
  float accg[NV][VN], accb[NV][VN], gam[NV][VN];
  {
    const __amdgpu_buffer_rsrc_t rg = span_rsrc(g, row_bytes);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      Vec<T> v;
      span_load<T>(v, rg, (uint32_t)(i * 64 + lane) * 16);
      v.unpack(gam[i]);
#pragma unroll
      for (int k = 0; k < VN; ++k) { accg[i][k] = 0.f; accb[i][k] = 0.f; }
    }
  }
  struct RowRaw { Vec<T> x[NV], dy[NV], rs[NV]; float mean, rstd; };
  auto fetch = [&](RowRaw& q, int64_t r) __attribute__((always_inline)) {
    const bool have = r < rows;
    const int64_t rr = have ? r : 0;
    const __amdgpu_buffer_rsrc_t rx = span_rsrc(x + rr * H, have ? row_bytes : 0u), rd = span_rsrc(dy + rr * H, have ? row_bytes : 0u),
                                 rs = span_rsrc(dres ? dres + rr * H : x, have && dres ? row_bytes : 0u);
    q.mean = stats[2 * rr]; q.rstd = stats[2 * rr + 1];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const uint32_t off = (uint32_t)(i * 64 + lane) * 16;
      span_load<T>(q.x[i], rx, off);
      span_load<T>(q.dy[i], rd, off);
      span_load<T>(q.rs[i], rs, off);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto work = [&](RowRaw& cur, int64_t r) __attribute__((always_inline)) {
    const bool have = r < rows;
    const float mean = cur.mean, rstd = cur.rstd;
    float xh[NV][VN], dxh[NV][VN];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float xv[VN], dv[VN];
      cur.x[i].unpack(xv);
      cur.dy[i].unpack(dv);
#pragma unroll
      for (int k = 0; k < VN; ++k) {
        xh[i][k] = (xv[k] - mean) * rstd;
        dxh[i][k] = dv[k] * gam[i][k];
        accg[i][k] += dv[k] * xh[i][k];
        accb[i][k] += dv[k];
        s1 += dxh[i][k];
        s2 += dxh[i][k] * xh[i][k];
      }
    }
    s1 = RMS ? 0.f : wave_sum(s1) / H;
    s2 = wave_sum(s2) / H;
    const __amdgpu_buffer_rsrc_t ro = span_rsrc(dx + (have ? r : 0) * H, have ? row_bytes : 0u);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float o[VN], rs[VN];
      cur.rs[i].unpack(rs);
#pragma unroll
      for (int k = 0; k < VN; ++k) o[k] = rstd * (dxh[i][k] - s1 - xh[i][k] * s2) + rs[k];
      Vec<T> v; v.pack(o);
      span_store<T>(v, ro, (uint32_t)(i * 64 + lane) * 16);
    }
  };
  if (wave < rows) {
    RowRaw qa, qb;
    int64_t r = wave;
    fetch(qa, r);
    {
      // a row's worth of stores to nowhere: the loop is entered with the operations in flight it is re-entered with
      const __amdgpu_buffer_rsrc_t none = span_rsrc(dx, 0u);
      Vec<T> z; float zf[VN];
#pragma unroll
      for (int k = 0; k < VN; ++k) zf[k] = 0.f;
      z.pack(zf);
#pragma unroll
      for (int i = 0; i < NV; ++i) span_store<T>(z, none, (uint32_t)i * 16);   // distinct offsets: identical stores would be merged
      __builtin_amdgcn_sched_barrier(0);
    }
    do {
      fetch(qb, r + nwaves);
      work(qa, r);
      fetch(qa, r + 2 * nwaves);
      work(qb, r + nwaves);
      r += 2 * nwaves;
    } while (r < rows);
  }
  // block reduction of the per-wave column sums
  extern __shared__ float lds[];  // [4][2][H]
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * VN;
    if (c < H) {
#pragma unroll
      for (int k = 0; k < VN; ++k) {
        lds[(wv * 2 + 0) * H + c + k] = accg[i][k];
        lds[(wv * 2 + 1) * H + c + k] = accb[i][k];
      }
    }
  }
  __syncthreads();
  float* outp = partials + (int64_t)blockIdx.x * 2 * H;
  for (int j = threadIdx.x; j < 2 * H; j += 256)
    outp[j] = lds[j] + lds[2 * H + j] + lds[4 * H + j] + lds[6 * H + j];
}

// The same for wide rows (hidden above 1024), where a row no longer fits one wave's registers: a block of four
// waves per row, thread t owning vectors t, t + 256, ... (at most NVW); the two row sums cross the waves through
// LDS (one barrier per row, slots alternating); every column belongs to one thread, so the block's gamma / beta
// partial sums go straight from registers to `partials` [nblocks, 2, H] (beta half unused for RMSNorm).
template <typename T, int NVW, bool RMS>
__global__ void __launch_bounds__(256) norm_bwd_wide_kernel(const T* __restrict__ dy, const T* __restrict__ x, const T* __restrict__ g,
                                                             const float* __restrict__ stats, const T* __restrict__ dres,
                                                             T* __restrict__ dx, float* __restrict__ partials, int64_t rows, int H) {
  constexpr int VN = Vec<T>::N;
  const int wv = threadIdx.x >> 6;
  const uint32_t row_bytes = (uint32_t)H * sizeof(T);
  float accg[NVW][VN], accb[NVW][VN], gam[NVW][VN];
  {
    const __amdgpu_buffer_rsrc_t rg = span_rsrc(g, row_bytes);
#pragma unroll
    for (int i = 0; i < NVW; ++i) {
      Vec<T> v;
      span_load<T>(v, rg, (uint32_t)(i * 256 + threadIdx.x) * 16);
      v.unpack(gam[i]);
#pragma unroll
      for (int k = 0; k < VN; ++k) { accg[i][k] = 0.f; accb[i][k] = 0.f; }
    }
  }
  struct RowRaw { Vec<T> x[NVW], dy[NVW], rs[NVW]; float mean, rstd; };
  __shared__ float red[2][2][4];
  const int64_t step = gridDim.x;
  auto fetch = [&](RowRaw& q, int64_t r) __attribute__((always_inline)) {
    const bool have = r < rows;
    const int64_t rr = have ? r : 0;
    const __amdgpu_buffer_rsrc_t rx = span_rsrc(x + rr * H, have ? row_bytes : 0u), rd = span_rsrc(dy + rr * H, have ? row_bytes : 0u),
                                 rs = span_rsrc(dres ? dres + rr * H : x, have && dres ? row_bytes : 0u);
    q.mean = stats[2 * rr]; q.rstd = stats[2 * rr + 1];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NVW; ++i) {
      const uint32_t off = (uint32_t)(i * 256 + threadIdx.x) * 16;
      span_load<T>(q.x[i], rx, off);
      span_load<T>(q.dy[i], rd, off);
      span_load<T>(q.rs[i], rs, off);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // par: which of the two LDS slots this row uses; a wave cannot be two rows ahead of another (one barrier per row),
  // so the slots of a parity are free again when it writes them
  auto work = [&](RowRaw& cur, int64_t r, int par) __attribute__((always_inline)) {
    const bool have = r < rows;
    const float mean = cur.mean, rstd = cur.rstd;
    float xh[NVW][VN], dxh[NVW][VN];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NVW; ++i) {
      float xv[VN], dv[VN];
      cur.x[i].unpack(xv);
      cur.dy[i].unpack(dv);
#pragma unroll
      for (int k = 0; k < VN; ++k) {
        xh[i][k] = (xv[k] - mean) * rstd;
        dxh[i][k] = dv[k] * gam[i][k];
        accg[i][k] += dv[k] * xh[i][k];
        if (!RMS) accb[i][k] += dv[k];
        s1 += dxh[i][k];
        s2 += dxh[i][k] * xh[i][k];
      }
    }
    s1 = RMS ? 0.f : wave_sum(s1);
    s2 = wave_sum(s2);
    red[par][0][wv] = s1; red[par][1][wv] = s2;   // every lane of the wave writes the same two values: no branch in the row loop
    block_sync_lds();
    s1 = (red[par][0][0] + red[par][0][1] + red[par][0][2] + red[par][0][3]) / H;
    s2 = (red[par][1][0] + red[par][1][1] + red[par][1][2] + red[par][1][3]) / H;
    const __amdgpu_buffer_rsrc_t ro = span_rsrc(dx + (have ? r : 0) * H, have ? row_bytes : 0u);
#pragma unroll
    for (int i = 0; i < NVW; ++i) {
      float o[VN], rs[VN];
      cur.rs[i].unpack(rs);
#pragma unroll
      for (int k = 0; k < VN; ++k) o[k] = rstd * (dxh[i][k] - s1 - xh[i][k] * s2) + rs[k];
      Vec<T> v; v.pack(o);
      span_store<T>(v, ro, (uint32_t)(i * 256 + threadIdx.x) * 16);
    }
  };
  if ((int64_t)blockIdx.x < rows) {
    RowRaw qa, qb;
    int64_t r = blockIdx.x;
    fetch(qa, r);
    {
      const __amdgpu_buffer_rsrc_t none = span_rsrc(dx, 0u);
      Vec<T> z; float zf[VN];
#pragma unroll
      for (int k = 0; k < VN; ++k) zf[k] = 0.f;
      z.pack(zf);
#pragma unroll
      for (int i = 0; i < NVW; ++i) span_store<T>(z, none, (uint32_t)i * 16);   // distinct offsets: identical stores would be merged
      __builtin_amdgcn_sched_barrier(0);
    }
    do {
      fetch(qb, r + step);
      work(qa, r, 0);
      fetch(qa, r + 2 * step);
      work(qb, r + step, 1);
      r += 2 * step;
    } while (r < rows);
  }
  float* outp = partials + (int64_t)blockIdx.x * 2 * H;
#pragma unroll
  for (int i = 0; i < NVW; ++i) {
    const int c = (i * 256 + threadIdx.x) * VN;
    if (c < H) {
#pragma unroll
      for (int k = 0; k < VN; ++k) {
        outp[c + k] = accg[i][k];
        if (!RMS) outp[H + c + k] = accb[i][k];
      }
    }
  }
}

// out[j] (+)= sum_c partials[c * stride + j], for up to REDUCE_MAX_JOBS independent jobs in one launch.
// 1024 threads = 32 columns x 32 chunk lanes: a block sums all chunks of its 32
// columns (128-byte reads), the 32 lanes of a column meet in LDS in a fixed
// order.  Columns [0, n0) of a job go to out0, columns [n0, n) to out1 (dgamma | dbeta).
struct ReduceGroup { ReduceJob j[REDUCE_MAX_JOBS]; int block0[REDUCE_MAX_JOBS + 1]; int n; };
__global__ void __launch_bounds__(1024) reduce_group_kernel(ReduceGroup g, int accumulate) {
  int ji = 0;
#pragma unroll
  for (int i = 1; i < REDUCE_MAX_JOBS; ++i)
    if (i < g.n && (int)blockIdx.x >= g.block0[i]) ji = i;
  const ReduceJob& jb = g.j[ji];
  const int col = threadIdx.x & 31, cl = threadIdx.x >> 5;
  const int64_t j = (int64_t)((int)blockIdx.x - g.block0[ji]) * 32 + col;
  float acc = 0.f;
  if (j < jb.n) {
    // eight independent partial sums: eight loads in flight per thread instead of a chain of dependent ones
    float a[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] = 0.f;
    int c = cl;
    for (; c + 7 * 32 < jb.nchunks; c += 8 * 32) {
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] += jb.partials[(c + u * 32) * jb.stride + j];
    }
    for (; c < jb.nchunks; c += 32) a[0] += jb.partials[c * jb.stride + j];
    acc = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
  }
  __shared__ float red[32][33];
  red[cl][col] = acc;
  __syncthreads();
  if (cl == 0 && j < jb.n) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 32; ++k) t += red[k][col];
    float* o = j < jb.n0 ? jb.out0 + j : jb.out1 + (j - jb.n0);
    *o = accumulate ? *o + t : t;
  }
}

int reduce_group(hipStream_t s, const ReduceJob* jobs, int n, int accumulate) {
  if (n < 1) return POPLAR_OK;
  if (n > REDUCE_MAX_JOBS) return poplar_fail(POPLAR_ERR_INVALID, "at most %d reductions per launch", REDUCE_MAX_JOBS);
  ReduceGroup g;
  int blocks = 0;
  for (int i = 0; i < n; ++i) {
    g.j[i] = jobs[i];
    g.block0[i] = blocks;
    blocks += (int)cdiv(jobs[i].n, 32);
  }
  for (int i = n; i < REDUCE_MAX_JOBS; ++i) g.j[i] = jobs[0];
  for (int i = n; i <= REDUCE_MAX_JOBS; ++i) g.block0[i] = blocks;
  g.n = n;
  if (blocks == 0) return POPLAR_OK;
  hipLaunchKernelGGL(reduce_group_kernel, dim3(blocks), dim3(1024), 0, s, g, accumulate);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

// wide rows: a block per row at a time; two blocks per CU keep enough loads in flight, more would only add partials
static int norm_bwd_wide_blocks(int64_t rows, int vectors_per_thread) {
  return (int)std::min<int64_t>(rows, vectors_per_thread == 1 ? 768 : 512);   // thin threads: a third block per CU for the loads in flight
}

static int norm_bwd_blocks(int64_t rows) {
  int64_t b = cdiv(rows, 16);  // at least 4 rows per wave; at most three blocks per CU of a 256-CU chip (what its registers allow: whole rounds)
  if (b > 768) b = 768;
  if (b < 1) b = 1;
  return (int)b;
}

template <typename T, bool RMS>
static int norm_bwd_launch(hipStream_t s, int64_t rows, int H, const T* dy, const T* x, const T* g, const float* stats, const T* dres,
                           T* dx, float* partials, int grid) {
  constexpr int VN = Vec<T>::N;
  int need = (int)cdiv(H, 64 * VN);
  if (need > 2) {   // the row-per-wave kernel would run out of registers
    const int needw = (int)cdiv(H, 256 * VN);
#define NORM_BWD_WIDE(NVW) \
  hipLaunchKernelGGL((norm_bwd_wide_kernel<T, NVW, RMS>), dim3(grid), dim3(256), 0, s, dy, x, g, stats, dres, dx, partials, rows, H)
    if (needw <= 1) NORM_BWD_WIDE(1);
    else if (needw <= 2) NORM_BWD_WIDE(2);
    else if (needw <= 4) NORM_BWD_WIDE(4);
    else return poplar_fail(POPLAR_ERR_INVALID, "hidden %d too large for the norm backward kernel", H);
#undef NORM_BWD_WIDE
    POPLAR_LAUNCH_CHECK();
    return POPLAR_OK;
  }
  size_t lds = (size_t)8 * H * sizeof(float);
#define NORM_BWD_CASE(NVV) \
  hipLaunchKernelGGL((norm_bwd_kernel<T, NVV, RMS>), dim3(grid), dim3(256), lds, s, dy, x, g, stats, dres, dx, partials, rows, H)
  if (need <= 1) NORM_BWD_CASE(1);
  else NORM_BWD_CASE(2);
#undef NORM_BWD_CASE
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int layernorm_bwd_partial(hipStream_t s, int dtype, int64_t T_, int H, const void* dy, const void* x, const void* g, const float* stats,
                          const void* dres, void* dx, float* dg, float* db, float* partials, int64_t partials_elems, int rms, ReduceJob* job) {
  job->n = 0;
  if (T_ == 0) return POPLAR_OK;
  const bool wide = cdiv(H, 64 * (dtype == POPLAR_BF16 ? 8 : 4)) > 2;
  int grid = wide ? norm_bwd_wide_blocks(T_, (int)cdiv(H, 256 * (dtype == POPLAR_BF16 ? 8 : 4))) : norm_bwd_blocks(T_);
  if ((int64_t)grid * 2 * H > partials_elems) return poplar_fail(POPLAR_ERR_OOM, "norm backward scratch too small");
  DISPATCH_DTYPE(dtype, {
    if (rms) POPLAR_TRY((norm_bwd_launch<T, true>(s, T_, H, (const T*)dy, (const T*)x, (const T*)g, stats, (const T*)dres, (T*)dx, partials, grid)));
    else POPLAR_TRY((norm_bwd_launch<T, false>(s, T_, H, (const T*)dy, (const T*)x, (const T*)g, stats, (const T*)dres, (T*)dx, partials, grid)));
  });
  // dgamma = partials[:, 0, :], dbeta = partials[:, 1, :]: one job covers both
  job->partials = partials; job->nchunks = grid; job->stride = (int64_t)2 * H;
  job->out0 = dg; job->out1 = db; job->n0 = H; job->n = rms ? H : 2 * (int64_t)H;
  return POPLAR_OK;
}

int layernorm_bwd(hipStream_t s, int dtype, int64_t T_, int H, const void* dy, const void* x, const void* g, const float* stats,
                  const void* dres, void* dx, float* dg, float* db, int accumulate, float* partials, int64_t partials_elems, int rms) {
  ReduceJob job;
  POPLAR_TRY(layernorm_bwd_partial(s, dtype, T_, H, dy, x, g, stats, dres, dx, dg, db, partials, partials_elems, rms, &job));
  return job.n ? reduce_group(s, &job, 1, accumulate) : POPLAR_OK;
}

// ---------------------------------------------------------------------------
// Column sums (bias gradients): out[n] (+)= sum_t x[t, n].
// grid = (column strips of 64*VN, row chunks); 4 waves split the chunk's rows.
// ---------------------------------------------------------------------------
struct ColsumGroup { ColsumProblem p[COLSUM_MAX_GROUP]; int strip0[COLSUM_MAX_GROUP + 1]; int64_t col0[COLSUM_MAX_GROUP]; int n; int64_t ncat; };
// Up to COLSUM_MAX_GROUP matrices of one row count in a launch; partials[chunk][ncat] holds their columns side by side.
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(ColsumGroup g, int64_t rows, int rows_per_chunk, float* __restrict__ partials) {
  constexpr int VN = Vec<T>::N;
  int pi = 0;
#pragma unroll
  for (int i = 1; i < COLSUM_MAX_GROUP; ++i)
    if (i < g.n && (int)blockIdx.x >= g.strip0[i]) pi = i;
  const T* __restrict__ x = (const T*)g.p[pi].x;
  const int64_t ldx = g.p[pi].ldx, N = g.p[pi].N;
  const int strip = (int)blockIdx.x - g.strip0[pi];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int64_t c = ((int64_t)strip * 64 + lane) * VN;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
  int64_t r1 = r0 + rows_per_chunk;
  if (r1 > rows) r1 = rows;
  float acc[VN];
#pragma unroll
  for (int k = 0; k < VN; ++k) acc[k] = 0.f;
  if (c < N) {
    for (int64_t r = r0 + wv; r < r1; r += 4) {
      float f[VN];
      Vec<T> v; v.load(x + r * ldx + c); v.unpack(f);
#pragma unroll
      for (int k = 0; k < VN; ++k) acc[k] += f[k];
    }
  }
  __shared__ float lds[4][64 * VN];
#pragma unroll
  for (int k = 0; k < VN; ++k) lds[wv][lane * VN + k] = acc[k];
  __syncthreads();
  for (int j = threadIdx.x; j < 64 * VN; j += 256) {
    int64_t col = (int64_t)strip * 64 * VN + j;
    if (col < N) partials[(int64_t)blockIdx.y * g.ncat + g.col0[pi] + col] = lds[0][j] + lds[1][j] + lds[2][j] + lds[3][j];
  }
}

// first pass only: jobs[i] receives the reduction that finishes problem i
int colsum_partial(hipStream_t s, int dtype, int64_t T_, const ColsumProblem* p, int n, float* partials, int64_t partials_elems,
                   ReduceJob* jobs) {
  if (n < 1 || n > COLSUM_MAX_GROUP) return poplar_fail(POPLAR_ERR_INVALID, "1 to %d column sums per launch", COLSUM_MAX_GROUP);
  for (int i = 0; i < n; ++i) jobs[i].n = 0;
  if (T_ == 0) return POPLAR_OK;
  const int VN = dtype == POPLAR_BF16 ? 8 : 4;
  ColsumGroup g;
  int strips = 0;
  int64_t ncat = 0;
  for (int i = 0; i < n; ++i) {
    if (p[i].N % VN) return poplar_fail(POPLAR_ERR_INVALID, "colsum needs N %% %d == 0", VN);
    g.p[i] = p[i];
    g.strip0[i] = strips; g.col0[i] = ncat;
    strips += (int)cdiv(p[i].N, 64 * VN);
    ncat += p[i].N;
  }
  for (int i = n; i < COLSUM_MAX_GROUP; ++i) { g.p[i] = p[0]; g.col0[i] = 0; }
  for (int i = n; i <= COLSUM_MAX_GROUP; ++i) g.strip0[i] = strips;
  g.n = n; g.ncat = ncat;
  if (strips == 0) return POPLAR_OK;
  int chunks = (int)cdiv(2048, strips);
  if (chunks > cdiv(T_, 32)) chunks = (int)cdiv(T_, 32);
  if (chunks < 1) chunks = 1;
  int rpc = (int)cdiv(T_, chunks);
  chunks = (int)cdiv(T_, rpc);
  if ((int64_t)chunks * ncat > partials_elems) return poplar_fail(POPLAR_ERR_OOM, "colsum scratch too small");
  DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(colsum_kernel<T>, dim3(strips, chunks), dim3(256), 0, s, g, T_, rpc, partials));
  POPLAR_LAUNCH_CHECK();
  for (int i = 0; i < n; ++i) {
    jobs[i].partials = partials + g.col0[i]; jobs[i].nchunks = chunks; jobs[i].stride = ncat;
    jobs[i].out0 = p[i].out; jobs[i].out1 = p[i].out; jobs[i].n0 = p[i].N; jobs[i].n = p[i].N;
  }
  return POPLAR_OK;
}

int colsum(hipStream_t s, int dtype, int64_t T_, int64_t N, const void* x, int64_t ldx, float* out, int accumulate,
           float* partials, int64_t partials_elems) {
  if (T_ == 0 || N == 0) return POPLAR_OK;
  ColsumProblem p = {x, ldx, N, out};
  ReduceJob job;
  POPLAR_TRY(colsum_partial(s, dtype, T_, &p, 1, partials, partials_elems, &job));
  return reduce_group(s, &job, 1, accumulate);
}

// ---------------------------------------------------------------------------
// SwiGLU on the fused [T, 2F] gate|up activation: g = silu(hg) * hu
// ---------------------------------------------------------------------------
// A block column owns 256 vectors of a row, a block row walks the rows two at a time (both rows' loads in flight
// before either is worked on; four at a time measured the same); no index division anywhere; streaming accesses (the
// forward kernel 95 -> 85 us on 8192 x 11008, 0.80 of the HBM rate; the backward kernel, five streams, stays at 0.72).  sigmoid(a) = 1 / (1 + 2^(-a log2 e)) with the hardware
// exp2, and for bfloat16 outputs the hardware reciprocal (1 ulp; the quotient in float costs ten instructions a value).
template <typename T>
__device__ inline float swiglu_sigmoid(float a) {
  const float e = __builtin_amdgcn_exp2f(a * -1.4426950408889634f);
  if (std::is_same<T, float>::value) return 1.0f / (1.0f + e);
  return __builtin_amdgcn_rcpf(1.0f + e);
}
template <typename T>
__global__ void __launch_bounds__(256) swiglu_fwd_kernel(const T* __restrict__ hgu, T* __restrict__ g, int64_t rows, int F) {
  constexpr int VN = Vec<T>::N, R = 2;
  const int c = (int)(blockIdx.x * 256 + threadIdx.x) * VN;
  if (c >= F) return;
  for (int64_t r0 = (int64_t)blockIdx.y * R; r0 < rows; r0 += (int64_t)gridDim.y * R) {
    Vec<T> va[R], vb[R];
#pragma unroll
    for (int u = 0; u < R; ++u)
      if (r0 + u < rows) {
        vec_load_nt(va[u], hgu + (r0 + u) * 2 * F + c);
        vec_load_nt(vb[u], hgu + (r0 + u) * 2 * F + F + c);
      }
#pragma unroll
    for (int u = 0; u < R; ++u)
      if (r0 + u < rows) {
        float a[VN], b[VN], o[VN];
        va[u].unpack(a);
        vb[u].unpack(b);
#pragma unroll
        for (int k = 0; k < VN; ++k) o[k] = a[k] * swiglu_sigmoid<T>(a[k]) * b[k];
        Vec<T> v;
        v.pack(o);
        vec_store_nt(v, g + (r0 + u) * F + c);
      }
  }
}
template <typename T>
__global__ void __launch_bounds__(256) swiglu_bwd_kernel(const T* __restrict__ dg, const T* __restrict__ hgu, T* __restrict__ dhgu, int64_t rows, int F) {
  constexpr int VN = Vec<T>::N, R = 2;
  const int c = (int)(blockIdx.x * 256 + threadIdx.x) * VN;
  if (c >= F) return;
  for (int64_t r0 = (int64_t)blockIdx.y * R; r0 < rows; r0 += (int64_t)gridDim.y * R) {
    Vec<T> va[R], vb[R], vd[R];
#pragma unroll
    for (int u = 0; u < R; ++u)
      if (r0 + u < rows) {
        vec_load_nt(va[u], hgu + (r0 + u) * 2 * F + c);
        vec_load_nt(vb[u], hgu + (r0 + u) * 2 * F + F + c);
        vec_load_nt(vd[u], dg + (r0 + u) * F + c);
      }
#pragma unroll
    for (int u = 0; u < R; ++u)
      if (r0 + u < rows) {
        float a[VN], b[VN], d[VN], oa[VN], ob[VN];
        va[u].unpack(a);
        vb[u].unpack(b);
        vd[u].unpack(d);
#pragma unroll
        for (int k = 0; k < VN; ++k) {
          const float sg = swiglu_sigmoid<T>(a[k]);
          oa[k] = d[k] * b[k] * (sg + a[k] * sg * (1.0f - sg));
          ob[k] = d[k] * a[k] * sg;
        }
        Vec<T> v;
        v.pack(oa);
        vec_store_nt(v, dhgu + (r0 + u) * 2 * F + c);
        v.pack(ob);
        vec_store_nt(v, dhgu + (r0 + u) * 2 * F + F + c);
      }
  }
}
static dim3 swiglu_grid(int64_t rows, int F, int vn) {
  return dim3((unsigned)cdiv(F / vn, 256), (unsigned)std::min<int64_t>(cdiv(rows, 2), 65535));
}
int swiglu_fwd(hipStream_t s, int dtype, int64_t T_, int F, const void* hgu, void* g) {
  if (T_ == 0) return POPLAR_OK;
  DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(swiglu_fwd_kernel<T>, swiglu_grid(T_, F, Vec<T>::N), dim3(256), 0, s, (const T*)hgu, (T*)g, T_, F));
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
int swiglu_bwd(hipStream_t s, int dtype, int64_t T_, int F, const void* dg, const void* hgu, void* dhgu) {
  if (T_ == 0) return POPLAR_OK;
  DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(swiglu_bwd_kernel<T>, swiglu_grid(T_, F, Vec<T>::N), dim3(256), 0, s, (const T*)dg, (const T*)hgu, (T*)dhgu, T_, F));
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

// ---------------------------------------------------------------------------
// RoPE in place on the q and k thirds of qkv [B*S, ld]: element i of a head is
// paired with i + d/2 and rotated by pos * 10000^(-2i/d).  sign = -1 applies the
// inverse rotation (the backward pass).
// rope_vec_kernel: one thread owns 16 bytes' worth of consecutive i of one token
// (8 bfloat16 or 4 float), evaluates those angles once in double and walks all
// heads of q and k with 16-byte accesses: eight (four) neighbouring lanes cover
// the contiguous half of a head.  rope_kernel: one element pair per thread, for
// head dims and alignments the vector form does not take.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) rope_vec_kernel(T* __restrict__ qkv, int64_t ld, int64_t tokens, int S, int nh, int d, float sign) {
  constexpr int N = Vec<T>::N;
  constexpr int HEADS = 8;       // heads per thread (blockIdx.y picks the run of heads), UNROLL of them in flight at a time
  constexpr int UNROLL = 4;
  const int half = d / 2, groups = half / N;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= tokens * groups) return;
  const int64_t t = idx / groups;
  const int i0 = (int)(idx % groups) * N;
  const int pos = (int)(t % S);
  float c[N], sn[N];   // cosines and signed sines of this thread's N angles
#pragma unroll
  for (int k = 0; k < N; ++k) {
    if (std::is_same<T, float>::value) {
      // angle and its reduction to [-pi, pi] in double (positions reach the thousands of radians), sine and cosine of
      // the reduced angle in float
      const double ang = (double)pos * exp(-9.210340371976184 * (2.0 * (double)(i0 + k) / (double)d));   // ln 10000
      const double turns = rint(ang * 0.15915494309189535);
      const float r = (float)fma(turns, -1.2246467991473532e-16 * 2.0, fma(turns, -6.283185307179586, ang));
      float sf, cf;
      sincosf(r, &sf, &cf);
      c[k] = cf;
      sn[k] = sign * sf;
    } else {
      // bfloat16 rows: the angle in turns in float (its error at position 2048 is 2.5e-4 rad, a sixteenth of the
      // rounding of the values it rotates), its fraction through the hardware sine and cosine, which take turns
      const float turns = (float)pos * __builtin_amdgcn_exp2f(-13.287712379549449f * (2.0f * (float)(i0 + k) / (float)d)) * 0.15915494309189535f;   // log2 10000
      const float fr = __builtin_amdgcn_fractf(turns);
      c[k] = __builtin_amdgcn_cosf(fr);
      sn[k] = sign * __builtin_amdgcn_sinf(fr);
    }
  }
  const int heads = 2 * nh;   // q heads, then k heads: the two thirds are adjacent
  const int h_begin = blockIdx.y * HEADS, h_end = min(heads, h_begin + HEADS);
  T* row = qkv + t * ld + i0;
  for (int h0 = h_begin; h0 < h_end; h0 += UNROLL) {
    Vec<T> a[UNROLL], b[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (h0 + u < h_end) {
        a[u].load(row + (int64_t)(h0 + u) * d);
        b[u].load(row + (int64_t)(h0 + u) * d + half);
      }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (h0 + u < h_end) {
        float x1[N], x2[N], y1[N], y2[N];
        a[u].unpack(x1);
        b[u].unpack(x2);
#pragma unroll
        for (int k = 0; k < N; ++k) {
          y1[k] = x1[k] * c[k] - x2[k] * sn[k];
          y2[k] = x2[k] * c[k] + x1[k] * sn[k];
        }
        a[u].pack(y1);
        b[u].pack(y2);
        a[u].store(row + (int64_t)(h0 + u) * d);
        b[u].store(row + (int64_t)(h0 + u) * d + half);
      }
  }
}
template <typename T>
__global__ void rope_kernel(T* __restrict__ qkv, int64_t ld, int64_t tokens, int S, int nh, int d, float sign) {
  const int half = d / 2;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= tokens * half) return;
  const int64_t t = idx / half;
  const int i = (int)(idx % half);
  const int pos = (int)(t % S);
  const double ang = (double)pos * pow(10000.0, -2.0 * (double)i / (double)d);
  double sd, cd;
  sincos(ang, &sd, &cd);
  const float c = (float)cd, sn = sign * (float)sd;
  const int H = nh * d;
  T* row = qkv + t * ld;
  for (int part = 0; part < 2; ++part) {
    for (int h = 0; h < nh; ++h) {
      T* p = row + part * H + h * d + i;
      float x1 = to_float<T>(p[0]), x2 = to_float<T>(p[half]);
      p[0] = from_float<T>(x1 * c - x2 * sn);
      p[half] = from_float<T>(x2 * c + x1 * sn);
    }
  }
}
int rope_inplace(hipStream_t s, int dtype, int B, int S, int nh, int d, void* qkv, int64_t ld, float sign) {
  int64_t work = (int64_t)B * S * (d / 2);
  if (work == 0) return POPLAR_OK;
  const int vec = dtype == POPLAR_BF16 ? 8 : 4;
  // the vector form needs whole 16-byte groups in half a head and 16-byte aligned rows
  if ((d / 2) % vec == 0 && ((uintptr_t)qkv & 15) == 0 && (ld * (int64_t)elt_size(dtype)) % 16 == 0) {
    work /= vec;
    const dim3 grid((unsigned)cdiv(work, 256), (unsigned)cdiv(2 * nh, 8));   // y: runs of eight heads
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(rope_vec_kernel<T>, grid, dim3(256), 0, s, (T*)qkv, ld, (int64_t)B * S, S, nh, d, sign));
  } else {
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(rope_kernel<T>, dim3((unsigned)cdiv(work, 256)), dim3(256), 0, s, (T*)qkv, ld, (int64_t)B * S, S, nh, d, sign));
  }
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

// ---------------------------------------------------------------------------
// Embedding
// ---------------------------------------------------------------------------
template <typename T>
__global__ void embed_fwd_kernel(const int32_t* __restrict__ tok, int64_t tok_ld, const T* __restrict__ wte, const T* __restrict__ wpe,
                                 T* __restrict__ x, int64_t tokens, int S, int H, int V) {
  constexpr int VN = Vec<T>::N;
  const int per_row = H / VN;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < tokens * per_row; i += stride) {
    int64_t t = i / per_row;
    int c = (int)(i % per_row) * VN;
    int64_t b = t / S, sp = t % S;
    int id = tok[b * tok_ld + sp];
    float a[VN], p[VN];
    Vec<T> v;
#pragma unroll
    for (int k = 0; k < VN; ++k) a[k] = 0.f;
    // an id outside [0, V) embeds as zero (and receives no gradient): nothing outside the table is touched
    if (id >= 0 && id < V) { v.load(wte + (int64_t)id * H + c); v.unpack(a); }
    if (wpe) {
      v.load(wpe + sp * H + c); v.unpack(p);
#pragma unroll
      for (int k = 0; k < VN; ++k) a[k] += p[k];
    }
    v.pack(a); v.store(x + t * H + c);
  }
}
int embed_fwd(hipStream_t s, int dtype, int B, int S, int H, int V, const int32_t* tok, int64_t tok_ld, const void* wte, const void* wpe, void* x) {
  int64_t tokens = (int64_t)B * S;
  if (tokens == 0) return POPLAR_OK;
  DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(embed_fwd_kernel<T>, dim3(grid_for(tokens * H / Vec<T>::N, 256)), dim3(256), 0, s, tok, tok_ld,
                                           (const T*)wte, (const T*)wpe, (T*)x, tokens, S, H, V));
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

// One element per lane: the 64 atomics of a wavefront instruction fall on 256 consecutive bytes of one
// (or two) rows of dwte.  With a vector of columns per lane they would be 32 bytes apart and every
// atomic a memory transaction of its own (measured 4x slower).
template <typename T>
__global__ void embed_bwd_wte_kernel(const int32_t* __restrict__ tok, int64_t tok_ld, const T* __restrict__ dx, float* __restrict__ dwte,
                                     int64_t tokens, int S, int H, int V) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < tokens * H; i += stride) {
    const int64_t t = i / H;
    const int c = (int)(i - t * H);
    const int id = tok[(t / S) * tok_ld + (t % S)];
    if (id >= 0 && id < V) unsafeAtomicAdd(dwte + (int64_t)id * H + c, to_float<T>(dx[i]));
  }
}
// The same sums in a fixed order, without atomics.  One block per token t: if an earlier token carries the same
// id the block has nothing to do; otherwise it owns row id of dwte and adds to it the rows of dx of t and of every
// later token with that id, in sequence order.  Tokens are compared 256 at a time (one per thread, a ballot per
// wavefront); each thread keeps its columns of the sum in registers and adds them to dwte once at the end.
template <typename T, int COLS>
__global__ void __launch_bounds__(256) embed_bwd_wte_ordered_kernel(const int32_t* __restrict__ tok, int64_t tok_ld, const T* __restrict__ dx,
                                                                    float* __restrict__ dwte, int64_t tokens, int S, int H, int V) {
  __shared__ unsigned long long hits[4];
  const int64_t t0 = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6;
  const int id = tok[(t0 / S) * tok_ld + (t0 % S)];
  if (id < 0 || id >= V) return;
  auto scan = [&](int64_t base, int64_t end) {   // hits[w] <- which of tokens base + 64 w .. + 63 (below end) carry `id`
    const int64_t t = base + tid;
    const bool same = t < end && tok[(t / S) * tok_ld + (t % S)] == id;
    const unsigned long long m = __builtin_amdgcn_ballot_w64(same);
    __syncthreads();                               // the previous chunk's masks have been read
    if ((tid & 63) == 0) hits[wave] = m;
    __syncthreads();
  };
  for (int64_t base = 0; base < t0; base += 256) {  // an earlier token with this id owns the row
    scan(base, t0);
    if (hits[0] | hits[1] | hits[2] | hits[3]) return;
  }
  float acc[COLS];
#pragma unroll
  for (int k = 0; k < COLS; ++k) acc[k] = 0.f;
  for (int64_t first = t0; first < tokens; first += 256) {   // thread i looks at token first + i; the first chunk holds t0 itself
    scan(first, tokens);
    for (int w = 0; w < 4; ++w) {
      unsigned long long m = hits[w];
      while (m) {
        const int bit = __builtin_ctzll(m);
        m &= m - 1;
        const T* row = dx + (first + w * 64 + bit) * H;
#pragma unroll
        for (int k = 0; k < COLS; ++k) {
          const int c = tid + k * 256;
          if (c < H) acc[k] += to_float<T>(row[c]);
        }
      }
    }
  }
  float* out = dwte + (int64_t)id * H;
#pragma unroll
  for (int k = 0; k < COLS; ++k) {
    const int c = tid + k * 256;
    if (c < H) out[c] += acc[k];
  }
}
template <typename T>
__global__ void embed_bwd_wpe_kernel(const T* __restrict__ dx, float* __restrict__ dwpe, int B, int S, int H, int accumulate) {
  constexpr int VN = Vec<T>::N;
  const int per_row = H / VN;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)S * per_row) return;
  int64_t sp = i / per_row;
  int c = (int)(i % per_row) * VN;
  float acc[VN];
#pragma unroll
  for (int k = 0; k < VN; ++k) acc[k] = 0.f;
  for (int b = 0; b < B; ++b) {
    float a[VN];
    Vec<T> v; v.load(dx + ((int64_t)b * S + sp) * H + c); v.unpack(a);
#pragma unroll
    for (int k = 0; k < VN; ++k) acc[k] += a[k];
  }
  float* o = dwpe + sp * H + c;
#pragma unroll
  for (int k = 0; k < VN; ++k) o[k] = accumulate ? o[k] + acc[k] : acc[k];
}
template <typename T>
static int embed_bwd_wte_ordered(hipStream_t s, const int32_t* tok, int64_t tok_ld, const T* dx, float* dwte, int64_t tokens, int S, int H, int V) {
  if (H > 32 * 256) return poplar_fail(POPLAR_ERR_UNIMPLEMENTED, "ordered embedding gradient: hidden %d above %d", H, 32 * 256);
  if (tokens > 0x7fffffff) return poplar_fail(POPLAR_ERR_INVALID, "too many tokens for one launch");
  const dim3 grid((unsigned)tokens), block(256);
#define ORDERED(C) hipLaunchKernelGGL((embed_bwd_wte_ordered_kernel<T, C>), grid, block, 0, s, tok, tok_ld, dx, dwte, tokens, S, H, V)
  const int cols = (H + 255) / 256;
  if (cols <= 1) ORDERED(1);
  else if (cols <= 2) ORDERED(2);
  else if (cols <= 4) ORDERED(4);
  else if (cols <= 8) ORDERED(8);
  else if (cols <= 16) ORDERED(16);
  else ORDERED(32);
#undef ORDERED
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int embed_bwd(hipStream_t s, int dtype, int B, int S, int H, int V, const int32_t* tok, int64_t tok_ld, const void* dx, float* dwte, float* dwpe, int accumulate,
              int ordered) {
  int64_t tokens = (int64_t)B * S;
  if (tokens == 0) return POPLAR_OK;
  DISPATCH_DTYPE(dtype, {
    if (ordered) POPLAR_TRY(embed_bwd_wte_ordered<T>(s, tok, tok_ld, (const T*)dx, dwte, tokens, S, H, V));
    else hipLaunchKernelGGL(embed_bwd_wte_kernel<T>, dim3(grid_for(tokens * H, 256)), dim3(256), 0, s, tok, tok_ld, (const T*)dx, dwte, tokens, S, H, V);
    POPLAR_LAUNCH_CHECK();
    if (dwpe) {
      hipLaunchKernelGGL(embed_bwd_wpe_kernel<T>, dim3((unsigned)cdiv((int64_t)S * H / Vec<T>::N, 256)), dim3(256), 0, s, (const T*)dx, dwpe, B, S, H, accumulate);
      POPLAR_LAUNCH_CHECK();
    }
  });
  return POPLAR_OK;
}

// ---------------------------------------------------------------------------
// Softmax cross-entropy over logits [T, ld] (V valid columns), in place:
// logits <- loss_scale * (softmax - onehot(target)), columns V..ld-1 <- 0;
// row_loss[t] = logsumexp - logit[target].  One block per row, two passes over
// the row (online max / sum first, gradient second).  A negative target marks a
// position without a prediction (masked-language-model batches): its row of
// the gradient is zero and it adds nothing to the loss.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) xent_kernel(T* __restrict__ logits, int64_t ld, int V, const int32_t* __restrict__ targets,
                                                    int64_t tgt_ld, int S, float loss_scale, float* __restrict__ row_loss) {
  constexpr int VN = Vec<T>::N;
  const int64_t t = blockIdx.x;
  T* row = logits + t * ld;
  const int nvec = (int)(ld / VN);
  int tgt = targets[(t / S) * tgt_ld + (t % S)];
  if (tgt >= V) tgt = -1;   // a class that does not exist is treated like a position without a prediction, never read
  if (tgt < 0) {   // a position that is not predicted: no loss, zero gradient
    Vec<T> z;
    float f[VN];
#pragma unroll
    for (int k = 0; k < VN; ++k) f[k] = 0.f;
    z.pack(f);
    for (int i = threadIdx.x; i < nvec; i += 256) z.store(row + i * VN);
    if (threadIdx.x == 0) row_loss[t] = 0.f;
    return;
  }
  float mx = -INFINITY, sum = 0.f;
  for (int i = threadIdx.x; i < nvec; i += 256) {
    float f[VN];
    Vec<T> v; v.load(row + i * VN); v.unpack(f);
    float lm = -INFINITY;
#pragma unroll
    for (int k = 0; k < VN; ++k) if (i * VN + k < V) lm = fmaxf(lm, f[k]);
    if (lm > mx) { sum *= __expf(mx - lm); mx = lm; }
#pragma unroll
    for (int k = 0; k < VN; ++k) if (i * VN + k < V) sum += __expf(f[k] - mx);
  }
  __shared__ float smx[4], ssum[4];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float wm = wave_max(mx);
  sum = (mx == -INFINITY) ? 0.f : sum * __expf(mx - wm);
  sum = wave_sum(sum);
  if (lane == 0) { smx[wv] = wm; ssum[wv] = sum; }
  __syncthreads();
  float bm = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) bs += (smx[w] == -INFINITY) ? 0.f : ssum[w] * __expf(smx[w] - bm);
  const float lse = bm + logf(bs);
  if (threadIdx.x == 0) row_loss[t] = lse - to_float<T>(row[tgt]);
  __syncthreads();  // the target logit is read before anyone overwrites it
  for (int i = threadIdx.x; i < nvec; i += 256) {
    float f[VN];
    Vec<T> v; v.load(row + i * VN); v.unpack(f);
#pragma unroll
    for (int k = 0; k < VN; ++k) {
      int col = i * VN + k;
      float p = col < V ? __expf(f[k] - lse) : 0.f;
      if (col == tgt) p -= 1.0f;
      f[k] = p * loss_scale;
    }
    v.pack(f); v.store(row + i * VN);
  }
}

// The same operation with each row held in registers between the two passes, so that the logits cross the
// memory system once in each direction (the two-pass kernel above reads them twice: a row of 100 KB times the
// rows in flight is far beyond the L2).  One block of 1024 threads per CU walks rows blockIdx.x, + gridDim.x, ...;
// a thread owns vectors tid, tid + 1024, ... of the row: exactly NV of them, so that only the last can hold columns
// past V (the launcher checks (NV - 1) * 1024 vectors <= V columns).  The row loop is built like the norm kernels':
// rows in pairs in a body without a branch, two register sets, all accesses through row descriptors, so that the
// next row's loads and the previous row's stores stay in flight while a row is worked on.  For that reason a row
// without a prediction is not skipped: its sums are formed and its gradient is scaled by zero.
template <typename T, int NV>
__global__ void __launch_bounds__(1024) xent_row_kernel(T* __restrict__ logits, int64_t ld, int V, int64_t rows,
                                                         const int32_t* __restrict__ targets, int64_t tgt_ld, int S,
                                                         float loss_scale, float* __restrict__ row_loss) {
  constexpr int VN = Vec<T>::N;
  constexpr float L2E = 1.4426950408889634f;
  const int wv = threadIdx.x >> 6;
  const uint32_t row_bytes = (uint32_t)ld * sizeof(T);
  __shared__ float smx[2][16], ssum[2][16], stl[2], junk[64];
  const int64_t step = gridDim.x;
  auto fetch = [&](Vec<T> (&q)[NV], int64_t t) __attribute__((always_inline)) {
    const bool have = t < rows;
    const __amdgpu_buffer_rsrc_t rs = span_rsrc(logits + (have ? t : 0) * ld, have ? row_bytes : 0u);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NV; ++j) span_load<T, 2>(q[j], rs, (uint32_t)(threadIdx.x + j * 1024) * 16);   // streamed once in each direction: non-temporal
    __builtin_amdgcn_sched_barrier(0);
  };
  auto work = [&](Vec<T> (&q)[NV], int64_t t, int par) __attribute__((always_inline)) {
    const bool have = t < rows;
    const int64_t tt = have ? t : 0;
    const uint32_t ts = (uint32_t)tt / (uint32_t)S;   // rows fit 32 bits (the launcher checks): a 64-bit division would bring a branch into the loop
    int tgt = targets[(int64_t)ts * tgt_ld + ((uint32_t)tt - ts * (uint32_t)S)];
    if (tgt >= V || !have) tgt = -1;   // a class that does not exist is treated like a position without a prediction
    const int tv = tgt >= 0 ? tgt / VN : -1;
    // columns past V in the row's last vector (and whole vectors past the row's end, which read as zeros) count as
    // minus infinity: they drop out of the maximum and the sum and come out of the last pass as zeros
    {
      float f[VN];
      q[NV - 1].unpack(f);
      const int c0 = (int)(threadIdx.x + (NV - 1) * 1024) * VN;
#pragma unroll
      for (int k = 0; k < VN; ++k) f[k] = c0 + k < V ? f[k] : -INFINITY;
      q[NV - 1].pack(f);
    }
    // this thread's share of max and sum; exponentials in the base-2 domain (one fma + v_exp_f32 each); the vector
    // that holds the target logit is kept aside on the way
    float mx = -INFINITY, sum = 0.f;
    Vec<T> hit = q[0];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      float f[VN];
      q[j].unpack(f);
#pragma unroll
      for (int k = 0; k < VN; ++k) mx = fmaxf(mx, f[k]);
      if (j > 0) {
        const bool mine = (int)(threadIdx.x + j * 1024) == tv;
        hit.raw.x = mine ? q[j].raw.x : hit.raw.x; hit.raw.y = mine ? q[j].raw.y : hit.raw.y;
        hit.raw.z = mine ? q[j].raw.z : hit.raw.z; hit.raw.w = mine ? q[j].raw.w : hit.raw.w;
      }
    }
    const float m2 = mx * L2E;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      float f[VN];
      q[j].unpack(f);
#pragma unroll
      for (int k = 0; k < VN; ++k) sum += __builtin_amdgcn_exp2f(fmaf(f[k], L2E, -m2));
    }
    const float wm = wave_max(mx);
    sum = (mx == -INFINITY) ? 0.f : sum * __expf(mx - wm);
    sum = wave_sum(sum);
    smx[par][wv] = wm; ssum[par][wv] = sum;   // every lane writes the same two values: no branch in the row loop
    float own_tl; bool is_owner;
    {
      // the thread whose vectors include the target's puts the logit where thread 0 finds it; the others write aside
      float f[VN];
      hit.unpack(f);
      float tl = f[0];
#pragma unroll
      for (int k = 1; k < VN; ++k) tl = (tgt % VN) == k ? f[k] : tl;
      const bool owner = tv >= 0 && (tv & 1023) == (int)threadIdx.x;
      float* dst = owner ? &stl[par] : &junk[threadIdx.x & 63];
      *dst = tl;
      own_tl = tl; is_owner = owner;
    }
    block_sync_lds();   // one barrier per row: the LDS slots alternate, a wave two rows ahead is impossible
    float bm = -INFINITY;
#pragma unroll
    for (int w = 0; w < 16; ++w) bm = fmaxf(bm, smx[par][w]);
    float bs = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) bs += (smx[par][w] == -INFINITY) ? 0.f : ssum[par][w] * __expf(smx[par][w] - bm);
    const float lse = bm + logf(bs);
    span_store_f1((lse - stl[par]) * (tgt >= 0 ? 1.f : 0.f), span_rsrc(row_loss + tt, have ? 4u : 0u), (uint32_t)threadIdx.x * 4);
    const float l2 = lse * L2E;
    const float scale = tgt >= 0 ? loss_scale : 0.f;   // a row without a prediction gets zeros
    const __amdgpu_buffer_rsrc_t ro = span_rsrc(logits + tt * ld, have ? row_bytes : 0u);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      float f[VN];
      q[j].unpack(f);
#pragma unroll
      for (int k = 0; k < VN; ++k) f[k] = __builtin_amdgcn_exp2f(fmaf(f[k], L2E, -l2)) * scale;
      Vec<T> o; o.pack(f);
      span_store<T, 2>(o, ro, (uint32_t)(threadIdx.x + j * 1024) * 16);
    }
    // the target's entry is softmax - 1: its owner stores that one value again, after the vector that holds it (same
    // thread, same address: in order), formed in float and rounded once; every other lane's offset points past the row
    const T fix = from_float<T>(__builtin_amdgcn_exp2f(fmaf(own_tl, L2E, -l2)) * scale - scale);
    static_assert(sizeof(T) == 2, "one 16-bit store");
    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(short, fix), ro, (int)(is_owner ? (uint32_t)tgt * 2u : row_bytes), 0, 2);
  };
  Vec<T> qa[NV], qb[NV];
  int64_t t = blockIdx.x;   // the launcher starts no more blocks than there are rows
  fetch(qa, t);
  {
    // a row's worth of stores to nowhere: the loop is entered with the operations in flight it is re-entered with
    const __amdgpu_buffer_rsrc_t none = span_rsrc(logits, 0u);
    Vec<T> z; float zf[VN];
#pragma unroll
    for (int k = 0; k < VN; ++k) zf[k] = 0.f;
    z.pack(zf);
    span_store_f1(0.f, none, 0u);
#pragma unroll
    for (int j = 0; j < NV; ++j) span_store<T, 2>(z, none, (uint32_t)j * 16);   // distinct offsets: identical stores would be merged
    __builtin_amdgcn_raw_buffer_store_b16((short)0, none, 0, 0, 2);
    __builtin_amdgcn_sched_barrier(0);
  }
  do {
    fetch(qb, t + step);
    work(qa, t, 0);
    fetch(qa, t + 2 * step);
    work(qb, t + step, 1);
    t += 2 * step;
  } while (t < rows);
}

__global__ void __launch_bounds__(1024) loss_sum_kernel(const float* __restrict__ row_loss, int64_t n, float scale, float* __restrict__ loss) {
  // one block: four independent partial sums per thread keep four loads in flight
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int64_t i = threadIdx.x;
  for (; i + 3 * 1024 < n; i += 4 * 1024) {
    a0 += row_loss[i]; a1 += row_loss[i + 1024]; a2 += row_loss[i + 2 * 1024]; a3 += row_loss[i + 3 * 1024];
  }
  for (; i < n; i += 1024) a0 += row_loss[i];
  float acc = (a0 + a1) + (a2 + a3);
  __shared__ float sw[16];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sw[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) t += sw[w];
    *loss = t * scale;
  }
}

int xent_fwd_bwd(hipStream_t s, int dtype, int64_t T_, int V, int64_t ld, void* logits, const int32_t* targets, int64_t tgt_ld, int S,
                 float loss_scale, float* loss, float* row_loss) {
  if (T_ == 0) return POPLAR_OK;
  const int VN = dtype == POPLAR_BF16 ? 8 : 4;
  if (ld % VN || ld < V) return poplar_fail(POPLAR_ERR_INVALID, "logit row stride %lld invalid for V=%d", (long long)ld, V);
  const int64_t nvec = ld / VN;
  const int nv = (int)cdiv(nvec, 1024);
  if (dtype == POPLAR_BF16 && nv <= 8 && (int64_t)(nv - 1) * 1024 * VN <= V && T_ < (1ll << 31)) {
    static int cus = 0;   // one block per CU (1024 threads with the row in registers fill it)
    if (!cus) {
      int dev = 0;
      POPLAR_CHECK_HIP(hipGetDevice(&dev));
      POPLAR_CHECK_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    }
    const dim3 grid((unsigned)std::min<int64_t>(T_, cus));
#define XENT_ROW_CASE(NVV) \
  case NVV: hipLaunchKernelGGL((xent_row_kernel<bf16, NVV>), grid, dim3(1024), 0, s, (bf16*)logits, ld, V, T_, targets, tgt_ld, S, loss_scale, row_loss); break
    switch (nv) {
      XENT_ROW_CASE(1); XENT_ROW_CASE(2); XENT_ROW_CASE(3); XENT_ROW_CASE(4);
      XENT_ROW_CASE(5); XENT_ROW_CASE(6); XENT_ROW_CASE(7); XENT_ROW_CASE(8);
    }
#undef XENT_ROW_CASE
  } else {
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(xent_kernel<T>, dim3((unsigned)T_), dim3(256), 0, s, (T*)logits, ld, V, targets, tgt_ld, S, loss_scale, row_loss));
  }
  POPLAR_LAUNCH_CHECK();
  hipLaunchKernelGGL(loss_sum_kernel, dim3(1), dim3(1024), 0, s, row_loss, T_, loss_scale, loss);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
