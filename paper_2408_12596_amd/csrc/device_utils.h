// Device-side helpers: 16-byte vector access for float / bfloat16 rows and
// 64-lane wavefront reductions.
#pragma once
#include "common.h"

#define WAVE 64

template <typename T> struct Vec;  // 16 bytes of T
template <> struct Vec<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ void load(const float* p) { raw = *reinterpret_cast<const float4*>(p); }
  __device__ void store(float* p) const { *reinterpret_cast<float4*>(p) = raw; }
  __device__ void unpack(float* f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
  __device__ void pack(const float* f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};

__device__ inline float bf16_bits_to_float(uint32_t hi16) { return __uint_as_float(hi16 << 16); }
// round-to-nearest-even float -> bfloat16 bits (NaN kept quiet)
__device__ inline uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <> struct Vec<bf16> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ void load(const bf16* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ void store(bf16* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ void unpack(float* f) const {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ void pack(const float* f) {
    // v_cvt_pk_bf16_f32: two floats to packed bfloat16, round to nearest even
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      floatx2_t p2 = {f[2 * i], f[2 * i + 1]};
      bf16x2_t h = __builtin_convertvector(p2, bf16x2_t);
      w[i] = *reinterpret_cast<uint32_t*>(&h);
    }
    raw = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

template <typename T> __device__ inline float to_float(T v);
template <> __device__ inline float to_float<float>(float v) { return v; }
template <> __device__ inline float to_float<bf16>(bf16 v) {
  return bf16_bits_to_float(*reinterpret_cast<const uint16_t*>(&v));
}
template <typename T> __device__ inline T from_float(float f);
template <> __device__ inline float from_float<float>(float f) { return f; }
template <> __device__ inline bf16 from_float<bf16>(float f) {
  uint16_t b = (uint16_t)float_to_bf16_bits(f);
  return *reinterpret_cast<bf16*>(&b);
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// make LDS writes of this wavefront visible to its other lanes
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// tanh-form GeLU and its derivative (the form GPT-2 uses)
__device__ inline float gelu_tanh(float h) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  float t = tanhf(k0 * (h + k1 * h * h * h));
  return 0.5f * h * (1.0f + t);
}
__device__ inline float gelu_tanh_grad(float h) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  float t = tanhf(k0 * (h + k1 * h * h * h));
  float dt = (1.0f - t * t) * k0 * (1.0f + 3.0f * k1 * h * h);
  return 0.5f * (1.0f + t) + 0.5f * h * dt;
}

// fast variants for bf16 outputs, on the identity 0.5 (1 + tanh u) = sigmoid(2u) = 1 / (1 + 2^(-2u log2 e))
// with the hardware exp2 and reciprocal: gelu(h) = h s,  gelu'(h) = s + h s (1 - s) 2u'.
// Large |h| saturate the right way: 2^z = inf gives s = 0, 2^z = 0 gives s = 1.
__device__ inline float gelu_sigmoid_fast(float h, float h2) {
  const float c0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f, c1 = c0 * 0.044715f;
  const float z = h * __builtin_fmaf(h2, c1, c0);
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z));
}
__device__ inline float gelu_tanh_fast(float h) { return h * gelu_sigmoid_fast(h, h * h); }
// value and derivative together: the sigmoid is shared, the derivative costs five more operations
__device__ inline void gelu_tanh_both_fast(float h, float* g, float* dg) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  const float h2 = h * h;
  const float s = gelu_sigmoid_fast(h, h2);
  const float du2 = __builtin_fmaf(h2, 6.0f * k0 * k1, 2.0f * k0);   // 2 u'
  *g = h * s;
  *dg = __builtin_fmaf(h * du2 * s, 1.0f - s, s);
}
__device__ inline float gelu_tanh_grad_fast(float h) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  const float h2 = h * h;
  const float s = gelu_sigmoid_fast(h, h2);
  const float du2 = __builtin_fmaf(h2, 6.0f * k0 * k1, 2.0f * k0);   // 2 u'
  return __builtin_fmaf(h * du2 * s, 1.0f - s, s);
}

// Row accesses through a buffer descriptor.  The descriptor spans `bytes` bytes at p; a lane whose byte offset lies
// at or beyond that reads zeros and writes nothing, and the instruction is issued all the same.  The row kernels
// below rely on both halves of that: no lane needs a branch around its loads and stores (a row tail reads as zeros),
// and every pass over a row issues the same number of memory instructions whatever the row length, so that the
// compiler can count exactly how many newer ones may stay in flight when it waits for an older one (the counter is
// in order): a row fetched one step ahead stays in flight while the current one is worked on and stored.  A branch
// around a load or store (even one that is always taken) makes that count a guess, and the guess is zero; a branch
// between a load and its first use lets the compiler sink the load down to the use.  So the row loops below are
// single blocks that handle rows in pairs, a missing second row being a descriptor of zero bytes.
// AUX: 0 = cached, 2 = non-temporal.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ inline __amdgpu_buffer_rsrc_t span_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
template <typename T, int AUX = 0>
__device__ inline void span_load(Vec<T>& v, __amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
  v.raw = __builtin_bit_cast(decltype(v.raw), __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, AUX));
}
template <typename T, int AUX = 0>
__device__ inline void span_store(const Vec<T>& v, __amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v.raw), rs, (int)byte_off, 0, AUX);
}
// one value stored by the lane with in_range_lane_off == 0 only: the others point past the descriptor's 4 or 8 bytes
__device__ inline void span_store_f1(float a, __amdgpu_buffer_rsrc_t rs, uint32_t lane_off) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a), rs, (int)lane_off, 0, 0);
}
__device__ inline void span_store_f2(float a, float b, __amdgpu_buffer_rsrc_t rs, uint32_t lane_off) {
  u32x2 t = {__float_as_uint(a), __float_as_uint(b)};
  __builtin_amdgcn_raw_buffer_store_b64(t, rs, (int)lane_off, 0, 0);
}
// Barrier of the block for LDS traffic only: waits for this wave's LDS operations and meets the others.  Unlike
// __syncthreads() it carries no fence over global memory, which would wait for every load and store in flight.
__device__ inline void block_sync_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// streaming (non-temporal) access to the 16 bytes of a Vec
template <typename T>
__device__ inline void vec_load_nt(Vec<T>& v, const T* p) {
  v.raw = __builtin_bit_cast(decltype(v.raw), __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}
template <typename T>
__device__ inline void vec_store_nt(const Vec<T>& v, T* p) {
  __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v.raw), reinterpret_cast<u32x4*>(p));
}

// streaming (non-temporal) 16-byte / 8-byte accesses: index i counts vectors
typedef float nt_f4 __attribute__((ext_vector_type(4)));
typedef uint32_t nt_u2 __attribute__((ext_vector_type(2)));
__device__ inline float4 nt_load4(const float* base, int64_t i) {
  nt_f4 v = __builtin_nontemporal_load(reinterpret_cast<const nt_f4*>(base) + i);
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ inline void nt_store4(float* base, int64_t i, float4 v) {
  nt_f4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<nt_f4*>(base) + i);
}
__device__ inline void nt_store2(uint32_t* base, int64_t i, uint2 v) {
  nt_u2 t = {v.x, v.y};
  __builtin_nontemporal_store(t, reinterpret_cast<nt_u2*>(base) + i);
}
