// Flash-style causal attention on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16): forward, and backward as two kernels (dK/dV per
// key tile, dQ per query tile) so that no result depends on atomics.
//
// Data: the fused projection output qkv [B*S, 3H] (q | k | v thirds, head h in
// columns h*D..(h+1)*D of each), o and dout [B*S, H], lse and delta float
// [B, nh, S].  D is 64 or 128.
//
// MFMA conventions used below (32x32 tile, K = 16 per instruction):
//   A fragment: lane holds row  (lane % 32), k-slots (lane / 32) * 8 + 0..7
//   B fragment: lane holds col  (lane % 32), the same k-slots
//   C tile    : lane holds col  (lane % 32); register i is row (i/4)*8 + (lane/32)*4 + i%4
// A probability tile therefore leaves the softmax already in B-fragment form
// if the k-slot e of lane half g inside a 16-row chunk is read as row
// (e/4)*8 + g*4 + e%4.  The matching A operand (V^T, K^T, Q^T, dO^T) is built
// when its tile is copied to LDS: a thread loads the 8 rows 16j + 4g +
// {0,1,2,3,8,9,10,11} (16 bytes each), transposes them in registers and writes
// one 16-byte chunk per column, so the fragment read is a single 16-byte LDS
// load and the probabilities never touch LDS.
//
// Forward and dQ work on S^T = K Q^T (lane = query), which keeps the running
// max / sum / rescale of a query inside one lane (plus one exchange between the
// two lane halves).  dK/dV works on S = Q K^T (lane = key).
#include "device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f

__device__ inline bf16x8 as_frag(uint4 v) { return *reinterpret_cast<bf16x8*>(&v); }

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
// two floats to packed bfloat16 (round to nearest even) with one v_cvt_pk_bf16_f32
__device__ inline uint32_t pack_bf16(float a, float b) {
  floatx2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return *reinterpret_cast<uint32_t*>(&h);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// registers 8s .. 8s+7 of a C tile as a B fragment
__device__ inline bf16x8 regs_to_frag(const floatx16& c, int s) {
  uint4 v = make_uint4(pack_bf16(c[8 * s + 0], c[8 * s + 1]), pack_bf16(c[8 * s + 2], c[8 * s + 3]),
                       pack_bf16(c[8 * s + 4], c[8 * s + 5]), pack_bf16(c[8 * s + 6], c[8 * s + 7]));
  return as_frag(v);
}

// ---- 64-row tile with D contiguous columns, copied as it is ("direct") -------
template <int D>
struct DirectRows {
  static constexpr int NC = 64 * D / 8 / 256;  // 16-byte chunks per thread
  static constexpr int ROWB = D * 2;
  uint4 v[NC];
  // rows r0 .. r0+63 of a [*, ld] matrix starting at column 0 of `p`; rows >= rlim read as zero
  __device__ void load(const bf16* __restrict__ p, int64_t ld, int r0, int rlim) {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int row = idx / (D / 8), c = idx % (D / 8);
      if (r0 + row < rlim) v[i] = *reinterpret_cast<const uint4*>(p + (int64_t)(r0 + row) * ld + c * 8);
      else v[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ void store(char* lds) const {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int row = idx / (D / 8), c = idx % (D / 8);
      *reinterpret_cast<uint4*>(lds + row * ROWB + ((c ^ (row & 7)) << 4)) = v[i];
    }
  }
  // A fragment: row `row` of the tile, k-slice s (16 columns), lane half g
  __device__ static bf16x8 frag(const char* lds, int row, int s, int g) {
    return *reinterpret_cast<const bf16x8*>(lds + row * ROWB + (((2 * s + g) ^ (row & 7)) << 4));
  }
};

// ---- 64-row tile copied transposed, rows permuted into k-slot order -----------
// LDS image: D rows (one per column of the source) of 64 values = 128 bytes.
// Threads tid0 .. tid0+D-1 each own one 8x8 block.
template <int D>
struct PermutedTranspose {
  uint4 v[8];
  __device__ static bool mine(int tid0) { return (int)threadIdx.x >= tid0 && (int)threadIdx.x < tid0 + D; }
  __device__ void load(const bf16* __restrict__ p, int64_t ld, int r0, int rlim, int tid0) {
    const int bid = threadIdx.x - tid0;
    const int jg = bid & 7, cx = bid >> 3;   // 8 lanes share a column chunk: their LDS writes fill one 128-byte row
    const int rbase = r0 + 16 * (jg >> 1) + 4 * (jg & 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rbase + (i & 3) + (i >> 2) * 8;
      if (r < rlim) v[i] = *reinterpret_cast<const uint4*>(p + (int64_t)r * ld + cx * 8);
      else v[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ void store(char* lds, int tid0) const {
    const int bid = threadIdx.x - tid0;
    const int jg = bid & 7, cx = bid >> 3;
    const uint32_t* w = reinterpret_cast<const uint32_t*>(&v[0]);  // w[row * 4 + word]
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      uint32_t o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t lo = w[(2 * j) * 4 + (x >> 1)], hi = w[(2 * j + 1) * 4 + (x >> 1)];
        o[j] = (x & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
      const int row = cx * 8 + x;
      *reinterpret_cast<uint4*>(lds + row * 128 + ((jg ^ (row & 7)) << 4)) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
  // A fragment: row `row` (a source column), 16-row chunk j of the source, lane half g
  __device__ static bf16x8 frag(const char* lds, int row, int j, int g) {
    return *reinterpret_cast<const bf16x8*>(lds + row * 128 + (((2 * j + g) ^ (row & 7)) << 4));
  }
};

// B fragments of one row of a [*, ld] matrix kept in registers: D/16 slices
template <int D>
__device__ inline void load_row_frags(bf16x8* f, const bf16* __restrict__ p, int64_t ld, int row, int rlim, int g) {
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < rlim) v = *reinterpret_cast<const uint4*>(p + (int64_t)row * ld + s * 16 + g * 8);
    f[s] = as_frag(v);
  }
}

// store a transposed accumulator (lane = row of the output, 4 consecutive columns per register group)
template <int D>
__device__ inline void store_rows_from_transposed(bf16* __restrict__ p, int64_t ld, int row, int rlim, int g,
                                                  const floatx16* acc, float scale) {
  if (row >= rlim) return;
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      uint2 w;
      w.x = pack_bf16(acc[ct][4 * q4 + 0] * scale, acc[ct][4 * q4 + 1] * scale);
      w.y = pack_bf16(acc[ct][4 * q4 + 2] * scale, acc[ct][4 * q4 + 3] * scale);
      *reinterpret_cast<uint2*>(p + (int64_t)row * ld + ct * 32 + q4 * 8 + g * 4) = w;
    }
}

__device__ inline void zero_acc(floatx16& a) {
#pragma unroll
  for (int i = 0; i < 16; ++i) a[i] = 0.f;
}

// =============================================================================
// forward
// =============================================================================
template <int D>
__global__ void __launch_bounds__(256) flash_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ o, float* __restrict__ lse,
                                                         int S, int nh, int causal, float scale) {
  __shared__ __attribute__((aligned(16))) char k_lds[64 * D * 2];
  __shared__ __attribute__((aligned(16))) char vt_lds[D * 128];
  const int H = nh * D;
  const int64_t ld = 3 * (int64_t)H;
  const int qtiles = (S + 127) / 128;
  const int qt = qtiles - 1 - (int)(blockIdx.x % qtiles);  // heavy (late) query tiles first
  const int h = (int)((blockIdx.x / qtiles) % nh);
  const int b = (int)(blockIdx.x / ((int64_t)qtiles * nh));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int q0 = qt * 128;
  const int q = q0 + wave * 32 + lr;
  const bf16* base = qkv + (int64_t)b * S * ld + h * D;
  const bf16* kp = base + H;
  const bf16* vp = base + 2 * H;

  bf16x8 qf[D / 16];
  load_row_frags<D>(qf, base, ld, q, S, g);
  floatx16 oacc[D / 32];
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct) zero_acc(oacc[ct]);
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = scale * LOG2E;
  const int kv_end = causal ? min(S, q0 + 128) : S;

  DirectRows<D> kt;
  PermutedTranspose<D> vt;
  const bool vmine = PermutedTranspose<D>::mine(0);
  kt.load(kp, ld, 0, S);
  if (vmine) vt.load(vp, ld, 0, S, 0);
  for (int kv0 = 0; kv0 < kv_end; kv0 += 64) {
    kt.store(k_lds);
    if (vmine) vt.store(vt_lds, 0);
    __syncthreads();
    if (kv0 + 64 < kv_end) {
      kt.load(kp, ld, kv0 + 64, S);
      if (vmine) vt.load(vp, ld, kv0 + 64, S, 0);
    }
    // S^T tiles: rows = keys kv0 + u*32 + .., cols = this wave's queries
    floatx16 st[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      zero_acc(st[u]);
#pragma unroll
      for (int s = 0; s < D / 16; ++s)
        st[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(DirectRows<D>::frag(k_lds, u * 32 + lr, s, g), qf[s], st[u], 0, 0, 0);
    }
    // only tiles that touch the diagonal of this wave's queries or the end of the sequence need the mask
    const int qw0 = q0 + wave * 32;
    if ((causal && kv0 + 63 > qw0) || kv0 + 64 > S) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kv = kv0 + u * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          const bool ok = kv < S && (!causal || kv <= q);
          st[u][i] = ok ? st[u][i] : -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, st[u][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);                   // running max of the raw scores
    const float mc = (m_new == -INFINITY ? 0.f : m_new) * c2;
    const float alpha = fast_exp2(m_run * c2 - mc);         // m_run = -inf gives 0
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        st[u][i] = fast_exp2(__builtin_fmaf(st[u][i], c2, -mc));
        psum += st[u][i];
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[ct][i] *= alpha;
    // O^T += V^T P^T
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x8 pb = regs_to_frag(st[j >> 1], j & 1);
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct)
        oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(PermutedTranspose<D>::frag(vt_lds, ct * 32 + lr, j, g), pb, oacc[ct], 0, 0, 0);
    }
    __syncthreads();
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  store_rows_from_transposed<D>(o + (int64_t)b * S * H + h * D, H, q, S, g, oacc, inv);
  if (g == 0 && q < S) lse[((int64_t)b * nh + h) * S + q] = (m_run * c2 + log2f(l_tot)) * LN2;
}

// =============================================================================
// delta[b,h,i] = sum_c dout[i,c] * o[i,c]
// =============================================================================
__global__ void __launch_bounds__(256) flash_delta_kernel(const bf16* __restrict__ o, const bf16* __restrict__ dout, float* __restrict__ delta,
                                                           int64_t rows, int S, int nh, int D) {
  // one thread per 8 columns; D/8 consecutive threads share a (token, head) row
  const int per = D / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = idx / per;  // over tokens * nh
  float acc = 0.f;
  if (row < rows) {
    const int c = (int)(idx % per) * 8;
    const int64_t t = row / nh;
    const int h = (int)(row % nh);
    const int64_t off = t * (int64_t)nh * D + h * D + c;
    float a[8], d[8];
    Vec<bf16> v; v.load(o + off); v.unpack(a);
    v.load(dout + off); v.unpack(d);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += a[k] * d[k];
  }
  for (int ofs = per >> 1; ofs > 0; ofs >>= 1) acc += __shfl_xor(acc, ofs, 64);
  if (row < rows && (idx % per) == 0) {
    const int64_t t = row / nh;
    const int h = (int)(row % nh);
    delta[((t / S) * nh + h) * S + (t % S)] = acc;
  }
}

// =============================================================================
// backward, dQ: block = 128 queries, loop over key tiles (S^T form, lane = query)
// =============================================================================
template <int D>
__global__ void __launch_bounds__(256) flash_bwd_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            bf16* __restrict__ dqkv, int S, int nh, int causal, float scale) {
  __shared__ __attribute__((aligned(16))) char k_lds[64 * D * 2];
  __shared__ __attribute__((aligned(16))) char v_lds[64 * D * 2];
  __shared__ __attribute__((aligned(16))) char kt_lds[D * 128];
  const int H = nh * D;
  const int64_t ld = 3 * (int64_t)H;
  const int qtiles = (S + 127) / 128;
  const int qt = qtiles - 1 - (int)(blockIdx.x % qtiles);
  const int h = (int)((blockIdx.x / qtiles) % nh);
  const int b = (int)(blockIdx.x / ((int64_t)qtiles * nh));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int q0 = qt * 128;
  const int q = q0 + wave * 32 + lr;
  const bf16* base = qkv + (int64_t)b * S * ld + h * D;
  const bf16* kp = base + H;
  const bf16* vp = base + 2 * H;

  bf16x8 qf[D / 16], dof[D / 16];
  load_row_frags<D>(qf, base, ld, q, S, g);
  load_row_frags<D>(dof, dout + (int64_t)b * S * H + h * D, H, q, S, g);
  const float c2 = scale * LOG2E;
  const int64_t stat = ((int64_t)b * nh + h) * S + q;
  const float lse2 = q < S ? lse[stat] * LOG2E : 0.f;
  const float dl = q < S ? delta[stat] : 0.f;
  floatx16 dq[D / 32];
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct) zero_acc(dq[ct]);
  const int kv_end = causal ? min(S, q0 + 128) : S;

  DirectRows<D> kt, vt;
  PermutedTranspose<D> ktt;
  const bool tmine = PermutedTranspose<D>::mine(0);
  kt.load(kp, ld, 0, S);
  vt.load(vp, ld, 0, S);
  if (tmine) ktt.load(kp, ld, 0, S, 0);
  for (int kv0 = 0; kv0 < kv_end; kv0 += 64) {
    kt.store(k_lds);
    vt.store(v_lds);
    if (tmine) ktt.store(kt_lds, 0);
    __syncthreads();
    if (kv0 + 64 < kv_end) {
      kt.load(kp, ld, kv0 + 64, S);
      vt.load(vp, ld, kv0 + 64, S);
      if (tmine) ktt.load(kp, ld, kv0 + 64, S, 0);
    }
    floatx16 st[2], dpt[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      zero_acc(st[u]);
      zero_acc(dpt[u]);
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        st[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(DirectRows<D>::frag(k_lds, u * 32 + lr, s, g), qf[s], st[u], 0, 0, 0);
        dpt[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(DirectRows<D>::frag(v_lds, u * 32 + lr, s, g), dof[s], dpt[u], 0, 0, 0);
      }
      if ((causal && kv0 + 63 > q0 + wave * 32) || kv0 + 64 > S || q0 + 128 > S) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kv = kv0 + u * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          const bool ok = kv < S && q < S && (!causal || kv <= q);
          const float p = ok ? fast_exp2(__builtin_fmaf(st[u][i], c2, -lse2)) : 0.f;
          st[u][i] = p * (dpt[u][i] - dl);   // dS^T
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = fast_exp2(__builtin_fmaf(st[u][i], c2, -lse2));
          st[u][i] = p * (dpt[u][i] - dl);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x8 dsb = regs_to_frag(st[j >> 1], j & 1);
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct)
        dq[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(PermutedTranspose<D>::frag(kt_lds, ct * 32 + lr, j, g), dsb, dq[ct], 0, 0, 0);
    }
    __syncthreads();
  }
  store_rows_from_transposed<D>(dqkv + (int64_t)b * S * ld + h * D, ld, q, S, g, dq, scale);
}

// =============================================================================
// backward, dK and dV: block = 128 keys, loop over query tiles (S form, lane = key)
// =============================================================================
template <int D>
__global__ void __launch_bounds__(256) flash_bwd_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                             const float* __restrict__ lse, const float* __restrict__ delta,
                                                             bf16* __restrict__ dqkv, int S, int nh, int causal, float scale) {
  __shared__ __attribute__((aligned(16))) char q_lds[64 * D * 2];
  __shared__ __attribute__((aligned(16))) char do_lds[64 * D * 2];
  __shared__ __attribute__((aligned(16))) char qt_lds[D * 128];
  __shared__ __attribute__((aligned(16))) char dot_lds[D * 128];
  __shared__ __attribute__((aligned(16))) float lse_lds[64];
  __shared__ __attribute__((aligned(16))) float delta_lds[64];
  const int H = nh * D;
  const int64_t ld = 3 * (int64_t)H;
  const int ktiles = (S + 127) / 128;
  const int ktile = (int)(blockIdx.x % ktiles);   // early key tiles see the most queries: they come first
  const int h = (int)((blockIdx.x / ktiles) % nh);
  const int b = (int)(blockIdx.x / ((int64_t)ktiles * nh));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int kvb = ktile * 128;
  const int kv = kvb + wave * 32 + lr;
  const bf16* qp = qkv + (int64_t)b * S * ld + h * D;
  const bf16* dop = dout + (int64_t)b * S * H + h * D;
  const float* lsep = lse + ((int64_t)b * nh + h) * S;
  const float* delp = delta + ((int64_t)b * nh + h) * S;

  bf16x8 kf[D / 16], vf[D / 16];
  load_row_frags<D>(kf, qp + H, ld, kv, S, g);
  load_row_frags<D>(vf, qp + 2 * H, ld, kv, S, g);
  floatx16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct) { zero_acc(dk[ct]); zero_acc(dv[ct]); }
  const float c2 = scale * LOG2E;
  const int q_begin = causal ? (kvb / 64) * 64 : 0;

  DirectRows<D> qd, dod;
  PermutedTranspose<D> qtt, dott;
  constexpr int T1 = D == 64 ? 128 : 128;  // first thread of the dO^T loaders
  const bool qmine = PermutedTranspose<D>::mine(0), dmine = PermutedTranspose<D>::mine(T1);
  float lse_r = 0.f, del_r = 0.f;
  auto load_tile = [&](int q0) {
    qd.load(qp, ld, q0, S);
    dod.load(dop, H, q0, S);
    if (qmine) qtt.load(qp, ld, q0, S, 0);
    if (dmine) dott.load(dop, H, q0, S, T1);
    if (threadIdx.x < 64) {
      const int qq = q0 + threadIdx.x;
      lse_r = qq < S ? lsep[qq] * LOG2E : 0.f;
      del_r = qq < S ? delp[qq] : 0.f;
    }
  };
  load_tile(q_begin);
  for (int q0 = q_begin; q0 < S; q0 += 64) {
    qd.store(q_lds);
    dod.store(do_lds);
    if (qmine) qtt.store(qt_lds, 0);
    if (dmine) dott.store(dot_lds, T1);
    if (threadIdx.x < 64) { lse_lds[threadIdx.x] = lse_r; delta_lds[threadIdx.x] = del_r; }
    __syncthreads();
    if (q0 + 64 < S) load_tile(q0 + 64);
    floatx16 sm[2], dp[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      zero_acc(sm[u]);
      zero_acc(dp[u]);
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        sm[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(DirectRows<D>::frag(q_lds, u * 32 + lr, s, g), kf[s], sm[u], 0, 0, 0);
        dp[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(DirectRows<D>::frag(do_lds, u * 32 + lr, s, g), vf[s], dp[u], 0, 0, 0);
      }
      if ((causal && q0 < kvb + wave * 32 + 31) || q0 + 64 > S || kvb + 128 > S) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ql = u * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          const int qq = q0 + ql;
          const bool ok = qq < S && kv < S && (!causal || kv <= qq);
          const float p = ok ? fast_exp2(__builtin_fmaf(sm[u][i], c2, -lse_lds[ql])) : 0.f;
          dp[u][i] = p * (dp[u][i] - delta_lds[ql]);   // dS
          sm[u][i] = p;                                 // P
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ql = u * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          const float p = fast_exp2(__builtin_fmaf(sm[u][i], c2, -lse_lds[ql]));
          dp[u][i] = p * (dp[u][i] - delta_lds[ql]);
          sm[u][i] = p;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x8 pb = regs_to_frag(sm[j >> 1], j & 1);
      const bf16x8 dsb = regs_to_frag(dp[j >> 1], j & 1);
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct) {
        dv[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(PermutedTranspose<D>::frag(dot_lds, ct * 32 + lr, j, g), pb, dv[ct], 0, 0, 0);
        dk[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(PermutedTranspose<D>::frag(qt_lds, ct * 32 + lr, j, g), dsb, dk[ct], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  bf16* outp = dqkv + (int64_t)b * S * ld + h * D;
  store_rows_from_transposed<D>(outp + H, ld, kv, S, g, dk, scale);
  store_rows_from_transposed<D>(outp + 2 * H, ld, kv, S, g, dv, 1.0f);
}

// =============================================================================
// launchers
// =============================================================================
static int check_flash(int B, int S, int nh, int d, const void* qkv) {
  if (d != 64 && d != 128) return poplar_fail(POPLAR_ERR_INVALID, "bf16 attention needs head_dim 64 or 128, got %d", d);
  if ((uintptr_t)qkv & 15) return poplar_fail(POPLAR_ERR_INVALID, "qkv must be 16-byte aligned");
  if ((int64_t)B * nh * ((S + 127) / 128) > 0x7fffffff) return poplar_fail(POPLAR_ERR_INVALID, "attention grid too large");
  return POPLAR_OK;
}

int attn_fwd_flash(hipStream_t s, int B, int S, int nh, int d, int causal, const void* qkv, void* o, float* lse) {
  POPLAR_TRY(check_flash(B, S, nh, d, qkv));
  if (B == 0 || S == 0) return POPLAR_OK;
  const float scale = 1.0f / sqrtf((float)d);
  dim3 grid((unsigned)((int64_t)B * nh * ((S + 127) / 128)));
  if (d == 64) hipLaunchKernelGGL(flash_fwd_kernel<64>, grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, S, nh, causal, scale);
  else hipLaunchKernelGGL(flash_fwd_kernel<128>, grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, S, nh, causal, scale);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int attn_bwd_flash(hipStream_t s, int B, int S, int nh, int d, int causal, const void* qkv, const void* o, const void* dout,
                   const float* lse, void* dqkv, float* delta) {
  POPLAR_TRY(check_flash(B, S, nh, d, qkv));
  if (B == 0 || S == 0) return POPLAR_OK;
  const float scale = 1.0f / sqrtf((float)d);
  const int64_t rows = (int64_t)B * S * nh;
  hipLaunchKernelGGL(flash_delta_kernel, dim3((unsigned)cdiv(rows * (d / 8), 256)), dim3(256), 0, s, (const bf16*)o, (const bf16*)dout, delta,
                     rows, S, nh, d);
  POPLAR_LAUNCH_CHECK();
  dim3 grid((unsigned)((int64_t)B * nh * ((S + 127) / 128)));
  if (d == 64) {
    hipLaunchKernelGGL(flash_bwd_dkv_kernel<64>, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, S, nh, causal, scale);
    hipLaunchKernelGGL(flash_bwd_dq_kernel<64>, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, S, nh, causal, scale);
  } else {
    hipLaunchKernelGGL(flash_bwd_dkv_kernel<128>, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, S, nh, causal, scale);
    hipLaunchKernelGGL(flash_bwd_dq_kernel<128>, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, S, nh, causal, scale);
  }
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
