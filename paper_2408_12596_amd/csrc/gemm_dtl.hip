// bf16 GEMM on the gfx950 matrix cores with global -> LDS direct loads
// (buffer_load_dwordx4 ... lds) and a two-stage LDS pipeline.
//
// Same math and operand layouts as gemm_mfma.hip (NT, NN, TN; float
// accumulation; fused epilogues); this kernel is the one the large projections
// run on.  What differs:
//  * Tiles travel HBM/L2 -> LDS without passing through registers: each
//    wavefront issues 16-byte-per-lane buffer loads whose 64 results land in
//    one contiguous KiB of LDS (lane L at base + 16 L; measured on the device).
//    The LDS image is swizzled (k-contiguous operands) or padded (k-strided
//    operands, read with ds_read_b64_tr_b16), so the permutation is applied on
//    the global side: every lane computes once which 16 bytes belong at its LDS
//    position.  Rows past the matrix are out of the buffer's range and arrive
//    as zeros.
//  * Two LDS stages, one barrier per K step of 64: the loads of step i+1 are in
//    flight while the MFMAs of step i run; no ds_write instructions at all.
//  * 256x256 block tile on 8 wavefronts (2 x 4, each 128x64) for large
//    problems, 128x128 on 4 wavefronts (two blocks per CU) for small ones.
// Preconditions checked by the launcher: K a multiple of 64 unless both operands
// are k-strided (their K tail is out of range, hence zero), operand extents
// below 4 GiB (32-bit buffer offsets).
#include "device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

struct DtlGemmParams {
  const bf16* A; const bf16* B; void* C;
  const bf16* bias; const bf16* residual; bf16* aux;
  int64_t M, N, K, lda, ldb, ldc, ldaux;
  uint32_t a_records, b_records;   // bytes of A / B that may be read
  int c_float, act;
  float beta;
  int tiles_m, tiles_n, k_per_split;
};

#define DTL_BK 64
#define OOB_OFFSET 0xfffffff0u

__device__ inline int dtl_swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// k-contiguous operand: R rows of 64 k-values (128 B), 16-byte chunks XOR-swizzled
template <int R>
struct DirectImage {
  static constexpr int BYTES = R * 128;
  static constexpr int LOADS = BYTES / 1024;
  static constexpr int FRAG_READS = 1;
  // byte offset (k = 0) of the 16 bytes that belong at LDS position idx*1024 + lane*16
  __device__ static uint32_t lane_offset(int idx, int lane, int64_t ld, int64_t r0) {
    const int row = idx * 8 + (lane >> 3);
    const int c = (lane & 7) ^ dtl_swz(row);
    const int64_t off = ((r0 + row) * ld + c * 8) * 2;
    return off < (int64_t)OOB_OFFSET ? (uint32_t)off : OOB_OFFSET;
  }
  __device__ static uint32_t k_step(int64_t ld) { return DTL_BK * 2; }   // bytes added per K step
  __device__ static bf16x8 frag(const char* lds, int ro, int kk, int lane) {
    const int row = ro + (lane & 31);
    return *reinterpret_cast<const bf16x8*>(lds + row * 128 + (((kk * 2 + (lane >> 5)) ^ dtl_swz(row)) << 4));
  }
};

// k-strided operand: the tile as it lies in memory, 64 k-rows of R values, row stride R*2 + 64 bytes
template <int R>
struct StridedImage {
  static constexpr int STRIDE = R * 2 + 64;
  static constexpr int BYTES = 64 * STRIDE;
  static constexpr int LOADS = BYTES / 1024;
  static constexpr int FRAG_READS = 2;
  static_assert(BYTES % 1024 == 0, "image must be whole KiB");
  __device__ static uint32_t lane_offset(int idx, int lane, int64_t ld, int64_t r0) {
    const int pos = idx * 1024 + lane * 16;
    const int krow = pos / STRIDE, col = pos % STRIDE;
    if (col >= R * 2) return OOB_OFFSET;   // padding
    const int64_t off = ((int64_t)krow * ld + r0 + col / 2) * 2;
    return off < (int64_t)OOB_OFFSET ? (uint32_t)off : OOB_OFFSET;
  }
  __device__ static uint32_t k_step(int64_t ld) { return (uint32_t)(DTL_BK * ld * 2); }
  __device__ static bf16x8 frag(const char* lds, int ro, int kk, int lane) {
    const int j = lane & 15, gi = (lane >> 4) & 1, lk = lane >> 5;
    const char* q = lds + (kk * 16 + lk * 8 + (j >> 2)) * STRIDE + (ro + gi * 16 + 4 * (j & 3)) * 2;
    typedef __attribute__((address_space(3))) bf16x4* lds_ptr;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(q));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(q + 4 * STRIDE));
    bf16x8 f;
    f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3]; f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
    return f;
  }
};

// One 16-byte-per-lane load of a wavefront straight into the KiB of LDS at `dst`
// (lane L lands at dst + 16 L).  Kept out of the kernel template: the host pass
// drops a kernel template whose body names this builtin directly.
__device__ inline void load_kib_to_lds(__amdgpu_buffer_rsrc_t rsrc, char* dst, uint32_t lane_byte_offset) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)dst, 16, lane_byte_offset, 0, 0, 0);
}

template <int LAYOUT, int R> struct ImageA { typedef DirectImage<R> type; };
template <int R> struct ImageA<GEMM_TN, R> { typedef StridedImage<R> type; };
template <int LAYOUT, int R> struct ImageB { typedef StridedImage<R> type; };
template <int R> struct ImageB<GEMM_NT, R> { typedef DirectImage<R> type; };

template <int LAYOUT, int WM, int WN, int TM, int TN, bool ATOMIC>
__global__ void __launch_bounds__(64 * WM * WN, 2) gemm_dtl_kernel(DtlGemmParams p) {
  constexpr int NW = WM * WN;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  typedef typename ImageA<LAYOUT, BM>::type ImA;
  typedef typename ImageB<LAYOUT, BN>::type ImB;
  constexpr int STAGE = ImA::BYTES + ImB::BYTES;
  // two separate arrays: the compiler can tell the stage being filled from the stage being read
  __shared__ __attribute__((aligned(1024))) char stage0[STAGE];
  __shared__ __attribute__((aligned(1024))) char stage1[STAGE];

  // XCD-aware renumbering, then bands of 8 tile rows with the column index fastest inside a band
  const int nt = p.tiles_m * p.tiles_n;
  int id = blockIdx.x;
  {
    const int per = nt / 8;
    if (id < per * 8) id = (id & 7) * per + (id >> 3);
  }
  const int band = 8 * p.tiles_n;
  const int band_id = id / band;
  const int rows_in_band = min(8, p.tiles_m - band_id * 8);
  const int in_band = id - band_id * band;
  const int tile_m = band_id * 8 + in_band % rows_in_band;
  const int tile_n = in_band / rows_in_band;
  const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
  const int64_t kbeg = (int64_t)blockIdx.y * p.k_per_split;
  const int64_t kend = min(p.K, kbeg + p.k_per_split);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / WN) * (TM * 32), wn = (wave % WN) * (TN * 32);
  const int lr = lane & 31, lk = lane >> 5;

  const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, p.a_records, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)p.B, 0, p.b_records, 0x00020000);

  // per-lane source offsets of this wave's loads (wave w takes loads w, w + NW, ...)
  constexpr int LA = (ImA::LOADS + NW - 1) / NW, LB = (ImB::LOADS + NW - 1) / NW;
  uint32_t offa[LA], offb[LB];
  const uint32_t stepa = ImA::k_step(p.lda), stepb = ImB::k_step(p.ldb);
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    offa[i] = ImA::lane_offset(wave + i * NW, lane, p.lda, m0);
    if (offa[i] != OOB_OFFSET) offa[i] += (uint32_t)(kbeg / DTL_BK) * stepa;
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    offb[i] = ImB::lane_offset(wave + i * NW, lane, p.ldb, n0);
    if (offb[i] != OOB_OFFSET) offb[i] += (uint32_t)(kbeg / DTL_BK) * stepb;
  }

  auto issue = [&](char* st) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int idx = wave + i * NW;
      if (idx < ImA::LOADS) {
        load_kib_to_lds(rsrc_a, st + idx * 1024, offa[i]);
        if (offa[i] != OOB_OFFSET) offa[i] += stepa;
      }
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int idx = wave + i * NW;
      if (idx < ImB::LOADS) {
        load_kib_to_lds(rsrc_b, st + ImA::BYTES + idx * 1024, offb[i]);
        if (offb[i] != OOB_OFFSET) offb[i] += stepb;
      }
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  auto compute = [&](const char* st) {
    const char* lds_a = st;
    const char* lds_b = st + ImA::BYTES;
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = ImA::frag(lds_a, wm + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = ImB::frag(lds_b, wn + j * 32, 0, lane);
#pragma unroll
    for (int kk = 0; kk < DTL_BK / 16; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < DTL_BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[nxt][i] = ImA::frag(lds_a, wm + i * 32, kk + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[nxt][j] = ImB::frag(lds_b, wn + j * 32, kk + 1, lane);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
      if (kk + 1 < DTL_BK / 16) {
#pragma unroll
        for (int x = 0; x < ImA::FRAG_READS * TM + ImB::FRAG_READS * TN; ++x) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if (x < TM * TN) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        if (ImA::FRAG_READS * TM + ImB::FRAG_READS * TN < TM * TN)
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (ImA::FRAG_READS * TM + ImB::FRAG_READS * TN), 0);
      }
    }
  };

  // two-stage pipeline: wait for this step's tile, let every wave leave the previous step, start the next
  // tile's loads into the other stage, compute.  (The generated loop waits on vmcnt only at its top: the
  // loads stay in flight during the MFMAs.)
  issue(stage0);
  if constexpr (TM * TN <= 4) {
    // small wave tile: unrolled by two, each stage a compile-time object (measured faster; the large
    // wave tile runs out of registers in this form)
    for (int64_t k0 = kbeg; k0 < kend; k0 += 2 * DTL_BK) {
      __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's tile loads have landed
      __syncthreads();
      if (k0 + DTL_BK < kend) issue(stage1);
      compute(stage0);
      if (k0 + DTL_BK >= kend) break;
      __builtin_amdgcn_s_waitcnt(0x0f70);
      __syncthreads();
      if (k0 + 2 * DTL_BK < kend) issue(stage0);
      compute(stage1);
    }
  } else {
    int par = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += DTL_BK, par ^= 1) {
      __builtin_amdgcn_s_waitcnt(0x0f70);
      __syncthreads();
      char* cur = par ? stage1 : stage0;
      char* nxt = par ? stage0 : stage1;
      if (k0 + DTL_BK < kend) issue(nxt);
      compute(cur);
    }
  }
  __syncthreads();

  if (ATOMIC) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t n = n0 + wn + j * 32 + lr;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int64_t m = m0 + wm + i * 32 + (q >> 2) * 8 + lk * 4 + (q & 3);
          if (m < p.M && n < p.N) unsafeAtomicAdd(reinterpret_cast<float*>(p.C) + m * p.ldc + n, acc[i][j][q]);
        }
    }
    return;
  }
  // epilogue through a per-wave float staging area (see gemm_mfma.hip)
  constexpr int SW = TN * 32 + 4;
  constexpr int GROUPS = TN * 4;
  float* stage = reinterpret_cast<float*>(stage0) + wave * (16 * SW);
  const int64_t n_ext = (p.N + 7) / 8 * 8;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 8; ++q)
          stage[((q >> 2) * 8 + lk * 4 + (q & 3)) * SW + j * 32 + lr] = acc[i][j][half * 8 + q];
      wave_lds_sync();
#pragma unroll
      for (int it = 0; it < 16 * GROUPS / 64; ++it) {
        const int gid = lane + it * 64;
        const int row = gid / GROUPS, cg = gid % GROUPS;
        const int64_t m = m0 + wm + i * 32 + half * 16 + row;
        const int64_t n = n0 + wn + cg * 8;
        float v[8];
        {
          const float4 lo = *reinterpret_cast<const float4*>(stage + row * SW + cg * 8);
          const float4 hi = *reinterpret_cast<const float4*>(stage + row * SW + cg * 8 + 4);
          v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
        }
        if (m < p.M && n < n_ext) {
          Vec<bf16> t;
          float f[8];
          if (p.bias) {
            t.load(p.bias + n); t.unpack(f);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += f[k];
          }
          if (p.act == ACT_GELU) {
            t.pack(v); t.store(p.aux + m * p.ldaux + n);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = gelu_tanh_fast(v[k]);
          } else if (p.act == ACT_GELU_BWD) {
            t.load(p.aux + m * p.ldaux + n); t.unpack(f);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] *= gelu_tanh_grad_fast(f[k]);
          }
          if (p.residual) {
            t.load(p.residual + m * p.ldc + n); t.unpack(f);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += f[k];
          }
          if (p.c_float) {
            float* c = reinterpret_cast<float*>(p.C) + m * p.ldc + n;
            float4 lo = make_float4(v[0], v[1], v[2], v[3]), hi = make_float4(v[4], v[5], v[6], v[7]);
            if (p.beta != 0.f) {
              const float4 ol = *reinterpret_cast<const float4*>(c), oh = *reinterpret_cast<const float4*>(c + 4);
              lo.x += p.beta * ol.x; lo.y += p.beta * ol.y; lo.z += p.beta * ol.z; lo.w += p.beta * ol.w;
              hi.x += p.beta * oh.x; hi.y += p.beta * oh.y; hi.z += p.beta * oh.z; hi.w += p.beta * oh.w;
            }
            *reinterpret_cast<float4*>(c) = lo;
            *reinterpret_cast<float4*>(c + 4) = hi;
          } else {
            t.pack(v); t.store(reinterpret_cast<bf16*>(p.C) + m * p.ldc + n);
          }
        }
      }
      wave_lds_sync();
    }
  }
}

template <int WM, int WN, int TM, int TN, bool ATOMIC>
static void launch_dtl(hipStream_t s, int layout, dim3 grid, const DtlGemmParams& p) {
  dim3 block(64 * WM * WN);
  switch (layout) {
    case GEMM_NT: hipLaunchKernelGGL((gemm_dtl_kernel<GEMM_NT, WM, WN, TM, TN, ATOMIC>), grid, block, 0, s, p); break;
    case GEMM_NN: hipLaunchKernelGGL((gemm_dtl_kernel<GEMM_NN, WM, WN, TM, TN, ATOMIC>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((gemm_dtl_kernel<GEMM_TN, WM, WN, TM, TN, ATOMIC>), grid, block, 0, s, p); break;
  }
}

// Returns POPLAR_ERR_UNIMPLEMENTED (without touching the error text's meaning for callers) when the
// shape is outside this kernel's preconditions; the caller then uses the register-staged kernel.
int gemm_bf16_dtl(hipStream_t s, const GemmArgs& a) {
  if (a.layout < GEMM_NT || a.layout > GEMM_TN) return POPLAR_ERR_UNIMPLEMENTED;
  // a K tail is fine when every operand reads zeros there: k-strided operands run out of range, a
  // k-contiguous A only if the caller vouches for zero padding up to the next multiple of 64
  const bool a_tail_ok = a.layout == GEMM_NN && a.a_k_pad_zero && a.lda >= round_up(a.K, DTL_BK);
  if (a.layout != GEMM_TN && a.K % DTL_BK && !a_tail_ok) return POPLAR_ERR_UNIMPLEMENTED;
  if (a.K < DTL_BK) return POPLAR_ERR_UNIMPLEMENTED;
  if (a.lda % 8 || a.ldb % 8 || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return POPLAR_ERR_UNIMPLEMENTED;
  if (a.ldc % 8 || a.ldc < round_up(a.N, 8) || ((uintptr_t)a.C & 15) || (a.aux && (a.ldaux % 8 || ((uintptr_t)a.aux & 15))) ||
      (a.bias && ((uintptr_t)a.bias & 15)) || (a.residual && ((uintptr_t)a.residual & 15)))
    return POPLAR_ERR_UNIMPLEMENTED;
  // rows and contiguous extent of each operand as stored
  const int64_t a_rows = a.layout == GEMM_TN ? a.K : a.M, a_cols = a.layout == GEMM_TN ? a.M : a.K;
  const int64_t b_rows = a.layout == GEMM_NT ? a.N : a.K, b_cols = a.layout == GEMM_NT ? a.K : a.N;
  if (round_up(a_cols, 8) > a.lda || round_up(b_cols, 8) > a.ldb) return POPLAR_ERR_UNIMPLEMENTED;
  const int64_t a_bytes = ((a_rows - 1) * a.lda + (a_tail_ok ? round_up(a_cols, DTL_BK) : round_up(a_cols, 8))) * 2;
  const int64_t b_bytes = ((b_rows - 1) * a.ldb + round_up(b_cols, 8)) * 2;
  // 32-bit offsets must also hold for the rows a tile reaches past the matrix
  const int64_t lim = (int64_t)0xfffffff0u - 1024;
  if ((round_up(a_rows, 256) + 64) * a.lda * 2 + 1024 > lim || (round_up(b_rows, 256) + 64) * a.ldb * 2 + 1024 > lim)
    return POPLAR_ERR_UNIMPLEMENTED;

  DtlGemmParams p;
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B; p.C = a.C;
  p.bias = (const bf16*)a.bias; p.residual = (const bf16*)a.residual; p.aux = (bf16*)a.aux;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc; p.ldaux = a.ldaux;
  p.a_records = (uint32_t)a_bytes; p.b_records = (uint32_t)b_bytes;
  p.c_float = a.c_float; p.act = a.act; p.beta = a.beta;

  // Tile shape and K split by a small cost model, in units of one K step of a 256x256 tile on its CU:
  // 256x256 tiles run one block per CU; 128x128 tiles two per CU, each step a quarter of the work at
  // ~85% of the efficiency; the epilogue costs a few K steps (more when it adds with atomics); the
  // launch takes ceil(blocks / slots) rounds.
  const bool plain = a.c_float && !a.bias && !a.residual && a.act == ACT_NONE;
  const int64_t ksteps = cdiv(a.K, DTL_BK);
  bool big = true;
  int splits = 1;
  double best = 1e300;
  for (int cfg = 0; cfg < 2; ++cfg) {
    const bool bg = cfg == 0;
    const int64_t t = cdiv(a.M, bg ? 256 : 128) * cdiv(a.N, bg ? 256 : 128);
    const double slots = bg ? 256.0 : 512.0, step = bg ? 1.0 : 0.59;
    static const int cand[] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16};
    for (int sp : cand) {
      if (sp > 1 && (!plain || ksteps / sp < 8)) break;
      const double epi = sp > 1 ? (bg ? 8.0 : 2.5) : (bg ? 4.0 : 1.2);
      const double rounds = ceil((double)(t * sp) / slots);
      const double cost = rounds * ((double)cdiv(ksteps, sp) * step + epi);
      if (cost < best) { best = cost; big = bg; splits = sp; }
    }
  }
  const int BM = big ? 256 : 128, BN = big ? 256 : 128;
  p.tiles_m = (int)cdiv(a.M, BM);
  p.tiles_n = (int)cdiv(a.N, BN);
  const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
  p.k_per_split = (int)round_up(cdiv(a.K, splits), DTL_BK);
  splits = (int)cdiv(a.K, p.k_per_split);
  const bool atomic = splits > 1;
  if (atomic && a.beta == 0.f) {
    if (a.ldc != a.N) {
      for (int64_t m = 0; m < a.M; ++m) POPLAR_TRY(fill_zero(s, (float*)a.C + m * a.ldc, a.N * 4));
    } else {
      POPLAR_TRY(fill_zero(s, a.C, a.M * a.N * 4));
    }
  }
  dim3 grid((unsigned)tiles, (unsigned)splits);
  if (big) {
    if (atomic) launch_dtl<2, 4, 4, 2, true>(s, a.layout, grid, p);
    else launch_dtl<2, 4, 4, 2, false>(s, a.layout, grid, p);
  } else {
    if (atomic) launch_dtl<2, 2, 2, 2, true>(s, a.layout, grid, p);
    else launch_dtl<2, 2, 2, 2, false>(s, a.layout, grid, p);
  }
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
