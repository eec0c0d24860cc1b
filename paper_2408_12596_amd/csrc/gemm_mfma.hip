// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), float
// accumulation, for the projections of the decoder layer in forward and
// backward:  NT  y = x W^T,   NN  dx = dy W,   TN  dW = dy^T x.
//
// Design
//  * 256 threads = 4 wavefronts in a 2x2 grid; each wavefront owns TM x TN
//    MFMA tiles of 32x32 (block tile 64*TM x 64*TN), K step 64.
//  * Both operands sit in LDS as rows of 64 k-contiguous bf16 (128 B), the
//    16-byte chunks XOR-swizzled with the row index so that the 16-byte
//    fragment reads of 8 consecutive rows cover all banks.
//  * An operand whose reduction index is not the contiguous one in memory (B in
//    NN, both in TN) is copied to LDS as it lies in memory and its fragments are
//    read with the transposing LDS load of gfx950 (ds_read_b64_tr_b16), so no
//    layout pays for a register transpose.
//  * Global loads of step i+1 are issued before the MFMAs of step i (register
//    prefetch); two blocks per CU overlap one block's LDS phase with the
//    other's MFMA phase.
//  * Blocks are renumbered so that each XCD (one L2 each, blocks are dealt
//    round-robin over 8 of them) works on a compact band of tiles.
//  * Gradient GEMMs with few output tiles split K over blockIdx.y and add
//    their partial sums into the float output with hardware atomics.
#include "device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct MfmaGemmParams {
  const bf16* A; const bf16* B; void* C;
  const bf16* bias; const bf16* residual; bf16* aux;
  int64_t M, N, K, lda, ldb, ldc, ldaux;
  int64_t a_ext, b_ext;   // readable extent (multiple of 8) of each operand's contiguous dimension
  int c_float, act, atomic;
  float beta;
  int tiles_m, tiles_n, k_per_split;
};

#define BK 64

__device__ inline int64_t round_up_dev(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
// 16-byte chunk c of row r sits at chunk position c ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1): sixteen consecutive rows
// reading the same logical chunk then touch sixteen different 16-byte slots of the 256-byte bank line
__device__ inline int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ ((row & 7) ^ ((row >> 3) & 1))) << 4); }

// ---- operand tile, reduction index contiguous in memory: elem(r, k) = p[(r0+r)*ld + k] ----
// LDS image: R rows of 64 k-values (128 B), 16-byte chunks XOR-swizzled with the row.
template <int R>
struct DirectTile {
  static constexpr int N = R / 32;
  static constexpr int LDS_BYTES = R * 128;
  static constexpr int FRAG_READS = 1;   // LDS instructions per fragment
  uint4 v[N];
  __device__ void load(const bf16* __restrict__ p, int64_t ld, int64_t r0, int64_t rlim, int64_t k0, int64_t kend) {
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
    const int64_t k = k0 + c * 8;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int64_t r = r0 + rr + i * 32;
      if (r < rlim && k < kend) v[i] = *reinterpret_cast<const uint4*>(p + r * ld + k);
      else v[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ void store(char* lds) const {
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < N; ++i) *reinterpret_cast<uint4*>(lds + lds_off(rr + i * 32, c)) = v[i];
  }
  // fragment of the 32-row MFMA tile starting at row `ro`, k-slice kk (16 values)
  __device__ static bf16x8 frag(const char* lds, int ro, int kk, int lane) {
    return *reinterpret_cast<const bf16x8*>(lds + lds_off(ro + (lane & 31), kk * 2 + (lane >> 5)));
  }
};

// ---- operand tile, reduction index strided in memory: elem(r, k) = p[k*ld + r0 + r] ----
// LDS image: the tile as it lies in memory, 64 k-rows of R values (row stride
// padded by 64 B so that four consecutive k-rows start in different bank
// quarters).  The fragment is read with the LDS transpose load of gfx950
// (ds_read_b64_tr_b16): inside a group of 16 lanes, lane j passes the address
// of 4 consecutive values of k-row j/4 at column 4*(j%4), and receives the 4
// k-values of column j - two such loads give the 8 k-values of an MFMA
// fragment.
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
template <int R>
struct TrTile {
  static constexpr int N = R / 32;              // 16-byte chunks per thread
  static constexpr int STRIDE = R * 2 + 64;     // bytes per k-row
  static constexpr int LDS_BYTES = 64 * STRIDE;
  static constexpr int FRAG_READS = 2;
  uint4 v[N];
  __device__ void load(const bf16* __restrict__ p, int64_t ld, int64_t r0, int64_t rext, int64_t k0, int64_t kend) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int k = idx / (R / 8), c = idx % (R / 8);
      const int64_t r = r0 + c * 8;
      if (k0 + k < kend && r < rext) v[i] = *reinterpret_cast<const uint4*>(p + (k0 + k) * ld + r);
      else v[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ void store(char* lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int idx = threadIdx.x + i * 256;
      const int k = idx / (R / 8), c = idx % (R / 8);
      *reinterpret_cast<uint4*>(lds + k * STRIDE + c * 16) = v[i];
    }
  }
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

template <int LAYOUT, int R> struct ATile { typedef DirectTile<R> type; };
template <int R> struct ATile<GEMM_TN, R> { typedef TrTile<R> type; };
template <int LAYOUT, int R> struct BTile { typedef TrTile<R> type; };
template <int R> struct BTile<GEMM_NT, R> { typedef DirectTile<R> type; };

template <int LAYOUT, int TM, int TN, bool ATOMIC>
__global__ void __launch_bounds__(256, (TM * TN > 4 && LAYOUT == GEMM_TN ? 1 : 2)) gemm_mfma_kernel(MfmaGemmParams p) {
  constexpr int BM = TM * 64, BN = TN * 64;
  typedef typename ATile<LAYOUT, BM>::type TileA;
  typedef typename BTile<LAYOUT, BN>::type TileB;
  __shared__ __attribute__((aligned(16))) char lds_all[TileA::LDS_BYTES + TileB::LDS_BYTES];
  char* const lds_a = lds_all;
  char* const lds_b = lds_all + TileA::LDS_BYTES;

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
  // reading limits: rows/cols past M, N give zeros; along k the contiguous operand may read its zero padding
  const int64_t ka_end = LAYOUT == GEMM_TN ? kend : min(kend, p.a_ext);
  const int64_t kb_end = LAYOUT == GEMM_NT ? min(kend, p.b_ext) : kend;
  const int64_t ra_lim = LAYOUT == GEMM_TN ? p.a_ext : p.M;
  const int64_t rb_lim = LAYOUT == GEMM_NT ? p.N : p.b_ext;

  TileA ta;
  TileB tb;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * (TM * 32), wn = (wave & 1) * (TN * 32);
  const int lr = lane & 31, lk = lane >> 5;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  ta.load(p.A, p.lda, m0, ra_lim, kbeg, ka_end);
  tb.load(p.B, p.ldb, n0, rb_lim, kbeg, kb_end);
  for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
    ta.store(lds_a);
    tb.store(lds_b);
    __syncthreads();
    if (k0 + BK < kend) {
      ta.load(p.A, p.lda, m0, ra_lim, k0 + BK, ka_end);
      tb.load(p.B, p.ldb, n0, rb_lim, k0 + BK, kb_end);
    }
    // fragments of k-slice kk+1 are fetched from LDS while the MFMAs of slice kk run
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = TileA::frag(lds_a, wm + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = TileB::frag(lds_b, wn + j * 32, 0, lane);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[nxt][i] = TileA::frag(lds_a, wm + i * 32, kk + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[nxt][j] = TileB::frag(lds_b, wn + j * 32, kk + 1, lane);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
      // ask the scheduler to keep that overlap: one LDS read in front of each of the first MFMAs of the slice
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int x = 0; x < TileA::FRAG_READS * TM + TileB::FRAG_READS * TN; ++x) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if (x < TM * TN) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        if (TileA::FRAG_READS * TM + TileB::FRAG_READS * TN < TM * TN)
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TileA::FRAG_READS * TM + TileB::FRAG_READS * TN), 0);
      }
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator q of a 32x32 tile is row (q/4)*8 + (lane/32)*4 + q%4,
  // column lane%32.  Each wavefront passes its tiles through a private float
  // staging area in LDS, 16 rows at a time, and reads them back as groups of 8
  // consecutive columns, so that bias / activation / residual work on vectors
  // and every global access is 16 bytes wide.
  if (ATOMIC) {
    // split-K partial sums: float atomics straight from the accumulators, 32
    // lanes on 32 consecutive columns of one row per instruction
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
  constexpr int SW = TN * 32 + 4;          // staging row stride in floats
  constexpr int GROUPS = TN * 4;           // 8-column groups per staging row
  float* stage = reinterpret_cast<float*>(lds_a) + wave * (16 * SW);
  const int64_t n_ext = round_up_dev(p.N, 8);
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
            // the backward pass needs the pre-activation only for gelu': that is what is stashed, formed here from the
            // fp32 value next to the activation itself (they share the sigmoid)
#pragma unroll
            for (int k = 0; k < 8; ++k) gelu_tanh_both_fast(v[k], &v[k], &f[k]);
            t.pack(f); t.store(p.aux + m * p.ldaux + n);
          } else if (p.act == ACT_GELU_BWD) {
            t.load(p.aux + m * p.ldaux + n); t.unpack(f);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] *= f[k];
          }
          if (p.residual) {
            t.load(p.residual + m * p.ldc + n); t.unpack(f);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += f[k];
          }
          if (p.c_float) {
            float* c = reinterpret_cast<float*>(p.C) + m * p.ldc + n;
            {
              float4 lo = make_float4(v[0], v[1], v[2], v[3]), hi = make_float4(v[4], v[5], v[6], v[7]);
              if (p.beta != 0.f) {
                const float4 ol = *reinterpret_cast<const float4*>(c), oh = *reinterpret_cast<const float4*>(c + 4);
                lo.x += p.beta * ol.x; lo.y += p.beta * ol.y; lo.z += p.beta * ol.z; lo.w += p.beta * ol.w;
                hi.x += p.beta * oh.x; hi.y += p.beta * oh.y; hi.z += p.beta * oh.z; hi.w += p.beta * oh.w;
              }
              *reinterpret_cast<float4*>(c) = lo;
              *reinterpret_cast<float4*>(c + 4) = hi;
            }
          } else {
            t.pack(v); t.store(reinterpret_cast<bf16*>(p.C) + m * p.ldc + n);
          }
        }
      }
      wave_lds_sync();
    }
  }
}

template <int TM, int TN, bool ATOMIC>
static void launch_tiles(hipStream_t s, int layout, dim3 grid, const MfmaGemmParams& p) {
  switch (layout) {
    case GEMM_NT: hipLaunchKernelGGL((gemm_mfma_kernel<GEMM_NT, TM, TN, ATOMIC>), grid, dim3(256), 0, s, p); break;
    case GEMM_NN: hipLaunchKernelGGL((gemm_mfma_kernel<GEMM_NN, TM, TN, ATOMIC>), grid, dim3(256), 0, s, p); break;
    default: hipLaunchKernelGGL((gemm_mfma_kernel<GEMM_TN, TM, TN, ATOMIC>), grid, dim3(256), 0, s, p); break;
  }
}

int gemm_bf16_mfma(hipStream_t s, const GemmArgs& a) {
  if (a.M == 0 || a.N == 0) return POPLAR_OK;
  if (a.layout < GEMM_NT || a.layout > GEMM_TN) return poplar_fail(POPLAR_ERR_INVALID, "unknown GEMM layout %d", a.layout);
  MfmaGemmParams p;
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B; p.C = a.C;
  p.bias = (const bf16*)a.bias; p.residual = (const bf16*)a.residual; p.aux = (bf16*)a.aux;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc; p.ldaux = a.ldaux;
  p.c_float = a.c_float; p.act = a.act; p.beta = a.beta; p.atomic = 0;
  // contiguous dimension of each operand: K for row-major [rows, K] operands, M or N for the transposed ones
  const int64_t a_dim = a.layout == GEMM_TN ? a.M : a.K;
  const int64_t b_dim = a.layout == GEMM_NT ? a.K : a.N;
  p.a_ext = round_up(a_dim, 8);
  p.b_ext = round_up(b_dim, 8);
  if (p.a_ext > a.lda || p.b_ext > a.ldb)
    return poplar_fail(POPLAR_ERR_INVALID, "bf16 GEMM needs contiguous dimensions padded to 8 elements (dims %lld/%lld, strides %lld/%lld)",
                       (long long)a_dim, (long long)b_dim, (long long)a.lda, (long long)a.ldb);
  if (a.lda % 8 || a.ldb % 8 || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15))
    return poplar_fail(POPLAR_ERR_INVALID, "bf16 GEMM operands need 16-byte aligned rows");
  // the epilogue moves 8 columns at a time
  if (a.ldc % 8 || a.ldc < round_up(a.N, 8) || ((uintptr_t)a.C & 15) || (a.aux && (a.ldaux % 8 || ((uintptr_t)a.aux & 15))) ||
      (a.bias && ((uintptr_t)a.bias & 15)) || (a.residual && ((uintptr_t)a.residual & 15)))
    return poplar_fail(POPLAR_ERR_INVALID, "bf16 GEMM output rows need 16-byte alignment and a stride covering N rounded up to 8");

  // tile shape: 256x128 when that still fills the chip, else 128x128
  const bool big = cdiv(a.M, 256) * cdiv(a.N, 128) >= 512;
  const int BM = big ? 256 : 128, BN = 128;
  p.tiles_m = (int)cdiv(a.M, BM);
  p.tiles_n = (int)cdiv(a.N, BN);
  const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
  // split K only for plain float-output GEMMs (weight gradients) that leave CUs idle
  int splits = 1;
  const bool plain = a.c_float && !a.bias && !a.residual && a.act == ACT_NONE;
  if (plain && tiles < 384 && !a.no_atomics) {
    splits = (int)std::min<int64_t>(cdiv(768, tiles), cdiv(a.K, 512));
    if (splits < 1) splits = 1;
  }
  p.k_per_split = (int)round_up(cdiv(a.K, splits), BK);
  splits = (int)cdiv(a.K, p.k_per_split);
  if (splits > 1) {
    p.atomic = 1;
    if (a.beta == 0.f) {
      if (a.ldc != a.N) {
        POPLAR_TRY(fill_zero_2d(s, a.C, a.M, a.N, a.ldc));
      } else {
        POPLAR_TRY(fill_zero(s, a.C, a.M * a.N * 4));
      }
    }
  }
  dim3 grid((unsigned)tiles, (unsigned)splits);
  poplar_gemm_kernel_launches += 1;
  if (p.atomic) {
    if (big) launch_tiles<4, 2, true>(s, a.layout, grid, p);
    else launch_tiles<2, 2, true>(s, a.layout, grid, p);
  } else {
    if (big) launch_tiles<4, 2, false>(s, a.layout, grid, p);
    else launch_tiles<2, 2, false>(s, a.layout, grid, p);
  }
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
