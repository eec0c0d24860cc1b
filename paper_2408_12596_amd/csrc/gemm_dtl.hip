// bf16 GEMM on the gfx950 matrix cores with global -> LDS direct loads
// (buffer_load_dwordx4 ... lds) and an LDS pipeline of 2 + 3 slots.
//
// Same math and operand layouts as gemm_mfma.hip (NT, NN, TN; float
// accumulation; fused epilogues); this kernel is the one the large projections
// run on.  What differs:
//  * Tiles travel HBM/L2 -> LDS without passing through registers: each
//    wavefront issues 16-byte-per-lane buffer loads whose 64 results land in
//    one contiguous KiB of LDS (lane L at base + 16 L; measured on the device).
//    The LDS image is swizzled, in 16-byte chunks for k-contiguous operands and
//    in 64-byte granules for k-strided ones (read with ds_read_b64_tr_b16), and
//    the permutation is applied on the global side: every lane computes once
//    which 16 bytes belong at its LDS position.  Rows past the matrix are out of the buffer's range and arrive
//    as zeros.
//  * Two LDS slots for A tiles and three for B tiles, one barrier per K step of
//    64 (four k-slices of 16), no ds_write instructions at all.  The step is
//    software-pipelined by hand: the barrier sits before the last k-slice; B's
//    loads of the tile after next are issued behind the MFMAs of the first two
//    slices (into B's third slot), A's behind those of the last slice (into the
//    slot the barrier has just freed), where the first fragments of the next
//    tile are read as well.  Issued in one burst the loads hold every wavefront
//    at the address unit's queue while the matrix cores idle (measured: 0.4 us
//    of a 1.5 us step at the top of a step; with all of them behind the last
//    slice, a fifth of the kernel's time).  Scheduling fences keep MFMAs, LDS
//    reads and loads in source order; every LDS read is assembly, because the
//    compiler cannot tell the slot being filled from the one being read.
//  * 256x256 block tile on 8 wavefronts (2 x 4, each 128x64) for large
//    problems, 256x192 (4 x 2, each 64x96) where that fills the CUs in whole
//    rounds, 128x128 on 4 wavefronts (two blocks per CU) for small ones.
// Preconditions checked by the launcher: K a multiple of 64 unless both operands
// are k-strided (their K tail is out of range, hence zero), operand extents
// below 4 GiB (32-bit buffer offsets).
#include <hip/hip_ext.h>
#include "device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

struct DtlGemmParams {
  const bf16* A; const bf16* B; void* C;
  const bf16* bias; const bf16* residual; bf16* aux;
  int64_t M, N, K, lda, ldb, ldc, ldaux;
  uint32_t a_records, b_records;   // bytes of A / B that may be read
  int c_float, act;
  float beta;
  int tiles_m, tiles_n, k_per_split;
  float* rowsum;        // TN only, may be null: rowsum[m] (+)= sum_k A(k, m)
  int rowsum_accumulate;
};

// Up to four problems of one layout, tile shape and K extent in a single launch: the block index runs
// over the tiles of all of them (start[i] = first tile of problem i).  Eight slots: a group whose K is cut in
// two runs as twice as many problems (the halves of each).
#define DTL_MAX_GROUP 8
#define DTL_MAX_PROBLEMS 4
struct DtlGroupParams {
  DtlGemmParams g[DTL_MAX_GROUP];
  int start[DTL_MAX_GROUP + 1];
  int n;
};

#define DTL_BK 64

__device__ inline int dtl_swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// k-contiguous operand: R rows of 64 k-values (128 B), 16-byte chunks XOR-swizzled
template <int R>
struct DirectImage {
  static constexpr int BYTES = R * 128;
  static constexpr int LOADS = BYTES / 1024;
  // byte offset (k = 0) of the 16 bytes that belong at LDS position idx*1024 + lane*16
  __device__ static uint32_t lane_offset(int idx, int lane, int64_t ld, int64_t r0) {
    const int row = idx * 8 + (lane >> 3);
    const int c = (lane & 7) ^ dtl_swz(row);
    return (uint32_t)(((r0 + row) * ld + c * 8) * 2);
  }
  __device__ static uint32_t k_step(int64_t ld) { return DTL_BK * 2; }   // bytes added per K step
  // One 16-byte read per fragment, written as assembly like the transposing reads of StridedImage and for the same
  // reason; the invariant stated there holds for it.
  __device__ static bf16x8 frag(const char* lds, int ro, int kk, int lane) {
    const int row = ro + (lane & 31);
    const char* q = lds + row * 128 + (((kk * 2 + (lane >> 5)) ^ dtl_swz(row)) << 4);
    const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)q;
    intx4 f;
    asm volatile("ds_read_b128 %0, %1" : "=v"(f) : "v"(addr));
    return __builtin_bit_cast(bf16x8, f);
  }
};

// k-strided operand: the tile as it lies in memory, 64 k-rows of R values (R * 2 bytes each, no padding); the 64-byte
// granules of k-row r change places by XOR with swz(r), chosen so that four consecutive k-rows (what 32 lanes of a
// transposing read address, 64 bytes of each) fall into four different quarters of the 64 banks: rows of 512 or 256
// bytes all start at bank 0 (swz = r % 4), rows of 384 or 128 bytes alternate between banks 0 and 32 (swz = (r / 2) % 2).
// The permutation is applied on the global side: a granule is 64 consecutive bytes of the row there, too.
template <int R>
struct StridedImage {
  static constexpr int STRIDE = R * 2;
  static constexpr int BYTES = 64 * STRIDE;
  static constexpr int LOADS = BYTES / 1024;
  static_assert(R % 64 == 0 && BYTES % 1024 == 0, "whole granule pairs, whole KiB");
  __device__ static int swz(int krow) { return (STRIDE % 256 == 0) ? (krow & 3) : ((krow >> 1) & 1); }
  __device__ static uint32_t lane_offset(int idx, int lane, int64_t ld, int64_t r0) {
    const int pos = idx * 1024 + lane * 16;
    const int krow = pos / STRIDE, within = pos % STRIDE;
    const int col = (((within >> 6) ^ swz(krow)) << 5) + ((within & 63) >> 1);   // in values
    return (uint32_t)(((int64_t)krow * ld + r0 + col) * 2);
  }
  __device__ static uint32_t k_step(int64_t ld) { return (uint32_t)(DTL_BK * ld * 2); }
  // INVARIANT for the caller: a fragment returned here may feed an MFMA only after an s_waitcnt lgkmcnt(0) that
  // follows this call (slice() begins with one), and a fragment that is read but never used must be named as an input
  // of an empty asm statement after such a wait (the kernel does so for the last K step's reads), or the compiler may
  // hand its registers to something else while the read is still in flight.
  // The reads are written as assembly: the compiler orders the builtin form after every global -> LDS load in
  // flight (the slots rotate, it cannot tell the one being filled from the one being read), which would serialise
  // the pipeline.  The price: the compiler does not see these reads complete either, so the kernel waits on
  // lgkmcnt by hand before it uses a fragment.
  __device__ static bf16x8 frag(const char* lds, int ro, int kk, int lane) {
    // rows ro .. ro + 31 are one granule of every k-row; both reads take k-rows with the same remainder mod 4
    const int j = lane & 15, gi = (lane >> 4) & 1, lk = lane >> 5;
    const int krow = kk * 16 + lk * 8 + (j >> 2);
    const char* q = lds + krow * STRIDE + (((ro >> 5) ^ swz(krow)) << 6) + gi * 32 + 8 * (j & 3);
    const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)q;
    intx2 lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr));
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(hi) : "v"(addr + 4 * STRIDE));
    intx4 f = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, f);
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

// EPI selects the epilogue: 0 float staging (any output and fused operand), 1 float atomics (split K), 2 transposed
// bf16 staging (bf16 output, nothing fused that is indexed by row), 3 float output with nothing fused (the weight
// gradients), stored straight from the accumulators
template <int LAYOUT, int WM, int WN, int TM, int TN, int EPI>
__global__ void __launch_bounds__(64 * WM * WN, 2) gemm_dtl_kernel(DtlGroupParams gp) {
  constexpr bool ATOMIC = EPI == 1, TRANSPOSED = EPI == 2, DIRECT = EPI == 3;
  constexpr int NW = WM * WN;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  typedef typename ImageA<LAYOUT, BM>::type ImA;
  typedef typename ImageB<LAYOUT, BN>::type ImB;
  constexpr int STAGE = ImA::BYTES + ImB::BYTES;
  // LDS: two slots for A tiles, three for B tiles (160 KB at 256 x 256, all there is; 136 KB at 256 x 192; 80 and 40
  // KB for the shapes that run two and four blocks per CU).  With two slots a tile's loads can only go out once its
  // slot is free, i.e. behind the MFMAs of the last k-slice: eight loads per wave in a quarter of the step, and the
  // waves queue at the address unit while the matrix cores idle.  With its third slot B's loads of the tile after
  // next go out behind the first two k-slices (the tile that last held that slot is two steps gone) with more than a
  // step to land, and only A's wait for the barrier.  The slots rotate with period three against A's two, the
  // compiler cannot tell which is being filled and which read, and every LDS read of the K loop is assembly.
  // stage0 / stage1 (A slot + B slot each) double as the epilogue's staging memory.
  __shared__ __attribute__((aligned(1024))) char stage0[STAGE];
  __shared__ __attribute__((aligned(1024))) char stage1[STAGE];
  __shared__ __attribute__((aligned(1024))) char slot3[ImB::BYTES];

  // XCD-aware renumbering over the tiles of the whole group (blocks are dealt round-robin to the 8 XCDs; each
  // XCD gets a contiguous run of tiles), then the problem the tile belongs to, then bands of 8 tile rows
  // (order inside a band: see below)
  int id = blockIdx.x;
  {
    const int per = gp.start[DTL_MAX_GROUP] / 8;
    if (id < per * 8) id = (id & 7) * per + (id >> 3);
  }
  int pi = 0;
#pragma unroll
  for (int i = 1; i < DTL_MAX_GROUP; ++i)
    if (i < gp.n && id >= gp.start[i]) pi = i;
  const DtlGemmParams& p = gp.g[pi];
  id -= gp.start[pi];
  const int band = 8 * p.tiles_n;
  const int band_id = id / band;
  const int rows_in_band = min(8, p.tiles_m - band_id * 8);
  const int in_band = id - band_id * band;
  // Order inside a band: the tiles that run on an XCD at one time (32 CUs, one or two blocks each) should share as
  // few operand panels as possible, i.e. form a near-square patch.  With many tile columns the row index runs
  // fastest (8 rows x 4-8 columns at a time); with up to 8 columns the column index does (whole tile rows: 4-9 rows x
  // all columns), which also keeps a row's tiles in the same round when a band is smaller than a round.
  const bool n_fast = p.tiles_n <= 8;
  const int tile_m = band_id * 8 + (n_fast ? in_band / p.tiles_n : in_band % rows_in_band);
  const int tile_n = n_fast ? in_band % p.tiles_n : in_band / rows_in_band;
  const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
  const int64_t kbeg = (int64_t)blockIdx.y * p.k_per_split;
  const int64_t kend = min(p.K, kbeg + p.k_per_split);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
  const int wm = (wave / WN) * (TM * 32), wn = (wave % WN) * (TN * 32);
  const int lr = lane & 31, lk = lane >> 5;

  // buffer descriptors are rebuilt per step: with zero records every lane is out of range, which turns
  // the loads past the last tile into zero fills without a branch in the MFMA stream
  __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, p.a_records, 0x00020000);
  __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)p.B, 0, p.b_records, 0x00020000);

  // Per-lane source offsets of this wave's loads: wave w takes KiB w, w + NW, ... of each image
  constexpr int LA = ImA::LOADS / NW, LB = ImB::LOADS / NW, NL = LA + LB;
  static_assert(ImA::LOADS % NW == 0 && ImB::LOADS % NW == 0 && LB >= 2 && LB <= 15, "whole loads per wave; B's in two parts; the wait's field");
  uint32_t offa[LA], offb[LB];
  const uint32_t stepa = ImA::k_step(p.lda), stepb = ImB::k_step(p.ldb);
#pragma unroll
  for (int i = 0; i < LA; ++i) offa[i] = ImA::lane_offset(wave + i * NW, lane, p.lda, m0) + (uint32_t)(kbeg / DTL_BK) * stepa;
#pragma unroll
  for (int i = 0; i < LB; ++i) offb[i] = ImB::lane_offset(wave + i * NW, lane, p.ldb, n0) + (uint32_t)(kbeg / DTL_BK) * stepb;

  // load number l (0 .. NL-1) of this wave's share of a tile: A's first (into slot sta), then B's (into slot stb)
  auto load_ab = [&](char* sta, char* stb, int l) __attribute__((always_inline)) {
    if (l < LA) {
      load_kib_to_lds(rsrc_a, sta + (wave + l * NW) * 1024, offa[l]);
      offa[l] += stepa;
    } else {
      load_kib_to_lds(rsrc_b, stb + (wave + (l - LA) * NW) * 1024, offb[l - LA]);
      offb[l - LA] += stepb;
    }
  };
  auto load_tile = [&](char* st) __attribute__((always_inline)) {
#pragma unroll
    for (int l = 0; l < NL; ++l) load_ab(st, st + ImA::BYTES, l);
  };

  // Second operand of the epilogue (the stashed gelu' factor for the backward of GeLU, or the residual; the launcher admits
  // one of the two), 16 bytes per lane for each 16-row group of the wave tile.  The first TMC tile rows are
  // fetched here, before the K loop, the rest at the start of the epilogue behind the first chunk's work: the
  // epilogue then never waits on memory for them.
  constexpr int SW = TN * 32 + 4;
  constexpr int GROUPS = TN * 4;
  constexpr int ITS = 16 * GROUPS / 64;
  constexpr int TMC = TM >= 4 ? 2 : TM;
  static_assert(TM == TMC || TM == 2 * TMC, "one or two chunks");
  const int64_t n_ext = (p.N + 7) / 8 * 8;
  const bf16* extra = p.act == ACT_GELU_BWD ? p.aux : p.residual;
  const int64_t ldx = p.act == ACT_GELU_BWD ? p.ldaux : p.ldc;
  uint4 pre[2][TMC][2][ITS];
  auto prefetch = [&](int c) __attribute__((always_inline)) {
    if (!extra) return;
#pragma unroll
    for (int i = 0; i < TMC; ++i)
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
          const int gid = lane + it * 64;
          const int64_t m = m0 + wm + (c * TMC + i) * 32 + half * 16 + gid / GROUPS;
          const int64_t n = n0 + wn + (gid % GROUPS) * 8;
          pre[c][i][half][it] = make_uint4(0, 0, 0, 0);
          if (m < p.M && n < n_ext) pre[c][i][half][it] = *reinterpret_cast<const uint4*>(extra + m * ldx + n);
        }
  };
  if (EPI == 0) prefetch(0);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  // Row sums of A (the bias gradient that belongs to a weight gradient): the waves on the first column of tiles
  // also add up their A fragments, lane by lane (a lane holds 8 k-values of one row: four two-element dot
  // products with ones); the two k-halves of a row meet in the epilogue.
  const bool do_rs = LAYOUT == GEMM_TN && p.rowsum != nullptr && tile_n == 0 && wn == 0;
  float rs[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) rs[i] = 0.f;

  // Fragments of k-slice kk of a stage; f = 0 .. TM+TN-1 in the order the MFMAs first need them
  bf16x8 fa[2][TM], fb[2][TN];
  auto read_frag = [&](const char* sta, const char* stb, int kk, int buf, int f) __attribute__((always_inline)) {
    // order: a0, b0, b1 .., a1, a2 ..
    if (f == 0) fa[buf][0] = ImA::frag(sta, wm, kk, lane);
    else if (f <= TN) fb[buf][f - 1] = ImB::frag(stb, wn + (f - 1) * 32, kk, lane);
    else fa[buf][f - TN] = ImA::frag(sta, wm + (f - TN) * 32, kk, lane);
  };
  constexpr int NM = TM * TN, NF = TM + TN;
  // One k-slice: the NM MFMAs in source order, with the fragment reads of the next slice (slots rsta / rstb, slice rkk) and the tile loads number l0 .. l0 + nload - 1 of the wave's share
  // (A's into slot lsta, B's into lstb) dealt evenly between them.  The fences keep the order as written: without them the reads drift together and the MFMAs wait on LDS.
  auto slice = [&](int buf, const char* rsta, const char* rstb, int rkk, char* lsta, char* lstb, int l0, int nload) __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this slice's fragments, read during the previous one
    __builtin_amdgcn_sched_barrier(0);
    constexpr int SLACK = NM >= 6 ? 2 : 1;   // MFMAs left after the last read is issued
#pragma unroll
    for (int x = 0; x < NM; ++x) {
      const int i = x / TN, j = x % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int f = 0; f < NF; ++f)
        if (f * (NM - SLACK) / NF == x) read_frag(rsta, rstb, rkk, buf ^ 1, f);
#pragma unroll
      for (int l = 0; l < nload; ++l)
        if (l * NM / nload == x) load_ab(lsta, lstb, l0 + l);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (LAYOUT == GEMM_TN && __builtin_expect(do_rs, 0)) {   // rare (the first column of tiles, models with biases): kept out of the MFMA stream's straight path
      typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
      const bf16x2_t one2 = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const bf16x8 a8 = fa[buf][i];
        const bf16x2_t a01 = {a8[0], a8[1]}, a23 = {a8[2], a8[3]}, a45 = {a8[4], a8[5]}, a67 = {a8[6], a8[7]};
        rs[i] = __builtin_amdgcn_fdot2_f32_bf16(a01, one2, rs[i], false);
        rs[i] = __builtin_amdgcn_fdot2_f32_bf16(a23, one2, rs[i], false);
        rs[i] = __builtin_amdgcn_fdot2_f32_bf16(a45, one2, rs[i], false);
        rs[i] = __builtin_amdgcn_fdot2_f32_bf16(a67, one2, rs[i], false);
      }
    }
  };

  // Software pipeline over K steps of 64 (four k-slices).  At the top of step i the fragments of slice 0 are in
  // registers and tile i+1 is in flight or landed.  Slices 0..2 run, B's loads of tile i+2 going out behind the first
  // two; then the wave waits for its own loads of tile i+1 and for its last LDS reads, the barrier tells it that
  // every wave has done so (tile i+1 complete, slots of tile i no longer read); slice 3 runs while A's loads of tile
  // i+2 start into the freed A slot and slice 0 of tile i+1 is read.
  const int nsteps = (int)((kend - kbeg + DTL_BK - 1) / DTL_BK);
  load_tile(stage0);
  if (nsteps > 1) load_tile(stage1);
  if (nsteps > 1) __builtin_amdgcn_s_waitcnt(0x0f70 | (NL & 15) | ((NL >> 4) << 14));   // vmcnt(NL): tile 0 landed, tile 1 may be on its way
  else __builtin_amdgcn_s_waitcnt(0x0f70);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int f = 0; f < NF; ++f) read_frag(stage0, stage0 + ImA::BYTES, 0, 0, f);
  __builtin_amdgcn_sched_barrier(0);
  char *a_cur = stage0, *a_nxt = stage1;
  char *b_cur = stage0 + ImA::BYTES, *b_nxt = stage1 + ImA::BYTES, *b_free = slot3;
  for (int i = 0; i < nsteps; ++i) {
    // the last two steps have no tile to fetch: their loads zero-fill slots nobody reads again, and the last step's
    // fragment reads of the next slots are never used
    const bool more = i + 2 < nsteps;
    rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)p.B, 0, more ? p.b_records : 0u, 0x00020000);
    slice(0, a_cur, b_cur, 1, nullptr, b_free, LA, LB / 2);
    slice(1, a_cur, b_cur, 2, nullptr, b_free, LA + LB / 2, LB - LB / 2);
    slice(0, a_cur, b_cur, 3, nullptr, nullptr, 0, 0);
    // Tile i+1 has landed for this wave (loads complete in order: only B's of tile i+2, just issued, may be on
    // their way) and its LDS reads have returned; then every wave's.  A bare barrier: a fence over global memory
    // would wait for the loads that are meant to stay in flight.
    __builtin_amdgcn_s_waitcnt(0x0070 | LB);   // vmcnt(LB) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, more ? p.a_records : 0u, 0x00020000);
    slice(1, a_nxt, b_nxt, 0, a_cur, nullptr, 0, LA);
    char* t = a_cur; a_cur = a_nxt; a_nxt = t;
    t = b_cur; b_cur = b_nxt; b_nxt = b_free; b_free = t;
  }
  // The zero fills must have landed before the stages are reused below.  The last step's fragment reads
  // must have landed too: the compiler does not know the assembly reads are in flight, their destination
  // registers are dead here, and a late return would overwrite whatever the epilogue keeps there (an
  // address, for one).
  // The empty statements after the wait name those registers as inputs, which keeps them reserved up to
  // that point.
  __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
#pragma unroll
  for (int i = 0; i < TM; ++i) asm volatile("" ::"v"(fa[0][i]));
#pragma unroll
  for (int j = 0; j < TN; ++j) asm volatile("" ::"v"(fb[0][j]));
  __syncthreads();

  if (LAYOUT == GEMM_TN && do_rs) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const float v = rs[i] + __shfl_xor(rs[i], 32, 64);   // lanes l and l + 32 hold the two k-halves of row l
      const int64_t m = m0 + wm + i * 32 + lr;
      if (lk == 0 && m < p.M) {
        float* o = p.rowsum + m;
        if (ATOMIC) unsafeAtomicAdd(o, v);
        else *o = p.rowsum_accumulate ? *o + v : v;
      }
    }
  }

  // Float outputs with nothing fused: a lane holds one column of four consecutive rows per register group, so one
  // store instruction writes two rows of 32 consecutive floats, whole 128-byte lines, straight from the accumulators.
  // No staging through LDS and none of its registers: with them this instance of the kernel ran its K loop slower
  // (a 12288 x 4096 x 8192 weight gradient took 806 us against 673 us with a bfloat16 output).
  if (DIRECT) {
    float* cbase = reinterpret_cast<float*>(p.C);
    const bool add = p.beta != 0.f;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t n = n0 + wn + j * 32 + lr;
      if (n < p.N) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            const int64_t m = m0 + wm + i * 32 + (q >> 2) * 8 + lk * 4 + (q & 3);
            if (m < p.M) {
              float* c = cbase + m * p.ldc + n;
              *c = add ? acc[i][j][q] + p.beta * *c : acc[i][j][q];
            }
          }
      }
    }
    return;
  }
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
  // bf16 outputs whose epilogue is elementwise in the accumulator's own layout (bias, GeLU; no second operand
  // indexed by row): bias and activation are applied in registers in fp32, the results are rounded once, written
  // to LDS as the transpose (a lane holds four consecutive rows of one column: one 8-byte write), and read back
  // with transposing reads that hand each lane eight consecutive columns of one row for a 16-byte store.  A
  // quarter of the LDS instructions and half the LDS bytes of the float staging below, which costs 3.7 us per
  // 256x256 tile (measured), more than the stores themselves.
  if (TRANSPOSED) {
    constexpr int IC = TM >= 2 ? 2 : 1;                 // 32-row tiles per round
    constexpr int P = IC * 64 + 16;                     // bytes per image row (one column of C, IC*32 rows), padded
    constexpr int IMG = TN * 32 * P;
    static_assert((NW / 2) * IMG <= STAGE, "transposed staging must fit the stages");
    static_assert(TM % IC == 0, "whole rounds");
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    char* img = (wave < NW / 2 ? stage0 : stage1) + (wave % (NW / 2)) * IMG;
    // a wave's epilogue is bound by its instruction count (two waves share a SIMD and nothing else runs): every
    // address below is a per-lane base plus a compile-time offset, and what is uniform is decided outside the loops
    char* wbase = img + lr * P + lk * 8;                                   // + (j*32)*P + (ii*32 + g4*8)*2
    const int j16 = lane & 15, grp = lane >> 4;
    const uint32_t rbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)(img + (grp * 8 + (j16 >> 2)) * P + (4 * (j16 & 3)) * 2);
    float bcol[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t n = n0 + wn + j * 32 + lr;
      bcol[j] = (p.bias && n < p.N) ? to_float<bf16>(p.bias[n]) : 0.f;
    }
    const bool gelu = p.act == ACT_GELU;                // GeLU has two outputs: the activation, then gelu' for the backward pass
    const bool has_bias = p.bias != nullptr;
    bool ncol_ok[TN];
#pragma unroll
    for (int nb = 0; nb < TN; ++nb) ncol_ok[nb] = n0 + wn + nb * 32 + grp * 8 < n_ext;
    auto put = [&](int ii, int j, int g4, float v0, float v1, float v2, float v3) __attribute__((always_inline)) {
      const bf16x2_t h0 = __builtin_convertvector(floatx2_t{v0, v1}, bf16x2_t);
      const bf16x2_t h1 = __builtin_convertvector(floatx2_t{v2, v3}, bf16x2_t);
      // column j*32 + lr of the wave tile, rows ii*32 + g4*8 + lk*4 .. +3
      *reinterpret_cast<uint2*>(wbase + (j * 32) * P + (ii * 32 + g4 * 8) * 2) =
          make_uint2(__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1));
    };
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if (pass == 1 && !gelu) break;
      bf16* outp = pass == 0 ? reinterpret_cast<bf16*>(p.C) : p.aux;
      const int64_t ldo = pass == 0 ? p.ldc : p.ldaux;
#pragma unroll
      for (int r = 0; r < TM / IC; ++r) {
        if (gelu) {
#pragma unroll
          for (int ii = 0; ii < IC; ++ii)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
              for (int g4 = 0; g4 < 4; ++g4) {
                float v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                  float gv, dg;
                  gelu_tanh_both_fast(acc[r * IC + ii][j][g4 * 4 + k] + bcol[j], &gv, &dg);
                  v[k] = pass == 0 ? gv : dg;
                }
                put(ii, j, g4, v[0], v[1], v[2], v[3]);
              }
        } else if (has_bias) {
#pragma unroll
          for (int ii = 0; ii < IC; ++ii)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
              for (int g4 = 0; g4 < 4; ++g4) {
                const floatx16& t = acc[r * IC + ii][j];
                put(ii, j, g4, t[g4 * 4] + bcol[j], t[g4 * 4 + 1] + bcol[j], t[g4 * 4 + 2] + bcol[j], t[g4 * 4 + 3] + bcol[j]);
              }
        } else {
#pragma unroll
          for (int ii = 0; ii < IC; ++ii)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
              for (int g4 = 0; g4 < 4; ++g4) {
                const floatx16& t = acc[r * IC + ii][j];
                put(ii, j, g4, t[g4 * 4], t[g4 * 4 + 1], t[g4 * 4 + 2], t[g4 * 4 + 3]);
              }
        }
        wave_lds_sync();
        // 16 lanes: lane j16 addresses image row (j16 >> 2) of a 4 x 16 block at element 4 (j16 & 3) and receives element
        // j16 of the four rows, i.e. C[row mb*16 + j16][four consecutive columns]; two reads give eight columns.
        // All reads of a 16-row block are issued before the one wait.
        // INVARIANT (the compiler does not see these reads complete): every register pair written by issue() is
        // named as an in/out operand of the empty statement after the matching s_waitcnt below, which both keeps the
        // pair reserved until the data has landed and orders every use behind the wait; issue(mb + 1) runs only when
        // block mb + 1 exists, so no read is left without such a statement.
        const int64_t mrow = m0 + wm + (r * IC * 32) + j16;
        bf16* orow = outp + mrow * ldo + (n0 + wn + grp * 8);
        constexpr int NMB = IC * 2;
        intx2 lo[2][TN], hi[2][TN];
        auto issue = [&](int mb, int buf) __attribute__((always_inline)) {
#pragma unroll
          for (int nb = 0; nb < TN; ++nb) {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo[buf][nb]) : "v"(rbase), "n"(nb * 32 * P + mb * 32));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi[buf][nb]) : "v"(rbase), "n"(nb * 32 * P + mb * 32 + 4 * P));
          }
        };
        issue(0, 0);
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb) {
          // the reads of the next 16-row block are in flight while this one is stored
          if (mb + 1 < NMB) {
            issue(mb + 1, (mb + 1) & 1);
            asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(2 * TN) : "memory");
          } else {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          }
#pragma unroll
          for (int nb = 0; nb < TN; ++nb) asm volatile("" : "+v"(lo[mb & 1][nb]), "+v"(hi[mb & 1][nb]));   // landed: only now may the values be used
          if (mrow + mb * 16 < p.M) {
#pragma unroll
            for (int nb = 0; nb < TN; ++nb)
              if (ncol_ok[nb])
                *reinterpret_cast<uint4*>(orow + nb * 32) = make_uint4(lo[mb & 1][nb][0], lo[mb & 1][nb][1], hi[mb & 1][nb][0], hi[mb & 1][nb][1]);
          }
          orow += 16 * ldo;
        }
        wave_lds_sync();
      }
    }
    return;
  }
  // Everything else goes through a per-wave float staging area (see gemm_mfma.hip).  The bias depends on the column only
  // and is read once.
  float* stage = reinterpret_cast<float*>(stage0) + wave * (16 * SW);
  uint4 bias_raw[ITS];
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int64_t n = n0 + wn + ((lane + it * 64) % GROUPS) * 8;
    bias_raw[it] = make_uint4(0, 0, 0, 0);
    if (p.bias && n < n_ext) bias_raw[it] = *reinterpret_cast<const uint4*>(p.bias + n);
  }
  if (TM > TMC) prefetch(1);
#pragma unroll
  for (int ic = 0; ic < TM; ic += TMC) {
    const int c = ic / TMC;
#pragma unroll
    for (int ii = 0; ii < TMC; ++ii) {
      const int i = ic + ii;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 8; ++q)
            stage[((q >> 2) * 8 + lk * 4 + (q & 3)) * SW + j * 32 + lr] = acc[i][j][half * 8 + q];
        wave_lds_sync();
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
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
              t.raw = bias_raw[it]; t.unpack(f);
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
              t.raw = pre[c][ii][half][it]; t.unpack(f);
#pragma unroll
              for (int k = 0; k < 8; ++k) v[k] *= f[k];
            }
            if (p.residual) {   // never together with GeLU' (the launcher refuses that pair): pre holds the residual
              t.raw = pre[c][ii][half][it]; t.unpack(f);
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
}

// dst[i] += src[i] over up to eight segments in one launch: the second pass of a K split whose second half went to
// a buffer of its own.  Segments whose two pointers are 16-byte aligned go four floats at a time (4096 per block).
struct AddSeg { float* dst; const float* src; int64_t n; int vec; };
struct AddGroup { AddSeg s[2 * DTL_MAX_PROBLEMS]; int start[2 * DTL_MAX_PROBLEMS + 1]; int n; };
__global__ void __launch_bounds__(256) splitk_add_kernel(AddGroup g) {
  int si = 0;
#pragma unroll
  for (int i = 1; i < 2 * DTL_MAX_PROBLEMS; ++i)
    if (i < g.n && (int)blockIdx.x >= g.start[i]) si = i;
  const AddSeg& sg = g.s[si];
  const int64_t base = (int64_t)((int)blockIdx.x - g.start[si]) * 4096;
  if (sg.vec) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t i = base + k * 1024 + threadIdx.x * 4;
      if (i + 3 < sg.n) {
        float4 d = *reinterpret_cast<const float4*>(sg.dst + i);
        const float4 v = nt_load4(sg.src, i / 4);
        d.x += v.x; d.y += v.y; d.z += v.z; d.w += v.w;
        *reinterpret_cast<float4*>(sg.dst + i) = d;
      } else {
        for (int64_t j = i; j < sg.n; ++j) sg.dst[j] += sg.src[j];
      }
    }
  } else {
    for (int64_t i = base + threadIdx.x; i < min(sg.n, base + 4096); i += 256) sg.dst[i] += sg.src[i];
  }
}

template <int WM, int WN, int TM, int TN, int EPI>
static void launch_dtl(hipStream_t s, int layout, dim3 grid, const DtlGroupParams& gp, hipEvent_t e0, hipEvent_t e1) {
  dim3 block(64 * WM * WN);
  poplar_gemm_kernel_launches += 1;
  // with events the launch itself carries them: they receive the kernel's own start and end
  switch (layout) {
    case GEMM_NT: hipExtLaunchKernelGGL((gemm_dtl_kernel<GEMM_NT, WM, WN, TM, TN, EPI>), grid, block, 0, s, e0, e1, 0, gp); break;
    case GEMM_NN: hipExtLaunchKernelGGL((gemm_dtl_kernel<GEMM_NN, WM, WN, TM, TN, EPI>), grid, block, 0, s, e0, e1, 0, gp); break;
    default: hipExtLaunchKernelGGL((gemm_dtl_kernel<GEMM_TN, WM, WN, TM, TN, EPI>), grid, block, 0, s, e0, e1, 0, gp); break;
  }
}

// Checks one problem against the kernel's preconditions and fills its parameters (not the tiling).
static int dtl_prepare(const GemmArgs& a, DtlGemmParams& p) {
  if (a.layout < GEMM_NT || a.layout > GEMM_TN) return POPLAR_ERR_UNIMPLEMENTED;
  // a K tail is fine when every operand reads zeros there: k-strided operands run out of range, a
  // k-contiguous A only if the caller vouches for zero padding up to the next multiple of 64
  const bool a_tail_ok = a.layout == GEMM_NN && a.a_k_pad_zero && a.lda >= round_up(a.K, DTL_BK);
  if (a.layout != GEMM_TN && a.K % DTL_BK && !a_tail_ok) return POPLAR_ERR_UNIMPLEMENTED;
  if (a.K < DTL_BK) return POPLAR_ERR_UNIMPLEMENTED;
  if (a.act == ACT_GELU_BWD && a.residual) return POPLAR_ERR_UNIMPLEMENTED;   // the epilogue prefetches one extra operand
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
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B; p.C = a.C;
  p.bias = (const bf16*)a.bias; p.residual = (const bf16*)a.residual; p.aux = (bf16*)a.aux;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc; p.ldaux = a.ldaux;
  p.a_records = (uint32_t)a_bytes; p.b_records = (uint32_t)b_bytes;
  p.c_float = a.c_float; p.act = a.act; p.beta = a.beta;
  if (a.a_rowsum && a.layout != GEMM_TN) return POPLAR_ERR_UNIMPLEMENTED;
  p.rowsum = a.a_rowsum; p.rowsum_accumulate = a.a_rowsum_accumulate;
  return POPLAR_OK;
}

// true when the direct-to-LDS kernel takes these problems as one launch (n > 1) or one each (n == 1)
bool gemm_bf16_dtl_accepts(const GemmArgs* a, int n) {
  if (n < 1 || n > DTL_MAX_PROBLEMS) return false;
  DtlGemmParams p;
  for (int i = 0; i < n; ++i)
    if (a[i].layout != a[0].layout || a[i].K != a[0].K || dtl_prepare(a[i], p) != POPLAR_OK) return false;
  return true;
}

// Tile shape and K split by a small cost model, in units of one K step of a 256x256 tile on its CU.
// 256x256 and 256x192 tiles run one block per CU, 128x128 tiles two per CU (each step a quarter of the
// work at ~80% of the efficiency), 64x64 tiles four per CU (latency-bound steps: they only pay when the
// larger tiles would leave most CUs idle, i.e. few rows and a narrow output); the epilogue costs a few
// K steps; the launch takes ceil(blocks / slots) rounds.  The 256x192 tile exists for the block count: widths such as 768 or
// 2304 give whole rounds with it where 256-wide tiles leave a quarter of the CUs idle.  A split adds a
// zero fill and float atomics, which the chip retires at a fixed rate (about 250 G/s measured)
// whatever the tile shape: that term is what keeps the split count low.
struct TileCfg { int bm, bn; double slots, step, epi, epi_atomic; };
static const TileCfg cfgs[4] = {{256, 256, 256.0, 1.0, 4.0, 6.0}, {256, 192, 256.0, 0.84, 3.0, 5.0}, {128, 128, 512.0, 0.6, 1.2, 2.0},
                                {64, 64, 1024.0, 0.36, 0.5, 0.8}};

// plain: every problem writes a float matrix with no bias / activation / residual, so K may be split
// *halves_out (may be null): the plan is a cut of K in two whose second half goes to the problems' k_partial buffers
// and is added afterwards: no zero fill and no atomics, one pass over the outputs instead (14.6 us for the 7.1 M
// elements of a GPT-2-small layer's weight gradients; the coefficient is set so that the cut begins where it was
// measured to pay on that layer: above 8192 tokens).  Offered when every problem brings the buffer.
static double dtl_plan(const GemmArgs* a, int n, bool plain, int* pick_out, int* splits_out, bool* halves_out = nullptr) {
  const int64_t ksteps = cdiv(a[0].K, DTL_BK);
  bool can_halve = halves_out != nullptr && plain && a[0].layout == GEMM_TN && n <= DTL_MAX_PROBLEMS && ksteps >= 16;
  // (dense outputs only: the second pass runs over M * ldc floats of C and of the buffer alike)
  for (int i = 0; i < n; ++i) can_halve = can_halve && a[i].k_partial != nullptr && ((uintptr_t)a[i].k_partial & 15) == 0 && a[i].ldc == a[i].N;
  bool halves = false;
  double mn = 0.0;
  for (int i = 0; i < n; ++i) mn += (double)a[i].M * (double)a[i].N;
  int pick = 0, splits = 1;
  double best = 1e300;
  for (int cfg = 0; cfg < 4; ++cfg) {
    const TileCfg& tc = cfgs[cfg];
    int64_t t = 0;
    for (int i = 0; i < n; ++i) t += cdiv(a[i].M, tc.bm) * cdiv(a[i].N, tc.bn);
    static const int cand[] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16};
    for (int sp : cand) {
      if (sp > 1 && (!plain || ksteps / sp < 8 || a[0].no_atomics)) break;
      const double rounds = ceil((double)(t * sp) / tc.slots);
      // two 128x128 blocks that really share a CU slow each other down a little more
      // (measured; likewise the 64x64 blocks as a CU fills up: four to a CU they cost almost twice the lone block's
      // step, more again with two strided operands)
      const double step3 = t * sp > 768 ? (a[0].layout == GEMM_TN ? 0.75 : 0.66) : t * sp > 256 ? 0.50 : tc.step;
      const double step = cfg == 2 ? (t * sp > 256 ? 0.68 : tc.step) : cfg == 3 ? step3 : tc.step;
      const double cost = rounds * ((double)cdiv(ksteps, sp) * step + (sp > 1 ? tc.epi_atomic : tc.epi)) +
                          (sp > 1 ? 3.0 * n + 2.7e-6 * (double)sp * mn : 0.0);   // one zero fill per problem, atomics
      if (cost < best) { best = cost; pick = cfg; splits = sp; halves = false; }
    }
    if (can_halve && cfg < 3) {
      const double rounds = ceil((double)(2 * t) / tc.slots);
      const double step = cfg == 2 ? (2 * t > 256 ? 0.68 : tc.step) : tc.step;
      const double cost = rounds * ((double)cdiv(ksteps, 2) * step + tc.epi) + 2.0 + 2.6e-6 * mn;
      if (cost < best) { best = cost; pick = cfg; splits = 1; halves = true; }
    }
  }
  *pick_out = pick; *splits_out = splits;
  if (halves_out) *halves_out = halves;
  return best;
}

static int dtl_group_impl(hipStream_t s, const GemmArgs* a, int n, bool may_cut, int forced_pick = -1);

// Up to DTL_MAX_GROUP problems of one layout and one K in a single launch (a plain GEMM is a group of one).
// Returns POPLAR_ERR_UNIMPLEMENTED, with nothing launched, when a problem is outside the kernel's
// preconditions or the group is not uniform; the caller then runs the problems one by one.
int gemm_bf16_dtl_group(hipStream_t s, const GemmArgs* a, int n) { return dtl_group_impl(s, a, n, true); }

// forced_pick >= 0: the halves of a group whose K was cut in two (tile shape given, no further split or cut; the
// second halves may be shorter than the first by a part of a K step)
static int dtl_group_impl(hipStream_t s, const GemmArgs* a, int n, bool may_cut, int forced_pick) {
  if (n < 1 || n > (forced_pick >= 0 ? DTL_MAX_GROUP : DTL_MAX_PROBLEMS)) return POPLAR_ERR_UNIMPLEMENTED;
  DtlGroupParams gp;
  bool plain = true;
  for (int i = 0; i < n; ++i) {
    if (a[i].layout != a[0].layout || (forced_pick < 0 && a[i].K != a[0].K)) return POPLAR_ERR_UNIMPLEMENTED;
    const int st = dtl_prepare(a[i], gp.g[i]);
    if (st != POPLAR_OK) return st;
    plain = plain && a[i].c_float && !a[i].bias && !a[i].residual && a[i].act == ACT_NONE;
  }
  gp.n = n;
  int64_t K = a[0].K;
  for (int i = 1; i < n; ++i) K = std::max(K, a[i].K);
  int pick = 0, splits = 1;
  bool halves = false;
  const double best = forced_pick >= 0 ? 0.0 : dtl_plan(a, n, plain, &pick, &splits, &halves);
  if (forced_pick >= 0) { pick = forced_pick; may_cut = false; }

  // K cut in two: the first halves write (or add to) the outputs as asked, the second halves their sums to the
  // problems' own buffers, all 2n as one launch; one more pass adds the buffers to the outputs.  The events go
  // to the first and the last of the two launches.
  if (halves) {
    GemmArgs b[DTL_MAX_GROUP];
    AddGroup ag;
    ag.n = 0;
    int blocks = 0;
    const int64_t kh = round_up(K / 2, DTL_BK);
    for (int i = 0; i < n; ++i) {
      GemmArgs& lo = b[i];
      GemmArgs& hi = b[n + i];
      lo = a[i]; lo.K = kh; lo.k_partial = nullptr; lo.ev_start = nullptr; lo.ev_stop = nullptr;
      hi = lo; hi.K = K - kh;
      hi.A = (const bf16*)a[i].A + kh * a[i].lda;           // TN: both operands are stored [K, .]
      hi.B = (const bf16*)a[i].B + kh * a[i].ldb;
      hi.C = a[i].k_partial; hi.beta = 0.f;
      const int64_t cn = a[i].M * a[i].ldc;
      ag.s[ag.n] = AddSeg{(float*)a[i].C, a[i].k_partial, cn, 1};
      ag.start[ag.n++] = blocks;
      blocks += (int)cdiv(cn, 4096);
      if (a[i].a_rowsum) {
        hi.a_rowsum = a[i].k_partial + cn; hi.a_rowsum_accumulate = 0;
        ag.s[ag.n] = AddSeg{a[i].a_rowsum, hi.a_rowsum, a[i].M, 0};
        ag.start[ag.n++] = blocks;
        blocks += (int)cdiv(a[i].M, 4096);
      }
    }
    for (int i = 0; i < ag.n; ++i)
      if (((uintptr_t)ag.s[i].dst | (uintptr_t)ag.s[i].src) & 15) ag.s[i].vec = 0;
    for (int i = ag.n; i <= 2 * DTL_MAX_PROBLEMS; ++i) ag.start[i] = blocks;
    b[0].ev_start = a[0].ev_start;
    POPLAR_TRY(dtl_group_impl(s, b, 2 * n, false, pick));
    hipExtLaunchKernelGGL(splitk_add_kernel, dim3(blocks), dim3(256), 0, s, nullptr, a[0].ev_stop, 0, ag);
    POPLAR_LAUNCH_CHECK();
    return POPLAR_OK;
  }

  // Weight gradients on 256x256 tiles whose last round would be mostly empty (the head: 591 tiles on 256 CUs; the four
  // of a Llama-7B layer: 3088) are cut along M of the last problem: the tile rows that fill whole rounds run as they
  // are, the rest as a problem of its own, for which the model finds a K split that spreads it over the chip.
  if (may_cut && n <= DTL_MAX_PROBLEMS && plain && a[0].layout == GEMM_TN && pick == 0 && splits == 1 && !halves) {
    int64_t tiles = 0;
    for (int i = 0; i < n; ++i) tiles += cdiv(a[i].M, 256) * cdiv(a[i].N, 256);
    const GemmArgs& last = a[n - 1];
    const int64_t tm = cdiv(last.M, 256), tn = cdiv(last.N, 256);
    const int64_t rest = tiles % 256;                      // tiles of the last, partial round
    if (tiles > 256 && rest != 0 && rest % tn == 0 && rest / tn < tm) {
      const int64_t keep_rows = tm - rest / tn;
      GemmArgs h[DTL_MAX_PROBLEMS];
      for (int i = 0; i < n; ++i) h[i] = a[i];
      GemmArgs t = last;
      h[n - 1].M = keep_rows * 256;
      t.M = last.M - h[n - 1].M;
      t.A = (const bf16*)last.A + h[n - 1].M;              // TN: A is stored [K, M]
      t.C = (float*)last.C + h[n - 1].M * last.ldc;
      if (last.a_rowsum) t.a_rowsum = last.a_rowsum + h[n - 1].M;
      if (last.k_partial) t.k_partial = nullptr;
      h[0].ev_stop = nullptr; t.ev_start = nullptr; t.ev_stop = a[0].ev_stop;
      int pk, sp;
      const double cut = dtl_plan(h, n, true, &pk, &sp) + dtl_plan(&t, 1, true, &pk, &sp);
      DtlGemmParams probe;
      if (cut < 0.95 * best && dtl_prepare(t, probe) == POPLAR_OK) {
        POPLAR_TRY(dtl_group_impl(s, h, n, false));
        return dtl_group_impl(s, &t, 1, false);
      }
    }
  }
  // A forward or input-gradient product (one problem, 256x256 tiles, rows = tokens) whose last round would be partly
  // empty is cut along N: the tile columns that fill whole rounds run as they are, the remaining columns as a problem
  // of their own, on whatever tile shape fills the chip best for them (8192 x 11008: 1376 tiles = 5.4 rounds become
  // five whole rounds and 384 blocks of 128 x 128, two to a CU).  Taken for products without a second matrix operand
  // (residual, GeLU factor): the bias is indexed by column and moves with the cut.
  if (may_cut && n == 1 && a[0].layout != GEMM_TN && pick == 0 && splits == 1 && !a[0].residual && !a[0].aux) {
    const GemmArgs& g = a[0];
    const int64_t tm = cdiv(g.M, 256), tn = cdiv(g.N, 256), tiles = tm * tn, rest = tiles % 256;
    if (tiles > 256 && rest != 0 && rest % tm == 0 && rest / tm < tn) {
      const int64_t keep = (tn - rest / tm) * 256;         // columns of the main part
      const int64_t es_c = g.c_float ? 4 : 2;
      GemmArgs h = g, t = g;
      h.N = keep;
      t.N = g.N - keep;
      t.B = g.layout == GEMM_NT ? (const void*)((const bf16*)g.B + keep * g.ldb) : (const void*)((const bf16*)g.B + keep);
      t.C = (char*)g.C + keep * es_c;
      if (g.bias) t.bias = (const bf16*)g.bias + keep;
      h.ev_stop = nullptr; t.ev_start = nullptr;
      int pk, sp;
      const double cut = dtl_plan(&h, 1, plain, &pk, &sp) + dtl_plan(&t, 1, plain, &pk, &sp);
      DtlGemmParams probe;
      if (cut < 0.96 * best && dtl_prepare(h, probe) == POPLAR_OK && dtl_prepare(t, probe) == POPLAR_OK) {
        POPLAR_TRY(dtl_group_impl(s, &h, 1, false));
        return dtl_group_impl(s, &t, 1, false);
      }
    }
  }
  const int BM = cfgs[pick].bm, BN = cfgs[pick].bn;
  const int k_per_split = (int)round_up(cdiv(K, splits), DTL_BK);
  splits = (int)cdiv(K, k_per_split);
  const bool atomic = splits > 1;
  int64_t tiles = 0;
  for (int i = 0; i < n; ++i) {
    DtlGemmParams& p = gp.g[i];
    p.tiles_m = (int)cdiv(a[i].M, BM);
    p.tiles_n = (int)cdiv(a[i].N, BN);
    p.k_per_split = k_per_split;
    gp.start[i] = (int)tiles;
    tiles += (int64_t)p.tiles_m * p.tiles_n;
    if (tiles > 0x7fffffff) return POPLAR_ERR_UNIMPLEMENTED;
  }
  for (int i = n; i <= DTL_MAX_GROUP; ++i) gp.start[i] = (int)tiles;
  for (int i = n; i < DTL_MAX_GROUP; ++i) gp.g[i] = gp.g[0];
  if (atomic) {
    for (int i = 0; i < n; ++i)
      if (a[i].a_rowsum && !a[i].a_rowsum_accumulate) POPLAR_TRY(fill_zero(s, a[i].a_rowsum, a[i].M * 4));
    for (int i = 0; i < n; ++i) {
      if (a[i].beta != 0.f) continue;
      if (a[i].ldc != a[i].N) {
        POPLAR_TRY(fill_zero_2d(s, a[i].C, a[i].M, a[i].N, a[i].ldc));
      } else {
        POPLAR_TRY(fill_zero(s, a[i].C, a[i].M * a[i].N * 4));
      }
    }
  }
  dim3 grid((unsigned)tiles, (unsigned)splits);
  // which epilogue: split K -> atomics; bf16 outputs with nothing fused that is indexed by row -> transposed staging
  bool transposed = !atomic;
  for (int i = 0; i < n; ++i) transposed = transposed && !a[i].c_float && !a[i].residual && a[i].act != ACT_GELU_BWD;
  const int epi = atomic ? 1 : transposed ? 2 : plain ? 3 : 0;
#define DTL_LAUNCH(WM, WN, TM, TN)                                                                        \
  do {                                                                                                    \
    if (epi == 1) launch_dtl<WM, WN, TM, TN, 1>(s, a[0].layout, grid, gp, a[0].ev_start, a[0].ev_stop);      \
    else if (epi == 2) launch_dtl<WM, WN, TM, TN, 2>(s, a[0].layout, grid, gp, a[0].ev_start, a[0].ev_stop); \
    else if (epi == 3) launch_dtl<WM, WN, TM, TN, 3>(s, a[0].layout, grid, gp, a[0].ev_start, a[0].ev_stop); \
    else launch_dtl<WM, WN, TM, TN, 0>(s, a[0].layout, grid, gp, a[0].ev_start, a[0].ev_stop);               \
  } while (0)
  if (pick == 0) DTL_LAUNCH(2, 4, 4, 2);
  else if (pick == 1) DTL_LAUNCH(4, 2, 2, 3);
  else if (pick == 2) DTL_LAUNCH(2, 2, 2, 2);
  else DTL_LAUNCH(2, 2, 1, 1);
#undef DTL_LAUNCH
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int gemm_bf16_dtl(hipStream_t s, const GemmArgs& a) { return gemm_bf16_dtl_group(s, &a, 1); }
