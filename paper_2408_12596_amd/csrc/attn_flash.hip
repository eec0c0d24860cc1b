// Flash-style causal attention on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16): forward, and backward as two kernels (dK/dV per
// key tile, dQ per query tile) so that no result depends on atomics.
//
// Data: the fused projection output qkv [B*S, 3H] (q | k | v thirds, head h in
// columns h*D..(h+1)*D of each), o and dout [B*S, H], lse and delta float
// [B, nh, S].  D is 64 or 128.  lse is kept in the base-2 domain:
// lse2 = log2(sum_j exp(s_ij / sqrt(D))).
//
// MFMA conventions used below (32x32 tile, K = 16 per instruction):
//   A fragment: lane holds row  (lane % 32), k-slots (lane / 32) * 8 + 0..7
//   B fragment: lane holds col  (lane % 32), the same k-slots
//   C tile    : lane holds col  (lane % 32); register i is row (i/4)*8 + (lane/32)*4 + i%4
// A probability tile therefore leaves the softmax already in B-fragment form
// if k-slot e of lane half g inside a 16-row chunk is read as row
// (e/4)*8 + g*4 + e%4: the probabilities never touch LDS.
//
// Tiles (64 rows of K, V, Q or dO, D values each) go from global memory to LDS
// with direct loads (buffer_load ... lds, 16 bytes per lane, lane L of a
// wavefront landing at base + 16 L), two stages deep, one barrier per tile.
// The LDS image keeps the rows as they are, 16-byte chunks XOR-swizzled with
// the row, and serves both operand forms:
//   * rows as the M index (K for S^T = K Q^T, V for dP^T, Q and dO in dK/dV):
//     one 16-byte read per fragment;
//   * rows as the reduction index (V^T for O^T += V^T P^T, K^T for dQ, Q^T and
//     dO^T for dK/dV): two transposing reads (ds_read_b64_tr_b16) per fragment,
//     taken at rows 16j + 4g + {0..3} and 16j + 8 + 4g + {0..3}, which is exactly
//     the k-slot order of the probability fragments.
//
// Forward and dQ work on S^T = K Q^T (lane = query), which keeps the running
// max / sum / rescale of a query inside one lane (plus one exchange between the
// two lane halves).  dK/dV works on S = Q K^T (lane = key).
#include <hip/hip_ext.h>
#include <type_traits>
#include "device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

#define LOG2E 1.4426950408889634f
// LDS stages of the two backward kernels: three at either head dim (48 or 96-102 KB of the CU's 160)
#define FA_BWD_STAGES 3
#define FA_OOB 0xfffffff0u

__device__ inline bf16x8 as_frag(uint4 v) { return *reinterpret_cast<bf16x8*>(&v); }

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

// one 16-byte-per-lane load of a wavefront straight into the KiB of LDS at dst (lane L lands at dst + 16 L);
// offsets at or past the resource's size deliver zeros
__device__ inline void fa_load_kib(__amdgpu_buffer_rsrc_t rsrc, char* dst, uint32_t lane_byte_offset) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)dst, 16, lane_byte_offset, 0, 0, 0);
}

// ---- LDS image of 64 rows x D values ----------------------------------------------------------
// 16-byte chunk c of row r lies at chunk position c ^ fa_swz<D>(r) of the row.  The LDS serves 64 banks of
// 4 bytes per cycle (counters: with a swizzle built for 32 banks half of the LDS cycles were bank conflicts), so a
// 16-byte read is conflict-free when 16 consecutive rows land on the 16 chunk slots of a 256-byte window, and a
// transposing read (four rows x 64 bytes per 32 lanes) when rows R .. R+3 land on its four 64-byte slots.
//   D = 64 (128-byte rows: the row's parity is address bit 7): position bit 2 <- row bit 1, bits 1, 0 <- row bits 2, 3
//   D = 128 (256-byte rows): position bits 3, 2 <- row bits 1, 0; bits 1, 0 <- row bits 3, 2
template <int D>
__device__ inline int fa_swz(int row) {
  if (D == 64) return (((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1);
  return ((row & 3) << 2) | ((row >> 2) & 3);
}

template <int D>
struct Rows64 {
  static constexpr int ROWB = D * 2;            // 128 or 256 bytes
  static constexpr int CPR = D / 8;             // 16-byte chunks per row
  static constexpr int RPL = 1024 / ROWB;       // rows per wave load
  static constexpr int BYTES = 64 * ROWB;
  static constexpr int LOADS = BYTES / 1024;    // wave loads per tile: 8 or 16
  static constexpr int PER_WAVE = LOADS / 4;    // four wavefronts share a tile

  // byte offset, relative to row 0 of the tile, of the 16 bytes that belong at LDS position idx*1024 + lane*16
  __device__ static uint32_t lane_offset(int idx, int lane, int64_t ld) {
    const int row = idx * RPL + lane / CPR;
    const int c = (lane % CPR) ^ fa_swz<D>(row);
    return (uint32_t)(((int64_t)row * ld + c * 8) * 2);
  }
  // A fragment, rows as M index: row `row` of the tile, k-slice s (16 columns), lane half g
  __device__ static bf16x8 frag(const char* lds, int row, int s, int g) {
    return *reinterpret_cast<const bf16x8*>(lds + row * ROWB + (((2 * s + g) ^ fa_swz<D>(row)) << 4));
  }
  // per-lane bases of the transposed fragments of column tile ct (32 columns): first read (rows 0-7 of a
  // 16-row chunk) in .x, second read (rows 8-15) in .y
  __device__ static int2 tr_base(int ct, int lane) {
    const int l16 = lane & 15, gi = (lane >> 4) & 1, g = lane >> 5;
    const int row = 4 * g + (l16 >> 2);                       // row inside the 16-row chunk (first read)
    const int chunk = ct * 4 + gi * 2 + ((l16 & 3) >> 1);     // logical 16-byte chunk of the lane's 4 values
    return make_int2(row * ROWB + ((chunk ^ fa_swz<D>(row)) << 4) + (l16 & 1) * 8,
                     (row + 8) * ROWB + ((chunk ^ fa_swz<D>(row + 8)) << 4) + (l16 & 1) * 8);
  }
  // A fragment, rows as reduction index: 16-row chunk j, k-slots in probability order.
  // Written as assembly: the compiler would make the builtin form wait for every global -> LDS load in
  // flight (it cannot tell the stage being filled from the one being read).  It does not see these reads
  // complete either: the caller waits with fa_wait_lds() before it uses the fragment.
  // The chunk index (0 .. 3, a constant wherever this is called) goes into the instruction's offset field: a chunk
  // is 16 rows further on, which leaves the swizzle of a row unchanged.
  // INVARIANT for every caller (the compiler cannot check it): (1) a fragment read here is used only after a
  // fa_wait_lds() that follows the read in program order; (2) every fragment that is read IS used after that wait,
  // by an MFMA: a read whose result is dead would leave its destination registers free for the compiler to reuse while
  // the data is still on its way, and the late return would overwrite whatever was put there (this happened once in
  // the GEMM kernel, as a memory fault).  The three kernels below keep to it by prefetching the next group of
  // fragments only under the same condition under which that group's MFMAs run (c + 1 < 4 / PF; u == 0).
  template <int J>
  __device__ static bf16x8 frag_tr_at(uint32_t a0, uint32_t a1) {
    intx2 lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a0), "n"(J * 16 * ROWB));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a1), "n"(J * 16 * ROWB));
    intx4 f = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, f);
  }
  __device__ static bf16x8 frag_tr(const char* lds, int2 base, int j) {
    const uint32_t a0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)(lds + base.x);
    const uint32_t a1 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)(lds + base.y);
    switch (j) {
      case 0: return frag_tr_at<0>(a0, a1);
      case 1: return frag_tr_at<1>(a0, a1);
      case 2: return frag_tr_at<2>(a0, a1);
      default: return frag_tr_at<3>(a0, a1);
    }
  }
};

// component c (a constant after unrolling) of a float4
__device__ inline float f4_at(const float4& v, int c) { return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w; }

// at most N vector-memory operations of this wave still in flight (they complete in order)
template <int N>
__device__ inline void fa_wait_vm() {
  static_assert(N >= 0 && N < 64, "the counter has six bits");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}
// The current tile has landed for this wave: `later` tiles (0 .. 2) were requested after it, each with PER_TILE loads
template <int PER_TILE>
__device__ inline void fa_wait_tile(int later) {
  if (later >= 2) fa_wait_vm<2 * PER_TILE>();
  else if (later == 1) fa_wait_vm<PER_TILE>();
  else fa_wait_vm<0>();
}

// all LDS reads issued so far have returned; nothing moves across
__device__ inline void fa_wait_lds() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
  __builtin_amdgcn_sched_barrier(0);
}

// Four floats from LDS, written as assembly for the same reason as the transposing reads: the statistics tile is
// filled by direct loads, and the compiler would wait for every such load in flight (the next tile's) before a read
// of it that it can see.  Same invariant: used only after a later fa_wait_lds(), and always used.
typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ inline floatx4 lds_read_f4(const float* p) {
  floatx4 v;
  const uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(a));
  return v;
}

// Two chains of MFMAs over the D/16 k-slices of two LDS tiles (rows `row` of each, as A operands) against two sets of
// B fragments held in registers: acc0 += A0 B0^T, acc1 += A1 B1^T.  The A fragments are requested AHEAD MFMAs ahead of
// their use (three is where the gain ends; one costs 15 %) and the order is pinned: left to itself the compiler issues each read right before its MFMA (it keeps the
// register count down), and every MFMA then waits out an LDS round trip.
template <int D, int AHEAD = 3>
__device__ inline void mfma_two_chains(floatx16& acc0, floatx16& acc1, const char* lds0, const char* lds1, int row, int g,
                                       const bf16x8* b0, const bf16x8* b1) {
  typedef Rows64<D> Img;
  constexpr int N = D / 8;
  auto frag = [&](int n) { return (n & 1) ? Img::frag(lds1, row, n >> 1, g) : Img::frag(lds0, row, n >> 1, g); };
  bf16x8 fa[AHEAD + 1];
#pragma unroll
  for (int n = 0; n < AHEAD; ++n) fa[n] = frag(n);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int n = 0; n < N; ++n) {
    if (n + AHEAD < N) fa[(n + AHEAD) % (AHEAD + 1)] = frag(n + AHEAD);
    if (n & 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[n % (AHEAD + 1)], b1[n >> 1], acc1, 0, 0, 0);
    else acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[n % (AHEAD + 1)], b0[n >> 1], acc0, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

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

// bytes of a [rows, ld] bf16 matrix from `row0` to its end, clamped to the 32-bit range of a buffer resource
__device__ inline uint32_t records_from(int64_t rows_total, int64_t row0, int64_t ld, int64_t last_cols) {
  const int64_t bytes = ((rows_total - row0 - 1) * ld + last_cols) * 2;
  return bytes < (int64_t)FA_OOB ? (uint32_t)bytes : FA_OOB;
}

// Block id -> (sequence and head, tile): tile by tile over all heads, `t` counting a head's tiles in the order they
// should start (the callers put the longest first, so that the grid ends on its shortest blocks).  Orders that keep
// the blocks of a few heads together on an XCD, so that its L2 serves their shared K / V (or Q / dO) tiles, were
// measured and are slower at every group size: the blocks that run at one time then differ in length.
__device__ inline void fa_block_map(int bid, int heads, int tiles, int* head, int* t) {
  *head = bid % heads;
  *t = bid / heads;
}

// =============================================================================
// forward
// =============================================================================
// A block is WAVES waves of 32 queries each that share every K / V tile.  Four at either head dim: at head dim 128 two
// such blocks share a CU and its LDS, which leaves two stages each, and the kernel waits for its tile loads a third
// of its time (measured by taking the loads out); eight waves on one set of tiles (half the loads per CU, LDS for four
// stages) were measured and are no faster in the forward pass and 16 % slower in dQ: under the causal mask the waves
// of a block have unequal work, and with one block per CU nothing fills the SIMDs of those that are done.
template <int D>
__global__ void __launch_bounds__(256, D == 64 ? 3 : 2) flash_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ o, float* __restrict__ lse,
                                                         int B, int S, int nh, int causal, float scale) {
  typedef Rows64<D> Img;
  constexpr int WAVES = 4;
  constexpr int QB = 32 * WAVES;            // queries per block
  constexpr int NS = D == 64 ? 3 : 2;       // LDS stages: tiles t+1 .. t+NS-2 are in flight while tile t is used, t+NS-1 is requested
  constexpr int PW = Img::LOADS / WAVES;    // a wave's loads per K tile (and per V tile)
  __shared__ __attribute__((aligned(1024))) char lds[NS * 2 * Img::BYTES];   // [stage][K | V]
  const int H = nh * D;
  const int64_t ld = 3 * (int64_t)H;
  const int qtiles = (S + QB - 1) / QB;
  // longest blocks first over the whole grid (late query tiles see the most keys): the last blocks to start are the shortest
  int bh, tq;
  fa_block_map((int)blockIdx.x, B * nh, qtiles, &bh, &tq);
  const int qt = qtiles - 1 - tq;   // late query tiles see the most keys
  const int h = bh % nh, b = bh / nh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int q0 = qt * QB;
  const int q = q0 + wave * 32 + lr;
  const bf16* base = qkv + (int64_t)b * S * ld + h * D;   // row 0 of this sequence, q columns of head h
  // K and V tiles of this head: rows past the sequence are the next sequence's (finite, masked) or out of range (zero)
  const uint32_t recs = records_from((int64_t)B * S, (int64_t)b * S, ld, D);
  const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc((void*)(base + H), 0, recs, 0x00020000);
  const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void*)(base + 2 * H), 0, recs, 0x00020000);
  // this lane's offset in the wave's first load of a tile; its further loads lie WAVES * RPL rows further on (a multiple
  // of 16 rows, which leaves the swizzle as it is)
  const uint32_t off0 = Img::lane_offset(wave, lane, ld);
  const uint32_t load_step = (uint32_t)(WAVES * Img::RPL * ld * 2);
  const uint32_t tile_step = (uint32_t)(64 * ld * 2);
  auto issue = [&](char* st, uint32_t tile_off) {
#pragma unroll
    for (int i = 0; i < PW; ++i) {
      fa_load_kib(rk, st + (wave + WAVES * i) * 1024, off0 + i * load_step + tile_off);
      fa_load_kib(rv, st + Img::BYTES + (wave + WAVES * i) * 1024, off0 + i * load_step + tile_off);
    }
  };

  bf16x8 qf[D / 16];
  load_row_frags<D>(qf, base, ld, q, S, g);
  floatx16 oacc[D / 32];
  int2 trb[D / 32];
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct) { zero_acc(oacc[ct]); trb[ct] = Img::tr_base(ct, lane); }
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = scale * LOG2E;
  const int kv_end = causal ? min(S, q0 + QB) : S;
  const int qw0 = q0 + wave * 32;

#pragma unroll
  for (int j = 0; j < NS - 1; ++j)
    if (j * 64 < kv_end) issue(lds + j * 2 * Img::BYTES, (uint32_t)j * tile_step);
  int sc = 0;   // stage of the current tile
  for (int kv0 = 0; kv0 < kv_end; kv0 += 64, sc = sc == NS - 1 ? 0 : sc + 1) {
    // this wave's part of the current tile has landed (loads complete in order; those of up to NS - 2 later tiles may be pending)
    fa_wait_tile<2 * PW>(min(NS - 2, (kv_end - kv0 + 63) / 64 - 1));
    // every wave's part of the tile has landed and its LDS reads of the stage that is filled next have returned; no
    // fence over global memory, which would wait for the tiles that are meant to stay in flight
    block_sync_lds();
    char* cur = lds + sc * 2 * Img::BYTES;
    if (kv0 + 64 * (NS - 1) < kv_end) issue(lds + (sc == 0 ? NS - 1 : sc - 1) * 2 * Img::BYTES, (uint32_t)(kv0 / 64 + NS - 1) * tile_step);
    // a tile that lies wholly behind this wave's queries under the causal mask adds nothing: the wave only keeps step
    if (causal && kv0 > qw0 + 31) continue;
    const char* k_lds = cur;
    const char* v_lds = cur + Img::BYTES;
    // S^T tiles: rows = keys kv0 + u*32 + .., cols = this wave's queries
    floatx16 st[2];
    zero_acc(st[0]);
    zero_acc(st[1]);
    // keys 0-31 and 32-63 of the tile as two chains against the same Q fragments (32 rows further on the swizzle repeats)
    mfma_two_chains<D, 3>(st[0], st[1], k_lds, k_lds + 32 * Img::ROWB, lr, g, qf, qf);
    // V^T fragments, PF 16-row chunks at a time: the first group is issued now and returns behind the
    // softmax arithmetic, each later group behind the MFMAs of the one before
    constexpr int PF = D == 64 ? 2 : 1;
    bf16x8 vf[2][PF][D / 32];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < PF; ++j)
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct) vf[0][j][ct] = Img::frag_tr(v_lds, trb[ct], j);
    __builtin_amdgcn_sched_barrier(0);
    // only tiles that touch the diagonal of this wave's queries or the end of the sequence need the mask
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
    // once the running maxima have settled alpha is exactly 1 in every lane: skip the rescale then
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[ct][i] *= alpha;
    }
    // O^T += V^T P^T
#pragma unroll
    for (int c = 0; c < 4 / PF; ++c) {
      fa_wait_lds();
      if (c + 1 < 4 / PF) {
#pragma unroll
        for (int j = 0; j < PF; ++j)
#pragma unroll
          for (int ct = 0; ct < D / 32; ++ct) vf[(c + 1) & 1][j][ct] = Img::frag_tr(v_lds, trb[ct], (c + 1) * PF + j);
      }
#pragma unroll
      for (int j = 0; j < PF; ++j) {
        const int jj = c * PF + j;
        const bf16x8 pb = regs_to_frag(st[jj >> 1], jj & 1);
#pragma unroll
        for (int ct = 0; ct < D / 32; ++ct)
          oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[c & 1][j][ct], pb, oacc[ct], 0, 0, 0);
      }
    }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  store_rows_from_transposed<D>(o + (int64_t)b * S * H + h * D, H, q, S, g, oacc, inv);
  if (g == 0 && q < S) lse[((int64_t)b * nh + h) * S + q] = m_run * c2 + log2f(l_tot);
}

// =============================================================================
// backward, dQ: block = 128 queries, loop over key tiles (S^T form, lane = query)
// =============================================================================
template <int D>
__global__ void __launch_bounds__(256, D == 64 ? 3 : 2) flash_bwd_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                            const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                            float* __restrict__ delta, bf16* __restrict__ dqkv, int B, int S, int nh,
                                                            int causal, float scale) {
  typedef Rows64<D> Img;
  constexpr int WAVES = 4;                  // waves of 32 queries that share every K / V tile (see the forward kernel)
  constexpr int QB = 32 * WAVES;
  constexpr int NS = D == 64 ? 3 : 2;       // LDS stages
  constexpr int PW = Img::LOADS / WAVES;    // a wave's loads per K tile (and per V tile)
  __shared__ __attribute__((aligned(1024))) char lds[NS * 2 * Img::BYTES];   // [stage][K | V]
  const int H = nh * D;
  const int64_t ld = 3 * (int64_t)H;
  const int qtiles = (S + QB - 1) / QB;
  int bh, tq;
  fa_block_map((int)blockIdx.x, B * nh, qtiles, &bh, &tq);
  const int qt = qtiles - 1 - tq;   // late query tiles see the most keys
  const int h = bh % nh, b = bh / nh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int q0 = qt * QB;
  const int q = q0 + wave * 32 + lr;
  const bf16* base = qkv + (int64_t)b * S * ld + h * D;
  const uint32_t recs = records_from((int64_t)B * S, (int64_t)b * S, ld, D);
  const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc((void*)(base + H), 0, recs, 0x00020000);
  const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void*)(base + 2 * H), 0, recs, 0x00020000);
  // this lane's offset in the wave's first load of a tile; the wave's further loads lie whole rows further on (a
  // multiple of 16 rows, which leaves the swizzle as it is).  One register instead of one per load: the sums are
  // formed where they are used (the empty statement keeps the compiler from forming them once, before the loop, and
  // holding or spilling them)
  const uint32_t off0 = Img::lane_offset(wave, lane, ld);
  const uint32_t load_step = (uint32_t)(WAVES * Img::RPL * ld * 2);
  const uint32_t tile_step = (uint32_t)(64 * ld * 2);
  auto issue = [&](char* st, uint32_t tile_off) {
    uint32_t o = off0 + tile_off;
    asm volatile("" : "+v"(o));
#pragma unroll
    for (int i = 0; i < PW; ++i) {
      fa_load_kib(rk, st + (wave + WAVES * i) * 1024, o + i * load_step);
      fa_load_kib(rv, st + Img::BYTES + (wave + WAVES * i) * 1024, o + i * load_step);
    }
  };

  bf16x8 qf[D / 16], dof[D / 16];
  load_row_frags<D>(qf, base, ld, q, S, g);
  load_row_frags<D>(dof, dout + (int64_t)b * S * H + h * D, H, q, S, g);
  const float c2 = scale * LOG2E;
  const int64_t stat = ((int64_t)b * nh + h) * S + q;
  const float lse2 = q < S ? lse[stat] : 0.f;
  // delta = sum_c dO[q, c] O[q, c]: the lane holds half of dO's row already; O's row is read the same way, once.  The
  // sums are stored for the dK/dV kernel, which runs after this one.
  float dl = 0.f;
  {
    bf16x8 of[D / 16];
    load_row_frags<D>(of, o + (int64_t)b * S * H + h * D, H, q, S, g);
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
#pragma unroll
      for (int k = 0; k < 8; ++k) dl = __builtin_fmaf((float)dof[s][k], (float)of[s][k], dl);
    dl += __shfl_xor(dl, 32, 64);
    if (g == 0 && q < S) delta[stat] = dl;
  }
  floatx16 dq[D / 32];
  int2 trb[D / 32];
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct) { zero_acc(dq[ct]); trb[ct] = Img::tr_base(ct, lane); }
  const int kv_end = causal ? min(S, q0 + QB) : S;

#pragma unroll
  for (int j = 0; j < NS - 1; ++j)
    if (j * 64 < kv_end) issue(lds + j * 2 * Img::BYTES, (uint32_t)j * tile_step);
  int sc = 0;
  for (int kv0 = 0; kv0 < kv_end; kv0 += 64, sc = sc == NS - 1 ? 0 : sc + 1) {
    fa_wait_tile<2 * PW>(min(NS - 2, (kv_end - kv0 + 63) / 64 - 1));
    // every wave's part of the tile has landed and its LDS reads of the stage that is filled next have returned; no
    // fence over global memory, which would wait for the tiles that are meant to stay in flight
    block_sync_lds();
    char* cur = lds + sc * 2 * Img::BYTES;
    if (kv0 + 64 * (NS - 1) < kv_end) issue(lds + (sc == 0 ? NS - 1 : sc - 1) * 2 * Img::BYTES, (uint32_t)(kv0 / 64 + NS - 1) * tile_step);
    // a tile that lies wholly behind this wave's queries under the causal mask adds nothing: the wave only keeps step
    if (causal && kv0 > q0 + wave * 32 + 31) continue;
    const char* k_lds = cur;
    const char* v_lds = cur + Img::BYTES;
    // K^T fragments of the first 32 keys: issued now, they return behind the MFMAs and the exponentials
    bf16x8 kt[2][D / 32];   // K^T fragments of one half (two 16-key chunks)
    // 32 keys at a time, through to dQ: half the score registers of a whole-tile pass.  A half's K^T fragments are
    // requested at its start and return behind its MFMAs and exponentials; one set of registers for them keeps the
    // kernel within 256 registers at head dim 128, which is worth more than the second set: the MFMAs then write
    // ordinary registers (with more than 256 the compiler puts every MFMA result into accumulation registers and
    // copies each score out and in around the vector arithmetic), and two blocks share a CU.
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int ct = 0; ct < D / 32; ++ct) kt[jj][ct] = Img::frag_tr(k_lds, trb[ct], 2 * u + jj);
      __builtin_amdgcn_sched_barrier(0);
      floatx16 st, dpt;
      zero_acc(st);
      zero_acc(dpt);
      mfma_two_chains<D, D == 64 ? 3 : 2>(st, dpt, k_lds, v_lds, u * 32 + lr, g, qf, dof);
      if ((causal && kv0 + 63 > q0 + wave * 32) || kv0 + 64 > S || q0 + QB > S) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kv = kv0 + u * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          const bool ok = kv < S && q < S && (!causal || kv <= q);
          const float p = ok ? fast_exp2(__builtin_fmaf(st[i], c2, -lse2)) : 0.f;
          st[i] = p * (dpt[i] - dl);   // dS^T
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = fast_exp2(__builtin_fmaf(st[i], c2, -lse2));
          st[i] = p * (dpt[i] - dl);
        }
      }
      // dQ^T += K^T dS^T
      fa_wait_lds();
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const bf16x8 dsb = regs_to_frag(st, jj);
#pragma unroll
        for (int ct = 0; ct < D / 32; ++ct)
          dq[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt[jj][ct], dsb, dq[ct], 0, 0, 0);
      }
    }
  }
  store_rows_from_transposed<D>(dqkv + (int64_t)b * S * ld + h * D, ld, q, S, g, dq, scale);
}

// =============================================================================
// backward, dK and dV: block = 128 keys, loop over query tiles (S form, lane = key)
// =============================================================================
template <int D>
__global__ void __launch_bounds__(256, D == 64 ? 2 : 1) flash_bwd_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                             const float* __restrict__ lse, const float* __restrict__ delta,
                                                             bf16* __restrict__ dqkv, int B, int S, int nh, int causal, float scale) {
  typedef Rows64<D> Img;
  constexpr int STAGE = 2 * Img::BYTES + 2048;   // Q | dO | lse2 (first 256 bytes of a KiB) | delta (first 256 bytes of a KiB)
  constexpr int NS = FA_BWD_STAGES;
  __shared__ __attribute__((aligned(1024))) char lds[NS * STAGE];
  const int H = nh * D;
  const int64_t ld = 3 * (int64_t)H;
  // longest blocks first over the whole grid: with the causal mask early key tiles see the most queries
  int bh, ktile;   // with the causal mask early key tiles see the most queries: they come first as they are
  fa_block_map((int)blockIdx.x, B * nh, (S + 127) / 128, &bh, &ktile);
  const int h = bh % nh, b = bh / nh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int kvb = ktile * 128;
  const int kv = kvb + wave * 32 + lr;
  const bf16* qp = qkv + (int64_t)b * S * ld + h * D;
  const bf16* dop = dout + (int64_t)b * S * H + h * D;
  const float* lsep = lse + ((int64_t)b * nh + h) * S;
  const float* delp = delta + ((int64_t)b * nh + h) * S;
  const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc((void*)qp, 0, records_from((int64_t)B * S, (int64_t)b * S, ld, D), 0x00020000);
  const __amdgpu_buffer_rsrc_t rdo = __builtin_amdgcn_make_buffer_rsrc((void*)dop, 0, records_from((int64_t)B * S, (int64_t)b * S, H, D), 0x00020000);
  // statistics of this (sequence, head): S floats each; queries past S are out of range and read as zero
  const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc((void*)lsep, 0, (uint32_t)(S * 4), 0x00020000);
  const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc((void*)delp, 0, (uint32_t)(S * 4), 0x00020000);
  uint32_t offq[Img::PER_WAVE], offd[Img::PER_WAVE];
#pragma unroll
  for (int i = 0; i < Img::PER_WAVE; ++i) {
    offq[i] = Img::lane_offset(wave + 4 * i, lane, ld);
    offd[i] = Img::lane_offset(wave + 4 * i, lane, H);
  }
  const uint32_t stepq = (uint32_t)(64 * ld * 2), stepd = (uint32_t)(64 * (int64_t)H * 2);
  auto issue = [&](char* st, int q0) {
    const uint32_t t = (uint32_t)(q0 / 64);
#pragma unroll
    for (int i = 0; i < Img::PER_WAVE; ++i) {
      fa_load_kib(rq, st + (wave + 4 * i) * 1024, offq[i] + t * stepq);
      fa_load_kib(rdo, st + Img::BYTES + (wave + 4 * i) * 1024, offd[i] + t * stepd);
    }
    // 64 floats = 16 lanes x 16 bytes; the other lanes are parked out of range and write zeros behind them
    const uint32_t so = lane < 16 ? (uint32_t)(q0 * 4 + lane * 16) : FA_OOB;
    if (wave == 0) fa_load_kib(rl, st + 2 * Img::BYTES, so);
    if (wave == 1) fa_load_kib(rd, st + 2 * Img::BYTES + 1024, so);
  };

  bf16x8 kf[D / 16], vf[D / 16];
  load_row_frags<D>(kf, qp + H, ld, kv, S, g);
  load_row_frags<D>(vf, qp + 2 * H, ld, kv, S, g);
  floatx16 dk[D / 32], dv[D / 32];
  int2 trb[D / 32];
#pragma unroll
  for (int ct = 0; ct < D / 32; ++ct) { zero_acc(dk[ct]); zero_acc(dv[ct]); trb[ct] = Img::tr_base(ct, lane); }
  const float c2 = scale * LOG2E;
  const int q_begin = causal ? (kvb / 64) * 64 : 0;

  // waves 0 and 1 issue one load more per tile (the statistics), so waiting until at most NLD loads are
  // pending covers the current tile for every wave
  constexpr int NLD = 2 * Img::PER_WAVE;
  issue(lds, q_begin);
  if (NS == 3 && q_begin + 64 < S) issue(lds + STAGE, q_begin + 64);
  int sc = 0;
  for (int q0 = q_begin; q0 < S; q0 += 64, sc = sc == NS - 1 ? 0 : sc + 1) {
    if (NS == 3 && q0 + 64 < S) __builtin_amdgcn_s_waitcnt(0x0f70 | NLD);
    else __builtin_amdgcn_s_waitcnt(0x0f70);
    // every wave's part of the tile has landed and its LDS reads of the stage that is filled next have returned; no
    // fence over global memory, which would wait for the tile that is meant to stay in flight
    block_sync_lds();
    char* cur = lds + sc * STAGE;
    if (q0 + 64 * (NS - 1) < S) issue(lds + (sc == 0 ? NS - 1 : sc - 1) * STAGE, q0 + 64 * (NS - 1));
    const char* q_lds = cur;
    const char* do_lds = cur + Img::BYTES;
    const float* lse_lds = reinterpret_cast<const float*>(cur + 2 * Img::BYTES);
    const float* delta_lds = reinterpret_cast<const float*>(cur + 2 * Img::BYTES + 1024);
    // dO^T and Q^T fragments of the first 32 queries: issued now, they return behind the MFMAs and the exponentials
    bf16x8 dot[2][2][D / 32], qt[2][2][D / 32];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int ct = 0; ct < D / 32; ++ct) {
        dot[0][jj][ct] = Img::frag_tr(do_lds, trb[ct], jj);
        qt[0][jj][ct] = Img::frag_tr(q_lds, trb[ct], jj);
      }
    __builtin_amdgcn_sched_barrier(0);
    // 32 queries at a time, through to dV and dK: half the score registers of a whole-tile pass
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      floatx16 sm, dp;
      zero_acc(sm);
      zero_acc(dp);
      // statistics of this lane's 16 queries: four runs of four consecutive floats each, requested before the MFMAs
      floatx4 l4[4], d4[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        l4[r] = lds_read_f4(lse_lds + u * 32 + r * 8 + g * 4);
        d4[r] = lds_read_f4(delta_lds + u * 32 + r * 8 + g * 4);
      }
      mfma_two_chains<D>(sm, dp, q_lds, do_lds, u * 32 + lr, g, kf, vf);
      fa_wait_lds();   // the statistics (the transposed fragments too: all LDS reads return in order)
      if ((causal && q0 < kvb + wave * 32 + 31) || q0 + 64 > S || kvb + 128 > S) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int qq = q0 + u * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
          const bool ok = qq < S && kv < S && (!causal || kv <= qq);
          const float e = fast_exp2(__builtin_fmaf(sm[i], c2, -l4[i >> 2][i & 3]));
          const float p = ok ? e : 0.f;
          dp[i] = p * (dp[i] - d4[i >> 2][i & 3]);   // dS
          sm[i] = p;                                          // P
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = fast_exp2(__builtin_fmaf(sm[i], c2, -l4[i >> 2][i & 3]));
          dp[i] = p * (dp[i] - d4[i >> 2][i & 3]);
          sm[i] = p;
        }
      }
      // dV^T += dO^T P,  dK^T += Q^T dS
      fa_wait_lds();
      if (u == 0) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int ct = 0; ct < D / 32; ++ct) {
            dot[1][jj][ct] = Img::frag_tr(do_lds, trb[ct], 2 + jj);
            qt[1][jj][ct] = Img::frag_tr(q_lds, trb[ct], 2 + jj);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const bf16x8 pb = regs_to_frag(sm, jj);
        const bf16x8 dsb = regs_to_frag(dp, jj);
#pragma unroll
        for (int ct = 0; ct < D / 32; ++ct) {
          dv[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot[u][jj][ct], pb, dv[ct], 0, 0, 0);
          dk[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt[u][jj][ct], dsb, dk[ct], 0, 0, 0);
        }
      }
    }
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
  // 32-bit buffer offsets: one sequence of the fused projection must stay well below 4 GiB
  if (((int64_t)S + 128) * 3 * nh * d * 2 >= (int64_t)0xf0000000) return poplar_fail(POPLAR_ERR_INVALID, "sequence too long for the attention kernels");
  return POPLAR_OK;
}

int attn_fwd_flash(hipStream_t s, int B, int S, int nh, int d, int causal, const void* qkv, void* o, float* lse,
                   hipEvent_t ev_start, hipEvent_t ev_stop) {
  POPLAR_TRY(check_flash(B, S, nh, d, qkv));
  if (B == 0 || S == 0) return POPLAR_OK;
  const float scale = 1.0f / sqrtf((float)d);
  dim3 grid((unsigned)((int64_t)B * nh * ((S + 127) / 128)));
  if (d == 64) hipExtLaunchKernelGGL(flash_fwd_kernel<64>, grid, dim3(256), 0, s, ev_start, ev_stop, 0, (const bf16*)qkv, (bf16*)o, lse, B, S, nh, causal, scale);
  else hipExtLaunchKernelGGL(flash_fwd_kernel<128>, grid, dim3(256), 0, s, ev_start, ev_stop, 0, (const bf16*)qkv, (bf16*)o, lse, B, S, nh, causal, scale);
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}

int attn_bwd_flash(hipStream_t s, int B, int S, int nh, int d, int causal, const void* qkv, const void* o, const void* dout,
                   const float* lse, void* dqkv, float* delta, hipEvent_t ev_start, hipEvent_t ev_stop) {
  POPLAR_TRY(check_flash(B, S, nh, d, qkv));
  if (B == 0 || S == 0) return POPLAR_OK;
  const float scale = 1.0f / sqrtf((float)d);
  // dQ first: it also forms delta = rowsum(dO * O), which dK/dV reads.  The first launch carries the start event, the
  // last one the stop event.
  dim3 grid((unsigned)((int64_t)B * nh * ((S + 127) / 128)));
  if (d == 64) {
    hipExtLaunchKernelGGL(flash_bwd_dq_kernel<64>, grid, dim3(256), 0, s, ev_start, nullptr, 0, (const bf16*)qkv, (const bf16*)o, (const bf16*)dout, lse, delta, (bf16*)dqkv, B, S, nh, causal, scale);
    hipExtLaunchKernelGGL(flash_bwd_dkv_kernel<64>, grid, dim3(256), 0, s, nullptr, ev_stop, 0, (const bf16*)qkv, (const bf16*)dout, lse, (const float*)delta, (bf16*)dqkv, B, S, nh, causal, scale);
  } else {
    hipExtLaunchKernelGGL(flash_bwd_dq_kernel<128>, grid, dim3(256), 0, s, ev_start, nullptr, 0, (const bf16*)qkv, (const bf16*)o, (const bf16*)dout, lse, delta, (bf16*)dqkv, B, S, nh, causal, scale);
    hipExtLaunchKernelGGL(flash_bwd_dkv_kernel<128>, grid, dim3(256), 0, s, nullptr, ev_stop, 0, (const bf16*)qkv, (const bf16*)dout, lse, (const float*)delta, (bf16*)dqkv, B, S, nh, causal, scale);
  }
  POPLAR_LAUNCH_CHECK();
  return POPLAR_OK;
}
