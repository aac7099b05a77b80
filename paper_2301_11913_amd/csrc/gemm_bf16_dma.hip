// bf16 MFMA GEMM, pipelined variant for tile-aligned shapes:  C[M,N] (+)= sum_k A(m,k) B(n,k).
//
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, 16 bytes per lane,
// no staging registers) through a ring of NS stages of K-depth DBK, so NS-1 slices are in flight while
// one is multiplied.
// A load instruction fills 1 KiB of contiguous LDS; which 16-byte global chunk a lane fetches is free,
// which gives the bank-conflict-avoiding XOR swizzles below for nothing.
//
//   operand with k contiguous in memory  : LDS tile [rows][DBK k], fragment = one
//                                          ds_read_b128 per 32x16 operand block;
//   operand with k as the slow index     : LDS tile [k][rows] exactly as in memory, fragment = two
//   (W in dgrad, both operands in wgrad)   ds_read_b64_tr_b16 (the LDS transpose read hands lane n the
//                                          four k-consecutive values of column n).  One pass of that
//                                          read serves 32 lanes = 4 k-rows x 64 bytes; rows alias in the
//                                          banks, so 32-byte pairs are XOR-ed with 2*(k-row & 3).
//
// One workgroup owns one output tile and walks K in order: deterministic.
//
// Three kernels share this file: gemm_bf16_dma_kernel (128 x 128 tiles, v_mfma_f32_32x32x16_bf16),
// gemm_bf16_k32_kernel (256 x 256 and 256 x 128 tiles on eight wavefronts, v_mfma_f32_16x16x32_bf16: the dgrad and
// wgrad layouts, the rotary and GeGLU epilogues) and gemm_bf16_w4_kernel (256 x 256 tiles on four wavefronts: the
// forward layout with the store / bias / residual / int8-encoding / GeLU epilogues).  The two 16 x 16 x 32 kernels
// accumulate a tile in the same order and give the same bits; the 32 x 32 x 16 kernel agrees with them to fp32
// rounding of the sums.
#include <algorithm>
#include <type_traits>
#include <utility>

#include "gemm_bf16_common.h"

namespace swarm {
namespace {

typedef __attribute__((ext_vector_type(4))) short i16x4;

constexpr int DBK = 64;        // K depth of a stage (32 or 64; 64 measured faster: full 128-byte lines per row)
constexpr int NS = 2;          // LDS stages (NS x (BM+BN) x DBK x 2 bytes must fit 160 KiB)
constexpr int KCH = DBK / 8;   // 16-byte chunks per row of a non-transposed tile

// chunk swizzle of a non-transposed tile: makes the 16 rows that one LDS pass reads (64 banks x 4 B)
// hit 16 distinct 16-byte bank groups
__device__ __forceinline__ int swz_rows(int row) {
  return DBK == 64 ? ((row & 7) ^ ((row >> 3) & 1)) : ((row >> 2) & 3);
}
// The same for the fragments of the 16 x 16 x 32 kernel, whose lanes read 16 rows x 4 k-quarters: measured with a
// read-only loop, the swizzle above gives that lane order 151 B/clk per compute unit (two-way conflicts) and this
// one 277 B/clk, the rate of a linear read.
__device__ __forceinline__ int swz_rows16(int row) { return row & 7; }
template <bool K32>
__device__ __forceinline__ int swz_rows_of(int row) { return K32 ? swz_rows16(row) : swz_rows(row); }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant expression
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Issue the loads of one operand tile (BR rows of the GEMM x 32 k) into LDS at `lds` (BR*32 elements).
// NW wavefronts share the BR/16 load instructions round-robin.
// The t-th of this wavefront's BR*DBK/512/NW load instructions for the tile.
// glu_split != 0 (GeGLU forward, B = W1 [2*split, K]): the tile's rows are gathered so that every 64-row group
// (one wavefront column) holds 32 gate rows followed by the 32 up rows of the same features; r0 then counts
// features: tile row 64*w + c -> W1 row r0 + 32*w + (c & 31) + (c >= 32 ? split : 0).
template <int BR, int NW, bool TRANS, bool K32 = false>
__device__ __forceinline__ void issue_tile_one(const bf16_raw* __restrict__ g, int ld, int r0, int k0, bf16_raw* lds,
                                               int wave, int lane, int t, int glu_split = 0) {
  {
    const int q = wave + t * NW;            // wave-uniform instruction index; fills lds + q*512 .. +512
    const bf16_raw* src;
    if constexpr (!TRANS) {
      const int row = q * (64 / KCH) + lane / KCH;
      const int chunk = (lane % KCH) ^ swz_rows_of<K32>(row);
      const int grow = glu_split ? r0 + 32 * (row >> 6) + (row & 31) + ((row & 32) ? glu_split : 0) : r0 + row;
      src = g + (size_t)grow * ld + k0 + chunk * 8;
    } else {
      constexpr int CPR = BR / 8;           // 16-byte chunks per k-row
      const int krow = q * (64 / CPR) + lane / CPR;
      // K32: the 16 x 16 x 32 kernel's transpose reads take k-rows 8 apart in one pass; one more swizzle bit keeps
      // them off each other's banks (148 -> 208 B/clk per compute unit in a read-only loop)
      const int chunk = (lane % CPR) ^ (4 * (krow & 3)) ^ (K32 ? 2 * ((krow >> 3) & 1) : 0);
      src = g + (size_t)(k0 + krow) * ld + r0 + chunk * 8;
    }
    __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(lds + q * 512), 16, 0, 0);
  }
}

// The same load with its address split into a wave-uniform 64-bit base (tile origin, slice, instruction index:
// scalar arithmetic) and ONE 32-bit per-lane byte offset that is computed once per kernel.  issue_tile_one forms
// the whole 64-bit address per lane and instruction, and for an operand whose rows are `ld` apart the compiler
// re-multiplies by ld inside the loop (two v_mul_lo_u32 and a v_mad_u64_u32 per load, all quarter rate) rather
// than keep 16 address registers; here a load costs a few scalar instructions.
//   rows as tile rows   : lane offset = ((wave * 8 + lane / 8) * ld + chunk * 8) * 2,
//                         base(t) = g + ((r0 + t * NW * 8) * ld + k0) * 2
//   k-rows as tile rows : lane offset = ((wave * RPI + lane / CPR) * ld + chunk * 8) * 2,
//                         base(t) = g + ((k0 + t * NW * RPI) * ld + r0) * 2          (RPI = 64 / CPR k-rows per load)
// The chunk swizzle is the one of issue_tile_one; it does not depend on t except for (TRANS, K32, BR = 256, NW = 4),
// where it alternates with t (off[t & 1]).
template <int BR, int NW, bool TRANS, bool K32>
struct TileLoad {
  static constexpr bool ALT = TRANS && K32 && BR == 256 && NW == 4;
  uint32_t off[ALT ? 2 : 1];
  __device__ __forceinline__ void init(int ld, int wave, int lane) {
#pragma unroll
    for (int a = 0; a < (ALT ? 2 : 1); ++a) {
      const int q = wave + a * NW;
      if constexpr (!TRANS) {
        const int row = q * (64 / KCH) + lane / KCH;
        const int chunk = (lane % KCH) ^ swz_rows_of<K32>(row);
        off[a] = (uint32_t)((wave * (64 / KCH) + lane / KCH) * ld + chunk * 8) * 2u;
      } else {
        constexpr int CPR = BR / 8;
        const int krow = q * (64 / CPR) + lane / CPR;
        const int chunk = (lane % CPR) ^ (4 * (krow & 3)) ^ (K32 ? 2 * ((krow >> 3) & 1) : 0);
        off[a] = (uint32_t)((wave * (64 / CPR) + lane / CPR) * ld + chunk * 8) * 2u;
      }
    }
  }
  // the t-th of this wavefront's loads of the tile (r0, k0) into the stage at `lds`
  __device__ __forceinline__ void issue(const bf16_raw* __restrict__ g, int ld, int r0, int k0, bf16_raw* lds,
                                        int wave, int t) const {
    const int q = wave + t * NW;
    size_t base;
    if constexpr (!TRANS) base = ((size_t)(r0 + t * NW * (64 / KCH)) * ld + k0) * 2;
    else base = ((size_t)(k0 + t * NW * (64 / (BR / 8))) * ld + r0) * 2;
    const char* src = reinterpret_cast<const char*>(g) + base + off[ALT ? (t & 1) : 0];
    __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(lds + q * 512), 16, 0, 0);
  }
};

template <int BR, int NW, bool TRANS, bool K32 = false>
__device__ __forceinline__ void issue_tile(const bf16_raw* __restrict__ g, int ld, int r0, int k0, bf16_raw* lds,
                                           int wave, int lane, int glu_split = 0) {
  constexpr int NINST = BR * DBK / 512;
  static_assert(NINST % NW == 0, "tile rows must split evenly over the wavefronts");
#pragma unroll
  for (int t = 0; t < NINST / NW; ++t) issue_tile_one<BR, NW, TRANS, K32>(g, ld, r0, k0, lds, wave, lane, t, glu_split);
}

// Fragment (32 GEMM rows x 16 k) for v_mfma_f32_32x32x16_bf16 from a non-transposed tile.
__device__ __forceinline__ bf16x8 frag_rows(const bf16_raw* tile, int row_base, int kk, int l32, int lg) {
  const int row = row_base + l32;
  const int chunk = (2 * kk + lg) ^ swz_rows(l32);
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + row * DBK + chunk * 8));
}

// Same fragment from a [32 k][BR] tile through the LDS transpose read.
template <int BR>
__device__ __forceinline__ bf16x8 frag_trans(const bf16_raw* tile, int col_base, int kk, int lane) {
  const int l16 = lane & 15, grp = lane >> 4;
  const int lg = grp >> 1;
  const int col = col_base + 16 * (grp & 1) + 4 * (l16 & 3);
  const int kq = l16 >> 2;                                   // k-row inside the group of four
  const int chunk = (col >> 3) ^ (4 * kq);
  const int off = chunk * 8 + (col & 4);
  const int krow = 16 * kk + 8 * lg + kq;
  const bf16_raw* p0 = tile + krow * BR + off;
  // Issued as plain instructions: behind the compiler's builtin for this read every pending global -> LDS load
  // is taken as a possible writer of the bytes read and waited for (vmcnt(0)), which would serialise the loads
  // of the next slice with the reads of this one.  The stages are disjoint by construction.  The price: the
  // compiler does not count these reads, so the caller waits for them itself (lds_reads_done) before use.
  const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p0;
  uint2 a, b;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(a) : "v"(addr) : "memory");
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(b) : "v"(addr), "n"(8 * BR) : "memory");
  return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
}

// All LDS reads of this wavefront have returned (also those the compiler does not know of); nothing is
// scheduled across.
__device__ __forceinline__ void lds_reads_done() {
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_sched_barrier(0);
}

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_dma_kernel(KArgs p) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int STAGE = (BM + BN) * DBK;              // elements
  constexpr int IPW = (BM + BN) * DBK / 512 / NW;       // load instructions per wavefront per stage
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];

  int tile_m, tile_n;
  if (p.ksplit > 1) {
    // workgroups [i * ntiles, (i+1) * ntiles) take the i-th part of K of every tile
    const int ntiles = p.tiles_m * p.tiles_n;
    const int part = blockIdx.x / ntiles;
    tile_of_block(p, tile_m, tile_n, blockIdx.x - part * ntiles);
    p.K /= p.ksplit;
    p.A += A_T ? (size_t)part * p.K * p.lda : (size_t)part * p.K;
    p.B += B_T ? (size_t)part * p.K * p.ldb : (size_t)part * p.K;
    p.C = p.part + (size_t)part * p.M * p.N;
    p.ldc = p.N;
    p.epilogue = EPI_PART_F32;
  } else {
    tile_of_block(p, tile_m, tile_n);
  }
  const int m0 = tile_m * BM;
  // GeGLU forward: a tile of BN gathered rows covers BN/2 features; n0 then counts features
  const int glu = (!B_T && p.epilogue == EPI_BIAS_GEGLU) ? p.split : 0;
  const int n0 = glu ? tile_n * (BN / 2) : tile_n * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lg = lane >> 5;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = p.K / DBK;
  auto issue = [&](int kt, int stage) {   // slice kt -> LDS stage `stage`
    bf16_raw* st = lds + stage * STAGE;
    issue_tile<BM, NW, A_T>(p.A, p.lda, m0, kt * DBK, st, wave, lane);
    issue_tile<BN, NW, B_T>(p.B, p.ldb, n0, kt * DBK, st + BM * DBK, wave, lane, glu);
  };
  // When is the stage that a barrier frees refilled?  EARLY: in the sub-step right behind that barrier (slices 0
  // and 1 are requested up front, slice kt+2 behind the barrier that ends slice kt); otherwise one sub-step
  // later, at the top of the next iteration.  Measured: EARLY gains 1-3 % on the 256 x 256 tile and loses 5 % on
  // the 128 x 128 one (two workgroups per compute unit already overlap each other's loads).
  constexpr bool EARLY = BM == 256;
  issue(0, 0);
  if constexpr (EARLY) {
    issue(min(1, KT - 1), 1);
    wait_vmcnt<IPW>();
  } else {
    wait_vmcnt<0>();
  }
  __builtin_amdgcn_s_barrier();

  constexpr int KK = DBK / 16;
  static_assert(NS == 2 && KK % 2 == 0, "the fragment pipeline below assumes two stages and an even slice depth");
  auto load_frags = [&](const bf16_raw* sA, const bf16_raw* sB, int kk, bf16x8 (&a)[FM], bf16x8 (&b)[FN]) {
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      if constexpr (A_T) a[i] = frag_trans<BM>(sA, wm * WTM + i * 32, kk, lane);
      else a[i] = frag_rows(sA, wm * WTM + i * 32, kk, l32, lg);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      if constexpr (B_T) b[j] = frag_trans<BN>(sB, wn * WTN + j * 32, kk, lane);
      else b[j] = frag_rows(sB, wn * WTN + j * 32, kk, l32, lg);
    }
  };
  auto mma = [&](const bf16x8 (&a)[FM], const bf16x8 (&b)[FN]) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };

  // Software pipeline, written out instruction by instruction: every MFMA of sub-step kk is followed by one
  // LDS read of a fragment of sub-step kk+1 (and, in the first sub-step of a slice, by this wavefront's next
  // global -> LDS load of slice kt+1), and a scheduling barrier keeps that order.  Reads are thus spread under
  // the multiplies and the waits in front of the next sub-step are partial.  The last sub-step of a slice is
  // multiplied AFTER the barrier, behind the reads of the next slice's first fragments, so the matrix pipe has
  // work queued across the barrier.  The loop body is one basic block: the last iteration re-fetches the last
  // slice into the free stage instead of branching.
  constexpr int NMMA = FM * FN, NF = FM + FN;
  constexpr int IPA = BM * DBK / 512 / NW;          // this wavefront's load instructions for the A tile
  constexpr int LPM = (IPW + NMMA - 1) / NMMA;      // loads behind one MFMA
  constexpr int RPM = 1;                            // fragment reads behind one MFMA (2 and 3 measured no faster)
  static_assert(NMMA >= NF, "one fragment read per MFMA");
  // reads in the order the next sub-step needs them: A row 0, all of B, the other A rows
  auto read_nth = [&](const bf16_raw* sA, const bf16_raw* sB, int kk, int n, bf16x8 (&a)[FM], bf16x8 (&b)[FN]) {
    if (n == 0 || n > FN) {
      const int i = n == 0 ? 0 : n - FN;
      if constexpr (A_T) a[i] = frag_trans<BM>(sA, wm * WTM + i * 32, kk, lane);
      else a[i] = frag_rows(sA, wm * WTM + i * 32, kk, l32, lg);
    } else {
      const int j = n - 1;
      if constexpr (B_T) b[j] = frag_trans<BN>(sB, wn * WTN + j * 32, kk, lane);
      else b[j] = frag_rows(sB, wn * WTN + j * 32, kk, l32, lg);
    }
  };
  // multiply (ca, cb); read the fragments of sub-step nkk of the tile at nA into (na, nb); with LOADS, issue the
  // loads of slice `lk` into stage `ls`
  // loads inside the loop: split addresses where an operand is transposed (see TileLoad)
  constexpr bool SPLIT_ADDR = A_T || B_T;
  TileLoad<BM, NW, A_T, false> ldA;
  TileLoad<BN, NW, B_T, false> ldB;
  if constexpr (SPLIT_ADDR) {
    ldA.init(p.lda, wave, lane);
    ldB.init(p.ldb, wave, lane);
  }
  auto substep = [&](const bf16x8 (&ca)[FM], const bf16x8 (&cb)[FN], const bf16_raw* nA, int nkk, bf16x8 (&na)[FM],
                     bf16x8 (&nb)[FN], bool loads, int lk, int ls) {
    bf16_raw* st = lds + ls * STAGE;
    if constexpr (A_T || B_T) lds_reads_done();   // (ca, cb) were read by the previous sub-step
#pragma unroll
    for (int n = 0; n < NMMA; ++n) {
      const int i = n / FN, j = n % FN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[i], cb[j], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int r = n * RPM; r < (n + 1) * RPM && r < NF; ++r) read_nth(nA, nA + BM * DBK, nkk, r, na, nb);
      if (loads) {
#pragma unroll
        for (int t = n * LPM; t < (n + 1) * LPM && t < IPW; ++t) {
          if constexpr (SPLIT_ADDR) {
            if (t < IPA) ldA.issue(p.A, p.lda, m0, lk * DBK, st, wave, t);
            else ldB.issue(p.B, p.ldb, n0, lk * DBK, st + BM * DBK, wave, t - IPA);
          } else {
            if (t < IPA) issue_tile_one<BM, NW, A_T>(p.A, p.lda, m0, lk * DBK, st, wave, lane, t);
            else issue_tile_one<BN, NW, B_T>(p.B, p.ldb, n0, lk * DBK, st + BM * DBK, wave, lane, t - IPA, glu);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  bf16x8 fa[2][FM], fb[2][FN];
  load_frags(lds, lds + BM * DBK, 0, fa[0], fb[0]);
  for (int kt = 0; kt < KT; ++kt) {
    const bf16_raw* sA = lds + (kt & 1) * STAGE;
    const bf16_raw* nA = lds + ((kt + 1) & 1) * STAGE;
#pragma unroll
    for (int kk = 0; kk + 1 < KK; ++kk)
      substep(fa[kk & 1], fb[kk & 1], sA, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1], !EARLY && kk == 0,
              min(kt + 1, KT - 1), (kt + 1) & 1);
    // slice kt+1 must have landed (this wavefront's part) and this wavefront's reads of slice kt be complete;
    // then all wavefronts meet
    wait_vmcnt<0>();
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
    // the stage of slice kt is free (the last iterations re-fetch the last slice instead of branching)
    substep(fa[(KK - 1) & 1], fb[(KK - 1) & 1], nA, 0, fa[0], fb[0], EARLY, min(kt + 2, KT - 1), kt & 1);
  }
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();   // all MFMAs read registers only, but keep the epilogue's LDS reuse fenced

  // every wavefront is past the last barrier: the operand stages are free to serve as epilogue patches
  gemm_epilogue<FM, FN, false>(p, acc, m0 + wm * WTM, glu ? n0 + wn * (WTN / 2) : n0 + wn * WTN, l32, lg,
                               reinterpret_cast<float*>(lds) + wave * 32 * kEpiPitch);
}

// ------------------------------------------------------------------------------------------------------------
// The same product on v_mfma_f32_16x16x32_bf16.  A loop of nothing but MFMAs on random operands sustains 5-12 %
// more flops with the 16 x 16 x 32 shape than with 32 x 32 x 16 (the chip is power-limited there), and this kernel
// keeps that margin.  Per 32-deep sub-step a wavefront holds WTM/16 A fragments (16 rows x 32 k, 8 k-values per
// lane: lane % 16 -> row, lane / 16 -> k quarter) and WTN/16 B fragments; the MFMAs go row by row, and the A
// fragment of a row is re-read for the next sub-step as soon as the row is done (single buffer), the B fragments
// alternate between two buffers.  Two sub-steps per 64-deep slice; the second starts with one row of MFMAs, then
// the per-slice load wait and barrier, then the reads of the next slice and the refill of the freed stage.

// 16 rows x 32 k fragment of a non-transposed tile (rows of DBK k)
__device__ __forceinline__ bf16x8 frag_rows16(const bf16_raw* tile, int row_base, int kk, int l16, int q) {
  const int row = row_base + l16;
  const int chunk = (4 * kk + q) ^ swz_rows16(l16);
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + row * DBK + chunk * 8));
}
// the same fragment from a [k][BR] tile through the LDS transpose read (two plain instructions, caller waits)
template <int BR>
__device__ __forceinline__ bf16x8 frag_trans16(const bf16_raw* tile, int col_base, int kk, int lane) {
  const int l16 = lane & 15, q = lane >> 4;
  const int col = col_base + 4 * (l16 & 3);
  const int kq = l16 >> 2;                                   // k-row inside the group of four
  const int chunk = (col >> 3) ^ (4 * kq) ^ (2 * (q & 1));   // as written by issue_tile_one<..., K32 = true>
  const int off = chunk * 8 + (col & 4);
  const int krow = 32 * kk + 8 * q + kq;
  const bf16_raw* p0 = tile + krow * BR + off;
  const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p0;
  uint2 a, b;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(a) : "v"(addr) : "memory");
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(b) : "v"(addr), "n"(8 * BR) : "memory");
  return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
}

// Which fragment of the NEXT sub-step is requested behind MFMA slot n (slot = FN * row + column): 0 .. FM-1 = A row,
// FM + j = B column j, -1 = none.  kind 0: a sub-step without barrier; kind 1: barrier behind slot FN - 1, nothing
// of the next slice may be read before it.  No slot holds two fragments: B sits in column 1 of a row (column 0
// when a row has only two), A in the last column (A_0 of kind 1: the first one behind the barrier).
template <int FM, int FN>
constexpr int k32_read_at(int kind, int n) {
  constexpr int BCOL = FN > 2 ? 1 : 0;
  if (n % FN == FN - 1 && n / FN >= 1) return n / FN;                      // A_i behind the last MFMA of row i >= 1
  if (kind == 0) {
    if (n == FN - 1) return 0;                                             // A_0 behind the last MFMA of row 0
    if (n % FN == BCOL && n / FN < FN) return FM + n / FN;                 // B_j in row j
  } else {
    constexpr int R0 = FN > 2 ? 1 : 2;                                     // first row with a B request
    if (n == FN) return 0;                                                 // A_0 behind the first MFMA after the barrier
    if (n % FN == BCOL && n / FN >= R0 && n / FN < R0 + FN) return FM + n / FN - R0;   // B_j in row j + R0
  }
  return -1;
}
// LDS read instructions younger than the fragment(s) that row i of a sub-step of kind `cur` needs (A_i; for i = 0
// also every B), `prev` being the kind of the sub-step before it; ia / ib = instructions per A / B fragment
template <int FM, int FN>
constexpr int k32_younger(int prev, int cur, int i, int ia, int ib) {
  int needed = -1;
  for (int n = 0; n < FM * FN; ++n) {
    const int f = k32_read_at<FM, FN>(prev, n);
    if (f == i || (i == 0 && f >= FM)) needed = n > needed ? n : needed;
  }
  int cnt = 0;
  for (int n = needed + 1; n < FM * FN; ++n) {
    const int f = k32_read_at<FM, FN>(prev, n);
    if (f >= 0) cnt += f < FM ? ia : ib;
  }
  for (int n = 0; n < FN * i; ++n) {
    const int f = k32_read_at<FM, FN>(cur, n);
    if (f >= 0) cnt += f < FM ? ia : ib;
  }
  return cnt > 15 ? 15 : cnt;
}

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_k32_kernel(KArgs p) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int FM = WTM / 16, FN = WTN / 16;
  constexpr int STAGE = (BM + BN) * DBK;              // elements
  constexpr int IPW = (BM + BN) * DBK / 512 / NW;       // load instructions per wavefront per stage
  constexpr int IPA = BM * DBK / 512 / NW;
  static_assert(DBK == 64 && NS == 2, "two 32-deep sub-steps per slice, two stages");
  static_assert(FN >= 2 && FM >= FN + 2 && 2 * IPW + FN + 2 <= FM * FN, "read / load slots of a sub-step");
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];
#ifdef SWARM_KERNEL_HOOKS
  // Instrumented build: wall-clock stamps (100 MHz counter) at the start, at the first barrier, behind the loop
  // and when the epilogue's stores have left; written only when the caller asks (p.stamps).
  long long stamp[4], cyc[2];
  stamp[0] = wall_clock64();
#endif

  int tile_m, tile_n;
  if (p.ksplit > 1) {
    const int ntiles = p.tiles_m * p.tiles_n;
    const int part = blockIdx.x / ntiles;
    tile_of_block(p, tile_m, tile_n, blockIdx.x - part * ntiles);
    p.K /= p.ksplit;
    p.A += A_T ? (size_t)part * p.K * p.lda : (size_t)part * p.K;
    p.B += B_T ? (size_t)part * p.K * p.ldb : (size_t)part * p.K;
    p.C = p.part + (size_t)part * p.M * p.N;
    p.ldc = p.N;
    p.epilogue = EPI_PART_F32;
  } else {
    tile_of_block(p, tile_m, tile_n);
  }
  const int m0 = tile_m * BM;
  const int glu = (!B_T && p.epilogue == EPI_BIAS_GEGLU) ? p.split : 0;
  const int n0 = glu ? tile_n * (BN / 2) : tile_n * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l16 = lane & 15, q = lane >> 4;

  Acc16<WTM / 32, WTN / 32> acc;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc.blk[i][j][r] = 0.f;

  const int KT = p.K / DBK;
  issue_tile<BM, NW, A_T, true>(p.A, p.lda, m0, 0, lds, wave, lane);
  issue_tile<BN, NW, B_T, true>(p.B, p.ldb, n0, 0, lds + BM * DBK, wave, lane, glu);
  {
    const int k1 = min(1, KT - 1) * DBK;
    issue_tile<BM, NW, A_T, true>(p.A, p.lda, m0, k1, lds + STAGE, wave, lane);
    issue_tile<BN, NW, B_T, true>(p.B, p.ldb, n0, k1, lds + STAGE + BM * DBK, wave, lane, glu);
  }
  wait_vmcnt<IPW>();
  __builtin_amdgcn_s_barrier();
#ifdef SWARM_KERNEL_HOOKS
  stamp[1] = wall_clock64();
  cyc[0] = clock64();
#endif

  auto read_a = [&](const bf16_raw* sA, int i, int kk) __attribute__((always_inline)) {
    if constexpr (A_T) return frag_trans16<BM>(sA, wm * WTM + 16 * i, kk, lane);
    else return frag_rows16(sA, wm * WTM + 16 * i, kk, l16, q);
  };
  auto read_b = [&](const bf16_raw* sA, int j, int kk) __attribute__((always_inline)) {
    const bf16_raw* sB = sA + BM * DBK;
    if constexpr (B_T) return frag_trans16<BN>(sB, wn * WTN + 16 * j, kk, lane);
    else return frag_rows16(sB, wn * WTN + 16 * j, kk, l16, q);
  };
  bf16x8 fa[FM], fb[2][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) fa[i] = read_a(lds, i, 0);
#pragma unroll
  for (int j = 0; j < FN; ++j) fb[0][j] = read_b(lds, j, 0);
  lds_reads_done();

  // loads inside the loop: split addresses where an operand is transposed (the k-contiguous forward layout keeps
  // issue_tile_one, which also knows the GeGLU row gather)
  constexpr bool SPLIT_ADDR = A_T || B_T;
  TileLoad<BM, NW, A_T, true> ldA;
  TileLoad<BN, NW, B_T, true> ldB;
  if constexpr (SPLIT_ADDR) {
    ldA.init(p.lda, wave, lane);
    ldB.init(p.ldb, wave, lane);
  }
  constexpr int IA = A_T ? 2 : 1, IB = B_T ? 2 : 1;
  // One sub-step: FM * FN MFMAs on (fa, cb); behind them the reads of the next sub-step's fragments from the tile
  // at nA, sub-step nkk (A in place, B into nb).  KIND 1: the per-slice wait and barrier sit behind the first row,
  // and the loads of slice lk go into stage ls behind the MFMAs that follow it.
  auto substep = [&](auto kind_c, const bf16x8 (&cb)[FN], bf16x8 (&nb)[FN], const bf16_raw* nA, int nkk, int lk,
                     int ls) __attribute__((always_inline)) {
    constexpr int KIND = decltype(kind_c)::value;
    bf16_raw* st = lds + ls * STAGE;
    static_for<FM * FN>([&](auto nc) __attribute__((always_inline)) {
      constexpr int n = decltype(nc)::value;
      constexpr int i = n / FN, j = n % FN;
      if constexpr (j == 0 && (A_T || B_T)) {
        // fragments requested with plain instructions: wait until A_i (row 0: and every B) has arrived
        constexpr int younger = k32_younger<FM, FN>(1 - KIND, KIND, i, IA, IB);
        __builtin_amdgcn_s_waitcnt(0xC07F | (younger << 8));
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (KIND == 1 && n == FN) {
        // slice kt+1 must have landed (this wavefront's part) and this wavefront's reads of slice kt be complete;
        // then all wavefronts meet
        wait_vmcnt<0>();
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
      }
      acc.blk[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], cb[j], acc.blk[i][j], 0, 0, 0);
      constexpr int f = k32_read_at<FM, FN>(KIND, n);
      if constexpr (f >= 0 && f < FM) fa[f] = read_a(nA, f, nkk);
      if constexpr (f >= FM) nb[f - FM] = read_b(nA, f - FM, nkk);
      if constexpr (KIND == 1 && n >= FN + 2 && (n - FN) % 2 == 0 && (n - FN - 2) / 2 < IPW) {
        constexpr int t = (n - FN - 2) / 2;
        if constexpr (SPLIT_ADDR) {
          if constexpr (t < IPA) ldA.issue(p.A, p.lda, m0, lk * DBK, st, wave, t);
          else ldB.issue(p.B, p.ldb, n0, lk * DBK, st + BM * DBK, wave, t - IPA);
        } else {
          if constexpr (t < IPA) issue_tile_one<BM, NW, A_T, true>(p.A, p.lda, m0, lk * DBK, st, wave, lane, t);
          else issue_tile_one<BN, NW, B_T, true>(p.B, p.ldb, n0, lk * DBK, st + BM * DBK, wave, lane, t - IPA, glu);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  for (int kt = 0; kt < KT; ++kt) {
    const bf16_raw* sA = lds + (kt & 1) * STAGE;
    const bf16_raw* nA = lds + ((kt + 1) & 1) * STAGE;
    substep(std::integral_constant<int, 0>{}, fb[0], fb[1], sA, 1, 0, 0);
    // the stage of slice kt is free behind the barrier (the last iterations re-fetch the last slice instead of
    // branching)
    substep(std::integral_constant<int, 1>{}, fb[1], fb[0], nA, 0, min(kt + 2, KT - 1), kt & 1);
  }
  wait_vmcnt<0>();
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_s_barrier();   // every wavefront is past its last LDS read: the stages become epilogue patches
#ifdef SWARM_KERNEL_HOOKS
  stamp[2] = wall_clock64();
  cyc[1] = clock64();
#endif

  gemm_epilogue<WTM / 32, WTN / 32, false>(p, acc, m0 + wm * WTM, glu ? n0 + wn * (WTN / 2) : n0 + wn * WTN,
                                          lane & 31, lane >> 5,
                                          reinterpret_cast<float*>(lds) + wave * 32 * kEpiPitch);
#ifdef SWARM_KERNEL_HOOKS
  if (p.stamps) {
    wait_vmcnt<0>();   // the stores have left
    stamp[3] = wall_clock64();
    if (threadIdx.x == 0) {
      long long* out = p.stamps + (size_t)blockIdx.x * 16;
      out[0] = stamp[0]; out[1] = stamp[1]; out[2] = stamp[2]; out[3] = stamp[3];
      out[4] = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));    // HW_ID: compute unit, shader engine
      out[5] = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (31 << 11));   // XCC_ID
      out[6] = tile_m; out[7] = tile_n;
      out[8] = cyc[1] - cyc[0];   // shader cycles spent in the loop
    }
  }
#endif
}

// ------------------------------------------------------------------------------------------------------------
// The 256 x 256 tile on FOUR wavefronts of 128 x 128, both operands k-contiguous (forward products).  A wavefront's
// sub-step reads 8 + 8 fragments for 64 MFMAs where the 128 x 64 sub-tiles above read 8 + 4 for 32: a third fewer
// LDS bytes per flop, and LDS reads are what costs clock next to the matrix pipes.  One wavefront per SIMD has no
// partner to cover its waits, so nothing here may wait for anything recent:
//   - the 256 accumulator registers live in the accumulation half of the register file and the MFMAs work on them
//     in place (inline assembly: left to the compiler the products are formed in vector registers and copied over);
//   - both fragment sets are double-buffered (128 vector registers) and every read of the next sub-step is requested
//     during the first half of the current one, with plain instructions: the compiler turns each wait for an LDS read
//     it knows of into a wait for all of them while global -> LDS loads are in flight, and would put one in front of
//     every sub-step;
//   - the per-slice barrier sits behind the second MFMA of the slice's second sub-step, the reads of the next slice
//     and the refill of the freed stage follow it.
typedef uint32_t u32x4_frag __attribute__((ext_vector_type(4)));
template <int BYTE_OFF>
__device__ __forceinline__ bf16x8 lds_frag_plain(uint32_t addr) {
  static_assert(BYTE_OFF >= 0 && BYTE_OFF < 65536, "ds offset field");
  u32x4_frag v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(BYTE_OFF) : "memory");
  return __builtin_bit_cast(bf16x8, v);
}

// Epilogue of the four-wavefront kernel.  Its MFMAs take the B fragment as the first operand, so a lane's block
// registers are FOUR CONSECUTIVE COLUMNS of one row: blk[i][j][r] = C(row0 + 16 i + lane % 16, col0 + 16 j +
// 4 (lane / 16) + r).  One wavefront alone on its SIMD issues vector instructions at about half the rate two reach
// together, so the epilogue is kept short: the arithmetic (bias, residual) runs on the accumulator layout, the
// results are rounded to bf16 and turned into row order through ONE pass over a private 128 x 128 bf16 patch
// (8-byte cells in, 16-byte row pieces out), and the residual rows take the same patch the other way (16-byte row
// pieces in, the lane's own 8-byte cell out).  Same arithmetic, in the same order, as gemm_epilogue: the two kernels
// give the same bits.  Handles EPI_STORE, EPI_BIAS, EPI_BIAS_RESID, EPI_BIAS_RESID_ENCODE and EPI_PART_F32.
constexpr int kW4PatchPitch = 272;                       // bytes per patch row: 256 + 16 (rows 4 banks apart)
constexpr int kW4PatchBytes = 128 * kW4PatchPitch;       // per wavefront

inline bool w4_epilogue_ok(int epi) {
  return epi == EPI_STORE || epi == EPI_BIAS || epi == EPI_BIAS_RESID || epi == EPI_BIAS_RESID_ENCODE ||
         epi == EPI_BIAS_GELU;
}

// one accumulator register into a vector register, where it is used (left to itself the compiler moves all 256
// over at the start of the epilogue and spills)
__device__ __forceinline__ float acc_read(const float& a) {
  float v;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

template <int EPI, bool NT>
__device__ __forceinline__ void w4_epilogue_nt(const KArgs& p, const Acc16<4, 4>& acc, int row0, int col0, int lane,
                                               char* patch) {
  const int l16 = lane & 15, q = lane >> 4;
  if constexpr (EPI == EPI_PART_F32) {   // fp32 partial tile of a product cut along K: 16 bytes per lane, as they are
    float* c = reinterpret_cast<float*>(p.C) + (size_t)(row0 + l16) * p.ldc + col0 + 4 * q;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float4 v = make_float4(acc_read(acc.blk[i][j][0]), acc_read(acc.blk[i][j][1]),
                                     acc_read(acc.blk[i][j][2]), acc_read(acc.blk[i][j][3]));
        *reinterpret_cast<float4*>(c + (size_t)(16 * i) * p.ldc + 16 * j) = v;
        if (j == 7) __builtin_amdgcn_sched_barrier(0);
      }
    return;
  }
  constexpr bool has_aux = EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_RESID_ENCODE;
  // row-order accesses: 16 lanes cover the 256 bytes of a patch row, an instruction covers 4 rows
  const int c16 = lane & 15, r4 = lane >> 4;
  if constexpr (has_aux) {
#pragma unroll 1
    for (int t0 = 0; t0 < 32; t0 += 8) {      // eight loads in flight
      uint4 v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t)
        v[t] = load_stream<NT>(p.aux + (size_t)(row0 + 4 * (t0 + t) + r4) * p.ldaux + col0 + 8 * c16);
#pragma unroll
      for (int t = 0; t < 8; ++t)
        *reinterpret_cast<uint4*>(patch + (4 * (t0 + t) + r4) * kW4PatchPitch + 16 * c16) = v[t];
    }
  }
  float bias[8][4];
  if constexpr (EPI != EPI_STORE) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint2 b = *reinterpret_cast<const uint2*>(p.bias + col0 + 16 * j + 4 * q);
      bias[j][0] = __uint_as_float(b.x << 16); bias[j][1] = __uint_as_float(b.x & 0xFFFF0000u);
      bias[j][2] = __uint_as_float(b.y << 16); bias[j][3] = __uint_as_float(b.y & 0xFFFF0000u);
    }
  }
  char* cell0 = patch + l16 * kW4PatchPitch + 8 * q;      // block (i, j): + 16 i rows + 32 j bytes
  if constexpr (EPI == EPI_BIAS_GELU) {
    // two outputs, two passes through the patch: the pre-activations u = acc + bias (when the caller keeps them),
    // then gelu(u) of the same fp32 values
    if (p.C2) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          float x[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) x[r] = acc_read(acc.blk[i][j][r]) + bias[j][r];
          *reinterpret_cast<uint2*>(cell0 + 16 * i * kW4PatchPitch + 32 * j) =
              make_uint2(cvt_pk_bf16(x[0], x[1]), cvt_pk_bf16(x[2], x[3]));
          if (j == 7) __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll 1
      for (int t0 = 0; t0 < 32; t0 += 8)
#pragma unroll
        for (int tt = 0; tt < 8; ++tt) {
          const int row = 4 * (t0 + tt) + r4;
          const uint4 v = *reinterpret_cast<const uint4*>(patch + row * kW4PatchPitch + 16 * c16);
          store_stream<NT>(p.C2 + (size_t)(row0 + row) * p.ldc2 + col0 + 8 * c16, v);
        }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      char* cell = cell0 + 16 * i * kW4PatchPitch + 32 * j;
      float x[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = acc_read(acc.blk[i][j][r]);
      if constexpr (EPI == EPI_BIAS_GELU) {
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = gelu_fast(x[r] + bias[j][r]);
      } else if constexpr (has_aux) {
        const uint2 a = *reinterpret_cast<const uint2*>(cell);
        const float av[4] = {__uint_as_float(a.x << 16), __uint_as_float(a.x & 0xFFFF0000u),
                             __uint_as_float(a.y << 16), __uint_as_float(a.y & 0xFFFF0000u)};
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = x[r] + bias[j][r] + av[r];
      } else if constexpr (EPI == EPI_BIAS) {
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] += bias[j][r];
      }
      *reinterpret_cast<uint2*>(cell) = make_uint2(cvt_pk_bf16(x[0], x[1]), cvt_pk_bf16(x[2], x[3]));
      if (j == 7) __builtin_amdgcn_sched_barrier(0);     // a block row at a time: few registers
    }
  bf16_raw* C = reinterpret_cast<bf16_raw*>(p.C);
#pragma unroll 1
  for (int t0 = 0; t0 < 32; t0 += 8)
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) {
      const int row = 4 * (t0 + tt) + r4;
      const uint4 v = *reinterpret_cast<const uint4*>(patch + row * kW4PatchPitch + 16 * c16);
      const int col = col0 + 8 * c16;
      if constexpr (EPI == EPI_BIAS_RESID_ENCODE) {
        // the 8 lanes of a row segment hold one 64-element block of the bf16 values that a plain store would write
        float x[8];
        unpack8(v, x);
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
        amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
        amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
        amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
        const float sc = block_scale_rounded(amax / 127.0f, p.scales16);
        uint32_t w[2] = {0u, 0u};
        if (sc != 0.0f) {
          const BlockDivisor div(sc);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float qv = fminf(fmaxf(rintf(div.quotient(x[e])), -127.0f), 127.0f);
            w[e >> 2] |= ((uint32_t)(int)qv & 0xFFu) << (8 * (e & 3));
          }
        }
        const size_t e0 = (size_t)(row0 + row) * p.ldc + col;
        *reinterpret_cast<uint2*>(reinterpret_cast<int8_t*>(p.C) + e0) = make_uint2(w[0], w[1]);
        if ((c16 & 7) == 0) block_scale_store(p.scales, e0 >> 6, sc, p.scales16);
      } else {
        store_stream<NT>(C + (size_t)(row0 + row) * p.ldc + col, v);
      }
    }
}

// one uniform branch per epilogue kind and store kind: every copy is straight-line code
__device__ __forceinline__ void w4_epilogue(const KArgs& p, const Acc16<4, 4>& acc, int row0, int col0, int lane,
                                            char* patch) {
  const int epi = p.epilogue;
  if (epi == EPI_PART_F32) return w4_epilogue_nt<EPI_PART_F32, false>(p, acc, row0, col0, lane, patch);
  if (p.stream) {
    if (epi == EPI_STORE) return w4_epilogue_nt<EPI_STORE, true>(p, acc, row0, col0, lane, patch);
    if (epi == EPI_BIAS) return w4_epilogue_nt<EPI_BIAS, true>(p, acc, row0, col0, lane, patch);
    if (epi == EPI_BIAS_RESID) return w4_epilogue_nt<EPI_BIAS_RESID, true>(p, acc, row0, col0, lane, patch);
    if (epi == EPI_BIAS_GELU) return w4_epilogue_nt<EPI_BIAS_GELU, true>(p, acc, row0, col0, lane, patch);
    return w4_epilogue_nt<EPI_BIAS_RESID_ENCODE, true>(p, acc, row0, col0, lane, patch);
  }
  if (epi == EPI_STORE) return w4_epilogue_nt<EPI_STORE, false>(p, acc, row0, col0, lane, patch);
  if (epi == EPI_BIAS) return w4_epilogue_nt<EPI_BIAS, false>(p, acc, row0, col0, lane, patch);
  if (epi == EPI_BIAS_RESID) return w4_epilogue_nt<EPI_BIAS_RESID, false>(p, acc, row0, col0, lane, patch);
  if (epi == EPI_BIAS_GELU) return w4_epilogue_nt<EPI_BIAS_GELU, false>(p, acc, row0, col0, lane, patch);
  return w4_epilogue_nt<EPI_BIAS_RESID_ENCODE, false>(p, acc, row0, col0, lane, patch);
}

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_bf16_w4_kernel(KArgs p) {
  constexpr int NW = 4, WN = 2;
  constexpr int WTM = BM / 2, WTN = BN / 2;
  constexpr int FM = WTM / 16, FN = WTN / 16;
  constexpr int STAGE = (BM + BN) * DBK;              // elements
  constexpr int IPW = (BM + BN) * DBK / 512 / NW;       // load instructions per wavefront per stage
  constexpr int IPA = BM * DBK / 512 / NW;
  constexpr int NR = FM + FN;                           // fragment reads per sub-step
  static_assert(DBK == 64 && NS == 2, "two 32-deep sub-steps per slice, two stages");
  static_assert(2 * NR + 2 <= FM * FN && 4 * IPW <= FM * FN, "read / load slots of a sub-step");
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];
#ifdef SWARM_KERNEL_HOOKS
  long long stamp[4], cyc[2];
  stamp[0] = wall_clock64();
#endif

  int tile_m, tile_n;
  if (p.ksplit > 1) {
    const int ntiles = p.tiles_m * p.tiles_n;
    const int part = blockIdx.x / ntiles;
    tile_of_block(p, tile_m, tile_n, blockIdx.x - part * ntiles);
    p.K /= p.ksplit;
    p.A += (size_t)part * p.K;
    p.B += (size_t)part * p.K;
    p.C = p.part + (size_t)part * p.M * p.N;
    p.ldc = p.N;
    p.epilogue = EPI_PART_F32;
  } else {
    tile_of_block(p, tile_m, tile_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l16 = lane & 15, q = lane >> 4;

  Acc16<WTM / 32, WTN / 32> acc;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc.blk[i][j][r] = 0.f;

  const int KT = p.K / DBK;
  issue_tile<BM, NW, false, true>(p.A, p.lda, m0, 0, lds, wave, lane);
  issue_tile<BN, NW, false, true>(p.B, p.ldb, n0, 0, lds + BM * DBK, wave, lane);
  {
    const int k1 = min(1, KT - 1) * DBK;
    issue_tile<BM, NW, false, true>(p.A, p.lda, m0, k1, lds + STAGE, wave, lane);
    issue_tile<BN, NW, false, true>(p.B, p.ldb, n0, k1, lds + STAGE + BM * DBK, wave, lane);
  }
  wait_vmcnt<IPW>();
  __builtin_amdgcn_s_barrier();
#ifdef SWARM_KERNEL_HOOKS
  stamp[1] = wall_clock64();
  cyc[0] = clock64();
#endif

  // byte address of this lane's 16 bytes of fragment 0 of A resp. B in stage 0, sub-step kk (fragment i adds
  // 16 rows = 2048 bytes as an immediate; the chunk swizzle depends on the row's low bits only)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds;
  uint32_t offA[2], offB[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const uint32_t chunk = (uint32_t)((4 * kk + q) ^ swz_rows16(l16)) * 16u;
    offA[kk] = lds0 + (uint32_t)(wm * WTM + l16) * (DBK * 2) + chunk;
    offB[kk] = lds0 + (uint32_t)(BM + wn * WTN + l16) * (DBK * 2) + chunk;
  }
  bf16x8 fa[2][FM], fb[2][FN];
  static_for<FM>([&](auto ic) __attribute__((always_inline)) {
    fa[0][decltype(ic)::value] = lds_frag_plain<2048 * decltype(ic)::value>(offA[0]);
  });
  static_for<FN>([&](auto jc) __attribute__((always_inline)) {
    fb[0][decltype(jc)::value] = lds_frag_plain<2048 * decltype(jc)::value>(offB[0]);
  });

  // One sub-step: FM * FN MFMAs on buffer CUR; the fragments of the next sub-step (stage byte offset nst, sub-step
  // nkk) go into the other buffer behind the even MFMAs 2 r.  KIND 1: wait and barrier behind MFMA 1, the reads start
  // behind MFMA 2, and the loads of slice lk go into stage ls behind the MFMAs 4 t + 3.
  auto substep = [&](auto kind_c, auto cur_c, uint32_t nst, int nkk, int lk, int ls) __attribute__((always_inline)) {
    constexpr int KIND = decltype(kind_c)::value;
    constexpr int CUR = decltype(cur_c)::value, NXT = 1 - CUR;
    constexpr int R0 = KIND == 1 ? 2 : 0;     // MFMA slot of the first read
    bf16_raw* st = lds + ls * STAGE;
    const uint32_t na = offA[nkk] + nst, nb = offB[nkk] + nst;
    static_for<FM * FN>([&](auto nc) __attribute__((always_inline)) {
      constexpr int n = decltype(nc)::value;
      constexpr int i = n / FN;
      constexpr int j = (i & 1) ? FN - 1 - n % FN : n % FN;    // rows alternate direction: one operand changes per MFMA
      if constexpr (n == 0) {
        // buffer CUR was requested during the first half of the previous sub-step
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (KIND == 1 && n == 2) {
        // slice kt+1 has landed (this wavefront's part), this wavefront's reads of slice kt are complete: all meet
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
      // B fragment first: the block comes out with the lane's four registers along a row of C (see w4_epilogue_nt)
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc.blk[i][j]) : "v"(fb[CUR][j]), "v"(fa[CUR][i]));
      if constexpr (n >= R0 && (n - R0) % 2 == 0 && (n - R0) / 2 < NR) {
        constexpr int r = (n - R0) / 2;
        if constexpr (r < FN) fb[NXT][r < FN ? r : 0] = lds_frag_plain<2048 * (r < FN ? r : 0)>(nb);
        else fa[NXT][r >= FN ? r - FN : 0] = lds_frag_plain<2048 * (r >= FN ? r - FN : 0)>(na);
      }
      if constexpr (KIND == 1 && n % 4 == 3 && n / 4 < IPW) {
        constexpr int t = n / 4;
        if constexpr (t < IPA) issue_tile_one<BM, NW, false, true>(p.A, p.lda, m0, lk * DBK, st, wave, lane, t);
        else issue_tile_one<BN, NW, false, true>(p.B, p.ldb, n0, lk * DBK, st + BM * DBK, wave, lane, t - IPA);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  for (int kt = 0; kt < KT; ++kt) {
    const uint32_t cst = (uint32_t)(kt & 1) * (STAGE * 2), nst = (uint32_t)((kt + 1) & 1) * (STAGE * 2);
    substep(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, cst, 1, 0, 0);
    // the stage of slice kt is free behind the barrier (the last iterations re-fetch the last slice instead of
    // branching)
    substep(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, nst, 0, min(kt + 2, KT - 1), kt & 1);
  }
  wait_vmcnt<0>();
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_s_barrier();   // every wavefront is past its last LDS read: the stages become epilogue patches
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last in-place MFMAs retire before their results are read
#ifdef SWARM_KERNEL_HOOKS
  stamp[2] = wall_clock64();
  cyc[1] = clock64();
#endif

  static_assert(WTM == 128 && WTN == 128, "the epilogue's patch is 128 x 128");
  char* patch = reinterpret_cast<char*>(lds) + wave * kW4PatchBytes;
  w4_epilogue(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane, patch);
#ifdef SWARM_KERNEL_HOOKS
  if (p.stamps) {
    wait_vmcnt<0>();   // the stores have left
    stamp[3] = wall_clock64();
    if (threadIdx.x == 0) {
      long long* out = p.stamps + (size_t)blockIdx.x * 16;
      out[0] = stamp[0]; out[1] = stamp[1]; out[2] = stamp[2]; out[3] = stamp[3];
      out[4] = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));    // HW_ID: compute unit, shader engine
      out[5] = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (31 << 11));   // XCC_ID
      out[6] = tile_m; out[7] = tile_n;
      out[8] = cyc[1] - cyc[0];   // shader cycles spent in the loop
    }
  }
#endif
}

#ifdef SWARM_KERNEL_HOOKS
int g_gemm_four_waves = 1;   // measurement switch of the instrumented build (swarm_kernel_gemm_four_waves)
#endif

swarm_status launch_w4(const KArgs& k, hipStream_t st) {
  constexpr size_t stage_bytes = (size_t)NS * 512 * DBK * sizeof(bf16_raw);
  constexpr size_t lds_bytes = stage_bytes > 4 * (size_t)kW4PatchBytes ? stage_bytes : 4 * (size_t)kW4PatchBytes;
  void (*kern)(KArgs) = gemm_bf16_w4_kernel<256, 256>;
  static LdsOptIn opted;
  if (lds_opt_in((const void*)kern, lds_bytes, opted) != SWARM_OK) return SWARM_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3(k.tiles_m * k.tiles_n * (k.ksplit > 1 ? k.ksplit : 1)), dim3(256), lds_bytes, st, k);
  return launch_status();
}

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T>
swarm_status launch_dma(const KArgs& k, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)NS * (BM + BN) * DBK * sizeof(bf16_raw);
  // 256-row tiles: the 16 x 16 x 32 kernel; the 128 x 128 tile stays on 32 x 32 x 16 (measured 2 % faster there)
  void (*kern)(KArgs);
  if constexpr (BM == 256) kern = gemm_bf16_k32_kernel<BM, BN, WM, WN, A_T, B_T>;
  else kern = gemm_bf16_dma_kernel<BM, BN, WM, WN, A_T, B_T>;
  static LdsOptIn opted;   // per instantiation
  if (lds_opt_in((const void*)kern, lds_bytes, opted) != SWARM_OK) return SWARM_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3(k.tiles_m * k.tiles_n * (k.ksplit > 1 ? k.ksplit : 1)), dim3(WM * WN * 64), lds_bytes,
                     st, k);
  return launch_status();
}

template <int BM, int BN, int WM, int WN>
swarm_status launch_dma_layout(const KArgs& k, bool a_t, bool b_t, hipStream_t st) {
  if constexpr (BM == 256 && BN == 256) {
    // both operands k-contiguous and a short epilogue: four wavefronts of 128 x 128.  The epilogues with much
    // vector arithmetic (GeLU, rotary, GeGLU) stay on eight wavefronts: two per SIMD issue it twice as fast.
    bool w4 = !a_t && !b_t && w4_epilogue_ok(k.epilogue);
#ifdef SWARM_KERNEL_HOOKS
    w4 = w4 && g_gemm_four_waves;
#endif
    if (w4) return launch_w4(k, st);
  }
  if (!a_t && !b_t) return launch_dma<BM, BN, WM, WN, false, false>(k, st);
  if (!a_t && b_t) return launch_dma<BM, BN, WM, WN, false, true>(k, st);
  if (a_t && b_t) return launch_dma<BM, BN, WM, WN, true, true>(k, st);
  return SWARM_ERR_SHAPE;
}

// ---- split-K: second kernel.  C = epilogue(part_0 + part_1 + ...), summed in index order; a lane owns 8 columns.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(KArgs p) {
  const size_t chunks_per_row = (size_t)p.N / 8;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)p.M * chunks_per_row) return;         // whole lane octets leave together (N % 64 == 0)
  const size_t row = idx / chunks_per_row;
  const int col = (int)(idx % chunks_per_row) * 8;
  const size_t mn = (size_t)p.M * p.N;
  float x[8];
  {
    const float4* q = reinterpret_cast<const float4*>(p.part + row * p.N + col);
    const float4 a = q[0], b = q[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
  for (int i = 1; i < p.ksplit; ++i) {
    const float4* q = reinterpret_cast<const float4*>(p.part + i * mn + row * p.N + col);
    const float4 a = q[0], b = q[1];
    x[0] += a.x; x[1] += a.y; x[2] += a.z; x[3] += a.w; x[4] += b.x; x[5] += b.y; x[6] += b.z; x[7] += b.w;
  }
  if constexpr (EPI != EPI_STORE) {
    float bias[8];
    unpack8(*reinterpret_cast<const uint4*>(p.bias + col), bias);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] += bias[e];
  }
  if constexpr (EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_RESID_ENCODE) {
    float a[8];
    unpack8(*reinterpret_cast<const uint4*>(p.aux + row * p.ldaux + col), a);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] += a[e];
  }
  if constexpr (EPI == EPI_BIAS_RESID_ENCODE) {
    // the 8 lanes of a row segment hold one 64-element block; same arithmetic as the one-kernel epilogue
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      x[e] = bf16_bits_to_float(float_to_bf16_bits(x[e]));
      amax = fmaxf(amax, fabsf(x[e]));
    }
    amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
    const float sc = block_scale_rounded(amax / 127.0f, p.scales16);
    uint32_t w[2] = {0u, 0u};
    if (sc != 0.0f) {
      const BlockDivisor div(sc);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float q = fminf(fmaxf(rintf(div.quotient(x[e])), -127.0f), 127.0f);
        w[e >> 2] |= ((uint32_t)(int)q & 0xFFu) << (8 * (e & 3));
      }
    }
    const size_t e0 = row * p.ldc + col;
    *reinterpret_cast<uint2*>(reinterpret_cast<int8_t*>(p.C) + e0) = make_uint2(w[0], w[1]);
    if ((col & 63) == 0) block_scale_store(p.scales, e0 >> 6, sc, p.scales16);
  } else {
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_raw*>(p.C) + row * p.ldc + col) = pack8_bf16(x);
  }
}

// How many parts of K for an [M, N] output of 256 x 256 tiles: as many as keep every workgroup resident at once.
int splitk_parts_max(int M, int N) {
  if (M % 256 || N % 256) return 1;
  const long tiles = (long)(M / 256) * (N / 256);
  return tiles <= 64 ? 4 : tiles <= 128 ? 2 : 1;
}

}  // namespace

size_t gemm_splitk_floats(int M, int N) {
  const int parts = splitk_parts_max(M, N);
  return parts > 1 ? (size_t)parts * M * N : 0;
}

// Returns SWARM_ERR_SHAPE when the problem is not tile-aligned (the caller then uses the guarded kernel).
swarm_status gemm_bf16_dma(const GemmArgs& g, hipStream_t st) {
  if (g.a_trans && !g.b_trans) return SWARM_ERR_SHAPE;
  if (g.epilogue == EPI_BIAS_GEGLU && (g.a_trans || g.b_trans || g.N != 2 * g.split || g.split % 64)) return SWARM_ERR_SHAPE;
  if (g.K % DBK || g.lda % 8 || g.ldb % 8 || ((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return SWARM_ERR_SHAPE;
  KArgs k;
  k.group_m = 8;   // measured best of {2,4,8,16,32} on the d=4096 shapes
  k.A = (const bf16_raw*)g.A; k.B = (const bf16_raw*)g.B; k.M = g.M; k.N = g.N; k.K = g.K; k.lda = g.lda;
  k.ldb = g.ldb; k.C = g.C; k.ldc = g.ldc; k.epilogue = g.epilogue; k.bias = (const bf16_raw*)g.bias;
  k.aux = (const bf16_raw*)g.aux; k.ldaux = g.ldaux; k.C2 = (bf16_raw*)g.C2; k.ldc2 = g.ldc2; k.scales = g.scales; k.scales16 = g.scales16;
  k.rope = g.rope; k.rope_S = g.rope_S; k.rope_dh = g.rope_dh; k.rope_cols = g.rope_cols; k.split = g.split;
  k.ksplit = 1; k.part = nullptr; k.stamps = g.stamps;
  // An output of at least twice the 32 MB of L2 cannot wait there for its consumer; written (and its residual /
  // pre-activation / gradient rows read) non-temporally it leaves the operand panels in the L2 instead.
  k.stream = (size_t)g.M * g.N * (g.epilogue == EPI_ACCUM_F32 ? 4 : 2) >= ((size_t)64 << 20);
  // Few output tiles, long K, no transposed A (forward and dgrad products of short microbatches): the 256 x 256
  // tiles at ksplit workgroups per tile fill the chip where 128 x 128 tiles would run at their lower rate.
  // Every part keeps at least 4096 of K, which is where the second kernel's pass over the partial sums pays.
  const bool epi_ok = g.epilogue == EPI_STORE || g.epilogue == EPI_BIAS || g.epilogue == EPI_BIAS_RESID ||
                      g.epilogue == EPI_BIAS_RESID_ENCODE;
  if (g.splitk_ws && !g.a_trans && epi_ok && g.N % 64 == 0 && ((uintptr_t)g.splitk_ws & 15) == 0) {
    int parts = splitk_parts_max(g.M, g.N);
    while (parts > 1 && (g.K / parts < 4096 || g.K % (parts * DBK))) parts >>= 1;
    if (parts > 1 && g.splitk_floats >= (size_t)parts * g.M * g.N) {
      k.ksplit = parts; k.part = g.splitk_ws;
      k.tiles_m = g.M / 256; k.tiles_n = g.N / 256;
      const swarm_status s = launch_dma_layout<256, 256, 2, 4>(k, g.a_trans, g.b_trans, st);
      if (s != SWARM_OK) return s;
      const unsigned blocks = (unsigned)(((size_t)g.M * (g.N / 8) + 255) / 256);
      if (g.epilogue == EPI_STORE) hipLaunchKernelGGL(splitk_reduce_kernel<EPI_STORE>, dim3(blocks), dim3(256), 0, st, k);
      else if (g.epilogue == EPI_BIAS) hipLaunchKernelGGL(splitk_reduce_kernel<EPI_BIAS>, dim3(blocks), dim3(256), 0, st, k);
      else if (g.epilogue == EPI_BIAS_RESID)
        hipLaunchKernelGGL(splitk_reduce_kernel<EPI_BIAS_RESID>, dim3(blocks), dim3(256), 0, st, k);
      else hipLaunchKernelGGL(splitk_reduce_kernel<EPI_BIAS_RESID_ENCODE>, dim3(blocks), dim3(256), 0, st, k);
      return launch_status();
    }
  }
  // A tile count that leaves the last round of 256 workgroups at most half full (384 tiles = 1.5 rounds for the
  // QKV product of a 2048-row microbatch): the columns that make whole rounds go first, the rest is a product of
  // its own (smaller tiles or a cut along K fill the chip there).  Column-local epilogues only.
  if (!g.a_trans && g.M % 256 == 0 && g.N % 256 == 0 &&
      (g.epilogue == EPI_STORE || g.epilogue == EPI_BIAS || g.epilogue == EPI_BIAS_RESID ||
       g.epilogue == EPI_BIAS_GELU || g.epilogue == EPI_DGELU || g.epilogue == EPI_BIAS_ROPE)) {
    const long tm = g.M / 256, tn = g.N / 256, tiles = tm * tn;
    const long whole = (tiles / 256) * 256;
    if (tiles > 256 && tiles - whole > 0 && tiles - whole <= 128 && whole % tm == 0) {
      const int n1 = (int)(whole / tm) * 256;
      GemmArgs a = g, r = g;
      a.N = n1;
      r.N = g.N - n1;
      r.B = (const bf16_raw*)g.B + (g.b_trans ? (size_t)n1 : (size_t)n1 * g.ldb);
      r.C = (bf16_raw*)g.C + n1;
      if (g.bias) r.bias = (const bf16_raw*)g.bias + n1;
      if (g.aux) r.aux = (const bf16_raw*)g.aux + n1;
      if (g.C2) r.C2 = (bf16_raw*)g.C2 + n1;
      if (g.epilogue == EPI_BIAS_ROPE) {
        a.rope_cols = std::min(g.rope_cols, n1);
        r.rope_cols = g.rope_cols - n1;
        if (r.rope_cols <= 0) { r.rope_cols = 0; r.epilogue = EPI_BIAS; }
      }
      const swarm_status s = gemm_bf16_dma(a, st);
      if (s != SWARM_OK) return s;
      return gemm_bf16_dma(r, st);
    }
  }
  if (g.M % 256 == 0 && g.N % 256 == 0 && (long)(g.M / 256) * (g.N / 256) >= 160) {
    k.tiles_m = g.M / 256; k.tiles_n = g.N / 256;
    return launch_dma_layout<256, 256, 2, 4>(k, g.a_trans, g.b_trans, st);
  }
  // Too few 256 x 256 tiles, but 256 x 128 tiles make one nearly full round (a 2048-row microbatch times a
  // 4096-wide weight: 256 tiles): one round of those beats two rounds of 128 x 128.  A wavefront's sub-tile is
  // 32 columns wide there, so the epilogues that need 64 (fused encode, GeGLU) stay on the 128 x 128 tiles.
  if (!g.a_trans && g.M % 256 == 0 && g.N % 128 == 0 && g.epilogue != EPI_BIAS_RESID_ENCODE &&
      g.epilogue != EPI_BIAS_GEGLU) {
    const long tiles = (long)(g.M / 256) * (g.N / 128);
    if (tiles >= 192 && tiles <= 256) {
      k.tiles_m = g.M / 256; k.tiles_n = g.N / 128;
      return launch_dma_layout<256, 128, 2, 4>(k, g.a_trans, g.b_trans, st);
    }
  }
  if (g.M % 128 == 0 && g.N % 128 == 0) {
    k.tiles_m = g.M / 128; k.tiles_n = g.N / 128;
    return launch_dma_layout<128, 128, 2, 2>(k, g.a_trans, g.b_trans, st);
  }
  return SWARM_ERR_SHAPE;
}

}  // namespace swarm

#ifdef SWARM_KERNEL_HOOKS
// instrumented build: 0 = forward products on the eight-wavefront kernel as well (for A/B measurements)
extern "C" void swarm_kernel_gemm_four_waves(int on) { swarm::g_gemm_four_waves = on; }
#endif
