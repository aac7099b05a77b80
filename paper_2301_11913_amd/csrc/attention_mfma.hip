// Causal flash attention for bf16 on gfx950 MFMA (v_mfma_f32_32x32x16_bf16), forward and backward.
//
// Score tiles are computed TRANSPOSED where that puts the softmax row in one lane:
//   forward / dq:  S^T[kv][q] = K Q^T, so a lane owns one query column, its 16+16 kv values sit in
//                  its own registers and in lane^32: row max / row sum cost one cross-lane step, the
//                  online-softmax rescale of O^T[dh][q] is lane-local, and P^T (resp. dS^T) is already
//                  in the B-operand layout of the next MFMA (O^T = V^T P^T, dQ^T = K^T dS^T).
//   dk/dv:         S[q][kv] = Q K^T, so a lane owns one key column and P / dS are in the B-operand
//                  layout of dV^T = dO^T P and dK^T = Q^T dS.
//
// Tiles of 64 rows x d_head go from global memory straight into LDS (global_load_lds_dwordx4, two
// stages, no staging registers) in their memory layout.  A tile is read in two ways:
//   rows as MFMA rows      (contraction along d_head): one ds_read_b128 per operand block;
//   rows as the contraction (V^T, K^T, Q^T, dO^T)    : two ds_read_b64_tr_b16 (LDS transpose read),
//     whose row bases follow the accumulator's row order {4g..4g+3, 8+4g..8+4g+3}.
// One XOR swizzle of the 16-byte chunks (swz) keeps both kinds of read bank-conflict free.
// Rows past the sequence end are loaded from the last valid row; the causal mask zeroes them.
//
// Deterministic: dq and dk/dv come from two kernels that each own their output rows (no atomics).
#include "kernels.h"

namespace swarm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short i16x4;

constexpr int kThreads = 256;   // 4 wavefronts
constexpr float kLog2e = 1.4426950408889634f;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }    // vmcnt(0) only
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }  // lgkmcnt(0) only
// at most N LDS reads of this wavefront still in flight (LDS returns in order); nothing is scheduled across
template <int N>
__device__ __forceinline__ void wait_lds_reads() {
  __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
  __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& p, int base) {
  uint4 u;
  u.x = pack2(p[base + 0], p[base + 1]); u.y = pack2(p[base + 2], p[base + 3]);
  u.z = pack2(p[base + 4], p[base + 5]); u.w = pack2(p[base + 6], p[base + 7]);
  return __builtin_bit_cast(bf16x8, u);
}

// ---- 64 x DH tiles in LDS -----------------------------------------------------------------------
// chunk swizzle.  DH = 128 (256-byte rows): a 16-lane b128 pass reads 16 consecutive rows -> needs a
// bijection of row&15; a 32-lane transpose-read pass reads rows r..r+3 x four adjacent chunks ->
// bits [3:2] must separate rows r..r+3.  DH = 64 (128-byte rows): same idea with 8 chunks per row.
template <int DH>
__device__ __forceinline__ int swz(int row) {
  if constexpr (DH == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  const int x = (row >> 1) & 7;
  return ((x & 1) << 2) | (x >> 1);
}

template <int DH>
struct Tile64 {
  static constexpr int CH = DH / 8;          // 16-byte chunks per row
  static constexpr int RPI = 64 / CH;        // rows filled by one load instruction (1 KiB)
  static constexpr int NINST = CH;           // instructions per tile
  static constexpr int ELEMS = 64 * DH;

  // src = element (row 0, col 0) of the matrix; rows >= nrows are taken from row nrows-1
  static __device__ __forceinline__ void issue(const bf16_raw* __restrict__ src, int ld, int row0, int nrows,
                                               bf16_raw* lds, int wave, int lane) {
#pragma unroll
    for (int t = 0; t < NINST / 4; ++t) {
      const int q = wave + 4 * t;
      const int r = q * RPI + lane / CH;
      const int chunk = (lane % CH) ^ swz<DH>(r);
      const int grow = min(row0 + r, nrows - 1);
      __builtin_amdgcn_global_load_lds(GLB_PTR(src + (size_t)grow * ld + chunk * 8), LDS_PTR(lds + q * 512), 16, 0,
                                       0);
    }
  }
  // operand block with tile rows as MFMA rows: lane l32 -> row, 8 contraction values from chunk
  static __device__ __forceinline__ bf16x8 rows(const bf16_raw* tile, int row, int chunk) {
    return __builtin_bit_cast(bf16x8,
                              *reinterpret_cast<const uint4*>(tile + row * DH + ((chunk ^ swz<DH>(row)) << 3)));
  }
  // operand block with tile rows as the contraction: MFMA row = column cbase + (lane & 31); the 8 contraction
  // slots of lane group lg are tile rows rbase + 4*lg + {0..3} and rbase + 8 + 4*lg + {0..3}
  static __device__ __forceinline__ bf16x8 cols(const bf16_raw* tile, int cbase, int rbase, int lane) {
    const int l16 = lane & 15, grp = lane >> 4;
    const int col = cbase + 16 * (grp & 1) + 4 * (l16 & 3);
    const int r0 = rbase + 4 * (grp >> 1) + (l16 >> 2);
    const int r1 = r0 + 8;
    const bf16_raw* p0 = tile + r0 * DH + (((col >> 3) ^ swz<DH>(r0)) << 3) + (col & 4);
    const bf16_raw* p1 = tile + r1 * DH + (((col >> 3) ^ swz<DH>(r1)) << 3) + (col & 4);
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p0);
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p1);
    const uint2 a = __builtin_bit_cast(uint2, lo), b = __builtin_bit_cast(uint2, hi);
    return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
  }
  // Loop-invariant parts of the two reads above, as byte offsets inside a tile: the kernels compute them once
  // per lane before their tile loops, so that a fragment read costs one address add instead of the swizzle
  // arithmetic (which otherwise makes these kernels VALU-bound).
  static __device__ __forceinline__ uint32_t rows_off(int row, int chunk) {
    return (uint32_t)(row * DH + ((chunk ^ swz<DH>(row)) << 3)) * 2u;
  }
  static __device__ __forceinline__ bf16x8 rows_at(const bf16_raw* tile, uint32_t off) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(tile) + off));
  }
  // offsets of the two transpose reads of cols(tile, cbase, 0, lane); the swizzle of a row depends on its low four
  // bits only, so a row base that is a multiple of 16 just adds rbase * DH * 2 bytes (an immediate offset)
  static __device__ __forceinline__ void cols_off(int cbase, int lane, uint32_t& o0, uint32_t& o1) {
    const int l16 = lane & 15, grp = lane >> 4;
    const int col = cbase + 16 * (grp & 1) + 4 * (l16 & 3);
    const int r0 = 4 * (grp >> 1) + (l16 >> 2);
    const int r1 = r0 + 8;
    o0 = (uint32_t)(r0 * DH + (((col >> 3) ^ swz<DH>(r0)) << 3) + (col & 4)) * 2u;
    o1 = (uint32_t)(r1 * DH + (((col >> 3) ^ swz<DH>(r1)) << 3) + (col & 4)) * 2u;
  }
  template <int RB>
  static __device__ __forceinline__ bf16x8 cols_at_rb(uint32_t base, uint32_t o0, uint32_t o1) {
    uint2 a, b;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(a) : "v"(base + o0), "n"(RB * DH * 2) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(b) : "v"(base + o1), "n"(RB * DH * 2) : "memory");
    return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
  }
  // cols_raw(tile, cbase, rbase, lane) with rbase in {0, 16, 32, 48} and (o0, o1) = cols_off(cbase, lane)
  static __device__ __forceinline__ bf16x8 cols_at(const bf16_raw* tile, int rbase, uint32_t o0, uint32_t o1) {
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)tile;
    if (rbase == 0) return cols_at_rb<0>(base, o0, o1);
    if (rbase == 16) return cols_at_rb<16>(base, o0, o1);
    if (rbase == 32) return cols_at_rb<32>(base, o0, o1);
    return cols_at_rb<48>(base, o0, o1);
  }
  // The same block, read with plain instructions (two LDS reads).  Behind the compiler's builtin every pending
  // global -> LDS load counts as a possible writer of the bytes read and is waited for (vmcnt(0)), which would
  // serialise the next tile's loads with this tile's reads; the stages are disjoint by construction.  The
  // compiler does not count these reads: the caller waits for them itself (wait_lds_reads) before use.
  static __device__ __forceinline__ bf16x8 cols_raw(const bf16_raw* tile, int cbase, int rbase, int lane) {
    const int l16 = lane & 15, grp = lane >> 4;
    const int col = cbase + 16 * (grp & 1) + 4 * (l16 & 3);
    const int r0 = rbase + 4 * (grp >> 1) + (l16 >> 2);
    const int r1 = r0 + 8;
    const bf16_raw* p0 = tile + r0 * DH + (((col >> 3) ^ swz<DH>(r0)) << 3) + (col & 4);
    const bf16_raw* p1 = tile + r1 * DH + (((col >> 3) ^ swz<DH>(r1)) << 3) + (col & 4);
    const uint32_t a0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p0;
    const uint32_t a1 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p1;
    uint2 a, b;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(a) : "v"(a0) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(b) : "v"(a1) : "memory");
    return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
  }
};

// 8 contraction values of row `row` (columns col ..) straight from global memory, zero past nrows
__device__ __forceinline__ bf16x8 global_frag(const bf16_raw* base, int ld, int row, int nrows, int col) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < nrows) v = *reinterpret_cast<const uint4*>(base + (size_t)row * ld + col);
  return __builtin_bit_cast(bf16x8, v);
}

template <int N>
__device__ __forceinline__ void zero(f32x16 (&a)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) a[i][r] = 0.f;
}

// store a transposed accumulator (acc[i][r] = value at dh = 32i + 8(r/4) + 4lg + r%4 of this lane's row)
template <int DB>
__device__ __forceinline__ void store_rowT(bf16_raw* row, const f32x16 (&acc)[DB], float mul, int lg) {
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 v;
      v.x = pack2(acc[i][4 * g + 0] * mul, acc[i][4 * g + 1] * mul);
      v.y = pack2(acc[i][4 * g + 2] * mul, acc[i][4 * g + 3] * mul);
      *reinterpret_cast<uint2*>(row + 32 * i + 8 * g + 4 * lg) = v;
    }
}

// Workgroup -> (tile along the sequence, head, batch element) for a 1-D grid of nt * H * B workgroups.
// Consecutive workgroup ids go round-robin over the 8 XCDs; the workgroups of one (batch, head) pair all read
// the same K / V (or Q / dO) rows, so they are placed on ONE XCD (pair index mod 8), next to each other in that
// XCD's launch order: its L2 then fetches those rows once.  Inside a pair the tile index runs as given.
__device__ __forceinline__ void tile_head_batch(int nt, int H, int& tile, int& h, int& b) {
  const int id = blockIdx.x, npair = gridDim.x / nt;
  int pair, ti;
  if ((npair & 7) == 0) {
    const int j = id >> 3;
    pair = (j / nt) * 8 + (id & 7);
    ti = j % nt;
  } else {
    pair = id / nt;
    ti = id % nt;
  }
  tile = ti; h = pair % H; b = pair / H;
}

// ---- forward ------------------------------------------------------------------------------------
// grid (ceil(S/128), H, B); wavefront w owns query rows q0+32w .. q0+32w+31; KV tiles of 64.
template <int DH>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(const bf16_raw* __restrict__ qkv,
                                                               bf16_raw* __restrict__ o, float* __restrict__ lse,
                                                               int S, int H) {
  using T = Tile64<DH>;
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int STAGE = 2 * T::ELEMS;
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lg = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Causal rows get longer with the query index: a workgroup takes query tile nqt-1-pi and then tile pi, so every
  // workgroup does the same amount of work and the launch has no tail of long rows.
  const int nqt = (S + 127) / 128;
  int pi, h, b;
  tile_head_batch((nqt + 1) / 2, H, pi, h, b);
  const int d = H * DH, ld = 3 * d;
  const bf16_raw* Q = qkv + (size_t)b * S * ld + h * DH;
  const bf16_raw* K = Q + d;
  const bf16_raw* V = Q + 2 * d;
  const float c = kLog2e / sqrtf((float)DH);
  for (int pass = 0; pass < 2; ++pass) {
  const int qt = pass == 0 ? nqt - 1 - pi : pi;
  if (pass == 1 && qt == nqt - 1 - pi) break;     // odd tile count: the middle tile has no partner
  const int q0 = qt * 128;

  const int qrow = q0 + 32 * w + l32;
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = global_frag(Q, ld, qrow, S, 16 * ks + 8 * lg);

  f32x16 oacc[DB];
  zero(oacc);
  float m = -INFINITY, l = 0.f;

  const int ntile = (min(S, q0 + 128) + 63) / 64;
  auto issue = [&](int t) {
    bf16_raw* st = lds + (t & 1) * STAGE;
    T::issue(K, ld, t * 64, S, st, w, lane);
    T::issue(V, ld, t * 64, S, st + T::ELEMS, w, lane);
  };
  issue(0);
  wait_vm0();
  __builtin_amdgcn_s_barrier();

  const int wq_min = q0 + 32 * w, wq_max = wq_min + 31;
  uint32_t koff[2 * KS], voff[DB][2];      // per-lane tile offsets of the K-row and V^T fragment reads
#pragma unroll
  for (int n = 0; n < 2 * KS; ++n) koff[n] = T::rows_off(32 * (n & 1) + l32, 2 * (n >> 1) + lg);
#pragma unroll
  for (int i = 0; i < DB; ++i) T::cols_off(32 * i, lane, voff[i][0], voff[i][1]);
  for (int t = 0; t < ntile; ++t) {
    const bf16_raw* sK = lds + (t & 1) * STAGE;
    const bf16_raw* sV = sK + T::ELEMS;
    const int kv0 = t * 64;
    if (t + 1 < ntile) issue(t + 1);
    if (kv0 <= wq_max) {
      // S^T = K Q^T: NQK MFMAs, fragment n = (ks = n / 2, key block n % 2); the read of fragment n+PF sits behind
      // MFMA n, so reads run PF multiplies ahead of their use
      constexpr int NQK = 2 * KS, PF = 4, RING = 8;
      // The score MFMAs run at raised wavefront priority, the softmax and the P V MFMAs at the normal one: the two
      // wavefronts of a SIMD (from different workgroups) then fall out of step instead of both wanting the matrix
      // pipe, then both the vector unit (-5 % on this kernel at B = 4, S = 2048; the backward kernels do not react).
      __builtin_amdgcn_s_setprio(2);
      f32x16 s[2];
      zero(s);
      bf16x8 kr[RING];
#pragma unroll
      for (int n = 0; n < PF; ++n) kr[n] = T::rows_at(sK, koff[n]);
#pragma unroll
      for (int n = 0; n < NQK; ++n) {
        s[n & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[n % RING], qf[n >> 1], s[n & 1], 0, 0, 0);
        if (n + PF < NQK) {
          const int f = n + PF;
          kr[f % RING] = T::rows_at(sK, koff[f]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // O^T += V^T P^T: NPV MFMAs, fragment n = (dh block n % DB, key group n / DB); the first PF fragments of
      // V^T are requested now and arrive under the softmax arithmetic
      __builtin_amdgcn_s_setprio(0);
      constexpr int NPV = 4 * DB;
      bf16x8 vr[RING];
#pragma unroll
      for (int n = 0; n < PF; ++n) vr[n] = T::cols_at(sV, 16 * (n / DB), voff[n % DB][0], voff[n % DB][1]);
      if (kv0 + 63 > wq_min) {   // tile touches the diagonal (or the sequence end): mask kv > q
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = kv0 + 32 * kb + 8 * (r >> 2) + 4 * lg + (r & 3);
            if (kv > qrow) s[kb][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // The running maximum only has to keep exp2 in range: it is raised (and O^T, l rescaled) only when some
      // query of the wavefront exceeds its reference by more than 2^kSlack; until then p <= 2^kSlack.
      constexpr float kSlack = 8.0f;
      if (__builtin_amdgcn_ballot_w64((mx - m) * c > kSlack) != 0) {
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
        l *= alpha;
        m = m_new;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
      }
      const float mc = m * c;
      float sum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][r], c, -mc));
          s[kb][r] = p;
          sum += p;
        }
      sum += __shfl_xor(sum, 32, 64);
      l += sum;
      bf16x8 pf[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) pf[tt] = pack8(s[tt >> 1], 8 * (tt & 1));
#pragma unroll
      for (int n = 0; n < NPV; ++n) {
        // fragments n+1 .. min(n+PF, NPV)-1 may still be in flight: two reads each
        constexpr int kMaxAhead = PF - 1;
        const int ahead = (NPV - 1 - n) < kMaxAhead ? (NPV - 1 - n) : kMaxAhead;
        if (ahead == 3) wait_lds_reads<6>();
        else if (ahead == 2) wait_lds_reads<4>();
        else if (ahead == 1) wait_lds_reads<2>();
        else wait_lds_reads<0>();
        oacc[n % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[n % RING], pf[n / DB], oacc[n % DB], 0, 0, 0);
        if (n + PF < NPV) {
          const int f = n + PF;
          vr[f % RING] = T::cols_at(sV, 16 * (f / DB), voff[f % DB][0], voff[f % DB][1]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    wait_vm0();
    wait_lgkm0();
    __builtin_amdgcn_s_barrier();
  }

  if (qrow < S) {
    store_rowT<DB>(o + ((size_t)b * S + qrow) * d + h * DH, oacc, 1.0f / l, lg);
    if (lg == 0) lse[((size_t)b * H + h) * S + qrow] = m * (c / kLog2e) + logf(l);
  }
  }   // pass
}

// ---- backward -----------------------------------------------------------------------------------
// delta[b,h,s] = sum_c dO[s, h, c] * O[s, h, c].  One workgroup per token; a head's dh/8 chunks sit in
// adjacent lanes.
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_delta_kernel(const bf16_raw* __restrict__ o,
                                                              const bf16_raw* __restrict__ dout,
                                                              float* __restrict__ delta, int S, int H) {
  constexpr int LPH = DH / 8;   // lanes per head
  const int token = blockIdx.x;
  const int b = token / S, sidx = token % S;
  const int d = H * DH;
  for (int ch = threadIdx.x; ch < d / 8; ch += kThreads) {   // d/8 is a multiple of LPH, so whole heads stay together
    const uint4 a = *reinterpret_cast<const uint4*>(o + (size_t)token * d + ch * 8);
    const uint4 g = *reinterpret_cast<const uint4*>(dout + (size_t)token * d + ch * 8);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, gw[4] = {g.x, g.y, g.z, g.w};
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc = fmaf(__uint_as_float(aw[i] << 16), __uint_as_float(gw[i] << 16), acc);
      acc = fmaf(__uint_as_float(aw[i] & 0xFFFF0000u), __uint_as_float(gw[i] & 0xFFFF0000u), acc);
    }
#pragma unroll
    for (int msk = LPH / 2; msk >= 1; msk >>= 1) acc += __shfl_xor(acc, msk, 64);
    if ((ch % LPH) == 0) delta[((size_t)b * H + ch / LPH) * S + sidx] = acc;
  }
}

// dK, dV: grid (ceil(S/128), H, B), 8 wavefronts.  Wavefronts w and w+4 both own key rows kv0+32w..+31;
// the first computes dV (S -> P, dV^T += dO^T P), the second dK (S, dP -> dS, dK^T += Q^T dS), so each holds
// one 32 x d_head accumulator and two wavefronts fit a SIMD.  Both read the same Q / dO tiles of 64 queries.
constexpr int kDkDvThreads = 512;
template <int DH>
__global__ __launch_bounds__(kDkDvThreads) void attn_bwd_dkdv_kernel(const bf16_raw* __restrict__ qkv,
                                                                     const bf16_raw* __restrict__ dout,
                                                                     const float* __restrict__ lse,
                                                                     const float* __restrict__ delta,
                                                                     bf16_raw* __restrict__ dqkv, int S, int H) {
  using T = Tile64<DH>;
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int STAGE = 2 * T::ELEMS + 256;     // Q, dO + (lse, delta) as 2 x 64 floats
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lg = lane >> 5;
  const int w8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int w = w8 & 3;
  const bool is_dk = w8 >= 4;
  // key block pi (the longest sweep over the query tiles), then its partner nkb-1-pi: equal work per workgroup
  const int nkb = (S + 127) / 128;
  int pi, h, b;
  tile_head_batch((nkb + 1) / 2, H, pi, h, b);
  for (int pass = 0; pass < 2; ++pass) {
  const int kb = pass == 0 ? pi : nkb - 1 - pi;
  if (pass == 1 && kb == pi) break;
  const int d = H * DH, ld = 3 * d;
  const bf16_raw* Q = qkv + (size_t)b * S * ld + h * DH;
  const bf16_raw* K = Q + d;
  const bf16_raw* V = Q + 2 * d;
  const bf16_raw* dO = dout + (size_t)b * S * d + h * DH;
  const float* lse_r = lse + ((size_t)b * H + h) * S;
  const float* del_r = delta + ((size_t)b * H + h) * S;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = kLog2e * scale;

  const int kvrow = kb * 128 + 32 * w + l32;
  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = global_frag(K, ld, kvrow, S, 16 * ks + 8 * lg);
    vf[ks] = is_dk ? global_frag(V, ld, kvrow, S, 16 * ks + 8 * lg) : kf[ks];
  }
  f32x16 acc[DB];     // dV^T or dK^T
  zero(acc);

  const int t_begin = (kb * 128) / 64, t_end = (S + 63) / 64;
  auto issue = [&](int t) {
    bf16_raw* st = lds + ((t - t_begin) & 1) * STAGE;
    if (!is_dk) T::issue(Q, ld, t * 64, S, st, w, lane);
    else T::issue(dO, d, t * 64, S, st + T::ELEMS, w, lane);
    if (w == 0) {   // wavefront 0: lse of the tile's 64 rows, wavefront 4: delta
      const int row = min(t * 64 + lane, S - 1);
      __builtin_amdgcn_global_load_lds(GLB_PTR((is_dk ? del_r : lse_r) + row),
                                       LDS_PTR(st + 2 * T::ELEMS + (is_dk ? 128 : 0)), 4, 0, 0);
    }
  };
  issue(t_begin);
  wait_vm0();
  __builtin_amdgcn_s_barrier();

  const int wkv_min = kb * 128 + 32 * w;
  for (int t = t_begin; t < t_end; ++t) {
    const bf16_raw* sQ = lds + ((t - t_begin) & 1) * STAGE;
    const bf16_raw* sdO = sQ + T::ELEMS;
    const float* sstat = reinterpret_cast<const float*>(sQ + 2 * T::ELEMS);
    const int q0 = t * 64;
    if (t + 1 < t_end) issue(t + 1);
    if (q0 + 63 >= wkv_min) {
      const bool diag = q0 < wkv_min + 32;   // some q in the tile is below some kv of this wavefront
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        // S = Q K^T (both roles) and dP = dO V^T (dK role): fragment reads run PF MFMAs ahead of their use.
        // dV role: N1 = KS fragments of Q rows; dK role: 2 KS fragments, Q rows (even) and dO rows (odd).
        constexpr int PF = 3, RING = 4;
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
        bf16x8 fr[RING];
        if (is_dk) {
          constexpr int N1 = 2 * KS;
          auto frag1 = [&](int n) { return T::rows((n & 1) ? sdO : sQ, 32 * qb + l32, 2 * (n >> 1) + lg); };
#pragma unroll
          for (int n = 0; n < PF; ++n) fr[n] = frag1(n);
#pragma unroll
          for (int n = 0; n < N1; ++n) {
            if (n & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % RING], vf[n >> 1], dp, 0, 0, 0);
            else s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % RING], kf[n >> 1], s, 0, 0, 0);
            if (n + PF < N1) fr[(n + PF) % RING] = frag1(n + PF);
            __builtin_amdgcn_sched_barrier(0);
          }
        } else {
          constexpr int N1 = KS;
          auto frag1 = [&](int n) { return T::rows(sQ, 32 * qb + l32, 2 * n + lg); };
#pragma unroll
          for (int n = 0; n < PF; ++n) fr[n] = frag1(n);
#pragma unroll
          for (int n = 0; n < N1; ++n) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % RING], kf[n], s, 0, 0, 0);
            if (n + PF < N1) fr[(n + PF) % RING] = frag1(n + PF);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // dK^T += Q^T dS resp. dV^T += dO^T P: N2 MFMAs, fragment n = (dh block n % DB, query group n / DB); the
        // first PF fragments are requested now and arrive under the softmax arithmetic
        constexpr int N2 = 2 * DB;
        const bf16_raw* src = is_dk ? sQ : sdO;
        bf16x8 ct[RING];
        auto frag2 = [&](int n) { return T::cols_raw(src, 32 * (n % DB), 32 * qb + 16 * (n / DB), lane); };
#pragma unroll
        for (int n = 0; n < PF; ++n) ct[n] = frag2(n);
        // (the row statistics below are ordinary LDS loads issued AFTER those transpose reads: LDS returns in
        // order, so whatever count the compiler waits for before using them only over-waits)
        {
          // p = 0 for queries before this lane's key (diagonal tiles only) and past the sequence end: one unsigned
          // comparison of q - lo against S - lo, with lo = the lane's key on a diagonal tile and 0 elsewhere.
          // The row statistics are read four queries at a time, right where they are used (few live registers).
          const int lo = diag ? kvrow : 0;
          const uint32_t span = (uint32_t)(S - lo);
          const int qrel = q0 + 32 * qb + 4 * lg - lo;
          if (is_dk) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int rbase = 32 * qb + 8 * g + 4 * lg;
              const float4 L = *reinterpret_cast<const float4*>(sstat + rbase);
              const float4 D = *reinterpret_cast<const float4*>(sstat + 64 + rbase);
              const float Lg[4] = {L.x, L.y, L.z, L.w}, Dg[4] = {D.x, D.y, D.z, D.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const int r = 4 * g + e;
                float p = __builtin_amdgcn_exp2f(fmaf(s[r], c, -Lg[e] * kLog2e));
                if ((uint32_t)(qrel + 8 * g + e) >= span) p = 0.f;
                s[r] = p * (dp[r] - Dg[e]);                        // dS
              }
              if constexpr (DH == 128) __builtin_amdgcn_sched_barrier(0);
            }
          } else {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const float4 L = *reinterpret_cast<const float4*>(sstat + 32 * qb + 8 * g + 4 * lg);
              const float Lg[4] = {L.x, L.y, L.z, L.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const int r = 4 * g + e;
                const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c, -Lg[e] * kLog2e));
                s[r] = (uint32_t)(qrel + 8 * g + e) >= span ? 0.f : p;   // P
              }
              if constexpr (DH == 128) __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        bf16x8 bf[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) bf[tt] = pack8(s, 8 * tt);
#pragma unroll
        for (int n = 0; n < N2; ++n) {
          // fragments n+1 .. min(n+PF, N2)-1 may still be in flight: two reads each
          const int ahead = (N2 - 1 - n) < (PF - 1) ? (N2 - 1 - n) : (PF - 1);
          if (ahead == 2) wait_lds_reads<4>();
          else if (ahead == 1) wait_lds_reads<2>();
          else wait_lds_reads<0>();
          acc[n % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ct[n % RING], bf[n / DB], acc[n % DB], 0, 0, 0);
          if (n + PF < N2) ct[(n + PF) % RING] = frag2(n + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    wait_vm0();
    wait_lgkm0();
    __builtin_amdgcn_s_barrier();
  }

  if (kvrow < S) {
    bf16_raw* dkrow = dqkv + ((size_t)b * S + kvrow) * ld + d + h * DH;
    if (is_dk) store_rowT<DB>(dkrow, acc, scale, lg);
    else store_rowT<DB>(dkrow + d, acc, 1.0f, lg);
  }
  }   // pass
}

// dQ: grid (ceil(S/128), H, B); wavefront w owns query rows q0+32w..+31; KV tiles of 64.
template <int DH>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(const bf16_raw* __restrict__ qkv,
                                                                  const bf16_raw* __restrict__ dout,
                                                                  const float* __restrict__ lse,
                                                                  const float* __restrict__ delta,
                                                                  bf16_raw* __restrict__ dqkv, int S, int H) {
  using T = Tile64<DH>;
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int STAGE = 2 * T::ELEMS;           // K, V
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lg = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqt = (S + 127) / 128;
  int pi, h, b;
  tile_head_batch((nqt + 1) / 2, H, pi, h, b);
  const int d = H * DH, ld = 3 * d;
  for (int pass = 0; pass < 2; ++pass) {          // query tile nqt-1-pi, then its partner pi (equal work per workgroup)
  const int qtile = pass == 0 ? nqt - 1 - pi : pi;
  if (pass == 1 && qtile == nqt - 1 - pi) break;
  const int q0 = qtile * 128;
  const bf16_raw* Q = qkv + (size_t)b * S * ld + h * DH;
  const bf16_raw* K = Q + d;
  const bf16_raw* V = Q + 2 * d;
  const bf16_raw* dO = dout + (size_t)b * S * d + h * DH;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = kLog2e * scale;

  const int qrow = q0 + 32 * w + l32;
  bf16x8 qf[KS], dof[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = global_frag(Q, ld, qrow, S, 16 * ks + 8 * lg);
    dof[ks] = global_frag(dO, d, qrow, S, 16 * ks + 8 * lg);
  }
  float L2 = 0.f, dl = 0.f;
  if (qrow < S) {
    L2 = lse[((size_t)b * H + h) * S + qrow] * kLog2e;
    dl = delta[((size_t)b * H + h) * S + qrow];
  }
  f32x16 dqacc[DB];
  zero(dqacc);

  const int ntile = (min(S, q0 + 128) + 63) / 64;
  auto issue = [&](int t) {
    bf16_raw* st = lds + (t & 1) * STAGE;
    T::issue(K, ld, t * 64, S, st, w, lane);
    T::issue(V, ld, t * 64, S, st + T::ELEMS, w, lane);
  };
  issue(0);
  wait_vm0();
  __builtin_amdgcn_s_barrier();

  const int wq_min = q0 + 32 * w, wq_max = wq_min + 31;
  for (int t = 0; t < ntile; ++t) {
    const bf16_raw* sK = lds + (t & 1) * STAGE;
    const bf16_raw* sV = sK + T::ELEMS;
    const int kv0 = t * 64;
    if (t + 1 < ntile) issue(t + 1);
    if (kv0 <= wq_max) {
      const bool diag = kv0 + 63 > wq_min;
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2) {
        // S^T = K Q^T and dP^T = V dO^T: N1 MFMAs, fragment n = (ks = n / 2; n even: K rows, n odd: V rows);
        // the read of fragment n+PF sits behind MFMA n
        constexpr int N1 = 2 * KS, PF = 3, RING = 4;
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
        bf16x8 fr[RING];
        auto frag1 = [&](int n) { return T::rows((n & 1) ? sV : sK, 32 * kb2 + l32, 2 * (n >> 1) + lg); };
#pragma unroll
        for (int n = 0; n < PF; ++n) fr[n] = frag1(n);
#pragma unroll
        for (int n = 0; n < N1; ++n) {
          if (n & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % RING], dof[n >> 1], dp, 0, 0, 0);
          else s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % RING], qf[n >> 1], s, 0, 0, 0);
          if (n + PF < N1) fr[(n + PF) % RING] = frag1(n + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
        // dQ^T += K^T dS^T: N2 MFMAs, fragment n = (dh block n % DB, key group n / DB); the first PF fragments of
        // K^T are requested now and arrive under the softmax-gradient arithmetic
        constexpr int N2 = 2 * DB;
        bf16x8 kt[RING];
        auto frag2 = [&](int n) { return T::cols_raw(sK, 32 * (n % DB), 32 * kb2 + 16 * (n / DB), lane); };
#pragma unroll
        for (int n = 0; n < PF; ++n) kt[n] = frag2(n);
        if (diag) {   // only a tile on the diagonal (or past the sequence end) has keys to mask
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float p = __builtin_amdgcn_exp2f(fmaf(s[r], c, -L2));
            const int kv = kv0 + 32 * kb2 + 8 * (r >> 2) + 4 * lg + (r & 3);
            if (kv > qrow) p = 0.f;
            dp[r] = p * (dp[r] - dl);
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) dp[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c, -L2)) * (dp[r] - dl);
        }
        bf16x8 dsf[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) dsf[tt] = pack8(dp, 8 * tt);
#pragma unroll
        for (int n = 0; n < N2; ++n) {
          // fragments n+1 .. min(n+PF, N2)-1 may still be in flight: two reads each
          const int ahead = (N2 - 1 - n) < (PF - 1) ? (N2 - 1 - n) : (PF - 1);
          if (ahead == 2) wait_lds_reads<4>();
          else if (ahead == 1) wait_lds_reads<2>();
          else wait_lds_reads<0>();
          dqacc[n % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt[n % RING], dsf[n / DB], dqacc[n % DB], 0, 0, 0);
          if (n + PF < N2) kt[(n + PF) % RING] = frag2(n + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    wait_vm0();
    wait_lgkm0();
    __builtin_amdgcn_s_barrier();
  }

  if (qrow < S) store_rowT<DB>(dqkv + ((size_t)b * S + qrow) * ld + h * DH, dqacc, scale, lg);
  }   // pass
}

template <int DH>
swarm_status launch_fwd(const bf16_raw* qkv, bf16_raw* o, float* lse, int B, int S, int H, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)2 * 2 * 64 * DH * sizeof(bf16_raw);
  static LdsOptIn a0;
  if (lds_opt_in((const void*)attn_fwd_kernel<DH>, lds_bytes, a0) != SWARM_OK) return SWARM_ERR_LAUNCH;
  hipLaunchKernelGGL(attn_fwd_kernel<DH>, dim3((((S + 127) / 128 + 1) / 2) * H * B), dim3(kThreads), lds_bytes, st,
                     qkv, o, lse, S, H);
  return launch_status();
}

template <int DH>
swarm_status launch_bwd(const bf16_raw* qkv, const bf16_raw* o, const bf16_raw* dout, const float* lse, float* delta,
                        bf16_raw* dqkv, int B, int S, int H, hipStream_t st) {
  constexpr size_t lds_dkdv = (size_t)2 * (2 * 64 * DH + 256) * sizeof(bf16_raw);
  constexpr size_t lds_dq = (size_t)2 * 2 * 64 * DH * sizeof(bf16_raw);
  static LdsOptIn a1, a2;
  if (lds_opt_in((const void*)attn_bwd_dkdv_kernel<DH>, lds_dkdv, a1) != SWARM_OK) return SWARM_ERR_LAUNCH;
  if (lds_opt_in((const void*)attn_bwd_dq_kernel<DH>, lds_dq, a2) != SWARM_OK) return SWARM_ERR_LAUNCH;
  hipLaunchKernelGGL(attn_delta_kernel<DH>, dim3(B * S), dim3(kThreads), 0, st, o, dout, delta, S, H);
  dim3 grid((((S + 127) / 128 + 1) / 2) * H * B);   // workgroups take pairs of tiles
  hipLaunchKernelGGL(attn_bwd_dkdv_kernel<DH>, grid, dim3(kDkDvThreads), lds_dkdv, st, qkv, dout, lse, delta, dqkv, S,
                     H);
  hipLaunchKernelGGL(attn_bwd_dq_kernel<DH>, grid, dim3(kThreads), lds_dq, st, qkv, dout, lse, delta, dqkv, S, H);
  return launch_status();
}

}  // namespace

swarm_status attention_fwd_mfma(const void* qkv, void* o, float* lse, int B, int S, int H, int dh, hipStream_t st) {
  if (dh == 128) return launch_fwd<128>((const bf16_raw*)qkv, (bf16_raw*)o, lse, B, S, H, st);
  if (dh == 64) return launch_fwd<64>((const bf16_raw*)qkv, (bf16_raw*)o, lse, B, S, H, st);
  return SWARM_ERR_SHAPE;
}

swarm_status attention_bwd_mfma(const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                                void* dqkv, int B, int S, int H, int dh, hipStream_t st) {
  if (dh == 128)
    return launch_bwd<128>((const bf16_raw*)qkv, (const bf16_raw*)o, (const bf16_raw*)dout, lse, delta,
                           (bf16_raw*)dqkv, B, S, H, st);
  if (dh == 64)
    return launch_bwd<64>((const bf16_raw*)qkv, (const bf16_raw*)o, (const bf16_raw*)dout, lse, delta,
                          (bf16_raw*)dqkv, B, S, H, st);
  return SWARM_ERR_SHAPE;
}

}  // namespace swarm
