// Causal flash attention for bf16 on gfx950 MFMA (v_mfma_f32_32x32x16_bf16), forward and backward.
//
// All kernels compute score tiles TRANSPOSED where that puts the softmax row in one lane:
//   forward / dq:  S^T[kv][q] = K Q^T, so a lane owns one query column, its 16+16 kv values sit in
//                  its own registers and in lane^32: row max / row sum cost one cross-lane step, the
//                  online-softmax rescale of O^T[dh][q] is lane-local, and P^T (resp. dS^T) is already
//                  in the B-operand layout of the next MFMA (O^T = V^T P^T, dQ^T = K^T dS^T).
//   dk/dv:         S[q][kv] = Q K^T, so a lane owns one key column and P / dS are in the B-operand
//                  layout of dV^T = dO^T P and dK^T = Q^T dS.
// The operand that must be read along the contraction index (V^T, K^T, Q^T, dO^T) is transposed in
// registers on its way into LDS (8 x 4 patches, 8-byte global loads, 16-byte LDS rows); the 8 slots
// of a 16-byte LDS row follow the accumulator's row order {4g..4g+3, 8+4g..8+4g+3}, so one 16-byte
// LDS read feeds one MFMA.
//
// Deterministic: dq and dk/dv come from two kernels that each own their output rows (no atomics).
#include "kernels.h"

namespace swarm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 256;   // 4 wavefronts
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ int swz8(int row) { return (row & 7) ^ ((row >> 3) & 1); }

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

__device__ __forceinline__ bf16x8 lds_frag(const bf16_raw* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

// ---- tile movers ------------------------------------------------------------------------------
// Row-major tile [ROWS][DH] (contraction along DH): 16-byte chunks, chunk index XOR (row & 7).
template <int ROWS, int DH>
struct RowTile {
  static constexpr int CH = DH / 8;
  static constexpr int NI = ROWS * CH / kThreads;
  uint4 r[NI];
  // src points at element (row 0, col 0) of the tile's matrix; row pitch ld; rows >= nrows read as zero
  __device__ __forceinline__ void load(const bf16_raw* __restrict__ src, int ld, int row0, int nrows, int tid) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int it = tid + i * kThreads;
      const int row = it / CH, chunk = it % CH;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row0 + row < nrows) v = *reinterpret_cast<const uint4*>(src + (size_t)(row0 + row) * ld + chunk * 8);
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store(bf16_raw* __restrict__ lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int it = tid + i * kThreads;
      const int row = it / CH, chunk = it % CH;
      *reinterpret_cast<uint4*>(lds + row * DH + ((chunk ^ (row & 7)) << 3)) = r[i];
    }
  }
  static __device__ __forceinline__ int frag_off(int row, int chunk) {
    return row * DH + ((chunk ^ (row & 7)) << 3);
  }
};

// Transposed tile: memory [64 rows (contraction index)][DH]  ->  LDS [DH][64], where 16-byte chunk
// c = 2t+g of an LDS row holds contraction rows {16t+4g..+3, 16t+8+4g..+3} (accumulator row order).
template <int DH>
struct TransTile {
  static constexpr int NP = 8 * (DH / 4);                 // patches
  static constexpr int NI = (NP + kThreads - 1) / kThreads;
  uint2 r[NI][8];
  __device__ __forceinline__ void load(const bf16_raw* __restrict__ src, int ld, int row0, int nrows, int tid) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int it = tid + i * kThreads;
      const int dc = it % (DH / 4), c = it / (DH / 4);
      const int base = 16 * (c >> 1) + 4 * (c & 1);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = row0 + base + (j < 4 ? j : j + 4);
        uint2 v = make_uint2(0, 0);
        if (it < NP && row < nrows) v = *reinterpret_cast<const uint2*>(src + (size_t)row * ld + dc * 4);
        r[i][j] = v;
      }
    }
  }
  __device__ __forceinline__ void store(bf16_raw* __restrict__ lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int it = tid + i * kThreads;
      if (it >= NP) continue;
      const int dc = it % (DH / 4), c = it / (DH / 4);
      const uint2* q = r[i];
      uint4 o0, o1, o2, o3;
      o0.x = __builtin_amdgcn_perm(q[1].x, q[0].x, 0x05040100u); o1.x = __builtin_amdgcn_perm(q[1].x, q[0].x, 0x07060302u);
      o0.y = __builtin_amdgcn_perm(q[3].x, q[2].x, 0x05040100u); o1.y = __builtin_amdgcn_perm(q[3].x, q[2].x, 0x07060302u);
      o0.z = __builtin_amdgcn_perm(q[5].x, q[4].x, 0x05040100u); o1.z = __builtin_amdgcn_perm(q[5].x, q[4].x, 0x07060302u);
      o0.w = __builtin_amdgcn_perm(q[7].x, q[6].x, 0x05040100u); o1.w = __builtin_amdgcn_perm(q[7].x, q[6].x, 0x07060302u);
      o2.x = __builtin_amdgcn_perm(q[1].y, q[0].y, 0x05040100u); o3.x = __builtin_amdgcn_perm(q[1].y, q[0].y, 0x07060302u);
      o2.y = __builtin_amdgcn_perm(q[3].y, q[2].y, 0x05040100u); o3.y = __builtin_amdgcn_perm(q[3].y, q[2].y, 0x07060302u);
      o2.z = __builtin_amdgcn_perm(q[5].y, q[4].y, 0x05040100u); o3.z = __builtin_amdgcn_perm(q[5].y, q[4].y, 0x07060302u);
      o2.w = __builtin_amdgcn_perm(q[7].y, q[6].y, 0x05040100u); o3.w = __builtin_amdgcn_perm(q[7].y, q[6].y, 0x07060302u);
      const int row = dc * 4;
      *reinterpret_cast<uint4*>(lds + frag_off(row + 0, c)) = o0;
      *reinterpret_cast<uint4*>(lds + frag_off(row + 1, c)) = o1;
      *reinterpret_cast<uint4*>(lds + frag_off(row + 2, c)) = o2;
      *reinterpret_cast<uint4*>(lds + frag_off(row + 3, c)) = o3;
    }
  }
  static __device__ __forceinline__ int frag_off(int row, int chunk) {
    return row * 64 + ((chunk ^ swz8(row)) << 3);
  }
};

// ---- forward ------------------------------------------------------------------------------------
// grid (ceil(S/128), H, B); wavefront w owns query rows q0+32w .. q0+32w+31; KV tiles of 64.
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(const bf16_raw* __restrict__ qkv,
                                                            bf16_raw* __restrict__ o, float* __restrict__ lse,
                                                            int S, int H) {
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int STAGE = 2 * 64 * DH;
  extern __shared__ __attribute__((aligned(16))) bf16_raw lds[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lg = lane >> 5;
  const int qt = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = H * DH, ld = 3 * d;
  const int q0 = qt * 128;
  const bf16_raw* Q = qkv + (size_t)b * S * ld + h * DH;
  const bf16_raw* K = Q + d;
  const bf16_raw* V = Q + 2 * d;
  const float c = kLog2e / sqrtf((float)DH);

  const int qrow = q0 + 32 * w + l32;
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (qrow < S) v = *reinterpret_cast<const uint4*>(Q + (size_t)qrow * ld + 16 * ks + 8 * lg);
    qf[ks] = __builtin_bit_cast(bf16x8, v);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int kv_end = min(S, q0 + 128);
  const int ntile = (kv_end + 63) / 64;
  RowTile<64, DH> kt;
  TransTile<DH> vt;
  kt.load(K, ld, 0, S, tid);
  vt.load(V, ld, 0, S, tid);
  kt.store(lds, tid);
  vt.store(lds + 64 * DH, tid);
  __syncthreads();

  const int wq_min = q0 + 32 * w, wq_max = wq_min + 31;
  for (int t = 0; t < ntile; ++t) {
    const bf16_raw* sK = lds + (t & 1) * STAGE;
    const bf16_raw* sV = sK + 64 * DH;
    const int kv0 = t * 64;
    const bool more = t + 1 < ntile;
    if (more) {
      kt.load(K, ld, kv0 + 64, S, tid);
      vt.load(V, ld, kv0 + 64, S, tid);
    }
    if (kv0 <= wq_max) {
      f32x16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 a = lds_frag(sK + RowTile<64, DH>::frag_off(32 * kb + l32, 2 * ks + lg));
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
        }
      }
      if (kv0 + 63 > wq_min) {   // tile touches the diagonal: mask kv > q
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
      const float m_new = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
      const float mc = m_new * c;
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
      l = l * alpha + sum;
      m = m_new;
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
      bf16x8 pf[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) pf[tt] = pack8(s[tt >> 1], 8 * (tt & 1));
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const bf16x8 a = lds_frag(sV + TransTile<DH>::frag_off(32 * i + l32, 2 * tt + lg));
          oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[tt], oacc[i], 0, 0, 0);
        }
    }
    if (more) {
      bf16_raw* dK = lds + ((t + 1) & 1) * STAGE;
      kt.store(dK, tid);
      vt.store(dK + 64 * DH, tid);
    }
    __syncthreads();
  }

  if (qrow < S) {
    const float inv = 1.0f / l;
    bf16_raw* orow = o + ((size_t)b * S + qrow) * d + h * DH;
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack2(oacc[i][4 * g + 0] * inv, oacc[i][4 * g + 1] * inv);
        v.y = pack2(oacc[i][4 * g + 2] * inv, oacc[i][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(orow + 32 * i + 8 * g + 4 * lg) = v;
      }
    if (lg == 0) lse[((size_t)b * H + h) * S + qrow] = m * (c / kLog2e) + logf(l);
  }
}

template <int DH>
swarm_status launch_fwd(const bf16_raw* qkv, bf16_raw* o, float* lse, int B, int S, int H, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)2 * 2 * 64 * DH * sizeof(bf16_raw);
  auto kern = attn_fwd_kernel<DH>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) !=
        hipSuccess)
      return SWARM_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((S + 127) / 128, H, B), dim3(kThreads), lds_bytes, st, qkv, o, lse, S, H);
  return launch_status();
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

// dK, dV: grid (ceil(S/128), H, B); wavefront w owns key rows kv0+32w..+31; query tiles of 64.
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_bwd_dkdv_kernel(const bf16_raw* __restrict__ qkv,
                                                                 const bf16_raw* __restrict__ dout,
                                                                 const float* __restrict__ lse,
                                                                 const float* __restrict__ delta,
                                                                 bf16_raw* __restrict__ dqkv, int S, int H) {
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int TILE = 64 * DH;                 // elements of one 64-row tile
  constexpr int STAGE = 4 * TILE + 256;         // Q, Q^T, dO, dO^T + (lse, delta) as 2 x 64 floats
  extern __shared__ __attribute__((aligned(16))) bf16_raw lds[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lg = lane >> 5;
  const int kb = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
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
    uint4 a = make_uint4(0, 0, 0, 0), v = make_uint4(0, 0, 0, 0);
    if (kvrow < S) {
      a = *reinterpret_cast<const uint4*>(K + (size_t)kvrow * ld + 16 * ks + 8 * lg);
      v = *reinterpret_cast<const uint4*>(V + (size_t)kvrow * ld + 16 * ks + 8 * lg);
    }
    kf[ks] = __builtin_bit_cast(bf16x8, a);
    vf[ks] = __builtin_bit_cast(bf16x8, v);
  }
  f32x16 dvacc[DB], dkacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dvacc[i][r] = 0.f; dkacc[i][r] = 0.f; }

  const int t_begin = (kb * 128) / 64, t_end = (S + 63) / 64;
  RowTile<64, DH> qt, dot;
  TransTile<DH> qtt, dott;
  float stat = 0.f;   // threads 0..63: lse of row tid; 64..127: delta of row tid-64
  auto load_tile = [&](int q0) {
    qt.load(Q, ld, q0, S, tid);
    qtt.load(Q, ld, q0, S, tid);
    dot.load(dO, d, q0, S, tid);
    dott.load(dO, d, q0, S, tid);
    if (tid < 128) {
      const int row = q0 + (tid & 63);
      stat = row < S ? (tid < 64 ? lse_r[row] : del_r[row]) : 0.f;
    }
  };
  auto store_tile = [&](bf16_raw* st) {
    qt.store(st, tid);
    qtt.store(st + TILE, tid);
    dot.store(st + 2 * TILE, tid);
    dott.store(st + 3 * TILE, tid);
    if (tid < 128) reinterpret_cast<float*>(st + 4 * TILE)[tid] = stat;
  };
  load_tile(t_begin * 64);
  store_tile(lds);
  __syncthreads();

  const int wkv_min = kb * 128 + 32 * w;
  for (int t = t_begin; t < t_end; ++t) {
    const bf16_raw* sQ = lds + ((t - t_begin) & 1) * STAGE;
    const bf16_raw* sQt = sQ + TILE;
    const bf16_raw* sdO = sQ + 2 * TILE;
    const bf16_raw* sdOt = sQ + 3 * TILE;
    const float* sstat = reinterpret_cast<const float*>(sQ + 4 * TILE);
    const int q0 = t * 64;
    const bool more = t + 1 < t_end;
    if (more) load_tile(q0 + 64);
    if (q0 + 63 >= wkv_min) {
      f32x16 s[2], dp[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[qb][r] = 0.f; dp[qb][r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const bf16x8 a = lds_frag(sQ + RowTile<64, DH>::frag_off(32 * qb + l32, 2 * ks + lg));
          s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[ks], s[qb], 0, 0, 0);
          const bf16x8 g = lds_frag(sdO + RowTile<64, DH>::frag_off(32 * qb + l32, 2 * ks + lg));
          dp[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(g, vf[ks], dp[qb], 0, 0, 0);
        }
      const bool diag = q0 < wkv_min + 32;   // some q in the tile is below some kv of this wavefront
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int rbase = 32 * qb + 8 * g + 4 * lg;
          const float4 L = *reinterpret_cast<const float4*>(sstat + rbase);
          const float4 D = *reinterpret_cast<const float4*>(sstat + 64 + rbase);
          const float Ls[4] = {L.x, L.y, L.z, L.w}, Ds[4] = {D.x, D.y, D.z, D.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * g + e;
            float p = __builtin_amdgcn_exp2f(fmaf(s[qb][r], c, -Ls[e] * kLog2e));
            const int q = q0 + rbase + e;
            if ((diag && kvrow > q) || q >= S) p = 0.f;
            s[qb][r] = p;
            dp[qb][r] = p * (dp[qb][r] - Ds[e]);
          }
        }
      bf16x8 pf[4], dsf[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        pf[tt] = pack8(s[tt >> 1], 8 * (tt & 1));
        dsf[tt] = pack8(dp[tt >> 1], 8 * (tt & 1));
      }
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const bf16x8 a = lds_frag(sdOt + TransTile<DH>::frag_off(32 * i + l32, 2 * tt + lg));
          dvacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[tt], dvacc[i], 0, 0, 0);
          const bf16x8 a2 = lds_frag(sQt + TransTile<DH>::frag_off(32 * i + l32, 2 * tt + lg));
          dkacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, dsf[tt], dkacc[i], 0, 0, 0);
        }
    }
    if (more) store_tile(lds + ((t + 1 - t_begin) & 1) * STAGE);
    __syncthreads();
  }

  if (kvrow < S) {
    bf16_raw* dkrow = dqkv + ((size_t)b * S + kvrow) * ld + d + h * DH;
    bf16_raw* dvrow = dkrow + d;
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack2(dkacc[i][4 * g + 0] * scale, dkacc[i][4 * g + 1] * scale);
        v.y = pack2(dkacc[i][4 * g + 2] * scale, dkacc[i][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(dkrow + 32 * i + 8 * g + 4 * lg) = v;
        v.x = pack2(dvacc[i][4 * g + 0], dvacc[i][4 * g + 1]);
        v.y = pack2(dvacc[i][4 * g + 2], dvacc[i][4 * g + 3]);
        *reinterpret_cast<uint2*>(dvrow + 32 * i + 8 * g + 4 * lg) = v;
      }
  }
}

// dQ: grid (ceil(S/128), H, B); wavefront w owns query rows q0+32w..+31; KV tiles of 64.
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_bwd_dq_kernel(const bf16_raw* __restrict__ qkv,
                                                               const bf16_raw* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta,
                                                               bf16_raw* __restrict__ dqkv, int S, int H) {
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int TILE = 64 * DH;
  constexpr int STAGE = 3 * TILE;               // K, V, K^T
  extern __shared__ __attribute__((aligned(16))) bf16_raw lds[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lg = lane >> 5;
  const int qtile = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = H * DH, ld = 3 * d;
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
    uint4 a = make_uint4(0, 0, 0, 0), g = make_uint4(0, 0, 0, 0);
    if (qrow < S) {
      a = *reinterpret_cast<const uint4*>(Q + (size_t)qrow * ld + 16 * ks + 8 * lg);
      g = *reinterpret_cast<const uint4*>(dO + (size_t)qrow * d + 16 * ks + 8 * lg);
    }
    qf[ks] = __builtin_bit_cast(bf16x8, a);
    dof[ks] = __builtin_bit_cast(bf16x8, g);
  }
  float L2 = 0.f, dl = 0.f;
  if (qrow < S) {
    L2 = lse[((size_t)b * H + h) * S + qrow] * kLog2e;
    dl = delta[((size_t)b * H + h) * S + qrow];
  }
  f32x16 dqacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[i][r] = 0.f;

  const int kv_end = min(S, q0 + 128);
  const int ntile = (kv_end + 63) / 64;
  RowTile<64, DH> kt, vt;
  TransTile<DH> ktt;
  kt.load(K, ld, 0, S, tid);
  vt.load(V, ld, 0, S, tid);
  ktt.load(K, ld, 0, S, tid);
  kt.store(lds, tid);
  vt.store(lds + TILE, tid);
  ktt.store(lds + 2 * TILE, tid);
  __syncthreads();

  const int wq_min = q0 + 32 * w, wq_max = wq_min + 31;
  for (int t = 0; t < ntile; ++t) {
    const bf16_raw* sK = lds + (t & 1) * STAGE;
    const bf16_raw* sV = sK + TILE;
    const bf16_raw* sKt = sK + 2 * TILE;
    const int kv0 = t * 64;
    const bool more = t + 1 < ntile;
    if (more) {
      kt.load(K, ld, kv0 + 64, S, tid);
      vt.load(V, ld, kv0 + 64, S, tid);
      ktt.load(K, ld, kv0 + 64, S, tid);
    }
    if (kv0 <= wq_max) {
      f32x16 s[2], dp[2];
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[kb2][r] = 0.f; dp[kb2][r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
          const bf16x8 a = lds_frag(sK + RowTile<64, DH>::frag_off(32 * kb2 + l32, 2 * ks + lg));
          s[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb2], 0, 0, 0);
          const bf16x8 v = lds_frag(sV + RowTile<64, DH>::frag_off(32 * kb2 + l32, 2 * ks + lg));
          dp[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v, dof[ks], dp[kb2], 0, 0, 0);
        }
      const bool diag = kv0 + 63 > wq_min;
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(fmaf(s[kb2][r], c, -L2));
          const int kv = kv0 + 32 * kb2 + 8 * (r >> 2) + 4 * lg + (r & 3);
          if (diag && kv > qrow) p = 0.f;
          dp[kb2][r] = p * (dp[kb2][r] - dl);
        }
      bf16x8 dsf[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) dsf[tt] = pack8(dp[tt >> 1], 8 * (tt & 1));
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const bf16x8 a = lds_frag(sKt + TransTile<DH>::frag_off(32 * i + l32, 2 * tt + lg));
          dqacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf[tt], dqacc[i], 0, 0, 0);
        }
    }
    if (more) {
      bf16_raw* dK = lds + ((t + 1) & 1) * STAGE;
      kt.store(dK, tid);
      vt.store(dK + TILE, tid);
      ktt.store(dK + 2 * TILE, tid);
    }
    __syncthreads();
  }

  if (qrow < S) {
    bf16_raw* dqrow = dqkv + ((size_t)b * S + qrow) * ld + h * DH;
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack2(dqacc[i][4 * g + 0] * scale, dqacc[i][4 * g + 1] * scale);
        v.y = pack2(dqacc[i][4 * g + 2] * scale, dqacc[i][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(dqrow + 32 * i + 8 * g + 4 * lg) = v;
      }
  }
}

template <typename Kern>
swarm_status set_lds(Kern kern, size_t bytes, bool& done) {
  if (!done) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
      return SWARM_ERR_LAUNCH;
    done = true;
  }
  return SWARM_OK;
}

template <int DH>
swarm_status launch_bwd(const bf16_raw* qkv, const bf16_raw* o, const bf16_raw* dout, const float* lse, float* delta,
                        bf16_raw* dqkv, int B, int S, int H, hipStream_t st) {
  constexpr size_t lds_dkdv = (size_t)2 * (4 * 64 * DH + 256) * sizeof(bf16_raw);
  constexpr size_t lds_dq = (size_t)2 * 3 * 64 * DH * sizeof(bf16_raw);
  static bool a1 = false, a2 = false;
  if (set_lds(attn_bwd_dkdv_kernel<DH>, lds_dkdv, a1) != SWARM_OK) return SWARM_ERR_LAUNCH;
  if (set_lds(attn_bwd_dq_kernel<DH>, lds_dq, a2) != SWARM_OK) return SWARM_ERR_LAUNCH;
  hipLaunchKernelGGL(attn_delta_kernel<DH>, dim3(B * S), dim3(kThreads), 0, st, o, dout, delta, S, H);
  dim3 grid((S + 127) / 128, H, B);
  hipLaunchKernelGGL(attn_bwd_dkdv_kernel<DH>, grid, dim3(kThreads), lds_dkdv, st, qkv, dout, lse, delta, dqkv, S, H);
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
