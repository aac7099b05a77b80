// Pieces shared by the bf16 MFMA GEMM kernels: argument block, tile order, fused epilogue.
#pragma once
#include "kernels.h"
#include "gelu.h"

namespace swarm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct KArgs {
  const bf16_raw* A; const bf16_raw* B;
  int M, N, K, lda, ldb;
  void* C; int ldc;
  int epilogue;
  const bf16_raw* bias; const bf16_raw* aux; int ldaux;
  bf16_raw* C2; int ldc2;
  void* scales; int scales16;   // EPI_BIAS_RESID_ENCODE (scales16: bf16 bit patterns instead of fp32)
  const float* rope; int rope_S, rope_dh, rope_cols;   // EPI_BIAS_ROPE
  int split;       // EPI_DGEGLU, EPI_BIAS_GEGLU
  int tiles_m, tiles_n;
  int group_m;   // tile rows walked together (L2 reuse of the B panel)
  int stream;    // != 0: the epilogue's global accesses are non-temporal (see store_stream)
  int ksplit;    // > 1: the grid holds ksplit workgroups per tile, each takes K / ksplit and stores its fp32 partial
  float* part;   //      tile sums to part + index * M * N (a second kernel adds them and applies the epilogue)
  long long* stamps;   // instrumented build only (nullptr otherwise): 16 words per workgroup, see gemm_bf16_k32_kernel
};

constexpr int EPI_PART_F32 = 100;   // kernel-internal: C (fp32, ldc = N) = acc, no read

// Launch order maps consecutive workgroups to the 8 XCDs round-robin; give every XCD a contiguous band
// of tiles (its own L2 then sees the reuse) and walk tiles in groups of 8 rows to keep a B panel resident.
__device__ __forceinline__ void tile_of_block(const KArgs& p, int& tile_m, int& tile_n, int pid = blockIdx.x) {
  const int ntiles = p.tiles_m * p.tiles_n;
  if ((ntiles & 7) == 0) pid = (pid & 7) * (ntiles >> 3) + (pid >> 3);
  const int GM = p.group_m;
  const int per_group = GM * p.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GM;
  const int gsz = min(p.tiles_m - first_m, GM);
  tile_m = first_m + (pid % per_group) % gsz;
  tile_n = (pid % per_group) / gsz;
}

// acc[i][j][r] is C(row, col) with row = row0 + i*32 + 8*(r/4) + 4*lg + (r%4), col = col0 + j*32 + l32
// (row0/col0 = first row/column of this wavefront's sub-tile).
//
// bf16 outputs: an accumulator lane holds one column and scattered rows, which would mean 2-byte stores.
// Each wavefront therefore turns its sub-tile 32 rows at a time through a private LDS patch
// (`stage`, 32 x kEpiPitch floats) and writes rows out with 16-byte loads/stores: 8 lanes cover 128
// contiguous bytes of a row, for C, for the residual / pre-activation input and for the second output.
// fp32 accumulate (wgrad) already touches 128 contiguous bytes per row and stays direct.
constexpr int kEpiPitch = 68;   // floats; 4-bank skew between consecutive rows keeps the row reads conflict free

__device__ __forceinline__ void unpack8(const uint4& v, float (&x)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(w[i] << 16);
    x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Streaming accesses of the epilogues: an output tile is written once and the residual / pre-activation / gradient
// rows are read once, so they are marked non-temporal and do not push the operand panels out of the L2.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ void store_stream(void* dst, const uint4& v) {
  const u32x4_t t = {v.x, v.y, v.z, v.w};
  if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(dst));
  else *reinterpret_cast<u32x4_t*>(dst) = t;
}
template <bool NT>
__device__ __forceinline__ void store_stream(float* dst, const float4& v) {
  const f32x4_t t = {v.x, v.y, v.z, v.w};
  if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<f32x4_t*>(dst));
  else *reinterpret_cast<f32x4_t*>(dst) = t;
}
template <bool NT>
__device__ __forceinline__ uint4 load_stream(const bf16_raw* src) {
  u32x4_t t;
  if constexpr (NT) t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src));
  else t = *reinterpret_cast<const u32x4_t*>(src);
  return make_uint4(t[0], t[1], t[2], t[3]);
}
template <bool NT>
__device__ __forceinline__ float4 load_stream(const float* src) {
  f32x4_t t;
  if constexpr (NT) t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(src));
  else t = *reinterpret_cast<const f32x4_t*>(src);
  return make_float4(t[0], t[1], t[2], t[3]);
}

__device__ __forceinline__ uint4 pack8_bf16(const float (&x)[8]) {
  return make_uint4(cvt_pk_bf16(x[0], x[1]), cvt_pk_bf16(x[2], x[3]), cvt_pk_bf16(x[4], x[5]), cvt_pk_bf16(x[6], x[7]));
}

// Rows 32 i .. 32 i + 31 of a wavefront's accumulator sub-tile into its LDS patch (row-major, pitch kEpiPitch).
// 32 x 32 blocks: acc[i][j][r] is the element (8 (r / 4) + 4 lg + r % 4, 32 j + l32) of row group i.
template <int FM, int FN>
__device__ __forceinline__ void stage_rows32(const f32x16 (&acc)[FM][FN], int i, float* stage, int lane) {
  const int l32 = lane & 31, lg = lane >> 5;
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * lg + (r & 3)) * kEpiPitch + 32 * j + l32] = acc[i][j][r];
}
// 16 x 16 blocks (v_mfma_f32_16x16x32): blk[i16][j16][r] is the element (4 (lane / 16) + r, lane % 16) of block
// (i16, j16); a 32-row group holds the block rows 2 i and 2 i + 1.
typedef __attribute__((ext_vector_type(4))) float f32x4;
template <int FM, int FN>
struct Acc16 {
  f32x4 blk[2 * FM][2 * FN];
};
template <int FM, int FN>
__device__ __forceinline__ void stage_rows32(const Acc16<FM, FN>& acc, int i, float* stage, int lane) {
  const int l16 = lane & 15, q = lane >> 4;
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int j = 0; j < 2 * FN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) stage[(16 * h + 4 * q + r) * kEpiPitch + 16 * j + l16] = acc.blk[2 * i + h][j][r];
}

template <int FM, int FN, bool GUARD, bool NT, typename Acc>
__device__ __forceinline__ void gemm_epilogue_nt(const KArgs& p, const Acc& acc, int row0, int col0, int l32,
                                              int lg, float* stage) {
  static_assert(32 * FN <= kEpiPitch - 4, "the LDS patch holds 64 columns");
  const int epi = p.epilogue;
  constexpr int COLS = 32 * FN;
  const int lane = l32 + 32 * lg;
  if (epi == EPI_ACCUM_F32 || epi == EPI_PART_F32) {
    // C (fp32) += acc (or = acc), 16 bytes per lane: 16 lanes cover one 64-column row of the sub-tile
    constexpr int LPR4 = COLS / 4, RPP4 = 64 / LPR4;
    float* c = reinterpret_cast<float*>(p.C);
    const int c4 = lane % LPR4, rsub4 = lane / LPR4;
    const int colf = col0 + 4 * c4;
    const bool colf_ok = !GUARD || colf < p.N;
    // The gradient values a row group adds to are requested one group ahead: their latency is then paid once,
    // not once per group.
    constexpr int NPS4 = 32 / RPP4;
    const bool accum = epi == EPI_ACCUM_F32;
    float4 cn[NPS4];
    auto load_c = [&](int i) __attribute__((always_inline)) {
#pragma unroll
      for (int ps = 0; ps < NPS4; ++ps) {
        const int row = row0 + i * 32 + ps * RPP4 + rsub4;
        if (accum && colf_ok && (!GUARD || row < p.M))
          cn[ps] = load_stream<NT>(c + (size_t)row * p.ldc + colf);
      }
    };
    load_c(0);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      stage_rows32<FM, FN>(acc, i, stage, lane);
      float4 cc[NPS4];
#pragma unroll
      for (int ps = 0; ps < NPS4; ++ps) cc[ps] = cn[ps];
      if (i + 1 < FM) load_c(i + 1);
#pragma unroll
      for (int ps = 0; ps < NPS4; ++ps) {
        const int rl = ps * RPP4 + rsub4;
        const int row = row0 + i * 32 + rl;
        const float4 v = *reinterpret_cast<const float4*>(stage + rl * kEpiPitch + 4 * c4);
        if (!colf_ok || (GUARD && row >= p.M)) continue;
        float4 o = v;
        if (accum) {
          o = cc[ps];
          o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
        }
        store_stream<NT>(c + (size_t)row * p.ldc + colf, o);
      }
    }
    return;
  }
  if constexpr (FN == 2 && !GUARD) if (epi == EPI_BIAS_GEGLU) {
    // The B tile was gathered so that this sub-tile's columns 0..31 are the gate and 32..63 the up pre-activations
    // of the SAME 32 features col0 .. col0+31 (col0 counts features here).  4 lanes per row, 8 features each.
    const int c4 = lane & 3, rsub = lane >> 2;
    const int feat = col0 + 8 * c4;
    float bg[8], bu[8];
    unpack8(*reinterpret_cast<const uint4*>(p.bias + feat), bg);
    unpack8(*reinterpret_cast<const uint4*>(p.bias + p.split + feat), bu);
    bf16_raw* G = reinterpret_cast<bf16_raw*>(p.C);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      stage_rows32<FM, FN>(acc, i, stage, lane);
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        const int rl = ps * 16 + rsub;
        const size_t row = row0 + i * 32 + rl;
        const float* sp = stage + rl * kEpiPitch + 8 * c4;
        const float4 g0 = *reinterpret_cast<const float4*>(sp), g1 = *reinterpret_cast<const float4*>(sp + 4);
        const float4 u0 = *reinterpret_cast<const float4*>(sp + 32), u1 = *reinterpret_cast<const float4*>(sp + 36);
        float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) { g[e] += bg[e]; u[e] += bu[e]; }
        if (p.C2) {
          store_stream<NT>(p.C2 + row * p.ldc2 + feat, pack8_bf16(g));
          store_stream<NT>(p.C2 + row * p.ldc2 + p.split + feat, pack8_bf16(u));
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = gelu_fast(g[e]) * u[e];
        store_stream<NT>(G + row * p.ldc + feat, pack8_bf16(g));
      }
    }
    return;
  }
  constexpr int LPR = COLS / 8;          // lanes per row on the way out
  constexpr int RPP = 64 / LPR;          // rows per pass
  const int c8 = lane % LPR, rsub = lane / LPR;
  const int col = col0 + 8 * c8;
  const bool col_ok = !GUARD || col < p.N;     // N is a multiple of 8, so a chunk is all in or all out
  float bias[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) bias[e] = 0.f;
  if (col_ok && (epi == EPI_BIAS || epi == EPI_BIAS_RESID || epi == EPI_BIAS_GELU || epi == EPI_BIAS_RESID_ENCODE ||
                 epi == EPI_BIAS_ROPE))
    unpack8(*reinterpret_cast<const uint4*>(p.bias + col), bias);
  bf16_raw* C = reinterpret_cast<bf16_raw*>(p.C);
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    stage_rows32<FM, FN>(acc, i, stage, lane);
#pragma unroll
    for (int ps = 0; ps < 32 / RPP; ++ps) {
      const int rl = ps * RPP + rsub;
      const int row = row0 + i * 32 + rl;
      const float4 v0 = *reinterpret_cast<const float4*>(stage + rl * kEpiPitch + 8 * c8);
      const float4 v1 = *reinterpret_cast<const float4*>(stage + rl * kEpiPitch + 8 * c8 + 4);
      if (!col_ok || (GUARD && row >= p.M)) continue;     // uniform over a lane octet (N % 64 == 0 when encoding)
      float x[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
      if (epi == EPI_BIAS_RESID_ENCODE) {
        // stage-exit codec fused: the 8 lanes of a row segment hold one 64-element block.  Values are
        // rounded to bf16 first, so codes and scales equal the stand-alone encode of the stored tensor.
        float a[8];
        unpack8(load_stream<NT>(p.aux + (size_t)row * p.ldaux + col), a);
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          x[e] = bf16_bits_to_float(float_to_bf16_bits(x[e] + bias[e] + a[e]));
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
        const size_t e0 = (size_t)row * p.ldc + col;
        *reinterpret_cast<uint2*>(reinterpret_cast<int8_t*>(p.C) + e0) = make_uint2(w[0], w[1]);
        if (c8 == 0) block_scale_store(p.scales, e0 >> 6, sc, p.scales16);
        continue;
      }
      if (epi == EPI_BIAS) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] += bias[e];
      } else if (epi == EPI_BIAS_RESID) {
        float a[8];
        unpack8(load_stream<NT>(p.aux + (size_t)row * p.ldaux + col), a);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = x[e] + bias[e] + a[e];
      } else if (epi == EPI_BIAS_GELU) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] += bias[e];
        if (p.C2) store_stream<NT>(p.C2 + (size_t)row * p.ldc2 + col, pack8_bf16(x));
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = gelu_fast(x[e]);
      } else if (epi == EPI_DGELU) {
        float a[8];
        unpack8(load_stream<NT>(p.aux + (size_t)row * p.ldaux + col), a);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] *= gelu_grad_fast(a[e]);
      } else if (epi == EPI_BIAS_ROPE) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] += bias[e];
        if (col < p.rope_cols) {   // pair (2i, 2i+1) of a head turns by pos * 10000^(-2i/d_head)
          const int half = p.rope_dh >> 1;
          const float* t = p.rope + 2 * ((size_t)(row % p.rope_S) * half + ((col % p.rope_dh) >> 1));
          const float4 t0 = *reinterpret_cast<const float4*>(t), t1 = *reinterpret_cast<const float4*>(t + 4);
          const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float a = x[2 * e], b = x[2 * e + 1];
            x[2 * e] = a * cs[e] - b * sn[e];
            x[2 * e + 1] = a * sn[e] + b * cs[e];
          }
        }
      } else if (epi == EPI_DGEGLU) {
        float gt[8], up[8], o2[8];
        unpack8(load_stream<NT>(p.aux + (size_t)row * p.ldaux + col), gt);
        unpack8(load_stream<NT>(p.aux + (size_t)row * p.ldaux + p.split + col), up);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          o2[e] = x[e] * gelu_fast(gt[e]);
          x[e] = x[e] * up[e] * gelu_grad_fast(gt[e]);
        }
        store_stream<NT>(C + (size_t)row * p.ldc + p.split + col, pack8_bf16(o2));
      }
      store_stream<NT>(C + (size_t)row * p.ldc + col, pack8_bf16(x));
    }
  }
}

// NT (p.stream): the epilogue's global accesses are non-temporal; two copies of the code, one uniform branch.
template <int FM, int FN, bool GUARD, typename Acc>
__device__ __forceinline__ void gemm_epilogue(const KArgs& p, const Acc& acc, int row0, int col0, int l32,
                                              int lg, float* stage) {
  if (p.stream) gemm_epilogue_nt<FM, FN, GUARD, true>(p, acc, row0, col0, l32, lg, stage);
  else gemm_epilogue_nt<FM, FN, GUARD, false>(p, acc, row0, col0, l32, lg, stage);
}

}  // namespace
}  // namespace swarm
