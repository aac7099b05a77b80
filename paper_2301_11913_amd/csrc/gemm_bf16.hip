// bf16 MFMA GEMM for gfx950 with fp32 accumulation:  C[M,N] (+)= sum_k A(m,k) B(n,k).
//
// Workgroup tile BM x BN x 64, WM x WN wavefronts, each owning a (BM/WM) x (BN/WN) sub-tile made
// of 32x32 accumulators fed by v_mfma_f32_32x32x16_bf16.  Both operand tiles live in LDS as
// [rows][64 k] bf16 (128-byte rows) with the 16-byte chunks of a row XOR-swizzled so that the
// 64-lane 16-byte fragment reads are bank-conflict free; LDS is double buffered and the next
// K-slice is prefetched into registers while the current one is multiplied (one barrier per slice).
//
// Operands whose contraction index is the slow (row) index in memory - W in the data-gradient
// GEMM, both operands in the weight-gradient GEMM - are transposed on their way into LDS: a lane
// loads an 8(k) x 4 patch with 8-byte loads and permutes it in registers into four 16-byte LDS
// rows.  Nothing is transposed through HBM.
//
// Launch order maps consecutive workgroups to the 8 XCDs round-robin, so tile ids are remapped
// to give every XCD a contiguous band of tiles (its own L2 then sees the reuse), and tiles are
// walked in groups of rows to keep the B panel resident.
//
// Deterministic: one workgroup owns an output tile and walks K in order.
#include <vector>

#include "gemm_bf16_common.h"

namespace swarm {
namespace {

constexpr int BK = 64;

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }
// element offset of 16-byte chunk `chunk` (0..7) of row `row` in a [rows][64] bf16 tile
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * BK + ((chunk ^ swz(row)) << 3); }


// Global -> registers for one operand tile (BR rows of the GEMM x 64 k).
template <int BR, int NT, bool TRANS, bool GUARD>
struct TileLoader {
  // non-transposed: BR*8 16-byte chunks; transposed: (BR/4)*8 patches of 8(k) x 4
  static constexpr int NI = TRANS ? ((BR / 4) * 8 + NT - 1) / NT : (BR * 8) / NT;
  static constexpr int REGS = TRANS ? NI * 8 : NI * 2;   // in uint2 units
  uint2 r[REGS];

  __device__ __forceinline__ void load(const bf16_raw* __restrict__ p, int ld, int rows, int kdim, int r0, int k0,
                                       int tid) {
    if constexpr (!TRANS) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int it = tid + i * NT;
        const int row = it >> 3, chunk = it & 7;
        const int gr = r0 + row, gk = k0 + chunk * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (!GUARD || (gr < rows && gk < kdim)) v = *reinterpret_cast<const uint4*>(p + (size_t)gr * ld + gk);
        r[2 * i] = make_uint2(v.x, v.y);
        r[2 * i + 1] = make_uint2(v.z, v.w);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int it = tid + i * NT;
        const int xc = it % (BR / 4), kg = it / (BR / 4);
        const int col = r0 + xc * 4;
        const bool in = (NI * NT == (BR / 4) * 8) || kg < 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int gk = k0 + kg * 8 + j;
          uint2 v = make_uint2(0, 0);
          if (in && (!GUARD || (gk < kdim && col < rows)))
            v = *reinterpret_cast<const uint2*>(p + (size_t)gk * ld + col);
          r[i * 8 + j] = v;
        }
      }
    }
  }

  __device__ __forceinline__ void store(bf16_raw* __restrict__ lds, int tid) const {
    if constexpr (!TRANS) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int it = tid + i * NT;
        const int row = it >> 3, chunk = it & 7;
        *reinterpret_cast<uint4*>(lds + tile_off(row, chunk)) =
            make_uint4(r[2 * i].x, r[2 * i].y, r[2 * i + 1].x, r[2 * i + 1].y);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int it = tid + i * NT;
        const int xc = it % (BR / 4), kg = it / (BR / 4);
        if ((NI * NT != (BR / 4) * 8) && kg >= 8) continue;
        const uint2* q = r + i * 8;
        // q[j] = 4 consecutive columns of k-row j; build, per column x, the 8 k values
        uint4 o0, o1, o2, o3;
        o0.x = __builtin_amdgcn_perm(q[1].x, q[0].x, 0x05040100u); o1.x = __builtin_amdgcn_perm(q[1].x, q[0].x, 0x07060302u);
        o0.y = __builtin_amdgcn_perm(q[3].x, q[2].x, 0x05040100u); o1.y = __builtin_amdgcn_perm(q[3].x, q[2].x, 0x07060302u);
        o0.z = __builtin_amdgcn_perm(q[5].x, q[4].x, 0x05040100u); o1.z = __builtin_amdgcn_perm(q[5].x, q[4].x, 0x07060302u);
        o0.w = __builtin_amdgcn_perm(q[7].x, q[6].x, 0x05040100u); o1.w = __builtin_amdgcn_perm(q[7].x, q[6].x, 0x07060302u);
        o2.x = __builtin_amdgcn_perm(q[1].y, q[0].y, 0x05040100u); o3.x = __builtin_amdgcn_perm(q[1].y, q[0].y, 0x07060302u);
        o2.y = __builtin_amdgcn_perm(q[3].y, q[2].y, 0x05040100u); o3.y = __builtin_amdgcn_perm(q[3].y, q[2].y, 0x07060302u);
        o2.z = __builtin_amdgcn_perm(q[5].y, q[4].y, 0x05040100u); o3.z = __builtin_amdgcn_perm(q[5].y, q[4].y, 0x07060302u);
        o2.w = __builtin_amdgcn_perm(q[7].y, q[6].y, 0x05040100u); o3.w = __builtin_amdgcn_perm(q[7].y, q[6].y, 0x07060302u);
        const int row = xc * 4;
        *reinterpret_cast<uint4*>(lds + tile_off(row + 0, kg)) = o0;
        *reinterpret_cast<uint4*>(lds + tile_off(row + 1, kg)) = o1;
        *reinterpret_cast<uint4*>(lds + tile_off(row + 2, kg)) = o2;
        *reinterpret_cast<uint4*>(lds + tile_off(row + 3, kg)) = o3;
      }
    }
  }
};

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T, bool GUARD>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(KArgs p) {
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int STAGE = (BM + BN) * BK;   // elements per LDS stage
  extern __shared__ __attribute__((aligned(16))) bf16_raw lds[];

  int tile_m, tile_n;
  tile_of_block(p, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lg = lane >> 5;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  TileLoader<BM, NT, A_T, GUARD> la;
  TileLoader<BN, NT, B_T, GUARD> lb;

  const int KT = (p.K + BK - 1) / BK;
  la.load(p.A, p.lda, p.M, p.K, m0, 0, tid);
  lb.load(p.B, p.ldb, p.N, p.K, n0, 0, tid);
  la.store(lds, tid);
  lb.store(lds + BM * BK, tid);
  __syncthreads();

  // per-lane fragment offsets: row (l32) fixes the swizzle, chunk = 2*kk + lg
  int foff[4];
  {
    const int s = swz(l32);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) foff[kk] = l32 * BK + (((2 * kk + lg) ^ s) << 3);
  }

  for (int kt = 0; kt < KT; ++kt) {
    const bf16_raw* sA = lds + (kt & 1) * STAGE;
    const bf16_raw* sB = sA + BM * BK;
    const bool more = kt + 1 < KT;
    if (more) {
      la.load(p.A, p.lda, p.M, p.K, m0, (kt + 1) * BK, tid);
      lb.load(p.B, p.ldb, p.N, p.K, n0, (kt + 1) * BK, tid);
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 a[FM], b[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i)
        a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sA + (wm * WTM + i * 32) * BK + foff[kk]));
#pragma unroll
      for (int j = 0; j < FN; ++j)
        b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sB + (wn * WTN + j * 32) * BK + foff[kk]));
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      bf16_raw* dA = lds + ((kt + 1) & 1) * STAGE;
      la.store(dA, tid);
      lb.store(dA + BM * BK, tid);
    }
    __syncthreads();
  }

  // every wavefront is past the last barrier: the operand stages are free to serve as epilogue patches
  gemm_epilogue<FM, FN, GUARD>(p, acc, m0 + wm * WTM, n0 + wn * WTN, l32, lg,
                               reinterpret_cast<float*>(lds) + wave * 32 * kEpiPitch);
}

template <int BM, int BN, int WM, int WN, bool A_T, bool B_T, bool GUARD>
swarm_status launch(const KArgs& k, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)2 * (BM + BN) * BK * sizeof(bf16_raw);
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, A_T, B_T, GUARD>;
  static LdsOptIn opted;   // per instantiation
  if (lds_opt_in((const void*)kern, lds_bytes, opted) != SWARM_OK) return SWARM_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3(k.tiles_m * k.tiles_n), dim3(WM * WN * 64), lds_bytes, st, k);
  return launch_status();
}

template <int BM, int BN, int WM, int WN, bool GUARD>
swarm_status launch_layout(const KArgs& k, bool a_t, bool b_t, hipStream_t st) {
  if (!a_t && !b_t) return launch<BM, BN, WM, WN, false, false, GUARD>(k, st);
  if (!a_t && b_t) return launch<BM, BN, WM, WN, false, true, GUARD>(k, st);
  if (a_t && b_t) return launch<BM, BN, WM, WN, true, true, GUARD>(k, st);
  return SWARM_ERR_SHAPE;
}

#ifdef SWARM_KERNEL_HOOKS
// Per-launch timing of the MFMA GEMM, compiled into the instrumented build only (libswarm_hooks.so; off until
// enabled): an event pair on the launch stream around every launch, read back by swarm_kernel_timing_collect().
struct GemmTimer {
  static constexpr int kMax = 8192;
  bool enabled = false;
  int used = 0;
  std::vector<hipEvent_t> ev;      // 2 per launch
  std::vector<double> flops;
  std::vector<int> shape;          // 6 per launch: M, N, K, a_trans, b_trans, epilogue
} g_timer;
#endif

}  // namespace

swarm_status gemm_bf16_launch(const GemmArgs& g, hipStream_t st);
swarm_status gemm_bf16_dma(const GemmArgs& g, hipStream_t st);

swarm_status gemm_bf16(const GemmArgs& g, hipStream_t st) {
#ifdef SWARM_KERNEL_HOOKS
  if (g_timer.enabled && g_timer.used < GemmTimer::kMax) {
    const int i = g_timer.used++;
    g_timer.flops[i] = 2.0 * g.M * g.N * g.K;
    int* sh = &g_timer.shape[6 * i];
    sh[0] = g.M; sh[1] = g.N; sh[2] = g.K; sh[3] = g.a_trans; sh[4] = g.b_trans; sh[5] = g.epilogue;
    (void)hipEventRecord(g_timer.ev[2 * i], st);
    swarm_status s = gemm_bf16_launch(g, st);
    (void)hipEventRecord(g_timer.ev[2 * i + 1], st);
    return s;
  }
#endif
  return gemm_bf16_launch(g, st);
}

swarm_status gemm_bf16_launch(const GemmArgs& g, hipStream_t st) {
  // vector loads need 8-element alignment of every contiguous run
  auto al16 = [](const void* q) { return ((uintptr_t)q & 15) == 0; };
  bool vec_ok = (g.lda % 8 == 0) && (g.ldb % 8 == 0) && al16(g.A) && al16(g.B) &&
                (g.a_trans ? g.M % 8 == 0 : g.K % 8 == 0) && (g.b_trans ? g.N % 8 == 0 : g.K % 8 == 0);
  if (g.epilogue == EPI_ACCUM_F32) vec_ok = vec_ok && g.N % 4 == 0 && g.ldc % 4 == 0 && al16(g.C);
  if (g.epilogue != EPI_ACCUM_F32)   // the bf16 epilogue moves 8-element chunks
    vec_ok = vec_ok && g.N % 8 == 0 && g.ldc % 8 == 0 && al16(g.C) && (!g.bias || al16(g.bias)) &&
             (!g.aux || (al16(g.aux) && g.ldaux % 8 == 0)) && (!g.C2 || (al16(g.C2) && g.ldc2 % 8 == 0));
  if (g.epilogue == EPI_BIAS_RESID_ENCODE && (!vec_ok || g.N % 64 || g.ldc != g.N || !g.scales)) return SWARM_ERR_SHAPE;
  // epilogues that only the MFMA kernels have: refuse (before any launch) what they cannot take
  const bool mfma_only = g.epilogue == EPI_BIAS_ROPE || g.epilogue == EPI_DGEGLU || g.epilogue == EPI_BIAS_GEGLU;
  if (mfma_only && (!vec_ok || (g.a_trans && !g.b_trans))) return SWARM_ERR_SHAPE;
  if (g.epilogue == EPI_BIAS_ROPE && (!g.rope || g.rope_S < 1 || g.rope_dh % 8 || g.rope_cols % 8)) return SWARM_ERR_SHAPE;
  if (g.epilogue == EPI_DGEGLU && (g.split != g.N || !g.aux)) return SWARM_ERR_SHAPE;
  if (!vec_ok || (g.a_trans && !g.b_trans)) return gemm_generic(g, true, st);
  if (g.epilogue == EPI_BIAS_GEGLU)   // needs the gathered B tile of the direct-to-LDS kernel
    return gemm_bf16_dma(g, st);
  {
    const swarm_status s = gemm_bf16_dma(g, st);   // tile-aligned shapes: pipelined direct-to-LDS kernel
    if (s != SWARM_ERR_SHAPE) return s;
  }
  KArgs k;
  k.group_m = 8;   // measured best of {2,4,8,16,32} on the d=4096 shapes
  k.A = (const bf16_raw*)g.A; k.B = (const bf16_raw*)g.B; k.M = g.M; k.N = g.N; k.K = g.K; k.lda = g.lda;
  k.ldb = g.ldb; k.C = g.C; k.ldc = g.ldc; k.epilogue = g.epilogue; k.bias = (const bf16_raw*)g.bias;
  k.aux = (const bf16_raw*)g.aux; k.ldaux = g.ldaux; k.C2 = (bf16_raw*)g.C2; k.ldc2 = g.ldc2; k.scales = g.scales; k.scales16 = g.scales16;
  k.rope = g.rope; k.rope_S = g.rope_S; k.rope_dh = g.rope_dh; k.rope_cols = g.rope_cols; k.split = g.split;
  k.ksplit = 1; k.part = nullptr; k.stream = 0; k.stamps = nullptr;
  const long big_tiles = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
  // What arrives here has a ragged M, N or K (whole tiles with K % 64 == 0 went to the direct-to-LDS kernels above):
  // the bounds-checked instantiations only.
  if (big_tiles >= 160) {
    k.tiles_m = (g.M + 255) / 256; k.tiles_n = (g.N + 255) / 256;
    return launch_layout<256, 256, 2, 4, true>(k, g.a_trans, g.b_trans, st);
  }
  k.tiles_m = (g.M + 127) / 128; k.tiles_n = (g.N + 127) / 128;
  return launch_layout<128, 128, 2, 2, true>(k, g.a_trans, g.b_trans, st);
}

}  // namespace swarm

#ifdef SWARM_KERNEL_HOOKS
// Turn per-launch GEMM timing on (creates the event pool once) or off; resets the counters.
extern "C" int swarm_kernel_timing_enable(int on) {
  using namespace swarm;
  if (on && g_timer.ev.empty()) {
    g_timer.ev.resize(2 * GemmTimer::kMax);
    g_timer.flops.resize(GemmTimer::kMax);
    g_timer.shape.resize(6 * GemmTimer::kMax);
    for (auto& e : g_timer.ev)
      if (hipEventCreate(&e) != hipSuccess) return -1;
  }
  g_timer.enabled = on != 0;
  g_timer.used = 0;
  return 0;
}

// Synchronises, then returns the number of timed launches and their summed duration / flops.  With per_launch_ms
// and shapes not NULL (room for `room` launches: room doubles, 6 * room ints) every launch's duration and its
// M, N, K, a_trans, b_trans, epilogue are written too.
extern "C" int swarm_kernel_timing_collect_launches(double* total_ms, double* total_flops, double* per_launch_ms,
                                                    int* shapes, int room) {
  using namespace swarm;
  double ms = 0, fl = 0;
  for (int i = 0; i < g_timer.used; ++i) {
    if (hipEventSynchronize(g_timer.ev[2 * i + 1]) != hipSuccess) return -1;
    float t = 0;
    if (hipEventElapsedTime(&t, g_timer.ev[2 * i], g_timer.ev[2 * i + 1]) != hipSuccess) return -1;
    ms += t;
    fl += g_timer.flops[i];
    if (per_launch_ms && shapes && i < room) {
      per_launch_ms[i] = t;
      for (int k = 0; k < 6; ++k) shapes[6 * i + k] = g_timer.shape[6 * i + k];
    }
  }
  *total_ms = ms;
  *total_flops = fl;
  const int n = g_timer.used;
  g_timer.used = 0;
  return n;
}
extern "C" int swarm_kernel_timing_collect(double* total_ms, double* total_flops) {
  return swarm_kernel_timing_collect_launches(total_ms, total_flops, nullptr, nullptr, 0);
}
#endif  // SWARM_KERNEL_HOOKS
