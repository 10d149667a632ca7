// bf16 GEMM on the CDNA4 matrix cores: C[M,N] = sum_k A(m,k) B(n,k), fp32 accumulation.
// This is the dense contraction behind every fully connected layer of the transformer
// workloads (KARMA Sec. III-C "Fully-Connected Layer": |X| x |Y| multiply-adds) and its
// two gradients (dX = dY W, dW = dY^T X).
//
// Operands may have the reduction index contiguous ("k-contiguous": A[M][K], B[N][K]) or
// strided (A[K][M], B[K][N]); strided tiles are transposed in registers on their way into
// LDS, so the MFMA loop always reads 16-byte k-runs.  Tiles are staged through LDS with
// one register-resident tile in flight (double buffer); v_mfma_f32_32x32x16_bf16 does the
// arithmetic; the workgroup -> tile map keeps each XCD's L2 on a compact patch of C.
#include <hip/hip_runtime.h>

#include "karma.h"
#include "device_utils.h"
#include "kernels.h"

namespace karma {

struct GemmEpilogue {
  void* C;                 // bf16 or fp32 [M][ldc]
  const bf16_t* bias;      // [N] or null
  const bf16_t* residual;  // [M][ldc] or null (bf16 output only)
  int ldc;
  int out_f32;             // store fp32 instead of bf16
  int accumulate;          // fp32 output only: C += result
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    if (bias) v += bf2f(bias[n]);
    size_t at = (size_t)m * ldc + n;
    if (out_f32) {
      float* c = (float*)C;
      c[at] = accumulate ? c[at] + v : v;
    } else {
      if (residual) v += bf2f(residual[at]);
      ((bf16_t*)C)[at] = f2bf(v);
    }
  }
};

template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                   const bf16_t* __restrict__ B, int M, int N, int K,
                                                                   int lda, int ldb, int tiles_m, int tiles_n,
                                                                   GemmEpilogue ep) {
  constexpr int T = WGM * WGN * 64;
  constexpr int PITCH = BK + LDS_PAD;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = (bf16_t*)smem;          // [2][BM][PITCH]
  bf16_t* Bs = As + 2 * BM * PITCH;    // [2][BN][PITCH]

  // workgroup -> tile: consecutive ids go round-robin over the 8 XCDs, so give each XCD a
  // contiguous range of tiles, and walk tiles in bands of 8 tile-rows so that a band's B
  // panel stays in that XCD's L2.
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
  constexpr int BAND = 8;
  const int band_sz = BAND * tiles_n;
  const int first_m = (id / band_sz) * BAND;
  const int rows_in_band = min(tiles_m - first_m, BAND);
  const int tile_m = first_m + (id % band_sz) % rows_in_band;
  const int tile_n = (id % band_sz) / rows_in_band;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int lrow = lane & 31, lk = (lane >> 5) * 8;

  TileMover<BM, BK, T, A_KC> ma;
  TileMover<BN, BK, T, B_KC> mb;
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = (K + BK - 1) / BK;
  ma.load(A, lda, m0, 0, M, K, tid);
  mb.load(B, ldb, n0, 0, N, K, tid);
  ma.store(As, tid);
  mb.store(Bs, tid);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      ma.load(A, lda, m0, (kt + 1) * BK, M, K, tid);
      mb.load(B, ldb, n0, (kt + 1) * BK, N, K, tid);
    }
    const bf16_t* as = As + cur * BM * PITCH + (wm * WTM + lrow) * PITCH + lk;
    const bf16_t* bs = Bs + cur * BN * PITCH + (wn * WTN + lrow) * PITCH + lk;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8*)(as + i * 32 * PITCH + kk * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = *(const bf16x8*)(bs + j * 32 * PITCH + kk * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      ma.store(As + (cur ^ 1) * BM * PITCH, tid);
      mb.store(Bs + (cur ^ 1) * BN * PITCH, tid);
    }
    __syncthreads();
  }

  // accumulator layout of the 32x32 MFMA: register r of lane l is row (r/4)*8 + (l/32)*4 + r%4,
  // column l%32
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WTN + j * 32 + lrow;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * WTM + i * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r & 3);
        if (m < M && n < N) ep(m, n, acc[i][j][r]);
      }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN>
static int launch_cfg(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const size_t lds = (size_t)2 * (BM + BN) * (BK + LDS_PAD) * sizeof(bf16_t);
  GemmEpilogue ep{g.C, g.bias, g.residual, g.ldc, g.out_f32, g.accumulate};
  dim3 grid(tiles_m * tiles_n), block(WGM * WGN * 64);
#define KARMA_GEMM_LAUNCH(AK, BKC)                                                                      \
  do {                                                                                                  \
    auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, AK, BKC>;                                        \
    if (lds > 64 * 1024) (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
    hipLaunchKernelGGL(kern, grid, block, lds, s, g.A, g.B, g.M, g.N, g.K, g.lda, g.ldb, tiles_m, tiles_n, ep);  \
  } while (0)
  if (g.a_kc && g.b_kc) KARMA_GEMM_LAUNCH(true, true);
  else if (g.a_kc && !g.b_kc) KARMA_GEMM_LAUNCH(true, false);
  else if (!g.a_kc && g.b_kc) KARMA_GEMM_LAUNCH(false, true);
  else KARMA_GEMM_LAUNCH(false, false);
#undef KARMA_GEMM_LAUNCH
  return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP;
}

int gemm_bf16(const GemmArgs& g, hipStream_t s) {
  if (!g.A || !g.B || !g.C || g.M <= 0 || g.N <= 0 || g.K <= 0) return KARMA_E_INVAL;
  // 16-byte k-runs (k-contiguous) or 8-byte row runs (strided) must stay aligned and whole
  if (g.K % 8) return KARMA_E_INVAL;
  if (g.a_kc ? (g.lda % 8) : (g.lda % 4 || g.M % 4)) return KARMA_E_INVAL;
  if (g.b_kc ? (g.ldb % 8) : (g.ldb % 4 || g.N % 4)) return KARMA_E_INVAL;
  if (g.accumulate && !g.out_f32) return KARMA_E_INVAL;
  if (g.residual && g.out_f32) return KARMA_E_INVAL;
  return launch_cfg<128, 128, 64, 2, 2>(g, s);
}

}  // namespace karma

using namespace karma;

extern "C" int karma_k_gemm_bf16(const void* a, const void* b, void* c, const void* bias, const void* residual,
                                 uint32_t m, uint32_t n, uint32_t k, uint32_t flags, void* stream) {
  GemmArgs g{};
  g.A = (const bf16_t*)a;
  g.B = (const bf16_t*)b;
  g.C = c;
  g.bias = (const bf16_t*)bias;
  g.residual = (const bf16_t*)residual;
  g.M = (int)m; g.N = (int)n; g.K = (int)k;
  g.a_kc = !(flags & KARMA_GEMM_A_STRIDED);
  g.b_kc = !(flags & KARMA_GEMM_B_STRIDED);
  g.lda = g.a_kc ? (int)k : (int)m;
  g.ldb = g.b_kc ? (int)k : (int)n;
  g.ldc = (int)n;
  g.out_f32 = (flags & KARMA_GEMM_OUT_F32) != 0;
  g.accumulate = (flags & KARMA_GEMM_ACCUMULATE) != 0;
  return gemm_bf16(g, (hipStream_t)stream);
}
