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
#include "kernels.h"

namespace karma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

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

constexpr int LDS_PAD = 8;   // elements: a 16-byte skew per row keeps ds_read_b128 conflict-free

// One operand tile (ROWS x BK) on its way global -> registers -> LDS.
// KC: global is [rows][k] (k contiguous): each thread moves 16-byte k-runs unchanged.
// !KC: global is [k][rows]: each thread loads an 8(k) x 4(rows) patch as eight 8-byte
//      pieces and writes four transposed 16-byte k-runs.
template <int ROWS, int BK, int T, bool KC>
struct TileMover {
  static constexpr int PITCH = BK + LDS_PAD;
  static constexpr int VECS = ROWS * BK / 8 / T;
  static_assert(ROWS * BK % (8 * T) == 0 && VECS >= 1, "tile does not divide over the workgroup");
  static_assert(KC || VECS % 4 == 0, "transposing mover needs whole 8x4 patches per thread");
  u32x4 reg[VECS];

  __device__ __forceinline__ void load(const bf16_t* __restrict__ G, int ld, int row0, int k0, int rows_total,
                                       int k_total, int tid) {
    if (KC) {
#pragma unroll
      for (int i = 0; i < VECS; ++i) {
        int v = tid + i * T, row = v / (BK / 8), kc = v % (BK / 8);
        int gr = row0 + row, gk = k0 + kc * 8;
        u32x4 z = {0, 0, 0, 0};
        reg[i] = (gr < rows_total && gk < k_total) ? *(const u32x4*)(G + (size_t)gr * ld + gk) : z;
      }
    } else {
#pragma unroll
      for (int b = 0; b < VECS / 4; ++b) {
        int v = tid + b * T, rg = v % (ROWS / 4), kg = v / (ROWS / 4);
        int gr = row0 + rg * 4;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          int gk = k0 + kg * 8 + q;
          u32x2 z = {0, 0};
          u32x2 r = (gr < rows_total && gk < k_total) ? *(const u32x2*)(G + (size_t)gk * ld + gr) : z;
          reg[b * 4 + q / 2][(q & 1) * 2] = r.x;
          reg[b * 4 + q / 2][(q & 1) * 2 + 1] = r.y;
        }
      }
    }
  }

  __device__ __forceinline__ void store(bf16_t* __restrict__ S, int tid) const {
    if (KC) {
#pragma unroll
      for (int i = 0; i < VECS; ++i) {
        int v = tid + i * T, row = v / (BK / 8), kc = v % (BK / 8);
        *(u32x4*)(S + row * PITCH + kc * 8) = reg[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < VECS / 4; ++b) {
        int v = tid + b * T, rg = v % (ROWS / 4), kg = v / (ROWS / 4);
        // reg[b*4 + p] = { k=2p: (r0 r1 | r2 r3), k=2p+1: (r0 r1 | r2 r3) } as dwords x y z w
        u32x4 t[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          unsigned e0 = reg[b * 4 + p].x, e1 = reg[b * 4 + p].y;   // row k = 2p
          unsigned o0 = reg[b * 4 + p].z, o1 = reg[b * 4 + p].w;   // row k = 2p + 1
          t[0][p] = (e0 & 0xffffu) | (o0 << 16);
          t[1][p] = (e0 >> 16) | (o0 & 0xffff0000u);
          t[2][p] = (e1 & 0xffffu) | (o1 << 16);
          t[3][p] = (e1 >> 16) | (o1 & 0xffff0000u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) *(u32x4*)(S + (rg * 4 + j) * PITCH + kg * 8) = t[j];
      }
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
