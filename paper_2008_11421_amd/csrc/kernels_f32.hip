// fp32 kernels of the MLP workload: fully connected layer with ReLU (KARMA Sec. III-C,
// "Fully-Connected Layer", "ReLu Layer"), its backward, and the mean-squared-error loss.
// The shapes are tiny (32 x 256 x 256), so these are plain LDS-tiled FMA kernels; every
// output element is produced by one thread summing in a fixed order (deterministic).
#include <hip/hip_runtime.h>

#include "karma.h"
#include "kernels.h"

namespace karma {

constexpr int TS = 32;   // output tile edge
constexpr int TK = 16;   // reduction step

// C[m,n] = sum_k A(m,k) * B(n,k);  A row-major [M,K] (or [K,M] when A_T), B row-major
// [N,K] (or [K,N] when B_T).  Each of the 16x16 threads owns a 2x2 patch.
template <bool A_T, bool B_T, class Epilogue>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                        int M, int N, int K, Epilogue ep) {
  __shared__ float As[TK][TS + 1];
  __shared__ float Bs[TK][TS + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  for (int k0 = 0; k0 < K; k0 += TK) {
    // 512 elements per operand tile, 2 per thread
    for (int e = threadIdx.x; e < TS * TK; e += 256) {
      int r, c;   // r: row within tile (m or n), c: k within step
      if (A_T) { r = e % TS; c = e / TS; } else { r = e / TK; c = e % TK; }
      int gm = m0 + r, gk = k0 + c;
      float v = 0.f;
      if (gm < M && gk < K) v = A_T ? A[(size_t)gk * M + gm] : A[(size_t)gm * K + gk];
      As[c][r] = v;
      if (B_T) { r = e % TS; c = e / TS; } else { r = e / TK; c = e % TK; }
      int gn = n0 + r;
      gk = k0 + c;
      v = 0.f;
      if (gn < N && gk < K) v = B_T ? B[(size_t)gk * N + gn] : B[(size_t)gn * K + gk];
      Bs[c][r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a0 = As[k][ty], a1 = As[k][ty + 16], b0 = Bs[k][tx], b1 = Bs[k][tx + 16];
      acc[0][0] = fmaf(a0, b0, acc[0][0]);
      acc[0][1] = fmaf(a0, b1, acc[0][1]);
      acc[1][0] = fmaf(a1, b0, acc[1][0]);
      acc[1][1] = fmaf(a1, b1, acc[1][1]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int m = m0 + ty + 16 * i, n = n0 + tx + 16 * j;
      if (m < M && n < N) ep(m, n, acc[i][j]);
    }
}

struct EpBiasRelu {
  const float* b; float* z; float* y; int N;
  __device__ void operator()(int m, int n, float v) const {
    v += b[n];
    z[(size_t)m * N + n] = v;
    y[(size_t)m * N + n] = v > 0.f ? v : 0.f;
  }
};
struct EpStore {
  float* c; int N;
  __device__ void operator()(int m, int n, float v) const { c[(size_t)m * N + n] = v; }
};

// dz = dy * (z > 0)
__global__ void relu_mask_kernel(const float* __restrict__ z, const float* __restrict__ dy, float* __restrict__ dz, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dz[i] = z[i] > 0.f ? dy[i] : 0.f;
}

// db[n] = sum_m dz[m,n], rows in ascending order
__global__ void colsum_kernel(const float* __restrict__ dz, float* __restrict__ db, int M, int N) {
  int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float s = 0.f;
  for (int m = 0; m < M; ++m) s += dz[(size_t)m * N + n];
  db[n] = s;
}

// stage 1 of the loss: dy and per-block partial sums of (y - t)^2
__global__ __launch_bounds__(256) void mse_partial_kernel(const float* __restrict__ y, const float* __restrict__ t,
                                                           float* __restrict__ dy, float* __restrict__ partial, size_t n) {
  __shared__ float red[256];
  float s = 0.f;
  const float scale = 2.0f / (float)n;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    float d = y[i] - t[i];
    s = fmaf(d, d, s);
    dy[i] = d * scale;
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// stage 2: fixed-order sum of up to 1024 partials, scaled
__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ partial, int count, float scale,
                                                            float* __restrict__ out) {
  __shared__ float red[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < count; i += 256) s += partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0] * scale;
}

static inline dim3 tiles(int M, int N) { return dim3((N + TS - 1) / TS, (M + TS - 1) / TS); }

int linear_relu_fwd_f32(const float* x, const float* w, const float* b, float* z, float* y, int m, int n, int k,
                        hipStream_t s) {
  hipLaunchKernelGGL((gemm_f32_kernel<false, false, EpBiasRelu>), tiles(m, n), dim3(256), 0, s, x, w, m, n, k,
                     EpBiasRelu{b, z, y, n});
  return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP;
}

int linear_relu_bwd_f32(const float* x, const float* w, const float* z, const float* dy, float* dz, float* dx,
                        float* dw, float* db, int m, int n, int k, hipStream_t s) {
  size_t cnt = (size_t)m * n;
  hipLaunchKernelGGL(relu_mask_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, z, dy, dz, cnt);
  // dx[m,k] = sum_n dz[m,n] w[n,k]  -> A = dz [M,N] (reduction contiguous), B = w as [N,K] read transposed
  if (dx)
    hipLaunchKernelGGL((gemm_f32_kernel<false, true, EpStore>), tiles(m, k), dim3(256), 0, s, dz, w, m, k, n,
                       EpStore{dx, k});
  // dw[n,k] = sum_m dz[m,n] x[m,k] -> both operands read transposed, reduction over m
  hipLaunchKernelGGL((gemm_f32_kernel<true, true, EpStore>), tiles(n, k), dim3(256), 0, s, dz, x, n, k, m,
                     EpStore{dw, k});
  hipLaunchKernelGGL(colsum_kernel, dim3((n + 255) / 256), dim3(256), 0, s, dz, db, m, n);
  return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP;
}

int mse_f32(const float* y, const float* t, float* dy, float* loss, float* partial, size_t n, hipStream_t s) {
  int blocks = (int)std::min<size_t>(1024, (n + 255) / 256);
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(mse_partial_kernel, dim3(blocks), dim3(256), 0, s, y, t, dy, partial, n);
  hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, s, partial, blocks, 1.0f / (float)n, loss);
  return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP;
}

}  // namespace karma

using namespace karma;

extern "C" int karma_k_linear_relu_fwd_f32(const float* x, const float* w, const float* b, float* z, float* y,
                                           uint32_t m, uint32_t n, uint32_t k, void* stream) {
  if (!x || !w || !b || !z || !y || !m || !n || !k) return KARMA_E_INVAL;
  return linear_relu_fwd_f32(x, w, b, z, y, (int)m, (int)n, (int)k, (hipStream_t)stream);
}

extern "C" int karma_k_linear_relu_bwd_f32(const float* x, const float* w, const float* z, const float* dy,
                                           float* dz_ws, float* dx, float* dw, float* db, uint32_t m, uint32_t n,
                                           uint32_t k, void* stream) {
  if (!x || !w || !z || !dy || !dz_ws || !dw || !db || !m || !n || !k) return KARMA_E_INVAL;
  return linear_relu_bwd_f32(x, w, z, dy, dz_ws, dx, dw, db, (int)m, (int)n, (int)k, (hipStream_t)stream);
}

extern "C" int karma_k_mse_f32(const float* y, const float* t, float* dy, float* loss, float* partial_ws, uint64_t n,
                               void* stream) {
  if (!y || !t || !dy || !loss || !partial_ws || !n) return KARMA_E_INVAL;
  return mse_f32(y, t, dy, loss, partial_ws, (size_t)n, (hipStream_t)stream);
}
