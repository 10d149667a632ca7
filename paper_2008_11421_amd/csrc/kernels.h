// Internal launchers of the HIP kernels (C++ side of the kernel-level C ABI).
// All pointers are device pointers; every launcher is asynchronous on `s` and returns a
// karma_status.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace karma {

typedef uint16_t bf16_t;   // bit pattern of a bfloat16

// ---- fp32 MLP kernels (kernels_f32.hip)
int linear_relu_fwd_f32(const float* x, const float* w, const float* b, float* z, float* y, int m, int n, int k,
                        hipStream_t s);
int linear_relu_bwd_f32(const float* x, const float* w, const float* z, const float* dy, float* dz, float* dx,
                        float* dw, float* db, int m, int n, int k, hipStream_t s);
int mse_f32(const float* y, const float* t, float* dy, float* loss, float* partial, size_t n, hipStream_t s);

// ---- bf16 GEMM on the matrix cores (gemm_bf16.hip)
// C[M,N] = sum_k A(m,k) B(n,k) (+ bias[n]) (+ residual[m,n]).  a_kc: A is [M][lda] with k
// contiguous, else [K][lda] with m contiguous; same for B with n.
struct GemmArgs {
  const bf16_t* A; const bf16_t* B; void* C;
  const bf16_t* bias; const bf16_t* residual;
  int M, N, K, lda, ldb, ldc;
  bool a_kc, b_kc, out_f32, accumulate;
};
int gemm_bf16(const GemmArgs& g, hipStream_t s);

}  // namespace karma
