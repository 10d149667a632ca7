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

}  // namespace karma
