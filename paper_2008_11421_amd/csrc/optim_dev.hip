// The optimiser's update as a device kernel, for parameters whose optimiser state lives in HBM
// (karma_config.device_update_first): the tensors of the first record are the last the backward
// pass completes and the first the next forward pass reads, so a host update of them (gradient
// copy out, update, weight copy back) cannot hide behind anything; updated where they are, the
// step has no such tail.  Same arithmetic as the host loops (csrc/host_optim_loops.h): fp32
// master weights and moments, bias-corrected Adam without weight decay, SGD with momentum
// without dampening, plain SGD; the device copy of the weight is rounded to nearest even.
#include <hip/hip_runtime.h>

#include <cmath>

#include "device_utils.h"
#include "karma.h"
#include "kernels.h"

namespace karma {
namespace {

template <int KIND, bool G_BF16, bool O_BF16>
__global__ __launch_bounds__(256) void optim_update_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                                                            const void* __restrict__ g, size_t n, float lr, float beta1,
                                                            float beta2, float eps, float c1, float c2, void* __restrict__ out) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const float gi = G_BF16 ? bf2f(((const bf16_t*)g)[i]) : ((const float*)g)[i];
    float nw;
    if (KIND == KARMA_OPT_ADAM) {
      const float mi = beta1 * m[i] + (1.0f - beta1) * gi;
      const float vi = beta2 * v[i] + (1.0f - beta2) * gi * gi;
      m[i] = mi;
      v[i] = vi;
      nw = w[i] - lr * (mi * c1) / (sqrtf(vi * c2) + eps);
    } else if (KIND == KARMA_OPT_SGD_MOMENTUM) {
      const float bi = beta1 * m[i] + gi;
      m[i] = bi;
      nw = w[i] - lr * bi;
    } else {
      nw = w[i] - lr * gi;
    }
    w[i] = nw;
    if (O_BF16) ((bf16_t*)out)[i] = f2bf(nw);
    else ((float*)out)[i] = nw;
  }
}

}  // namespace

int optim_update_dev(int kind, float* w, float* m, float* v, const void* g, bool g_bf16, size_t n, float lr, float beta1,
                     float beta2, float eps, uint64_t step, void* out, bool out_bf16, hipStream_t s) {
  if (!w || !g || !out || !n) return KARMA_E_INVAL;
  const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 16);
#define KARMA_OPT_LAUNCH(K, GB, OB) \
  hipLaunchKernelGGL((optim_update_kernel<K, GB, OB>), dim3(blocks), dim3(256), 0, s, w, m, v, g, n, lr, beta1, beta2, eps, c1, c2, out)
#define KARMA_OPT_FORMATS(K)                           \
  do {                                                 \
    if (g_bf16 && out_bf16) KARMA_OPT_LAUNCH(K, true, true);   \
    else if (g_bf16) KARMA_OPT_LAUNCH(K, true, false);         \
    else if (out_bf16) KARMA_OPT_LAUNCH(K, false, true);       \
    else KARMA_OPT_LAUNCH(K, false, false);                    \
  } while (0)
  if (kind == KARMA_OPT_ADAM) {
    if (!m || !v) return KARMA_E_INVAL;
    KARMA_OPT_FORMATS(KARMA_OPT_ADAM);
  } else if (kind == KARMA_OPT_SGD_MOMENTUM) {
    if (!m) return KARMA_E_INVAL;
    KARMA_OPT_FORMATS(KARMA_OPT_SGD_MOMENTUM);
  } else if (kind == KARMA_OPT_SGD) {
    KARMA_OPT_FORMATS(KARMA_OPT_SGD);
  } else {
    return KARMA_E_INVAL;
  }
#undef KARMA_OPT_FORMATS
#undef KARMA_OPT_LAUNCH
  return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP;
}

}  // namespace karma
