// The host optimiser's update loops built for AVX-512 (this file alone is compiled with the
// AVX-512 target features; host_optim.cpp calls in here only when the CPU has them).
#define HOST_OPTIM_NS avx512_impl
#include "host_optim_loops.h"
#undef HOST_OPTIM_NS

namespace karma {
namespace avx512 {

void sgd_update(float* w, const void* g, bool g_is_bf16, size_t n, float lr, void* out, bool out_is_bf16) {
  avx512_impl::sgd_entry(w, g, g_is_bf16, n, lr, out, out_is_bf16);
}
void sgd_momentum_update(float* w, float* buf, const void* g, bool g_is_bf16, size_t n, float lr, float mu, void* out,
                         bool out_is_bf16) {
  avx512_impl::sgd_momentum_entry(w, buf, g, g_is_bf16, n, lr, mu, out, out_is_bf16);
}
void adam_update(float* w, float* m, float* v, const void* g, bool g_is_bf16, size_t n, float lr, float beta1, float beta2,
                 float eps, float c1, float c2, void* out, bool out_is_bf16) {
  avx512_impl::adam_entry(w, m, v, g, g_is_bf16, n, lr, beta1, beta2, eps, c1, c2, out, out_is_bf16);
}

}  // namespace avx512
}  // namespace karma
