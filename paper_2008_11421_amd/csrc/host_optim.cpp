#include "host_optim.h"
#include "karma.h"

#include <cmath>
#include <cstring>

namespace karma {

HostPool::HostPool(unsigned threads) {
  if (threads < 1) threads = 1;
  for (unsigned i = 1; i < threads; ++i) workers_.emplace_back([this, i] { worker(i); });
}

HostPool::~HostPool() {
  {
    std::lock_guard<std::mutex> lk(mu_);
    stop_ = true;
  }
  cv_.notify_all();
  for (auto& t : workers_) t.join();
}

void HostPool::worker(unsigned id) {
  uint64_t seen = 0;
  for (;;) {
    const std::function<void(size_t, size_t)>* fn;
    size_t n;
    {
      std::unique_lock<std::mutex> lk(mu_);
      cv_.wait(lk, [&] { return stop_ || epoch_ != seen; });
      if (stop_) return;
      seen = epoch_;
      fn = fn_;
      n = n_;
    }
    unsigned parts = size();
    size_t chunk = (n + parts - 1) / parts;
    chunk = (chunk + 63) / 64 * 64;
    size_t lo = std::min(n, (size_t)id * chunk), hi = std::min(n, lo + chunk);
    if (lo < hi) (*fn)(lo, hi);
    {
      std::lock_guard<std::mutex> lk(mu_);
      if (--pending_ == 0) done_cv_.notify_one();
    }
  }
}

void HostPool::parallel_for(size_t n, const std::function<void(size_t, size_t)>& fn) {
  unsigned parts = size();
  if (parts == 1 || n < 16384) {
    fn(0, n);
    return;
  }
  {
    std::lock_guard<std::mutex> lk(mu_);
    fn_ = &fn;
    n_ = n;
    pending_ = parts - 1;
    ++epoch_;
  }
  cv_.notify_all();
  size_t chunk = (n + parts - 1) / parts;
  chunk = (chunk + 63) / 64 * 64;
  size_t hi = std::min(n, chunk);
  if (hi > 0) fn(0, hi);
  std::unique_lock<std::mutex> lk(mu_);
  done_cv_.wait(lk, [&] { return pending_ == 0; });
}

float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace karma

#define HOST_OPTIM_NS avx2
#include "host_optim_loops.h"
#undef HOST_OPTIM_NS

namespace karma {

// the same loops built for AVX-512 (host_optim_avx512.cpp)
namespace avx512 {
void sgd_update(float* w, const void* g, bool g_is_bf16, size_t n, float lr, void* out, bool out_is_bf16);
void sgd_momentum_update(float* w, float* buf, const void* g, bool g_is_bf16, size_t n, float lr, float mu, void* out,
                         bool out_is_bf16);
void adam_update(float* w, float* m, float* v, const void* g, bool g_is_bf16, size_t n, float lr, float beta1, float beta2,
                 float eps, float c1, float c2, void* out, bool out_is_bf16);
}  // namespace avx512

static bool g_force_narrow = false;
void host_optim_force_narrow(bool on) { g_force_narrow = on; }

static bool wide_vectors() {
  static const bool yes = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
                          __builtin_cpu_supports("avx512vl") && __builtin_cpu_supports("avx512dq");
  return yes && !g_force_narrow;
}

void sgd_momentum_update(float* w, float* buf, const void* g, bool g_is_bf16, size_t n, float lr, float mu, void* out,
                         bool out_is_bf16) {
  if (wide_vectors()) avx512::sgd_momentum_update(w, buf, g, g_is_bf16, n, lr, mu, out, out_is_bf16);
  else avx2::sgd_momentum_entry(w, buf, g, g_is_bf16, n, lr, mu, out, out_is_bf16);
}

void sgd_update(float* w, const void* g, bool g_is_bf16, size_t n, float lr, void* out, bool out_is_bf16) {
  if (wide_vectors()) avx512::sgd_update(w, g, g_is_bf16, n, lr, out, out_is_bf16);
  else avx2::sgd_entry(w, g, g_is_bf16, n, lr, out, out_is_bf16);
}

void adam_update(float* w, float* m, float* v, const void* g, bool g_is_bf16, size_t n, float lr, float beta1,
                 float beta2, float eps, uint64_t step, void* out, bool out_is_bf16) {
  const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  if (wide_vectors()) avx512::adam_update(w, m, v, g, g_is_bf16, n, lr, beta1, beta2, eps, c1, c2, out, out_is_bf16);
  else avx2::adam_entry(w, m, v, g, g_is_bf16, n, lr, beta1, beta2, eps, c1, c2, out, out_is_bf16);
}

}  // namespace karma

// One update of n parameters through the same loops the executor uses per record.
extern "C" int karma_host_update(uint32_t optimizer, float* master, float* m, float* v, const void* grad,
                                 uint32_t grad_is_bf16, uint64_t n, float lr, float beta1, float beta2, float eps,
                                 uint64_t step, void* out, uint32_t out_is_bf16, uint32_t narrow_vectors) {
  using namespace karma;
  if (!master || !grad || !out) return KARMA_E_INVAL;
  if (grad == out && (grad_is_bf16 != 0) != (out_is_bf16 != 0)) return KARMA_E_INVAL;   // in place needs equal element types
  host_optim_force_narrow(narrow_vectors != 0);
  int st = KARMA_OK;
  if (optimizer == KARMA_OPT_SGD) sgd_update(master, grad, grad_is_bf16 != 0, (size_t)n, lr, out, out_is_bf16 != 0);
  else if (optimizer == KARMA_OPT_SGD_MOMENTUM && m)
    sgd_momentum_update(master, m, grad, grad_is_bf16 != 0, (size_t)n, lr, beta1, out, out_is_bf16 != 0);
  else if (optimizer == KARMA_OPT_ADAM && m && v && step >= 1)
    adam_update(master, m, v, grad, grad_is_bf16 != 0, (size_t)n, lr, beta1, beta2, eps, step, out, out_is_bf16 != 0);
  else st = KARMA_E_INVAL;
  host_optim_force_narrow(false);
  return st;
}
