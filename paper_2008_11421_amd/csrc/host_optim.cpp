#include "host_optim.h"

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

// The update loops are instantiated per gradient / output format so that the inner loop is
// branch-free and the compiler can vectorise it (AVX2 + FMA).
template <bool G_BF16>
static inline float load_g(const void* g, size_t i) {
  if (G_BF16) {
    uint32_t u = (uint32_t)((const uint16_t*)g)[i] << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
  }
  return ((const float*)g)[i];
}
template <bool O_BF16>
static inline void store_w(void* out, size_t i, float w) {
  if (O_BF16) {
    uint32_t u;
    std::memcpy(&u, &w, 4);
    uint32_t r = u + 0x7fffu + ((u >> 16) & 1u);
    // NaN stays NaN (quiet bit set); weights are finite in practice, the select keeps the loop branch-free
    uint32_t is_nan = (u & 0x7fffffffu) > 0x7f800000u ? 0xffffffffu : 0u;
    r = (r & ~is_nan) | ((u | 0x400000u) & is_nan);
    ((uint16_t*)out)[i] = (uint16_t)(r >> 16);
  } else {
    ((float*)out)[i] = w;
  }
}

template <bool G_BF16, bool O_BF16>
static void sgd_loop(float* __restrict__ w, const void* __restrict__ g, size_t n, float lr, void* __restrict__ out) {
  for (size_t i = 0; i < n; ++i) {
    float nw = w[i] - lr * load_g<G_BF16>(g, i);
    w[i] = nw;
    store_w<O_BF16>(out, i, nw);
  }
}

template <bool G_BF16, bool O_BF16>
static void adam_loop(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v, const void* __restrict__ g,
                      size_t n, float lr, float beta1, float beta2, float eps, float c1, float c2,
                      void* __restrict__ out) {
  const float ob1 = 1.0f - beta1, ob2 = 1.0f - beta2;
  for (size_t i = 0; i < n; ++i) {
    float gi = load_g<G_BF16>(g, i);
    float mi = beta1 * m[i] + ob1 * gi;
    float vi = beta2 * v[i] + ob2 * gi * gi;
    m[i] = mi;
    v[i] = vi;
    float nw = w[i] - lr * (mi * c1) / (std::sqrt(vi * c2) + eps);
    w[i] = nw;
    store_w<O_BF16>(out, i, nw);
  }
}

template <bool G_BF16, bool O_BF16>
static void sgd_momentum_loop(float* __restrict__ w, float* __restrict__ buf, const void* __restrict__ g, size_t n, float lr,
                              float mu, void* __restrict__ out) {
  for (size_t i = 0; i < n; ++i) {
    float bi = mu * buf[i] + load_g<G_BF16>(g, i);
    buf[i] = bi;
    float nw = w[i] - lr * bi;
    w[i] = nw;
    store_w<O_BF16>(out, i, nw);
  }
}

void sgd_momentum_update(float* w, float* buf, const void* g, bool g_is_bf16, size_t n, float lr, float mu, void* out,
                         bool out_is_bf16) {
  if (g_is_bf16) {
    if (out_is_bf16) sgd_momentum_loop<true, true>(w, buf, g, n, lr, mu, out);
    else sgd_momentum_loop<true, false>(w, buf, g, n, lr, mu, out);
  } else {
    if (out_is_bf16) sgd_momentum_loop<false, true>(w, buf, g, n, lr, mu, out);
    else sgd_momentum_loop<false, false>(w, buf, g, n, lr, mu, out);
  }
}

void sgd_update(float* w, const void* g, bool g_is_bf16, size_t n, float lr, void* out, bool out_is_bf16) {
  if (g_is_bf16) {
    if (out_is_bf16) sgd_loop<true, true>(w, g, n, lr, out); else sgd_loop<true, false>(w, g, n, lr, out);
  } else {
    if (out_is_bf16) sgd_loop<false, true>(w, g, n, lr, out); else sgd_loop<false, false>(w, g, n, lr, out);
  }
}

void adam_update(float* w, float* m, float* v, const void* g, bool g_is_bf16, size_t n, float lr, float beta1,
                 float beta2, float eps, uint64_t step, void* out, bool out_is_bf16) {
  const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  if (g_is_bf16) {
    if (out_is_bf16) adam_loop<true, true>(w, m, v, g, n, lr, beta1, beta2, eps, c1, c2, out);
    else adam_loop<true, false>(w, m, v, g, n, lr, beta1, beta2, eps, c1, c2, out);
  } else {
    if (out_is_bf16) adam_loop<false, true>(w, m, v, g, n, lr, beta1, beta2, eps, c1, c2, out);
    else adam_loop<false, false>(w, m, v, g, n, lr, beta1, beta2, eps, c1, c2, out);
  }
}

}  // namespace karma
