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

static inline float load_g(const void* g, bool is_bf16, size_t i) {
  return is_bf16 ? bf16_to_f32(((const uint16_t*)g)[i]) : ((const float*)g)[i];
}
static inline void store_w(void* out, bool is_bf16, size_t i, float w) {
  if (is_bf16) ((uint16_t*)out)[i] = f32_to_bf16_rne(w);
  else ((float*)out)[i] = w;
}

void sgd_update(float* w, const void* g, bool g_is_bf16, size_t n, float lr, void* out, bool out_is_bf16) {
  for (size_t i = 0; i < n; ++i) {
    float nw = w[i] - lr * load_g(g, g_is_bf16, i);
    w[i] = nw;
    store_w(out, out_is_bf16, i, nw);
  }
}

void adam_update(float* w, float* m, float* v, const void* g, bool g_is_bf16, size_t n, float lr, float beta1,
                 float beta2, float eps, uint64_t step, void* out, bool out_is_bf16) {
  const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  const float ob1 = 1.0f - beta1, ob2 = 1.0f - beta2;
  for (size_t i = 0; i < n; ++i) {
    float gi = load_g(g, g_is_bf16, i);
    float mi = beta1 * m[i] + ob1 * gi;
    float vi = beta2 * v[i] + ob2 * gi * gi;
    m[i] = mi;
    v[i] = vi;
    float nw = w[i] - lr * (mi * c1) / (std::sqrt(vi * c2) + eps);
    w[i] = nw;
    store_w(out, out_is_bf16, i, nw);
  }
}

}  // namespace karma
