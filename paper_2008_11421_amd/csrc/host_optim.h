// Host-side optimiser on fp32 master weights (KARMA Sec. III-G, pipeline stage 5: the
// weights of a block are updated on the CPU once its gradients have been moved out).
#pragma once
#include <condition_variable>
#include <cstddef>
#include <cstdint>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace karma {

// Persistent worker pool; parallel_for splits [0, n) into one contiguous range per worker.
class HostPool {
 public:
  explicit HostPool(unsigned threads);
  ~HostPool();
  void parallel_for(size_t n, const std::function<void(size_t, size_t)>& fn);
  unsigned size() const { return (unsigned)workers_.size() + 1; }

 private:
  void worker(unsigned id);
  std::vector<std::thread> workers_;
  std::mutex mu_;
  std::condition_variable cv_, done_cv_;
  const std::function<void(size_t, size_t)>* fn_ = nullptr;
  size_t n_ = 0;
  uint64_t epoch_ = 0;
  unsigned pending_ = 0;
  bool stop_ = false;
};

float bf16_to_f32(uint16_t b);
uint16_t f32_to_bf16_rne(float f);

// w -= lr * g ; new weights also written in device format to `out`.
void sgd_update(float* w, const void* g, bool g_is_bf16, size_t n, float lr, void* out, bool out_is_bf16);
// buf = mu * buf + g; w -= lr * buf (no dampening, no Nesterov)
void sgd_momentum_update(float* w, float* buf, const void* g, bool g_is_bf16, size_t n, float lr, float mu, void* out,
                         bool out_is_bf16);
// Bias-corrected Adam without weight decay; `step` counts from 1.
void adam_update(float* w, float* m, float* v, const void* g, bool g_is_bf16, size_t n, float lr, float beta1,
                 float beta2, float eps, uint64_t step, void* out, bool out_is_bf16);

}  // namespace karma
