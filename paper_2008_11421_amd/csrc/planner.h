// Host-side planner internals shared by the C ABI wrappers and the executor.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "karma.h"

namespace karma {

struct Problem {
  const karma_layer_cost* layers;
  uint32_t n;
  karma_link link;
  karma_loss_cost loss;
  uint64_t budget, fixed;
  // connections between non-consecutive layers: the output of layer src is read again by layer dst
  const karma_skip* skips = nullptr;
  uint32_t n_skips = 0;
};

// Two-ended first-fit allocator with a coalescing hole list.  Long-lived buffers come
// from the low end, short-lived ones from the high end.
struct Arena {
  struct Hole { int64_t off, size; };
  std::vector<Hole> holes;
  int64_t cap = 0, used = 0, peak = 0;
  void reset(int64_t capacity);
  int64_t take(int64_t size, bool low);   // -1 when nothing fits
  void give(int64_t off, int64_t size);
};

int64_t copy_ns(uint64_t bytes, uint64_t bw, int64_t lat);
// a chained layer drops its input: the input of a layer that is read again (skips[k].src + 1) cannot be chained
bool actions_valid(const uint8_t* a, uint32_t n, const karma_skip* skips = nullptr, uint32_t n_skips = 0);
bool skips_valid(const karma_skip* skips, uint32_t n_skips, uint32_t n);
// keepw: per layer, streamed weights stay in HBM from F_i to B_i (null = no layer keeps them)
bool simulate(const Problem& P, const uint8_t* actions, const uint8_t* keepw, karma_plan_summary* out,
              std::vector<karma_op>* ops);
bool plan(const Problem& P, std::vector<uint8_t>& actions, std::vector<uint8_t>& keepw, karma_plan_summary* out);
bool plan_grouped(const Problem& P, uint32_t max_group, std::vector<uint8_t>& actions, std::vector<uint8_t>& keepw,
                  karma_plan_summary* out, uint32_t* group_out);
std::string stage_string(const karma_op* ops, uint32_t n);

}  // namespace karma
