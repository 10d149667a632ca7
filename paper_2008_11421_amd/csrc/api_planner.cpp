// C ABI of the pure planner functions declared in karma.h.
#include <cstring>

#include "planner.h"

using namespace karma;

static bool graph_ok(const karma_skip* skips, uint32_t n_skips, uint32_t n_layers) {
  return (n_skips == 0 || skips) && skips_valid(skips, n_skips, n_layers);
}

extern "C" int karma_simulate_graph(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                                    const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                                    const karma_skip* skips, uint32_t n_skips, const uint8_t* actions,
                                    const uint8_t* weights_kept, karma_plan_summary* summary_out, karma_op* ops_out,
                                    uint32_t* n_ops_inout) {
  if (!layers || !n_layers || !link || !loss || !actions || !link->bw_h2d || !link->bw_d2h) return KARMA_E_INVAL;
  if (ops_out && !n_ops_inout) return KARMA_E_INVAL;
  if (!graph_ok(skips, n_skips, n_layers) || !actions_valid(actions, n_layers, skips, n_skips)) return KARMA_E_INVAL;
  Problem P{layers, n_layers, *link, *loss, budget_bytes, fixed_bytes, skips, n_skips};
  std::vector<karma_op> ops;
  karma_plan_summary s;
  if (!simulate(P, actions, weights_kept, &s, ops_out ? &ops : nullptr)) return KARMA_E_BUDGET;
  if (summary_out) *summary_out = s;
  if (ops_out) {
    if (ops.size() > *n_ops_inout) { *n_ops_inout = (uint32_t)ops.size(); return KARMA_E_OOM; }
    std::memcpy(ops_out, ops.data(), ops.size() * sizeof(karma_op));
    *n_ops_inout = (uint32_t)ops.size();
  }
  return KARMA_OK;
}

extern "C" int karma_simulate(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                              const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                              const uint8_t* actions, const uint8_t* weights_kept, karma_plan_summary* summary_out,
                              karma_op* ops_out, uint32_t* n_ops_inout) {
  return karma_simulate_graph(layers, n_layers, link, loss, budget_bytes, fixed_bytes, nullptr, 0, actions, weights_kept,
                              summary_out, ops_out, n_ops_inout);
}

extern "C" int karma_plan_graph(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                                const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                                const karma_skip* skips, uint32_t n_skips, uint8_t* actions_out,
                                uint8_t* weights_kept_out, karma_plan_summary* summary_out) {
  if (!layers || !n_layers || !link || !loss || !actions_out || !link->bw_h2d || !link->bw_d2h) return KARMA_E_INVAL;
  if (!graph_ok(skips, n_skips, n_layers)) return KARMA_E_INVAL;
  Problem P{layers, n_layers, *link, *loss, budget_bytes, fixed_bytes, skips, n_skips};
  std::vector<uint8_t> a, kw;
  karma_plan_summary s;
  if (!plan(P, a, kw, &s)) return KARMA_E_BUDGET;
  std::memcpy(actions_out, a.data(), n_layers);
  if (weights_kept_out) std::memcpy(weights_kept_out, kw.data(), n_layers);
  if (summary_out) *summary_out = s;
  return KARMA_OK;
}

extern "C" int karma_plan_pure(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                               const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                               uint8_t* actions_out, uint8_t* weights_kept_out, karma_plan_summary* summary_out) {
  return karma_plan_graph(layers, n_layers, link, loss, budget_bytes, fixed_bytes, nullptr, 0, actions_out,
                          weights_kept_out, summary_out);
}

extern "C" int karma_plan_grouped_graph(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                                        const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                                        const karma_skip* skips, uint32_t n_skips, uint32_t max_group,
                                        uint8_t* actions_out, uint8_t* weights_kept_out,
                                        karma_plan_summary* summary_out, uint32_t* group_out) {
  if (!layers || !n_layers || !link || !loss || !actions_out || !link->bw_h2d || !link->bw_d2h || !max_group) return KARMA_E_INVAL;
  if (!graph_ok(skips, n_skips, n_layers)) return KARMA_E_INVAL;
  Problem P{layers, n_layers, *link, *loss, budget_bytes, fixed_bytes, skips, n_skips};
  std::vector<uint8_t> a, kw;
  karma_plan_summary s;
  uint32_t g = 1;
  if (!plan_grouped(P, max_group, a, kw, &s, &g)) return KARMA_E_BUDGET;
  std::memcpy(actions_out, a.data(), n_layers);
  if (weights_kept_out) std::memcpy(weights_kept_out, kw.data(), n_layers);
  if (summary_out) *summary_out = s;
  if (group_out) *group_out = g;
  return KARMA_OK;
}

extern "C" int karma_plan_grouped_pure(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                                       const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                                       uint32_t max_group, uint8_t* actions_out, uint8_t* weights_kept_out,
                                       karma_plan_summary* summary_out, uint32_t* group_out) {
  return karma_plan_grouped_graph(layers, n_layers, link, loss, budget_bytes, fixed_bytes, nullptr, 0, max_group,
                                  actions_out, weights_kept_out, summary_out, group_out);
}

extern "C" int karma_stage_string(const karma_op* ops, uint32_t n_ops, char* buf, size_t buf_len) {
  if (!ops || !buf) return KARMA_E_INVAL;
  std::string s = stage_string(ops, n_ops);
  if (s.size() + 1 > buf_len) return KARMA_E_OOM;
  std::memcpy(buf, s.c_str(), s.size() + 1);
  return KARMA_OK;
}
