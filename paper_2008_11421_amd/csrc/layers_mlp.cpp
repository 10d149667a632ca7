// MLP workload: L x (Linear + ReLU) in fp32 with a mean-squared-error loss.
// Per layer: input x_i [batch, width], internals = pre-activation z_i, output relu(z_i).
#include <cstring>

#include "kernels.h"
#include "layers.h"

namespace karma {

int mlp_build_records(Ctx& c) {
  const karma_model_desc& d = c.desc;
  if (!d.n_layers || !d.width || !d.batch) return KARMA_E_INVAL;
  const uint64_t act = (uint64_t)d.batch * d.width * sizeof(float);
  c.rec.clear();
  for (uint32_t i = 0; i < d.n_layers; ++i) {
    Record r;
    r.kind = REC_LINEAR_RELU;
    r.p.resize(2);
    r.p[0].n = (uint64_t)d.width * d.width;   // W [out, in]
    r.p[1].n = d.width;                       // b
    r.out_bytes = act;
    r.sav_bytes = act;   // z
    r.ws_bytes = act;    // dz in backward
    r.streamed = d.stream_weights != 0;
    c.rec.push_back(std::move(r));
  }
  Record loss;
  loss.kind = REC_LOSS_MSE;
  loss.ws_bytes = 1024 * sizeof(float);
  c.rec.push_back(std::move(loss));
  c.in_bytes = act;
  c.lab_bytes = act;
  c.misc_bytes = 0;
  return KARMA_OK;
}

int mlp_prepare_step(Ctx& c, const void* in, const void* lab) {
  std::memcpy(c.stage_in, in, c.in_bytes);
  std::memcpy(c.stage_lab, lab, c.lab_bytes);
  return KARMA_OK;
}

int mlp_prepare_late(Ctx&) { return KARMA_OK; }

int mlp_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  const int m = (int)c.desc.batch, n = (int)c.desc.width;
  // a recompute whose output is not needed still writes y somewhere: the workspace
  float* y = io.out ? (float*)io.out : (float*)io.ws;
  return linear_relu_fwd_f32((const float*)io.x, (const float*)c.w_ptr(i, 0, io.w), (const float*)c.w_ptr(i, 1, io.w),
                             (float*)io.sav, y, m, n, n, s);
}

int mlp_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  const int m = (int)c.desc.batch, n = (int)c.desc.width;
  return linear_relu_bwd_f32((const float*)io.x, (const float*)c.w_ptr(i, 0, io.w), (const float*)io.sav,
                             (const float*)io.dy, (float*)io.ws, (float*)io.dx, (float*)c.g_ptr(i, 0, io.g),
                             (float*)c.g_ptr(i, 1, io.g), m, n, n, s);
}

int mlp_loss(Ctx& c, const LayerIO& io, hipStream_t s) {
  const size_t n = (size_t)c.desc.batch * c.desc.width;
  return mse_f32((const float*)io.x, (const float*)c.fixed_ptr(c.lab_off), (float*)io.dx,
                 (float*)c.fixed_ptr(c.loss_off), (float*)io.ws, n, s);
}

}  // namespace karma
