// Dispatch of the model-specific layer ops by model kind.
#include "context.h"
#include "layers.h"

namespace karma {

int model_build_records(Ctx& c) {
  switch (c.desc.kind) {
    case KARMA_MODEL_MLP: return mlp_build_records(c);
    case KARMA_MODEL_GPT: return gpt_build_records(c);
  }
  return KARMA_E_INVAL;
}
int model_prepare_step(Ctx& c, const void* in, const void* lab) {
  return c.desc.kind == KARMA_MODEL_MLP ? mlp_prepare_step(c, in, lab) : gpt_prepare_step(c, in, lab);
}
int model_prepare_late(Ctx& c) { return c.desc.kind == KARMA_MODEL_MLP ? mlp_prepare_late(c) : gpt_prepare_late(c); }
int layer_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  return c.desc.kind == KARMA_MODEL_MLP ? mlp_forward(c, i, io, s) : gpt_forward(c, i, io, s);
}
int layer_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  return c.desc.kind == KARMA_MODEL_MLP ? mlp_backward(c, i, io, s) : gpt_backward(c, i, io, s);
}
int loss_op(Ctx& c, const LayerIO& io, hipStream_t s) {
  return c.desc.kind == KARMA_MODEL_MLP ? mlp_loss(c, io, s) : gpt_loss(c, io, s);
}

}  // namespace karma
