// Dispatch of the model-specific layer ops by model kind.
#include "context.h"
#include "layers.h"

namespace karma {

#define KARMA_BY_KIND(call_mlp, call_gpt, call_cnn, call_wrn, call_unet) \
  switch (c.desc.kind) {                                      \
    case KARMA_MODEL_MLP: return call_mlp;                    \
    case KARMA_MODEL_GPT: return call_gpt;                    \
    case KARMA_MODEL_CNN: return call_cnn;                    \
    case KARMA_MODEL_WRN: return call_wrn;                    \
    case KARMA_MODEL_UNET: return call_unet;                  \
  }                                                           \
  return KARMA_E_INVAL

int model_build_records(Ctx& c) {
  KARMA_BY_KIND(mlp_build_records(c), gpt_build_records(c), cnn_build_records(c), wrn_build_records(c), unet_build_records(c));
}
int model_prepare_step(Ctx& c, const void* in, const void* lab) {
  KARMA_BY_KIND(mlp_prepare_step(c, in, lab), gpt_prepare_step(c, in, lab), cnn_prepare_step(c, in, lab),
                wrn_prepare_step(c, in, lab), unet_prepare_step(c, in, lab));
}
int model_prepare_late(Ctx& c) {
  KARMA_BY_KIND(mlp_prepare_late(c), gpt_prepare_late(c), cnn_prepare_late(c), wrn_prepare_late(c), unet_prepare_late(c));
}
int layer_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  KARMA_BY_KIND(mlp_forward(c, i, io, s), gpt_forward(c, i, io, s), cnn_forward(c, i, io, s), wrn_forward(c, i, io, s),
                unet_forward(c, i, io, s));
}
int layer_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  KARMA_BY_KIND(mlp_backward(c, i, io, s), gpt_backward(c, i, io, s), cnn_backward(c, i, io, s), wrn_backward(c, i, io, s),
                unet_backward(c, i, io, s));
}
int loss_op(Ctx& c, const LayerIO& io, hipStream_t s) {
  KARMA_BY_KIND(mlp_loss(c, io, s), gpt_loss(c, io, s), cnn_loss(c, io, s), wrn_loss(c, io, s), unet_loss(c, io, s));
}

}  // namespace karma
