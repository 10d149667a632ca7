// GPT workload (placeholder until the bf16 kernels land).
#include "layers.h"

namespace karma {
int gpt_build_records(Ctx&) { return KARMA_E_INVAL; }
int gpt_prepare_step(Ctx&, const void*, const void*) { return KARMA_E_INVAL; }
int gpt_forward(Ctx&, uint32_t, const LayerIO&, hipStream_t) { return KARMA_E_INVAL; }
int gpt_backward(Ctx&, uint32_t, const LayerIO&, hipStream_t) { return KARMA_E_INVAL; }
int gpt_loss(Ctx&, const LayerIO&, hipStream_t) { return KARMA_E_INVAL; }
}  // namespace karma
