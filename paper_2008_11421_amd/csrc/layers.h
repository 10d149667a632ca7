#pragma once
#include "context.h"

namespace karma {
int mlp_build_records(Ctx& c);
int mlp_prepare_step(Ctx& c, const void* in, const void* lab);
int mlp_prepare_late(Ctx& c);
int mlp_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int mlp_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int mlp_loss(Ctx& c, const LayerIO& io, hipStream_t s);

int gpt_build_records(Ctx& c);
int gpt_prepare_step(Ctx& c, const void* in, const void* lab);
int gpt_prepare_late(Ctx& c);
int gpt_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int gpt_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int gpt_loss(Ctx& c, const LayerIO& io, hipStream_t s);

int cnn_build_records(Ctx& c);
int cnn_prepare_step(Ctx& c, const void* in, const void* lab);
int cnn_prepare_late(Ctx& c);
int cnn_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int cnn_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int cnn_loss(Ctx& c, const LayerIO& io, hipStream_t s);

int wrn_build_records(Ctx& c);
int wrn_prepare_step(Ctx& c, const void* in, const void* lab);
int wrn_prepare_late(Ctx& c);
int wrn_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int wrn_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int wrn_loss(Ctx& c, const LayerIO& io, hipStream_t s);

int unet_build_records(Ctx& c);   // also fills c.skips
int unet_skips(const karma_model_desc& d, std::vector<karma_skip>& out);
int unet_prepare_step(Ctx& c, const void* in, const void* lab);
int unet_prepare_late(Ctx& c);
int unet_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int unet_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int unet_loss(Ctx& c, const LayerIO& io, hipStream_t s);
}  // namespace karma
