// Analytic cost model (KARMA Sec. III-C, III-D): the cost of a block is the number of
// arithmetic operations of its layers, projected on the device's throughput; its memory
// comes from the shapes.  With it the planner runs without any measurement on a GPU, e.g. to
// project how a model behaves across batch sizes (the x-axis of Fig. 5).
//
// Operation counts per sample as Sec. III-C lists them (one multiply-add = one operation):
// convolution |Y| K K C_in; ReLU |Y|; pooling |Y| K K (global average pooling: one per input
// element); batch normalisation 3|B| + 4|X| + 2|Y| = 9 per element; fully connected |X| |Y|;
// softmax 2|X|; element-wise operations and tensor adds one per element.  Where the paper
// gives nothing usable: self-attention is counted as S S d multiply-adds for Q K^T and for
// P V per head plus a softmax over the S S scores (the printed count has no sequence
// length), layer normalisation like batch normalisation, GELU and the embedding as
// element-wise, cross entropy as a softmax.  Backward = twice forward, recompute = forward,
// the loss op = three times its forward count (its gradients are part of it).
// Matrix operations (convolutions, fully connected layers, the attention products) and the
// rest are kept apart because the device runs them at different rates.
#include <cstring>
#include <utility>
#include <vector>

#include "context.h"
#include "karma.h"

namespace karma {
namespace {

typedef std::pair<uint64_t, uint64_t> Ops;   // matrix operations, other operations

int out_dim(int n, int k, int stride, int pad) { return (n + 2 * pad - k) / stride + 1; }

void count_mlp(const karma_model_desc& d, std::vector<Ops>& blocks, Ops& loss) {
  const uint64_t b = d.batch, w = d.width;
  for (uint32_t i = 0; i < d.n_layers; ++i) blocks.push_back(Ops(b * w * w, b * w));   // Linear + ReLU
  loss = Ops(0, b * w);                                                                // squared error per element
}

void count_gpt(const karma_model_desc& d, std::vector<Ops>& blocks, Ops& loss) {
  const uint64_t B = d.batch, S = d.seq, h = d.width, H = d.n_heads, f = d.ffn, V = d.vocab;
  const uint64_t T = B * S, dk = h / H;
  blocks.push_back(Ops(0, T * h));   // token + position embedding
  // attention half: layer normalisation, QKV and output projections, the two attention products, the
  // softmax of the scores, a residual add; feed-forward half: layer normalisation, FC1, GELU, FC2, residual add
  const Ops attn(T * (3 * h * h + h * h) + B * H * 2 * S * S * dk, 9 * T * h + B * H * 2 * S * S + T * h);
  const Ops ffn(T * 2 * h * f, 9 * T * h + T * f + T * h);
  for (uint32_t i = 0; i < d.n_layers; ++i) {
    if (d.split_blocks) {
      blocks.push_back(attn);
      blocks.push_back(ffn);
    } else {
      blocks.push_back(Ops(attn.first + ffn.first, attn.second + ffn.second));
    }
  }
  loss = Ops(T * h * V, 9 * T * h + 2 * T * V);   // final layer norm, tied LM head, softmax cross entropy
}

void count_cnn(const karma_model_desc& d, std::vector<Ops>& blocks, Ops& loss) {
  const uint64_t N = d.batch, width = d.width;
  const int h1 = out_dim((int)d.seq, 7, 2, 3), h2 = out_dim(h1, 3, 2, 1);
  const uint64_t y0 = N * h1 * h1 * width;
  // stem: 7x7 convolution over 3 channels, batch norm, ReLU, 3x3 max pooling
  blocks.push_back(Ops(y0 * 49 * 3, 9 * y0 + y0 + N * h2 * h2 * width * 9));
  int hw = h2;
  uint64_t cin = width;
  for (int st = 0; st < 4; ++st) {
    const uint64_t mid = width << st, cout = 4 * mid;
    for (uint32_t k = 0; k < d.stage_blocks[st]; ++k) {
      const int stride = (k == 0 && st > 0) ? 2 : 1;
      const int ho = out_dim(hw, 3, stride, 1);
      const uint64_t pin = N * hw * hw, pout = N * ho * ho;
      uint64_t m = pin * mid * cin + pout * mid * 9 * mid + pout * cout * mid;
      uint64_t o = 10 * pin * mid + 10 * pout * mid + 9 * pout * cout;   // batch norm (9) + ReLU (1) twice, batch norm
      if (k == 0) {   // projection shortcut: 1x1 convolution and its batch norm
        m += pout * cout * cin;
        o += 9 * pout * cout;
      }
      o += 2 * pout * cout;   // residual add, ReLU
      blocks.push_back(Ops(m, o));
      hw = ho;
      cin = cout;
    }
  }
  loss = Ops(N * cin * d.vocab, N * hw * hw * cin + 2 * N * d.vocab);   // average pooling, FC, softmax cross entropy
}

// Wide residual network: first 3x3 convolution; basic blocks (batch norm + ReLU on the input, 3x3 convolution
// carrying the stride, batch norm + ReLU, 3x3 convolution, residual add; 1x1 shortcut convolution where the shape
// changes); loss record: batch norm, ReLU, average pooling, FC, softmax cross entropy.
void count_wrn(const karma_model_desc& d, std::vector<Ops>& blocks, Ops& loss) {
  const uint64_t N = d.batch;
  int hw = (int)d.seq;
  uint64_t cin = 16;
  blocks.push_back(Ops(N * hw * hw * cin * 9 * 3, 0));
  for (int gr = 0; gr < 3; ++gr) {
    const uint64_t cout = (uint64_t)d.width << gr;
    for (uint32_t k = 0; k < d.stage_blocks[gr]; ++k) {
      const int stride = (k == 0 && gr > 0) ? 2 : 1;
      const int ho = out_dim(hw, 3, stride, 1);
      const uint64_t pin = N * hw * hw, pout = N * ho * ho;
      uint64_t m = pout * cout * 9 * cin + pout * cout * 9 * cout;
      const uint64_t o = 10 * pin * cin + 10 * pout * cout + pout * cout;
      if (cin != cout) m += pout * cout * cin;
      blocks.push_back(Ops(m, o));
      hw = ho;
      cin = cout;
    }
  }
  const uint64_t pix = N * hw * hw;
  loss = Ops(N * cin * d.vocab, 10 * pix * cin + pix * cin + 2 * N * d.vocab);
}

// Fully convolutional network: contracting levels (2x2 max pooling except at level 0, then twice 3x3 convolution,
// batch norm, ReLU), expansive levels (2x2 up-convolution: every fine pixel takes one tap, |Y| C_in; then the two
// convolutions, the first over twice the channels), loss record: 1x1 classifier, softmax cross entropy per pixel.
void count_unet(const karma_model_desc& d, std::vector<Ops>& blocks, Ops& loss) {
  const uint64_t N = d.batch, D = d.n_layers;
  auto pixels = [&](uint64_t l) { return N * (d.seq >> l) * (d.seq >> l); };
  auto chans = [&](uint64_t l) { return (uint64_t)d.width << l; };
  for (uint64_t l = 0; l <= D; ++l) {
    const uint64_t p = pixels(l), c = chans(l), cin = l ? chans(l - 1) : 1;
    blocks.push_back(Ops(p * c * 9 * cin + p * c * 9 * c, (l ? p * cin * 4 : 0) + 20 * p * c));
  }
  for (uint64_t l = D; l-- > 0;) {
    const uint64_t p = pixels(l), c = chans(l);
    blocks.push_back(Ops(p * c * chans(l + 1) + p * c * 9 * 2 * c + p * c * 9 * c, 20 * p * c));
  }
  loss = Ops(pixels(0) * chans(0) * d.vocab, 2 * pixels(0) * d.vocab);
}

// ceil(ops * 1e9 / rate) with a 128-bit intermediate
int64_t ops_time_ns(uint64_t ops, uint64_t rate) {
  const unsigned __int128 num = (unsigned __int128)ops * 1000000000ull;
  return (int64_t)((num + rate - 1) / rate);
}
int64_t time_ns(const Ops& o, const karma_device_rates& r) { return ops_time_ns(o.first, r.matrix_ops_per_s) + ops_time_ns(o.second, r.other_ops_per_s); }

}  // namespace
}  // namespace karma

using namespace karma;

extern "C" int karma_model_costs(const karma_model_desc* desc, const karma_device_rates* rates, karma_layer_cost* layers_out,
                                 uint32_t* n_inout, karma_loss_cost* loss_out, uint64_t* fixed_out) {
  if (!desc || !rates || !layers_out || !n_inout || !rates->matrix_ops_per_s || !rates->other_ops_per_s) return KARMA_E_INVAL;
  Ctx c;
  c.desc = *desc;
  int st = derive_layout(c);
  if (st) return st;
  if (*n_inout < c.L) {
    *n_inout = c.L;
    return KARMA_E_OOM;
  }
  std::vector<Ops> blocks;
  Ops loss;
  if (desc->kind == KARMA_MODEL_MLP) count_mlp(*desc, blocks, loss);
  else if (desc->kind == KARMA_MODEL_GPT) count_gpt(*desc, blocks, loss);
  else if (desc->kind == KARMA_MODEL_CNN) count_cnn(*desc, blocks, loss);
  else if (desc->kind == KARMA_MODEL_WRN) count_wrn(*desc, blocks, loss);
  else if (desc->kind == KARMA_MODEL_UNET) count_unet(*desc, blocks, loss);
  else return KARMA_E_INVAL;
  if (blocks.size() != c.L) return KARMA_E_STATE;
  for (uint32_t i = 0; i < c.L; ++i) {
    karma_layer_cost k = c.cost[i];
    k.tf_ns = time_ns(blocks[i], *rates);
    k.tb_ns = 2 * k.tf_ns;
    k.trc_ns = k.tf_ns;
    k.th_ns = 0;   // the analytic model prices the device and the link, not the host optimiser
    k.hg_bytes = k.hw_bytes = 0;
    layers_out[i] = k;
  }
  *n_inout = c.L;
  if (loss_out) *loss_out = karma_loss_cost{3 * time_ns(loss, *rates), c.loss_cost.ws_bytes, 0, 0, 0};
  if (fixed_out) *fixed_out = c.fixed_bytes;
  return KARMA_OK;
}
