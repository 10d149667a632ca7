// Wide residual network (the WRN-28-10 row of KARMA's Table III) as layer records of the
// out-of-core executor: record 0 is the first 3x3 convolution (to 16 channels), records 1..
// are pre-activated basic blocks (batch norm, ReLU, 3x3 convolution carrying the stride,
// batch norm, ReLU, 3x3 convolution, residual sum; where the shape changes the shortcut is a
// 1x1 convolution of the activated input with the block's stride), the loss record is batch
// norm, ReLU, global average pooling, the fully connected layer and mean cross entropy.
// One record = one block of the paper: a block's input is its checkpoint, its saved set the
// two activated tensors the convolutions read, the first convolution's output and the batch
// statistics.  Activations are NHWC bf16.  No dropout between the convolutions.
#include <algorithm>
#include <cstring>

#include "context.h"
#include "kernels.h"
#include "layers.h"

namespace karma {
namespace {

inline uint64_t up256(uint64_t b) { return (b + 255) / 256 * 256; }
constexpr int IMG_C = 8;     // the three image channels are stored as eight (zeros), so that a pixel is 16 bytes
constexpr int STEM_C = 16;   // channels of the first convolution (not widened)

struct BasicGeom {
  int N, H, W, cin, cout, stride, Ho, Wo;
  bool conv_shortcut;
  int P() const { return N * H * W; }
  int P2() const { return N * Ho * Wo; }
};

struct WideNet {
  int N, S, classes;
  std::vector<BasicGeom> blocks;   // index = record - 1
  int final_c, final_hw;
  explicit WideNet(const karma_model_desc& d) {
    N = (int)d.batch; S = (int)d.seq; classes = (int)d.vocab;
    int hw = S, cin = STEM_C;
    for (int gr = 0; gr < 3; ++gr) {
      const int cout = (int)d.width << gr;
      for (uint32_t k = 0; k < d.stage_blocks[gr]; ++k) {
        BasicGeom g;
        g.N = N; g.H = g.W = hw; g.cin = cin; g.cout = cout;
        g.stride = (k == 0 && gr > 0) ? 2 : 1;
        g.conv_shortcut = cin != cout;
        g.Ho = g.Wo = conv_out_dim(hw, 3, g.stride, 1);
        blocks.push_back(g);
        hw = g.Ho;
        cin = cout;
      }
    }
    final_c = cin;
    final_hw = hw * hw;
  }
};

enum BasicParam { G1, B1, W1, G2, B2, W2, WS };
enum HeadParam { HG, HB, HW, HBIAS };

Param matrix(uint64_t n) {
  Param p;
  p.n = n; p.dev_bf16 = true; p.grad_bf16 = true;
  return p;
}
Param vector_f32_grad(uint64_t n) {   // batch-norm gain / shift, bias
  Param p;
  p.n = n; p.dev_bf16 = true; p.grad_bf16 = false;
  return p;
}

uint64_t splitk_want(uint64_t m, uint64_t n) {
  const uint64_t tiles = ((m + 127) / 128) * ((n + 127) / 128);
  const uint64_t splits = std::min<uint64_t>(256, (512 + tiles - 1) / tiles);
  return splits * m * n * 4;
}

struct BasicSaved {
  uint64_t o1, c1, o2, st1, st2, total;
  explicit BasicSaved(const BasicGeom& g) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    o1 = take((uint64_t)g.P() * g.cin * 2);
    c1 = take((uint64_t)g.P2() * g.cout * 2);
    o2 = take((uint64_t)g.P2() * g.cout * 2);
    st1 = take((uint64_t)2 * g.cin * 4);
    st2 = take((uint64_t)2 * g.cout * 4);
    total = o;
  }
};

struct BasicWs {
  uint64_t sc, m2, m1, dxs, wt, bn, splitk, splitk_bytes, total;
  explicit BasicWs(const BasicGeom& g) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    sc = take(g.conv_shortcut ? (uint64_t)g.P2() * g.cout * 2 : 0);   // forward: the shortcut convolution's output
    m2 = take((uint64_t)g.P2() * g.cout * 2);                         // do2 -> dc1
    m1 = take((uint64_t)g.P() * g.cin * 2);                           // do1
    dxs = take(g.conv_shortcut ? (uint64_t)g.P() * g.cin * 2 : 0);    // do1's part through the shortcut convolution
    wt = take((uint64_t)9 * g.cout * std::max(g.cin, g.cout) * 2);    // transposed weights of an input-gradient product
    bn = take(std::max(bn_ws_bytes(g.P(), g.cin), bn_ws_bytes(g.P2(), g.cout)));
    splitk_bytes = std::max({splitk_want(g.cout, 9 * g.cin), splitk_want(g.cout, 9 * g.cout),
                             g.conv_shortcut ? splitk_want(g.cout, g.cin) : 0});
    splitk = take(splitk_bytes);
    total = o;
  }
};

struct StemWs {
  uint64_t splitk, splitk_bytes, total;
  StemWs() {
    splitk_bytes = splitk_want(STEM_C, 9 * IMG_C);
    splitk = 0;
    total = up256(splitk_bytes);
  }
};

struct HeadWs {
  uint64_t act, st, bn, feat, logits, dfeat, rowloss, part, total;
  explicit HeadWs(const WideNet& n) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    const uint64_t pixels = (uint64_t)n.N * n.final_hw;
    act = take(pixels * n.final_c * 2);            // ReLU(BN(x)), then its gradient
    st = take((uint64_t)2 * n.final_c * 4);
    bn = take(bn_ws_bytes((int)pixels, n.final_c));
    feat = take((uint64_t)n.N * n.final_c * 2);
    logits = take((uint64_t)n.N * n.classes * 2);
    dfeat = take((uint64_t)n.N * n.final_c * 2);
    rowloss = take((uint64_t)n.N * 4);
    part = take(std::max<uint64_t>(colsum_ws_bytes(n.N, n.classes), 1024 * 4));
    total = o;
  }
};

#define TRY(call)          \
  do {                     \
    int st_ = (call);      \
    if (st_) return st_;   \
  } while (0)

int gemm_plain(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* bias, int M, int N, int K, bool a_kc, bool b_kc,
               hipStream_t s) {
  GemmArgs g{};
  g.A = A; g.B = B; g.C = C; g.bias = bias;
  g.M = M; g.N = N; g.K = K;
  g.a_kc = a_kc; g.b_kc = b_kc;
  g.lda = a_kc ? K : M;
  g.ldb = b_kc ? K : N;
  g.ldc = N;
  return gemm_bf16(g, s);
}

}  // namespace

int wrn_build_records(Ctx& c) {
  const karma_model_desc& d = c.desc;
  if (!d.batch || !d.seq || !d.vocab || !d.width || d.seq % 4 || d.vocab % 8 || d.width % 8) return KARMA_E_INVAL;
  if ((uint64_t)d.vocab * 2 > 150 * 1024 || d.stage_blocks[3]) return KARMA_E_INVAL;
  if (!d.stage_blocks[0]) return KARMA_E_INVAL;
  for (int k = 1; k < 3; ++k)
    if (d.stage_blocks[k] && !d.stage_blocks[k - 1]) return KARMA_E_INVAL;
  WideNet net(d);
  c.rec.clear();
  Record stem;
  stem.kind = REC_WRN_STEM;
  stem.p.push_back(matrix((uint64_t)STEM_C * 9 * IMG_C));
  stem.out_bytes = (uint64_t)net.N * net.S * net.S * STEM_C * 2;
  stem.sav_bytes = 0;
  stem.ws_bytes = StemWs().total;
  c.rec.push_back(std::move(stem));
  for (const BasicGeom& g : net.blocks) {
    Record r;
    r.kind = REC_WRN_BLOCK;
    r.p.push_back(vector_f32_grad(g.cin)); r.p.push_back(vector_f32_grad(g.cin));
    r.p.push_back(matrix((uint64_t)g.cout * 9 * g.cin));
    r.p.push_back(vector_f32_grad(g.cout)); r.p.push_back(vector_f32_grad(g.cout));
    r.p.push_back(matrix((uint64_t)g.cout * 9 * g.cout));
    if (g.conv_shortcut) r.p.push_back(matrix((uint64_t)g.cout * g.cin));
    r.out_bytes = (uint64_t)g.P2() * g.cout * 2;
    r.sav_bytes = BasicSaved(g).total;
    r.ws_bytes = BasicWs(g).total;
    r.streamed = d.stream_weights != 0;
    c.rec.push_back(std::move(r));
  }
  Record head;
  head.kind = REC_LOSS_WRN_HEAD;
  head.p.push_back(vector_f32_grad(net.final_c));
  head.p.push_back(vector_f32_grad(net.final_c));
  head.p.push_back(matrix((uint64_t)net.classes * net.final_c));
  head.p.push_back(vector_f32_grad(net.classes));
  head.ws_bytes = HeadWs(net).total;
  c.rec.push_back(std::move(head));
  c.in_bytes = (uint64_t)net.N * net.S * net.S * IMG_C * 2;
  c.lab_bytes = (uint64_t)net.N * 4;
  c.misc_bytes = 0;
  return KARMA_OK;
}

// images fp32 [N][S][S][3] -> bf16 [N][S][S][8] (round to nearest even, channels 3..7 zero)
int wrn_prepare_step(Ctx& c, const void* in, const void* lab) {
  WideNet net(c.desc);
  const int32_t* labels = (const int32_t*)lab;
  for (int i = 0; i < net.N; ++i)
    if (labels[i] < 0 || labels[i] >= net.classes) {
      c.err = "label outside the classes";
      return KARMA_E_INVAL;
    }
  const float* img = (const float*)in;
  uint16_t* out = (uint16_t*)c.stage_in;
  const size_t pixels = (size_t)net.N * net.S * net.S;
  c.pool->parallel_for(pixels, [&](size_t lo, size_t hi) {
    for (size_t p = lo; p < hi; ++p) {
      uint16_t* o = out + p * IMG_C;
      for (int ch = 0; ch < 3; ++ch) o[ch] = f32_to_bf16_rne(img[p * 3 + ch]);
      for (int ch = 3; ch < IMG_C; ++ch) o[ch] = 0;
    }
  });
  std::memcpy(c.stage_lab, lab, c.lab_bytes);
  return KARMA_OK;
}

int wrn_prepare_late(Ctx&) { return KARMA_OK; }

int wrn_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  WideNet net(c.desc);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t, io.w); };
  if (i == 0) {
    if (!io.out) return KARMA_OK;   // nothing is saved: a recompute whose output nobody needs is empty
    StemWs wl;
    return conv2d_fwd((const bf16_t*)io.x, W(0), (bf16_t*)io.out, ConvShape{net.N, net.S, net.S, IMG_C, STEM_C, 3, 3, 1, 1}, s,
                      Wk + wl.splitk, wl.splitk_bytes);
  }
  const BasicGeom& g = net.blocks[i - 1];
  BasicSaved sv(g);
  BasicWs wl(g);
  const bf16_t* x = (const bf16_t*)io.x;
  bf16_t* o1 = (bf16_t*)(S + sv.o1);
  bf16_t* c1 = (bf16_t*)(S + sv.c1);
  bf16_t* o2 = (bf16_t*)(S + sv.o2);
  float* bnws = (float*)(Wk + wl.bn);
  void* sk = Wk + wl.splitk;
  TRY(bn_fwd(x, W(G1), W(B1), nullptr, o1, (float*)(S + sv.st1), bnws, g.P(), g.cin, 1, s));
  TRY(conv2d_fwd(o1, W(W1), c1, ConvShape{g.N, g.H, g.W, g.cin, g.cout, 3, 3, g.stride, 1}, s, sk, wl.splitk_bytes));
  TRY(bn_fwd(c1, W(G2), W(B2), nullptr, o2, (float*)(S + sv.st2), bnws, g.P2(), g.cout, 1, s));
  // the second convolution and the shortcut produce the output only: a recompute whose output
  // still exists as the next record's input stops here
  if (!io.out) return KARMA_OK;
  const bf16_t* shortcut = x;
  if (g.conv_shortcut) {
    bf16_t* sc = (bf16_t*)(Wk + wl.sc);
    TRY(conv2d_fwd(o1, W(WS), sc, ConvShape{g.N, g.H, g.W, g.cin, g.cout, 1, 1, g.stride, 0}, s, sk, wl.splitk_bytes));
    shortcut = sc;
  }
  return conv2d_fwd(o2, W(W2), (bf16_t*)io.out, ConvShape{g.N, g.Ho, g.Wo, g.cout, g.cout, 3, 3, 1, 1}, s, sk, wl.splitk_bytes,
                    shortcut);
}

int wrn_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  WideNet net(c.desc);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  const bf16_t* dy = (const bf16_t*)io.dy;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t, io.w); };
  auto G = [&](int t) { return c.g_ptr(i, t, io.g); };
  if (i == 0) {
    StemWs wl;
    return conv2d_wgrad(dy, (const bf16_t*)io.x, (bf16_t*)G(0), Wk + wl.splitk, wl.splitk_bytes,
                        ConvShape{net.N, net.S, net.S, IMG_C, STEM_C, 3, 3, 1, 1}, s);
  }
  const BasicGeom& g = net.blocks[i - 1];
  BasicSaved sv(g);
  BasicWs wl(g);
  const bf16_t* x = (const bf16_t*)io.x;
  const bf16_t* o1 = (const bf16_t*)(S + sv.o1);
  const bf16_t* c1 = (const bf16_t*)(S + sv.c1);
  const bf16_t* o2 = (const bf16_t*)(S + sv.o2);
  const float* st1 = (const float*)(S + sv.st1);
  const float* st2 = (const float*)(S + sv.st2);
  bf16_t* m2 = (bf16_t*)(Wk + wl.m2);
  bf16_t* m1 = (bf16_t*)(Wk + wl.m1);
  bf16_t* dxs = (bf16_t*)(Wk + wl.dxs);
  bf16_t* wt = (bf16_t*)(Wk + wl.wt);
  float* bnws = (float*)(Wk + wl.bn);
  void* sk = Wk + wl.splitk;
  const ConvShape s1{g.N, g.H, g.W, g.cin, g.cout, 3, 3, g.stride, 1}, s2{g.N, g.Ho, g.Wo, g.cout, g.cout, 3, 3, 1, 1},
      ss{g.N, g.H, g.W, g.cin, g.cout, 1, 1, g.stride, 0};
  TRY(conv2d_wgrad(dy, o2, (bf16_t*)G(W2), sk, wl.splitk_bytes, s2, s));
  TRY(conv2d_dgrad(dy, W(W2), wt, nullptr, m2, s2, s, sk, wl.splitk_bytes));                                          // do2
  TRY(bn_bwd(m2, c1, st2, W(G2), W(B2), 1, m2, (float*)G(G2), (float*)G(B2), bnws, g.P2(), g.cout, s));              // dc1
  TRY(conv2d_wgrad(m2, o1, (bf16_t*)G(W1), sk, wl.splitk_bytes, s1, s));
  if (g.conv_shortcut) {
    TRY(conv2d_wgrad(dy, o1, (bf16_t*)G(WS), sk, wl.splitk_bytes, ss, s));
    TRY(conv2d_dgrad(dy, W(WS), wt, nullptr, dxs, ss, s, sk, wl.splitk_bytes));
    TRY(conv2d_dgrad(m2, W(W1), wt, dxs, m1, s1, s, sk, wl.splitk_bytes));                                            // do1, both paths
    TRY(bn_bwd(m1, x, st1, W(G1), W(B1), 1, (bf16_t*)io.dx, (float*)G(G1), (float*)G(B1), bnws, g.P(), g.cin, s));
  } else {
    TRY(conv2d_dgrad(m2, W(W1), wt, nullptr, m1, s1, s, sk, wl.splitk_bytes));                                        // do1
    TRY(bn_bwd(m1, x, st1, W(G1), W(B1), 1, (bf16_t*)io.dx, (float*)G(G1), (float*)G(B1), bnws, g.P(), g.cin, s, dy));
  }
  return KARMA_OK;
}

// Batch norm, ReLU, global average pooling, fully connected layer, mean cross entropy, and their gradients.
int wrn_loss(Ctx& c, const LayerIO& io, hipStream_t s) {
  WideNet net(c.desc);
  HeadWs wl(net);
  const uint32_t R = c.L;
  char* Wk = (char*)io.ws;
  bf16_t* act = (bf16_t*)(Wk + wl.act);
  float* st = (float*)(Wk + wl.st);
  float* bnws = (float*)(Wk + wl.bn);
  bf16_t* feat = (bf16_t*)(Wk + wl.feat);
  bf16_t* logits = (bf16_t*)(Wk + wl.logits);
  bf16_t* dfeat = (bf16_t*)(Wk + wl.dfeat);
  float* rowloss = (float*)(Wk + wl.rowloss);
  float* part = (float*)(Wk + wl.part);
  const bf16_t* x = (const bf16_t*)io.x;
  const bf16_t* gain = (const bf16_t*)c.w_ptr(R, HG);
  const bf16_t* shift = (const bf16_t*)c.w_ptr(R, HB);
  const bf16_t* w = (const bf16_t*)c.w_ptr(R, HW);
  const bf16_t* bias = (const bf16_t*)c.w_ptr(R, HBIAS);
  const int* labels = (const int*)c.fixed_ptr(c.lab_off);
  const int pixels = net.N * net.final_hw;
  TRY(bn_fwd(x, gain, shift, nullptr, act, st, bnws, pixels, net.final_c, 1, s));
  TRY(avgpool_fwd(act, feat, net.N, net.final_hw, net.final_c, s));
  TRY(gemm_plain(feat, w, logits, bias, net.N, net.classes, net.final_c, true, true, s));
  TRY(softmax_ce(logits, labels, rowloss, net.N, net.classes, 1.f / (float)net.N, s));   // logits -> dlogits
  TRY(sum_f32(rowloss, (float*)c.fixed_ptr(c.loss_off), part, (size_t)net.N, 1.f / (float)net.N, s));
  TRY(gemm_plain(logits, feat, c.g_ptr(R, HW), nullptr, net.classes, net.final_c, net.N, false, false, s));   // dW = dlogits^T feat
  TRY(colsum_bf16(logits, (float*)c.g_ptr(R, HBIAS), part, net.N, net.classes, s));
  TRY(gemm_plain(logits, w, dfeat, nullptr, net.N, net.final_c, net.classes, true, false, s));               // dfeat = dlogits W
  TRY(avgpool_bwd(dfeat, act, net.N, net.final_hw, net.final_c, s));
  TRY(bn_bwd(act, x, st, gain, shift, 1, (bf16_t*)io.dx, (float*)c.g_ptr(R, HG), (float*)c.g_ptr(R, HB), bnws, pixels,
             net.final_c, s));
  return KARMA_OK;
}

}  // namespace karma
