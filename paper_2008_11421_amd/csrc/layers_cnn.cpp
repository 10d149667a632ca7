// Bottleneck residual network (the ResNet-200 row of KARMA's Table III) as layer records
// of the out-of-core executor: record 0 is the stem (7x7 stride-2 convolution, batch norm,
// ReLU, 3x3 stride-2 max pooling), records 1.. are bottleneck blocks (1x1, 3x3 carrying
// the stride, 1x1, each followed by batch norm; projection shortcut where the shape
// changes; ReLU after the residual sum), the loss record is global average pooling, the
// fully connected layer and mean cross entropy.  One record = one block of the paper: a
// block's input is its checkpoint, its saved set the convolution outputs, the activations
// the next convolution reads, and the batch statistics.  Activations are NHWC bf16.
#include <algorithm>
#include <cstring>

#include "context.h"
#include "kernels.h"
#include "layers.h"

namespace karma {
namespace {

inline uint64_t up256(uint64_t b) { return (b + 255) / 256 * 256; }

struct BlockGeom {
  int N, H, W, cin, mid, cout, stride, Ho, Wo;
  bool proj;
  int P() const { return N * H * W; }      // pixels of the input
  int P2() const { return N * Ho * Wo; }   // pixels of the output
};

// fp32 workspace that lets a weight-gradient GEMM (M x N result, reduction over the pixels)
// split its reduction far enough to fill the chip: few output tiles need many splits
uint64_t splitk_want(uint64_t m, uint64_t n) {
  const uint64_t tiles = ((m + 127) / 128) * ((n + 127) / 128);
  const uint64_t splits = std::min<uint64_t>(256, (512 + tiles - 1) / tiles);
  return splits * m * n * 4;
}

struct Net {
  int N, S, classes, width, stem_c;
  std::vector<BlockGeom> blocks;   // index = record - 1
  int final_c, final_hw;
  explicit Net(const karma_model_desc& d) {
    N = (int)d.batch; S = (int)d.seq; classes = (int)d.vocab; width = (int)d.width;
    stem_c = width;
    int hw = S / 4, cin = stem_c;
    for (int st = 0; st < 4; ++st) {
      const int mid = width << st, cout = 4 * mid;
      for (uint32_t k = 0; k < d.stage_blocks[st]; ++k) {
        BlockGeom g;
        g.N = N; g.H = g.W = hw; g.cin = cin; g.mid = mid; g.cout = cout;
        g.stride = (k == 0 && st > 0) ? 2 : 1;
        g.proj = k == 0;
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

enum BlockParam { W1, G1, B1, W2, G2, B2, W3, G3, B3, WP, GP, BP };
enum StemParam { SW, SG, SB };

Param conv_weight(uint64_t n) {
  Param p;
  p.n = n; p.dev_bf16 = true; p.grad_bf16 = true;
  return p;
}
Param channel_vector(uint64_t n) {   // batch-norm gain / shift, biases: fp32 gradients
  Param p;
  p.n = n; p.dev_bf16 = true; p.grad_bf16 = false;
  return p;
}

// internals of one bottleneck block
struct BlockSaved {
  uint64_t c1, a1, c2, a2, c3, cp, st1, st2, st3, stp, total;
  explicit BlockSaved(const BlockGeom& g) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    c1 = take((uint64_t)g.P() * g.mid * 2);
    a1 = take((uint64_t)g.P() * g.mid * 2);
    c2 = take((uint64_t)g.P2() * g.mid * 2);
    a2 = take((uint64_t)g.P2() * g.mid * 2);
    c3 = take((uint64_t)g.P2() * g.cout * 2);
    cp = take(g.proj ? (uint64_t)g.P2() * g.cout * 2 : 0);
    st1 = take((uint64_t)2 * g.mid * 4);
    st2 = take((uint64_t)2 * g.mid * 4);
    st3 = take((uint64_t)2 * g.cout * 4);
    stp = take(g.proj ? (uint64_t)2 * g.cout * 4 : 0);
    total = o;
  }
};

// workspace of a block's forward (shortcut) and backward
struct BlockWs {
  uint64_t big, mid2, mid1, dxa, wt, bn, splitk, splitk_bytes, total;
  explicit BlockWs(const BlockGeom& g) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    big = take((uint64_t)2 * g.P2() * g.cout * 2);   // forward: normalised shortcut; backward: recomputed output -> dz, and dc3 / dcp
    mid2 = take((uint64_t)g.P2() * g.mid * 2);       // da2 -> dc2
    mid1 = take((uint64_t)g.P() * g.mid * 2);        // da1 -> dc1
    dxa = take(g.proj ? (uint64_t)g.P() * g.cin * 2 : 0);   // input gradient through the projection
    wt = take((uint64_t)std::max(9 * g.mid * g.mid, g.proj && g.stride > 1 ? g.cin * g.cout : 0) * 2);
    bn = take(std::max(bn_ws_bytes(g.P(), g.mid), bn_ws_bytes(g.P2(), g.cout)));
    splitk_bytes = std::max({splitk_want(g.mid, 9 * g.mid), splitk_want(g.cout, g.mid), splitk_want(g.mid, g.cin),
                             g.proj ? splitk_want(g.cout, g.cin) : 0});
    splitk = take(splitk_bytes);
    total = o;
  }
};

struct StemGeom {
  int N, S, C, H1, H2;   // image size, stem channels, size after the convolution, after pooling
};
StemGeom stem_geom(const Net& n) { return StemGeom{n.N, n.S, n.stem_c, n.S / 2, n.S / 4}; }
constexpr int IMG_C = 8;   // the three image channels are stored as eight (zeros), so that rows are 16 bytes

struct StemSaved {
  uint64_t c0, a0, st, total;
  explicit StemSaved(const StemGeom& g) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    const uint64_t act = (uint64_t)g.N * g.H1 * g.H1 * g.C * 2;
    c0 = take(act);
    a0 = take(act);
    st = take((uint64_t)2 * g.C * 4);
    total = o;
  }
};
struct StemWs {
  uint64_t da0, bn, splitk, splitk_bytes, total;
  explicit StemWs(const StemGeom& g) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    da0 = take((uint64_t)g.N * g.H1 * g.H1 * g.C * 2);
    bn = take(bn_ws_bytes(g.N * g.H1 * g.H1, g.C));
    splitk_bytes = splitk_want(g.C, 49 * IMG_C);
    splitk = take(splitk_bytes);
    total = o;
  }
};

struct HeadWs {
  uint64_t feat, logits, dfeat, rowloss, part, total;
  explicit HeadWs(const Net& n) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
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

int cnn_build_records(Ctx& c) {
  const karma_model_desc& d = c.desc;
  if (!d.batch || !d.seq || !d.vocab || !d.width || d.seq % 32 || d.vocab % 8 || d.width % 8) return KARMA_E_INVAL;
  if ((uint64_t)d.vocab * 2 > 150 * 1024) return KARMA_E_INVAL;
  uint32_t nb = 0;
  for (int k = 0; k < 4; ++k) nb += d.stage_blocks[k];
  if (!nb) return KARMA_E_INVAL;
  for (int k = 1; k < 4; ++k)
    if (d.stage_blocks[k] && !d.stage_blocks[k - 1]) return KARMA_E_INVAL;
  Net net(d);
  c.rec.clear();
  const StemGeom sg = stem_geom(net);
  Record stem;
  stem.kind = REC_CNN_STEM;
  stem.p.push_back(conv_weight((uint64_t)sg.C * 49 * IMG_C));
  stem.p.push_back(channel_vector(sg.C));
  stem.p.push_back(channel_vector(sg.C));
  stem.out_bytes = (uint64_t)sg.N * sg.H2 * sg.H2 * sg.C * 2;
  stem.sav_bytes = StemSaved(sg).total;
  stem.ws_bytes = StemWs(sg).total;
  c.rec.push_back(std::move(stem));
  for (const BlockGeom& g : net.blocks) {
    Record r;
    r.kind = REC_CNN_BLOCK;
    r.p.push_back(conv_weight((uint64_t)g.mid * g.cin));
    r.p.push_back(channel_vector(g.mid)); r.p.push_back(channel_vector(g.mid));
    r.p.push_back(conv_weight((uint64_t)g.mid * 9 * g.mid));
    r.p.push_back(channel_vector(g.mid)); r.p.push_back(channel_vector(g.mid));
    r.p.push_back(conv_weight((uint64_t)g.cout * g.mid));
    r.p.push_back(channel_vector(g.cout)); r.p.push_back(channel_vector(g.cout));
    if (g.proj) {
      r.p.push_back(conv_weight((uint64_t)g.cout * g.cin));
      r.p.push_back(channel_vector(g.cout)); r.p.push_back(channel_vector(g.cout));
    }
    r.out_bytes = (uint64_t)g.P2() * g.cout * 2;
    r.sav_bytes = BlockSaved(g).total;
    r.ws_bytes = BlockWs(g).total;
    r.streamed = d.stream_weights != 0;
    c.rec.push_back(std::move(r));
  }
  Record head;
  head.kind = REC_LOSS_CNN_HEAD;
  head.p.push_back(conv_weight((uint64_t)net.classes * net.final_c));
  head.p.push_back(channel_vector(net.classes));
  head.ws_bytes = HeadWs(net).total;
  c.rec.push_back(std::move(head));
  c.in_bytes = (uint64_t)net.N * net.S * net.S * IMG_C * 2;
  c.lab_bytes = (uint64_t)net.N * 4;
  c.misc_bytes = 0;
  return KARMA_OK;
}

// images fp32 [N][S][S][3] -> bf16 [N][S][S][8] (round to nearest even, channels 3..7 zero)
int cnn_prepare_step(Ctx& c, const void* in, const void* lab) {
  Net net(c.desc);
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

int cnn_prepare_late(Ctx&) { return KARMA_OK; }

int cnn_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  Net net(c.desc);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t, io.w); };
  if (i == 0) {
    const StemGeom g = stem_geom(net);
    StemSaved sv(g);
    StemWs wl(g);
    bf16_t* c0 = (bf16_t*)(S + sv.c0);
    bf16_t* a0 = (bf16_t*)(S + sv.a0);
    const int rows = g.N * g.H1 * g.H1;
    TRY(conv2d_fwd((const bf16_t*)io.x, W(SW), c0, ConvShape{g.N, g.S, g.S, IMG_C, g.C, 7, 7, 2, 3}, s, Wk + wl.splitk, wl.splitk_bytes));
    TRY(bn_fwd(c0, W(SG), W(SB), nullptr, a0, (float*)(S + sv.st), (float*)(Wk + wl.bn), rows, g.C, 1, s));
    if (io.out) TRY(maxpool_fwd(a0, (bf16_t*)io.out, g.N, g.H1, g.H1, g.C, s));
    return KARMA_OK;
  }
  const BlockGeom& g = net.blocks[i - 1];
  BlockSaved sv(g);
  BlockWs wl(g);
  const bf16_t* x = (const bf16_t*)io.x;
  bf16_t* c1 = (bf16_t*)(S + sv.c1);
  bf16_t* a1 = (bf16_t*)(S + sv.a1);
  bf16_t* c2 = (bf16_t*)(S + sv.c2);
  bf16_t* a2 = (bf16_t*)(S + sv.a2);
  bf16_t* c3 = (bf16_t*)(S + sv.c3);
  bf16_t* cp = (bf16_t*)(S + sv.cp);
  float* bnws = (float*)(Wk + wl.bn);
  TRY(conv2d_fwd(x, W(W1), c1, ConvShape{g.N, g.H, g.W, g.cin, g.mid, 1, 1, 1, 0}, s, Wk + wl.splitk, wl.splitk_bytes));
  TRY(bn_fwd(c1, W(G1), W(B1), nullptr, a1, (float*)(S + sv.st1), bnws, g.P(), g.mid, 1, s));
  TRY(conv2d_fwd(a1, W(W2), c2, ConvShape{g.N, g.H, g.W, g.mid, g.mid, 3, 3, g.stride, 1}, s, Wk + wl.splitk, wl.splitk_bytes));
  TRY(bn_fwd(c2, W(G2), W(B2), nullptr, a2, (float*)(S + sv.st2), bnws, g.P2(), g.mid, 1, s));
  TRY(conv2d_fwd(a2, W(W3), c3, ConvShape{g.N, g.Ho, g.Wo, g.mid, g.cout, 1, 1, 1, 0}, s, Wk + wl.splitk, wl.splitk_bytes));
  // a recompute whose output nobody needs still has to produce every saved tensor, statistics
  // included; only the last elementwise pass can be dropped
  bf16_t* y = io.out ? (bf16_t*)io.out : (bf16_t*)(Wk + wl.big) + (size_t)g.P2() * g.cout;
  if (g.proj) {
    bf16_t* sc = (bf16_t*)(Wk + wl.big);
    TRY(conv2d_fwd(x, W(WP), cp, ConvShape{g.N, g.H, g.W, g.cin, g.cout, 1, 1, g.stride, 0}, s, Wk + wl.splitk, wl.splitk_bytes));
    TRY(bn_fwd(cp, W(GP), W(BP), nullptr, sc, (float*)(S + sv.stp), bnws, g.P2(), g.cout, 0, s));
    TRY(bn_fwd(c3, W(G3), W(B3), sc, y, (float*)(S + sv.st3), bnws, g.P2(), g.cout, 1, s));
  } else {
    TRY(bn_fwd(c3, W(G3), W(B3), x, y, (float*)(S + sv.st3), bnws, g.P2(), g.cout, 1, s));
  }
  return KARMA_OK;
}

int cnn_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  Net net(c.desc);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  const bf16_t* dy = (const bf16_t*)io.dy;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t, io.w); };
  auto G = [&](int t) { return c.g_ptr(i, t, io.g); };
  if (i == 0) {
    const StemGeom g = stem_geom(net);
    StemSaved sv(g);
    StemWs wl(g);
    const bf16_t* c0 = (const bf16_t*)(S + sv.c0);
    const bf16_t* a0 = (const bf16_t*)(S + sv.a0);
    bf16_t* da0 = (bf16_t*)(Wk + wl.da0);
    const int rows = g.N * g.H1 * g.H1;
    TRY(maxpool_bwd(a0, dy, da0, g.N, g.H1, g.H1, g.C, s));
    TRY(bn_bwd(da0, c0, (const float*)(S + sv.st), W(SG), W(SB), 1, da0, (float*)G(SG), (float*)G(SB), (float*)(Wk + wl.bn),
               rows, g.C, s));
    TRY(conv2d_wgrad(da0, (const bf16_t*)io.x, (bf16_t*)G(SW), Wk + wl.splitk, wl.splitk_bytes,
                     ConvShape{g.N, g.S, g.S, IMG_C, g.C, 7, 7, 2, 3}, s));
    return KARMA_OK;
  }
  const BlockGeom& g = net.blocks[i - 1];
  BlockSaved sv(g);
  BlockWs wl(g);
  const bf16_t* x = (const bf16_t*)io.x;
  const bf16_t* c1 = (const bf16_t*)(S + sv.c1);
  const bf16_t* a1 = (const bf16_t*)(S + sv.a1);
  const bf16_t* c2 = (const bf16_t*)(S + sv.c2);
  const bf16_t* a2 = (const bf16_t*)(S + sv.a2);
  const bf16_t* c3 = (const bf16_t*)(S + sv.c3);
  const bf16_t* cp = (const bf16_t*)(S + sv.cp);
  const float* st1 = (const float*)(S + sv.st1);
  const float* st2 = (const float*)(S + sv.st2);
  const float* st3 = (const float*)(S + sv.st3);
  const float* stp = (const float*)(S + sv.stp);
  bf16_t* dz = (bf16_t*)(Wk + wl.big);
  bf16_t* big2 = dz + (size_t)g.P2() * g.cout;
  bf16_t* m2 = (bf16_t*)(Wk + wl.mid2);
  bf16_t* m1 = (bf16_t*)(Wk + wl.mid1);
  bf16_t* dxa = (bf16_t*)(Wk + wl.dxa);
  bf16_t* wt = (bf16_t*)(Wk + wl.wt);
  float* bnws = (float*)(Wk + wl.bn);
  void* sk = Wk + wl.splitk;
  const ConvShape s1{g.N, g.H, g.W, g.cin, g.mid, 1, 1, 1, 0}, s2{g.N, g.H, g.W, g.mid, g.mid, 3, 3, g.stride, 1},
      s3{g.N, g.Ho, g.Wo, g.mid, g.cout, 1, 1, 1, 0}, sp{g.N, g.H, g.W, g.cin, g.cout, 1, 1, g.stride, 0};
  // gradient through the last ReLU: the block's output is recomputed from saved tensors
  // (it is the next block's input and may be gone by now)
  if (g.proj) {
    TRY(bn_apply(cp, stp, W(GP), W(BP), nullptr, big2, g.P2(), g.cout, 0, s));
    TRY(bn_apply(c3, st3, W(G3), W(B3), big2, dz, g.P2(), g.cout, 1, s, dy));
  } else {
    TRY(bn_apply(c3, st3, W(G3), W(B3), x, dz, g.P2(), g.cout, 1, s, dy));
  }
  // main branch
  TRY(bn_bwd(dz, c3, st3, W(G3), W(B3), 0, big2, (float*)G(G3), (float*)G(B3), bnws, g.P2(), g.cout, s));   // dc3
  TRY(conv2d_wgrad(big2, a2, (bf16_t*)G(W3), sk, wl.splitk_bytes, s3, s));
  TRY(conv2d_dgrad(big2, W(W3), nullptr, nullptr, m2, s3, s, sk, wl.splitk_bytes));                                               // da2
  TRY(bn_bwd(m2, c2, st2, W(G2), W(B2), 1, m2, (float*)G(G2), (float*)G(B2), bnws, g.P2(), g.mid, s));       // dc2
  TRY(conv2d_wgrad(m2, a1, (bf16_t*)G(W2), sk, wl.splitk_bytes, s2, s));
  TRY(conv2d_dgrad(m2, W(W2), wt, nullptr, m1, s2, s, sk, wl.splitk_bytes));                                                      // da1
  TRY(bn_bwd(m1, c1, st1, W(G1), W(B1), 1, m1, (float*)G(G1), (float*)G(B1), bnws, g.P(), g.mid, s));        // dc1
  TRY(conv2d_wgrad(m1, x, (bf16_t*)G(W1), sk, wl.splitk_bytes, s1, s));
  // shortcut, then dx = gradient through the first convolution + gradient through the shortcut
  if (g.proj) {
    TRY(bn_bwd(dz, cp, stp, W(GP), W(BP), 0, big2, (float*)G(GP), (float*)G(BP), bnws, g.P2(), g.cout, s));  // dcp
    TRY(conv2d_wgrad(big2, x, (bf16_t*)G(WP), sk, wl.splitk_bytes, sp, s));
    TRY(conv2d_dgrad(big2, W(WP), wt, nullptr, dxa, sp, s, sk, wl.splitk_bytes));
    TRY(conv2d_dgrad(m1, W(W1), nullptr, dxa, (bf16_t*)io.dx, s1, s, sk, wl.splitk_bytes));
  } else {
    TRY(conv2d_dgrad(m1, W(W1), nullptr, dz, (bf16_t*)io.dx, s1, s, sk, wl.splitk_bytes));
  }
  return KARMA_OK;
}

// Global average pooling, fully connected layer, mean cross entropy, and their gradients.
int cnn_loss(Ctx& c, const LayerIO& io, hipStream_t s) {
  Net net(c.desc);
  HeadWs wl(net);
  const uint32_t R = c.L;
  char* Wk = (char*)io.ws;
  bf16_t* feat = (bf16_t*)(Wk + wl.feat);
  bf16_t* logits = (bf16_t*)(Wk + wl.logits);
  bf16_t* dfeat = (bf16_t*)(Wk + wl.dfeat);
  float* rowloss = (float*)(Wk + wl.rowloss);
  float* part = (float*)(Wk + wl.part);
  const bf16_t* w = (const bf16_t*)c.w_ptr(R, 0);
  const bf16_t* b = (const bf16_t*)c.w_ptr(R, 1);
  const int* labels = (const int*)c.fixed_ptr(c.lab_off);
  TRY(avgpool_fwd((const bf16_t*)io.x, feat, net.N, net.final_hw, net.final_c, s));
  TRY(gemm_plain(feat, w, logits, b, net.N, net.classes, net.final_c, true, true, s));
  TRY(softmax_ce(logits, labels, rowloss, net.N, net.classes, 1.f / (float)net.N, s));   // logits -> dlogits
  TRY(sum_f32(rowloss, (float*)c.fixed_ptr(c.loss_off), part, (size_t)net.N, 1.f / (float)net.N, s));
  TRY(gemm_plain(logits, feat, c.g_ptr(R, 0), nullptr, net.classes, net.final_c, net.N, false, false, s));   // dW = dlogits^T feat
  TRY(colsum_bf16(logits, (float*)c.g_ptr(R, 1), part, net.N, net.classes, s));
  TRY(gemm_plain(logits, w, dfeat, nullptr, net.N, net.final_c, net.classes, true, false, s));               // dfeat = dlogits W
  TRY(avgpool_bwd(dfeat, (bf16_t*)io.dx, net.N, net.final_hw, net.final_c, s));
  return KARMA_OK;
}

}  // namespace karma
