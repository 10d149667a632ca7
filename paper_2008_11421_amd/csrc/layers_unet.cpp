// Fully convolutional network (the U-Net row of KARMA's Table III; Sec. III-F.3 names it as the
// model with connections from the contracting to the expansive path) as layer records of the
// out-of-core executor.  depth D, level l: width << l channels at (image >> l)^2 pixels.
// Records 0 .. D: contracting levels (2x2 max pooling of the level above, except level 0; two
// 3x3 convolutions, each followed by batch normalisation and ReLU); records D+1 .. 2D:
// expansive levels D-1 .. 0 (2x2 stride-2 up-convolution of the level below, two 3x3
// convolutions of which the first reads the contracting output of the same level and the
// up-convolution's result as one concatenated tensor); loss record: 1x1 classifier and the
// mean cross entropy over all pixels.  The pooling belongs to the record BELOW it, so that a
// contracting record's output is the tensor the expansive path reads again: record 2D - l
// reads the output of record l (l < D), a connection between non-consecutive records that the
// planner and the executor handle (premature swap-in, gradient held until the contracting
// record's successor runs backward).  The concatenation is never built: the convolution over it
// is the sum of two convolutions, one per half, with the weight stored as two tensors.
// Activations are NHWC bf16; the single image channel is stored as eight (zeros).
#include <algorithm>
#include <atomic>
#include <cstring>

#include "context.h"
#include "kernels.h"
#include "layers.h"

namespace karma {
namespace {

inline uint64_t up256(uint64_t b) { return (b + 255) / 256 * 256; }
constexpr int IMG_C = 8;

struct Level {
  int N, S, C;            // images, pixels a side, channels of this level
  int P() const { return N * S * S; }
};

struct UNet {
  int N, S, D, width, classes;
  explicit UNet(const karma_model_desc& d)
      : N((int)d.batch), S((int)d.seq), D((int)d.n_layers), width((int)d.width), classes((int)d.vocab) {}
  Level level(int l) const { return Level{N, S >> l, width << l}; }
  bool down(uint32_t r) const { return (int)r <= D; }
  int level_of(uint32_t r) const { return down(r) ? (int)r : 2 * D - (int)r; }
};

enum DownParam { DW1, DG1, DB1, DW2, DG2, DB2 };
enum UpParam { UWU, UW1S, UW1U, UG1, UB1, UW2, UG2, UB2 };
enum HeadParam { HW, HBIAS };

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

// Saved set of a record: [pooled input | up-convolution's result], first convolution's output, its
// activation, second convolution's output, the two batch statistics.
struct Saved {
  uint64_t head, c1, a1, c2, st1, st2, total;
  Saved(const Level& v, uint64_t head_elems) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    const uint64_t t = (uint64_t)v.P() * v.C * 2;
    head = take(head_elems * 2);
    c1 = take(t); a1 = take(t); c2 = take(t);
    st1 = take((uint64_t)2 * v.C * 4);
    st2 = take((uint64_t)2 * v.C * 4);
    total = o;
  }
};

// Workspace of a record: two tensors of the level's size (gradients on their way down; in an
// expansive record's forward pass the first half of the split convolution), the transposed
// weights of an input-gradient product, batch-norm partial sums, split-k partial sums.
struct Work {
  uint64_t m1, m2, wt, bn, splitk, splitk_bytes, total;
  Work(const Level& v, int cin_max, uint64_t wt_elems, uint64_t splitk_need) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    const uint64_t t = (uint64_t)v.P() * std::max(v.C, cin_max) * 2;
    m1 = take(t); m2 = take(t);
    wt = take(wt_elems * 2);
    bn = take(bn_ws_bytes(v.P(), v.C));
    splitk_bytes = splitk_need;
    splitk = take(splitk_bytes);
    total = o;
  }
};

struct DownGeom {
  Level v;
  int cin;          // channels of the tensor the first convolution reads
  bool pooled;
  DownGeom(const UNet& n, int l) : v(n.level(l)), cin(l ? n.width << (l - 1) : IMG_C), pooled(l > 0) {}
  Saved saved() const { return Saved(v, pooled ? (uint64_t)v.P() * cin : 0); }
  Work work() const {
    return Work(v, cin, (uint64_t)9 * v.C * std::max(cin, v.C), std::max(splitk_want(v.C, 9 * (uint64_t)cin), splitk_want(v.C, 9 * (uint64_t)v.C)));
  }
};

struct UpGeom {
  Level v, below;
  UpGeom(const UNet& n, int l) : v(n.level(l)), below(n.level(l + 1)) {}
  Saved saved() const { return Saved(v, (uint64_t)v.P() * v.C); }
  Work work() const {
    return Work(v, v.C, (uint64_t)9 * v.C * v.C, std::max(splitk_want(v.C, 9 * (uint64_t)v.C), splitk_want(below.C, 4 * (uint64_t)v.C)));
  }
  // the up-convolution is the input gradient of this 2x2 stride-2 convolution from the fine grid to the coarse one
  ConvShape conv_of_up() const { return ConvShape{v.N, v.S, v.S, v.C, below.C, 2, 2, 2, 0}; }
};

struct HeadWs {
  uint64_t logits, rowloss, part, splitk, splitk_bytes, total;
  explicit HeadWs(const UNet& n) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    const uint64_t pixels = (uint64_t)n.level(0).P();
    logits = take(pixels * n.classes * 2);
    rowloss = take(pixels * 4);
    part = take(std::max<uint64_t>(colsum_ws_bytes((int)pixels, n.classes), 1024 * 4));
    splitk_bytes = (uint64_t)256 * n.classes * n.width * 4;
    splitk = take(splitk_bytes);
    total = o;
  }
};

#define TRY(call)          \
  do {                     \
    int st_ = (call);      \
    if (st_) return st_;   \
  } while (0)

ConvShape conv3(const Level& v, int cin) { return ConvShape{v.N, v.S, v.S, cin, v.C, 3, 3, 1, 1}; }

}  // namespace

int unet_skips(const karma_model_desc& d, std::vector<karma_skip>& out) {
  out.clear();
  for (uint32_t l = 0; l < d.n_layers; ++l) out.push_back(karma_skip{l, 2 * d.n_layers - l});
  return KARMA_OK;
}

int unet_build_records(Ctx& c) {
  const karma_model_desc& d = c.desc;
  if (!d.batch || !d.seq || !d.vocab || !d.width || !d.n_layers || d.n_layers > 6 || d.width % 8 || d.vocab % 8) return KARMA_E_INVAL;
  if (d.vocab > 16 || d.stream_weights || d.seq % (1u << d.n_layers) || (d.seq >> d.n_layers) < 2) return KARMA_E_INVAL;
  if ((uint64_t)d.batch * d.seq * d.seq >= (1u << 30)) return KARMA_E_INVAL;
  UNet net(d);
  c.rec.clear();
  for (int l = 0; l <= net.D; ++l) {
    DownGeom g(net, l);
    Record r;
    r.kind = REC_UNET_DOWN;
    r.p.push_back(matrix((uint64_t)g.v.C * 9 * g.cin));
    r.p.push_back(vector_f32_grad(g.v.C)); r.p.push_back(vector_f32_grad(g.v.C));
    r.p.push_back(matrix((uint64_t)g.v.C * 9 * g.v.C));
    r.p.push_back(vector_f32_grad(g.v.C)); r.p.push_back(vector_f32_grad(g.v.C));
    r.out_bytes = (uint64_t)g.v.P() * g.v.C * 2;
    r.sav_bytes = g.saved().total;
    r.ws_bytes = g.work().total;
    c.rec.push_back(std::move(r));
  }
  for (int l = net.D - 1; l >= 0; --l) {
    UpGeom g(net, l);
    Record r;
    r.kind = REC_UNET_UP;
    r.p.push_back(matrix((uint64_t)g.below.C * 4 * g.v.C));
    r.p.push_back(matrix((uint64_t)g.v.C * 9 * g.v.C));
    r.p.push_back(matrix((uint64_t)g.v.C * 9 * g.v.C));
    r.p.push_back(vector_f32_grad(g.v.C)); r.p.push_back(vector_f32_grad(g.v.C));
    r.p.push_back(matrix((uint64_t)g.v.C * 9 * g.v.C));
    r.p.push_back(vector_f32_grad(g.v.C)); r.p.push_back(vector_f32_grad(g.v.C));
    r.out_bytes = (uint64_t)g.v.P() * g.v.C * 2;
    r.sav_bytes = g.saved().total;
    r.ws_bytes = g.work().total;
    c.rec.push_back(std::move(r));
  }
  Record head;
  head.kind = REC_LOSS_UNET_HEAD;
  head.p.push_back(matrix((uint64_t)net.classes * net.width));
  head.p.push_back(vector_f32_grad(net.classes));
  head.ws_bytes = HeadWs(net).total;
  c.rec.push_back(std::move(head));
  c.in_bytes = (uint64_t)net.N * net.S * net.S * IMG_C * 2;
  c.lab_bytes = (uint64_t)net.N * net.S * net.S * 4;
  c.misc_bytes = 0;
  return unet_skips(d, c.skips);
}

// images fp32 [N][S][S] (one channel) -> bf16 [N][S][S][8] (round to nearest even, channels 1..7 zero);
// labels int32 [N][S][S]
int unet_prepare_step(Ctx& c, const void* in, const void* lab) {
  UNet net(c.desc);
  const size_t pixels = (size_t)net.N * net.S * net.S;
  const int32_t* labels = (const int32_t*)lab;
  std::atomic<bool> bad{false};
  c.pool->parallel_for(pixels, [&](size_t lo, size_t hi) {
    bool b = false;
    for (size_t p = lo; p < hi; ++p) b |= labels[p] < 0 || labels[p] >= net.classes;
    if (b) bad = true;
  });
  if (bad) {
    c.err = "label outside the classes";
    return KARMA_E_INVAL;
  }
  const float* img = (const float*)in;
  uint16_t* out = (uint16_t*)c.stage_in;
  c.pool->parallel_for(pixels, [&](size_t lo, size_t hi) {
    for (size_t p = lo; p < hi; ++p) {
      uint16_t* o = out + p * IMG_C;
      o[0] = f32_to_bf16_rne(img[p]);
      for (int ch = 1; ch < IMG_C; ++ch) o[ch] = 0;
    }
  });
  std::memcpy(c.stage_lab, lab, c.lab_bytes);
  return KARMA_OK;
}

int unet_prepare_late(Ctx&) { return KARMA_OK; }

namespace {

// the two convolutions with their normalisations, from the first convolution's output on
int level_tail_fwd(const Level& v, const Saved& sv, const Work& wl, char* S, char* Wk, const bf16_t* g1, const bf16_t* b1,
                   const bf16_t* w2, const bf16_t* g2, const bf16_t* b2, void* out, hipStream_t s) {
  bf16_t* c1 = (bf16_t*)(S + sv.c1);
  bf16_t* a1 = (bf16_t*)(S + sv.a1);
  bf16_t* c2 = (bf16_t*)(S + sv.c2);
  float* bnws = (float*)(Wk + wl.bn);
  TRY(bn_fwd(c1, g1, b1, nullptr, a1, (float*)(S + sv.st1), bnws, v.P(), v.C, 1, s));
  TRY(conv2d_fwd(a1, w2, c2, conv3(v, v.C), s, Wk + wl.splitk, wl.splitk_bytes));
  if (out) return bn_fwd(c2, g2, b2, nullptr, (bf16_t*)out, (float*)(S + sv.st2), bnws, v.P(), v.C, 1, s);
  // a recompute whose output still exists needs the statistics only; the normalised tensor goes to the workspace
  return bn_fwd(c2, g2, b2, nullptr, (bf16_t*)(Wk + wl.m1), (float*)(S + sv.st2), bnws, v.P(), v.C, 1, s);
}

}  // namespace

int unet_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  UNet net(c.desc);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t, io.w); };
  const int l = net.level_of(i);
  if (net.down(i)) {
    DownGeom g(net, l);
    Saved sv = g.saved();
    Work wl = g.work();
    const bf16_t* first = (const bf16_t*)io.x;
    if (g.pooled) {
      bf16_t* pooled = (bf16_t*)(S + sv.head);
      TRY(maxpool2_fwd((const bf16_t*)io.x, pooled, g.v.N, 2 * g.v.S, 2 * g.v.S, g.cin, s));
      first = pooled;
    }
    TRY(conv2d_fwd(first, W(DW1), (bf16_t*)(S + sv.c1), conv3(g.v, g.cin), s, Wk + wl.splitk, wl.splitk_bytes));
    return level_tail_fwd(g.v, sv, wl, S, Wk, W(DG1), W(DB1), W(DW2), W(DG2), W(DB2), io.out, s);
  }
  if (io.n_skips != 1 || !io.skip_x[0]) return KARMA_E_INVAL;
  UpGeom g(net, l);
  Saved sv = g.saved();
  Work wl = g.work();
  bf16_t* up = (bf16_t*)(S + sv.head);
  bf16_t* half = (bf16_t*)(Wk + wl.m1);
  TRY(conv2d_dgrad((const bf16_t*)io.x, W(UWU), (bf16_t*)(Wk + wl.wt), nullptr, up, g.conv_of_up(), s, Wk + wl.splitk,
                   wl.splitk_bytes));
  TRY(conv2d_fwd((const bf16_t*)io.skip_x[0], W(UW1S), half, conv3(g.v, g.v.C), s, Wk + wl.splitk, wl.splitk_bytes));
  TRY(conv2d_fwd(up, W(UW1U), (bf16_t*)(S + sv.c1), conv3(g.v, g.v.C), s, Wk + wl.splitk, wl.splitk_bytes, half));
  return level_tail_fwd(g.v, sv, wl, S, Wk, W(UG1), W(UB1), W(UW2), W(UG2), W(UB2), io.out, s);
}

int unet_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  UNet net(c.desc);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  const bf16_t* dy = (const bf16_t*)io.dy;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t, io.w); };
  auto G = [&](int t) { return c.g_ptr(i, t, io.g); };
  const int l = net.level_of(i);
  const bool down = net.down(i);
  const Level v = net.level(l);
  Saved sv = down ? DownGeom(net, l).saved() : UpGeom(net, l).saved();
  Work wl = down ? DownGeom(net, l).work() : UpGeom(net, l).work();
  const int g1 = down ? DG1 : UG1, b1 = down ? DB1 : UB1, w2 = down ? DW2 : UW2, g2 = down ? DG2 : UG2, b2 = down ? DB2 : UB2;
  const bf16_t* c1 = (const bf16_t*)(S + sv.c1);
  const bf16_t* a1 = (const bf16_t*)(S + sv.a1);
  const bf16_t* c2 = (const bf16_t*)(S + sv.c2);
  const float* st1 = (const float*)(S + sv.st1);
  const float* st2 = (const float*)(S + sv.st2);
  bf16_t* m1 = (bf16_t*)(Wk + wl.m1);
  bf16_t* m2 = (bf16_t*)(Wk + wl.m2);
  bf16_t* wt = (bf16_t*)(Wk + wl.wt);
  float* bnws = (float*)(Wk + wl.bn);
  void* sk = Wk + wl.splitk;
  const ConvShape inner = conv3(v, v.C);
  // through the second normalisation and convolution, then the first normalisation: m1 = gradient of the
  // first convolution's output
  TRY(bn_bwd(dy, c2, st2, W(g2), W(b2), 1, m2, (float*)G(g2), (float*)G(b2), bnws, v.P(), v.C, s));
  TRY(conv2d_wgrad(m2, a1, (bf16_t*)G(w2), sk, wl.splitk_bytes, inner, s));
  TRY(conv2d_dgrad(m2, W(w2), wt, nullptr, m1, inner, s, sk, wl.splitk_bytes));
  TRY(bn_bwd(m1, c1, st1, W(g1), W(b1), 1, m1, (float*)G(g1), (float*)G(b1), bnws, v.P(), v.C, s));
  if (down) {
    DownGeom g(net, l);
    const bf16_t* first = g.pooled ? (const bf16_t*)(S + sv.head) : (const bf16_t*)io.x;
    TRY(conv2d_wgrad(m1, first, (bf16_t*)G(DW1), sk, wl.splitk_bytes, conv3(v, g.cin), s));
    if (!g.pooled) return KARMA_OK;   // level 0 reads the images
    TRY(conv2d_dgrad(m1, W(DW1), wt, nullptr, m2, conv3(v, g.cin), s, sk, wl.splitk_bytes));
    return maxpool2_bwd((const bf16_t*)io.x, m2, (bf16_t*)io.dx, v.N, 2 * v.S, 2 * v.S, g.cin, s);
  }
  if (io.n_skips != 1 || !io.skip_x[0] || !io.skip_dx[0]) return KARMA_E_INVAL;
  UpGeom g(net, l);
  const bf16_t* up = (const bf16_t*)(S + sv.head);
  const bf16_t* skip = (const bf16_t*)io.skip_x[0];
  TRY(conv2d_wgrad(m1, skip, (bf16_t*)G(UW1S), sk, wl.splitk_bytes, inner, s));
  TRY(conv2d_wgrad(m1, up, (bf16_t*)G(UW1U), sk, wl.splitk_bytes, inner, s));
  // the contracting output's share of the gradient, left for the backward op of the record that reads it as its input
  if (io.skip_dx_first[0]) {
    TRY(conv2d_dgrad(m1, W(UW1S), wt, nullptr, (bf16_t*)io.skip_dx[0], inner, s, sk, wl.splitk_bytes));
  } else {
    TRY(conv2d_dgrad(m1, W(UW1S), wt, nullptr, m2, inner, s, sk, wl.splitk_bytes));
    TRY(add_inplace_bf16((bf16_t*)io.skip_dx[0], m2, (size_t)v.P() * v.C, s));
  }
  TRY(conv2d_dgrad(m1, W(UW1U), wt, nullptr, m2, inner, s, sk, wl.splitk_bytes));   // gradient of the up-convolution's result
  const ConvShape k = g.conv_of_up();
  TRY(conv2d_wgrad((const bf16_t*)io.x, m2, (bf16_t*)G(UWU), sk, wl.splitk_bytes, k, s));
  return conv2d_fwd(m2, W(UWU), (bf16_t*)io.dx, k, s, sk, wl.splitk_bytes);
}

// 1x1 classifier, mean cross entropy over the pixels, and their gradients
int unet_loss(Ctx& c, const LayerIO& io, hipStream_t s) {
  UNet net(c.desc);
  HeadWs wl(net);
  const uint32_t R = c.L;
  char* Wk = (char*)io.ws;
  bf16_t* logits = (bf16_t*)(Wk + wl.logits);
  float* rowloss = (float*)(Wk + wl.rowloss);
  float* part = (float*)(Wk + wl.part);
  const bf16_t* x = (const bf16_t*)io.x;
  const bf16_t* w = (const bf16_t*)c.w_ptr(R, HW);
  const bf16_t* bias = (const bf16_t*)c.w_ptr(R, HBIAS);
  const int* labels = (const int*)c.fixed_ptr(c.lab_off);
  const int pixels = net.level(0).P(), C = net.width, K = net.classes;
  GemmArgs f{};   // logits = x w^T + bias
  f.A = x; f.B = w; f.C = logits; f.bias = bias;
  f.M = pixels; f.N = K; f.K = C; f.a_kc = f.b_kc = true; f.lda = C; f.ldb = C; f.ldc = K;
  TRY(gemm_bf16(f, s));
  TRY(softmax_ce(logits, labels, rowloss, pixels, K, 1.f / (float)pixels, s));   // logits -> dlogits
  TRY(sum_f32(rowloss, (float*)c.fixed_ptr(c.loss_off), part, (size_t)pixels, 1.f / (float)pixels, s));
  GemmArgs dw{};  // dW = dlogits^T x: a long reduction over the pixels, split
  dw.A = logits; dw.B = x; dw.C = c.g_ptr(R, HW);
  dw.M = K; dw.N = C; dw.K = pixels; dw.a_kc = dw.b_kc = false; dw.lda = K; dw.ldb = C; dw.ldc = C;
  dw.ws = Wk + wl.splitk; dw.ws_bytes = wl.splitk_bytes;
  TRY(gemm_bf16(dw, s));
  TRY(colsum_bf16(logits, (float*)c.g_ptr(R, HBIAS), part, pixels, K, s));
  GemmArgs dx{};  // dx = dlogits w
  dx.A = logits; dx.B = w; dx.C = io.dx;
  dx.M = pixels; dx.N = C; dx.K = K; dx.a_kc = true; dx.b_kc = false; dx.lda = K; dx.ldb = C; dx.ldc = C;
  return gemm_bf16(dx, s);
}

}  // namespace karma
