// GPT-style transformer workload: token + position embedding, pre-LN blocks
//   x += Proj(Attn(LN1(x)));  x += FC2(GELU(FC1(LN2(x))))
// and a loss op made of the final LayerNorm, the LM head tied to the token embedding and
// the mean next-token cross-entropy.  bf16 tensors in HBM, fp32 accumulation everywhere.
// The layer types are those of KARMA Sec. III-C (fully connected, self-attention, softmax);
// the block is the unit the planner keeps, swaps or recomputes.
#include <algorithm>
#include <cstring>
#include <numeric>

#include "kernels.h"
#include "layers.h"

namespace karma {

namespace {

inline uint64_t up256(uint64_t b) { return (b + 255) / 256 * 256; }

struct Dims {
  int B, S, H, D, h, ffn, V, T;
  explicit Dims(const karma_model_desc& d)
      : B((int)d.batch), S((int)d.seq), H((int)d.n_heads), D((int)(d.width / d.n_heads)), h((int)d.width),
        ffn((int)d.ffn), V((int)d.vocab), T((int)(d.batch * d.seq)) {}
};

// internals of one block, in the order they are produced
struct BlockSaved {
  uint64_t a, stats1, qkv, ctx, lse, r1, stats2, m, f1, g, total;
  explicit BlockSaved(const Dims& d) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    a = take((uint64_t)d.T * d.h * 2);
    stats1 = take((uint64_t)d.T * 2 * 4);
    qkv = take((uint64_t)d.T * 3 * d.h * 2);
    ctx = take((uint64_t)d.T * d.h * 2);
    lse = take((uint64_t)d.B * d.H * d.S * 4);
    r1 = take((uint64_t)d.T * d.h * 2);
    stats2 = take((uint64_t)d.T * 2 * 4);
    m = take((uint64_t)d.T * d.h * 2);
    f1 = take((uint64_t)d.T * d.ffn * 2);
    g = take((uint64_t)d.T * d.ffn * 2);
    total = o;
  }
};

// the same internals when a block is two records: the attention half keeps a .. lse and hands r1 on as its
// output, the feed-forward half (whose input is r1) keeps stats2 .. g
struct AttnSaved {
  uint64_t a, stats1, qkv, ctx, lse, total;
  explicit AttnSaved(const Dims& d) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    a = take((uint64_t)d.T * d.h * 2);
    stats1 = take((uint64_t)d.T * 2 * 4);
    qkv = take((uint64_t)d.T * 3 * d.h * 2);
    ctx = take((uint64_t)d.T * d.h * 2);
    lse = take((uint64_t)d.B * d.H * d.S * 4);
    total = o;
  }
};
struct FfnSaved {
  uint64_t stats2, m, f1, g, total;
  explicit FfnSaved(const Dims& d) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    stats2 = take((uint64_t)d.T * 2 * 4);
    m = take((uint64_t)d.T * d.h * 2);
    f1 = take((uint64_t)d.T * d.ffn * 2);
    g = take((uint64_t)d.T * d.ffn * 2);
    total = o;
  }
};

// backward workspace of one block
struct BlockWs {
  uint64_t wide, t1, t2, t3, delta, part, splitk, splitk_bytes, total;
  explicit BlockWs(const Dims& d) {
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    wide = take((uint64_t)d.T * std::max(d.ffn, 3 * d.h) * 2);   // dg -> df1, later dqkv
    t1 = take((uint64_t)d.T * d.h * 2);                           // dm, later dctx
    t2 = take((uint64_t)d.T * d.h * 2);                           // dr1
    t3 = take((uint64_t)d.T * d.h * 2);                           // da
    delta = take((uint64_t)d.B * d.H * d.S * 4);
    part = take(std::max({layernorm_bwd_ws_bytes(d.T, d.h), colsum_ws_bytes(d.T, std::max(d.ffn, 3 * d.h)),
                          attention_bwd_colsum_bytes(d.B, d.S, d.H, d.D)}));
    splitk_bytes = (uint64_t)8 * std::max(d.ffn, 3 * d.h) * d.h * 4;   // partial sums of the weight-gradient GEMMs
    splitk = take(splitk_bytes);
    total = o;
  }
};

constexpr int HEAD_CHUNK = 4096;   // tokens per LM-head chunk: the full logits never exist

struct LossWs {
  uint64_t xf, stats, logits, dxf, rowloss, part, splitk, splitk_bytes, total;
  int chunk;
  explicit LossWs(const Dims& d) {
    chunk = std::min(d.T, HEAD_CHUNK);
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o += up256(bytes); return at; };
    xf = take((uint64_t)d.T * d.h * 2);
    stats = take((uint64_t)d.T * 2 * 4);
    logits = take((uint64_t)chunk * d.V * 2);
    dxf = take((uint64_t)d.T * d.h * 2);
    rowloss = take((uint64_t)d.T * 4);
    part = take(std::max<uint64_t>(layernorm_bwd_ws_bytes(d.T, d.h), 1024 * 4));
    splitk_bytes = (uint64_t)8 * chunk * d.h * 4;   // the dx GEMM of a chunk has few tiles and a long reduction
    splitk = take(splitk_bytes);
    total = o;
  }
};

enum BlockParam { LN1_G, LN1_B, WQKV, BQKV, WO, BO, LN2_G, LN2_B, W1, B1, W2, B2 };

Param make_param(uint64_t n, bool matrix) {
  Param p;
  p.n = n;
  p.dev_bf16 = true;
  p.grad_bf16 = matrix;   // vectors (biases, LayerNorm parameters) keep fp32 gradients
  return p;
}

int gemm_raw(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* bias, const bf16_t* res, int M, int N, int K,
             bool a_kc, bool b_kc, bool out_f32, bool acc, hipStream_t s, void* ws, size_t ws_bytes) {
  GemmArgs g{};
  g.A = A; g.B = B; g.C = C; g.bias = bias; g.residual = res;
  g.M = M; g.N = N; g.K = K;
  g.a_kc = a_kc; g.b_kc = b_kc;
  g.lda = a_kc ? K : M;
  g.ldb = b_kc ? K : N;
  g.ldc = N;
  g.out_f32 = out_f32; g.accumulate = acc;
  g.ws = ws; g.ws_bytes = ws_bytes;
  return gemm_bf16(g, s);
}

int gemm(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* bias, const bf16_t* res, int M, int N, int K,
         bool a_kc, bool b_kc, bool out_f32, bool acc, hipStream_t s, void* ws = nullptr, size_t ws_bytes = 0) {
  return gemm_raw(A, B, C, bias, res, M, N, K, a_kc, b_kc, out_f32, acc, s, ws, ws_bytes);
}

// the product with the feed-forward GELU folded into its output stage (mode 1: aux = GELU(C) written;
// mode 2: C = (A B^T) * GELU'(aux))
int gemm_gelu(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* bias, bf16_t* aux, int M, int N, int K, bool a_kc,
              bool b_kc, int mode, hipStream_t s, float* colsum_partial = nullptr, int* colsum_rows = nullptr) {
  GemmArgs g{};
  g.A = A; g.B = B; g.C = C; g.bias = bias;
  g.M = M; g.N = N; g.K = K;
  g.a_kc = a_kc; g.b_kc = b_kc;
  g.lda = a_kc ? K : M;
  g.ldb = b_kc ? K : N;
  g.ldc = N;
  g.act = mode;
  g.aux = aux;
  g.colsum_partial = colsum_partial;
  g.colsum_rows = colsum_rows;
  return gemm_bf16(g, s);
}

#define TRY(call)          \
  do {                     \
    int st_ = (call);      \
    if (st_) return st_;   \
  } while (0)

}  // namespace

int gpt_build_records(Ctx& c) {
  const karma_model_desc& md = c.desc;
  if (!md.n_layers || !md.width || !md.batch || !md.seq || !md.n_heads || !md.ffn || !md.vocab) return KARMA_E_INVAL;
  if (md.width % md.n_heads) return KARMA_E_INVAL;
  if (md.split_blocks > 1) return KARMA_E_INVAL;
  Dims d(md);
  if ((d.D != 64 && d.D != 128 && d.D != 152) || d.S % 128 || d.h % 8 || d.ffn % 8 || d.V % 8) return KARMA_E_INVAL;
  if ((uint64_t)d.V * 2 > 150 * 1024) return KARMA_E_INVAL;
  const uint64_t act = (uint64_t)d.T * d.h * 2;
  c.rec.clear();
  Record emb;
  emb.kind = REC_EMBED;
  emb.p.push_back(make_param((uint64_t)d.V * d.h, true));
  emb.p.back().grad_bf16 = false;   // fp32 accumulator: LM head chunks + scatter-add land here
  emb.p.push_back(make_param((uint64_t)d.S * d.h, true));
  emb.out_bytes = act;
  c.rec.push_back(std::move(emb));
  BlockSaved sv(d);
  AttnSaved asv(d);
  FfnSaved fsv(d);
  BlockWs ws(d);
  for (uint32_t i = 0; i < md.n_layers; ++i) {
    std::vector<Param> p(12);
    p[LN1_G] = make_param(d.h, false); p[LN1_B] = make_param(d.h, false);
    p[WQKV] = make_param((uint64_t)3 * d.h * d.h, true); p[BQKV] = make_param(3 * d.h, false);
    p[WO] = make_param((uint64_t)d.h * d.h, true); p[BO] = make_param(d.h, false);
    p[LN2_G] = make_param(d.h, false); p[LN2_B] = make_param(d.h, false);
    p[W1] = make_param((uint64_t)d.ffn * d.h, true); p[B1] = make_param(d.ffn, false);
    p[W2] = make_param((uint64_t)d.h * d.ffn, true); p[B2] = make_param(d.h, false);
    // one record per block, or its two halves (tensors 0..5 and 6..11) as records of their own
    for (int half = 0; half < (md.split_blocks ? 2 : 1); ++half) {
      Record r;
      r.kind = md.split_blocks ? (half == 0 ? REC_ATTN : REC_FFN) : REC_BLOCK;
      if (!md.split_blocks) r.p = p;
      else r.p.assign(p.begin() + 6 * half, p.begin() + 6 * half + 6);
      r.out_bytes = act;
      r.sav_bytes = !md.split_blocks ? sv.total : half == 0 ? asv.total : fsv.total;
      r.ws_bytes = ws.total;
      r.streamed = md.stream_weights != 0;
      c.rec.push_back(std::move(r));
    }
  }
  Record loss;
  loss.kind = REC_LOSS_LMHEAD;
  loss.p.push_back(make_param(d.h, false));
  loss.p.push_back(make_param(d.h, false));
  loss.ws_bytes = LossWs(d).total;
  c.rec.push_back(std::move(loss));
  c.in_bytes = (uint64_t)d.T * 4;
  c.lab_bytes = (uint64_t)d.T * 4;
  c.misc_bytes = ((uint64_t)3 * d.T + 1) * 4;   // order[T], seg_start[T+1], seg_id[T]
  return KARMA_OK;
}

// Host-side preparation: ids/labels into the staging buffers.
int gpt_prepare_step(Ctx& c, const void* in, const void* lab) {
  Dims d(c.desc);
  const int32_t* ids = (const int32_t*)in;
  const int32_t* labels = (const int32_t*)lab;
  for (int t = 0; t < d.T; ++t)
    if (ids[t] < 0 || ids[t] >= d.V || labels[t] < 0 || labels[t] >= d.V) {
      c.err = "token id or label outside the vocabulary";
      return KARMA_E_INVAL;
    }
  std::memcpy(c.stage_in, in, c.in_bytes);
  std::memcpy(c.stage_lab, lab, c.lab_bytes);
  return KARMA_OK;
}

// Stable sort of the token positions by id for the atomic-free embedding gradient: only the
// very last backward op needs it, so it runs on the host while the GPU computes.
int gpt_prepare_late(Ctx& c) {
  Dims d(c.desc);
  const int32_t* ids = (const int32_t*)c.stage_in;
  int32_t* order = (int32_t*)c.stage_misc;
  int32_t* seg_start = order + d.T;
  int32_t* seg_id = seg_start + d.T + 1;
  std::iota(order, order + d.T, 0);
  std::stable_sort(order, order + d.T, [&](int32_t a, int32_t b) { return ids[a] < ids[b]; });
  int n = 0;
  for (int p = 0; p < d.T; ++p)
    if (p == 0 || ids[order[p]] != ids[order[p - 1]]) {
      seg_start[n] = p;
      seg_id[n] = ids[order[p]];
      ++n;
    }
  seg_start[n] = d.T;
  c.n_segments = (uint32_t)n;
  return KARMA_OK;
}

namespace {

// The two halves of a block.  Pointers into the saved set and the workspace are handed in, so that the same
// code serves a whole-block record (one saved set, r1 inside it) and the split records (r1 is the attention
// half's output and the feed-forward half's input).  W / G: the record's weight / gradient tensor of a
// BlockParam, wherever the record keeps it.
struct AttnBufs {
  bf16_t* a; float* stats1; bf16_t* qkv; bf16_t* ctx; float* lse;
};
struct FfnBufs {
  float* stats2; bf16_t* m; bf16_t* f1; bf16_t* g;
};
struct BwdBufs {
  bf16_t* wide; bf16_t* t1; bf16_t* t3; float* delta; float* part; char* splitk; uint64_t splitk_bytes;
};

template <class WF>
int attn_half_fwd(const Dims& d, const bf16_t* x, const AttnBufs& b, bf16_t* r1, WF W, hipStream_t s) {
  TRY(layernorm_fwd(x, W(LN1_G), W(LN1_B), b.a, b.stats1, d.T, d.h, s));
  TRY(gemm(b.a, W(WQKV), b.qkv, W(BQKV), nullptr, d.T, 3 * d.h, d.h, true, true, false, false, s));
  TRY(attention_fwd(b.qkv, b.ctx, b.lse, d.B, d.S, d.H, d.D, s));
  // a recompute whose output nobody needs stops here: backward only reads the internals
  if (r1) TRY(gemm(b.ctx, W(WO), r1, W(BO), x, d.T, d.h, d.h, true, true, false, false, s));
  return KARMA_OK;
}

template <class WF>
int ffn_half_fwd(const Dims& d, const bf16_t* r1, const FfnBufs& b, bf16_t* out, WF W, hipStream_t s) {
  TRY(layernorm_fwd(r1, W(LN2_G), W(LN2_B), b.m, b.stats2, d.T, d.h, s));
  TRY(gemm_gelu(b.m, W(W1), b.f1, W(B1), b.g, d.T, d.ffn, d.h, true, true, 1, s));   // f1 = m W1^T + b1, g = GELU(f1)
  if (out) TRY(gemm(b.g, W(W2), out, W(B2), r1, d.T, d.h, d.ffn, true, true, false, false, s));
  return KARMA_OK;
}

// y = r1 + g W2^T + b2 back to dr1 = LN2'(dm) + dy
template <class WF, class GF>
int ffn_half_bwd(const Dims& d, const bf16_t* dy, const bf16_t* r1, const FfnBufs& b, const BwdBufs& w, bf16_t* dr1, WF W,
                 GF G, hipStream_t s) {
  // df1 = (dy W2) * GELU'(f1); where the kernel can, it leaves partial column sums of df1 (FC1's bias gradient)
  int sum_rows = 0;
  TRY(gemm_gelu(dy, W(W2), w.wide, nullptr, b.f1, d.T, d.ffn, d.h, true, false, 2, s, w.part, &sum_rows));
  if (sum_rows) TRY(colsum_finish(w.part, sum_rows, d.ffn, (float*)G(B1), s));
  TRY(gemm(dy, b.g, G(W2), nullptr, nullptr, d.h, d.ffn, d.T, false, false, false, false, s, w.splitk, w.splitk_bytes));        // dW2 = dy^T g
  TRY(gemm(w.wide, W(W1), w.t1, nullptr, nullptr, d.T, d.h, d.ffn, true, false, false, false, s));      // dm = df1 W1
  TRY(gemm(w.wide, b.m, G(W1), nullptr, nullptr, d.ffn, d.h, d.T, false, false, false, false, s, w.splitk, w.splitk_bytes));    // dW1 = df1^T m
  if (!sum_rows) TRY(colsum_bf16(w.wide, (float*)G(B1), w.part, d.T, d.ffn, s));
  // dr1 = LN2'(dm) + dy; the same pass sums dy's columns: the gradient of FC2's bias
  TRY(layernorm_bwd(w.t1, r1, b.stats2, W(LN2_G), dy, dr1, (float*)G(LN2_G), (float*)G(LN2_B), w.part, d.T, d.h, s,
                    (float*)G(B2)));
  return KARMA_OK;
}

// r1 = x + ctx Wo^T + bo back to dx = LN1'(da) + dr1
template <class WF, class GF>
int attn_half_bwd(const Dims& d, const bf16_t* dr1, const bf16_t* x, const AttnBufs& b, const BwdBufs& w, bf16_t* dx, WF W,
                  GF G, hipStream_t s) {
  TRY(gemm(dr1, W(WO), w.t1, nullptr, nullptr, d.T, d.h, d.h, true, false, false, false, s));         // dctx = dr1 Wo
  TRY(gemm(dr1, b.ctx, G(WO), nullptr, nullptr, d.h, d.h, d.T, false, false, false, false, s, w.splitk, w.splitk_bytes));       // dWo = dr1^T ctx
  // where the kernels can they leave partial column sums of dqkv (the QKV bias gradient) in the workspace
  int sum_rows = 0;
  TRY(attention_bwd(b.qkv, b.ctx, w.t1, b.lse, w.delta, w.wide, d.B, d.S, d.H, d.D, s, w.part, &sum_rows));
  if (sum_rows) TRY(colsum_finish(w.part, sum_rows, 3 * d.h, (float*)G(BQKV), s));
  TRY(gemm(w.wide, W(WQKV), w.t3, nullptr, nullptr, d.T, d.h, 3 * d.h, true, false, false, false, s));  // da = dqkv Wqkv
  TRY(gemm(w.wide, b.a, G(WQKV), nullptr, nullptr, 3 * d.h, d.h, d.T, false, false, false, false, s, w.splitk, w.splitk_bytes));  // dWqkv = dqkv^T a
  if (!sum_rows) TRY(colsum_bf16(w.wide, (float*)G(BQKV), w.part, d.T, 3 * d.h, s));
  // dx = LN1'(da) + dr1; the same pass sums dr1's columns: the gradient of the output projection's bias
  TRY(layernorm_bwd(w.t3, x, b.stats1, W(LN1_G), dr1, dx, (float*)G(LN1_G), (float*)G(LN1_B), w.part, d.T, d.h, s,
                    (float*)G(BO)));
  return KARMA_OK;
}

}  // namespace

int gpt_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  Dims d(c.desc);
  if (i == 0) {
    if (!io.out) return KARMA_OK;
    return embed_fwd((const int*)io.x, (const bf16_t*)c.w_ptr(0, 0), (const bf16_t*)c.w_ptr(0, 1), (bf16_t*)io.out, d.T,
                     d.S, d.h, s);
  }
  char* S = (char*)io.sav;
  const bf16_t* x = (const bf16_t*)io.x;
  const int kind = c.rec[i].kind;
  // a split record holds six of the block's twelve tensors: the feed-forward half's start at LN2_G
  const int first = kind == REC_FFN ? (int)LN2_G : 0;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t - first, io.w); };
  if (kind == REC_ATTN) {
    AttnSaved sv(d);
    AttnBufs ab{(bf16_t*)(S + sv.a), (float*)(S + sv.stats1), (bf16_t*)(S + sv.qkv), (bf16_t*)(S + sv.ctx), (float*)(S + sv.lse)};
    return attn_half_fwd(d, x, ab, (bf16_t*)io.out, W, s);
  }
  if (kind == REC_FFN) {
    FfnSaved sv(d);
    FfnBufs fb{(float*)(S + sv.stats2), (bf16_t*)(S + sv.m), (bf16_t*)(S + sv.f1), (bf16_t*)(S + sv.g)};
    return ffn_half_fwd(d, x, fb, (bf16_t*)io.out, W, s);
  }
  BlockSaved sv(d);
  AttnBufs ab{(bf16_t*)(S + sv.a), (float*)(S + sv.stats1), (bf16_t*)(S + sv.qkv), (bf16_t*)(S + sv.ctx), (float*)(S + sv.lse)};
  FfnBufs fb{(float*)(S + sv.stats2), (bf16_t*)(S + sv.m), (bf16_t*)(S + sv.f1), (bf16_t*)(S + sv.g)};
  bf16_t* r1 = (bf16_t*)(S + sv.r1);
  TRY(attn_half_fwd(d, x, ab, r1, W, s));
  return ffn_half_fwd(d, r1, fb, (bf16_t*)io.out, W, s);
}

int gpt_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s) {
  Dims d(c.desc);
  const bf16_t* dy = (const bf16_t*)io.dy;
  if (i == 0) {
    const int32_t* order = (const int32_t*)c.fixed_ptr(c.misc_off);
    const int32_t* seg_start = order + d.T;
    const int32_t* seg_id = seg_start + d.T + 1;
    return embed_bwd(dy, order, seg_start, seg_id, (int)c.n_segments, (float*)c.g_ptr(0, 0), (bf16_t*)c.g_ptr(0, 1),
                     d.B, d.S, d.h, s);
  }
  BlockWs wl(d);
  char* S = (char*)io.sav;
  char* Wk = (char*)io.ws;
  const bf16_t* x = (const bf16_t*)io.x;
  BwdBufs wb{(bf16_t*)(Wk + wl.wide), (bf16_t*)(Wk + wl.t1), (bf16_t*)(Wk + wl.t3), (float*)(Wk + wl.delta),
             (float*)(Wk + wl.part), Wk + wl.splitk, wl.splitk_bytes};
  const int kind = c.rec[i].kind;
  const int first = kind == REC_FFN ? (int)LN2_G : 0;
  auto W = [&](int t) { return (const bf16_t*)c.w_ptr(i, t - first, io.w); };
  auto G = [&](int t) { return c.g_ptr(i, t - first, io.g); };
  if (kind == REC_ATTN) {
    AttnSaved sv(d);
    AttnBufs ab{(bf16_t*)(S + sv.a), (float*)(S + sv.stats1), (bf16_t*)(S + sv.qkv), (bf16_t*)(S + sv.ctx), (float*)(S + sv.lse)};
    return attn_half_bwd(d, dy, x, ab, wb, (bf16_t*)io.dx, W, G, s);
  }
  if (kind == REC_FFN) {
    FfnSaved sv(d);
    FfnBufs fb{(float*)(S + sv.stats2), (bf16_t*)(S + sv.m), (bf16_t*)(S + sv.f1), (bf16_t*)(S + sv.g)};
    return ffn_half_bwd(d, dy, x, fb, wb, (bf16_t*)io.dx, W, G, s);
  }
  BlockSaved sv(d);
  AttnBufs ab{(bf16_t*)(S + sv.a), (float*)(S + sv.stats1), (bf16_t*)(S + sv.qkv), (bf16_t*)(S + sv.ctx), (float*)(S + sv.lse)};
  FfnBufs fb{(float*)(S + sv.stats2), (bf16_t*)(S + sv.m), (bf16_t*)(S + sv.f1), (bf16_t*)(S + sv.g)};
  bf16_t* dr1 = (bf16_t*)(Wk + wl.t2);
  TRY(ffn_half_bwd(d, dy, (const bf16_t*)(S + sv.r1), fb, wb, dr1, W, G, s));
  return attn_half_bwd(d, dr1, x, ab, wb, (bf16_t*)io.dx, W, G, s);
}

// Final LayerNorm, tied LM head and mean cross-entropy with their gradients, chunked over
// tokens so that only HEAD_CHUNK rows of logits exist at a time.
int gpt_loss(Ctx& c, const LayerIO& io, hipStream_t s) {
  Dims d(c.desc);
  LossWs wl(d);
  const uint32_t R = c.L;   // the loss record
  char* Wk = (char*)io.ws;
  const bf16_t* x = (const bf16_t*)io.x;
  bf16_t* xf = (bf16_t*)(Wk + wl.xf);
  float* stats = (float*)(Wk + wl.stats);
  bf16_t* logits = (bf16_t*)(Wk + wl.logits);
  bf16_t* dxf = (bf16_t*)(Wk + wl.dxf);
  float* rowloss = (float*)(Wk + wl.rowloss);
  float* part = (float*)(Wk + wl.part);
  const bf16_t* wte = (const bf16_t*)c.w_ptr(0, 0);
  float* dwte = (float*)c.g_ptr(0, 0);
  const int* labels = (const int*)c.fixed_ptr(c.lab_off);
  TRY(fill_zero(dwte, (size_t)d.V * d.h * 4, s));
  TRY(layernorm_fwd(x, (const bf16_t*)c.w_ptr(R, 0), (const bf16_t*)c.w_ptr(R, 1), xf, stats, d.T, d.h, s));
  for (int t0 = 0; t0 < d.T; t0 += wl.chunk) {
    const int n = std::min(wl.chunk, d.T - t0);
    const bf16_t* xc = xf + (size_t)t0 * d.h;
    TRY(gemm(xc, wte, logits, nullptr, nullptr, n, d.V, d.h, true, true, false, false, s));          // logits = xf wte^T
    TRY(softmax_ce(logits, labels + t0, rowloss + t0, n, d.V, 1.0f / (float)d.T, s));                 // -> dlogits
    TRY(gemm(logits, wte, dxf + (size_t)t0 * d.h, nullptr, nullptr, n, d.h, d.V, true, false, false, false, s,
             Wk + wl.splitk, wl.splitk_bytes));
    TRY(gemm(logits, xc, dwte, nullptr, nullptr, d.V, d.h, n, false, false, true, true, s));          // dwte += dlogits^T xf
  }
  TRY(sum_f32(rowloss, (float*)c.fixed_ptr(c.loss_off), part, (size_t)d.T, 1.0f / (float)d.T, s));
  TRY(layernorm_bwd(dxf, x, stats, (const bf16_t*)c.w_ptr(R, 0), nullptr, (bf16_t*)io.dx, (float*)c.g_ptr(R, 0),
                    (float*)c.g_ptr(R, 1), part, d.T, d.h, s));
  return KARMA_OK;
}

}  // namespace karma
