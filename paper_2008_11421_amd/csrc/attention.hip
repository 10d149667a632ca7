// Fused causal self-attention on the matrix cores, forward and backward.
// Attention(Q, K, V) = Softmax(Q K^T / sqrt(d_k)) V (KARMA Sec. III-C "Self-Attention
// Layer"), one head at a time, with the S x S score matrix never leaving the chip: only
// the output and one log-sum-exp per query are saved for backward.
//
// Data layout: qkv [batch][seq][3*hidden] bf16 with q | k | v in thirds and head j in
// columns j*D..(j+1)*D of each third; ctx [batch][seq][hidden]; lse, delta [batch][head][seq]
// fp32.  lse is kept in the base-2 domain of the scaled scores: lse2 = log2 sum_j
// 2^(s_ij * scale * log2 e).
//
// All three kernels compute score tiles in the orientation that puts the softmax/row
// quantities on the lane (not across lanes): a 32x32 MFMA result holds column l%32 in lane
// l and 16 rows in its registers, so with queries on the columns every per-query reduction
// is a loop over registers plus one exchange between the two half-waves, and the
// probabilities can be fed back as the k-operand of the next MFMA straight from registers.
// Reductions over tiles run in a fixed order; there are no atomics (dQ has its own pass).
#include <hip/hip_runtime.h>

#include "karma.h"
#include "device_utils.h"
#include "kernels.h"

namespace karma {

constexpr float LOG2E = 1.4426950408889634f;

// v_exp_f32: 2^x without the range fix-ups of exp2f (arguments here are <= 0 or -inf)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

union Frag {
  bf16x8 v;
  u32x4 u;
  u32x2 h[2];
};

// k-operand fragment from two 8-byte pieces of an LDS row (keys/queries 4g..4g+3 and 8+4g..)
__device__ __forceinline__ bf16x8 frag2(const bf16_t* p) {
  Frag f;
  f.h[0] = *(const u32x2*)p;
  f.h[1] = *(const u32x2*)(p + 8);
  return f.v;
}
// k-operand fragment from eight accumulator registers
__device__ __forceinline__ bf16x8 frag_regs(const f32x16& a, int s, float mul) {
  Frag f;
#pragma unroll
  for (int e = 0; e < 4; ++e) f.u[e] = pack2(a[8 * s + 2 * e] * mul, a[8 * s + 2 * e + 1] * mul);
  return f.v;
}

// ------------------------------------------------------------------------------- forward
// grid (seq/128, heads, batch), 256 threads; wavefront w owns queries q0+32w .. q0+32w+31
// and walks the keys in tiles of 128 (four 32-key sub-tiles; sub-tiles entirely after the
// wavefront's queries are skipped).
// Workgroup -> (tile, head, batch).  Workgroup ids go round-robin over the 8 XCDs; all tiles
// of one (batch, head) are given to the same XCD, so that head's K and V are fetched into one
// L2 only, and the heaviest tile of the causal triangle goes first (heavy_high: the last
// tile is the heaviest).
__device__ __forceinline__ void attn_block(int& tile, int& head, int& b, bool heavy_high) {
  const int nt = gridDim.x, H = gridDim.y, hb_total = gridDim.y * gridDim.z;
  const int L = blockIdx.x + nt * (blockIdx.y + H * blockIdx.z);
  int t, hb;
  if (hb_total % 8 == 0) {
    const int slot = L / 8;
    hb = (slot / nt) * 8 + L % 8;
    t = slot % nt;
  } else {
    t = L % nt;
    hb = L / nt;
  }
  tile = heavy_high ? nt - 1 - t : t;
  head = hb % H;
  b = hb / H;
}

template <int D>
__global__ __launch_bounds__(256, (D == 64 ? 2 : 1)) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                        float* __restrict__ lse, int S, int H) {
  constexpr int KT = 128;   // keys per tile
  constexpr int PK = D + LDS_PAD, PV = KT + LDS_PAD;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[KT * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[D * PV];
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  int tile, head, b;
  attn_block(tile, head, b, true);
  const int q0 = tile * 128;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lrow = lane & 31, g = lane >> 5;
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * D;
  const bf16_t* Qg = base;
  const bf16_t* Kg = base + h;
  const bf16_t* Vg = base + 2 * h;
  const int qbase = q0 + 32 * w, query = qbase + lrow;
  const float c = LOG2E * rsqrtf((float)D);

  bf16x8 qf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    Frag f;
    f.u = *(const u32x4*)(Qg + (size_t)query * ld + ks * 16 + g * 8);
    qf[ks] = f.v;
  }
  f32x16 o[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;   // m: running maximum of the raw scores (before the 1/sqrt(d) scale)

  TileMover<KT, D, 256, true> mk;
  TileMover<D, KT, 256, false> mv;
  const int n_kt = (q0 + 128) / KT;
  mk.load(Kg, ld, 0, 0, S, D, tid, true);
  mv.load(Vg, ld, 0, 0, D, S, tid, true);
  for (int kt = 0; kt < n_kt; ++kt) {
    const int key0 = kt * KT;
    __syncthreads();   // previous tile fully consumed
    mk.store(Ks, tid);
    mv.store(Vt, tid);
    __syncthreads();
    if (kt + 1 < n_kt) {   // next tile's loads stay in flight while this one is computed
      mk.load(Kg, ld, key0 + KT, 0, S, D, tid, true);
      mv.load(Vg, ld, 0, key0 + KT, D, S, tid, true);
    }
    // sub-tiles this wavefront needs: keys key0 + 32*mt <= last query
    const int n_mt = min(4, (qbase + 31 - key0) / 32 + 1);
    f32x16 s[4];
    float tmax = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      if (mt < n_mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          bf16x8 kf = *(const bf16x8*)(Ks + (mt * 32 + lrow) * PK + ks * 16 + g * 8);
          s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[mt], 0, 0, 0);
        }
        if (key0 + mt * 32 + 31 > qbase) {   // sub-tile touches the diagonal: mask keys after the query
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + mt * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            if (key > query) s[mt][r] = -INFINITY;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[mt][r]);
      }
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m, tmax);
    const float mc = m_new * c;
    if (__any(m_new != m)) {   // rescale only when some query's maximum moved
      const float alpha = fast_exp2(m * c - mc);
      l *= alpha;
#pragma unroll
      for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
      m = m_new;
    }
    float psum = 0.f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      if (mt < n_mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = fast_exp2(fmaf(s[mt][r], c, -mc));
          s[mt][r] = p;
          psum += p;
        }
        // O^T += V^T P^T
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 pf = frag_regs(s[mt], st, 1.f);
#pragma unroll
          for (int i = 0; i < D / 32; ++i) {
            bf16x8 vf = frag2(Vt + (i * 32 + lrow) * PV + mt * 32 + st * 16 + g * 4);
            o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[i], 0, 0, 0);
          }
        }
      }
    }
    l += psum;
  }
  l += __shfl_xor(l, 32, 64);
  const float inv = 1.f / l;
  bf16_t* out = ctx + ((size_t)b * S + query) * h + (size_t)head * D;
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      u32x2 v;
      v.x = pack2(o[i][rg * 4 + 0] * inv, o[i][rg * 4 + 1] * inv);
      v.y = pack2(o[i][rg * 4 + 2] * inv, o[i][rg * 4 + 3] * inv);
      *(u32x2*)(out + i * 32 + rg * 8 + g * 4) = v;
    }
  if (g == 0) lse[((size_t)b * H + head) * S + query] = m * c + log2f(l);
}

// ------------------------------------------------------------------ backward: delta
// delta[b][head][q] = sum_d dO[b][q][head*D + d] * O[b][q][head*D + d]
template <int D>
__global__ void attn_delta_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                  float* __restrict__ delta, int S, int H, size_t total) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (b, q, head), head fastest
  if (i >= total) return;
  const int head = (int)(i % H);
  const size_t bq = i / H;
  const int q = (int)(bq % S);
  const size_t b = bq / S;
  const bf16_t* po = o + bq * (size_t)H * D + (size_t)head * D;
  const bf16_t* pd = dout + bq * (size_t)H * D + (size_t)head * D;
  float acc = 0.f;
#pragma unroll
  for (int v = 0; v < D / 8; ++v) {
    u32x4 a = *(const u32x4*)(po + v * 8), d = *(const u32x4*)(pd + v * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc = fmaf(__uint_as_float(a[e] << 16), __uint_as_float(d[e] << 16), acc);
      acc = fmaf(__uint_as_float(a[e] & 0xffff0000u), __uint_as_float(d[e] & 0xffff0000u), acc);
    }
  }
  delta[(b * H + head) * S + q] = acc;
}

// ------------------------------------------------------------------ backward: dQ
// Same tiling as forward: wavefront owns 32 queries, walks the keys in tiles of 128.
template <int D>
__global__ __launch_bounds__(256, (D == 64 ? 2 : 1)) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S, int H) {
  constexpr int KT = 128;
  constexpr int PK = D + LDS_PAD, PT = KT + LDS_PAD;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  bf16_t* Ks = (bf16_t*)smem_attn;   // [KT][PK]
  bf16_t* Vs = Ks + KT * PK;         // [KT][PK]
  bf16_t* Kt = Vs + KT * PK;         // [D][PT]   K transposed
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  int tile, head, b;
  attn_block(tile, head, b, true);
  const int q0 = tile * 128;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lrow = lane & 31, g = lane >> 5;
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * D;
  const bf16_t* Kg = base + h;
  const bf16_t* Vg = base + 2 * h;
  const int qbase = q0 + 32 * w, query = qbase + lrow;
  const float scale = rsqrtf((float)D), c = LOG2E * scale;

  bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    Frag f;
    f.u = *(const u32x4*)(base + (size_t)query * ld + ks * 16 + g * 8);
    qf[ks] = f.v;
    f.u = *(const u32x4*)(dout + ((size_t)b * S + query) * h + (size_t)head * D + ks * 16 + g * 8);
    dof[ks] = f.v;
  }
  const float my_lse = lse[((size_t)b * H + head) * S + query];
  const float my_delta = delta[((size_t)b * H + head) * S + query];
  f32x16 dq[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

  TileMover<KT, D, 256, true> mk, mv;
  TileMover<D, KT, 256, false> mkt;
  const int n_kt = (q0 + 128) / KT;
  mk.load(Kg, ld, 0, 0, S, D, tid, true);
  mv.load(Vg, ld, 0, 0, S, D, tid, true);
  mkt.load(Kg, ld, 0, 0, D, S, tid, true);
  for (int kt = 0; kt < n_kt; ++kt) {
    const int key0 = kt * KT;
    __syncthreads();
    mk.store(Ks, tid);
    mv.store(Vs, tid);
    mkt.store(Kt, tid);
    __syncthreads();
    if (kt + 1 < n_kt) {
      mk.load(Kg, ld, key0 + KT, 0, S, D, tid, true);
      mv.load(Vg, ld, key0 + KT, 0, S, D, tid, true);
      mkt.load(Kg, ld, 0, key0 + KT, D, S, tid, true);
    }
    const int n_mt = min(4, (qbase + 31 - key0) / 32 + 1);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      if (mt < n_mt) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          bf16x8 kf = *(const bf16x8*)(Ks + (mt * 32 + lrow) * PK + ks * 16 + g * 8);
          bf16x8 vf = *(const bf16x8*)(Vs + (mt * 32 + lrow) * PK + ks * 16 + g * 8);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[ks], dp, 0, 0, 0);
        }
        const bool diag = key0 + mt * 32 + 31 > qbase;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = fast_exp2(fmaf(s[r], c, -my_lse));
          if (diag) {
            const int key = key0 + mt * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            if (key > query) p = 0.f;
          }
          s[r] = p * (dp[r] - my_delta);   // dS^T (before the 1/sqrt(d) factor)
        }
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 dsf = frag_regs(s, st, scale);
#pragma unroll
          for (int i = 0; i < D / 32; ++i) {
            bf16x8 ktf = frag2(Kt + (i * 32 + lrow) * PT + mt * 32 + st * 16 + g * 4);
            dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf, dq[i], 0, 0, 0);
          }
        }
      }
    }
  }
  bf16_t* out = dqkv + ((size_t)b * S + query) * ld + (size_t)head * D;
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      u32x2 v;
      v.x = pack2(dq[i][rg * 4 + 0], dq[i][rg * 4 + 1]);
      v.y = pack2(dq[i][rg * 4 + 2], dq[i][rg * 4 + 3]);
      *(u32x2*)(out + i * 32 + rg * 8 + g * 4) = v;
    }
}

// ------------------------------------------------------------------ backward: dK, dV
// grid (seq/128, heads, batch); wavefront w owns keys k0+32w .. +31 and loops over the
// query tiles (64 queries, two 32-query sub-tiles) at or after them.  Scores are computed
// with queries on the rows so that the probabilities sit in registers as the (key x query)
// operand of dV = P^T dO and dK = dS^T Q.
template <int D>
__global__ __launch_bounds__(256, (D == 64 ? 2 : 1)) void attn_bwd_dkv_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S, int H) {
  constexpr int QT = 64;
  constexpr int TT = (D * QT / 32 < 256) ? D * QT / 32 : 256;   // threads of the transposing movers
  constexpr int PK = D + LDS_PAD, PT = QT + LDS_PAD;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  bf16_t* Qs = (bf16_t*)smem_attn;   // [QT][PK]
  bf16_t* Os = Qs + QT * PK;         // [QT][PK]   dO
  bf16_t* Qt = Os + QT * PK;         // [D][PT]    Q transposed
  bf16_t* Ot = Qt + D * PT;          // [D][PT]    dO transposed
  float* lse_s = (float*)(Ot + D * PT);
  float* delta_s = lse_s + QT;
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  int tile, head, b;
  attn_block(tile, head, b, false);
  const int k0 = tile * 128;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lrow = lane & 31, g = lane >> 5;
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * D;
  const bf16_t* dOg = dout + (size_t)b * S * h + (size_t)head * D;
  const int kbase = k0 + 32 * w, key = kbase + lrow;
  const float scale = rsqrtf((float)D), c = LOG2E * scale;

  bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    Frag f;
    f.u = *(const u32x4*)(base + h + (size_t)key * ld + ks * 16 + g * 8);
    kf[ks] = f.v;
    f.u = *(const u32x4*)(base + 2 * h + (size_t)key * ld + ks * 16 + g * 8);
    vf[ks] = f.v;
  }
  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[i][r] = 0.f; dv[i][r] = 0.f; }

  TileMover<QT, D, 256, true> mq, mo;
  TileMover<D, QT, TT, false> mqt, mot;
  auto fetch = [&](int qq) {
    mq.load(base, ld, qq, 0, S, D, tid, true);
    mo.load(dOg, (size_t)h, qq, 0, S, D, tid, true);
    if (tid < TT) {
      mqt.load(base, ld, 0, qq, D, S, tid, true);
      mot.load(dOg, (size_t)h, 0, qq, D, S, tid, true);
    }
  };
  fetch(k0);
  float lse_r = 0.f, delta_r = 0.f;
  if (tid < QT) {
    lse_r = lse[((size_t)b * H + head) * S + k0 + tid];
    delta_r = delta[((size_t)b * H + head) * S + k0 + tid];
  }
  for (int qq0 = k0; qq0 < S; qq0 += QT) {
    __syncthreads();
    mq.store(Qs, tid);
    mo.store(Os, tid);
    if (tid < TT) {
      mqt.store(Qt, tid);
      mot.store(Ot, tid);
    }
    if (tid < QT) {
      lse_s[tid] = lse_r;
      delta_s[tid] = delta_r;
    }
    __syncthreads();
    if (qq0 + QT < S) {
      fetch(qq0 + QT);
      if (tid < QT) {
        lse_r = lse[((size_t)b * H + head) * S + qq0 + QT + tid];
        delta_r = delta[((size_t)b * H + head) * S + qq0 + QT + tid];
      }
    }
    // sub-tiles of 32 queries; those entirely before this wavefront's keys contribute nothing
    const int first_mt = max(0, (kbase - qq0) / 32);
#pragma unroll
    for (int mt = 0; mt < QT / 32; ++mt) {
      if (mt >= first_mt) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          bf16x8 qfr = *(const bf16x8*)(Qs + (mt * 32 + lrow) * PK + ks * 16 + g * 8);
          bf16x8 ofr = *(const bf16x8*)(Os + (mt * 32 + lrow) * PK + ks * 16 + g * 8);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr, kf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ofr, vf[ks], dp, 0, 0, 0);
        }
        const bool diag = qq0 + mt * 32 < kbase + 31;
        // p in s, dS in dp (in place); the per-query statistics come four at a time
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int qb = mt * 32 + rg * 8 + g * 4;
          const float4 l4 = *(const float4*)(lse_s + qb);
          const float4 d4 = *(const float4*)(delta_s + qb);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = rg * 4 + e;
            float p = fast_exp2(fmaf(s[r], c, -lv[e]));
            if (diag && key > qq0 + qb + e) p = 0.f;
            s[r] = p;
            dp[r] = p * (dp[r] - dl[e]);
          }
        }
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 pf = frag_regs(s, st, 1.f);
          bf16x8 dsf = frag_regs(dp, st, scale);
#pragma unroll
          for (int i = 0; i < D / 32; ++i) {
            bf16x8 otf = frag2(Ot + (i * 32 + lrow) * PT + mt * 32 + st * 16 + g * 4);
            bf16x8 qtf = frag2(Qt + (i * 32 + lrow) * PT + mt * 32 + st * 16 + g * 4);
            dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf, otf, dv[i], 0, 0, 0);
            dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dsf, qtf, dk[i], 0, 0, 0);
          }
        }
      }
    }
  }
  // dk[i][r]: key = kbase + (r/4)*8 + 4g + r%4, d = i*32 + lane%32
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kk = kbase + (r >> 2) * 8 + g * 4 + (r & 3);
      bf16_t* row = dqkv + ((size_t)b * S + kk) * ld + (size_t)head * D + i * 32 + lrow;
      row[h] = f2bf(dk[i][r]);
      row[2 * h] = f2bf(dv[i][r]);
    }
}

template <int D>
constexpr size_t attn_dq_lds() { return (size_t)(2 * 128 * (D + LDS_PAD) + D * (128 + LDS_PAD)) * sizeof(bf16_t); }
template <int D>
constexpr size_t attn_dkv_lds() {
  return (size_t)(2 * 64 * (D + LDS_PAD) + 2 * D * (64 + LDS_PAD)) * sizeof(bf16_t) + 2 * 64 * sizeof(float);
}

// ------------------------------------------------------------------------------ launchers
static inline int ok() { return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP; }

int attention_fwd(const bf16_t* qkv, bf16_t* ctx, float* lse, int batch, int seq, int heads, int d, hipStream_t s) {
  if (seq % 128 || (d != 64 && d != 128) || batch <= 0 || heads <= 0) return KARMA_E_INVAL;
  dim3 grid(seq / 128, heads, batch);
  if (d == 64) hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(256), 0, s, qkv, ctx, lse, seq, heads);
  else hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(256), 0, s, qkv, ctx, lse, seq, heads);
  return ok();
}

template <int D>
static void launch_bwd(dim3 grid, hipStream_t s, const bf16_t* qkv, const bf16_t* dctx, const float* lse,
                       const float* delta, bf16_t* dqkv, int seq, int heads) {
  constexpr size_t l1 = attn_dq_lds<D>(), l2 = attn_dkv_lds<D>();
  if (l1 > 64 * 1024)
    (void)hipFuncSetAttribute((const void*)attn_bwd_dq_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l1);
  if (l2 > 64 * 1024)
    (void)hipFuncSetAttribute((const void*)attn_bwd_dkv_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l2);
  hipLaunchKernelGGL(attn_bwd_dq_kernel<D>, grid, dim3(256), l1, s, qkv, dctx, lse, delta, dqkv, seq, heads);
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<D>, grid, dim3(256), l2, s, qkv, dctx, lse, delta, dqkv, seq, heads);
}

int attention_bwd(const bf16_t* qkv, const bf16_t* ctx, const bf16_t* dctx, const float* lse, float* delta,
                  bf16_t* dqkv, int batch, int seq, int heads, int d, hipStream_t s) {
  if (seq % 128 || (d != 64 && d != 128) || batch <= 0 || heads <= 0) return KARMA_E_INVAL;
  dim3 grid(seq / 128, heads, batch);
  const size_t total = (size_t)batch * seq * heads;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (d == 64) {
    hipLaunchKernelGGL(attn_delta_kernel<64>, dim3(blocks), dim3(256), 0, s, ctx, dctx, delta, seq, heads, total);
    launch_bwd<64>(grid, s, qkv, dctx, lse, delta, dqkv, seq, heads);
  } else {
    hipLaunchKernelGGL(attn_delta_kernel<128>, dim3(blocks), dim3(256), 0, s, ctx, dctx, delta, seq, heads, total);
    launch_bwd<128>(grid, s, qkv, dctx, lse, delta, dqkv, seq, heads);
  }
  return ok();
}

}  // namespace karma

using namespace karma;

extern "C" int karma_k_attention_fwd_bf16(const void* qkv, void* ctx, float* lse, uint32_t batch, uint32_t seq,
                                          uint32_t heads, uint32_t d, void* stream) {
  if (!qkv || !ctx || !lse) return KARMA_E_INVAL;
  return attention_fwd((const bf16_t*)qkv, (bf16_t*)ctx, lse, (int)batch, (int)seq, (int)heads, (int)d,
                       (hipStream_t)stream);
}

extern "C" int karma_k_attention_bwd_bf16(const void* qkv, const void* ctx, const void* dctx, const float* lse,
                                          float* delta_ws, void* dqkv, uint32_t batch, uint32_t seq, uint32_t heads,
                                          uint32_t d, void* stream) {
  if (!qkv || !ctx || !dctx || !lse || !delta_ws || !dqkv) return KARMA_E_INVAL;
  return attention_bwd((const bf16_t*)qkv, (const bf16_t*)ctx, (const bf16_t*)dctx, lse, delta_ws, (bf16_t*)dqkv,
                       (int)batch, (int)seq, (int)heads, (int)d, (hipStream_t)stream);
}
