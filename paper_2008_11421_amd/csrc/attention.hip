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
// grid (seq/128, heads, batch), 256 threads; wavefront w owns queries q0+32w .. q0+32w+31.
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                        float* __restrict__ lse, int S, int H) {
  constexpr int PK = D + LDS_PAD, PV = 64 + LDS_PAD, TV = (D * 64 / 32 < 256) ? D * 64 / 32 : 256;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[64 * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[D * PV];
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  const int q0 = blockIdx.x * 128, head = blockIdx.y, b = blockIdx.z;
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
  float m = -INFINITY, l = 0.f;

  TileMover<64, D, 256, true> mk;
  TileMover<D, 64, TV, false> mv;
  const int n_kt = (q0 + 128) / 64;
  for (int kt = 0; kt < n_kt; ++kt) {
    const int key0 = kt * 64;
    mk.load(Kg, ld, key0, 0, S, D, tid);
    if (tid < TV) mv.load(Vg, ld, 0, key0, D, S, tid);
    __syncthreads();   // previous tile fully consumed
    mk.store(Ks, tid);
    if (tid < TV) mv.store(Vt, tid);
    __syncthreads();
    if (key0 <= qbase + 31) {
      f32x16 s[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          bf16x8 kf = *(const bf16x8*)(Ks + (mt * 32 + lrow) * PK + ks * 16 + g * 8);
          s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[mt], 0, 0, 0);
        }
      }
      // scale into the base-2 domain, mask keys after the query, tile maximum
      float tmax = -INFINITY;
      const bool diag = key0 + 63 > qbase;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = s[mt][r] * c;
          if (diag) {
            int key = key0 + mt * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            if (key > query) v = -INFINITY;
          }
          s[mt][r] = v;
          tmax = fmaxf(tmax, v);
        }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m, tmax);
      const float alpha = exp2f(m - m_new);
      m = m_new;
      float psum = 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = exp2f(s[mt][r] - m_new);
          s[mt][r] = p;
          psum += p;
        }
      l = l * alpha + psum;
#pragma unroll
      for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
      // O^T += V^T P^T
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
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
  if (g == 0) lse[((size_t)b * H + head) * S + query] = m + log2f(l);
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
// Same tiling as forward: wavefront owns 32 queries, loops over key tiles.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16_t* __restrict__ dqkv, int S, int H) {
  constexpr int PK = D + LDS_PAD, PT = 64 + LDS_PAD, TT = (D * 64 / 32 < 256) ? D * 64 / 32 : 256;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[64 * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[64 * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Kt[D * PT];
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  const int q0 = blockIdx.x * 128, head = blockIdx.y, b = blockIdx.z;
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

  TileMover<64, D, 256, true> mk, mv;
  TileMover<D, 64, TT, false> mkt;
  const int n_kt = (q0 + 128) / 64;
  for (int kt = 0; kt < n_kt; ++kt) {
    const int key0 = kt * 64;
    mk.load(Kg, ld, key0, 0, S, D, tid);
    mv.load(Vg, ld, key0, 0, S, D, tid);
    if (tid < TT) mkt.load(Kg, ld, 0, key0, D, S, tid);
    __syncthreads();
    mk.store(Ks, tid);
    mv.store(Vs, tid);
    if (tid < TT) mkt.store(Kt, tid);
    __syncthreads();
    if (key0 <= qbase + 31) {
      const bool diag = key0 + 63 > qbase;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
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
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = exp2f(s[r] * c - my_lse);
          if (diag) {
            int key = key0 + mt * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
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
// query tiles at or after them.  Scores are computed with queries on the rows so that the
// probabilities sit in registers as the (key x query) operand of dV = P^T dO and dK = dS^T Q.
template <int D>
__global__ __launch_bounds__(256, (D == 64 ? 2 : 1)) void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            bf16_t* __restrict__ dqkv, int S, int H) {
  constexpr int PK = D + LDS_PAD, PT = 64 + LDS_PAD, TT = (D * 64 / 32 < 256) ? D * 64 / 32 : 256;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[64 * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Os[64 * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Qt[D * PT];
  __shared__ __attribute__((aligned(16))) bf16_t Ot[D * PT];
  __shared__ __attribute__((aligned(16))) float lse_s[64], delta_s[64];
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  const int k0 = blockIdx.x * 128, head = blockIdx.y, b = blockIdx.z;
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

  TileMover<64, D, 256, true> mq, mo;
  TileMover<D, 64, TT, false> mqt, mot;
  for (int qt = k0 / 64; qt < S / 64; ++qt) {
    const int qq0 = qt * 64;
    mq.load(base, ld, qq0, 0, S, D, tid);
    mo.load(dOg, (size_t)h, qq0, 0, S, D, tid);
    if (tid < TT) {
      mqt.load(base, ld, 0, qq0, D, S, tid);
      mot.load(dOg, (size_t)h, 0, qq0, D, S, tid);
    }
    __syncthreads();
    mq.store(Qs, tid);
    mo.store(Os, tid);
    if (tid < TT) {
      mqt.store(Qt, tid);
      mot.store(Ot, tid);
    }
    if (tid < 64) {
      lse_s[tid] = lse[((size_t)b * H + head) * S + qq0 + tid];
      delta_s[tid] = delta[((size_t)b * H + head) * S + qq0 + tid];
    }
    __syncthreads();
    if (qq0 + 63 >= kbase) {
      const bool diag = qq0 < kbase + 31;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {   // 32 queries each
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
            float p = exp2f(s[r] * c - lv[e]);
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

// ------------------------------------------------------------------------------ launchers
static inline int ok() { return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP; }

int attention_fwd(const bf16_t* qkv, bf16_t* ctx, float* lse, int batch, int seq, int heads, int d, hipStream_t s) {
  if (seq % 128 || (d != 64 && d != 128) || batch <= 0 || heads <= 0) return KARMA_E_INVAL;
  dim3 grid(seq / 128, heads, batch);
  if (d == 64) hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(256), 0, s, qkv, ctx, lse, seq, heads);
  else hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(256), 0, s, qkv, ctx, lse, seq, heads);
  return ok();
}

int attention_bwd(const bf16_t* qkv, const bf16_t* ctx, const bf16_t* dctx, const float* lse, float* delta,
                  bf16_t* dqkv, int batch, int seq, int heads, int d, hipStream_t s) {
  if (seq % 128 || (d != 64 && d != 128) || batch <= 0 || heads <= 0) return KARMA_E_INVAL;
  dim3 grid(seq / 128, heads, batch);
  const size_t total = (size_t)batch * seq * heads;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (d == 64) {
    hipLaunchKernelGGL(attn_delta_kernel<64>, dim3(blocks), dim3(256), 0, s, ctx, dctx, delta, seq, heads, total);
    hipLaunchKernelGGL(attn_bwd_dq_kernel<64>, grid, dim3(256), 0, s, qkv, dctx, lse, delta, dqkv, seq, heads);
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<64>, grid, dim3(256), 0, s, qkv, dctx, lse, delta, dqkv, seq, heads);
  } else {
    hipLaunchKernelGGL(attn_delta_kernel<128>, dim3(blocks), dim3(256), 0, s, ctx, dctx, delta, seq, heads, total);
    hipLaunchKernelGGL(attn_bwd_dq_kernel<128>, grid, dim3(256), 0, s, qkv, dctx, lse, delta, dqkv, seq, heads);
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<128>, grid, dim3(256), 0, s, qkv, dctx, lse, delta, dqkv, seq, heads);
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
