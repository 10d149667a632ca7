// Kernels of the convolutional workload (KARMA Sec. III-C: convolution, batch
// normalisation, ReLU and pooling layers; the ResNet-200 row of Table III), NHWC bf16.
//
// Convolutions are implicit GEMMs on the matrix cores: the GEMM kernel gathers its A operand
// (forward, input gradient) or B operand (weight gradient) from the NHWC tensor, so no
// im2col buffer exists; 1x1 stride-1 convolutions are plain GEMMs.  Batch normalisation,
// ReLU masks and pooling are bandwidth-bound: 16-byte vectors along the channel axis, rows
// of pixels spread over the workgroup, per-channel sums reduced in a fixed order
// (workgroup partials, then a second kernel), so results are reproducible.
#include <hip/hip_runtime.h>

#include "karma.h"
#include "kernels.h"

namespace karma {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__device__ __forceinline__ bf16_t f2bf_(float f) {   // round to nearest even, NaN kept
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f_(bf16_t b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ void unpack8(const u32x4& v, float* f) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(v[i] << 16);
    f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ u32x4 pack8(const float* f) {
  u32x4 v;
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = (unsigned)f2bf_(f[2 * i]) | ((unsigned)f2bf_(f[2 * i + 1]) << 16);
  return v;
}
static inline int ok() { return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP; }
static inline unsigned blocks_for(size_t n, unsigned per) { return (unsigned)((n + per - 1) / per); }

constexpr float BN_EPS = 1e-5f;
// Rows of pixels per workgroup: eight per thread.  A workgroup is vc vector columns (8
// channels each, at most 256) times 256 / vc row lanes, so wide layers take short bands
// (enough workgroups even when only a few thousand pixels are left) and narrow ones long bands.
__host__ __device__ inline int bn_band(int C) {
  const int vc = C / 8 < 256 ? C / 8 : 256;
  const int band = 8 * (256 / vc);
  return band < 16 ? 16 : band;
}

// Rows per workgroup of the partial sums: the band above, or longer when that would make more than 2048 bands (a
// million pixels in 96-row bands are 11 000 partial rows, which the few workgroups of the finishing kernel then
// take longer to add up than the sums themselves took).
__host__ __device__ inline int bn_sum_band(int rows, int C) {
  const int b = bn_band(C), cap = (rows + 2047) / 2048;
  return b >= cap ? b : (cap + 7) / 8 * 8;
}

// Per-channel partial sums over a band of rows.  The 256 threads form vc vector columns (8
// channels each) times rl row lanes; a thread walks rows rl, rl + RL, ... of the band, the
// row lanes are then added in ascending order through LDS.
//   forward:  a0 = sum(x - pivot), a1 = sum((x - pivot)^2), pivot = the channel's value in row 0
//   backward: a0 = sum(dy'), a1 = sum(dy' * xhat), dy' = dy where the ReLU that follows let the
//             value through (mask recomputed from xhat*g + b), else 0
template <bool BWD>
__global__ __launch_bounds__(256) void bn_partial_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                          const float* __restrict__ stats, const bf16_t* __restrict__ g,
                                                          const bf16_t* __restrict__ b, float* __restrict__ partial,
                                                          int rows, int C, int relu) {
  __shared__ float red[2][256][8];
  const int nv = C / 8;
  const int VC = min(nv - (int)blockIdx.y * 256, 256), RL = 256 / VC;
  const int vc = threadIdx.x % VC, rl = threadIdx.x / VC;
  const int c8 = (blockIdx.y * 256 + vc) * 8;
  float a0[8], a1[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) a0[e] = a1[e] = 0.f;
  if (rl < RL) {
    float p0[8], p1[8], gg[8], bb[8];
    if (BWD) {
      unpack8(*(const u32x4*)(g + c8), gg);
      unpack8(*(const u32x4*)(b + c8), bb);
#pragma unroll
      for (int e = 0; e < 8; ++e) { p0[e] = stats[c8 + e]; p1[e] = stats[C + c8 + e]; }
    } else {
      unpack8(*(const u32x4*)(x + c8), p0);
    }
    const int band = bn_sum_band(rows, C);
    const int r0 = blockIdx.x * band, r1 = min(rows, r0 + band);
#pragma unroll 2
    for (int r = r0 + rl; r < r1; r += RL) {
      float v[8];
      unpack8(*(const u32x4*)(x + (size_t)r * C + c8), v);
      if (BWD) {
        float d[8];
        unpack8(*(const u32x4*)(dy + (size_t)r * C + c8), d);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (v[e] - p0[e]) * p1[e];
          const float dd = (relu && !(xh * gg[e] + bb[e] > 0.f)) ? 0.f : d[e];
          a0[e] += dd;
          a1[e] += dd * xh;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float t = v[e] - p0[e];
          a0[e] += t;
          a1[e] += t * t;
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { red[0][threadIdx.x][e] = a0[e]; red[1][threadIdx.x][e] = a1[e]; }
  __syncthreads();
  if (rl == 0) {
    for (int k = 1; k < RL; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) { a0[e] += red[0][k * VC + vc][e]; a1[e] += red[1][k * VC + vc][e]; }
    float* out = partial + (size_t)blockIdx.x * 2 * C;
#pragma unroll
    for (int e = 0; e < 8; ++e) { out[c8 + e] = a0[e]; out[C + c8 + e] = a1[e]; }
  }
}

// Adds the band partials in a fixed order: 32 interleaved slices of the bands per channel,
// then the slices in ascending order.
//   forward:  stats[0][c] = mean, stats[1][c] = 1/sqrt(var + eps) (biased variance)
//   backward: out0[c] = dbeta, out1[c] = dgamma
__global__ __launch_bounds__(256) void bn_finish_kernel(const float* __restrict__ partial, int bands, int C, int rows,
                                                         const bf16_t* __restrict__ x_row0, float* __restrict__ out0,
                                                         float* __restrict__ out1, int bwd) {
  __shared__ float red[2][32][8];
  const int cl = threadIdx.x & 7, slice = threadIdx.x >> 3;
  const int c = blockIdx.x * 8 + cl;
  float s0 = 0.f, s1 = 0.f;
  if (c < C) {
    int p = slice;
    for (; p + 96 < bands; p += 128) {   // four bands in flight, added in ascending order
      float a[4], b[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        a[k] = partial[(size_t)(p + 32 * k) * 2 * C + c];
        b[k] = partial[(size_t)(p + 32 * k) * 2 * C + C + c];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) { s0 += a[k]; s1 += b[k]; }
    }
    for (; p < bands; p += 32) {
      s0 += partial[(size_t)p * 2 * C + c];
      s1 += partial[(size_t)p * 2 * C + C + c];
    }
  }
  red[0][slice][cl] = s0;
  red[1][slice][cl] = s1;
  __syncthreads();
  if (slice == 0 && c < C) {
    float t0 = red[0][0][cl], t1 = red[1][0][cl];
#pragma unroll
    for (int k = 1; k < 32; ++k) { t0 += red[0][k][cl]; t1 += red[1][k][cl]; }
    if (bwd) {
      out0[c] = t0;
      out1[c] = t1;
    } else {
      const float inv = 1.f / (float)rows;
      const float m = t0 * inv;                       // mean of (x - pivot)
      const float var = fmaxf(t1 * inv - m * m, 0.f);
      out0[c] = bf2f_(x_row0[c]) + m;
      out1[c] = 1.f / sqrtf(var + BN_EPS);
    }
  }
}

// y = (x - mean) * rstd * g + b (+ add) (ReLU).  Same thread layout as the partial sums: a
// thread keeps its eight channels' scale and shift in registers and walks the rows of a band.
// gate (may be null): instead of the value itself, gate's element is written where the value as stored (bf16)
// is positive and zero elsewhere: the gradient through the ReLU, without a pass of its own.
__global__ __launch_bounds__(256) void bn_apply_fwd_kernel(const bf16_t* __restrict__ x, const float* __restrict__ stats,
                                                            const bf16_t* __restrict__ g, const bf16_t* __restrict__ b,
                                                            const bf16_t* __restrict__ add, const bf16_t* __restrict__ gate,
                                                            bf16_t* __restrict__ y, int rows, int C, int relu) {
  const int nv = C / 8;
  const int VC = min(nv - (int)blockIdx.y * 256, 256), RL = 256 / VC;
  const int vc = threadIdx.x % VC, rl = threadIdx.x / VC;
  if (rl >= RL) return;
  const int c8 = (blockIdx.y * 256 + vc) * 8;
  float gg[8], bb[8], mean[8], rstd[8];
  unpack8(*(const u32x4*)(g + c8), gg);
  unpack8(*(const u32x4*)(b + c8), bb);
#pragma unroll
  for (int e = 0; e < 8; ++e) { mean[e] = stats[c8 + e]; rstd[e] = stats[C + c8 + e]; }
  const int band = bn_band(C);
  const int r0 = blockIdx.x * band, r1 = min(rows, r0 + band);
  for (int r = r0 + rl; r < r1; r += RL) {
    const size_t at = (size_t)r * C + c8;
    float v[8], a[8];
    unpack8(*(const u32x4*)(x + at), v);
    if (add) unpack8(*(const u32x4*)(add + at), a);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // kept as (x - mean) * rstd * g + b: the backward pass recomputes exactly this expression
      float t = (v[e] - mean[e]) * rstd[e] * gg[e] + bb[e];
      if (add) t += a[e];
      v[e] = relu ? fmaxf(t, 0.f) : t;
    }
    u32x4 out = pack8(v);
    if (gate) {
      const u32x4 gv = *(const u32x4*)(gate + at);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const unsigned w = out[k];
        const unsigned keep = ((w & 0x7fffu) && !(w & 0x8000u) ? 0xffffu : 0u) | ((w & 0x7fff0000u) && !(w & 0x80000000u) ? 0xffff0000u : 0u);
        out[k] = gv[k] & keep;
      }
    }
    *(u32x4*)(y + at) = out;
  }
}

// dx = g * rstd * (dy' - dbeta/M - xhat * dgamma/M) (+ add)
__global__ __launch_bounds__(256) void bn_apply_bwd_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                            const float* __restrict__ stats, const bf16_t* __restrict__ g,
                                                            const bf16_t* __restrict__ b, const float* __restrict__ dgamma,
                                                            const float* __restrict__ dbeta, const bf16_t* __restrict__ add,
                                                            bf16_t* __restrict__ dx, int rows, int C, float inv_rows, int relu) {
  const int nv = C / 8;
  const int VC = min(nv - (int)blockIdx.y * 256, 256), RL = 256 / VC;
  const int vc = threadIdx.x % VC, rl = threadIdx.x / VC;
  if (rl >= RL) return;
  const int c8 = (blockIdx.y * 256 + vc) * 8;
  float gg[8], bb[8], mean[8], rstd[8], k0[8], k1[8];
  unpack8(*(const u32x4*)(g + c8), gg);
  unpack8(*(const u32x4*)(b + c8), bb);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    mean[e] = stats[c8 + e];
    rstd[e] = stats[C + c8 + e];
    k0[e] = dbeta[c8 + e] * inv_rows;
    k1[e] = dgamma[c8 + e] * inv_rows;
  }
  const int band = bn_band(C);
  const int r0 = blockIdx.x * band, r1 = min(rows, r0 + band);
  for (int r = r0 + rl; r < r1; r += RL) {
    const size_t at = (size_t)r * C + c8;
    float v[8], d[8];
    unpack8(*(const u32x4*)(x + at), v);
    unpack8(*(const u32x4*)(dy + at), d);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float xh = (v[e] - mean[e]) * rstd[e];
      const float dd = (relu && !(xh * gg[e] + bb[e] > 0.f)) ? 0.f : d[e];
      v[e] = gg[e] * rstd[e] * (dd - k0[e] - xh * k1[e]);
    }
    if (add) {
      float a[8];
      unpack8(*(const u32x4*)(add + at), a);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += a[e];
    }
    *(u32x4*)(dx + at) = pack8(v);
  }
}

// dz = dy where y > 0, else 0 (gradient through the ReLU that produced y)
__global__ void relu_mask_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ y, bf16_t* __restrict__ dz,
                                 size_t nvec) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  u32x4 d = ((const u32x4*)dy)[i], m = ((const u32x4*)y)[i], o;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    // a bf16 is positive iff its sign bit is clear and it is not zero
    const unsigned lo = m[k] & 0xffffu, hi = m[k] >> 16;
    const unsigned keep_lo = (lo & 0x7fffu) && !(lo & 0x8000u) ? 0xffffu : 0u;
    const unsigned keep_hi = (hi & 0x7fffu) && !(hi & 0x8000u) ? 0xffff0000u : 0u;
    o[k] = d[k] & (keep_lo | keep_hi);
  }
  ((u32x4*)dz)[i] = o;
}

// 3x3 max pooling, stride 2, padding 1 (padding never wins)
__global__ void maxpool_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, int N, int H, int W, int C,
                                   int Ho, int Wo) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nv = C / 8;
  if (i >= (size_t)N * Ho * Wo * nv) return;
  const int c8 = (int)(i % nv) * 8;
  size_t p = i / nv;
  const int wo = (int)(p % Wo); p /= Wo;
  const int ho = (int)(p % Ho);
  const int n = (int)(p / Ho);
  float best[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
  for (int r = 0; r < 3; ++r)
    for (int s = 0; s < 3; ++s) {
      const int hi = 2 * ho - 1 + r, wi = 2 * wo - 1 + s;
      if ((unsigned)hi >= (unsigned)H || (unsigned)wi >= (unsigned)W) continue;
      float v[8];
      unpack8(*(const u32x4*)(x + (((size_t)n * H + hi) * W + wi) * C + c8), v);
#pragma unroll
      for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], v[e]);
    }
  ((u32x4*)y)[i] = pack8(best);
}

// Gradient of the pooling in gather form: an input element collects dy from every window
// whose first maximum (row-major window order) it is.  No atomics.
__global__ void maxpool_bwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                   int N, int H, int W, int C, int Ho, int Wo) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nv = C / 8;
  if (i >= (size_t)N * H * W * nv) return;
  const int c8 = (int)(i % nv) * 8;
  size_t p = i / nv;
  const int w = (int)(p % W); p /= W;
  const int h = (int)(p % H);
  const int n = (int)(p / H);
  float mine[8], acc[8];
  unpack8(((const u32x4*)x)[i], mine);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int ho = max(0, h / 2); ho <= min(Ho - 1, (h + 1) / 2); ++ho)
    for (int wo = max(0, w / 2); wo <= min(Wo - 1, (w + 1) / 2); ++wo) {
      // my position inside this window, and whether an earlier or a larger element beats me
      const int mr = h - (2 * ho - 1), ms = w - (2 * wo - 1);
      if (mr < 0 || mr > 2 || ms < 0 || ms > 2) continue;
      bool win[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) win[e] = true;
      for (int r = 0; r < 3; ++r)
        for (int s = 0; s < 3; ++s) {
          const int hi = 2 * ho - 1 + r, wi = 2 * wo - 1 + s;
          if ((r == mr && s == ms) || (unsigned)hi >= (unsigned)H || (unsigned)wi >= (unsigned)W) continue;
          float v[8];
          unpack8(*(const u32x4*)(x + (((size_t)n * H + hi) * W + wi) * C + c8), v);
          const bool earlier = r * 3 + s < mr * 3 + ms;
#pragma unroll
          for (int e = 0; e < 8; ++e) win[e] = win[e] && (earlier ? v[e] < mine[e] : v[e] <= mine[e]);
        }
      float d[8];
      unpack8(*(const u32x4*)(dy + (((size_t)n * Ho + ho) * Wo + wo) * C + c8), d);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += win[e] ? d[e] : 0.f;
    }
  ((u32x4*)dx)[i] = pack8(acc);
}

// 2x2 max pooling, stride 2 (H and W even): one thread per output pixel and eight channels
__global__ void maxpool2_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, int N, int H, int W, int C) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nv = C / 8, Ho = H / 2, Wo = W / 2;
  if (i >= (size_t)N * Ho * Wo * nv) return;
  const int c8 = (int)(i % nv) * 8;
  size_t p = i / nv;
  const int wo = (int)(p % Wo); p /= Wo;
  const int ho = (int)(p % Ho);
  const int n = (int)(p / Ho);
  const bf16_t* at = x + (((size_t)n * H + 2 * ho) * W + 2 * wo) * C + c8;
  float best[8], v[8];
  unpack8(*(const u32x4*)at, best);
  unpack8(*(const u32x4*)(at + C), v);
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], v[e]);
  unpack8(*(const u32x4*)(at + (size_t)W * C), v);
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], v[e]);
  unpack8(*(const u32x4*)(at + (size_t)W * C + C), v);
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], v[e]);
  ((u32x4*)y)[i] = pack8(best);
}

// Its gradient: the windows are disjoint, so the thread of an output pixel writes all four input
// positions: dy to the first maximum in row-major window order, zero to the others.
__global__ void maxpool2_bwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                    int N, int H, int W, int C) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nv = C / 8, Ho = H / 2, Wo = W / 2;
  if (i >= (size_t)N * Ho * Wo * nv) return;
  const int c8 = (int)(i % nv) * 8;
  size_t p = i / nv;
  const int wo = (int)(p % Wo); p /= Wo;
  const int ho = (int)(p % Ho);
  const int n = (int)(p / Ho);
  const size_t base = (((size_t)n * H + 2 * ho) * W + 2 * wo) * C + c8;
  const size_t pos[4] = {base, base + C, base + (size_t)W * C, base + (size_t)W * C + C};
  float v[4][8], d[8];
#pragma unroll
  for (int k = 0; k < 4; ++k) unpack8(*(const u32x4*)(x + pos[k]), v[k]);
  unpack8(((const u32x4*)dy)[i], d);
  int first[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    first[e] = 0;
    float best = v[0][e];
#pragma unroll
    for (int k = 1; k < 4; ++k)
      if (v[k][e] > best) { best = v[k][e]; first[e] = k; }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = first[e] == k ? d[e] : 0.f;
    *(u32x4*)(dx + pos[k]) = pack8(o);
  }
}

// y += a, eight elements per thread (a gradient that arrived by another path)
__global__ void add_inplace_kernel(bf16_t* __restrict__ y, const bf16_t* __restrict__ a, size_t nvec) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float u[8], v[8];
  unpack8(((const u32x4*)y)[i], u);
  unpack8(((const u32x4*)a)[i], v);
#pragma unroll
  for (int e = 0; e < 8; ++e) u[e] += v[e];
  ((u32x4*)y)[i] = pack8(u);
}

// global average pooling: y[n][c] = mean over the HW positions, summed in position order
__global__ void avgpool_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, int N, int HW, int C) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nv = C / 8;
  if (i >= (size_t)N * nv) return;
  const int c8 = (int)(i % nv) * 8, n = (int)(i / nv);
  float a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int p = 0; p < HW; ++p) {
    float v[8];
    unpack8(*(const u32x4*)(x + ((size_t)n * HW + p) * C + c8), v);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] *= 1.f / (float)HW;
  ((u32x4*)y)[i] = pack8(a);
}

__global__ void avgpool_bwd_kernel(const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx, int N, int HW, int C) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nv = C / 8;
  if (i >= (size_t)N * HW * nv) return;
  const int c8 = (int)(i % nv) * 8, n = (int)(i / ((size_t)HW * nv));
  float d[8];
  unpack8(*(const u32x4*)(dy + (size_t)n * C + c8), d);
#pragma unroll
  for (int e = 0; e < 8; ++e) d[e] *= 1.f / (float)HW;
  ((u32x4*)dx)[i] = pack8(d);
}

// wt[ci][tap][co] = w[co][tap][ci]: the input-gradient pass reads the weights with the output
// channel as the contiguous reduction index
__global__ void conv_weight_transpose_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt, int Cout, int taps,
                                             int Cin) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)Cout * taps * Cin) return;
  const int co = (int)(i % Cout);
  const int t = (int)((i / Cout) % taps);
  const int ci = (int)(i / ((size_t)Cout * taps));
  wt[i] = w[((size_t)co * taps + t) * Cin + ci];
}

bool plain_gemm(const ConvShape& c) { return c.R == 1 && c.S == 1 && c.stride == 1 && c.pad == 0; }
bool shape_ok(const ConvShape& c) {
  return c.N > 0 && c.H > 0 && c.W > 0 && c.Cin > 0 && c.Cout > 0 && c.R > 0 && c.S > 0 && c.stride > 0 && c.pad >= 0 &&
         c.Cin % 8 == 0 && c.Cout % 8 == 0 && c.H + 2 * c.pad >= c.R && c.W + 2 * c.pad >= c.S &&
         (size_t)c.N * c.H * c.W < (1u << 30);
}

}  // namespace

int conv_out_dim(int n, int k, int stride, int pad) { return (n + 2 * pad - k) / stride + 1; }

int conv2d_fwd(const bf16_t* x, const bf16_t* w, bf16_t* y, const ConvShape& c, hipStream_t s, void* ws, size_t ws_bytes,
               const bf16_t* add) {
  if (!x || !w || !y || !shape_ok(c)) return KARMA_E_INVAL;
  const int Ho = conv_out_dim(c.H, c.R, c.stride, c.pad), Wo = conv_out_dim(c.W, c.S, c.stride, c.pad);
  GemmArgs g{};
  g.A = x; g.B = w; g.C = y; g.residual = add;
  g.M = c.N * Ho * Wo; g.N = c.Cout; g.K = c.R * c.S * c.Cin;
  g.a_kc = g.b_kc = true;
  g.lda = g.K; g.ldb = g.K; g.ldc = g.N;
  g.ws = ws; g.ws_bytes = ws_bytes;   // late stages: few output tiles, long reductions
  if (!plain_gemm(c)) {
    g.conv_mode = 1;
    g.conv = ConvGather{c.H, c.W, c.Cin, Ho, Wo, c.R, c.S, c.stride, c.pad, 0};
  }
  return gemm_bf16(g, s);
}

size_t conv2d_dgrad_ws_elems(const ConvShape& c) { return plain_gemm(c) ? 0 : (size_t)c.R * c.S * c.Cin * c.Cout; }

int conv2d_dgrad(const bf16_t* dy, const bf16_t* w, bf16_t* wt_ws, const bf16_t* add, bf16_t* dx, const ConvShape& c,
                 hipStream_t s, void* ws, size_t ws_bytes) {
  if (!dy || !w || !dx || !shape_ok(c)) return KARMA_E_INVAL;
  const int Ho = conv_out_dim(c.H, c.R, c.stride, c.pad), Wo = conv_out_dim(c.W, c.S, c.stride, c.pad);
  GemmArgs g{};
  g.A = dy; g.C = dx; g.residual = add;
  g.M = c.N * c.H * c.W; g.N = c.Cin; g.ldc = g.N;
  g.ws = ws; g.ws_bytes = ws_bytes;
  if (plain_gemm(c)) {
    g.B = w;            // B(n = ci, k = co) = w[co][ci]: strided
    g.K = c.Cout;
    g.a_kc = true; g.b_kc = false;
    g.lda = g.K; g.ldb = c.Cin;
    return gemm_bf16(g, s);
  }
  if (!wt_ws) return KARMA_E_INVAL;
  const size_t n = (size_t)c.R * c.S * c.Cin * c.Cout;
  hipLaunchKernelGGL(conv_weight_transpose_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, w, wt_ws, c.Cout, c.R * c.S,
                     c.Cin);
  g.B = wt_ws;          // [Cin][R*S*Cout], reduction index contiguous
  g.K = c.R * c.S * c.Cout;
  g.a_kc = g.b_kc = true;
  g.lda = g.K; g.ldb = g.K;
  g.conv_mode = 1;
  // rows are the pixels of x (H x W grid); the gathered tensor is dy (Ho x Wo x Cout)
  g.conv = ConvGather{Ho, Wo, c.Cout, c.H, c.W, c.R, c.S, c.stride, c.pad, 1};
  return gemm_bf16(g, s);
}

int conv2d_wgrad(const bf16_t* dy, const bf16_t* x, bf16_t* dw, void* ws, size_t ws_bytes, const ConvShape& c,
                 hipStream_t s) {
  if (!dy || !x || !dw || !shape_ok(c)) return KARMA_E_INVAL;
  const int Ho = conv_out_dim(c.H, c.R, c.stride, c.pad), Wo = conv_out_dim(c.W, c.S, c.stride, c.pad);
  GemmArgs g{};
  g.A = dy;             // A(m = co, k = pixel) = dy[pixel][co]: strided
  g.B = x;
  g.C = dw;
  g.M = c.Cout; g.N = c.R * c.S * c.Cin; g.K = c.N * Ho * Wo;
  g.a_kc = g.b_kc = false;
  g.lda = c.Cout; g.ldb = c.Cin; g.ldc = g.N;
  g.ws = ws; g.ws_bytes = ws_bytes;
  if (!plain_gemm(c)) {
    g.conv_mode = 2;
    g.conv = ConvGather{c.H, c.W, c.Cin, Ho, Wo, c.R, c.S, c.stride, c.pad, 0};
  }
  return gemm_bf16(g, s);
}

size_t bn_ws_bytes(int rows, int c) {
  const int band = bn_sum_band(rows, c > 8 ? c : 8);
  return (size_t)((rows + band - 1) / band) * 2 * c * sizeof(float);
}

int bn_fwd(const bf16_t* x, const bf16_t* g, const bf16_t* b, const bf16_t* add, bf16_t* y, float* stats, float* ws,
           int rows, int c, int relu, hipStream_t s) {
  if (!x || !g || !b || !y || !stats || !ws || rows <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  const int bands = (rows + bn_sum_band(rows, c) - 1) / bn_sum_band(rows, c);
  hipLaunchKernelGGL(bn_partial_kernel<false>, dim3(bands, (c / 8 + 255) / 256), dim3(256), 0, s, x, (const bf16_t*)nullptr,
                     (const float*)nullptr, g, b, ws, rows, c, 0);
  hipLaunchKernelGGL(bn_finish_kernel, dim3((c + 7) / 8), dim3(256), 0, s, ws, bands, c, rows, x, stats, stats + c, 0);
  hipLaunchKernelGGL(bn_apply_fwd_kernel, dim3((rows + bn_band(c) - 1) / bn_band(c), (c / 8 + 255) / 256), dim3(256), 0, s, x, stats,
                     g, b, add, (const bf16_t*)nullptr, y, rows, c, relu);
  return ok();
}

int bn_apply(const bf16_t* x, const float* stats, const bf16_t* g, const bf16_t* b, const bf16_t* add, bf16_t* y, int rows,
             int c, int relu, hipStream_t s, const bf16_t* gate) {
  if (!x || !stats || !g || !b || !y || rows <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(bn_apply_fwd_kernel, dim3((rows + bn_band(c) - 1) / bn_band(c), (c / 8 + 255) / 256), dim3(256), 0, s, x, stats,
                     g, b, add, gate, y, rows, c, relu);
  return ok();
}

int bn_bwd(const bf16_t* dy, const bf16_t* x, const float* stats, const bf16_t* g, const bf16_t* b, int relu, bf16_t* dx,
           float* dgamma, float* dbeta, float* ws, int rows, int c, hipStream_t s, const bf16_t* add) {
  if (!dy || !x || !stats || !g || !b || !dx || !dgamma || !dbeta || !ws || rows <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  const int bands = (rows + bn_sum_band(rows, c) - 1) / bn_sum_band(rows, c);
  hipLaunchKernelGGL(bn_partial_kernel<true>, dim3(bands, (c / 8 + 255) / 256), dim3(256), 0, s, x, dy, stats, g, b, ws, rows,
                     c, relu);
  hipLaunchKernelGGL(bn_finish_kernel, dim3((c + 7) / 8), dim3(256), 0, s, ws, bands, c, rows, (const bf16_t*)nullptr, dbeta,
                     dgamma, 1);
  hipLaunchKernelGGL(bn_apply_bwd_kernel, dim3((rows + bn_band(c) - 1) / bn_band(c), (c / 8 + 255) / 256), dim3(256), 0, s, dy, x, stats, g, b, dgamma, dbeta,
                     add, dx, rows, c, 1.f / (float)rows, relu);
  return ok();
}

int relu_mask_bwd(const bf16_t* dy, const bf16_t* y, bf16_t* dz, size_t n, hipStream_t s) {
  if (!dy || !y || !dz || n % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(relu_mask_kernel, dim3(blocks_for(n / 8, 256)), dim3(256), 0, s, dy, y, dz, n / 8);
  return ok();
}

int maxpool_fwd(const bf16_t* x, bf16_t* y, int n, int h, int w, int c, hipStream_t s) {
  if (!x || !y || n <= 0 || h <= 0 || w <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  const int ho = conv_out_dim(h, 3, 2, 1), wo = conv_out_dim(w, 3, 2, 1);
  hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(blocks_for((size_t)n * ho * wo * (c / 8), 256)), dim3(256), 0, s, x, y, n, h, w,
                     c, ho, wo);
  return ok();
}

int maxpool_bwd(const bf16_t* x, const bf16_t* dy, bf16_t* dx, int n, int h, int w, int c, hipStream_t s) {
  if (!x || !dy || !dx || n <= 0 || h <= 0 || w <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  const int ho = conv_out_dim(h, 3, 2, 1), wo = conv_out_dim(w, 3, 2, 1);
  hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(blocks_for((size_t)n * h * w * (c / 8), 256)), dim3(256), 0, s, x, dy, dx, n, h,
                     w, c, ho, wo);
  return ok();
}

int maxpool2_fwd(const bf16_t* x, bf16_t* y, int n, int h, int w, int c, hipStream_t s) {
  if (!x || !y || n <= 0 || h <= 0 || w <= 0 || c <= 0 || c % 8 || h % 2 || w % 2) return KARMA_E_INVAL;
  hipLaunchKernelGGL(maxpool2_fwd_kernel, dim3(blocks_for((size_t)n * (h / 2) * (w / 2) * (c / 8), 256)), dim3(256), 0, s, x, y,
                     n, h, w, c);
  return ok();
}

int maxpool2_bwd(const bf16_t* x, const bf16_t* dy, bf16_t* dx, int n, int h, int w, int c, hipStream_t s) {
  if (!x || !dy || !dx || n <= 0 || h <= 0 || w <= 0 || c <= 0 || c % 8 || h % 2 || w % 2) return KARMA_E_INVAL;
  hipLaunchKernelGGL(maxpool2_bwd_kernel, dim3(blocks_for((size_t)n * (h / 2) * (w / 2) * (c / 8), 256)), dim3(256), 0, s, x, dy,
                     dx, n, h, w, c);
  return ok();
}

int add_inplace_bf16(bf16_t* y, const bf16_t* a, size_t n, hipStream_t s) {
  if (!y || !a || n % 8) return KARMA_E_INVAL;
  if (!n) return KARMA_OK;
  hipLaunchKernelGGL(add_inplace_kernel, dim3(blocks_for(n / 8, 256)), dim3(256), 0, s, y, a, n / 8);
  return ok();
}

int avgpool_fwd(const bf16_t* x, bf16_t* y, int n, int hw, int c, hipStream_t s) {
  if (!x || !y || n <= 0 || hw <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(blocks_for((size_t)n * (c / 8), 256)), dim3(256), 0, s, x, y, n, hw, c);
  return ok();
}

int avgpool_bwd(const bf16_t* dy, bf16_t* dx, int n, int hw, int c, hipStream_t s) {
  if (!dy || !dx || n <= 0 || hw <= 0 || c <= 0 || c % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(blocks_for((size_t)n * hw * (c / 8), 256)), dim3(256), 0, s, dy, dx, n, hw, c);
  return ok();
}

}  // namespace karma

using namespace karma;

static ConvShape shape_of(const karma_conv_shape* c) {
  return ConvShape{(int)c->n, (int)c->h, (int)c->w, (int)c->c_in, (int)c->c_out, (int)c->r, (int)c->s, (int)c->stride,
                   (int)c->pad};
}

extern "C" int karma_k_conv2d_fwd_bf16(const void* x, const void* w, void* y, const karma_conv_shape* c, void* stream) {
  if (!c) return KARMA_E_INVAL;
  return conv2d_fwd((const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, shape_of(c), (hipStream_t)stream, nullptr, 0);
}

extern "C" int karma_k_conv2d_fwd_add_bf16(const void* x, const void* w, const void* add, void* y, const karma_conv_shape* c,
                                           void* stream) {
  if (!c) return KARMA_E_INVAL;
  return conv2d_fwd((const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, shape_of(c), (hipStream_t)stream, nullptr, 0,
                    (const bf16_t*)add);
}

extern "C" int karma_k_conv2d_dgrad_bf16(const void* dy, const void* w, void* wt_ws, const void* add, void* dx,
                                         const karma_conv_shape* c, void* stream) {
  if (!c) return KARMA_E_INVAL;
  return conv2d_dgrad((const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)wt_ws, (const bf16_t*)add, (bf16_t*)dx, shape_of(c),
                      (hipStream_t)stream, nullptr, 0);
}

extern "C" int karma_k_conv2d_wgrad_bf16(const void* dy, const void* x, void* dw, void* ws, uint64_t ws_bytes,
                                         const karma_conv_shape* c, void* stream) {
  if (!c) return KARMA_E_INVAL;
  return conv2d_wgrad((const bf16_t*)dy, (const bf16_t*)x, (bf16_t*)dw, ws, (size_t)ws_bytes, shape_of(c), (hipStream_t)stream);
}

extern "C" uint64_t karma_k_batchnorm_ws_bytes(uint32_t rows, uint32_t c) { return (uint64_t)bn_ws_bytes((int)rows, (int)c); }

extern "C" int karma_k_batchnorm_fwd_bf16(const void* x, const void* gamma, const void* beta, const void* add, void* y,
                                          void* stats, void* ws, uint32_t rows, uint32_t c, uint32_t relu, void* stream) {
  return bn_fwd((const bf16_t*)x, (const bf16_t*)gamma, (const bf16_t*)beta, (const bf16_t*)add, (bf16_t*)y, (float*)stats,
                (float*)ws, (int)rows, (int)c, (int)relu, (hipStream_t)stream);
}

extern "C" int karma_k_batchnorm_bwd_bf16(const void* dy, const void* x, const void* stats, const void* gamma,
                                          const void* beta, uint32_t relu, void* dx, void* dgamma, void* dbeta, void* ws,
                                          uint32_t rows, uint32_t c, void* stream) {
  return bn_bwd((const bf16_t*)dy, (const bf16_t*)x, (const float*)stats, (const bf16_t*)gamma, (const bf16_t*)beta, (int)relu,
                (bf16_t*)dx, (float*)dgamma, (float*)dbeta, (float*)ws, (int)rows, (int)c, (hipStream_t)stream);
}

extern "C" int karma_k_batchnorm_bwd_add_bf16(const void* dy, const void* x, const void* stats, const void* gamma,
                                              const void* beta, uint32_t relu, const void* add, void* dx, void* dgamma,
                                              void* dbeta, void* ws, uint32_t rows, uint32_t c, void* stream) {
  return bn_bwd((const bf16_t*)dy, (const bf16_t*)x, (const float*)stats, (const bf16_t*)gamma, (const bf16_t*)beta, (int)relu,
                (bf16_t*)dx, (float*)dgamma, (float*)dbeta, (float*)ws, (int)rows, (int)c, (hipStream_t)stream,
                (const bf16_t*)add);
}

extern "C" int karma_k_relu_mask_bwd_bf16(const void* dy, const void* y, void* dz, uint64_t n, void* stream) {
  return relu_mask_bwd((const bf16_t*)dy, (const bf16_t*)y, (bf16_t*)dz, (size_t)n, (hipStream_t)stream);
}

extern "C" int karma_k_maxpool_fwd_bf16(const void* x, void* y, uint32_t n, uint32_t h, uint32_t w, uint32_t c, void* stream) {
  return maxpool_fwd((const bf16_t*)x, (bf16_t*)y, (int)n, (int)h, (int)w, (int)c, (hipStream_t)stream);
}

extern "C" int karma_k_maxpool_bwd_bf16(const void* x, const void* dy, void* dx, uint32_t n, uint32_t h, uint32_t w,
                                        uint32_t c, void* stream) {
  return maxpool_bwd((const bf16_t*)x, (const bf16_t*)dy, (bf16_t*)dx, (int)n, (int)h, (int)w, (int)c, (hipStream_t)stream);
}

extern "C" int karma_k_maxpool2_fwd_bf16(const void* x, void* y, uint32_t n, uint32_t h, uint32_t w, uint32_t c, void* stream) {
  return maxpool2_fwd((const bf16_t*)x, (bf16_t*)y, (int)n, (int)h, (int)w, (int)c, (hipStream_t)stream);
}

extern "C" int karma_k_maxpool2_bwd_bf16(const void* x, const void* dy, void* dx, uint32_t n, uint32_t h, uint32_t w,
                                         uint32_t c, void* stream) {
  return maxpool2_bwd((const bf16_t*)x, (const bf16_t*)dy, (bf16_t*)dx, (int)n, (int)h, (int)w, (int)c, (hipStream_t)stream);
}

extern "C" int karma_k_add_inplace_bf16(void* y, const void* a, uint64_t n, void* stream) {
  return add_inplace_bf16((bf16_t*)y, (const bf16_t*)a, (size_t)n, (hipStream_t)stream);
}

extern "C" int karma_k_avgpool_fwd_bf16(const void* x, void* y, uint32_t n, uint32_t hw, uint32_t c, void* stream) {
  return avgpool_fwd((const bf16_t*)x, (bf16_t*)y, (int)n, (int)hw, (int)c, (hipStream_t)stream);
}

extern "C" int karma_k_avgpool_bwd_bf16(const void* dy, void* dx, uint32_t n, uint32_t hw, uint32_t c, void* stream) {
  return avgpool_bwd((const bf16_t*)dy, (bf16_t*)dx, (int)n, (int)hw, (int)c, (hipStream_t)stream);
}
