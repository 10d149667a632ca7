// HBM-bound kernels of the transformer workloads: LayerNorm, GELU, column sums (bias
// gradients), token/position embedding and its gradient, softmax cross-entropy, fills and
// casts.  KARMA Sec. III-C lists their op counts (softmax 2|X|, element-wise ops inferred);
// here they are bandwidth problems: 16-byte coalesced accesses, one wavefront per row with
// shuffle reductions for the normalisations, fixed-order two-stage sums wherever a
// reduction crosses workgroups (no atomics, so results are reproducible bit for bit).
#include <hip/hip_runtime.h>

#include "karma.h"
#include "device_utils.h"
#include "kernels.h"

namespace karma {

__device__ __forceinline__ float bf2f_(bf16_t b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ bf16_t f2bf_(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
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
// Wavefront reductions with data-parallel-primitive moves (full-rate vector instructions; a cross-lane read
// through the LDS crossbar costs an LDS round trip per step, and a row's two reductions are a chain of twelve).
// Steps: the other lane of a pair, the other pair of a quad, the other quad of a half-row (row_half_mirror), the
// other half of a row of 16 (row_mirror): every lane of a row then holds the row's value; lane 15 of rows 0 and 2
// goes to rows 1 and 3 (row_bcast:15), lane 31 to rows 2 and 3 (row_bcast:31): lane 63 holds the wavefront's value,
// which is read back as a scalar.  `old` is what a lane of a row that a step does not write combines with.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_from(float old, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v), CTRL,
                                                               ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float lane63(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_from<0xB1, 0xf>(0.f, v);    // quad_perm [1,0,3,2]
  v += dpp_from<0x4E, 0xf>(0.f, v);    // quad_perm [2,3,0,1]
  v += dpp_from<0x141, 0xf>(0.f, v);   // row_half_mirror
  v += dpp_from<0x140, 0xf>(0.f, v);   // row_mirror
  v += dpp_from<0x142, 0xa>(0.f, v);   // row_bcast:15 into rows 1 and 3
  v += dpp_from<0x143, 0xc>(0.f, v);   // row_bcast:31 into rows 2 and 3
  return lane63(v);
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_from<0xB1, 0xf>(v, v));
  v = fmaxf(v, dpp_from<0x4E, 0xf>(v, v));
  v = fmaxf(v, dpp_from<0x141, 0xf>(v, v));
  v = fmaxf(v, dpp_from<0x140, 0xf>(v, v));
  v = fmaxf(v, dpp_from<0x142, 0xa>(v, v));
  v = fmaxf(v, dpp_from<0x143, 0xc>(v, v));
  return lane63(v);
}

constexpr float LN_EPS = 1e-5f;
constexpr int LN_MAXV_LIMIT = 12;   // 16-byte vectors per lane: rows up to 64*8*12 = 6144 elements

// ---- LayerNorm forward: a wavefront takes RW rows at a time, held in registers, all loads issued
// before the first reduction.  RW = 1 is what runs: with several rows per wavefront the kernel
// measured slower (fewer wavefronts to spread over the chip outweigh the deeper load queue).
template <int LN_MAXV, int RW>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ g,
                                                             const bf16_t* __restrict__ b, bf16_t* __restrict__ y,
                                                             float* __restrict__ stats, int rows, int h) {
  const int lane = threadIdx.x & 63, row0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * RW;
  if (row0 >= rows) return;
  const int nv = h / 8;
  u32x4 raw[RW][LN_MAXV];
#pragma unroll
  for (int r = 0; r < RW; ++r)
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      const int c = lane + i * 64;
      if (c < nv && row0 + r < rows) raw[r][i] = *(const u32x4*)(x + (size_t)(row0 + r) * h + c * 8);
    }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int row = row0 + r;
    if (row >= rows) break;
    float v[LN_MAXV][8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      if (lane + i * 64 < nv) {
        unpack8(raw[r][i], v[i]);
#pragma unroll
        for (int e = 0; e < 8; ++e) s += v[i][e];
      }
    }
    const float mean = wave_sum(s) / (float)h;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i)
      if (lane + i * 64 < nv)
#pragma unroll
        for (int e = 0; e < 8; ++e) { float d = v[i][e] - mean; q = fmaf(d, d, q); }
    const float rstd = rsqrtf(wave_sum(q) / (float)h + LN_EPS);
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      int c = lane + i * 64;
      if (c < nv) {
        float gg[8], bb[8], o[8];
        unpack8(*(const u32x4*)(g + c * 8), gg);
        unpack8(*(const u32x4*)(b + c * 8), bb);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (v[i][e] - mean) * rstd * gg[e] + bb[e];
        *(u32x4*)(y + (size_t)row * h + c * 8) = pack8(o);
      }
    }
    if (lane == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
  }
}

// ---- LayerNorm backward: dx per row (one wavefront per row); per-workgroup partial sums
// of dgamma/dbeta over a contiguous band of rows, reduced by colsum_finish_kernel.
// dx = rstd * (dy*g - mean(dy*g) - xhat * mean(dy*g*xhat)) (+ add)
// ADDSUM: the column sums of `add` are reduced along with dgamma and dbeta (the added tensor is the gradient
// of the sum the LayerNorm's input went into, whose bias gradient is exactly that column sum: one pass less
// over it).  The partial rows then hold three vectors of h instead of two.
constexpr int LNB_ROWS = 64;   // rows per workgroup: 4 wavefronts x 16 rows
template <int LN_MAXV, bool ADDSUM>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                             const float* __restrict__ stats, const bf16_t* __restrict__ g,
                                                             const bf16_t* __restrict__ add, bf16_t* __restrict__ dx,
                                                             float* __restrict__ partial, int rows, int h) {
  constexpr int NS = ADDSUM ? 3 : 2;
  extern __shared__ float lds[];   // [4][NS][h]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int nv = h / 8;
  float dgam[LN_MAXV][8], dbet[LN_MAXV][8], gg[LN_MAXV][8], asum[ADDSUM ? LN_MAXV : 1][8];
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + i * 64;
    if (c < nv) unpack8(*(const u32x4*)(g + c * 8), gg[i]);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dgam[i][e] = 0.f;
      dbet[i][e] = 0.f;
      if (ADDSUM) asum[i][e] = 0.f;
    }
  }
  // the next row's vectors are requested before this row is reduced (a wavefront walks 16 rows)
  const int first = blockIdx.x * LNB_ROWS + w * (LNB_ROWS / 4);
  u32x4 nx[LN_MAXV], nd[LN_MAXV], na[LN_MAXV];
  auto fetch = [&](int row) {
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      const int c = lane + i * 64;
      if (c < nv && row < rows) {
        nx[i] = *(const u32x4*)(x + (size_t)row * h + c * 8);
        nd[i] = *(const u32x4*)(dy + (size_t)row * h + c * 8);
        if (add) na[i] = *(const u32x4*)(add + (size_t)row * h + c * 8);
      }
    }
  };
  fetch(first);
  for (int r = 0; r < LNB_ROWS / 4; ++r) {
    const int row = first + r;
    if (row >= rows) break;
    const float mean = stats[2 * row], rstd = stats[2 * row + 1];
    float xh[LN_MAXV][8], dyg[LN_MAXV][8];
    u32x4 cur_add[LN_MAXV];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      int c = lane + i * 64;
      if (c < nv) {
        float xv[8], dv[8];
        unpack8(nx[i], xv);
        unpack8(nd[i], dv);
        cur_add[i] = na[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xh[i][e] = (xv[e] - mean) * rstd;
          dyg[i][e] = dv[e] * gg[i][e];
          dgam[i][e] = fmaf(dv[e], xh[i][e], dgam[i][e]);
          dbet[i][e] += dv[e];
          s1 += dyg[i][e];
          s2 = fmaf(dyg[i][e], xh[i][e], s2);
        }
      }
    }
    if (r + 1 < LNB_ROWS / 4) fetch(row + 1);
    const float m1 = wave_sum(s1) / (float)h, m2 = wave_sum(s2) / (float)h;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      int c = lane + i * 64;
      if (c < nv) {
        float o[8], av[8];
        if (add) unpack8(cur_add[i], av);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          o[e] = rstd * (dyg[i][e] - m1 - xh[i][e] * m2);
          if (add) o[e] += av[e];
          if (ADDSUM) asum[i][e] += av[e];
        }
        *(u32x4*)(dx + (size_t)row * h + c * 8) = pack8(o);
      }
    }
  }
  // combine the four wavefronts in fixed order, write this workgroup's partial row
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + i * 64;
    if (c < nv)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        lds[(w * NS + 0) * h + c * 8 + e] = dgam[i][e];
        lds[(w * NS + 1) * h + c * 8 + e] = dbet[i][e];
        if (ADDSUM) lds[(w * NS + 2) * h + c * 8 + e] = asum[i][e];
      }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < NS * h; c += 256) {
    int which = c / h, col = c % h;
    float s = lds[(0 * NS + which) * h + col] + lds[(1 * NS + which) * h + col] + lds[(2 * NS + which) * h + col] +
              lds[(3 * NS + which) * h + col];
    partial[((size_t)blockIdx.x * NS + which) * h + col] = s;
  }
}

// out[c] = sum_p partial[p][c]: eight slices of threads sum every eighth partial, then the
// slices are added in ascending order (a fixed association, so results are reproducible)
// Columns split.. go to out_f32_b (two results that lie side by side in the partials, one launch).
__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ partial, int parts, int stride,
                                                             int cols, bf16_t* __restrict__ out_bf16,
                                                             float* __restrict__ out_f32, int split,
                                                             float* __restrict__ out_f32_b, int split2 = 1 << 30,
                                                             float* __restrict__ out_f32_c = nullptr) {
  __shared__ float red[8][32];
  const int cl = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cl;
  float s = 0.f;
  if (c < cols) {
    int p = slice;
    for (; p + 56 < parts; p += 64) {   // eight loads in flight, added in ascending order
      float v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = partial[(size_t)(p + 8 * k) * stride + c];
#pragma unroll
      for (int k = 0; k < 8; ++k) s += v[k];
    }
    for (; p < parts; p += 8) s += partial[(size_t)p * stride + c];
  }
  red[slice][cl] = s;
  __syncthreads();
  if (slice == 0 && c < cols) {
    float t = red[0][cl];
#pragma unroll
    for (int k = 1; k < 8; ++k) t += red[k][cl];
    if (out_bf16) out_bf16[c] = f2bf_(t);
    if (out_f32) {
      if (c < split) out_f32[c] = t;
      else if (c < split2) out_f32_b[c - split] = t;
      else out_f32_c[c - split2] = t;
    }
  }
}

// The same for many partial rows: 8 columns x 32 slices per workgroup, so that a thread walks parts / 32 rows
// (the walk is a chain of dependent-latency steps; with 8 slices and hundreds of parts it was most of the
// kernel's time).  Slices are added in ascending order.
__global__ __launch_bounds__(256) void colsum_finish_tall_kernel(const float* __restrict__ partial, int parts, int stride,
                                                                  int cols, float* __restrict__ out_f32, int split,
                                                                  float* __restrict__ out_f32_b, int split2,
                                                                  float* __restrict__ out_f32_c) {
  __shared__ float red[32][8];
  const int cl = threadIdx.x & 7, slice = threadIdx.x >> 3;
  const int c = blockIdx.x * 8 + cl;
  float s = 0.f;
  if (c < cols) {
    int p = slice;
    for (; p + 224 < parts; p += 256) {   // eight loads in flight, added in ascending order
      float v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = partial[(size_t)(p + 32 * k) * stride + c];
#pragma unroll
      for (int k = 0; k < 8; ++k) s += v[k];
    }
    for (; p < parts; p += 32) s += partial[(size_t)p * stride + c];
  }
  red[slice][cl] = s;
  __syncthreads();
  if (slice == 0 && c < cols) {
    float t = red[0][cl];
#pragma unroll
    for (int k = 1; k < 32; ++k) t += red[k][cl];
    if (c < split) out_f32[c] = t;
    else if (c < split2) out_f32_b[c - split] = t;
    else out_f32_c[c - split2] = t;
  }
}

// fp32 results from `parts` partial rows: the kernel that suits their number
static void launch_colsum_finish(const float* partial, int parts, int stride, int cols, float* out, int split, float* out_b,
                                 int split2, float* out_c, hipStream_t s) {
  if (parts >= 128)
    hipLaunchKernelGGL(colsum_finish_tall_kernel, dim3((cols + 7) / 8), dim3(256), 0, s, partial, parts, stride, cols, out,
                       split, out_b, split2, out_c);
  else
    hipLaunchKernelGGL(colsum_finish_kernel, dim3((cols + 31) / 32), dim3(256), 0, s, partial, parts, stride, cols,
                       (bf16_t*)nullptr, out, split, out_b, split2, out_c);
}

// column sums of a bf16 matrix [rows][cols]: each workgroup sums a band of rows
constexpr int CS_ROWS = 64;
__global__ __launch_bounds__(256) void colsum_partial_kernel(const bf16_t* __restrict__ x, float* __restrict__ partial,
                                                              int rows, int cols) {
  // thread owns 8 consecutive columns; 256 threads cover 2048 columns per blockIdx.y
  const int c8 = (blockIdx.y * 256 + threadIdx.x) * 8;
  if (c8 >= cols) return;
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const int r0 = blockIdx.x * CS_ROWS, r1 = min(rows, r0 + CS_ROWS);
  int r = r0;
  for (; r + 8 <= r1; r += 8) {   // eight independent loads in flight, added in row order
    u32x4 q[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) q[k] = *(const u32x4*)(x + (size_t)(r + k) * cols + c8);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float v[8];
      unpack8(q[k], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) s[e] += v[e];
    }
  }
  for (; r < r1; ++r) {
    float v[8];
    unpack8(*(const u32x4*)(x + (size_t)r * cols + c8), v);
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) partial[(size_t)blockIdx.x * cols + c8 + e] = s[e];
}

// ---- GELU (tanh form) ------------------------------------------------------------
__global__ void gelu_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, size_t nvec) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float v[8];
  unpack8(((const u32x4*)x)[i], v);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
  ((u32x4*)y)[i] = pack8(v);
}
__global__ void gelu_bwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                size_t nvec) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float v[8], d[8];
  unpack8(((const u32x4*)x)[i], v);
  unpack8(((const u32x4*)dy)[i], d);
#pragma unroll
  for (int e = 0; e < 8; ++e) d[e] *= gelu_grad_f(v[e]);
  ((u32x4*)dx)[i] = pack8(d);
}

// ---- embedding ---------------------------------------------------------------------
// out[t] = wte[ids[t]] + wpe[t % seq]
__global__ void embed_fwd_kernel(const int* __restrict__ ids, const bf16_t* __restrict__ wte,
                                 const bf16_t* __restrict__ wpe, bf16_t* __restrict__ out, int tokens, int seq, int h) {
  const int nv = h / 8;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)tokens * nv) return;
  int t = (int)(i / nv), c = (int)(i % nv);
  float a[8], b[8];
  unpack8(*(const u32x4*)(wte + (size_t)ids[t] * h + c * 8), a);
  unpack8(*(const u32x4*)(wpe + (size_t)(t % seq) * h + c * 8), b);
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] += b[e];
  *(u32x4*)(out + (size_t)t * h + c * 8) = pack8(a);
}
// Token-embedding gradient without atomics.  The host sorts token positions by id
// (stable): order[] lists positions, seg_start[u]..seg_start[u+1] is the run of the u-th
// distinct id seg_id[u].  One workgroup row per distinct id adds its rows in that order
// into the fp32 accumulator (which already holds the LM-head contribution).
__global__ void embed_bwd_wte_kernel(const bf16_t* __restrict__ dx, const int* __restrict__ order,
                                     const int* __restrict__ seg_start, const int* __restrict__ seg_id,
                                     float* __restrict__ dwte, int h) {
  const int u = blockIdx.x;
  const int s0 = seg_start[u], s1 = seg_start[u + 1];
  float* dst = dwte + (size_t)seg_id[u] * h;
  for (int c = threadIdx.x; c < h / 8; c += blockDim.x) {
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = dst[c * 8 + e];
    for (int p = s0; p < s1; ++p) {
      float v[8];
      unpack8(*(const u32x4*)(dx + (size_t)order[p] * h + c * 8), v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) dst[c * 8 + e] = acc[e];
  }
}
// dwpe[s] = sum_b dx[b, s], batch entries in ascending order
__global__ void embed_bwd_wpe_kernel(const bf16_t* __restrict__ dx, bf16_t* __restrict__ dwpe, int batch, int seq, int h) {
  const int nv = h / 8;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)seq * nv) return;
  int s = (int)(i / nv), c = (int)(i % nv);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int b = 0; b < batch; ++b) {
    float v[8];
    unpack8(*(const u32x4*)(dx + ((size_t)b * seq + s) * h + c * 8), v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  *(u32x4*)(dwpe + (size_t)s * h + c * 8) = pack8(acc);
}

// ---- softmax cross-entropy, forward and gradient fused -------------------------------
// One workgroup per row: the row of logits is read once into LDS, reduced (max, sum of
// exponentials), then overwritten with (softmax - onehot) * scale.  rowloss[row] = lse - z[label].
// CE_THREADS threads (16 wavefronts: with a 64 KB row two workgroups fill a compute unit's wave slots, which
// lets one row's loads, exponentials and stores overlap another's); partial results of the wavefronts are
// combined in ascending order.
constexpr int CE_THREADS = 1024, CE_WAVES = CE_THREADS / 64;
__global__ __launch_bounds__(CE_THREADS) void softmax_ce_kernel(bf16_t* __restrict__ logits, const int* __restrict__ labels,
                                                                 float* __restrict__ rowloss, int cols, float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_ce[];
  bf16_t* row = (bf16_t*)smem_ce;
  __shared__ float red[2 * CE_WAVES];
  const int r = blockIdx.x, nv = cols / 8, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  bf16_t* src = logits + (size_t)r * cols;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < nv; c += CE_THREADS) {
    u32x4 v = *(const u32x4*)(src + c * 8);
    *(u32x4*)(row + c * 8) = v;
    float f[8];
    unpack8(v, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) mx = fmaxf(mx, f[e]);
  }
  mx = wave_max(mx);
  if (lane == 0) red[w] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int k = 1; k < CE_WAVES; ++k) mx = fmaxf(mx, red[k]);
  float sum = 0.f;
  for (int c = threadIdx.x; c < nv; c += CE_THREADS) {
    float f[8];
    unpack8(*(const u32x4*)(row + c * 8), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) sum += __expf(f[e] - mx);
  }
  sum = wave_sum(sum);
  if (lane == 0) red[CE_WAVES + w] = sum;
  __syncthreads();
  sum = red[CE_WAVES];
#pragma unroll
  for (int k = 1; k < CE_WAVES; ++k) sum += red[CE_WAVES + k];
  const float lse = mx + __logf(sum);
  const int label = labels[r];
  if (threadIdx.x == 0) rowloss[r] = lse - bf2f_(row[label]);
  const float inv = 1.f / sum;
  for (int c = threadIdx.x; c < nv; c += CE_THREADS) {
    float f[8];
    unpack8(*(const u32x4*)(row + c * 8), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float p = __expf(f[e] - mx) * inv;
      if (c * 8 + e == label) p -= 1.f;
      f[e] = p * scale;
    }
    *(u32x4*)(src + c * 8) = pack8(f);
  }
}

// The same for many short rows (a per-pixel classifier: millions of rows of a few classes): one thread per row,
// the row in registers.  NV = cols / 8.
template <int NV>
__global__ __launch_bounds__(256) void softmax_ce_rows_kernel(bf16_t* __restrict__ logits, const int* __restrict__ labels,
                                                              float* __restrict__ rowloss, int rows, float scale) {
  const size_t r = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= (size_t)rows) return;
  bf16_t* src = logits + r * (NV * 8);
  float f[NV * 8];
#pragma unroll
  for (int c = 0; c < NV; ++c) unpack8(*(const u32x4*)(src + c * 8), f + c * 8);
  float mx = f[0];
#pragma unroll
  for (int e = 1; e < NV * 8; ++e) mx = fmaxf(mx, f[e]);
  float sum = 0.f;
#pragma unroll
  for (int e = 0; e < NV * 8; ++e) sum += __expf(f[e] - mx);
  const int label = labels[r];
  float at_label = 0.f;
  const float inv = 1.f / sum;
#pragma unroll
  for (int e = 0; e < NV * 8; ++e) {
    if (e == label) at_label = f[e];
    float p = __expf(f[e] - mx) * inv;
    if (e == label) p -= 1.f;
    f[e] = p * scale;
  }
  rowloss[r] = mx + __logf(sum) - at_label;
#pragma unroll
  for (int c = 0; c < NV; ++c) *(u32x4*)(src + c * 8) = pack8(f + c * 8);
}

// fixed-order sum of n floats (two stages) scaled: the mean loss
__global__ __launch_bounds__(256) void sum_stage1_kernel(const float* __restrict__ x, float* __restrict__ partial, size_t n) {
  __shared__ float red[256];
  float s = 0.f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) s += x[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int k = 128; k > 0; k >>= 1) {
    if ((int)threadIdx.x < k) red[threadIdx.x] += red[threadIdx.x + k];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}
__global__ __launch_bounds__(256) void sum_stage2_kernel(const float* __restrict__ partial, int count, float scale,
                                                          float* __restrict__ out) {
  __shared__ float red[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < count; i += 256) s += partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int k = 128; k > 0; k >>= 1) {
    if ((int)threadIdx.x < k) red[threadIdx.x] += red[threadIdx.x + k];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0] * scale;
}

// ---- fills and casts -----------------------------------------------------------------
__global__ void fill_u32_kernel(unsigned* __restrict__ p, unsigned v, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void f32_to_bf16_kernel(const float* __restrict__ x, bf16_t* __restrict__ y, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = f2bf_(x[i]);
}

// ------------------------------------------------------------------------------ launchers
static inline int ok() { return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP; }
static inline unsigned blocks_for(size_t n, unsigned per) { return (unsigned)((n + per - 1) / per); }

int layernorm_fwd(const bf16_t* x, const bf16_t* g, const bf16_t* b, bf16_t* y, float* stats, int rows, int h,
                  hipStream_t s) {
  if (h % 8 || h > 64 * 8 * LN_MAXV_LIMIT || rows <= 0) return KARMA_E_INVAL;
  const int per_lane = (h / 8 + 63) / 64;
#define KARMA_LN_FWD(V) hipLaunchKernelGGL((layernorm_fwd_kernel<V, 1>), dim3((rows + 3) / 4), dim3(256), 0, s, x, g, b, y, stats, rows, h)
  if (per_lane <= 2) KARMA_LN_FWD(2);
  else if (per_lane <= 4) KARMA_LN_FWD(4);
  else if (per_lane <= 6) KARMA_LN_FWD(6);
  else if (per_lane <= 9) KARMA_LN_FWD(9);
  else KARMA_LN_FWD(12);
#undef KARMA_LN_FWD
  return ok();
}

// room for three vectors per workgroup (dgamma, dbeta and, when asked for, the column sums of add)
size_t layernorm_bwd_ws_bytes(int rows, int h) { return (size_t)((rows + LNB_ROWS - 1) / LNB_ROWS) * 3 * h * sizeof(float); }

// add_colsum (may be null; needs add): out[c] = sum over rows of add[r][c]
int layernorm_bwd(const bf16_t* dy, const bf16_t* x, const float* stats, const bf16_t* g, const bf16_t* add, bf16_t* dx,
                  float* dgamma, float* dbeta, float* partial_ws, int rows, int h, hipStream_t s, float* add_colsum) {
  if (h % 8 || h > 64 * 8 * LN_MAXV_LIMIT || rows <= 0 || (add_colsum && !add)) return KARMA_E_INVAL;
  const int parts = (rows + LNB_ROWS - 1) / LNB_ROWS;
  const int per_lane = (h / 8 + 63) / 64;
  // rows too wide for three vectors per wavefront in LDS: the plain kernel, then a pass of its own over add
  if (add_colsum && (size_t)4 * 3 * h * sizeof(float) > 160 * 1024) {
    int st = layernorm_bwd(dy, x, stats, g, add, dx, dgamma, dbeta, partial_ws, rows, h, s, nullptr);
    if (st) return st;
    return colsum_bf16(add, add_colsum, partial_ws, rows, h, s);
  }
  const int ns = add_colsum ? 3 : 2;
  const size_t lds = (size_t)4 * ns * h * sizeof(float);
#define KARMA_LN_BWD_K(V, AS)                                                                                    \
  do {                                                                                                           \
    auto kern = layernorm_bwd_kernel<V, AS>;                                                                     \
    if (lds > 64 * 1024) (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
    hipLaunchKernelGGL(kern, dim3(parts), dim3(256), lds, s, dy, x, stats, g, add, dx, partial_ws, rows, h);      \
  } while (0)
#define KARMA_LN_BWD(V)                   \
  do {                                    \
    if (add_colsum) KARMA_LN_BWD_K(V, true); \
    else KARMA_LN_BWD_K(V, false);        \
  } while (0)
  if (per_lane <= 2) KARMA_LN_BWD(2);
  else if (per_lane <= 4) KARMA_LN_BWD(4);
  else if (per_lane <= 6) KARMA_LN_BWD(6);
  else if (per_lane <= 9) KARMA_LN_BWD(9);
  else KARMA_LN_BWD(12);
#undef KARMA_LN_BWD
#undef KARMA_LN_BWD_K
  launch_colsum_finish(partial_ws, parts, ns * h, ns * h, dgamma, h, dbeta, 2 * h, add_colsum, s);
  return ok();
}

size_t colsum_ws_bytes(int rows, int cols) { return (size_t)((rows + CS_ROWS - 1) / CS_ROWS) * cols * sizeof(float); }

int colsum_bf16(const bf16_t* x, float* out, float* partial_ws, int rows, int cols, hipStream_t s) {
  if (cols % 8 || rows <= 0) return KARMA_E_INVAL;
  const int parts = (rows + CS_ROWS - 1) / CS_ROWS;
  hipLaunchKernelGGL(colsum_partial_kernel, dim3(parts, (cols / 8 + 255) / 256), dim3(256), 0, s, x, partial_ws, rows, cols);
  launch_colsum_finish(partial_ws, parts, cols, cols, out, cols, nullptr, 1 << 30, nullptr, s);
  return ok();
}

int colsum_finish(const float* partial, int parts, int cols, float* out, hipStream_t s) {
  if (parts <= 0 || cols <= 0) return KARMA_E_INVAL;
  launch_colsum_finish(partial, parts, cols, cols, out, cols, nullptr, 1 << 30, nullptr, s);
  return ok();
}

int gelu_fwd(const bf16_t* x, bf16_t* y, size_t n, hipStream_t s) {
  if (n % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(gelu_fwd_kernel, dim3(blocks_for(n / 8, 256)), dim3(256), 0, s, x, y, n / 8);
  return ok();
}
int gelu_bwd(const bf16_t* x, const bf16_t* dy, bf16_t* dx, size_t n, hipStream_t s) {
  if (n % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(gelu_bwd_kernel, dim3(blocks_for(n / 8, 256)), dim3(256), 0, s, x, dy, dx, n / 8);
  return ok();
}

int embed_fwd(const int* ids, const bf16_t* wte, const bf16_t* wpe, bf16_t* out, int tokens, int seq, int h, hipStream_t s) {
  if (h % 8) return KARMA_E_INVAL;
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(blocks_for((size_t)tokens * (h / 8), 256)), dim3(256), 0, s, ids, wte, wpe,
                     out, tokens, seq, h);
  return ok();
}
int embed_bwd(const bf16_t* dx, const int* order, const int* seg_start, const int* seg_id, int n_seg, float* dwte_f32,
              bf16_t* dwpe, int batch, int seq, int h, hipStream_t s) {
  if (h % 8) return KARMA_E_INVAL;
  if (n_seg > 0)
    hipLaunchKernelGGL(embed_bwd_wte_kernel, dim3(n_seg), dim3(128), 0, s, dx, order, seg_start, seg_id, dwte_f32, h);
  hipLaunchKernelGGL(embed_bwd_wpe_kernel, dim3(blocks_for((size_t)seq * (h / 8), 256)), dim3(256), 0, s, dx, dwpe,
                     batch, seq, h);
  return ok();
}

int softmax_ce(bf16_t* logits, const int* labels, float* rowloss, int rows, int cols, float scale, hipStream_t s) {
  const size_t lds = (size_t)cols * sizeof(bf16_t);
  if (cols % 8 || rows <= 0 || lds > 150 * 1024) return KARMA_E_INVAL;
  if (cols <= 16 && rows >= 4096) {   // short rows, many of them: a thread per row
    if (cols == 8)
      hipLaunchKernelGGL(softmax_ce_rows_kernel<1>, dim3(blocks_for((size_t)rows, 256)), dim3(256), 0, s, logits, labels, rowloss,
                         rows, scale);
    else
      hipLaunchKernelGGL(softmax_ce_rows_kernel<2>, dim3(blocks_for((size_t)rows, 256)), dim3(256), 0, s, logits, labels, rowloss,
                         rows, scale);
    return ok();
  }
  if (lds > 64 * 1024)
    (void)hipFuncSetAttribute((const void*)softmax_ce_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(softmax_ce_kernel, dim3(rows), dim3(CE_THREADS), lds, s, logits, labels, rowloss, cols, scale);
  return ok();
}

int sum_f32(const float* x, float* out, float* partial_ws, size_t n, float scale, hipStream_t s) {
  int blocks = (int)std::min<size_t>(1024, (n + 255) / 256);
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(sum_stage1_kernel, dim3(blocks), dim3(256), 0, s, x, partial_ws, n);
  hipLaunchKernelGGL(sum_stage2_kernel, dim3(1), dim3(256), 0, s, partial_ws, blocks, scale, out);
  return ok();
}

int fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes % 4) return KARMA_E_INVAL;
  if (!bytes) return KARMA_OK;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(bytes / 4, 256)), dim3(256), 0, s, (unsigned*)p, 0u, bytes / 4);
  return ok();
}
int cast_f32_to_bf16(const float* x, bf16_t* y, size_t n, hipStream_t s) {
  if (!n) return KARMA_OK;
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, x, y, n);
  return ok();
}

}  // namespace karma

using namespace karma;

extern "C" int karma_k_layernorm_fwd_bf16(const void* x, const void* g, const void* b, void* y, float* stats,
                                          uint32_t rows, uint32_t h, void* stream) {
  if (!x || !g || !b || !y || !stats) return KARMA_E_INVAL;
  return layernorm_fwd((const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)y, stats, (int)rows, (int)h,
                       (hipStream_t)stream);
}
extern "C" int karma_k_layernorm_bwd_bf16(const void* dy, const void* x, const float* stats, const void* g,
                                          const void* add, void* dx, float* dgamma, float* dbeta, float* ws,
                                          uint64_t ws_bytes, uint32_t rows, uint32_t h, void* stream) {
  if (!dy || !x || !stats || !g || !dx || !dgamma || !dbeta || !ws) return KARMA_E_INVAL;
  if (ws_bytes < layernorm_bwd_ws_bytes((int)rows, (int)h)) return KARMA_E_OOM;
  return layernorm_bwd((const bf16_t*)dy, (const bf16_t*)x, stats, (const bf16_t*)g, (const bf16_t*)add, (bf16_t*)dx,
                       dgamma, dbeta, ws, (int)rows, (int)h, (hipStream_t)stream, nullptr);
}
extern "C" int karma_k_layernorm_bwd_addsum_bf16(const void* dy, const void* x, const float* stats, const void* g,
                                                 const void* add, void* dx, float* dgamma, float* dbeta,
                                                 float* add_colsum, float* ws, uint64_t ws_bytes, uint32_t rows, uint32_t h,
                                                 void* stream) {
  if (!dy || !x || !stats || !g || !add || !dx || !dgamma || !dbeta || !add_colsum || !ws) return KARMA_E_INVAL;
  if (ws_bytes < layernorm_bwd_ws_bytes((int)rows, (int)h)) return KARMA_E_OOM;
  return layernorm_bwd((const bf16_t*)dy, (const bf16_t*)x, stats, (const bf16_t*)g, (const bf16_t*)add, (bf16_t*)dx,
                       dgamma, dbeta, ws, (int)rows, (int)h, (hipStream_t)stream, add_colsum);
}
extern "C" int karma_k_colsum_bf16(const void* x, float* out, float* ws, uint64_t ws_bytes, uint32_t rows, uint32_t cols,
                                   void* stream) {
  if (!x || !out || !ws) return KARMA_E_INVAL;
  if (ws_bytes < colsum_ws_bytes((int)rows, (int)cols)) return KARMA_E_OOM;
  return colsum_bf16((const bf16_t*)x, out, ws, (int)rows, (int)cols, (hipStream_t)stream);
}
extern "C" int karma_k_gelu_fwd_bf16(const void* x, void* y, uint64_t n, void* stream) {
  if (!x || !y) return KARMA_E_INVAL;
  return gelu_fwd((const bf16_t*)x, (bf16_t*)y, (size_t)n, (hipStream_t)stream);
}
extern "C" int karma_k_gelu_bwd_bf16(const void* x, const void* dy, void* dx, uint64_t n, void* stream) {
  if (!x || !dy || !dx) return KARMA_E_INVAL;
  return gelu_bwd((const bf16_t*)x, (const bf16_t*)dy, (bf16_t*)dx, (size_t)n, (hipStream_t)stream);
}
extern "C" int karma_k_embed_fwd_bf16(const int32_t* ids, const void* wte, const void* wpe, void* out, uint32_t tokens,
                                      uint32_t seq, uint32_t h, void* stream) {
  if (!ids || !wte || !wpe || !out || !seq) return KARMA_E_INVAL;
  return embed_fwd(ids, (const bf16_t*)wte, (const bf16_t*)wpe, (bf16_t*)out, (int)tokens, (int)seq, (int)h,
                   (hipStream_t)stream);
}
extern "C" int karma_k_embed_bwd_bf16(const void* dx, const int32_t* order, const int32_t* seg_start,
                                      const int32_t* seg_id, uint32_t n_seg, float* dwte_f32, void* dwpe,
                                      uint32_t batch, uint32_t seq, uint32_t h, void* stream) {
  if (!dx || !order || !seg_start || !seg_id || !dwte_f32 || !dwpe) return KARMA_E_INVAL;
  return embed_bwd((const bf16_t*)dx, order, seg_start, seg_id, (int)n_seg, dwte_f32, (bf16_t*)dwpe, (int)batch,
                   (int)seq, (int)h, (hipStream_t)stream);
}
extern "C" int karma_k_softmax_ce_bf16(void* logits, const int32_t* labels, float* rowloss, uint32_t rows, uint32_t cols,
                                       float scale, void* stream) {
  if (!logits || !labels || !rowloss) return KARMA_E_INVAL;
  return softmax_ce((bf16_t*)logits, labels, rowloss, (int)rows, (int)cols, scale, (hipStream_t)stream);
}
extern "C" int karma_k_sum_f32(const float* x, float* out, float* ws, uint64_t n, float scale, void* stream) {
  if (!x || !out || !ws || !n) return KARMA_E_INVAL;
  return sum_f32(x, out, ws, (size_t)n, scale, (hipStream_t)stream);
}
