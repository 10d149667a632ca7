// Internal launchers of the HIP kernels (C++ side of the kernel-level C ABI).
// All pointers are device pointers; every launcher is asynchronous on `s` and returns a
// karma_status.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <vector>

namespace karma {

typedef uint16_t bf16_t;   // bit pattern of a bfloat16

// ---- fp32 MLP kernels (kernels_f32.hip)
int linear_relu_fwd_f32(const float* x, const float* w, const float* b, float* z, float* y, int m, int n, int k,
                        hipStream_t s);
int linear_relu_bwd_f32(const float* x, const float* w, const float* z, const float* dy, float* dz, float* dx,
                        float* dw, float* db, int m, int n, int k, hipStream_t s);
int mse_f32(const float* y, const float* t, float* dy, float* loss, float* partial, size_t n, hipStream_t s);

// ---- bf16 GEMM on the matrix cores (gemm_bf16.hip)
// An operand that is an NHWC tensor seen through a convolution (implicit GEMM): GEMM row (or,
// for the weight gradient, reduction index) p = (image, ho, wo) on the Ho x Wo grid and
// index j = (r*S + s)*C + c address element (image, hi, wi, c) of the H x W x C tensor with
//   hi = ho*stride - pad + r, wi = wo*stride - pad + s              (transposed = 0), or
//   hi = (ho + pad - r)/stride, wi = (wo + pad - s)/stride where both divide (transposed = 1:
//   the gradient of a strided convolution w.r.t. its input); positions outside count as zero.
struct ConvGather {
  int H, W, C, Ho, Wo, R, S, stride, pad, transposed;
};

// C[M,N] = sum_k A(m,k) B(n,k) (+ bias[n]) (+ residual[m,n]).  a_kc: A is [M][lda] with k
// contiguous, else [K][lda] with m contiguous; same for B with n.
struct GemmArgs {
  const bf16_t* A; const bf16_t* B; void* C;
  const bf16_t* bias; const bf16_t* residual;
  int M, N, K, lda, ldb, ldc;
  bool a_kc, b_kc, out_f32, accumulate;
  void* ws;          // optional fp32 workspace for split-k partial sums (dense C only)
  size_t ws_bytes;
  // conv_mode 1: A (k-contiguous) is gathered, rows = output pixels, k = (tap, channel);
  // conv_mode 2: B (strided) is gathered, k = output pixels, n = (tap, channel)
  int conv_mode;
  ConvGather conv;
  // act 1: C = A B^T + bias as usual and aux (bf16 [M][ldc], written) = GELU(C as stored);
  // act 2: C = (A B^T) * GELU'(aux), aux (read) holding the pre-activation.  bf16 C, no residual, no split.
  int act;
  void* aux;
  // act 2, optional: room for ceil(M / 128) rows of N floats.  When the product runs on the kernel that can do
  // it, partial column sums of C (fp32, before rounding) are left there and *colsum_rows (preset to 0 by the
  // caller) is set to their number; colsum_finish adds them up.  Otherwise nothing is written.
  float* colsum_partial;
  int* colsum_rows;
};
int gemm_bf16(const GemmArgs& g, hipStream_t s);
// While non-null on the calling thread, gemm_bf16 calls record an event before and after
// their launch (pairs appended from *used on, created on demand) and their flop count: the
// benchmark's per-launch timing of the dominant kernel.  One call in `stride` is timed (the
// one whose running index `seq` is congruent to `phase`), so that the events, each of which
// also keeps consecutive kernels from overlapping, stay a small part of the step; the caller
// rotates the phase from step to step so that every launch site is sampled.
struct GemmTimer {
  std::vector<hipEvent_t>* events;
  size_t* used;
  std::vector<double>* flops;
  unsigned stride, phase, seq;
};
extern thread_local GemmTimer* g_gemm_timer;


// ---- HBM-bound bf16 kernels (norm_act.hip)
int layernorm_fwd(const bf16_t* x, const bf16_t* g, const bf16_t* b, bf16_t* y, float* stats, int rows, int h, hipStream_t s);
size_t layernorm_bwd_ws_bytes(int rows, int h);
// dx = LayerNorm backward (+ add, may be null); dgamma/dbeta fp32 [h]
int layernorm_bwd(const bf16_t* dy, const bf16_t* x, const float* stats, const bf16_t* g, const bf16_t* add, bf16_t* dx,
                  float* dgamma, float* dbeta, float* partial_ws, int rows, int h, hipStream_t s,
                  float* add_colsum = nullptr);
size_t colsum_ws_bytes(int rows, int cols);
int colsum_bf16(const bf16_t* x, float* out, float* partial_ws, int rows, int cols, hipStream_t s);
// out[c] = sum over p < parts of partial[p][c] (rows of cols floats), in a fixed order
int colsum_finish(const float* partial, int parts, int cols, float* out, hipStream_t s);
int gelu_fwd(const bf16_t* x, bf16_t* y, size_t n, hipStream_t s);
int gelu_bwd(const bf16_t* x, const bf16_t* dy, bf16_t* dx, size_t n, hipStream_t s);
int embed_fwd(const int* ids, const bf16_t* wte, const bf16_t* wpe, bf16_t* out, int tokens, int seq, int h, hipStream_t s);
int embed_bwd(const bf16_t* dx, const int* order, const int* seg_start, const int* seg_id, int n_seg, float* dwte_f32,
              bf16_t* dwpe, int batch, int seq, int h, hipStream_t s);
int softmax_ce(bf16_t* logits, const int* labels, float* rowloss, int rows, int cols, float scale, hipStream_t s);
int sum_f32(const float* x, float* out, float* partial_ws, size_t n, float scale, hipStream_t s);
int fill_zero(void* p, size_t bytes, hipStream_t s);
int cast_f32_to_bf16(const float* x, bf16_t* y, size_t n, hipStream_t s);

// ---- convolutional workload (conv_bn.hip): NHWC bf16, weights [c_out][r][s][c_in]
struct ConvShape { int N, H, W, Cin, Cout, R, S, stride, pad; };
int conv_out_dim(int n, int k, int stride, int pad);
// ws / ws_bytes: optional fp32 workspace that lets a product with few output tiles split its reduction;
// add (may be null): a tensor of y's shape added to the result (a residual sum)
int conv2d_fwd(const bf16_t* x, const bf16_t* w, bf16_t* y, const ConvShape& c, hipStream_t s, void* ws = nullptr,
               size_t ws_bytes = 0, const bf16_t* add = nullptr);
size_t conv2d_dgrad_ws_elems(const ConvShape& c);   // elements of the transposed-weight buffer (0 for 1x1 stride 1)
// dx = gradient w.r.t. the input (+ add, may be null)
int conv2d_dgrad(const bf16_t* dy, const bf16_t* w, bf16_t* wt_ws, const bf16_t* add, bf16_t* dx, const ConvShape& c,
                 hipStream_t s, void* ws = nullptr, size_t ws_bytes = 0);
// dw [c_out][r][s][c_in]; ws: optional fp32 split-k workspace
int conv2d_wgrad(const bf16_t* dy, const bf16_t* x, bf16_t* dw, void* ws, size_t ws_bytes, const ConvShape& c, hipStream_t s);
size_t bn_ws_bytes(int rows, int c);
// training-mode batch normalisation over the rows of [rows][c]; stats = mean[c], rstd[c];
// y = xhat*g + b (+ add) (ReLU when relu != 0)
int bn_fwd(const bf16_t* x, const bf16_t* g, const bf16_t* b, const bf16_t* add, bf16_t* y, float* stats, float* ws,
           int rows, int c, int relu, hipStream_t s);
// the normalisation alone, from statistics already computed (recomputing an output)
// gate (may be null): y receives gate's element where the value as stored is positive, zero elsewhere
// (the gradient through the ReLU that follows the normalisation)
int bn_apply(const bf16_t* x, const float* stats, const bf16_t* g, const bf16_t* b, const bf16_t* add, bf16_t* y, int rows,
             int c, int relu, hipStream_t s, const bf16_t* gate = nullptr);
// relu != 0: dy first passes the ReLU that followed the normalisation (mask recomputed);
// add (may be null, may be dy): a tensor of x's shape added to dx (the gradient of a shortcut from x)
int bn_bwd(const bf16_t* dy, const bf16_t* x, const float* stats, const bf16_t* g, const bf16_t* b, int relu, bf16_t* dx,
           float* dgamma, float* dbeta, float* ws, int rows, int c, hipStream_t s, const bf16_t* add = nullptr);
int relu_mask_bwd(const bf16_t* dy, const bf16_t* y, bf16_t* dz, size_t n, hipStream_t s);
int maxpool_fwd(const bf16_t* x, bf16_t* y, int n, int h, int w, int c, hipStream_t s);   // 3x3, stride 2, pad 1
int maxpool_bwd(const bf16_t* x, const bf16_t* dy, bf16_t* dx, int n, int h, int w, int c, hipStream_t s);
int maxpool2_fwd(const bf16_t* x, bf16_t* y, int n, int h, int w, int c, hipStream_t s);  // 2x2, stride 2; h, w even
int maxpool2_bwd(const bf16_t* x, const bf16_t* dy, bf16_t* dx, int n, int h, int w, int c, hipStream_t s);
int add_inplace_bf16(bf16_t* y, const bf16_t* a, size_t n, hipStream_t s);                // y += a; n a multiple of 8
int avgpool_fwd(const bf16_t* x, bf16_t* y, int n, int hw, int c, hipStream_t s);         // global
int avgpool_bwd(const bf16_t* dy, bf16_t* dx, int n, int hw, int c, hipStream_t s);

// ---- the optimiser's update on the device (optim_dev.hip): kind = karma_opt_kind; fp32 master weights and state,
// g the gradient (bf16 or fp32), out the device copy of the weight (bf16 or fp32); step counts from 1
int optim_update_dev(int kind, float* w, float* m, float* v, const void* g, bool g_bf16, size_t n, float lr, float beta1,
                     float beta2, float eps, uint64_t step, void* out, bool out_bf16, hipStream_t s);

// ---- fused causal attention (attention.hip); seq multiple of 128, d in {64, 128}
int attention_fwd(const bf16_t* qkv, bf16_t* ctx, float* lse, int batch, int seq, int heads, int d, hipStream_t s);
int attention_bwd(const bf16_t* qkv, const bf16_t* ctx, const bf16_t* dctx, const float* lse, float* delta,
                  bf16_t* dqkv, int batch, int seq, int heads, int d, hipStream_t s, float* colsum_partial = nullptr,
                  int* colsum_rows = nullptr);
size_t attention_bwd_colsum_bytes(int batch, int seq, int heads, int d);

}  // namespace karma
