// Device-side helpers shared by the HIP kernels: bf16 conversion, vector types and the
// global -> register -> LDS tile mover used by every MFMA kernel.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace karma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {   // round to nearest even, NaN kept
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// two floats -> packed bf16 pair with the hardware converter (v_cvt_pk_bf16_f32, RNE)
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
// Workgroup barrier that orders LDS traffic only: waits for this wavefront's LDS operations,
// not for its global loads still in flight (a plain __syncthreads() waits for those too,
// which would put the latency of prefetched tiles back on the critical path).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ unsigned pack2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(unsigned, b);
}

// GELU, tanh form: 0.5 x (1 + tanh(u)), u = sqrt(2/pi) (x + 0.044715 x^3).  With
// sig = 1 / (1 + e^(-2u)) = (1 + tanh u) / 2 this is x * sig, and the derivative is
// sig + 2 x sig (1 - sig) u'(x): one hardware exponential and one reciprocal per element.
__device__ __forceinline__ float gelu_sig(float x) {
  const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-2.885390081777927f * u));   // 2 log2(e)
}
__device__ __forceinline__ float gelu_f(float x) { return x * gelu_sig(x); }
__device__ __forceinline__ float gelu_grad_f(float x) {
  const float sg = gelu_sig(x);
  const float du = 0.7978845608028654f * (1.f + 3.f * 0.044715f * x * x);
  return sg + 2.f * x * sg * (1.f - sg) * du;
}

// ---- gfx950: direct global -> LDS loads and transposing LDS reads
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
#define KARMA_LDS(T) __attribute__((address_space(3))) T

// 16 bytes per lane from g (per-lane address) to LDS byte address lds (wavefront-uniform) + 16*lane.
// The s_nop covers the SALU-writes-M0 -> LDS-DMA hazard, which the assembler does not see in inline code.
__device__ __forceinline__ void load_to_lds16(const bf16_t* g, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(__builtin_amdgcn_readfirstlane(lds)), "v"(g)
               : "memory");
}
// The same with the address split into a wavefront-uniform base (scalar registers) and a 32-bit
// per-lane byte offset: no vector arithmetic per load when the offsets are kept in registers.
__device__ __forceinline__ void load_to_lds16_s(const void* base, unsigned byte_off, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(__builtin_amdgcn_readfirstlane(lds)),
               "v"(byte_off), "s"(base)
               : "memory");
}
// LDS-only workgroup barrier written with builtins, so that the compiler's own wait-count
// bookkeeping knows that every LDS read issued before it has returned.
__device__ __forceinline__ void lds_barrier_visible() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), other counters untouched
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Two transposing 8-byte reads make one MFMA k-operand (k-slots 0..3 from `at`, 4..7 from `at2`).
// In each group of 16 lanes, lane 4e+q supplies the address of (k-row e, columns 4q..4q+3) and
// receives, for the column that is its own index in the group, k-rows 0..3.
__device__ __forceinline__ bf16x8 read_tr_pair(unsigned at, unsigned at2) {
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KARMA_LDS(s16x4_t)*)(uintptr_t)at);
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KARMA_LDS(s16x4_t)*)(uintptr_t)at2);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

constexpr int LDS_PAD = 8;   // elements: a 16-byte skew per row keeps ds_read_b128 conflict-free

// One operand tile (ROWS x BK) on its way global -> registers -> LDS [ROWS][BK + pad].
// KC: global is [rows][k] (k contiguous): each thread moves 16-byte k-runs unchanged.
// !KC: global is [k][rows]: each thread loads an 8(k) x 4(rows) patch as eight 8-byte
//      pieces and writes four transposed 16-byte k-runs.
// T threads take part (tid < T).
template <int ROWS, int BK, int T, bool KC>
struct TileMover {
  static constexpr int PITCH = BK + LDS_PAD;
  static constexpr int VECS = ROWS * BK / 8 / T;
  static_assert(ROWS * BK % (8 * T) == 0 && VECS >= 1, "tile does not divide over the workgroup");
  static_assert(KC || VECS % 4 == 0, "transposing mover needs whole 8x4 patches per thread");
  u32x4 reg[VECS];

  // full: the whole tile lies inside the matrix, no bounds checks needed
  __device__ __forceinline__ void load(const bf16_t* __restrict__ G, size_t ld, int row0, int k0, int rows_total,
                                       int k_total, int tid, bool full = false) {
    if (full) {
      if (KC) {
#pragma unroll
        for (int i = 0; i < VECS; ++i) {
          int v = tid + i * T, row = v / (BK / 8), kc = v % (BK / 8);
          reg[i] = *(const u32x4*)(G + (size_t)(row0 + row) * ld + k0 + kc * 8);
        }
      } else {
#pragma unroll
        for (int b = 0; b < VECS / 4; ++b) {
          int v = tid + b * T, rg = v % (ROWS / 4), kg = v / (ROWS / 4);
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            u32x2 r = *(const u32x2*)(G + (size_t)(k0 + kg * 8 + q) * ld + row0 + rg * 4);
            reg[b * 4 + q / 2][(q & 1) * 2] = r.x;
            reg[b * 4 + q / 2][(q & 1) * 2 + 1] = r.y;
          }
        }
      }
      return;
    }
    if (KC) {
#pragma unroll
      for (int i = 0; i < VECS; ++i) {
        int v = tid + i * T, row = v / (BK / 8), kc = v % (BK / 8);
        int gr = row0 + row, gk = k0 + kc * 8;
        u32x4 z = {0, 0, 0, 0};
        reg[i] = (gr < rows_total && gk < k_total) ? *(const u32x4*)(G + (size_t)gr * ld + gk) : z;
      }
    } else {
#pragma unroll
      for (int b = 0; b < VECS / 4; ++b) {
        int v = tid + b * T, rg = v % (ROWS / 4), kg = v / (ROWS / 4);
        int gr = row0 + rg * 4;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          int gk = k0 + kg * 8 + q;
          u32x2 z = {0, 0};
          u32x2 r = (gr < rows_total && gk < k_total) ? *(const u32x2*)(G + (size_t)gk * ld + gr) : z;
          reg[b * 4 + q / 2][(q & 1) * 2] = r.x;
          reg[b * 4 + q / 2][(q & 1) * 2 + 1] = r.y;
        }
      }
    }
  }

  // Element offset of (pixel p of the Ho x Wo grid, tap) in the gathered NHWC tensor, or -1
  // where the convolution reads padding.
  static __device__ __forceinline__ long conv_offset(const ConvGather& cg, int p, int tap) {
    const int hw = cg.Ho * cg.Wo;
    const int img = p / hw, rem = p - img * hw;
    const int ho = rem / cg.Wo, wo = rem - ho * cg.Wo;
    const int r = tap / cg.S, s = tap - r * cg.S;
    int hi, wi;
    if (!cg.transposed) {
      hi = ho * cg.stride - cg.pad + r;
      wi = wo * cg.stride - cg.pad + s;
    } else {
      const int th = ho + cg.pad - r, tw = wo + cg.pad - s;
      if (th < 0 || tw < 0 || th % cg.stride || tw % cg.stride) return -1;
      hi = th / cg.stride;
      wi = tw / cg.stride;
    }
    if ((unsigned)hi >= (unsigned)cg.H || (unsigned)wi >= (unsigned)cg.W) return -1;
    return ((long)(img * cg.H + hi) * cg.W + wi) * cg.C;
  }

  // k-contiguous operand gathered through a convolution: row = output pixel, k = (tap, channel)
  __device__ __forceinline__ void load_conv(const bf16_t* __restrict__ G, const ConvGather& cg, int row0, int k0,
                                            int rows_total, int k_total, int tid) {
    static_assert(KC || VECS % 4 == 0, "");
    if (KC) {
#pragma unroll
      for (int i = 0; i < VECS; ++i) {
        int v = tid + i * T, row = v / (BK / 8), kc = v % (BK / 8);
        int gr = row0 + row, gk = k0 + kc * 8;
        u32x4 z = {0, 0, 0, 0};
        reg[i] = z;
        if (gr < rows_total && gk < k_total) {
          const int tap = gk / cg.C, c = gk - tap * cg.C;
          const long at = conv_offset(cg, gr, tap);
          if (at >= 0) reg[i] = *(const u32x4*)(G + at + c);
        }
      }
    } else {
      // strided operand: row index n = (tap, channel), k = output pixel
#pragma unroll
      for (int b = 0; b < VECS / 4; ++b) {
        int v = tid + b * T, rg = v % (ROWS / 4), kg = v / (ROWS / 4);
        int gr = row0 + rg * 4;
        const int tap = gr / cg.C, c = gr - tap * cg.C;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          int gk = k0 + kg * 8 + q;
          u32x2 r = {0, 0};
          if (gr < rows_total && gk < k_total) {
            const long at = conv_offset(cg, gk, tap);
            if (at >= 0) r = *(const u32x2*)(G + at + c);
          }
          reg[b * 4 + q / 2][(q & 1) * 2] = r.x;
          reg[b * 4 + q / 2][(q & 1) * 2 + 1] = r.y;
        }
      }
    }
  }

  __device__ __forceinline__ void store(bf16_t* __restrict__ S, int tid) const {
    if (KC) {
#pragma unroll
      for (int i = 0; i < VECS; ++i) {
        int v = tid + i * T, row = v / (BK / 8), kc = v % (BK / 8);
        *(u32x4*)(S + row * PITCH + kc * 8) = reg[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < VECS / 4; ++b) {
        int v = tid + b * T, rg = v % (ROWS / 4), kg = v / (ROWS / 4);
        // reg[b*4 + p] = { k=2p: (r0 r1 | r2 r3), k=2p+1: (r0 r1 | r2 r3) } as dwords x y z w
        u32x4 t[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          unsigned e0 = reg[b * 4 + p].x, e1 = reg[b * 4 + p].y;   // row k = 2p
          unsigned o0 = reg[b * 4 + p].z, o1 = reg[b * 4 + p].w;   // row k = 2p + 1
          t[0][p] = (e0 & 0xffffu) | (o0 << 16);
          t[1][p] = (e0 >> 16) | (o0 & 0xffff0000u);
          t[2][p] = (e1 & 0xffffu) | (o1 << 16);
          t[3][p] = (e1 >> 16) | (o1 & 0xffff0000u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) *(u32x4*)(S + (rg * 4 + j) * PITCH + kg * 8) = t[j];
      }
    }
  }
};

}  // namespace karma
