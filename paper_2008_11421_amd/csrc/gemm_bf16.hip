// bf16 GEMM on the CDNA4 matrix cores: C[M,N] = sum_k A(m,k) B(n,k), fp32 accumulation.
// This is the dense contraction behind every fully connected layer of the transformer
// workloads (KARMA Sec. III-C "Fully-Connected Layer": |X| x |Y| multiply-adds) and its
// two gradients (dX = dY W, dW = dY^T X).
//
// Operands may have the reduction index contiguous ("k-contiguous": A[M][K], B[N][K]) or
// strided (A[K][M], B[K][N]); strided tiles are transposed in registers on their way into
// LDS, so the MFMA loop always reads 16-byte k-runs.  Tiles are staged through LDS with
// one register-resident tile in flight (double buffer); v_mfma_f32_32x32x16_bf16 does the
// arithmetic; the workgroup -> tile map keeps each XCD's L2 on a compact patch of C.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "karma.h"
#include "device_utils.h"
#include "kernels.h"

namespace karma {

struct GemmEpilogue {
  void* C;                 // bf16 or fp32 [M][ldc]
  const bf16_t* bias;      // [N] or null
  const bf16_t* residual;  // [M][ldc] or null (bf16 output only)
  int ldc;
  int out_f32;             // store fp32 instead of bf16
  int accumulate;          // fp32 output only: C += result
  bf16_t* aux;             // [M][ldc]: octet<1> writes GELU(C) there, octet<2> multiplies the result by GELU'(aux) (bf16 C only)
  float* colsum;           // direct-load kernel, octet<2> only, or null: [tiles_m * 2][N] partial column sums of the result
  // eight consecutive columns n..n+7 of row m (n multiple of 8); cols = how many are inside the matrix
  // pre (when have_pre): the eight residual (or, ACT 2, pre-activation) values of this octet, fetched by the caller
  template <int ACT = 0>
  __device__ __forceinline__ void octet(int m, int n, int cols, const float4& lo, const float4& hi,
                                        bool have_pre = false, u32x4 pre = u32x4{0, 0, 0, 0}) const {
    float unused[8];
    octet<ACT>(m, n, cols, lo, hi, have_pre, pre, false, unused);
  }
  // do_sum (octet<2>, full octets): the eight results are also added to sum8
  template <int ACT>
  __device__ __forceinline__ void octet(int m, int n, int cols, const float4& lo, const float4& hi, bool have_pre, u32x4 pre,
                                        bool do_sum, float (&sum8)[8]) const {
    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    const size_t at = (size_t)m * ldc + n;
    if (cols == 8 && (ldc & 7) == 0) {
      if (bias) {
        u32x4 b = *(const u32x4*)(bias + n);
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(b[e] << 16); v[2 * e + 1] += __uint_as_float(b[e] & 0xffff0000u); }
      }
      if (out_f32) {
        float4* c = (float4*)((float*)C + at);
        float4 o0 = make_float4(v[0], v[1], v[2], v[3]), o1 = make_float4(v[4], v[5], v[6], v[7]);
        if (accumulate) {
          float4 p0 = c[0], p1 = c[1];
          o0.x += p0.x; o0.y += p0.y; o0.z += p0.z; o0.w += p0.w;
          o1.x += p1.x; o1.y += p1.y; o1.z += p1.z; o1.w += p1.w;
        }
        c[0] = o0;
        c[1] = o1;
      } else {
        if (residual) {
          u32x4 r = have_pre ? pre : *(const u32x4*)(residual + at);
#pragma unroll
          for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(r[e] << 16); v[2 * e + 1] += __uint_as_float(r[e] & 0xffff0000u); }
        }
        if (ACT == 2) {
          u32x4 r = have_pre ? pre : *(const u32x4*)(aux + at);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[2 * e] *= gelu_grad_f(__uint_as_float(r[e] << 16));
            v[2 * e + 1] *= gelu_grad_f(__uint_as_float(r[e] & 0xffff0000u));
          }
          if (do_sum) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sum8[e] += v[e];
          }
        }
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = pack2(v[2 * e], v[2 * e + 1]);
        *(u32x4*)((bf16_t*)C + at) = o;
        if (ACT == 1) {   // the activation of the value as stored (what a separate pass over C would compute)
          u32x4 a2;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            a2[e] = pack2(gelu_f(__uint_as_float(o[e] << 16)), gelu_f(__uint_as_float(o[e] & 0xffff0000u)));
          *(u32x4*)(aux + at) = a2;
        }
      }
    } else {
      for (int e = 0; e < cols; ++e) {
        float x = v[e];
        if (bias) x += bf2f(bias[n + e]);
        if (out_f32) {
          float* c = (float*)C;
          c[at + e] = accumulate ? c[at + e] + x : x;
        } else {
          if (residual) x += bf2f(residual[at + e]);
          if (ACT == 2) x *= gelu_grad_f(bf2f(aux[at + e]));
          const bf16_t stored = f2bf(x);
          ((bf16_t*)C)[at + e] = stored;
          if (ACT == 1) aux[at + e] = f2bf(gelu_f(bf2f(stored)));
        }
      }
    }
  }
};

// Persistent kernel: each workgroup walks the work items (output tile x k-split) of its
// XCD's range.  Per item: the first k-tile is already in registers (loaded while the previous
// item's results were being written out), the main loop is software-pipelined by hand
// (fragments of step kk+1 are read from LDS while the MFMAs of step kk run; the next
// k-tile's global loads are issued at the top and parked in LDS half way through), and the
// results leave through a per-wavefront LDS strip so that stores are row-contiguous.  The
// stores are not waited for: they drain while the next item computes.
// CONV 1: A is an NHWC tensor gathered through a convolution (rows = output pixels, forward
// and input-gradient passes); CONV 2: B is (reduction index = output pixels, weight gradient).
template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int CONV = 0, int ACT = 0>
__global__ __launch_bounds__(WGM* WGN * 64, (BM <= 128 && BN <= 128 ? 2 : 1)) void gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                   const bf16_t* __restrict__ B, int M, int N, int K,
                                                                   int lda, int ldb, int tiles_m, int tiles_n,
                                                                   int splits, int k_per_split, GemmEpilogue ep,
                                                                   float* __restrict__ partial, ConvGather cg) {
  static_assert(CONV == 0 || (CONV == 1 && A_KC) || (CONV == 2 && !B_KC), "which operand a convolution gathers");
  constexpr int T = WGM * WGN * 64;
  constexpr int PITCH = BK + LDS_PAD;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int KSTEPS = BK / 16;
  static_assert(KSTEPS % 2 == 0 && KSTEPS >= 4, "fragment double buffer alternates per step; tiles are parked before the barrier of step KSTEPS-2");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = (bf16_t*)smem;          // [2][BM][PITCH]
  bf16_t* Bs = As + 2 * BM * PITCH;    // [2][BN][PITCH]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int lrow = lane & 31, lk = (lane >> 5) * 8;
  const int total_tiles = tiles_m * tiles_n;
  const int total_items = total_tiles * splits;

  // Work items are numbered split-major (item = split * tiles + tile) and cut into 8 equal
  // contiguous ranges, one per XCD: workgroup ids go round-robin over the XCDs, so workgroup
  // b serves range b % 8, starting at position b / 8 and advancing by gridDim.x / 8.  What
  // runs together on one XCD is then a compact patch of tiles inside one k-split (tiles are
  // walked in bands of 8 tile rows), so its L2 fetches every operand panel about once.
  const int per_xcd = (total_items + 7) / 8;
  const int xcd_first = (int)(blockIdx.x % 8) * per_xcd;
  const int xcd_step = (int)gridDim.x / 8;
  auto decode = [&](int pos, int& m0, int& n0, int& kb, int& ke, int& split) {
    const int item = xcd_first + pos;
    split = item / total_tiles;
    const int id = item % total_tiles;
    constexpr int BAND = 8;
    const int band_sz = BAND * tiles_n;
    const int first_m = (id / band_sz) * BAND;
    const int rows_in_band = min(tiles_m - first_m, BAND);
    m0 = (first_m + (id % band_sz) % rows_in_band) * BM;
    n0 = ((id % band_sz) / rows_in_band) * BN;
    kb = split * k_per_split;
    ke = min(K, kb + k_per_split);
  };
  auto valid = [&](int pos) { return pos < per_xcd && xcd_first + pos < total_items; };

  TileMover<BM, BK, T, A_KC> ma;
  TileMover<BN, BK, T, B_KC> mb;
  auto load_a = [&](int row0, int k0, int k_end, bool whole) {
    if (CONV == 1) ma.load_conv(A, cg, row0, k0, M, k_end, tid);
    else ma.load(A, lda, row0, k0, M, k_end, tid, whole);
  };
  auto load_b = [&](int row0, int k0, int k_end, bool whole) {
    if (CONV == 2) mb.load_conv(B, cg, row0, k0, N, k_end, tid);
    else mb.load(B, ldb, row0, k0, N, k_end, tid, whole);
  };
  bf16x8 af[2][TM], bfr[2][TN];
  auto read_frags = [&](int buf, int cur, int kk) {
    const bf16_t* as = As + cur * BM * PITCH + (wm * WTM + lrow) * PITCH + lk + kk * 16;
    const bf16_t* bs = Bs + cur * BN * PITCH + (wn * WTN + lrow) * PITCH + lk + kk * 16;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[buf][i] = *(const bf16x8*)(as + i * 32 * PITCH);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[buf][j] = *(const bf16x8*)(bs + j * 32 * PITCH);
  };

  int pos = blockIdx.x / 8;
  if (!valid(pos)) return;
  int m0, n0, kb, ke, split;
  decode(pos, m0, n0, kb, ke, split);
  bool full = m0 + BM <= M && n0 + BN <= N && (ke - kb) % BK == 0;
  load_a(m0, kb, ke, full);
  load_b(n0, kb, ke, full);

  for (;;) {
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    lds_barrier();   // every wavefront is done with the previous item's tiles
    ma.store(As, tid);
    mb.store(Bs, tid);
    lds_barrier();
    read_frags(0, 0, 0);
    const int KT = (ke - kb + BK - 1) / BK;
    // the second k-tile starts its trip right away: a tile's loads are issued one whole
    // tile time before they are parked in LDS (half way through the tile before it is used)
    if (KT > 1) {
      load_a(m0, kb + BK, ke, full);
      load_b(n0, kb + BK, ke, full);
    }
    for (int kt = 0; kt < KT; ++kt) {
      const int cur = kt & 1;
      const bool more = kt + 1 < KT;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        // fragments of the next step; the last step already reads the next tile (the barrier
        // after the step before it has made that tile visible and retired this one)
        if (kk + 1 < KSTEPS) read_frags((kk + 1) & 1, cur, kk + 1);
        else if (more) read_frags(0, cur ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // The next tile is parked in LDS half way through the current one and its registers
        // are refilled at once with the tile after next.  Transposed tiles, whose LDS writes
        // are slower, go in two halves (A after step 0, B after step 1) so that the eight
        // wavefronts' writes do not all land in the same step.
        constexpr int A_AT = 0;
        constexpr int B_AT = A_KC ? 0 : 1;
        if (kk == A_AT && more) {
          ma.store(As + (cur ^ 1) * BM * PITCH, tid);
          if (A_AT != B_AT && kt + 2 < KT) load_a(m0, kb + (kt + 2) * BK, ke, full);
        }
        if (kk == B_AT && more) {
          mb.store(Bs + (cur ^ 1) * BN * PITCH, tid);
          if (kt + 2 < KT) {
            if (A_AT == B_AT) load_a(m0, kb + (kt + 2) * BK, ke, full);
            load_b(n0, kb + (kt + 2) * BK, ke, full);
          }
        }
        if ((kk == A_AT || kk == B_AT) && more) __builtin_amdgcn_sched_barrier(0);
        if (kk == KSTEPS - 2) lds_barrier();
      }
    }
    lds_barrier();   // the last tile's reads are done: LDS is free for the epilogue

    // where the results of this item go
    const int out_m0 = m0, out_n0 = n0, out_split = split;
    // start fetching the next item's first k-tile before writing this one out
    pos += xcd_step;
    const bool have_next = valid(pos);
    if (have_next) {
      decode(pos, m0, n0, kb, ke, split);
      full = m0 + BM <= M && n0 + BN <= N && (ke - kb) % BK == 0;
      load_a(m0, kb, ke, full);
      load_b(n0, kb, ke, full);
    }

    // Epilogue through LDS (the operand tiles are dead now: the k-loop ended on a barrier).
    // The MFMAs ran with the operands exchanged, so each accumulator holds the transposed
    // tile: register r of lane l is column (r/4)*8 + (l/32)*4 + r%4 of row l%32, i.e. four
    // consecutive columns per register quad.  Each wavefront parks one 32-row strip of its
    // tile in its own fp32 [32][WTN] patch of LDS with 16-byte writes, then reads it back so
    // that a run of lanes stores one contiguous piece of a row (stores that scatter 16-byte
    // pieces over 32 rows are several times slower).  The patch is private to the wavefront,
    // whose LDS operations execute in order: no barrier in here.
    constexpr int SP = WTN + 4;   // fp32 pitch of the strip
    static_assert((size_t)WGM * WGN * 32 * SP * 4 <= (size_t)2 * (BM + BN) * PITCH * 2, "strip does not fit the tile LDS");
    float* strip = (float*)smem + wave * 32 * SP;
    constexpr int QPR = WTN / 8;              // octets per strip row
    constexpr int RPI = 64 / QPR;             // rows covered per pass of the wavefront
    static_assert(QPR >= 4 && 64 % QPR == 0 && RPI % 2 == 0 && 32 % RPI == 0, "strip read-out does not tile");
    // lane -> (octet q, row rr) such that eight consecutive lanes read two rows' worth of
    // alternate 16-byte units (conflict-free with the odd pitch in 16-byte units)
    const int q = (lane & 3) | (((lane >> 3) % (QPR / 4)) << 2);
    const int rr = ((lane >> 2) & 1) | ((lane / (2 * QPR)) << 1);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(float4*)(strip + lrow * SP + j * 32 + g * 8 + (lane >> 5) * 4) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      const int n = out_n0 + wn * WTN + q * 8;
#pragma unroll
      for (int pass = 0; pass < 32 / RPI; ++pass) {
        const int row = pass * RPI + rr;
        const int m = out_m0 + wm * WTM + i * 32 + row;
        const float4 v = *(const float4*)(strip + row * SP + q * 8);
        const float4 u = *(const float4*)(strip + row * SP + q * 8 + 4);
        if (m < M && n < N) {
          if (splits > 1) {
            float* dst = partial + ((size_t)out_split * M + m) * N + n;
            const float vv[8] = {v.x, v.y, v.z, v.w, u.x, u.y, u.z, u.w};
            if (n + 8 <= N && (N & 3) == 0) { *(float4*)dst = v; *(float4*)(dst + 4) = u; }
            else for (int e = 0; e < N - n && e < 8; ++e) dst[e] = vv[e];
          } else {
            ep.template octet<ACT>(m, n, min(8, N - n), v, u);
          }
        }
      }
    }
    if (!have_next) break;
  }
}

// ---------------------------------------------------------------------------------------
// The same product for shapes made of whole tiles, with the two gfx950 additions that take
// the operand tiles off the vector-register path:
//  * global_load_lds_dwordx4 copies 16 bytes per lane from global memory straight into LDS
//    (lane l's piece lands at M0 + 16*l): no staging registers, no ds_write burst in which
//    all eight wavefronts stall at once, and the loads are waited for only at the single
//    barrier per k-tile;
//  * ds_read_b64_tr_b16 reads a strided operand (k-rows of m-contiguous elements) out of LDS
//    already transposed into the MFMA's 8-consecutive-k-per-lane layout, so strided tiles
//    need no register transposes either.
// LDS holds two stages of (A tile, B tile) without padding; bank conflicts are avoided by
// choosing which 16-byte piece of global memory each lane fetches (an XOR swizzle of the
// piece index with low bits of the row), undone in the fragment addresses.
// The tile stream is continuous across work items: while the last k-tile of an item is being
// multiplied, the first k-tile of the next item is already landing in the other stage; the
// epilogue's fp32 strip aliases the stage of the last tile (plus a small margin).
// EDGE: the matrix need not be made of whole tiles.  Pieces of an operand tile that lie outside the matrix are
// not fetched (their lanes are masked out of the direct load) and their 16 bytes of LDS are zeroed instead, so
// that the products they enter vanish; results outside the matrix are not stored.
// CONV 1 (with EDGE, both operands k-contiguous): A is an NHWC tensor gathered through a convolution, rows =
// pixels of the grid cg.Ho x cg.Wo, k = (tap, channel).  A 16-byte piece is eight channels of one (pixel, tap), so
// the direct load takes it from wherever the convolution reads it, and pieces that fall on padding (or on the
// holes of a strided convolution's gradient) are zeroed in LDS like pieces outside the matrix.  The pixel of each
// of a lane's rows is decoded once per work item; per k-tile only (tap, channel) of the lane's two k offsets are
// (multiplications by reciprocals: magic_c = 2^32 / C + 1, magic_s = 2^32 / S + 1, exact for the sizes admitted).
// CONV 2 (with EDGE, both operands strided): B is gathered, k = pixels of the grid cg.Ho x cg.Wo, n = (tap, channel):
// the weight gradient.  A lane's four k-rows are four pixels that change with every k-tile: each is decoded per tile
// (image by a float reciprocal with an exact correction, row and column by reciprocal multiplication: magic_w =
// 2^32 / Wo + 1, inv_grid = 1 / (Ho * Wo)).
template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int ACT = 0, bool EDGE = false, int CONV = 0>
__global__ __launch_bounds__(WGM* WGN * 64, (BM == 256 && BN == 64) ? 4 : 1) void gemm_bf16_dl_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                                         int M, int N, int K, int lda, int ldb, int tiles_m,
                                                                         int tiles_n, int splits, int k_per_split,
                                                                         GemmEpilogue ep, float* __restrict__ partial,
                                                                         ConvGather cg, unsigned magic_c, unsigned magic_s,
                                                                         unsigned magic_w, float inv_grid) {
  static_assert(CONV == 0 || (CONV == 1 && A_KC && B_KC && EDGE && ACT == 0) || (CONV == 2 && !A_KC && !B_KC && EDGE && ACT == 0),
                "the gathered forms");
  constexpr int WAVES = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int KSTEPS = BK / 16;
  static_assert(BK == 64 && KSTEPS == 4, "swizzles below are written for 128-byte k-rows");
  // the narrow tile (BN = 64: convolutions with 64 output channels) exists for k-contiguous operands only
  static_assert((BM == 256 && BN == 256) || (BM == 256 && BN == 64 && A_KC && B_KC), "strided swizzle assumes 512-byte k-rows");
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int CH_A = A_BYTES / 1024 / WAVES, CH_B = B_BYTES / 1024 / WAVES;   // 1 KiB pieces per wavefront
  constexpr int LPT = CH_A + CH_B;                                               // direct loads per lane per k-tile
  constexpr int SP = WTN + 4;
  constexpr int STRIP = WAVES * 32 * SP * 4;
  constexpr int EXTRA = STRIP > STAGE ? STRIP - STAGE : 0;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [EXTRA][stage 0][stage 1][EXTRA]
  const unsigned lds0 = (unsigned)(uintptr_t)((KARMA_LDS(unsigned char)*)smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int lrow = lane & 31;
  const int total_tiles = tiles_m * tiles_n;
  const int total_items = total_tiles * splits;
  const int per_xcd = (total_items + 7) / 8;
  const int xcd_first = (int)(blockIdx.x % 8) * per_xcd;
  const int xcd_step = (int)gridDim.x / 8;
  auto decode = [&](int pos, int& m0, int& n0, int& kb, int& ke, int& split) {
    const int item = xcd_first + pos;
    split = item / total_tiles;
    const int id = item % total_tiles;
    constexpr int BAND = 8;
    const int band_sz = BAND * tiles_n;
    const int first_m = (id / band_sz) * BAND;
    const int rows_in_band = min(tiles_m - first_m, BAND);
    m0 = (first_m + (id % band_sz) % rows_in_band) * BM;
    n0 = ((id % band_sz) / rows_in_band) * BN;
    kb = split * k_per_split;
    ke = min(K, kb + k_per_split);
  };
  auto valid = [&](int pos) { return pos < per_xcd && xcd_first + pos < total_items; };

  // ---- global side of the direct loads.  A wavefront moves CH 1-KiB pieces per operand and
  // k-tile; piece i of wavefront w is rows 32w + 8i .. +7 of a k-contiguous tile (eight
  // 16-byte pieces per 128-byte row) or k-rows 8w + 2i, +1 of a strided one (32 pieces per
  // 512-byte k-row).  The lane at LDS piece p of a row fetches global piece p ^ swizzle(row):
  //   k-contiguous: swizzle = (row / 2) % 8     strided: swizzle = (k % 4) * 4
  // Both depend on i only through its parity, so two column offsets per lane suffice.
  // (a wavefront whose share of a k-contiguous B tile is a single piece of eight rows, BN / WAVES = 8, starts on an
  // odd or even piece depending on its number: B_ODD0 below)
  static_assert((BM / WAVES) % 16 == 0 && ((BN / WAVES) % 16 == 0 || (BN / WAVES == 8 && B_KC)) && (BK / WAVES) % 4 == 0,
                "swizzle parity per piece");
  const int B_ODD0 = (B_KC && (BN / WAVES) % 16 != 0) ? (wave & 1) : 0;
  const int a_row = A_KC ? wave * (BM / WAVES) + (lane >> 3) : wave * (BK / WAVES) + (lane >> 5);
  const int b_row = B_KC ? wave * (BN / WAVES) + (lane >> 3) : wave * (BK / WAVES) + (lane >> 5);
  // byte offset of each of this lane's pieces from the tile's first element; a tile is then a uniform
  // base address (scalar registers) plus these, and issuing it costs no vector arithmetic
  unsigned a_off[CH_A], b_off[CH_B];
#pragma unroll
  for (int i = 0; i < (CH_A > CH_B ? CH_A : CH_B); ++i) {
    const int odd = i & 1, odd_b = (i + B_ODD0) & 1;
    const int kc_col = ((lane & 7) ^ ((4 * odd + (lane >> 4)) & 7)) * 8;
    const int kc_col_b = ((lane & 7) ^ ((4 * odd_b + (lane >> 4)) & 7)) * 8;
    const int st_col = ((lane & 31) ^ ((2 * odd + (lane >> 5)) << 2)) * 8;
    if (i < CH_A) a_off[i] = (unsigned)(((size_t)(a_row + i * (A_KC ? 8 : 2)) * lda + (A_KC ? kc_col : st_col)) * sizeof(bf16_t));
    if (i < CH_B) b_off[i] = (unsigned)(((size_t)(b_row + i * (B_KC ? 8 : 2)) * ldb + (B_KC ? kc_col_b : st_col)) * sizeof(bf16_t));
  }
  // element offset of an item's k-tile 0 (the same in every lane)
  auto a_origin = [&](int m0, int kb) { return A_KC ? (size_t)m0 * lda + kb : (size_t)kb * lda + m0; };
  auto b_origin = [&](int n0, int kb) { return B_KC ? (size_t)n0 * ldb + kb : (size_t)kb * ldb + n0; };
  // EDGE: where piece i of this lane lies inside a tile: (row of the operand, k) for a k-contiguous tile,
  // (k, first of its eight rows) for a strided one; `rows` is how many rows the operand has from the tile's
  // first row on, `ks` how many k are left from the tile's first k on
  auto piece_inside = [&](bool kc, int rowbase, int i, int rows, int ks, int odd0 = 0) {
    const int odd = (i + odd0) & 1;
    if (kc) {
      const int r = rowbase + i * 8, k = ((lane & 7) ^ ((4 * odd + (lane >> 4)) & 7)) * 8;
      return r < rows && k < ks;
    }
    const int k = rowbase + i * 2, r = ((lane & 31) ^ ((2 * odd + (lane >> 5)) << 2)) * 8;
    return r < rows && k < ks;
  };
  auto fetch_piece = [&](const bf16_t* base, unsigned off, unsigned lds, bool inside) {
    if (!EDGE) {
      load_to_lds16_s(base, off, lds);
    } else if (inside) {
      load_to_lds16_s(base, off, lds);
    } else {
      *(KARMA_LDS(u32x4)*)(uintptr_t)(lds + 16 * lane) = u32x4{0, 0, 0, 0};
    }
  };
  // CONV: where the pixels of this lane's CH_A rows lie, for the item whose tiles are being issued (dec_m0)
  // one register per row: image << 20 | (h0 + CBIAS) << 10 | (w0 + CBIAS), (h0, w0) = top-left input position of
  // the pixel's window (or, transposed, the pixel's own position plus the padding); image 4095 = row outside the matrix
  constexpr int CBIAS = 64;   // keeps the packed coordinates non-negative
  unsigned c_pix[CONV ? CH_A : 1], c_pix_next[CONV ? CH_A : 1];   // of the current item's rows, of the next item's
  const int c_shift = cg.stride == 2 ? 1 : 0;
  auto conv_decode = [&](int m0x, unsigned (&pix)[CONV ? CH_A : 1]) {
    const int grid = cg.Ho * cg.Wo;
#pragma unroll
    for (int i = 0; i < CH_A; ++i) {
      const int row = m0x + a_row + 8 * i;
      const int img = row / grid, rem = row - img * grid;
      const int ho = rem / cg.Wo, wo = rem - ho * cg.Wo;
      const int h0 = cg.transposed ? ho + cg.pad : ho * cg.stride - cg.pad;
      const int w0 = cg.transposed ? wo + cg.pad : wo * cg.stride - cg.pad;
      pix[i] = ((unsigned)(row < M ? img : 4095) << 20) | ((unsigned)(h0 + CBIAS) << 10) | (unsigned)(w0 + CBIAS);
    }
  };
  // m0 / n0: the tile's first row of the operand; k0: the item's first k; kend: its last k + 1 (EDGE only)
  // nxt (CONV): the tile belongs to the next item (whose rows were decoded into c_pix_next)
  auto issue_a = [&](int stage, size_t ao, int t, int m0 = 0, int k0 = 0, int kend = 0, bool nxt = false) {
    const unsigned sa = lds0 + EXTRA + stage * STAGE + wave * (CH_A * 1024);
    if constexpr (CONV == 1) {
#pragma unroll
      for (int i = 0; i < CH_A; ++i) {
        // (tap, channel) of this piece's k; recomputed per piece: a few multiplications against registers held
        // across the MFMA steps
        const int k = k0 + t * BK + ((lane & 7) ^ ((4 * (i & 1) + (lane >> 4)) & 7)) * 8;
        const int tap = (int)__umulhi((unsigned)k, magic_c);
        const int ch = k - tap * cg.C;
        const int r = (int)__umulhi((unsigned)tap, magic_s), sx = tap - r * cg.S;
        const unsigned px = nxt ? c_pix_next[i] : c_pix[i];
        const int img = (int)(px >> 20), h0 = (int)((px >> 10) & 1023u) - CBIAS, w0 = (int)(px & 1023u) - CBIAS;
        int hi, wi;
        bool ok = k < kend && img != 4095;
        if (!cg.transposed) {
          hi = h0 + r;
          wi = w0 + sx;
        } else {
          const int th = h0 - r, tw = w0 - sx;
          ok = ok && th >= 0 && tw >= 0 && !((th | tw) & c_shift);
          hi = th >> c_shift;
          wi = tw >> c_shift;
        }
        ok = ok && (unsigned)hi < (unsigned)cg.H && (unsigned)wi < (unsigned)cg.W;
        const unsigned off = (unsigned)(((img * cg.H + hi) * cg.W + wi) * cg.C + ch) * 2u;
        fetch_piece(A, off, sa + i * 1024, ok);
        __builtin_amdgcn_sched_barrier(0);
      }
      return;
    }
    const bf16_t* pa = A + ao + (A_KC ? (size_t)t * BK : (size_t)t * BK * lda);
#pragma unroll
    for (int i = 0; i < CH_A; ++i)
      fetch_piece(pa, a_off[i], sa + i * 1024, !EDGE || piece_inside(A_KC, a_row, i, M - m0, kend - k0 - t * BK));
  };
  auto issue_b = [&](int stage, size_t bo, int t, int n0 = 0, int k0 = 0, int kend = 0) {
    const unsigned sb = lds0 + EXTRA + stage * STAGE + A_BYTES + wave * (CH_B * 1024);
    if constexpr (CONV == 2) {
      const int grid = cg.Ho * cg.Wo;
#pragma unroll
      for (int i = 0; i < CH_B; ++i) {
        // n = (tap, channel) of this piece's eight columns
        const int n = n0 + ((lane & 31) ^ ((2 * (i & 1) + (lane >> 5)) << 2)) * 8;
        const int tap = (int)__umulhi((unsigned)n, magic_c);
        const int ch = n - tap * cg.C;
        const int r = (int)__umulhi((unsigned)tap, magic_s), sx = tap - r * cg.S;
        // its k-row is one pixel
        const int p = k0 + t * BK + b_row + 2 * i;
        int img = (int)((float)p * inv_grid);
        int rem = p - img * grid;
        if (rem < 0) { --img; rem += grid; }
        if (rem >= grid) { ++img; rem -= grid; }
        const int ho = (int)__umulhi((unsigned)rem, magic_w), wo = rem - ho * cg.Wo;
        const int hi = ho * cg.stride - cg.pad + r, wi = wo * cg.stride - cg.pad + sx;
        const bool ok = p < kend && n < N && (unsigned)hi < (unsigned)cg.H && (unsigned)wi < (unsigned)cg.W;
        const unsigned off = (unsigned)(((img * cg.H + hi) * cg.W + wi) * cg.C + ch) * 2u;
        fetch_piece(B, off, sb + i * 1024, ok);
        __builtin_amdgcn_sched_barrier(0);
      }
      return;
    }
    const bf16_t* pb = B + bo + (B_KC ? (size_t)t * BK : (size_t)t * BK * ldb);
#pragma unroll
    for (int i = 0; i < CH_B; ++i)
      fetch_piece(pb, b_off[i], sb + i * 1024, !EDGE || piece_inside(B_KC, b_row, i, N - n0, kend - k0 - t * BK, B_ODD0));
  };
  auto issue = [&](int stage, size_t ao, size_t bo, int t, int m0 = 0, int n0 = 0, int k0 = 0, int kend = 0, bool nxt = false) {
    issue_a(stage, ao, t, m0, k0, kend, nxt);
    issue_b(stage, bo, t, n0, k0, kend);
  };

  // ---- LDS side: fragment addresses (bytes from the start of the operand's tile).
  // k-contiguous: lane reads 16 bytes: row = block row + lane%32, piece (lane/32 + 2*kk) ^ swizzle.
  // strided: two transposing 8-byte reads (k + 0..3 and k + 4..7); in each group of 16 lanes,
  // lane 4e+q supplies k-row e, columns 4q..4q+3, and receives column (its index in the group),
  // k-rows 0..3: lane group g covers block rows 16*(g%2).. and k offset 8*(g/2).
  const int grp = lane >> 4, e4 = (lane >> 2) & 3, q4 = lane & 3;
  auto frag_base = [&](bool kc, int wrow0, int blk) -> unsigned {
    if (kc) return (unsigned)((wrow0 + blk * 32 + lrow) * (BK * 2));
    const int m = wrow0 + blk * 32 + 16 * (grp & 1) + 4 * q4;
    const int piece = (m >> 3) ^ (e4 << 2);
    return (unsigned)((8 * (grp >> 1) + e4) * (BM * 2) + piece * 16 + (m & 7) * 2);
  };
  const unsigned kc_k0 = (unsigned)(((lane >> 5) ^ ((lrow >> 1) & 7)) * 16);   // piece for kk = 0; kk flips bits 5-6
  unsigned a_fb[TM], b_fb[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_fb[i] = frag_base(A_KC, wm * WTM, i) + (A_KC ? kc_k0 : 0u);
#pragma unroll
  for (int j = 0; j < TN; ++j) b_fb[j] = frag_base(B_KC, wn * WTN, j) + (B_KC ? kc_k0 : 0u);
  bf16x8 af[2][TM], bfr[2][TN];
  auto read_one = [&](bool kc, unsigned tile_lds, unsigned fb, int kk) -> bf16x8 {
    if (kc) return *(const KARMA_LDS(bf16x8)*)(uintptr_t)(tile_lds + (fb ^ (unsigned)(kk << 5)));
    const unsigned at = tile_lds + fb + (unsigned)(kk * 16 * (BM * 2));
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KARMA_LDS(s16x4_t)*)(uintptr_t)at);
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KARMA_LDS(s16x4_t)*)(uintptr_t)(at + 4 * (BM * 2)));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto read_frags = [&](int buf, int stage, int kk) {
    const unsigned ta = lds0 + EXTRA + stage * STAGE, tb = ta + A_BYTES;
    // in the order the MFMAs below want them: (a0, b0), (a0, b1), (a1, ...), ...
#pragma unroll
    for (int x = 0; x < (TM > TN ? TM : TN); ++x) {
      if (x < TN) bfr[buf][x] = read_one(B_KC, tb, b_fb[x], kk);
      if (x < TM) af[buf][x] = read_one(A_KC, ta, a_fb[x], kk);
    }
  };

  int pos = blockIdx.x / 8;
  if (!valid(pos)) return;
  int m0, n0, kb, ke, split;
  decode(pos, m0, n0, kb, ke, split);
  size_t ao = a_origin(m0, kb), bo = b_origin(n0, kb);
  int s0 = 0;   // stage of the current item's first k-tile
  if constexpr (CONV == 1) conv_decode(m0, c_pix);
  issue(s0, ao, bo, 0, m0, n0, kb, ke);

  for (;;) {
    const int KT = EDGE ? (ke - kb + BK - 1) / BK : (ke - kb) / BK;
    // the next item, whose first k-tile is fetched while this one is still computing
    int m0n = 0, n0n = 0, kbn = 0, ken = 0, splitn = 0;
    const bool have_next = valid(pos + xcd_step);
    size_t aon = 0, bon = 0;
    if (have_next) {
      decode(pos + xcd_step, m0n, n0n, kbn, ken, splitn);
      aon = a_origin(m0n, kbn);
      bon = b_origin(n0n, kbn);
      if constexpr (CONV == 1) conv_decode(m0n, c_pix_next);
    }
    lds_barrier_visible();   // the previous item's strip (which overlays stage s0 ^ 1) has been read out by every wavefront
    if (KT > 1) issue(s0 ^ 1, ao, bo, 1, m0, n0, kb, ke);
    else if (have_next) issue(s0 ^ 1, aon, bon, 0, m0n, n0n, kbn, ken, true);
    if (KT > 1 || have_next) wait_vm<LPT>();   // everything older than the loads just issued: tile 0 has landed
    else wait_vm<0>();
    lds_barrier_visible();
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    read_frags(0, s0, 0);
    int st = s0;
    for (int kt = 0; kt < KT; ++kt) {
      const bool more = kt + 1 < KT;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        if (kk + 1 < KSTEPS) read_frags((kk + 1) & 1, st, kk + 1);
        else read_frags(0, st ^ 1, 0);   // the next tile's first step (not used after the item's last tile)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
        // one LDS read in the shadow of each MFMA
#pragma unroll
        for (int r = 0; r < TM + TN; ++r) {
          if (r < TM * TN) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if constexpr (TM * TN > TM + TN) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);
        __builtin_amdgcn_sched_barrier(0);
        if (kk == KSTEPS - 2 && more) {
          // The next k-tile (issued one tile ago) must have landed, for every wavefront; past
          // the barrier nobody reads this stage any more (the last step's fragments were
          // fetched before this step's MFMAs), so the tile after next goes into it at once.
          wait_vm<0>();
          lds_barrier_visible();
          if (kt + 2 < KT) issue_a(st, ao, kt + 2, m0, kb, ke);
          else if (have_next) issue_a(st, aon, 0, m0n, kbn, ken, true);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (kk == KSTEPS - 1 && more) {
          if (kt + 2 < KT) issue_b(st, bo, kt + 2, n0, kb, ke);
          else if (have_next) issue_b(st, bon, 0, n0n, kbn, ken);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      st ^= 1;
    }
    lds_barrier_visible();   // the last tile's reads are done: its stage is free for the strip

    // Epilogue as in the kernel above: accumulators hold the transposed tile; each wavefront
    // parks a 32-row strip in its own fp32 patch of LDS and reads it back row-contiguously.
    float* strip = (float*)(smem + ((st ^ 1) == 0 ? 0 : EXTRA + STAGE)) + wave * 32 * SP;
    constexpr int QPR = WTN / 8;
    constexpr int RPI = 64 / QPR;
    static_assert(QPR >= 4 && 64 % QPR == 0 && RPI % 2 == 0 && 32 % RPI == 0, "strip read-out does not tile");
    const int q = (lane & 3) | (((lane >> 3) % (QPR / 4)) << 2);
    const int rr = ((lane >> 2) & 1) | ((lane / (2 * QPR)) << 1);
    // The output stage's per-element input (the residual, or with ACT 2 the saved pre-activation) is
    // fetched one strip ahead, octet by octet as the previous strip's octets are consumed, so that its
    // latency hides behind a whole strip's trip through LDS at the price of one vector per pass.
    constexpr int PASSES = 32 / RPI;
    const bf16_t* ein = ACT == 2 ? ep.aux : (ep.out_f32 ? nullptr : ep.residual);
    const bool fetch_in = ein != nullptr && splits == 1 && (ep.ldc & 7) == 0;
    const int n = n0 + wn * WTN + q * 8;
    auto fetch = [&](int i, int pass) {
      const int m = m0 + wm * WTM + i * 32 + pass * RPI + rr;
      if (EDGE && (m >= M || n >= N)) return u32x4{0, 0, 0, 0};
      return *(const u32x4*)(ein + (size_t)m * ep.ldc + n);
    };
    u32x4 pre[PASSES];
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) pre[pass] = fetch_in ? fetch(0, pass) : u32x4{0, 0, 0, 0};
    // column sums of this wavefront's part of the tile (the bias gradient of the layer whose input gradient
    // this product is): every octet of a lane lies in the same eight columns
    const bool col_sums = ACT == 2 && ep.colsum != nullptr && splits == 1;
    float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(float4*)(strip + lrow * SP + j * 32 + g * 8 + (lane >> 5) * 4) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
#pragma unroll
      for (int pass = 0; pass < PASSES; ++pass) {
        const int row = pass * RPI + rr;
        const int m = m0 + wm * WTM + i * 32 + row;
        const float4 v = *(const float4*)(strip + row * SP + q * 8);
        const float4 u = *(const float4*)(strip + row * SP + q * 8 + 4);
        const bool inside = !EDGE || (m < M && n < N);
        if (splits > 1) {
          if (inside) {
            float* dst = partial + ((size_t)split * M + m) * N + n;
            *(float4*)dst = v;
            *(float4*)(dst + 4) = u;
          }
        } else {
          const u32x4 cur = pre[pass];
          if (fetch_in && i + 1 < TM) pre[pass] = fetch(i + 1, pass);
          // (rows outside the matrix were multiplied from zeroed operand rows: they add nothing to the column sums)
          if (inside) ep.template octet<ACT>(m, n, 8, v, u, fetch_in, cur, col_sums, cs);
        }
      }
    }
    if (col_sums) {
      // lanes that share a column octet differ in lane bits 2, 4 and 5 (the row they take in a pass)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        cs[e] += __shfl_xor(cs[e], 4, 64);
        cs[e] += __shfl_xor(cs[e], 16, 64);
        cs[e] += __shfl_xor(cs[e], 32, 64);
      }
      if (rr == 0 && (!EDGE || n < N)) {
        float* dst = ep.colsum + ((size_t)(m0 / BM) * WGM + wm) * N + n;
        *(float4*)dst = make_float4(cs[0], cs[1], cs[2], cs[3]);
        *(float4*)(dst + 4) = make_float4(cs[4], cs[5], cs[6], cs[7]);
      }
    }
    if (!have_next) break;
    pos += xcd_step;
    m0 = m0n; n0 = n0n; kb = kbn; ke = ken; split = splitn;
    ao = aon; bo = bon;
    if constexpr (CONV == 1) {
#pragma unroll
      for (int i = 0; i < CH_A; ++i) c_pix[i] = c_pix_next[i];
    }
    s0 = st;
  }
}

// out = sum over splits (ascending) of partial[s], then the epilogue's conversions
__global__ void splitk_reduce_kernel(const float* __restrict__ partial, int splits, size_t mn, GemmEpilogue ep, int N) {
  size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= mn) return;
  const int cnt = (int)min((size_t)4, mn - i);
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s)
    for (int e = 0; e < cnt; ++e) v[e] += partial[(size_t)s * mn + i + e];
  // rows are dense (ldc == N) in the split-k path, so element i is (i / N, i % N)
  for (int e = 0; e < cnt; ++e) {
    const size_t at = i + e;
    float x = v[e];
    if (ep.bias) x += bf2f(ep.bias[at % N]);
    if (ep.out_f32) {
      float* c = (float*)ep.C;
      c[at] = ep.accumulate ? c[at] + x : x;
    } else {
      if (ep.residual) x += bf2f(ep.residual[at]);
      ((bf16_t*)ep.C)[at] = f2bf(x);
    }
  }
}

// The same reduction for many splits of a small result (weight gradients of convolutions:
// a few thousand elements, up to 256 splits): eight slices of threads each add every eighth
// partial in ascending order, then the slices are added in ascending order.  The association
// is fixed, so results are reproducible (it differs from the kernel above, which is used for
// few splits: the choice depends on the split count only).
__global__ __launch_bounds__(256) void splitk_reduce_sliced_kernel(const float* __restrict__ partial, int splits, size_t mn,
                                                                    GemmEpilogue ep, int N) {
  __shared__ float red[8][32][4];
  const int q = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const size_t i = ((size_t)blockIdx.x * 32 + q) * 4;
  const int cnt = i < mn ? (int)min((size_t)4, mn - i) : 0;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = slice; s < splits; s += 8)
    for (int e = 0; e < cnt; ++e) v[e] += partial[(size_t)s * mn + i + e];
#pragma unroll
  for (int e = 0; e < 4; ++e) red[slice][q][e] = v[e];
  __syncthreads();
  if (slice != 0 || cnt == 0) return;
  for (int k = 1; k < 8; ++k)
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += red[k][q][e];
  for (int e = 0; e < cnt; ++e) {
    const size_t at = i + e;
    float x = v[e];
    if (ep.bias) x += bf2f(ep.bias[at % N]);
    if (ep.out_f32) {
      float* c = (float*)ep.C;
      c[at] = ep.accumulate ? c[at] + x : x;
    } else {
      if (ep.residual) x += bf2f(ep.residual[at]);
      ((bf16_t*)ep.C)[at] = f2bf(x);
    }
  }
}

static int g_cus = 0;
static int compute_units() {
  if (!g_cus) {
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess) g_cus = p.multiProcessorCount;
    if (g_cus <= 0) g_cus = 256;
  }
  return g_cus;
}

template <int BM, int BN, int BK, int WGM, int WGN, bool EDGE>
static void launch_direct(const GemmArgs& g, hipStream_t s, dim3 grid, dim3 block, int tiles_m, int tiles_n, int splits,
                          int k_per_split, const GemmEpilogue& ep) {
  if constexpr (BM == 256 && BN == 64 && BK == 64 && EDGE) {
    // the narrow tile: a gathered first operand against 64 output channels
    constexpr int STAGE = (BM + BN) * BK * 2, STRIP = WGM * WGN * 32 * (BN / WGN + 4) * 4;
    constexpr int EXTRA = STRIP > STAGE ? STRIP - STAGE : 0;
    const int lds = 2 * STAGE + 2 * EXTRA;
    if (g.conv_mode == 1) {
      const unsigned magic_c = (unsigned)((1ull << 32) / (unsigned)g.conv.C + 1), magic_s = (unsigned)((1ull << 32) / (unsigned)g.conv.S + 1);
      auto kern = gemm_bf16_dl_kernel<BM, BN, BK, WGM, WGN, true, true, 0, true, 1>;
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      hipLaunchKernelGGL(kern, grid, block, lds, s, g.A, g.B, g.M, g.N, g.K, g.lda, g.ldb, tiles_m, tiles_n, splits,
                         k_per_split, ep, (float*)g.ws, g.conv, magic_c, magic_s, 0u, 0.f);
    }
  }
  if constexpr (BM == 256 && BN == 256 && BK == 64) {
    constexpr int STAGE = (BM + BN) * BK * 2, STRIP = WGM * WGN * 32 * (BN / WGN + 4) * 4;
    constexpr int EXTRA = STRIP > STAGE ? STRIP - STAGE : 0;
    const int lds = 2 * STAGE + 2 * EXTRA;
#define KARMA_DL_LAUNCH(AK, BKC, ACT)                                                                             \
  do {                                                                                                            \
    auto kern = gemm_bf16_dl_kernel<BM, BN, BK, WGM, WGN, AK, BKC, ACT, EDGE>;                                    \
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);                \
    hipLaunchKernelGGL(kern, grid, block, lds, s, g.A, g.B, g.M, g.N, g.K, g.lda, g.ldb, tiles_m, tiles_n, splits, \
                       k_per_split, ep, (float*)g.ws, g.conv, 0u, 0u, 0u, 0.f);                                   \
  } while (0)
    if (g.conv_mode) {
      if constexpr (EDGE) {
        const unsigned magic_c = (unsigned)((1ull << 32) / (unsigned)g.conv.C + 1), magic_s = (unsigned)((1ull << 32) / (unsigned)g.conv.S + 1);
        const unsigned magic_w = (unsigned)((1ull << 32) / (unsigned)g.conv.Wo + 1);
        const float inv_grid = 1.0f / (float)(g.conv.Ho * g.conv.Wo);
        if (g.conv_mode == 1) {
          auto kern = gemm_bf16_dl_kernel<BM, BN, BK, WGM, WGN, true, true, 0, true, 1>;
          (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
          hipLaunchKernelGGL(kern, grid, block, lds, s, g.A, g.B, g.M, g.N, g.K, g.lda, g.ldb, tiles_m, tiles_n, splits,
                             k_per_split, ep, (float*)g.ws, g.conv, magic_c, magic_s, magic_w, inv_grid);
        } else {
          auto kern = gemm_bf16_dl_kernel<BM, BN, BK, WGM, WGN, false, false, 0, true, 2>;
          (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
          hipLaunchKernelGGL(kern, grid, block, lds, s, g.A, g.B, g.M, g.N, g.K, g.lda, g.ldb, tiles_m, tiles_n, splits,
                             k_per_split, ep, (float*)g.ws, g.conv, magic_c, magic_s, magic_w, inv_grid);
        }
      }
    } else if (g.act == 1) KARMA_DL_LAUNCH(true, true, 1);          // the layouts were checked by the caller
    else if (g.act == 2) KARMA_DL_LAUNCH(true, false, 2);
    else if (g.a_kc && g.b_kc) KARMA_DL_LAUNCH(true, true, 0);
    else if (g.a_kc && !g.b_kc) KARMA_DL_LAUNCH(true, false, 0);
    else if (!g.a_kc && g.b_kc) KARMA_DL_LAUNCH(false, true, 0);
    else KARMA_DL_LAUNCH(false, false, 0);
#undef KARMA_DL_LAUNCH
  }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool CONVS = false>
static int launch_cfg(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const int tiles = tiles_m * tiles_n;
  // workgroups that run at once: the small tile leaves LDS and registers for two per compute unit
  const int cus = compute_units() * ((BM <= 128 && BN <= 128) || (BM == 256 && BN == 64) ? 2 : 1);
  // split the reduction when the tiles alone cannot fill the chip (weight gradients:
  // small M x N, K = tokens); partial sums are reduced in a fixed order afterwards
  int splits = 1;
  if (g.ws && g.ldc == g.N && tiles < cus && !g.act) {
    // the split count that best fills whole rounds of the chip, fewer splits preferred: every
    // split writes and re-reads an M x N fp32 partial, which is weighed against the operand
    // bytes of the whole product (a skinny weight gradient with a very long reduction takes
    // hundreds of splits, a square one a handful)
    const int max_splits = std::min(256, std::max(1, g.K / (4 * BK)));
    const double per_split = std::min(0.01, 0.5 * (8.0 * g.M * g.N) / (2.0 * ((double)g.M + g.N) * g.K));
    double best = -1.0;
    for (int sp = 1; sp <= max_splits; ++sp) {
      if (sp > 1 && (size_t)sp * g.M * g.N * sizeof(float) > g.ws_bytes) break;
      const int items = tiles * sp, rounds = (items + cus - 1) / cus;
      const double score = (double)items / ((double)rounds * cus) - per_split * sp;
      if (score > best) { best = score; splits = sp; }
    }
  }
  int k_per_split = (g.K + splits - 1) / splits;
  k_per_split = (k_per_split + BK - 1) / BK * BK;
  splits = (g.K + k_per_split - 1) / k_per_split;
  const size_t lds = (size_t)2 * (BM + BN) * (BK + LDS_PAD) * sizeof(bf16_t);
  GemmEpilogue ep{g.C, g.bias, g.residual, g.ldc, g.out_f32, g.accumulate, (bf16_t*)g.aux, nullptr};
  // a multiple of 8 workgroups: the kernel deals work items out per XCD
  dim3 grid(std::min((tiles * splits + 7) / 8 * 8, std::max(8, cus / 8 * 8))), block(WGM * WGN * 64);
#define KARMA_GEMM_LAUNCH(AK, BKC, CV, ACT)                                                                 \
  do {                                                                                                  \
    auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, AK, BKC, CV, ACT>;                               \
    if (lds > 64 * 1024) (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
    hipLaunchKernelGGL(kern, grid, block, lds, s, g.A, g.B, g.M, g.N, g.K, g.lda, g.ldb, tiles_m, tiles_n, splits,  \
                       k_per_split, ep, (float*)g.ws, g.conv);                                          \
  } while (0)
  // whole tiles, 16-byte aligned rows: the direct-to-LDS kernel
  bool direct = false, whole = false;
  if constexpr (CONVS && BM == 256) {
    // a gathered first operand through the direct-to-LDS kernel (eligibility was checked by the caller)
    launch_direct<BM, BN, BK, WGM, WGN, true>(g, s, grid, block, tiles_m, tiles_n, splits, k_per_split, ep);
  } else {
  if (!CONVS && BM == 256 && BN == 256 && BK == 64 && WGM == 2 && WGN == 4) {
    // (a lane's piece offsets inside a tile are kept as 32-bit byte counts)
    direct = g.M % 8 == 0 && g.N % 8 == 0 && g.K % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
             ((uintptr_t)g.A % 16) == 0 && ((uintptr_t)g.B % 16) == 0 && g.ldc % 8 == 0 &&
             (uint64_t)g.lda * 2 * 256 < (1ull << 31) && (uint64_t)g.ldb * 2 * 256 < (1ull << 31) &&
             // tiles that hang over the matrix pay for a whole tile: worth it when most of the work lies inside
             g.M >= BM && g.N >= BN && g.K >= 2 * BK;
    whole = g.M % BM == 0 && g.N % BN == 0 && g.K % BK == 0;
  }
  if (direct) {
    if (g.act == 2 && g.colsum_partial && splits == 1 && g.ldc == g.N) {
      ep.colsum = g.colsum_partial;
      if (g.colsum_rows) *g.colsum_rows = tiles_m * WGM;
    }
    if (whole) launch_direct<BM, BN, BK, WGM, WGN, false>(g, s, grid, block, tiles_m, tiles_n, splits, k_per_split, ep);
    else launch_direct<BM, BN, BK, WGM, WGN, true>(g, s, grid, block, tiles_m, tiles_n, splits, k_per_split, ep);
  } else if (CONVS) {   // the convolution variants exist for one tile shape only
    if (g.conv_mode == 1) KARMA_GEMM_LAUNCH(true, true, (CONVS ? 1 : 0), 0);
    else KARMA_GEMM_LAUNCH(false, false, (CONVS ? 2 : 0), 0);
  } else if (g.act == 1) KARMA_GEMM_LAUNCH(true, true, 0, 1);
  else if (g.act == 2) KARMA_GEMM_LAUNCH(true, false, 0, 2);
  else if (g.a_kc && g.b_kc) KARMA_GEMM_LAUNCH(true, true, 0, 0);
  else if (g.a_kc && !g.b_kc) KARMA_GEMM_LAUNCH(true, false, 0, 0);
  else if (!g.a_kc && g.b_kc) KARMA_GEMM_LAUNCH(false, true, 0, 0);
  else KARMA_GEMM_LAUNCH(false, false, 0, 0);
  }
#undef KARMA_GEMM_LAUNCH
  if (splits > 1) {
    const size_t mn = (size_t)g.M * g.N;
    if (splits >= 16)
      hipLaunchKernelGGL(splitk_reduce_sliced_kernel, dim3((unsigned)((mn / 4 + 31) / 32 + 1)), dim3(256), 0, s,
                         (const float*)g.ws, splits, mn, ep, g.N);
    else
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((mn / 4 + 255) / 256 + 1)), dim3(256), 0, s,
                         (const float*)g.ws, splits, mn, ep, g.N);
  }
  return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP;
}

thread_local GemmTimer* g_gemm_timer = nullptr;

static int gemm_bf16_launch(const GemmArgs& g, hipStream_t s);

int gemm_bf16(const GemmArgs& g, hipStream_t s) {
  GemmTimer* t = g_gemm_timer;
  if (!t) return gemm_bf16_launch(g, s);
  if (t->stride > 1 && (t->seq++ % t->stride) != t->phase % t->stride) return gemm_bf16_launch(g, s);
  while (t->events->size() < *t->used + 2) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return KARMA_E_HIP;
    t->events->push_back(e);
  }
  if (hipEventRecord((*t->events)[*t->used], s) != hipSuccess) return KARMA_E_HIP;
  const int st = gemm_bf16_launch(g, s);
  if (hipEventRecord((*t->events)[*t->used + 1], s) != hipSuccess) return KARMA_E_HIP;
  *t->used += 2;
  t->flops->push_back(2.0 * g.M * g.N * g.K);
  return st;
}

static int gemm_bf16_launch(const GemmArgs& g, hipStream_t s) {
  if (!g.A || !g.B || !g.C || g.M <= 0 || g.N <= 0 || g.K <= 0) return KARMA_E_INVAL;
  // 16-byte k-runs (k-contiguous) or 8-byte row runs (strided) must stay aligned and whole
  if ((g.a_kc || g.b_kc) && g.K % 8) return KARMA_E_INVAL;   // strided operands take any K: every k-row is bounds-checked
  if (g.conv_mode != 1 && (g.a_kc ? (g.lda % 8) : (g.lda % 4 || g.M % 4))) return KARMA_E_INVAL;
  if (g.conv_mode != 2 && (g.b_kc ? (g.ldb % 8) : (g.ldb % 4 || g.N % 4))) return KARMA_E_INVAL;
  if (g.conv_mode < 0 || g.conv_mode > 2) return KARMA_E_INVAL;
  if (g.accumulate && !g.out_f32) return KARMA_E_INVAL;
  if (g.act < 0 || g.act > 2 || (g.act && (!g.aux || g.out_f32 || g.residual || g.conv_mode))) return KARMA_E_INVAL;
  // the fused forms exist for the layouts of the feed-forward layer: forward x W1^T (both operands
  // k-contiguous), backward dy W2 (second operand strided)
  if ((g.act == 1 && !(g.a_kc && g.b_kc)) || (g.act == 2 && !(g.a_kc && !g.b_kc))) return KARMA_E_INVAL;
  if (g.residual && g.out_f32) return KARMA_E_INVAL;
  if (g.conv_mode) {
    const ConvGather& cg = g.conv;
    if (g.conv_mode == 1 ? !(g.a_kc && g.b_kc) : (g.a_kc || g.b_kc)) return KARMA_E_INVAL;
    if (cg.C % 8 || cg.H <= 0 || cg.W <= 0 || cg.Ho <= 0 || cg.Wo <= 0 || cg.R <= 0 || cg.S <= 0 || cg.stride <= 0 || cg.pad < 0)
      return KARMA_E_INVAL;
    // the gathered operand's index ranges must be what the convolution spans
    const long pixels = (long)cg.Ho * cg.Wo, taps_c = (long)cg.R * cg.S * cg.C;
    if (g.conv_mode == 1 ? (g.M % pixels || g.K != taps_c) : (g.K % pixels || g.N != taps_c)) return KARMA_E_INVAL;
    // Large products with a gathered first operand (forward and input gradient) take the direct-to-LDS kernel
    // with its 256 x 256 tile: worth it from 128 output channels on (below that most of the tile is empty).
    // Its piece offsets are 32-bit byte counts and its index arithmetic assumes strides 1 and 2.
    const uint64_t gathered_bytes = (uint64_t)(g.M / pixels) * cg.H * cg.W * cg.C * 2;
    const long tiles256 = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);   // enough of the large tiles to fill the chip
    if (g.conv_mode == 1 && g.N >= 128 && tiles256 >= 192 && g.K >= 128 && g.N % 8 == 0 && g.ldc % 8 == 0 && cg.stride <= 2 &&
        cg.H * cg.stride + cg.pad + 64 < 1024 && cg.W * cg.stride + cg.pad + 64 < 1024 && cg.Ho + cg.pad + 64 < 1024 &&
        cg.Wo + cg.pad + 64 < 1024 && g.M / pixels < 4095 && gathered_bytes < (1ull << 32) && (uint64_t)g.K * cg.C < (1ull << 31) &&
        ((uintptr_t)g.A % 16) == 0 && ((uintptr_t)g.B % 16) == 0 && (uint64_t)g.ldb * 2 * 256 < (1ull << 31))
      return launch_cfg<256, 256, 64, 2, 4, true>(g, s);
    // The same with 64 output channels (the first stage of the bottleneck network, the full-resolution level of the
    // fully convolutional one): a 256 x 64 tile, eight wavefronts of 64 x 32, two workgroups per compute unit (a
    // k-tile of this shape carries 16 MFMAs per wavefront, less than its loads' round trip: the second workgroup
    // multiplies while the first one waits)
    if (g.conv_mode == 1 && g.N == 64 && (g.M + 255) / 256 >= 384 && g.K >= 128 && g.ldc % 8 == 0 && cg.stride <= 2 &&
        cg.H * cg.stride + cg.pad + 64 < 1024 && cg.W * cg.stride + cg.pad + 64 < 1024 && cg.Ho + cg.pad + 64 < 1024 &&
        cg.Wo + cg.pad + 64 < 1024 && g.M / pixels < 4095 && gathered_bytes < (1ull << 32) && (uint64_t)g.K * cg.C < (1ull << 31) &&
        ((uintptr_t)g.A % 16) == 0 && ((uintptr_t)g.B % 16) == 0 && (uint64_t)g.ldb * 2 * 256 < (1ull << 31))
      return launch_cfg<256, 64, 64, 4, 2, true>(g, s);
    // The weight gradient (second operand gathered, reduction over the pixels): few output tiles and a very long
    // reduction, which the split fills the chip with; worth the large tile from 64 x 512 results on (with 64 output
    // channels three quarters of the tile's rows are zeros, and it is still faster than the small tile's gather).
    // (pixels * Wo < 2^32: the reciprocal multiplication by magic_w = 2^32 / Wo + 1 is exact for every n with
    // n * (magic_w * Wo - 2^32) < 2^32, and that excess is at most Wo)
    if (g.conv_mode == 2 && g.M >= 64 && g.N >= 512 && g.K >= 4096 && g.M % 8 == 0 && g.lda % 8 == 0 && g.ldc % 8 == 0 &&
        g.ws != nullptr && cg.H * cg.stride + cg.pad + 64 < 1024 && cg.W * cg.stride + cg.pad + 64 < 1024 &&
        (uint64_t)(g.K / pixels) * cg.H * cg.W * cg.C * 2 < (1ull << 32) && (uint64_t)g.N * cg.C < (1ull << 31) &&
        (uint64_t)pixels * cg.Wo < (1ull << 32) && g.K < (1 << 24) && ((uintptr_t)g.A % 16) == 0 && ((uintptr_t)g.B % 16) == 0 &&
        (uint64_t)g.lda * 2 * 256 < (1ull << 31))
      return launch_cfg<256, 256, 64, 2, 4, true>(g, s);
    return launch_cfg<128, 128, 64, 2, 2, true>(g, s);
  }
  if (g.M > 128 && g.N > 128) return launch_cfg<256, 256, 64, 2, 4>(g, s);
  return launch_cfg<128, 128, 64, 2, 2>(g, s);
}

}  // namespace karma

using namespace karma;

extern "C" int karma_k_gemm_gelu_bf16(const void* a, const void* b, void* c, const void* bias, void* aux, uint32_t m,
                                      uint32_t n, uint32_t k, uint32_t flags, uint32_t mode, void* stream) {
  if (mode != KARMA_GEMM_GELU_FWD && mode != KARMA_GEMM_GELU_BWD) return KARMA_E_INVAL;
  if (flags & (KARMA_GEMM_OUT_F32 | KARMA_GEMM_ACCUMULATE)) return KARMA_E_INVAL;
  GemmArgs g{};
  g.A = (const bf16_t*)a;
  g.B = (const bf16_t*)b;
  g.C = c;
  g.bias = (const bf16_t*)bias;
  g.M = (int)m; g.N = (int)n; g.K = (int)k;
  g.a_kc = !(flags & KARMA_GEMM_A_STRIDED);
  g.b_kc = !(flags & KARMA_GEMM_B_STRIDED);
  g.lda = g.a_kc ? (int)k : (int)m;
  g.ldb = g.b_kc ? (int)k : (int)n;
  g.ldc = (int)n;
  g.act = (int)mode;
  g.aux = aux;
  return gemm_bf16(g, (hipStream_t)stream);
}

// The backward product with GELU' and the column sums of its result (fused where the shape allows)
extern "C" int karma_k_gemm_gelu_bwd_colsum_bf16(const void* a, const void* b, void* c, const void* aux, float* colsum_out,
                                                 float* ws, uint64_t ws_bytes, uint32_t m, uint32_t n, uint32_t k,
                                                 void* stream) {
  if (!a || !b || !c || !aux || !colsum_out || !ws) return KARMA_E_INVAL;
  if (ws_bytes < colsum_ws_bytes((int)m, (int)n)) return KARMA_E_OOM;
  GemmArgs g{};
  g.A = (const bf16_t*)a;
  g.B = (const bf16_t*)b;
  g.C = c;
  g.M = (int)m; g.N = (int)n; g.K = (int)k;
  g.a_kc = true;
  g.b_kc = false;
  g.lda = (int)k;
  g.ldb = (int)n;
  g.ldc = (int)n;
  g.act = 2;
  g.aux = const_cast<void*>(aux);
  int rows = 0;
  g.colsum_partial = ws;
  g.colsum_rows = &rows;
  int st = gemm_bf16(g, (hipStream_t)stream);
  if (st) return st;
  if (rows) return colsum_finish(ws, rows, (int)n, colsum_out, (hipStream_t)stream);
  return colsum_bf16((const bf16_t*)c, colsum_out, ws, (int)m, (int)n, (hipStream_t)stream);
}

extern "C" int karma_k_gemm_bf16(const void* a, const void* b, void* c, const void* bias, const void* residual,
                                 uint32_t m, uint32_t n, uint32_t k, uint32_t flags, void* ws, uint64_t ws_bytes,
                                 void* stream) {
  GemmArgs g{};
  g.A = (const bf16_t*)a;
  g.B = (const bf16_t*)b;
  g.C = c;
  g.bias = (const bf16_t*)bias;
  g.residual = (const bf16_t*)residual;
  g.M = (int)m; g.N = (int)n; g.K = (int)k;
  g.a_kc = !(flags & KARMA_GEMM_A_STRIDED);
  g.b_kc = !(flags & KARMA_GEMM_B_STRIDED);
  g.lda = g.a_kc ? (int)k : (int)m;
  g.ldb = g.b_kc ? (int)k : (int)n;
  g.ldc = (int)n;
  g.out_f32 = (flags & KARMA_GEMM_OUT_F32) != 0;
  g.accumulate = (flags & KARMA_GEMM_ACCUMULATE) != 0;
  g.ws = ws;
  g.ws_bytes = ws ? (size_t)ws_bytes : 0;
  return gemm_bf16(g, (hipStream_t)stream);
}

// ---- the product for callers that cannot allocate -------------------------------------------
// The split-reduction workspace lives in a file-scope device array instead of a caller's buffer.
// In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device (each GPU holds its own copy at its own address).
namespace {
constexpr size_t STATIC_WS_BYTES = KARMA_GEMM_STATIC_WS_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_WS_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device, or nullptr (HIP error).
void* static_ws() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int karma_k_gemm_bf16_static_ws(const void* a, const void* b, void* c, const void* bias, const void* residual,
                                           uint32_t m, uint32_t n, uint32_t k, uint32_t flags, void* stream) {
  // two partial results must fit, or the workspace could not serve any split
  if ((uint64_t)m * n * sizeof(float) * 2 > STATIC_WS_BYTES) return KARMA_E_OOM;
  void* ws = static_ws();
  if (!ws) return KARMA_E_HIP;
  return karma_k_gemm_bf16(a, b, c, bias, residual, m, n, k, flags, ws, STATIC_WS_BYTES, stream);
}
