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

#include <algorithm>
#include <type_traits>

#include "karma.h"
#include "device_utils.h"
#include "kernels.h"

namespace karma {

constexpr float LOG2E = 1.4426950408889634f;

// Tile sizes of the head-dimension-64 kernels, from a sweep on 32 x 16 heads x 1024 x 64 (times of
// forward / dQ+dK/dV passes): forward 128, 64, 32 keys per tile: 143, 121, 139 us; dQ 128 -> 64 keys:
// -40 us; dK/dV 128, 64, 32 queries: 0, 0, -25 us.  Smaller tiles need fewer registers per
// wavefront and let the two workgroups of a compute unit drift apart, so that one's MFMAs overlap
// the other's exponentials; below these sizes the barrier per tile costs more than that gains.
constexpr int ATTN_FWD_KT = 64, ATTN_DQ_KT = 64, ATTN_DKV_QT = 32;

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

// Eight elements of a row starting at column col, zeros where the row (D columns) has ended
template <int D>
__device__ __forceinline__ bf16x8 row_frag(const bf16_t* row, int col) {
  Frag f;
  if (col < D) f.u = *(const u32x4*)(row + col);
  else f.u = u32x4{0, 0, 0, 0};
  return f.v;
}
// Threads that run a transposing TileMover over a [ROWS][COLS] tile: it hands out whole patches of
// 4 rows x 8 columns, so the thread count has to divide their number.
template <int ROWS, int COLS>
constexpr int transposer_threads() {
  constexpr int patches = ROWS * COLS / 32;
  return patches % 256 == 0 ? 256 : patches < 256 ? patches : patches % 160 == 0 ? 160 : 64;
}

// Sum over the 32 lanes of each half-wavefront, left in every lane: four data-parallel-primitive steps inside
// the rows of 16 lanes (swap neighbours, swap pairs, mirror the half row, mirror the row), one exchange across rows.
__device__ __forceinline__ float half_wave_sum(float v) {
  auto dpp_add = [](float x, auto ctrl) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, false);
    return x + __int_as_float(y);
  };
  v = dpp_add(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1, 0, 3, 2]
  v = dpp_add(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2, 3, 0, 1]
  v = dpp_add(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v = dpp_add(v, std::integral_constant<int, 0x140>{});   // row_mirror
  return v + __shfl_xor(v, 16, 64);
}

// ------------------------------------------------------------------------------- forward
// grid (seq/128, heads, batch), 256 threads; wavefront w owns queries q0+32w .. q0+32w+31
// and walks the keys in tiles of 128 (64 for head dimensions above 128) made of 32-key sub-tiles (those entirely after the
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

// Head dimensions that are no multiple of 32 (D = 152) run with the tiles padded to DP columns:
// the movers fill columns D..DP-1 with zeros, so the padded part of Q, K, V and dO adds nothing to
// any product, and the results' padded columns are not stored.
template <int D, int DP>
__global__ __launch_bounds__(256, (DP == 64 ? 2 : 1)) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                        float* __restrict__ lse, int S, int H) {
  constexpr int KT = DP > 128 ? 64 : 128;   // keys per tile (the score tiles of one step stay in registers)
  constexpr int NMT = KT / 32;
  constexpr bool EXACT = D == DP;
  constexpr int TV = transposer_threads<DP, KT>();
  constexpr int PK = DP + LDS_PAD, PV = KT + LDS_PAD;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[KT * PK];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DP * PV];
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

  bf16x8 qf[DP / 16];
#pragma unroll
  for (int ks = 0; ks < DP / 16; ++ks) qf[ks] = row_frag<D>(Qg + (size_t)query * ld, ks * 16 + g * 8);
  f32x16 o[DP / 32];
#pragma unroll
  for (int i = 0; i < DP / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;   // m: running maximum of the raw scores (before the 1/sqrt(d) scale)

  TileMover<KT, DP, 256, true> mk;
  TileMover<DP, KT, TV, false> mv;
  const int n_kt = (q0 + 128) / KT;
  mk.load(Kg, ld, 0, 0, S, D, tid, EXACT);
  if (tid < TV) mv.load(Vg, ld, 0, 0, D, S, tid, EXACT);
  for (int kt = 0; kt < n_kt; ++kt) {
    const int key0 = kt * KT;
    __syncthreads();   // previous tile fully consumed
    mk.store(Ks, tid);
    if (tid < TV) mv.store(Vt, tid);
    __syncthreads();
    if (kt + 1 < n_kt) {   // next tile's loads stay in flight while this one is computed
      mk.load(Kg, ld, key0 + KT, 0, S, D, tid, EXACT);
      if (tid < TV) mv.load(Vg, ld, 0, key0 + KT, D, S, tid, EXACT);
    }
    // sub-tiles this wavefront needs: keys key0 + 32*mt <= last query
    const int n_mt = min(NMT, (qbase + 31 - key0) / 32 + 1);
    f32x16 s[NMT];
    float tmax = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      if (mt < n_mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < DP / 16; ++ks) {
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
      for (int i = 0; i < DP / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
      m = m_new;
    }
    float psum = 0.f;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
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
          for (int i = 0; i < DP / 32; ++i) {
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
  for (int i = 0; i < DP / 32; ++i)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      u32x2 v;
      v.x = pack2(o[i][rg * 4 + 0] * inv, o[i][rg * 4 + 1] * inv);
      v.y = pack2(o[i][rg * 4 + 2] * inv, o[i][rg * 4 + 3] * inv);
      if (EXACT || i * 32 + rg * 8 + g * 4 < D) *(u32x2*)(out + i * 32 + rg * 8 + g * 4) = v;
    }
  if (g == 0) lse[((size_t)b * H + head) * S + query] = m * c + log2f(l);
}

// ---------------------------------------------------------- head dimension 64: direct loads
// The kernels below (D = 64) keep every operand tile as it lies in memory, [rows][64] with
// 128-byte rows, fetched straight into LDS by global_load_lds_dwordx4 (two stages, one
// barrier per tile) and read either by rows (ds_read_b128: the operand whose reduction index
// is the head dimension) or transposed (ds_read_b64_tr_b16: the operand whose reduction index
// is the tile's row index), so no tile is loaded twice or transposed in registers.
// 16-byte piece p of row r is stored at piece p ^ swz64(r): row reads (16 consecutive rows,
// one piece) and transposing reads (4 rows x 4 pieces) are both free of bank conflicts.
__device__ __forceinline__ int swz64(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }

// Direct loads of a [ROWS][64] tile (row pitch ld elements in memory) by WAVES wavefronts: the
// per-lane byte offsets (row, swizzled piece) are computed once, a tile is then a uniform base
// pointer plus those offsets.
template <int ROWS, int WAVES>
struct TileLoader64 {
  static constexpr int CH = ROWS / 8 / WAVES;   // 1 KiB pieces (8 rows) per wavefront
  static_assert(CH >= 1 && ROWS % (8 * WAVES) == 0, "tile does not divide over the wavefronts");
  unsigned off[CH];
  __device__ __forceinline__ void init(size_t ld, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int row = 8 * (wave * CH + i) + (lane >> 3);
      off[i] = (unsigned)(((size_t)row * ld + (size_t)(((lane & 7) ^ swz64(row)) * 8)) * sizeof(bf16_t));
    }
  }
  // tile: address of the tile's first row (the same in every lane); lds: byte address of the tile in LDS
  __device__ __forceinline__ void issue(const bf16_t* tile, unsigned lds, int wave) const {
#pragma unroll
    for (int i = 0; i < CH; ++i) load_to_lds16_s(tile, off[i], lds + (wave * CH + i) * 1024);
  }
};

// per-lane address parts of the two fragment kinds
struct Frag64 {
  unsigned row_off;      // row read: lane%32 * 128
  unsigned ko[4];        // row read: byte offset of the lane's piece for k-step ks (d = 16 ks + 8 g ..)
  unsigned tro[2][2];    // transposing read: [32-wide block of the transposed rows][first / second four k]
  __device__ __forceinline__ void init(int lane) {
    const int lrow = lane & 31, g = lane >> 5, grp = lane >> 4, e4 = (lane >> 2) & 3, q4 = lane & 3;
    row_off = (unsigned)(lrow * 128);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ko[ks] = (unsigned)(((2 * ks + g) ^ swz64(lrow)) * 16);
    // the lane supplies (tile row = base + 4 g + 8 h + e4, columns 32 i + 16 (grp % 2) + 4 q4 ..): base is a
    // multiple of 16, so the swizzle of that row is known here
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int f = ((e4 >> 1) << 2) | ((g + 2 * h) & 3);
        const int piece = (4 * i + 2 * (grp & 1) + (q4 >> 1)) ^ f;
        tro[i][h] = (unsigned)((4 * g + 8 * h + e4) * 128 + piece * 16 + (q4 & 1) * 8);
      }
  }
  // rows r0 + lane%32 of the tile, k = d in [16 ks + 8 g, +8)
  __device__ __forceinline__ bf16x8 rows(unsigned tile, int r0, int ks) const {
    return *(const KARMA_LDS(bf16x8)*)(uintptr_t)(tile + (unsigned)(r0 * 128) + row_off + ko[ks]);
  }
  // transposed: MFMA row = column 32 i + lane%32 of the tile, k-slots = tile rows base + 4g + {0..3, 8..11}
  __device__ __forceinline__ bf16x8 cols(unsigned tile, int base, int i) const {
    const unsigned at = tile + (unsigned)(base * 128);
    return read_tr_pair(at + tro[i][0], at + tro[i][1]);
  }
};

template <int KT, int WGS>
__global__ __launch_bounds__(256, WGS) void attn_fwd_dl_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                              float* __restrict__ lse, int S, int H) {
  constexpr int D = 64, NMT = KT / 32, TILE = KT * D * 2, STAGE = 2 * TILE;   // stage = K tile | V tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  const unsigned lds0 = (unsigned)(uintptr_t)((KARMA_LDS(unsigned char)*)smem_attn);
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  int tile, head, b;
  attn_block(tile, head, b, true);
  const int q0 = tile * 128;
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), lrow = lane & 31, g = lane >> 5;
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * D;
  const bf16_t* Kg = base + h;
  const bf16_t* Vg = base + 2 * h;
  const int qbase = q0 + 32 * w, query = qbase + lrow;
  const float c = LOG2E * rsqrtf((float)D);
  Frag64 fr;
  fr.init(lane);

  TileLoader64<KT, 4> tl;
  tl.init(ld, w, lane);
  auto issue = [&](int kt) {
    const unsigned st = lds0 + (kt & 1) * STAGE;
    tl.issue(Kg + (size_t)kt * KT * ld, st, w);
    tl.issue(Vg + (size_t)kt * KT * ld, st + TILE, w);
  };
  const int n_kt = (q0 + 128) / KT;
  issue(0);

  bf16x8 qf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    Frag f;
    f.u = *(const u32x4*)(base + (size_t)query * ld + ks * 16 + g * 8);
    qf[ks] = f.v;
  }
  f32x16 o[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;   // m: running maximum of the raw scores (before the 1/sqrt(d) scale)

  // One 128-key tile.  FULL: every key precedes every query of the workgroup (all tiles but the
  // last): no masking, no skipped sub-tiles, and the four sub-tiles' MFMA chains are independent
  // instruction streams the scheduler can interleave with each other and with the exponentials.
  auto tile_step = [&](int kt, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int key0 = kt * KT;
    wait_vm<0>();            // this wavefront's share of tile kt has landed
    lds_barrier_visible();   // ... and everybody's; tile kt - 1 is no longer read
    if (kt + 1 < n_kt) issue(kt + 1);
    const unsigned Ks = lds0 + (kt & 1) * STAGE, Vs = Ks + TILE;
    // sub-tiles this wavefront needs: keys key0 + 32*mt <= last query
    const int n_mt = FULL ? NMT : min(NMT, (qbase + 31 - key0) / 32 + 1);
    f32x16 s[NMT];
    float tmax = -INFINITY;
    if (FULL) {
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt)
          s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.rows(Ks, mt * 32, ks), qf[ks], s[mt], 0, 0, 0);
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[mt][r]);
    } else {
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt) {
        if (mt < n_mt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
          for (int ks = 0; ks < D / 16; ++ks) s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.rows(Ks, mt * 32, ks), qf[ks], s[mt], 0, 0, 0);
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
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // The reference maximum m follows the true maximum lazily: the accumulators are rescaled only when
    // some query's maximum has grown by more than 2^8 in the exponent's domain; until then its
    // probabilities are computed against the old reference and may reach 256 (harmless in fp32
    // accumulators and in bf16, whose relative precision does not depend on the magnitude).
    const float m_new = fmaxf(m, tmax);
    if (__any((m_new - m) * c > 8.f)) {
      const float alpha = fast_exp2((m - m_new) * c);
      l *= alpha;
#pragma unroll
      for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
      m = m_new;
    }
    const float mc = m * c;
    float psum = 0.f;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      if (FULL || mt < n_mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = fast_exp2(fmaf(s[mt][r], c, -mc));
          s[mt][r] = p;
          psum += p;
        }
        // O^T += V^T P^T: the probabilities' k-slots are keys 16 st + 4 g + {0..3, 8..11}, which is
        // exactly what the transposing read delivers
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 pf = frag_regs(s[mt], st, 1.f);
#pragma unroll
          for (int i = 0; i < D / 32; ++i) o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.cols(Vs, mt * 32 + st * 16, i), pf, o[i], 0, 0, 0);
        }
      }
    }
    l += psum;
  };
  const int n_full = q0 / KT;   // tiles whose keys all precede the workgroup's first query
  for (int kt = 0; kt < n_full; ++kt) tile_step(kt, std::true_type{});
  for (int kt = n_full; kt < n_kt; ++kt) tile_step(kt, std::false_type{});
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
// Same tiling as forward: wavefront owns 32 queries, walks the keys in tiles of 128 (or 64).
template <int D, int DP>
__global__ __launch_bounds__(256, (DP == 64 ? 2 : 1)) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S, int H) {
  constexpr int KT = DP > 128 ? 64 : 128, NMT = KT / 32;
  constexpr bool EXACT = D == DP;
  constexpr int TV = transposer_threads<DP, KT>();
  constexpr int PK = DP + LDS_PAD, PT = KT + LDS_PAD;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  bf16_t* Ks = (bf16_t*)smem_attn;   // [KT][PK]
  bf16_t* Vs = Ks + KT * PK;         // [KT][PK]
  bf16_t* Kt = Vs + KT * PK;         // [DP][PT]  K transposed
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

  bf16x8 qf[DP / 16], dof[DP / 16];
#pragma unroll
  for (int ks = 0; ks < DP / 16; ++ks) {
    qf[ks] = row_frag<D>(base + (size_t)query * ld, ks * 16 + g * 8);
    dof[ks] = row_frag<D>(dout + ((size_t)b * S + query) * h + (size_t)head * D, ks * 16 + g * 8);
  }
  const float my_lse = lse[((size_t)b * H + head) * S + query];
  const float my_delta = delta[((size_t)b * H + head) * S + query];
  f32x16 dq[DP / 32];
#pragma unroll
  for (int i = 0; i < DP / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

  TileMover<KT, DP, 256, true> mk, mv;
  TileMover<DP, KT, TV, false> mkt;
  const int n_kt = (q0 + 128) / KT;
  mk.load(Kg, ld, 0, 0, S, D, tid, EXACT);
  mv.load(Vg, ld, 0, 0, S, D, tid, EXACT);
  if (tid < TV) mkt.load(Kg, ld, 0, 0, D, S, tid, EXACT);
  for (int kt = 0; kt < n_kt; ++kt) {
    const int key0 = kt * KT;
    __syncthreads();
    mk.store(Ks, tid);
    mv.store(Vs, tid);
    if (tid < TV) mkt.store(Kt, tid);
    __syncthreads();
    if (kt + 1 < n_kt) {
      mk.load(Kg, ld, key0 + KT, 0, S, D, tid, EXACT);
      mv.load(Vg, ld, key0 + KT, 0, S, D, tid, EXACT);
      if (tid < TV) mkt.load(Kg, ld, 0, key0 + KT, D, S, tid, EXACT);
    }
    const int n_mt = min(NMT, (qbase + 31 - key0) / 32 + 1);
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      if (mt < n_mt) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < DP / 16; ++ks) {
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
          for (int i = 0; i < DP / 32; ++i) {
            bf16x8 ktf = frag2(Kt + (i * 32 + lrow) * PT + mt * 32 + st * 16 + g * 4);
            dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf, dq[i], 0, 0, 0);
          }
        }
      }
    }
  }
  bf16_t* out = dqkv + ((size_t)b * S + query) * ld + (size_t)head * D;
#pragma unroll
  for (int i = 0; i < DP / 32; ++i)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      u32x2 v;
      v.x = pack2(dq[i][rg * 4 + 0], dq[i][rg * 4 + 1]);
      v.y = pack2(dq[i][rg * 4 + 2], dq[i][rg * 4 + 3]);
      if (EXACT || i * 32 + rg * 8 + g * 4 < D) *(u32x2*)(out + i * 32 + rg * 8 + g * 4) = v;
    }
}

// dQ for head dimension 64 with direct loads: K and V tiles as they lie in memory; K is read by
// rows for the scores and transposed for dQ^T += K^T dS^T.
// It also computes delta[q] = sum_d dO[q][d] O[q][d] for its queries (each lane holds half a row of dO
// as MFMA fragments anyway) and stores it for the dK/dV pass.
template <int KT>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_dl_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                                 const bf16_t* __restrict__ dout, const float* __restrict__ lse,
                                                                 float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S, int H,
                                                                 float* __restrict__ colsum) {
  constexpr int D = 64, NMT = KT / 32, TILE = KT * D * 2, STAGE = 2 * TILE;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  const unsigned lds0 = (unsigned)(uintptr_t)((KARMA_LDS(unsigned char)*)smem_attn);
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  int tile, head, b;
  attn_block(tile, head, b, true);
  const int q0 = tile * 128;
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), lrow = lane & 31, g = lane >> 5;
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * D;
  const bf16_t* Kg = base + h;
  const bf16_t* Vg = base + 2 * h;
  const int qbase = q0 + 32 * w, query = qbase + lrow;
  const float scale = rsqrtf((float)D), c = LOG2E * scale;
  Frag64 fr;
  fr.init(lane);
  TileLoader64<KT, 4> tl;
  tl.init(ld, w, lane);
  auto issue = [&](int kt) {
    const unsigned st = lds0 + (kt & 1) * STAGE;
    tl.issue(Kg + (size_t)kt * KT * ld, st, w);
    tl.issue(Vg + (size_t)kt * KT * ld, st + TILE, w);
  };
  const int n_kt = (q0 + 128) / KT;
  issue(0);

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
  float my_delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    Frag fo, fd;
    fo.u = *(const u32x4*)(o + ((size_t)b * S + query) * h + (size_t)head * D + ks * 16 + g * 8);
    fd.v = dof[ks];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      my_delta = fmaf(__uint_as_float(fo.u[e] << 16), __uint_as_float(fd.u[e] << 16), my_delta);
      my_delta = fmaf(__uint_as_float(fo.u[e] & 0xffff0000u), __uint_as_float(fd.u[e] & 0xffff0000u), my_delta);
    }
  }
  my_delta += __shfl_xor(my_delta, 32, 64);   // the other half of the row
  if (g == 0) delta[((size_t)b * H + head) * S + query] = my_delta;
  f32x16 dq[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

  auto tile_step = [&](int kt, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int key0 = kt * KT;
    wait_vm<0>();
    lds_barrier_visible();
    if (kt + 1 < n_kt) issue(kt + 1);
    const unsigned Ks = lds0 + (kt & 1) * STAGE, Vs = Ks + TILE;
    const int n_mt = FULL ? NMT : min(NMT, (qbase + 31 - key0) / 32 + 1);
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      if (FULL || mt < n_mt) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.rows(Ks, mt * 32, ks), qf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.rows(Vs, mt * 32, ks), dof[ks], dp, 0, 0, 0);
        }
        const bool diag = !FULL && key0 + mt * 32 + 31 > qbase;
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
          for (int i = 0; i < D / 32; ++i) dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.cols(Ks, mt * 32 + st * 16, i), dsf, dq[i], 0, 0, 0);
        }
      }
    }
  };
  const int n_full = q0 / KT;   // tiles whose keys all precede the workgroup's first query
  for (int kt = 0; kt < n_full; ++kt) tile_step(kt, std::true_type{});
  for (int kt = n_full; kt < n_kt; ++kt) tile_step(kt, std::false_type{});

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
  // Column sums of dQ over this wavefront's 32 queries (the gradient of the QKV bias, first third): the
  // queries lie on the lanes of each half-wavefront, so five exchanges per register; one row of partial sums
  // per wavefront, [batch * S / 32][3 h], added up afterwards in a fixed order.
  if (colsum) {
    float* dst = colsum + ((size_t)b * (S / 32) + qbase / 32) * ld + (size_t)head * D;
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        float t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          t[e] = half_wave_sum(dq[i][rg * 4 + e]);
        }
        if (lrow == 0) *(float4*)(dst + i * 32 + rg * 8 + g * 4) = make_float4(t[0], t[1], t[2], t[3]);
      }
  }
}

// ------------------------------------------------------------------ backward: dK, dV
// grid (seq/128, heads, batch); wavefront w owns keys k0+32w .. +31 and loops over the
// query tiles (64 queries, two 32-query sub-tiles) at or after them.  Scores are computed
// with queries on the rows so that the probabilities sit in registers as the (key x query)
// operand of dV = P^T dO and dK = dS^T Q.
template <int D, int DP>
__global__ __launch_bounds__(256, (DP == 64 ? 2 : 1)) void attn_bwd_dkv_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S, int H) {
  constexpr int QT = 64;
  constexpr bool EXACT = D == DP;
  constexpr int TT = transposer_threads<DP, QT>();
  constexpr int PK = DP + LDS_PAD, PT = QT + LDS_PAD;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  bf16_t* Qs = (bf16_t*)smem_attn;   // [QT][PK]
  bf16_t* Os = Qs + QT * PK;         // [QT][PK]   dO
  bf16_t* Qt = Os + QT * PK;         // [DP][PT]   Q transposed
  bf16_t* Ot = Qt + DP * PT;         // [DP][PT]   dO transposed
  float* lse_s = (float*)(Ot + DP * PT);
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

  bf16x8 kf[DP / 16], vf[DP / 16];
#pragma unroll
  for (int ks = 0; ks < DP / 16; ++ks) {
    kf[ks] = row_frag<D>(base + h + (size_t)key * ld, ks * 16 + g * 8);
    vf[ks] = row_frag<D>(base + 2 * h + (size_t)key * ld, ks * 16 + g * 8);
  }
  f32x16 dk[DP / 32], dv[DP / 32];
#pragma unroll
  for (int i = 0; i < DP / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[i][r] = 0.f; dv[i][r] = 0.f; }

  TileMover<QT, DP, 256, true> mq, mo;
  TileMover<DP, QT, TT, false> mqt, mot;
  auto fetch = [&](int qq) {
    mq.load(base, ld, qq, 0, S, D, tid, EXACT);
    mo.load(dOg, (size_t)h, qq, 0, S, D, tid, EXACT);
    if (tid < TT) {
      mqt.load(base, ld, 0, qq, D, S, tid, EXACT);
      mot.load(dOg, (size_t)h, 0, qq, D, S, tid, EXACT);
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
        for (int ks = 0; ks < DP / 16; ++ks) {
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
          for (int i = 0; i < DP / 32; ++i) {
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
  for (int i = 0; i < DP / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kk = kbase + (r >> 2) * 8 + g * 4 + (r & 3);
      bf16_t* row = dqkv + ((size_t)b * S + kk) * ld + (size_t)head * D + i * 32 + lrow;
      if (EXACT || i * 32 + lrow < D) {
        row[h] = f2bf(dk[i][r]);
        row[2 * h] = f2bf(dv[i][r]);
      }
    }
}

// dK, dV for head dimension 64 with direct loads: Q and dO tiles of 128 queries as they lie in
// memory, read by rows for S = Q K^T and dP = dO V^T and transposed for dV += P^T dO, dK += dS^T Q.
template <int QT>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_dl_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                                  const float* __restrict__ lse, const float* __restrict__ delta,
                                                                  bf16_t* __restrict__ dqkv, int S, int H,
                                                                  float* __restrict__ colsum) {
  constexpr int D = 64, TILE = QT * D * 2, STAGE = 2 * TILE;   // stage = Q tile | dO tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];
  const unsigned lds0 = (unsigned)(uintptr_t)((KARMA_LDS(unsigned char)*)smem_attn);
  float* stat = (float*)(smem_attn + 2 * STAGE);   // [2 stages][lse | delta][QT]
  const int h = H * D;
  const size_t ld = 3 * (size_t)h;
  int tile, head, b;
  attn_block(tile, head, b, false);
  const int k0 = tile * 128;
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), lrow = lane & 31, g = lane >> 5;
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * D;
  const bf16_t* dOg = dout + (size_t)b * S * h + (size_t)head * D;
  const float* lse_g = lse + ((size_t)b * H + head) * S;
  const float* delta_g = delta + ((size_t)b * H + head) * S;
  const int kbase = k0 + 32 * w, key = kbase + lrow;
  const float scale = rsqrtf((float)D), c = LOG2E * scale;
  Frag64 fr;
  fr.init(lane);
  TileLoader64<QT, 4> tlq, tlo;   // Q rows lie 3 h apart, dO rows h
  tlq.init(ld, w, lane);
  tlo.init((size_t)h, w, lane);
  auto issue = [&](int t) {   // query tile t of this workgroup: queries k0 + QT t ..
    const unsigned st = lds0 + (t & 1) * STAGE;
    const int qq = k0 + t * QT;
    tlq.issue(base + (size_t)qq * ld, st, w);
    tlo.issue(dOg + (size_t)qq * h, st + TILE, w);
  };
  const int n_t = (S - k0) / QT;
  issue(0);

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
  float lse_r = 0.f, delta_r = 0.f;
  if (tid < QT) {
    lse_r = lse_g[k0 + tid];
    delta_r = delta_g[k0 + tid];
  }

  auto tile_step = [&](int t, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int qq0 = k0 + t * QT;
    float* lse_s = stat + (t & 1) * 2 * QT;
    float* delta_s = lse_s + QT;
    if (tid < QT) {   // this tile's per-query statistics (fetched one tile ago); the buffer was last read two tiles ago
      lse_s[tid] = lse_r;
      delta_s[tid] = delta_r;
    }
    wait_vm<0>();
    lds_barrier_visible();
    if (t + 1 < n_t) {
      issue(t + 1);
      if (tid < QT) {
        lse_r = lse_g[qq0 + QT + tid];
        delta_r = delta_g[qq0 + QT + tid];
      }
    }
    const unsigned Qs = lds0 + (t & 1) * STAGE, Os = Qs + TILE;
    // sub-tiles of 32 queries; those entirely before this wavefront's keys contribute nothing
    const int first_mt = FULL ? 0 : max(0, (kbase - qq0) / 32);
#pragma unroll
    for (int mt = 0; mt < QT / 32; ++mt) {
      if (FULL || mt >= first_mt) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.rows(Qs, mt * 32, ks), kf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.rows(Os, mt * 32, ks), vf[ks], dp, 0, 0, 0);
        }
        const bool diag = !FULL && qq0 + mt * 32 < kbase + 31;
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
            dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf, fr.cols(Os, mt * 32 + st * 16, i), dv[i], 0, 0, 0);
            dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dsf, fr.cols(Qs, mt * 32 + st * 16, i), dk[i], 0, 0, 0);
          }
        }
      }
    }
  };
  // the first 128 queries are the workgroup's own keys (the diagonal); all later tiles lie after them
  for (int t = 0; t < 128 / QT; ++t) tile_step(t, std::false_type{});
  for (int t = 128 / QT; t < n_t; ++t) tile_step(t, std::true_type{});

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
  // Column sums of dK and dV over this wavefront's 32 keys (second and third third of the QKV bias gradient):
  // a lane holds 16 keys of one column in its registers, the other half-wavefront the other 16.
  if (colsum) {
    float* dst = colsum + ((size_t)b * (S / 32) + kbase / 32) * ld + (size_t)head * D;
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
      float sk = 0.f, sv = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sk += dk[i][r]; sv += dv[i][r]; }
      sk += __shfl_xor(sk, 32, 64);
      sv += __shfl_xor(sv, 32, 64);
      if (g == 0) {
        dst[h + i * 32 + lrow] = sk;
        dst[2 * h + i * 32 + lrow] = sv;
      }
    }
  }
}

template <int D>
constexpr size_t attn_dq_lds() {
  constexpr int KT = D > 128 ? 64 : 128;
  return (size_t)(2 * KT * (D + LDS_PAD) + D * (KT + LDS_PAD)) * sizeof(bf16_t);
}
template <int D>
constexpr size_t attn_dkv_lds() {
  return (size_t)(2 * 64 * (D + LDS_PAD) + 2 * D * (64 + LDS_PAD)) * sizeof(bf16_t) + 2 * 64 * sizeof(float);
}

// ------------------------------------------------------------------------------ launchers
static inline int ok() { return hipGetLastError() == hipSuccess ? KARMA_OK : KARMA_E_HIP; }

int attention_fwd(const bf16_t* qkv, bf16_t* ctx, float* lse, int batch, int seq, int heads, int d, hipStream_t s) {
  if (seq % 128 || (d != 64 && d != 128 && d != 152) || batch <= 0 || heads <= 0) return KARMA_E_INVAL;
  dim3 grid(seq / 128, heads, batch);
  if (d == 64) {
    constexpr int KT = ATTN_FWD_KT, lds = 2 * 2 * KT * 64 * 2;   // two stages of (K tile, V tile)
    auto kern = attn_fwd_dl_kernel<KT, 2>;
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, qkv, ctx, lse, seq, heads);
  }
  else if (d == 128) hipLaunchKernelGGL((attn_fwd_kernel<128, 128>), grid, dim3(256), 0, s, qkv, ctx, lse, seq, heads);
  else hipLaunchKernelGGL((attn_fwd_kernel<152, 160>), grid, dim3(256), 0, s, qkv, ctx, lse, seq, heads);
  return ok();
}

template <int D, int DP = D>
static void launch_bwd(dim3 grid, hipStream_t s, const bf16_t* qkv, const bf16_t* ctx, const bf16_t* dctx, const float* lse,
                       float* delta, bf16_t* dqkv, int seq, int heads, float* colsum = nullptr) {
  if constexpr (D == 64) {
    constexpr int KT = ATTN_DQ_KT, QT = ATTN_DKV_QT;
    constexpr int l1 = 2 * 2 * KT * 64 * 2;                      // two stages of (K tile, V tile)
    constexpr int l2 = 2 * 2 * QT * 64 * 2 + 2 * 2 * QT * 4;     // two stages of (Q tile, dO tile) + their lse, delta
    auto kq = attn_bwd_dq_dl_kernel<KT>;
    auto kkv = attn_bwd_dkv_dl_kernel<QT>;
    (void)hipFuncSetAttribute((const void*)kq, hipFuncAttributeMaxDynamicSharedMemorySize, l1);
    (void)hipFuncSetAttribute((const void*)kkv, hipFuncAttributeMaxDynamicSharedMemorySize, l2);
    hipLaunchKernelGGL(kq, grid, dim3(256), l1, s, qkv, ctx, dctx, lse, delta, dqkv, seq, heads, colsum);
    hipLaunchKernelGGL(kkv, grid, dim3(256), l2, s, qkv, dctx, lse, delta, dqkv, seq, heads, colsum);
  } else {
    constexpr size_t l1 = attn_dq_lds<DP>(), l2 = attn_dkv_lds<DP>();
    auto kq = attn_bwd_dq_kernel<D, DP>;
    auto kkv = attn_bwd_dkv_kernel<D, DP>;
    if (l1 > 64 * 1024) (void)hipFuncSetAttribute((const void*)kq, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l1);
    if (l2 > 64 * 1024) (void)hipFuncSetAttribute((const void*)kkv, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l2);
    hipLaunchKernelGGL(kq, grid, dim3(256), l1, s, qkv, dctx, lse, delta, dqkv, seq, heads);
    hipLaunchKernelGGL(kkv, grid, dim3(256), l2, s, qkv, dctx, lse, delta, dqkv, seq, heads);
  }
}

size_t attention_bwd_colsum_bytes(int batch, int seq, int heads, int d) {
  return (size_t)batch * (seq / 32) * 3 * heads * d * sizeof(float);
}

// colsum_partial (may be null) with room for attention_bwd_colsum_bytes: where the kernels can (head dimension
// 64) they leave one row of column sums of dqkv per 32 tokens there and *colsum_rows is set to the number of
// rows (colsum_finish adds them up: the gradient of the QKV bias); otherwise *colsum_rows stays 0.
int attention_bwd(const bf16_t* qkv, const bf16_t* ctx, const bf16_t* dctx, const float* lse, float* delta,
                  bf16_t* dqkv, int batch, int seq, int heads, int d, hipStream_t s, float* colsum_partial,
                  int* colsum_rows) {
  if (seq % 128 || (d != 64 && d != 128 && d != 152) || batch <= 0 || heads <= 0) return KARMA_E_INVAL;
  if (colsum_rows) *colsum_rows = 0;
  dim3 grid(seq / 128, heads, batch);
  const size_t total = (size_t)batch * seq * heads;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (d == 64) {   // the dQ pass computes delta itself
    launch_bwd<64>(grid, s, qkv, ctx, dctx, lse, delta, dqkv, seq, heads, colsum_rows ? colsum_partial : nullptr);
    if (colsum_partial && colsum_rows) *colsum_rows = batch * (seq / 32);
  } else if (d == 128) {
    hipLaunchKernelGGL(attn_delta_kernel<128>, dim3(blocks), dim3(256), 0, s, ctx, dctx, delta, seq, heads, total);
    launch_bwd<128>(grid, s, qkv, ctx, dctx, lse, delta, dqkv, seq, heads);
  } else {
    hipLaunchKernelGGL(attn_delta_kernel<152>, dim3(blocks), dim3(256), 0, s, ctx, dctx, delta, seq, heads, total);
    launch_bwd<152, 160>(grid, s, qkv, ctx, dctx, lse, delta, dqkv, seq, heads);
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
                       (int)batch, (int)seq, (int)heads, (int)d, (hipStream_t)stream, nullptr, nullptr);
}

// The same with the column sums of dqkv (the QKV bias gradient), from the kernels where they can, else by a pass
// over dqkv.  ws: max(batch * seq / 32, ceil(batch * seq / 64)) * 3 * heads * d floats.
extern "C" int karma_k_attention_bwd_colsum_bf16(const void* qkv, const void* ctx, const void* dctx, const float* lse,
                                                 float* delta_ws, void* dqkv, float* colsum_out, float* ws, uint64_t ws_bytes,
                                                 uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d, void* stream) {
  if (!qkv || !ctx || !dctx || !lse || !delta_ws || !dqkv || !colsum_out || !ws) return KARMA_E_INVAL;
  const int rows = (int)(batch * seq), cols = (int)(3 * heads * d);
  if (ws_bytes < std::max(attention_bwd_colsum_bytes((int)batch, (int)seq, (int)heads, (int)d), colsum_ws_bytes(rows, cols)))
    return KARMA_E_OOM;
  int parts = 0;
  int st = attention_bwd((const bf16_t*)qkv, (const bf16_t*)ctx, (const bf16_t*)dctx, lse, delta_ws, (bf16_t*)dqkv,
                         (int)batch, (int)seq, (int)heads, (int)d, (hipStream_t)stream, ws, &parts);
  if (st) return st;
  if (parts) return colsum_finish(ws, parts, cols, colsum_out, (hipStream_t)stream);
  return colsum_bf16((const bf16_t*)dqkv, colsum_out, ws, rows, cols, (hipStream_t)stream);
}
