// GEMMs of the scheduled layer: the fused-QKV / output / FFN projections (paper section 2.2 step 1,
// appendix schedule) and the eight backward products, with the bias, bias+activation, activation
// derivative and residual-add epilogues applied to the fp32 accumulators in registers.
//
// bf16 path: 8 wavefronts in a 2x4 grid (or 2 x 2x2 with an in-block K split), each owning a block of
// v_mfma_f32_32x32x16_bf16 tiles. K slabs go global -> LDS by direct loads into a ring of LDS stages (or,
// for shapes with a K tail, through registers), one barrier per slab. Operands whose contraction index is
// contiguous in memory are read from LDS with 16-byte reads; operands whose contraction index is the
// strided one (the "N" operand of dY*W and both operands of dY^T*X) stay in their memory order in LDS and
// are read with the transposing ds_read_b64_tr_b16, so no transposed copy of any tensor is ever made.
// fp32 path: a plain LDS-tiled FMA kernel (correctness mode).
#include <stdio.h>
#include <stdlib.h>
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace slapo {

enum { ACT_GELU = 0, ACT_RELU = 1 };
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float act_fwd(float u, int act) {
  if (act == ACT_RELU) return u > 0.f ? u : 0.f;
  return 0.5f * u * (1.f + erff(u * 0.70710678118654752f));
}
__device__ __forceinline__ float act_grad(float u, int act) {
  if (act == ACT_RELU) return u > 0.f ? 1.f : 0.f;
  const float cdf = 0.5f * (1.f + erff(u * 0.70710678118654752f));
  const float pdf = 0.39894228040143268f * __expf(-0.5f * u * u);
  return cdf + u * pdf;
}

// GeLU for the bf16 epilogues. Phi(u) = 0.5 (1 + erf(u / sqrt 2)) with the erf of Abramowitz & Stegun 7.1.26
// (|error| <= 1.5e-7, far below one bf16 rounding): for x >= 0, erf(x) = 1 - t (a1 + t (a2 + ... a5 t)) exp(-x^2),
// t = 1 / (1 + 0.3275911 x). Written for h = 0.5 * poly * exp(-u^2/2): Phi(-|u|) = h, Phi(|u|) = 1 - h, so the
// negative tail has no cancellation. One exp2, one reciprocal and a dozen FMAs, about half the cost of erff.
struct GeluTerms { float phi, e; };   // Phi(u) and exp(-u^2 / 2)
__device__ __forceinline__ GeluTerms gelu_terms(float u) {
  const float t = __builtin_amdgcn_rcpf(fmaf(fabsf(u), 0.3275911f * 0.70710678118654752f, 1.0f));
  const float e = __builtin_amdgcn_exp2f(u * u * (-0.5f * 1.4426950408889634f));
  float p = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
  p = fmaf(t, p, 0.5f * 1.421413741f);
  p = fmaf(t, p, 0.5f * -0.284496736f);
  p = fmaf(t, p, 0.5f * 0.254829592f);
  const float h = p * t * e;
  GeluTerms g;
  g.phi = u < 0.f ? h : 1.0f - h;
  g.e = e;
  return g;
}

template <typename T>
__device__ __forceinline__ void epilogue_store(int epi, int act, float acc, int64_t m, int64_t n, int64_t ldc,
                                               T* __restrict__ C, const T* __restrict__ bias,
                                               const T* aux_in, T* __restrict__ aux_out) {
  const int64_t idx = m * ldc + n;
  float v = acc;
  if (epi == EPI_BIAS) {
    v += to_f32(bias[n]);
  } else if (epi == EPI_BIAS_ACT) {
    v += to_f32(bias[n]);
    if (aux_out) from_f32(aux_out[idx], act_grad(v, act));   // all that backward needs of the pre-activation
    v = act_fwd(v, act);
  } else if (epi == EPI_DACT) {
    const float u = to_f32(aux_in[idx]);
    v = act == ACT_RELU ? (u > 0.f ? v : 0.f) : v * u;
  } else if (epi == EPI_ADD) {
    v += to_f32(aux_in[idx]);
  }
  from_f32(C[idx], v);
}

// silu(u) = u * sigmoid(u) and the two factors the gated feed-forward block keeps for backward
struct GateTerms { float out, dgate, dup; };   // silu(u) * w, w * silu'(u), silu(u)
template <bool FAST>
__device__ __forceinline__ GateTerms gate_terms(float u, float w) {
  const float sg = FAST ? __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u * -1.4426950408889634f))
                        : 1.0f / (1.0f + expf(-u));
  const float s = u * sg;
  GateTerms g;
  g.out = s * w;
  g.dgate = w * (sg + s * (1.0f - sg));   // silu'(u) = sigmoid(u) (1 + u (1 - sigmoid(u)))
  g.dup = s;
  return g;
}

// LDS layouts. Every tile sits in LDS unpadded and in memory order, 16 bytes of thread t of a slab at byte
// 16 t of the stage, so that a slab can be brought in either through registers or by the direct
// global -> LDS loads of gfx950 (one wave-level load fills 1 KB of consecutive LDS, lane l at byte 16 l).
// Bank conflicts are avoided by permuting, inside each tile row, which 16-byte chunk of global memory a
// thread fetches. The LDS has 64 banks of 4 B: 16 lanes of a 16-byte access, and 32 lanes of a transposing
// 8-byte read, are checked against each other for conflicts. Measured peak rates per CU with conflict-free
// addresses and 8 or 16 wavefronts: 16-byte reads 257 B per clock, plain 8-byte reads 164, transposing
// 8-byte reads 120 (about the same instruction rate as the 16-byte read, half the bytes).
//  - K-contiguous tile [rows][BK]: position p of row r holds chunk p ^ swzK(r), swzK(r) = (r / RP) % (BK/8),
//    RP = rows per 256 B. A fragment read (one chunk of 16 consecutive rows) then lands in 16 different
//    16-byte bank groups. swzK depends on the lane only (wave tiles start at multiples of 32 rows), so a
//    fragment address is a per-lane base plus (2*ks ^ per-lane constant).
//  - M-contiguous tile [BK][W]: position p of k-row r holds chunk p ^ (swzM(r) << 1), i.e. 32-byte granules
//    are permuted by swzM(r) (defined in the kernel). A transposing 8-byte read is served 32 lanes at a time:
//    4 consecutive k-rows x 2 adjacent granules, whose 8 pieces the permutation spreads over the 8 bank
//    groups (the conflict counter read 49 % of the LDS cycles with a permutation that only separated the
//    four rows, 1 % of the K-contiguous level with this one).
//
// Why direct loads: a ds_write moves 64 B per clock and keeps the LDS busy meanwhile, so writing a slab
// costs as much LDS time as reading it three times; measured on the chip, fragment reads running beside
// register-staged stores take the sum of both times, beside direct loads the maximum.

// PF: slabs of register prefetch of the register-staged path (NS == 0, two LDS stages).
// NS: LDS stages of the direct-load path (0 = register-staged).
// PW: extra wavefronts that do nothing but issue the direct loads (0 = every wavefront loads its share). A
//     vector-memory instruction holds its wavefront at issue while the address unit is busy, and the 32 KB
//     a 128x128 tile needs per slab keep that unit (64 B per clock) busy for as long as the slab's MFMAs
//     take; with the loads on wavefronts of their own, that wait never stands in front of an MFMA.
// F16: the 16-bit elements are IEEE half instead of bf16 (same data movement; MFMA and conversions differ).
// Position of workgroup `bid` of a grid of tiles_m x tiles_n tiles. Workgroups are handed to the 8 XCDs round-robin;
// the ids are renumbered so that each XCD (own L2) gets a run of consecutive tile ids, and the ids are ordered in
// groups of 4 tile rows walked column by column, so that the tiles an XCD works on at the same time form a compact
// block: its workgroups walk K in step, and every A (B) slab that reaches the L2 is used by all tiles of its row
// (column) in the block. `copies`: the grid holds that many copies of the tile set (K ranges), copy after copy.
struct TilePos { int tile_m, tile_n, copy; };
__device__ __forceinline__ TilePos tile_position(int bid, int tiles_m, int tiles_n, int copies) {
  const int nblk = tiles_m * tiles_n;
  const int per_xcd = (nblk * copies) / 8;
  if (bid < per_xcd * 8) bid = (bid & 7) * per_xcd + (bid >> 3);
  TilePos t;
  t.copy = bid / nblk;
  bid -= t.copy * nblk;
  constexpr int GROUP_M = 4;
  const int group = bid / (GROUP_M * tiles_n);
  const int first_m = group * GROUP_M;
  const int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  const int in_group = bid - group * GROUP_M * tiles_n;
  t.tile_m = first_m + in_group % gsz;
  t.tile_n = in_group / gsz;
  return t;
}

// HYB: a grid whose tile count is not a multiple of the 256 CUs ends in a thin round that costs a full one. A
// hybrid launch runs the tiles of the full rounds as usual (workgroups below tail_begin) and cuts each tile of
// the remainder into tail_splits K ranges, one workgroup each, so that the last round is short instead of
// thin: workgroup tail_begin + r * (tiles in the tail) + t covers range r of tail tile t and leaves its fp32
// accumulators as a full tile in hyb_ws[(t * tail_splits + r)][BM][BN]; hybrid_reduce_kernel adds the ranges in
// order and applies the epilogue. Plain launches pass tail_begin = number of tiles.
template <int LAYOUT, int BM, int BN, int BK, int WGM, int WGN, int KS, int PF, int NS, int PW, bool KTAIL, int EPI,
          bool F16 = false, bool HYB = false>
__global__ __launch_bounds__((WGM * WGN * KS + PW) * 64) void gemm_bf16_kernel(int M, int N, int K,
                                                                  const bf16_t* __restrict__ A,
                                                                  const bf16_t* __restrict__ B,
                                                                  bf16_t* __restrict__ C,
                                                                  const bf16_t* __restrict__ bias,
                                                                  const bf16_t* aux_in,
                                                                  bf16_t* __restrict__ aux_out, int act,
                                                                  int tail_begin, int tail_splits,
                                                                  float* __restrict__ hyb_ws) {
  constexpr bool A_KC = (LAYOUT != GEMM_TN);  // A operand contiguous along K
  constexpr bool DBUF = (LAYOUT != GEMM_NT);  // second fragment register set (measured: +3 % TN, +2-5 % NN, -1 % NT)
  constexpr bool B_KC = (LAYOUT == GEMM_NT);
  // KS == 2: two sets of WGM x WGN wavefronts share the output tile; set g multiplies the g-th half of
  // every K slab and the two accumulator sets are added through LDS before the epilogue. This doubles the
  // wavefronts per SIMD without shrinking the per-wave tile (LDS traffic per flop stays that of the
  // larger wave tile).
  constexpr int NCOMP = WGM * WGN * KS * 64;         // threads that compute
  constexpr int NTHR = PW ? PW * 64 : NCOMP;         // threads that load
  static_assert(PW == 0 || NS > 0, "loader wavefronts belong to the direct path");
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  constexpr int A_LOADS = BM * BK / 8 / NTHR, B_LOADS = BN * BK / 8 / NTHR;
  static_assert(A_LOADS >= 1 && B_LOADS >= 1, "tile too small for the thread count");
  static_assert(BK == 32 || BK == 64 || BK == 128, "swizzles written for 64- to 256-byte tile rows");
  static_assert(!(KTAIL && NS), "a direct load cannot zero-fill the K tail");
  static_assert(NS == 0 || (NS >= 2 && NS <= 10), "stage count");
  constexpr int PA = A_KC ? BK : BM;        // row pitch of the A tile in elements (unpadded)
  constexpr int PB = B_KC ? BK : BN;
  constexpr int SA = BM * BK, SB = BN * BK;  // elements per stage
  constexpr int NSTG = NS ? NS : 2;
  auto swzK = [](int row) { constexpr int RP = BK >= 128 ? 1 : 128 / BK; return (row / RP) % (BK / 8); };
  auto swzM = [](int krow, auto width) {
    constexpr int W = decltype(width)::value;
    static_assert(W >= 64, "at least four 32-byte granules per tile row");
    constexpr int RPM = W >= 128 ? 1 : 128 / W;   // k-rows per 256 bytes of LDS
    const int q = krow / RPM;
    // One transposing read covers, per group of 32 lanes, four consecutive k-rows x two adjacent granules
    // (an even one and its successor): eight 32-byte pieces that must land in eight different bank groups.
    // The k-row picks bits 1-2 of the granule position (bit 1 only for 64-wide tiles, whose rows alternate
    // between the two halves of the 256 bytes by themselves), so the granule's own low bit still tells
    // the two halves apart; rows 8 apart (the other 32 lanes) differ in bit 0.
    return W >= 128 ? (((q & 3) << 1) ^ ((q >> 3) & 1)) : (((q & 1) << 1) ^ ((q >> 2) & 1));
  };
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* sA = smem;               // [NSTG][SA]
  bf16_t* sB = smem + NSTG * SA;   // [NSTG][SB]

  const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
  const int nblk = tiles_m * tiles_n;
  // Split-K instances: `act` K ranges per tile, every (range, tile) pair a workgroup; consecutive ids walk the
  // tiles of one range, so the blocks an XCD holds still share operand panels.
  constexpr bool SPLITK = (EPI == EPI_SPLITK);
  static_assert(!SPLITK || NS > 0, "split-K instances use the direct-load pipeline");
  static_assert(!(HYB && SPLITK) && (!HYB || NS > 0), "hybrid launches use the direct-load pipeline");
  int bid = blockIdx.x;
  bool is_tail = false;          // (uniform for the workgroup)
  int tail_range = 0, tail_tile = 0;
  if (HYB && bid >= tail_begin) {
    const int t = bid - tail_begin, tail_tiles = nblk - tail_begin;
    tail_range = t / tail_tiles;
    tail_tile = t - tail_range * tail_tiles;
    bid = tail_begin + tail_tile;
    is_tail = true;
  }
  const TilePos pos = tile_position(bid, tiles_m, tiles_n, SPLITK ? act : 1);
  const int splits = SPLITK ? act : (is_tail ? tail_splits : 1);
  const int split = SPLITK ? pos.copy : tail_range;
  const int tile_m = pos.tile_m, tile_n = pos.tile_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int lane = threadIdx.x & 63;
  const bool is_loader = PW ? threadIdx.x >= NCOMP : true;
  const int tid = PW ? (is_loader ? threadIdx.x - NCOMP : 0) : threadIdx.x;   // index among the loading threads
  const int cw = threadIdx.x >> 6;                                            // wavefront index
  const int kgroup = cw / (WGM * WGN), wave = cw % (WGM * WGN);
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

  // Each thread moves A_LOADS + B_LOADS 16-byte pieces per slab: thread t owns position t of the slab (tile
  // row t / CA, chunk position t % CA), piece i sits NTHR positions (RSA tile rows) further. Pieces outside
  // M or N are read from a clamped (valid) address and never reach a stored output, so only the K tail
  // needs zero fill; all loads are unconditional, which lets the compiler keep the next slabs' loads in
  // flight while it waits for the oldest ones only.
  constexpr int CA = A_KC ? BK / 8 : BM / 8, CB = B_KC ? BK / 8 : BN / 8;   // pieces per tile row
  constexpr int RSA = NTHR / CA, RSB = NTHR / CB;                            // tile rows between pieces
  static_assert(NS != 0 || (RSA % 16 == 0 && RSB % 16 == 0), "the K-tail test assumes one column per thread");
  const int ar = tid / CA, br = tid / CB;
  // column (in elements) of the chunk fetched for the position in tile row r
  auto col_a = [&](int r) {
    return A_KC ? ((tid % CA) ^ swzK(r)) * 8 : ((tid % CA) ^ (swzM(r, std::integral_constant<int, BM>{}) << 1)) * 8;
  };
  auto col_b = [&](int r) {
    return B_KC ? ((tid % CB) ^ swzK(r)) * 8 : ((tid % CB) ^ (swzM(r, std::integral_constant<int, BN>{}) << 1)) * 8;
  };
  const int ac = col_a(ar), bc = col_b(br);
  const int lda = A_KC ? K : M, ldb = B_KC ? K : N;
  const bf16_t* ga[A_LOADS];
  const bf16_t* gb[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int tr = ar + i * RSA;
    if (A_KC) { int r = m0 + tr; r = r < M ? r : M - 1; ga[i] = A + (int64_t)r * lda + col_a(tr); }
    else { int c = m0 + col_a(tr); c = c < M ? c : M - 8; ga[i] = A + (int64_t)tr * lda + c; }
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int tr = br + i * RSB;
    if (B_KC) { int r = n0 + tr; r = r < N ? r : N - 1; gb[i] = B + (int64_t)r * ldb + col_b(tr); }
    else { int c = n0 + col_b(tr); c = c < N ? c : N - 8; gb[i] = B + (int64_t)tr * ldb + c; }
  }
  const int64_t stepA = A_KC ? BK : (int64_t)BK * lda, stepB = B_KC ? BK : (int64_t)BK * ldb;

  // slabs of this workgroup: all of them, or the split's range (the host makes every range non-empty)
  const int nk_all = (K + BK - 1) / BK;
  const int nk_per = (nk_all + splits - 1) / splits;
  const int ks0 = split * nk_per;   // (split = 0, splits = 1 for workgroups that walk all of K)
  const int nk = nk_all - ks0 < nk_per ? nk_all - ks0 : nk_per;
  static_assert(PF == 1 || PF == 2, "register prefetch depth");
  u32x4_t ra0[A_LOADS], rb0[B_LOADS], ra1[A_LOADS], rb1[B_LOADS];   // register sets: slab k lives in set k % PF
  // Every call issues exactly A_LOADS + B_LOADS loads (slab index clamped to the last one), so the number
  // of loads in flight is the same on every path and the oldest slab can be awaited on its own.
  auto load_global = [&](int kstep, u32x4_t (&ra)[A_LOADS], u32x4_t (&rb)[B_LOADS]) {
    kstep = kstep < nk ? kstep : nk - 1;
    const int k0 = kstep * BK;
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
      const bf16_t* p = ga[i] + kstep * stepA;
      if (KTAIL) {  // pieces at or beyond K: read a valid address, zero the value
        const bool ok = A_KC ? (k0 + ac < K) : (k0 + ar + i * RSA < K);
        p = ok ? p : A;
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(p);
        ra[i] = ok ? v : u32x4_t{0, 0, 0, 0};
      } else {
        ra[i] = *reinterpret_cast<const u32x4_t*>(p);
      }
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
      const bf16_t* p = gb[i] + kstep * stepB;
      if (KTAIL) {
        const bool ok = B_KC ? (k0 + bc < K) : (k0 + br + i * RSB < K);
        p = ok ? p : B;
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(p);
        rb[i] = ok ? v : u32x4_t{0, 0, 0, 0};
      } else {
        rb[i] = *reinterpret_cast<const u32x4_t*>(p);
      }
    }
  };
  auto store_lds = [&](int stage, const u32x4_t (&ra)[A_LOADS], const u32x4_t (&rb)[B_LOADS]) {
    bf16_t* a = sA + stage * SA + tid * 8;
    bf16_t* b = sB + stage * SB + tid * 8;
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) *reinterpret_cast<u32x4_t*>(a + i * NTHR * 8) = ra[i];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) *reinterpret_cast<u32x4_t*>(b + i * NTHR * 8) = rb[i];
  };
  // Direct path: the same pieces, written by the memory system straight into LDS (wave-uniform LDS base,
  // lane l lands 16 l bytes behind it). Completion is tracked by the vector-memory counter. The loads are
  // buffer loads: resource = the operand from the tile's origin on, per-lane byte offset fixed for the whole
  // K loop, the K step in the scalar offset. Issuing a slab then takes no vector-ALU instruction at all,
  // which matters because the vector ALU is where the MFMAs run: address arithmetic of a loading wavefront
  // queues behind the MFMAs of the wavefronts that share its SIMD (measured: 64-bit per-lane addresses make
  // load time and MFMA time add up; this form overlaps them). Reads beyond the operand's end return zero.
  unsigned voa[A_LOADS], vob[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) voa[i] = (unsigned)(((ar + i * RSA) * lda + col_a(ar + i * RSA)) * 2);
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) vob[i] = (unsigned)(((br + i * RSB) * ldb + col_b(br + i * RSB)) * 2);
  const int64_t origin_a = A_KC ? (int64_t)m0 * lda : m0, origin_b = B_KC ? (int64_t)n0 * ldb : n0;
  auto records = [](int64_t elems) { const int64_t b = elems * 2; return (unsigned)(b < 0xffffffffll ? b : 0xffffffffll); };
  const bf16_t* base_a = A + origin_a;
  const bf16_t* base_b = B + origin_b;
  const unsigned bytes_a = records((int64_t)M * K - origin_a), bytes_b = records((int64_t)N * K - origin_b);
  const int lw = __builtin_amdgcn_readfirstlane(PW ? cw - NCOMP / 64 : cw);   // index among the loading wavefronts
  // Fragments of an operand that is not contiguous along K come through transposing reads, which the compiler would
  // hold back behind every direct load this wavefront has in flight (common.h): those instances issue their own.
  constexpr bool UNTRACKED = !(A_KC && B_KC) && PW == 0;
  auto dma16 = [](const bf16_t* base, unsigned bytes, bf16_t* lds, unsigned voffset, unsigned soffset) {
    if constexpr (UNTRACKED) buffer_load_lds_16_untracked(base, bytes, lds, voffset, soffset);
    else buffer_load_lds_16(base, bytes, lds, voffset, soffset);
  };
  auto load_direct = [&](int kstep, int stage) {
    bf16_t* a = sA + stage * SA + lw * 512;
    bf16_t* b = sB + stage * SB + lw * 512;
    const unsigned soa = (unsigned)(ks0 + kstep) * (unsigned)(stepA * 2), sob = (unsigned)(ks0 + kstep) * (unsigned)(stepB * 2);
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) dma16(base_a, bytes_a, a + i * NTHR * 8, voa[i], soa);
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) dma16(base_b, bytes_b, b + i * NTHR * 8, vob[i], sob);
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Per-lane fragment addressing (stage 0, k-step 0).
  // K-contiguous: chunk 2*ks + lane/32 of row lane%32, stored at position (2*ks + lane/32) ^ swzK =
  // (2*ks ^ fsw) with the low bit folded into the base.
  const int fsw = swzK(lane & 31) & ~1;
  const int kc_low = (((lane >> 5) ^ swzK(lane & 31)) & 1) << 3;
  const int fa_base = (wm0 + (lane & 31)) * PA + kc_low;
  const int fb_base = (wn0 + (lane & 31)) * PB + kc_low;
  // M-contiguous: the lane reads 4 elements at k-row krow_l (+4 for the upper half of the fragment), column
  // 16*((lane/16)%2) + 4*(lane%4) of the 32-wide tile; the 32-byte granule index g is stored at g ^ swzM.
  const int krow_l = 8 * (lane >> 5) + ((lane & 15) >> 2);
  int ma_lo[2], ma_sw[2], mb_lo[2], mb_sw[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int swa = swzM(krow_l + 4 * h, std::integral_constant<int, BM>{});
    const int swb = swzM(krow_l + 4 * h, std::integral_constant<int, BN>{});
    ma_lo[h] = (krow_l + 4 * h) * PA + (((((lane >> 4) ^ swa) & 1)) << 4) + 4 * (lane & 3);
    mb_lo[h] = (krow_l + 4 * h) * PB + (((((lane >> 4) ^ swb) & 1)) << 4) + 4 * (lane & 3);
    ma_sw[h] = swa & ~1;
    mb_sw[h] = swb & ~1;
  }
  auto frag_kc = [&](const bf16_t* tile, int base, int pitch, int t, int ks) -> bf16x8_t {
    return *reinterpret_cast<const bf16x8_t*>(tile + base + t * 32 * pitch + (((2 * ks) ^ fsw) << 3));
  };
  auto frag_mc = [&](const bf16_t* tile, const int (&lo)[2], const int (&sw)[2], int pitch, int g0, int ks) -> bf16x8_t {
    typedef s16x4_t __attribute__((address_space(3))) * lds4_t;
    const bf16_t* p = tile + ks * 16 * pitch;
    s16x4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(p + lo[0] + ((g0 ^ sw[0]) << 4)));
    s16x4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(p + lo[1] + ((g0 ^ sw[1]) << 4)));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    s16x8_t v = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  };
  auto compute = [&](int stage) {
    const bf16_t* a = sA + stage * SA;
    const bf16_t* b = sB + stage * SB;
    constexpr int KQ = BK / 16 / KS;
    if constexpr (DBUF && TM * TN >= TM + TN && KQ >= 2) {
      // Large wave tiles with both operands strided: one fragment of the NEXT k-step is requested in front of each
      // of the first TM + TN MFMAs of the current one, into a second register set, in the order the next
      // k-step uses them (A0, B0.., A1..). Every fragment then has at least six MFMAs of time, where the
      // single-set schedule the compiler produces waits for its last B fragment two MFMAs after asking for it.
      bf16x8_t fa[2][TM], fb[2][TN];
      auto read_a = [&](int kq, int i) {
        const int ks = kq + kgroup * KQ;
        return A_KC ? frag_kc(a, fa_base, PA, i, ks) : frag_mc(a, ma_lo, ma_sw, PA, (wm0 >> 4) + 2 * i, ks);
      };
      auto read_b = [&](int kq, int j) {
        const int ks = kq + kgroup * KQ;
        return B_KC ? frag_kc(b, fb_base, PB, j, ks) : frag_mc(b, mb_lo, mb_sw, PB, (wn0 >> 4) + 2 * j, ks);
      };
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[0][i] = read_a(0, i);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[0][j] = read_b(0, j);
#pragma unroll
      for (int kq = 0; kq < KQ; ++kq) {
        const int cur = kq & 1, nxt = cur ^ 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int m = i * TN + j;   // MFMA index inside the k-step = slot of the next k-step to request
            if (kq + 1 < KQ) {
              if (m == 0) fa[nxt][0] = read_a(kq + 1, 0);
              else if (m <= TN) fb[nxt][m - 1] = read_b(kq + 1, m - 1);
              else if (m < TM + TN) fa[nxt][m - TN] = read_a(kq + 1, m - TN);
            }
            acc[i][j] = mfma16<F16>(fa[cur][i], fb[cur][j], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);   // keep this order (the scheduler would sink the requests)
          }
      }
      return;
    }
    // scheduling hint for the slab: interleave the LDS reads with the MFMAs (variant chosen by measurement)
    __builtin_amdgcn_iglp_opt(LAYOUT == GEMM_TN ? 1 : 0);
#pragma unroll
    for (int kq = 0; kq < BK / 16 / KS; ++kq) {
      const int ks = kq + kgroup * (BK / 16 / KS);
      bf16x8_t fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = A_KC ? frag_kc(a, fa_base, PA, i, ks) : frag_mc(a, ma_lo, ma_sw, PA, (wm0 >> 4) + 2 * i, ks);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = B_KC ? frag_kc(b, fb_base, PB, j, ks) : frag_mc(b, mb_lo, mb_sw, PB, (wn0 >> 4) + 2 * j, ks);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma16<F16>(fa[i], fb[j], acc[i][j]);
    }
  };

  if constexpr (NS == 0) {
    // Register-staged pipeline: the slab of k-step k is computed from LDS stage k&1 while the global loads
    // of the next PF slabs are in flight in registers (register set k % PF holds slab k); a slab is written
    // to LDS right after the compute of the step before it. With PF == 2 the slab count must be even (the
    // host falls back to PF == 1 otherwise). Loads and stores are issued on every step (slab index
    // clamped; the last steps re-fetch the last slab into a stage nobody reads): with every step alike,
    // the wait before an LDS store covers the oldest slab only and the newer loads stay in flight.
    load_global(0, ra0, rb0);
    if (PF > 1) load_global(1, ra1, rb1);
    store_lds(0, ra0, rb0);
    __syncthreads();
    if (PF == 1) {
      for (int k = 0; k < nk; ++k) {
        load_global(k + 1, ra0, rb0);
        compute(k & 1);
        store_lds((k + 1) & 1, ra0, rb0);
        __syncthreads();
      }
    } else {
      for (int k = 0; k < nk; k += 2) {
        load_global(k + 2, ra0, rb0);
        compute(0);
        store_lds(1, ra1, rb1);
        __syncthreads();
        load_global(k + 3, ra1, rb1);
        compute(1);
        store_lds(0, ra0, rb0);
        __syncthreads();
      }
    }
  } else {
    // Direct pipeline over a ring of NS stages, slab j in stage j % NS (at least NS - 1 slabs). Step k issues the loads of slab k + NS - 1 into the stage that step k - 1 computed from (free
    // since the barrier that ended step k - 1), computes slab k, then waits until its own loads of slab
    // k + 1 have landed (the younger ones stay in flight) and meets the other wavefronts at the barrier.
    constexpr int LPS = A_LOADS + B_LOADS;   // loads per slab and loading wavefront
    if (is_loader) {
#pragma unroll
      for (int j = 0; j < NS - 1; ++j) load_direct(j, j);
    }
    wait_loads_and_lds<(NS - 2) * LPS>();
    block_barrier();
    if (PW && is_loader) {
      // loader wavefronts: issue, wait for the oldest slab, meet the others; nothing else
      for (int k0 = 0; k0 < nk; k0 += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          if (k0 + s >= nk) break;                  // uniform (slab counts that are no multiple of NS)
          const bool more = k0 + s + NS - 1 < nk;   // uniform
          if (more) load_direct(k0 + s + NS - 1, (s + NS - 1) % NS);
          if (more) wait_loads_and_lds<(NS - 2) * LPS>();
          else wait_loads_and_lds<0>();
          block_barrier();
        }
      }
    } else {
      for (int k0 = 0; k0 < nk; k0 += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          if (k0 + s >= nk) break;                  // uniform
          const bool more = k0 + s + NS - 1 < nk;   // uniform
          if (!PW && more) load_direct(k0 + s + NS - 1, (s + NS - 1) % NS);
          compute(s);
          if (PW) wait_loads_and_lds<63>();          // LDS reads done (no loads of its own)
          else if (more) wait_loads_and_lds<(NS - 2) * LPS>();
          else wait_loads_and_lds<0>();
          block_barrier();
        }
      }
    }
  }

  if (PW && is_loader) return;   // every load has landed (the last steps drain them); the rest is compute only

  // Epilogue. The accumulators (element r of a 32x32 tile: row (r/4)*8 + 4*(lane/32) + r%4, column
  // lane%32) go, one 32-row slab at a time, through a per-wave fp32 staging area in LDS so that every
  // global access of the epilogue (bias, auxiliary input, both outputs) is a 16-byte access of 8
  // consecutive columns of one row. The main loop ended with a barrier, so the stages are free.
  if (KS == 2) {   // add the second wave set's accumulators to the first; then only the first goes on
    float* red = reinterpret_cast<float*>(smem) + wave * (TM * TN * 16 * 64) + lane;
    if (kgroup == 1) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) red[((i * TN + j) * 16 + r) * 64] = acc[i][j][r];
    }
    __syncthreads();
    if (kgroup == 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] += red[((i * TN + j) * 16 + r) * 64];
    }
    __syncthreads();
    if (kgroup == 1) return;
  }
  constexpr int LDP = WN + 4;
  float* stage = reinterpret_cast<float*>(smem) + wave * (32 * LDP);
  constexpr int CPR = WN / 8;         // 8-column chunks per staged row
  constexpr int RPP = 64 / CPR;       // rows covered by one pass of the wave
  const int cc = lane % CPR, rr = lane / CPR;
  const int n = n0 + wn0 + cc * 8;
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if ((EPI == EPI_BIAS || EPI == EPI_BIAS_ACT) && n < N) load8h<F16>(bias + n, bv);
  // The auxiliary input of a 32-row slab is fetched one slab ahead (clamped addresses, so the loads are
  // unconditional): its latency passes while the slab before it is staged and written out.
  constexpr bool AUX = (EPI == EPI_DACT || EPI == EPI_ADD || EPI == EPI_DGATE);
  constexpr int NP = 32 / RPP;
  constexpr int NAUX = EPI == EPI_DGATE ? 2 : 1;   // 16-byte pieces of auxiliary input per 8 product columns
  u32x4_t au[TM][NP * NAUX];
  auto aux_fetch = [&](int i, u32x4_t (&dst)[NP * NAUX]) {
    const int nc = n < N ? n : N - 8;
#pragma unroll
    for (int pass = 0; pass < NP; ++pass) {
      int m = m0 + wm0 + i * 32 + pass * RPP + rr;
      m = m < M ? m : M - 1;
      if constexpr (EPI == EPI_DGATE) {   // the factor pairs of product columns nc..nc+7 sit in columns 2nc..2nc+15 of [M,2N]
        const bf16_t* q = aux_in + (int64_t)m * (2 * N) + 2 * nc;
        dst[2 * pass] = *reinterpret_cast<const u32x4_t*>(q);
        dst[2 * pass + NAUX - 1] = *reinterpret_cast<const u32x4_t*>(q + 8);
      } else {
        dst[pass] = *reinterpret_cast<const u32x4_t*>(aux_in + (int64_t)m * N + nc);
      }
    }
  };
  auto aux_get = [](const u32x4_t& w, float (&u)[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) { u[2 * e] = unpack_lo<F16>(w[e]); u[2 * e + 1] = unpack_hi<F16>(w[e]); }
  };
  if (AUX && !is_tail) aux_fetch(0, au[0]);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (AUX && !is_tail && i + 1 < TM) aux_fetch(i + 1, au[i + 1]);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stage[((r >> 2) * 8 + 4 * (lane >> 5) + (r & 3)) * LDP + j * 32 + (lane & 31)] = acc[i][j][r];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int pass = 0; pass < 32 / RPP; ++pass) {
      const int row = pass * RPP + rr;
      const int m = m0 + wm0 + i * 32 + row;
      float v[8];
      const float4 lo = *reinterpret_cast<const float4*>(stage + row * LDP + cc * 8);
      const float4 hi = *reinterpret_cast<const float4*>(stage + row * LDP + cc * 8 + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
      if (HYB && is_tail) {   // one K range of a tail tile: the bare accumulators, as a full tile of the workspace
        float* part = hyb_ws + ((size_t)(tail_tile * tail_splits + tail_range) * BM + (wm0 + i * 32 + row)) * BN + wn0 + cc * 8;
        *reinterpret_cast<float4*>(part) = lo;
        *reinterpret_cast<float4*>(part + 4) = hi;
      } else if (m < M && n < N) {
        const int64_t idx = (int64_t)m * N + n;
        if (EPI == EPI_BIAS) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bv[e];
        } else if (EPI == EPI_BIAS_ACT) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bv[e];
          // Activation and its derivative from the same fp32 pre-activation; the derivative is what is kept
          // for backward (the activation terms are at hand here, and backward is then one multiply).
          float dv[8];
          if (act == ACT_RELU) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { dv[e] = v[e] > 0.f ? 1.f : 0.f; v[e] = v[e] > 0.f ? v[e] : 0.f; }
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const GeluTerms g = gelu_terms(v[e]);
              dv[e] = fmaf(v[e] * g.e, 0.39894228040143268f, g.phi);
              v[e] *= g.phi;
            }
          }
          if (aux_out) store8h<F16>(aux_out + idx, dv);   // (a ReLU layer keeps nothing: its gate is read off the output)
        } else if (EPI == EPI_DACT) {
          float u[8];
          aux_get(au[i][pass], u);
          if (act == ACT_RELU) {   // aux_in is the activation output (or the stored 0/1 derivative): gate = [aux_in > 0]
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = u[e] > 0.f ? v[e] : 0.f;
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] *= u[e];
          }
        } else if (EPI == EPI_ADD) {
          float u[8];
          aux_get(au[i][pass], u);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += u[e];
        } else if (EPI == EPI_GATE) {
          // columns come as (gate, up) pairs: four gated values go to C [M,N/2], the backward factors stay [M,N]
          float f[8], o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const GateTerms g = gate_terms<true>(v[2 * e], v[2 * e + 1]);
            o[e] = g.out; f[2 * e] = g.dgate; f[2 * e + 1] = g.dup;
          }
          store8h<F16>(aux_out + idx, f);
          uint2 w;
          w.x = pack2<F16>(o[0], o[1]);
          w.y = pack2<F16>(o[2], o[3]);
          *reinterpret_cast<uint2*>(C + (int64_t)m * (N / 2) + n / 2) = w;
        } else if constexpr (EPI == EPI_DGATE) {
          float fa[8], fb[8], o0[8], o1[8];
          aux_get(au[i][2 * pass], fa);
          aux_get(au[i][2 * pass + NAUX - 1], fb);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o0[2 * e] = v[e] * fa[2 * e]; o0[2 * e + 1] = v[e] * fa[2 * e + 1];
            o1[2 * e] = v[4 + e] * fb[2 * e]; o1[2 * e + 1] = v[4 + e] * fb[2 * e + 1];
          }
          bf16_t* q = C + (int64_t)m * (2 * N) + 2 * n;
          store8h<F16>(q, o0);
          store8h<F16>(q + 8, o1);
        }
        else if (EPI == EPI_SPLITK) {
          float* part = reinterpret_cast<float*>(aux_out) + (int64_t)split * M * N + idx;
          *reinterpret_cast<float4*>(part) = make_float4(v[0], v[1], v[2], v[3]);
          *reinterpret_cast<float4*>(part + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
        if (EPI != EPI_GATE && EPI != EPI_DGATE && EPI != EPI_SPLITK) store8h<F16>(C + idx, v);
      }
    }
  }
}

template <int BM, int BN, int BK, int WGM, int WGN, int KS, int NS>
constexpr size_t gemm_lds_bytes() {
  constexpr size_t main_bytes = (size_t)(NS ? NS : 2) * (BM + BN) * BK * sizeof(bf16_t);
  constexpr size_t epi_bytes = (size_t)WGM * WGN * 32 * (BN / WGN + 4) * sizeof(float);
  constexpr size_t red_bytes = KS == 2 ? (size_t)BM * BN * sizeof(float) : 0;
  constexpr size_t m1 = main_bytes > epi_bytes ? main_bytes : epi_bytes;
  return m1 > red_bytes ? m1 : red_bytes;
}

// fp32 correctness kernel: 64x64 tile, 16-deep slabs, each thread a 4x4 block.
template <int LAYOUT>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int M, int N, int K, const float* __restrict__ A,
                                                       const float* __restrict__ B, float* __restrict__ C,
                                                       const float* __restrict__ bias, const float* aux_in,
                                                       float* __restrict__ aux_out, int epi, int act) {
  __shared__ float sA[16][65], sB[16][65];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int q = tid; q < 64 * 16; q += 256) {
      const int mm = q & 63, kk = q >> 6;
      const int m = m0 + mm, n = n0 + mm, k = k0 + kk;
      float av = 0.f, bv = 0.f;
      if (k < K) {
        if (m < M) av = (LAYOUT == GEMM_TN) ? A[(int64_t)k * M + m] : A[(int64_t)m * K + k];
        if (n < N) bv = (LAYOUT == GEMM_NT) ? B[(int64_t)n * K + k] : B[(int64_t)k * N + n];
      }
      sA[kk][mm] = av;
      sB[kk][mm] = bv;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[kk][ty * 4 + i]; b[i] = sB[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m >= M || n >= N) continue;
      if (epi == EPI_GATE) {          // (gate, up) pairs in adjacent columns; the even one does the work
        if (j & 1) continue;
        const GateTerms g = gate_terms<false>(acc[i][j], acc[i][j + 1]);
        C[(int64_t)m * (N / 2) + n / 2] = g.out;
        aux_out[(int64_t)m * N + n] = g.dgate;
        aux_out[(int64_t)m * N + n + 1] = g.dup;
      } else if (epi == EPI_DGATE) {
        const int64_t q = (int64_t)m * (2 * N) + 2 * n;
        C[q] = acc[i][j] * aux_in[q];
        C[q + 1] = acc[i][j] * aux_in[q + 1];
      } else {
        epilogue_store<float>(epi, act, acc[i][j], m, n, N, C, bias, aux_in, aux_out);
      }
    }
}

// epilogue / layout pairs the layer itself uses; only these get the tuned (deep-prefetch) kernels
constexpr bool epi_used(int layout, int epi) {
  return layout == GEMM_NT ? (epi == EPI_NONE || epi == EPI_BIAS || epi == EPI_BIAS_ACT || epi == EPI_GATE)
       : layout == GEMM_NN ? (epi == EPI_NONE || epi == EPI_DACT || epi == EPI_ADD || epi == EPI_DGATE)
                           : (epi == EPI_NONE || epi == EPI_ADD);
}

template <int LAYOUT, int BM, int BN, int BK, int WGM, int WGN, int KS, int PF, int NS, int PW, bool KTAIL, bool F16>
static void launch_bf16_tile(int epi, int act, int M, int N, int K, const void* A, const void* B, void* C,
                             const void* bias, const void* aux_in, void* aux_out, hipStream_t st) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const size_t lds = gemm_lds_bytes<BM, BN, BK, WGM, WGN, KS, NS>();
#define SLAPO_GEMM(E)                                                                                       \
  do {                                                                                                      \
    if constexpr (KTAIL || epi_used(LAYOUT, E)) {                                                           \
      auto kern = gemm_bf16_kernel<LAYOUT, BM, BN, BK, WGM, WGN, KS, PF, NS, PW, KTAIL, E, F16>;                           \
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);  \
      hipLaunchKernelGGL(kern, dim3(tiles), dim3((WGM * WGN * KS + PW) * 64), lds, st, M, N, K, (const bf16_t*)A,       \
                         (const bf16_t*)B, (bf16_t*)C, (const bf16_t*)bias, (const bf16_t*)aux_in,          \
                         (bf16_t*)aux_out, act, tiles, 1, (float*)nullptr);                                 \
    } else {                                                                                                \
      launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 2, 1, 1, 0, 0, true, F16>(epi, act, M, N, K, A, B, C, bias, aux_in,    \
                                                              aux_out, st);                                 \
    }                                                                                                       \
  } while (0)
  switch (epi) {
    case EPI_NONE: SLAPO_GEMM(EPI_NONE); break;
    case EPI_BIAS: SLAPO_GEMM(EPI_BIAS); break;
    case EPI_BIAS_ACT: SLAPO_GEMM(EPI_BIAS_ACT); break;
    case EPI_DACT: SLAPO_GEMM(EPI_DACT); break;
    case EPI_GATE: SLAPO_GEMM(EPI_GATE); break;
    case EPI_DGATE: SLAPO_GEMM(EPI_DGATE); break;
    default: SLAPO_GEMM(EPI_ADD); break;
  }
#undef SLAPO_GEMM
}

// ---- thin last rounds: the tail tiles of a 256x256 grid in several K ranges ----------------------------
// 320 tiles on 256 CUs take two rounds for 1.25 rounds of work. With a workspace at hand, the tiles beyond the
// last full round are cut into s = 256 / (their number) K ranges, so that the last round has about 256 workgroups
// of 1/s the length, and a second kernel adds the ranges in order (bitwise reproducible) and applies the
// epilogue. Worth it when the saved (1 - 1/s) of a round outweighs writing and re-reading the partial tiles,
// i.e. for long K; plain and add epilogues only (the others have so many tiles that a thin round matters little).
struct HybridPlan { int tail_begin, tail_tiles, splits; size_t ws_bytes; };
static HybridPlan hybrid_plan(int epi, int M, int N, int K) {
  const int tiles = ((M + 255) / 256) * ((N + 255) / 256);
  HybridPlan none = {tiles, 0, 1, 0}, p = none;
  static const bool disabled = debug_flag("no-hybrid");
  if (disabled || (epi != EPI_NONE && epi != EPI_ADD) || K % 128 != 0) return none;
  const int rem = tiles % 256, nk = K / 64;
  if (tiles <= 256 || rem == 0) return none;
  int s = 256 / rem;
  s = s > 8 ? 8 : s;
  while (s > 1 && ((s - 1) * ((nk + s - 1) / s) >= nk || nk / s < 8)) --s;   // every range non-empty, at least 8 slabs
  if (s < 2) return none;
  // a round of 64-deep slabs takes about 1.1 us per slab; the partial tiles are written and read once at ~4 TB/s
  const double saved_us = (1.0 - 1.0 / s) * nk * 1.1;
  const double cost_us = 2.0 * rem * s * 256.0 * 256.0 * 4.0 / 4.0e6;
  if (saved_us < 1.5 * cost_us) return none;
  p.tail_tiles = rem;
  p.tail_begin = tiles - rem;
  p.splits = s;
  p.ws_bytes = (size_t)rem * s * 256 * 256 * sizeof(float);
  return p;
}

// C tile of tail tile t = sum over the K ranges of hyb_ws[(t * splits + r)] (+ aux_in), eight columns per thread.
template <bool F16>
__global__ __launch_bounds__(256) void hybrid_reduce_kernel(int M, int N, int tail_begin, int splits,
                                                            const float* __restrict__ ws, bf16_t* C,
                                                            const bf16_t* aux_in) {
  constexpr int BM = 256, BN = 256, CPT = BM * BN / 8;   // 8-column chunks per tile
  const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
  const int q = blockIdx.x * 256 + threadIdx.x;
  const int t = q / CPT, in_tile = q - t * CPT;
  const TilePos pos = tile_position(tail_begin + t, tiles_m, tiles_n, 1);
  const int row = in_tile / (BN / 8), col = (in_tile % (BN / 8)) * 8;
  const int m = pos.tile_m * BM + row, n = pos.tile_n * BN + col;
  if (m >= M || n >= N) return;
  const float* part = ws + ((size_t)t * splits * BM + row) * BN + col;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = 0; r < splits; ++r) {
    float v[8];
    load8(part + (size_t)r * BM * BN, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  const int64_t idx = (int64_t)m * N + n;
  if (aux_in) {
    float v[8];
    load8h<F16>(aux_in + idx, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  store8h<F16>(C + idx, acc);
}

template <int LAYOUT, bool F16>
static void launch_hybrid(const HybridPlan& hp, int epi, int M, int N, int K, const void* A, const void* B, void* C,
                          const void* aux_in, float* ws, hipStream_t st) {
  constexpr int BM = 256, BN = 256, PW = LAYOUT == GEMM_NT ? 4 : 0;   // (loader wavefronts as in the plain launch)
  const size_t lds = gemm_lds_bytes<BM, BN, 64, 2, 4, 1, 2>();
  const int grid = hp.tail_begin + hp.tail_tiles * hp.splits;
#define SLAPO_HYB(E)                                                                                           \
  do {                                                                                                         \
    auto kern = gemm_bf16_kernel<LAYOUT, BM, BN, 64, 2, 4, 1, 2, 2, PW, false, E, F16, true>;                  \
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);       \
    hipLaunchKernelGGL(kern, dim3(grid), dim3((8 + PW) * 64), lds, st, M, N, K, (const bf16_t*)A, (const bf16_t*)B, \
                       (bf16_t*)C, (const bf16_t*)nullptr, (const bf16_t*)aux_in, (bf16_t*)nullptr, 0,         \
                       hp.tail_begin, hp.splits, ws);                                                          \
  } while (0)
  if (epi == EPI_ADD) SLAPO_HYB(EPI_ADD); else SLAPO_HYB(EPI_NONE);
#undef SLAPO_HYB
  const int chunks = hp.tail_tiles * (BM * BN / 8);
  hipLaunchKernelGGL(hybrid_reduce_kernel<F16>, dim3(chunks / 256), dim3(256), 0, st, M, N, hp.tail_begin, hp.splits,
                     (const float*)ws, (bf16_t*)C, epi == EPI_ADD ? (const bf16_t*)aux_in : (const bf16_t*)nullptr);
}

// Tile selection, from measurements on the layer's shapes. 256x256 tiles (8 wavefronts, 128x64 each, direct
// loads into two stages, issued by four more wavefronts in the NT layout) when they still cover at least three quarters of the 256 CUs. Otherwise 128x128
// tiles (8 wavefronts, 64x32 each): direct loads into a ring of four stages issued by four loader
// wavefronts when K is a multiple of four slabs; else register-staged with two slabs of prefetch. For outputs with few tiles, 128x64
// tiles: long K the same direct scheme with four computing wavefronts, else 128-deep slabs and two wave
// sets splitting each slab. Other K go to the general kernel (one slab of register prefetch, zero-filled
// tail).
enum TileKind { TILE_256, TILE_128_SPLITSLAB, TILE_128_LOADERS, TILE_128_REGS, TILE_128x64_LOADERS, TILE_128x64_DEEP, TILE_GENERAL };
static TileKind select_tile(int layout, int M, int N, int K, bool solo) {
  const int64_t t256 = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
  const int64_t t128 = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
  // A grid of 256x256 tiles runs in rounds of 256 (one workgroup per CU) and a thin last round costs a full one:
  // 320 tiles take two rounds for 1.25 rounds of work. A GEMM that has the chip to itself (`solo`: the forward
  // pass, the exported building block) therefore takes 128x128 tiles when their round count is the cheaper one,
  // at the long-K rates of the two kernels (PFLOP/s: 1.30 for all three layouts against 1.05 / 1.0 /
  // 1.0; a 256x256 tile is four small ones). In the backward pass the idle CUs of a thin round are exactly where
  // the other stream's kernels run, and the same rule makes the step slower (2.7B-shaped layer: 5.39 ms against
  // 4.99 ms; on a single stream 5.06 against 5.62), so it is not applied there.
  bool big = K % 128 == 0 && t256 >= 192;
  if (solo && big && K % 256 == 0 && K >= 2048) {
    const double e256 = 1.30, e128 = layout == GEMM_NT ? 1.05 : 1.0;
    const double c256 = (double)((t256 + 255) / 256) * 4.0 / e256, c128 = (double)((t128 + 255) / 256) / e128;
    big = c256 <= c128;
  }
  if (big) return TILE_256;
  // TN: both operands go through the transposing LDS reads (two per fragment): the 64x64 wave tile of the
  // split-slab form needs a third fewer of them per MFMA, worth 5-7 % on the weight-gradient shapes; the
  // K-contiguous layouts gain nothing from it
  if (K % 256 == 0 && t128 >= 160) return layout == GEMM_TN ? TILE_128_SPLITSLAB : TILE_128_LOADERS;
  if (K % 128 == 0 && (t128 >= 160 || K % 256 != 0)) return TILE_128_REGS;
  if (K % 256 == 0 && K >= 1024) return TILE_128x64_LOADERS;
  if (K % 256 == 0) return TILE_128x64_DEEP;
  return TILE_GENERAL;
}

template <int LAYOUT, bool F16>
static void launch_bf16(int epi, int act, int M, int N, int K, const void* A, const void* B, void* C,
                        const void* bias, const void* aux_in, void* aux_out, hipStream_t st, bool solo, float* ws,
                        size_t ws_bytes) {
  if (ws && select_tile(LAYOUT, M, N, K, false) == TILE_256) {
    // (with a workspace the thin last round in K ranges also beats the full grid of 128x128 tiles that a GEMM running
    // alone would otherwise take: 359 against 397 us for the 8192 x 2560 x 10240 NT product)
    const HybridPlan hp = hybrid_plan(epi, M, N, K);
    if (hp.ws_bytes && hp.ws_bytes <= ws_bytes) {
      launch_hybrid<LAYOUT, F16>(hp, epi, M, N, K, A, B, C, aux_in, ws, st);
      return;
    }
  }
  switch (select_tile(LAYOUT, M, N, K, solo)) {
    case TILE_256:
      // NT: four loader wavefronts beside the eight that compute (168 registers: three wavefronts per SIMD fit; the
      // NN/TN instances need 190-230, so their wavefronts load their own shares)
      if constexpr (LAYOUT == GEMM_NT) launch_bf16_tile<LAYOUT, 256, 256, 64, 2, 4, 1, 2, 2, 4, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
      else launch_bf16_tile<LAYOUT, 256, 256, 64, 2, 4, 1, 2, 2, 0, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
      break;
    case TILE_128_SPLITSLAB:
      launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 2, 2, 2, 4, 4, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st); break;
    case TILE_128_LOADERS:
      launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 4, 1, 2, 4, 4, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st); break;
    case TILE_128_REGS:
      launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 4, 1, 2, 0, 0, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st); break;
    case TILE_128x64_LOADERS:
      launch_bf16_tile<LAYOUT, 128, 64, 64, 2, 2, 1, 2, 4, 4, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st); break;
    case TILE_128x64_DEEP:
      launch_bf16_tile<LAYOUT, 128, 64, 128, 2, 2, 2, 2, 0, 0, false, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st); break;
    default:
      launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 2, 1, 1, 0, 0, true, F16>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st); break;
  }
}

// ---- weight gradients with few output tiles: several K ranges per tile ---------------------------------
// C (+)= sum over the ranges of the fp32 partial tiles, added in range order (so the result does not depend on
// which workgroup finished first), eight columns per thread.
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(int64_t chunks, int64_t mn, int splits,
                                                            const float* __restrict__ ws, T* C, int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= chunks) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    float v[8];
    load8(ws + (int64_t)s * mn + i * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  if (accumulate) {
    float v[8];
    load8(C + i * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  store8(C + i * 8, acc);
}

// Number of K ranges for a weight gradient: 1 (plain GEMM) unless the 128x128 tiles leave most of the chip idle
// and K is long; then as many as bring the grid to about one workgroup per CU, each range at least 48 slabs
// (measured: at M = N = 1024 four ranges take 41 us against 70 us at K = 16384, but 22.5 against 20.4 at K = 4096,
// where the second kernel and the partial tiles cost more than the idle CUs).
static int weight_grad_splits(int M, int N, int K) {
  static const bool disabled = debug_flag("no-splitk");   // A/B timing
  if (disabled || K % 256 != 0 || N % 8 != 0) return 1;
  const int64_t t128 = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
  if (t128 >= 160) return 1;
  int64_t s = 256 / t128;
  const int64_t by_len = (K / 64) / 48;
  if (s > by_len) s = by_len;
  if (s > 8) s = 8;
  return s < 2 ? 1 : (int)s;
}

size_t gemm_ws_bytes(int dtype, int epi, int M, int N, int K) {
  return dtype == DT_FP32 ? 0 : hybrid_plan(epi, M, N, K).ws_bytes;
}

size_t weight_grad_ws_bytes(int dtype, int M, int N, int K) {
  if (dtype == DT_FP32) return 0;
  const int s = weight_grad_splits(M, N, K);
  return s > 1 ? (size_t)s * M * N * sizeof(float) : hybrid_plan(EPI_NONE, M, N, K).ws_bytes;   // (same for the add epilogue)
}

template <bool F16>
static void launch_splitk(int splits, int accumulate, int M, int N, int K, const void* A, const void* B, void* C,
                          float* ws, hipStream_t st) {
  constexpr int BM = 128, BN = 128;
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const size_t lds = gemm_lds_bytes<BM, BN, 64, 2, 2, 2, 4>();
  auto kern = gemm_bf16_kernel<GEMM_TN, BM, BN, 64, 2, 2, 2, 2, 4, 4, false, EPI_SPLITK, F16>;
  (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(tiles * splits), dim3((2 * 2 * 2 + 4) * 64), lds, st, M, N, K, (const bf16_t*)A,
                     (const bf16_t*)B, (bf16_t*)C, (const bf16_t*)nullptr, (const bf16_t*)nullptr,
                     reinterpret_cast<bf16_t*>(ws), splits, tiles * splits, 1, (float*)nullptr);
  const int64_t mn = (int64_t)M * N, chunks = mn / 8;
  const dim3 grid((unsigned)((chunks + 255) / 256));
  if (F16) hipLaunchKernelGGL(splitk_reduce_kernel<f16_t>, grid, dim3(256), 0, st, chunks, mn, splits, ws, (f16_t*)C, accumulate);
  else hipLaunchKernelGGL(splitk_reduce_kernel<bf16_t>, grid, dim3(256), 0, st, chunks, mn, splits, ws, (bf16_t*)C, accumulate);
}

void launch_weight_grad(int dtype, int accumulate, int M, int N, int K, const void* A, const void* B, void* C,
                        float* ws, hipStream_t st, bool solo) {
  const int splits = (ws && dtype != DT_FP32) ? weight_grad_splits(M, N, K) : 1;
  if (splits == 1) {
    launch_gemm(dtype, GEMM_TN, accumulate ? EPI_ADD : EPI_NONE, 0, M, N, K, A, B, C, nullptr, accumulate ? C : nullptr,
                nullptr, st, solo, ws, ws ? weight_grad_ws_bytes(dtype, M, N, K) : 0);
    return;
  }
  if (dtype == DT_FP16) launch_splitk<true>(splits, accumulate, M, N, K, A, B, C, ws, st);
  else launch_splitk<false>(splits, accumulate, M, N, K, A, B, C, ws, st);
}

// The kernel instance a GEMM of this shape runs as, in the spelling of the kernel's template arguments
// (layout, BM, BN, BK, WGM, WGN, KS, PF, NS, PW, KTAIL, epilogue, F16, HYB), as the profiler prints the symbol; for
// the weight-gradient path (`weight_grad`) with its K ranges, if any.
void describe_gemm(int dtype, int layout, int epi, int M, int N, int K, bool solo, bool weight_grad, bool with_ws,
                   char* buf, size_t len) {
  if (dtype == DT_FP32) { snprintf(buf, len, "gemm_f32_kernel<%d>", layout); return; }
  const int f16 = dtype == DT_FP16 ? 1 : 0;
  const char* b = f16 ? "true" : "false";
  if (with_ws && !(weight_grad && weight_grad_splits(M, N, K) > 1) && select_tile(layout, M, N, K, false) == TILE_256) {
    const HybridPlan hp = hybrid_plan(weight_grad ? EPI_NONE : epi, M, N, K);
    if (hp.ws_bytes) {
      snprintf(buf, len, "gemm_bf16_kernel<%d, 256, 256, 64, 2, 4, 1, 2, 2, %d, false, %d, %s, true> (%d tiles + %d tiles in %d K ranges) + hybrid_reduce_kernel",
               layout, layout == GEMM_NT ? 4 : 0, epi, b, hp.tail_begin, hp.tail_tiles, hp.splits);
      return;
    }
  }
  if (weight_grad) {
    const int splits = weight_grad_splits(M, N, K);
    if (splits > 1) {
      snprintf(buf, len, "gemm_bf16_kernel<2, 128, 128, 64, 2, 2, 2, 2, 4, 4, false, %d, %s, false> in %d K ranges + splitk_reduce_kernel", EPI_SPLITK, b, splits);
      return;
    }
  }
  static const char* const shape[] = {"256, 256, 64, 2, 4, 1, 2, 2, 0, false", "128, 128, 64, 2, 2, 2, 2, 4, 4, false",
                                      "128, 128, 64, 2, 4, 1, 2, 4, 4, false", "128, 128, 64, 2, 4, 1, 2, 0, 0, false",
                                      "128, 64, 64, 2, 2, 1, 2, 4, 4, false", "128, 64, 128, 2, 2, 2, 2, 0, 0, false",
                                      "128, 128, 64, 2, 2, 1, 1, 0, 0, true"};
  TileKind k = select_tile(layout, M, N, K, solo);
  if (k != TILE_GENERAL && !epi_used(layout, epi)) k = TILE_GENERAL;   // epilogues the layer never pairs with this layout
  if (k == TILE_256 && layout == GEMM_NT) snprintf(buf, len, "gemm_bf16_kernel<0, 256, 256, 64, 2, 4, 1, 2, 2, 4, false, %d, %s, false>", epi, b);
  else snprintf(buf, len, "gemm_bf16_kernel<%d, %s, %d, %s, false>", layout, shape[(int)k], epi, b);
}

void launch_gemm(int dtype, int layout, int epi, int act, int M, int N, int K, const void* A, const void* B,
                 void* C, const void* bias, const void* aux_in, void* aux_out, hipStream_t st, bool solo, float* ws,
                 size_t ws_bytes) {
  if (dtype == DT_FP32) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
#define SLAPO_F32(L)                                                                                      \
  hipLaunchKernelGGL(gemm_f32_kernel<L>, grid, dim3(256), 0, st, M, N, K, (const float*)A, (const float*)B, \
                     (float*)C, (const float*)bias, (const float*)aux_in, (float*)aux_out, epi, act)
    if (layout == GEMM_NT) SLAPO_F32(GEMM_NT);
    else if (layout == GEMM_NN) SLAPO_F32(GEMM_NN);
    else SLAPO_F32(GEMM_TN);
#undef SLAPO_F32
    return;
  }
#define SLAPO_H(F)                                                                                          \
  if (layout == GEMM_NT) launch_bf16<GEMM_NT, F>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st, solo, ws, ws_bytes);     \
  else if (layout == GEMM_NN) launch_bf16<GEMM_NN, F>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st, solo, ws, ws_bytes); \
  else launch_bf16<GEMM_TN, F>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st, solo, ws, ws_bytes)
  if (dtype == DT_FP16) { SLAPO_H(true); } else { SLAPO_H(false); }
#undef SLAPO_H
}

}  // namespace slapo
