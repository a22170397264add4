// GEMMs of the scheduled layer: the fused-QKV / output / FFN projections (paper section 2.2 step 1,
// appendix schedule) and the eight backward products, with the bias, bias+activation, activation
// derivative and residual-add epilogues applied to the fp32 accumulators in registers.
//
// bf16 path: 256 threads = 4 wavefronts in a 2x2 grid, each owning a (BM/2)x(BN/2) block of
// v_mfma_f32_32x32x16_bf16 tiles; 64-deep K slabs are staged global -> registers -> LDS with two LDS
// stages and one barrier per slab. Operands whose contraction index is contiguous in memory are read
// from LDS with 16-byte reads; operands whose contraction index is the strided one (the "N" operand
// of dY*W and both operands of dY^T*X) stay in their memory order in LDS and are read with the
// transposing ds_read_b64_tr_b16, so no transposed copy of any tensor is ever made.
// fp32 path: a plain LDS-tiled FMA kernel (correctness mode).
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
__device__ __forceinline__ float gelu_fast(float u) { return u * gelu_terms(u).phi; }
__device__ __forceinline__ float gelu_grad_fast(float u) {
  const GeluTerms g = gelu_terms(u);
  return fmaf(u * g.e, 0.39894228040143268f, g.phi);
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
    T u;
    from_f32(u, v);
    aux_out[idx] = u;
    v = act_fwd(to_f32(u), act);  // activation of the stored pre-activation, as backward will see it
  } else if (epi == EPI_DACT) {
    v *= act_grad(to_f32(aux_in[idx]), act);
  } else if (epi == EPI_ADD) {
    v += to_f32(aux_in[idx]);
  }
  from_f32(C[idx], v);
}

// LDS layouts. The LDS serves 256 B per clock (64 banks of 4 B): 16 lanes of a 16-byte access, and 16
// lanes of a transposing 8-byte read, are served together, so both the stores of a slab and the fragment
// reads have to spread 16 lanes over all banks.
//  - K-contiguous tile [rows][BK], unpadded, 16-byte chunk c of row r stored at chunk c ^ swz(r) with
//    swz(r) = (r / RP) % (BK/8), RP = rows per 256 B: a store (16 lanes = 256 consecutive bytes of the
//    tile) stays a permutation inside each row, and a fragment read (one chunk of 16 consecutive rows)
//    lands in 16 different 16-byte bank groups. swz depends on the lane only (wave tiles start at
//    multiples of 32 rows), so a fragment address is a per-lane base plus (2*ks ^ per-lane constant).
//  - M-contiguous tile [BK][rows]: stores are whole rows; 16 lanes read 4 consecutive k-rows x 32 B, and a
//    pitch of 2*rows + 32 bytes keeps the four rows apart.
template <int LAYOUT, int BM, int BN, int BK, int WGM, int WGN, int KS, int PF, bool KTAIL, int EPI>
__global__ __launch_bounds__(WGM * WGN * KS * 64) void gemm_bf16_kernel(int M, int N, int K,
                                                                  const bf16_t* __restrict__ A,
                                                                  const bf16_t* __restrict__ B,
                                                                  bf16_t* __restrict__ C,
                                                                  const bf16_t* __restrict__ bias,
                                                                  const bf16_t* aux_in,
                                                                  bf16_t* __restrict__ aux_out, int act) {
  constexpr bool A_KC = (LAYOUT != GEMM_TN);  // A operand contiguous along K
  constexpr bool B_KC = (LAYOUT == GEMM_NT);
  // KS == 2: two sets of WGM x WGN wavefronts share the output tile; set g multiplies the g-th half of
  // every K slab and the two accumulator sets are added through LDS before the epilogue. This doubles the
  // wavefronts per SIMD without shrinking the per-wave tile (LDS traffic per flop stays that of the
  // larger wave tile).
  constexpr int NTHR = WGM * WGN * KS * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  constexpr int A_LOADS = BM * BK / 8 / NTHR, B_LOADS = BN * BK / 8 / NTHR;
  static_assert(A_LOADS >= 1 && B_LOADS >= 1, "tile too small for the thread count");
  static_assert(BK == 64 || BK == 128, "swizzle written for 128- and 256-byte tile rows");
  constexpr int PA = A_KC ? BK : BM + 16;   // row pitch of the A tile in elements
  constexpr int PB = B_KC ? BK : BN + 16;
  constexpr int RP = 128 / BK;              // K-contiguous tile rows per 256 B
  auto swz = [](int row) { return (row / RP) % (BK / 8); };
  constexpr int SA = A_KC ? BM * PA : BK * PA;  // elements per stage
  constexpr int SB = B_KC ? BN * PB : BK * PB;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* sA = smem;            // [2][SA]
  bf16_t* sB = smem + 2 * SA;   // [2][SB]

  // Workgroups are handed to the 8 XCDs round-robin. Renumber them so that each XCD (own L2) gets a
  // run of consecutive tile ids, and order the ids in groups of 4 tile rows walked column by column, so
  // that the tiles an XCD works on at the same time form a compact block: its workgroups walk K in step,
  // and every A (B) slab that reaches the L2 is used by all tiles of its row (column) in the block.
  const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
  const int nblk = tiles_m * tiles_n;
  int bid = blockIdx.x;
  const int per_xcd = nblk / 8;
  if (bid < per_xcd * 8) bid = (bid & 7) * per_xcd + (bid >> 3);
  constexpr int GROUP_M = 4;
  const int group = bid / (GROUP_M * tiles_n);
  const int first_m = group * GROUP_M;
  const int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  const int in_group = bid - group * GROUP_M * tiles_n;
  const int tile_m = first_m + in_group % gsz, tile_n = in_group / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int kgroup = (tid >> 6) / (WGM * WGN), wave = (tid >> 6) % (WGM * WGN);
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

  // Each thread moves A_LOADS + B_LOADS 16-byte pieces per slab. Piece i of a thread sits RSA (RSB) tile
  // rows below piece 0. Pieces outside M or N are read from a clamped (valid) address and never reach a
  // stored output, so only the K tail needs zero fill; all loads are unconditional, which lets the
  // compiler keep the next slabs' loads in flight while it waits for the oldest ones only.
  constexpr int CA = A_KC ? BK / 8 : BM / 8, CB = B_KC ? BK / 8 : BN / 8;   // pieces per tile row
  constexpr int RSA = NTHR / CA, RSB = NTHR / CB;                            // tile rows between pieces
  const int ar = tid / CA, ac = (tid % CA) * 8, br = tid / CB, bc = (tid % CB) * 8;
  const int lda = A_KC ? K : M, ldb = B_KC ? K : N;
  const bf16_t* ga[A_LOADS];
  const bf16_t* gb[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    if (A_KC) { int r = m0 + ar + i * RSA; r = r < M ? r : M - 1; ga[i] = A + (int64_t)r * lda + ac; }
    else { int c = m0 + ac; c = c < M ? c : M - 8; ga[i] = A + (int64_t)(ar + i * RSA) * lda + c; }
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    if (B_KC) { int r = n0 + br + i * RSB; r = r < N ? r : N - 1; gb[i] = B + (int64_t)r * ldb + bc; }
    else { int c = n0 + bc; c = c < N ? c : N - 8; gb[i] = B + (int64_t)(br + i * RSB) * ldb + c; }
  }
  const int64_t stepA = A_KC ? BK : (int64_t)BK * lda, stepB = B_KC ? BK : (int64_t)BK * ldb;
  static_assert(!A_KC || RSA % 32 == 0, "pieces of a thread must share the swizzle");
  static_assert(!B_KC || RSB % 32 == 0, "pieces of a thread must share the swizzle");
  const int la0 = A_KC ? ar * PA + (((ac >> 3) ^ swz(ar)) << 3) : ar * PA + ac;
  const int lb0 = B_KC ? br * PB + (((bc >> 3) ^ swz(br)) << 3) : br * PB + bc;

  const int nk = (K + BK - 1) / BK;
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
    bf16_t* a = sA + stage * SA + la0;
    bf16_t* b = sB + stage * SB + lb0;
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) *reinterpret_cast<u32x4_t*>(a + i * RSA * PA) = ra[i];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) *reinterpret_cast<u32x4_t*>(b + i * RSB * PB) = rb[i];
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per-lane fragment bases (stage 0, 32-row tile 0, k-step 0)
  // K-contiguous: chunk 2*ks + lane/32 of row lane%32, at (2*ks + lane/32) ^ swz = (2*ks ^ fsw) with the
  // low bit folded into the base
  const int fsw = swz(lane & 31) & ~1;
  const int fa_base = A_KC ? (wm0 + (lane & 31)) * PA + ((((lane >> 5) ^ swz(lane & 31)) & 1) << 3)
                           : (8 * (lane >> 5) + ((lane & 15) >> 2)) * PA + wm0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const int fb_base = B_KC ? (wn0 + (lane & 31)) * PB + ((((lane >> 5) ^ swz(lane & 31)) & 1) << 3)
                           : (8 * (lane >> 5) + ((lane & 15) >> 2)) * PB + wn0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  auto frag = [&](const bf16_t* tile, auto kc_tag, int base, int pitch, int t, int ks) -> bf16x8_t {
    if constexpr (decltype(kc_tag)::value) {
      return *reinterpret_cast<const bf16x8_t*>(tile + base + t * 32 * pitch + (((2 * ks) ^ fsw) << 3));
    } else {
      const bf16_t* p0 = tile + base + ks * 16 * pitch + t * 32;
      s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p0);
      s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p0 + 4 * pitch));
      typedef short s16x8_t __attribute__((ext_vector_type(8)));
      s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, v);
    }
  };
  auto compute = [&](int stage) {
    const bf16_t* a = sA + stage * SA;
    const bf16_t* b = sB + stage * SB;
    // scheduling hint for the slab: interleave the LDS reads with the MFMAs (variant chosen by measurement)
    __builtin_amdgcn_iglp_opt(LAYOUT == GEMM_TN ? 1 : 0);
#pragma unroll
    for (int kq = 0; kq < BK / 16 / KS; ++kq) {
      const int ks = kq + kgroup * (BK / 16 / KS);
      bf16x8_t fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = frag(a, std::integral_constant<bool, A_KC>{}, fa_base, PA, i, ks);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = frag(b, std::integral_constant<bool, B_KC>{}, fb_base, PB, j, ks);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  // Pipeline: the slab of k-step k is computed from LDS stage k&1 while the global loads of the next PF
  // slabs are in flight in registers (register set k % PF holds slab k); a slab is written to LDS right
  // after the compute of the step before it. With PF == 2 the slab count must be even (the host falls
  // back to PF == 1 otherwise). Loads and stores are issued on every step (slab index clamped; the last
  // steps re-fetch the last slab into a stage nobody reads): with every step alike, the wait before an
  // LDS store covers the oldest slab only and the newer loads stay in flight.
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
  if ((EPI == EPI_BIAS || EPI == EPI_BIAS_ACT) && n < N) load8(bias + n, bv);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
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
      if (m < M && n < N) {
        const int64_t idx = (int64_t)m * N + n;
        if (EPI == EPI_BIAS) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bv[e];
        } else if (EPI == EPI_BIAS_ACT) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bv[e];
          store8(aux_out + idx, v);
          // activation of the stored (rounded) pre-activation, the value backward will differentiate at
          if (act == ACT_RELU) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = gelu_fast(bf16_to_f32(f32_to_bf16(v[e])));
          }
        } else if (EPI == EPI_DACT) {
          float u[8];
          load8(aux_in + idx, u);
          if (act == ACT_RELU) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = u[e] > 0.f ? v[e] : 0.f;
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_fast(u[e]);
          }
        } else if (EPI == EPI_ADD) {
          float u[8];
          load8(aux_in + idx, u);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += u[e];
        }
        store8(C + idx, v);
      }
    }
  }
}

template <int LAYOUT, int BM, int BN, int BK, int WGM, int WGN, int KS>
constexpr size_t gemm_lds_bytes() {
  constexpr bool A_KC = (LAYOUT != GEMM_TN), B_KC = (LAYOUT == GEMM_NT);
  constexpr size_t SA = A_KC ? BM * BK : BK * (BM + 16);
  constexpr size_t SB = B_KC ? BN * BK : BK * (BN + 16);
  constexpr size_t main_bytes = 2 * (SA + SB) * sizeof(bf16_t);
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
      if (m < M && n < N) epilogue_store<float>(epi, act, acc[i][j], m, n, N, C, bias, aux_in, aux_out);
    }
}

// epilogue / layout pairs the layer itself uses; only these get the tuned (deep-prefetch) kernels
constexpr bool epi_used(int layout, int epi) {
  return layout == GEMM_NT ? (epi == EPI_NONE || epi == EPI_BIAS || epi == EPI_BIAS_ACT)
       : layout == GEMM_NN ? (epi == EPI_NONE || epi == EPI_DACT || epi == EPI_ADD)
                           : (epi == EPI_NONE || epi == EPI_ADD);
}

template <int LAYOUT, int BM, int BN, int BK, int WGM, int WGN, int KS, int PF, bool KTAIL>
static void launch_bf16_tile(int epi, int act, int M, int N, int K, const void* A, const void* B, void* C,
                             const void* bias, const void* aux_in, void* aux_out, hipStream_t st) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const size_t lds = gemm_lds_bytes<LAYOUT, BM, BN, BK, WGM, WGN, KS>();
#define SLAPO_GEMM(E)                                                                                       \
  do {                                                                                                      \
    if constexpr (KTAIL || epi_used(LAYOUT, E)) {                                                           \
      auto kern = gemm_bf16_kernel<LAYOUT, BM, BN, BK, WGM, WGN, KS, PF, KTAIL, E>;                             \
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);  \
      hipLaunchKernelGGL(kern, dim3(tiles), dim3(WGM * WGN * KS * 64), lds, st, M, N, K, (const bf16_t*)A,       \
                         (const bf16_t*)B, (bf16_t*)C, (const bf16_t*)bias, (const bf16_t*)aux_in,          \
                         (bf16_t*)aux_out, act);                                                            \
    } else {                                                                                                \
      launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 2, 1, 1, true>(epi, act, M, N, K, A, B, C, bias, aux_in,       \
                                                           aux_out, st);                                    \
    }                                                                                                       \
  } while (0)
  switch (epi) {
    case EPI_NONE: SLAPO_GEMM(EPI_NONE); break;
    case EPI_BIAS: SLAPO_GEMM(EPI_BIAS); break;
    case EPI_BIAS_ACT: SLAPO_GEMM(EPI_BIAS_ACT); break;
    case EPI_DACT: SLAPO_GEMM(EPI_DACT); break;
    default: SLAPO_GEMM(EPI_ADD); break;
  }
#undef SLAPO_GEMM
}

// Tile selection, from measurements on the layer's shapes: 256x256 tiles (8 wavefronts, 128x64 each) when
// they still cover at least three quarters of the 256 CUs; otherwise 128x128 (8 wavefronts, 64x32 each);
// for outputs with few tiles 128x64 tiles with 128-deep slabs and two wave sets splitting each slab. All
// use two slabs of register prefetch, which needs an even number of whole slabs; other K go to the general
// kernel (one slab, zero-filled tail).
template <int LAYOUT>
static void launch_bf16(int epi, int act, int M, int N, int K, const void* A, const void* B, void* C,
                        const void* bias, const void* aux_in, void* aux_out, hipStream_t st) {
  const int64_t t256 = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
  const int64_t t128 = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
  if (K % 128 == 0 && t256 >= 192)
    launch_bf16_tile<LAYOUT, 256, 256, 64, 2, 4, 1, 2, false>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
  else if (K % 128 == 0 && (t128 >= 160 || K % 256 != 0))
    launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 4, 1, 2, false>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
  else if (K % 256 == 0)
    launch_bf16_tile<LAYOUT, 128, 64, 128, 2, 2, 2, 2, false>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
  else
    launch_bf16_tile<LAYOUT, 128, 128, 64, 2, 2, 1, 1, true>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
}

void launch_gemm(int dtype_fp32, int layout, int epi, int act, int M, int N, int K, const void* A, const void* B,
                 void* C, const void* bias, const void* aux_in, void* aux_out, hipStream_t st) {
  if (dtype_fp32) {
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
  if (layout == GEMM_NT) launch_bf16<GEMM_NT>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
  else if (layout == GEMM_NN) launch_bf16<GEMM_NN>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
  else launch_bf16<GEMM_TN>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
}

}  // namespace slapo
