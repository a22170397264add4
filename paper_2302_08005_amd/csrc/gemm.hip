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
#include "common.h"
#include "kernels.h"

namespace slapo {

enum { ACT_GELU = 0, ACT_RELU = 1 };

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

constexpr int BK = 64;

// 16-byte chunk position inside an LDS row: rows that one LDS instruction touches together land in
// different bank groups. K-contiguous tiles are read 8 rows x 16 B at a time, transposed-read tiles
// 4 rows x 32 B at a time.
__device__ __forceinline__ int swz_kc(int row, int chunk) { return chunk ^ (row & 7); }
__device__ __forceinline__ int swz_mc(int krow, int chunk) { return chunk ^ ((krow & 3) << 1); }

template <int LAYOUT, int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                        const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
                                                        const bf16_t* __restrict__ bias, const bf16_t* aux_in,
                                                        bf16_t* __restrict__ aux_out, int act) {
  constexpr bool A_KC = (LAYOUT != GEMM_TN);  // A operand contiguous along K
  constexpr bool B_KC = (LAYOUT == GEMM_NT);
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  constexpr int A_LOADS = BM * BK / 8 / 256, B_LOADS = BN * BK / 8 / 256;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* sA = smem;                  // [2][BM*BK]
  bf16_t* sB = smem + 2 * BM * BK;    // [2][BN*BK]

  // Workgroups are handed to the 8 XCDs round-robin; renumber them so that each XCD (own L2) works
  // on a contiguous band of output tiles and re-reads the same operand panels.
  const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
  const int nblk = tiles_m * tiles_n;
  int bid = blockIdx.x;
  const int per_xcd = nblk / 8;
  if (bid < per_xcd * 8) bid = (bid & 7) * per_xcd + (bid >> 3);
  const int tile_m = bid / tiles_n, tile_n = bid % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
  const int lda = A_KC ? K : M, ldb = B_KC ? K : N;

  uint4 ra[A_LOADS], rb[B_LOADS];

  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
      const int q = tid + i * 256;
      int row, col;  // row/col in memory order of the tile
      if (A_KC) { row = m0 + q / 8; col = k0 + (q % 8) * 8; }
      else { row = k0 + q / (BM / 8); col = m0 + (q % (BM / 8)) * 8; }
      const bool ok = A_KC ? (row < M && col < K) : (row < K && col < M);
      ra[i] = ok ? *reinterpret_cast<const uint4*>(A + (int64_t)row * lda + col) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
      const int q = tid + i * 256;
      int row, col;
      if (B_KC) { row = n0 + q / 8; col = k0 + (q % 8) * 8; }
      else { row = k0 + q / (BN / 8); col = n0 + (q % (BN / 8)) * 8; }
      const bool ok = B_KC ? (row < N && col < K) : (row < K && col < N);
      rb[i] = ok ? *reinterpret_cast<const uint4*>(B + (int64_t)row * ldb + col) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_lds = [&](int stage) {
    bf16_t* a = sA + stage * BM * BK;
    bf16_t* b = sB + stage * BN * BK;
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
      const int q = tid + i * 256;
      int off;
      if (A_KC) { const int r = q / 8, c = q % 8; off = r * BK + swz_kc(r, c) * 8; }
      else { const int r = q / (BM / 8), c = q % (BM / 8); off = r * BM + swz_mc(r, c) * 8; }
      *reinterpret_cast<uint4*>(a + off) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
      const int q = tid + i * 256;
      int off;
      if (B_KC) { const int r = q / 8, c = q % 8; off = r * BK + swz_kc(r, c) * 8; }
      else { const int r = q / (BN / 8), c = q % (BN / 8); off = r * BN + swz_mc(r, c) * 8; }
      *reinterpret_cast<uint4*>(b + off) = rb[i];
    }
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment of a 32-row tile starting at `r0` (tile-local row) for the 16-deep step ks
  auto frag_kc = [&](const bf16_t* tile, int r0, int ks) -> bf16x8_t {
    const int r = r0 + (lane & 31), c = ks * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8_t*>(tile + r * BK + swz_kc(r, c) * 8);
  };
  auto frag_mc = [&](const bf16_t* tile, int ld, int r0, int ks) -> bf16x8_t {
    const int j = lane & 15, g = lane >> 4;
    const int k = ks * 16 + 8 * (g >> 1) + (j >> 2);
    const int m = r0 + 16 * (g & 1) + 4 * (j & 3);
    const bf16_t* p0 = tile + k * ld + swz_mc(k, m >> 3) * 8 + (m & 7);
    const bf16_t* p1 = tile + (k + 4) * ld + swz_mc(k + 4, m >> 3) * 8 + (m & 7);
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p0);
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p1);
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  };

  const int nk = (K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < nk) load_global((kt + 1) * BK);
    const bf16_t* a = sA + stage * BM * BK;
    const bf16_t* b = sB + stage * BN * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = A_KC ? frag_kc(a, wm0 + i * 32, ks) : frag_mc(a, BM, wm0 + i * 32, ks);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = B_KC ? frag_kc(b, wn0 + j * 32, ks) : frag_mc(b, BN, wn0 + j * 32, ks);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(stage ^ 1);
    __syncthreads();
  }

  // Epilogue. The accumulators (element r of a 32x32 tile: row (r/4)*8 + 4*(lane/32) + r%4, column
  // lane%32) go through a per-wave fp32 staging area in LDS so that every global access of the epilogue
  // (bias, auxiliary input, both outputs) is a 16-byte access of 8 consecutive columns of one row.
  // The main loop ended with a barrier, so the operand stages are free to be overwritten.
  constexpr int LDP = WN + 4;
  float* stage = reinterpret_cast<float*>(smem) + wave * (WM * LDP);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stage[(i * 32 + (r >> 2) * 8 + 4 * (lane >> 5) + (r & 3)) * LDP + j * 32 + (lane & 31)] = acc[i][j][r];
  __builtin_amdgcn_wave_barrier();
  constexpr int CPR = WN / 8;         // 8-column chunks per staged row
  constexpr int RPP = 64 / CPR;       // rows covered by one pass of the wave
  const int cc = lane % CPR, rr = lane / CPR;
  const int n = n0 + wn0 + cc * 8;
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if ((EPI == EPI_BIAS || EPI == EPI_BIAS_ACT) && n < N) load8(bias + n, bv);
#pragma unroll 4
  for (int pass = 0; pass < WM / RPP; ++pass) {
    const int row = pass * RPP + rr;
    const int m = m0 + wm0 + row;
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
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = act_fwd(bf16_to_f32(f32_to_bf16(v[e])), act);
      } else if (EPI == EPI_DACT) {
        float u[8];
        load8(aux_in + idx, u);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= act_grad(u[e], act);
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

template <int LAYOUT, int BM, int BN>
static void launch_bf16_tile(int epi, int act, int M, int N, int K, const void* A, const void* B, void* C,
                             const void* bias, const void* aux_in, void* aux_out, hipStream_t st) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const size_t lds_main = (size_t)2 * (BM + BN) * BK * sizeof(bf16_t);
  const size_t lds_epi = (size_t)4 * (BM / 2) * (BN / 2 + 4) * sizeof(float);
  const size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
#define SLAPO_GEMM(E)                                                                                       \
  do {                                                                                                      \
    auto kern = gemm_bf16_kernel<LAYOUT, BM, BN, E>;                                                        \
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);    \
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), lds, st, M, N, K, (const bf16_t*)A, (const bf16_t*)B,  \
                       (bf16_t*)C, (const bf16_t*)bias, (const bf16_t*)aux_in, (bf16_t*)aux_out, act);      \
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

template <int LAYOUT>
static void launch_bf16(int epi, int act, int M, int N, int K, const void* A, const void* B, void* C,
                        const void* bias, const void* aux_in, void* aux_out, hipStream_t st) {
  // 256x128 tiles when they still give every CU at least two tiles; otherwise 128x128 for occupancy
  const int64_t t_big = (int64_t)((M + 255) / 256) * ((N + 127) / 128);
  if (t_big >= 512) launch_bf16_tile<LAYOUT, 256, 128>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
  else launch_bf16_tile<LAYOUT, 128, 128>(epi, act, M, N, K, A, B, C, bias, aux_in, aux_out, st);
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
