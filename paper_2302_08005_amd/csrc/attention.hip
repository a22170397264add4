// Fused softmax attention, forward and backward (paper section 2.2 step 2: attention computed block
// by block so that the S x S matrix never reaches memory; the appendix schedule swaps it in for the
// matched scaled-dot-product pattern). Works in place on the packed projection [B,S,3H] = Q | K | V,
// so no head transposes are materialised.
//
// bf16 path. A workgroup of four wavefronts owns 128 query rows (forward, dQ) or 128 key rows (dK/dV)
// of one (sample, head); each wavefront owns 32 of them and walks the other sequence dimension in
// 64-row tiles staged through LDS (two stages, one barrier per tile). All products run on
// v_mfma_f32_32x32x16_bf16 and are arranged "transposed" (S^T = K Q^T, O^T = V^T P^T, ...), because
// then the accumulator layout of the score tile already is the B-operand layout of the next product
// and the per-row softmax state (max, sum, logsumexp, delta) is one scalar per lane; a row's maximum
// and sum need the lane's own 16..32 registers plus a single exchange with lane^32. The operand whose
// contraction index is the strided one in LDS is fetched with the transposing ds_read_b64_tr_b16.
// Backward recomputes the probabilities from the saved logsumexp and is split in two kernels (dK/dV
// per key tile, dQ per query tile) so that no floating-point atomics are needed.
//
// fp32 path: one wavefront per row, plain loops (correctness mode).
#include "common.h"
#include "kernels.h"

namespace slapo {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// ---- LDS tile [rows][D] of bf16, 16-byte chunks permuted inside each row -------------------------
// The LDS serves 256 B per clock (64 banks): 16 lanes of a 16-byte read, 32 lanes of a transposing
// 8-byte read. The same tile is read both ways -- 16 consecutive rows x one chunk, and 4 consecutive rows
// x four chunks -- and the XOR pattern below makes both conflict-free. With 128-byte rows (D = 64) rows
// of equal parity share banks; with 256-byte rows (D = 128) all rows do.
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  const int f = (D == 64) ? (((row & 2) << 1) | ((row >> 2) & 3)) : (((row & 3) << 2) | ((row >> 2) & 3));
  return row * D + ((chunk ^ f) << 3);
}
// MFMA operand whose 32 rows are tile rows r0.. and whose contraction runs along D (step s of 16)
template <int D>
__device__ __forceinline__ bf16x8_t frag_rows(const bf16_t* tile, int r0, int s, int lane) {
  const int r = r0 + (lane & 31);
  return *reinterpret_cast<const bf16x8_t*>(tile + tile_off<D>(r, 2 * s + (lane >> 5)));
}
// MFMA operand whose 32 rows are tile COLUMNS t*32.. and whose contraction runs over tile rows
// c0 + {4kc..4kc+3, 8+4kc..8+4kc+3} (kc = lane/32): the order in which a 32x32 accumulator holds them.
template <int D>
__device__ __forceinline__ bf16x8_t frag_tr(const bf16_t* tile, int c0, int t, int lane) {
  const int j = lane & 15, g = lane >> 4;
  const int row = c0 + 4 * (g >> 1) + (j >> 2);
  const int col = t * 32 + 16 * (g & 1) + 4 * (j & 3);
  const bf16_t* p0 = tile + tile_off<D>(row, col >> 3) + (col & 7);
  const bf16_t* p1 = tile + tile_off<D>(row + 8, col >> 3) + (col & 7);
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p0);
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p1);
  typedef short s16x8_t __attribute__((ext_vector_type(8)));
  s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}
// eight accumulator registers 8h..8h+7 as a bf16 operand
__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& v, int h) {
  uint4 w;
  w.x = pack_bf16x2(v[8 * h + 0], v[8 * h + 1]); w.y = pack_bf16x2(v[8 * h + 2], v[8 * h + 3]);
  w.z = pack_bf16x2(v[8 * h + 4], v[8 * h + 5]); w.w = pack_bf16x2(v[8 * h + 6], v[8 * h + 7]);
  return __builtin_bit_cast(bf16x8_t, w);
}
// row index inside a 32x32 accumulator tile of register r
__device__ __forceinline__ int acc_row(int r, int lane) { return (r >> 2) * 8 + 4 * (lane >> 5) + (r & 3); }

// 64 x D tile: global rows (clamped to `last_row`) -> registers -> LDS
template <int D>
struct TileMover {
  static constexpr int N = 64 * D / 8 / 256;
  uint4 r[N];
  __device__ __forceinline__ void load(const bf16_t* src, int64_t row_stride, int row0, int last_row, int tid,
                                       int zero_from) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int q = tid + i * 256, row = q / (D / 8), c = q % (D / 8);
      int gr = row0 + row;
      const bool zero = gr >= zero_from;
      gr = gr > last_row ? last_row : gr;
      r[i] = *reinterpret_cast<const uint4*>(src + (int64_t)gr * row_stride + c * 8);
      if (zero) r[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(bf16_t* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int q = tid + i * 256, row = q / (D / 8), c = q % (D / 8);
      *reinterpret_cast<uint4*>(tile + tile_off<D>(row, c)) = r[i];
    }
  }
};

__device__ __forceinline__ int visible_keys(const AttnShape& sh, const int32_t* seqlens, int b) {
  int n = sh.seq;
  if (seqlens) { const int v = seqlens[b]; n = v < n ? v : n; n = n < 0 ? 0 : n; }
  return n;
}

// =================================== forward =====================================================
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_bf16_kernel(AttnShape sh, const bf16_t* __restrict__ qkv,
                                                            const int32_t* __restrict__ seqlens,
                                                            bf16_t* __restrict__ out, float* __restrict__ lse) {
  constexpr int NS = D / 16, NT = D / 32;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];  // [2][K tile | V tile]
  const int S = sh.seq, H = sh.hidden;
  const int b = blockIdx.z, a = blockIdx.y, q_base = blockIdx.x * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kc = lane >> 5;
  const int64_t rs = 3 * (int64_t)H;
  const bf16_t* base = qkv + (int64_t)b * S * rs + a * D;
  const int kv_len = visible_keys(sh, seqlens, b);
  int kv_end = kv_len;
  if (sh.causal && q_base + 128 < kv_end) kv_end = q_base + 128;
  const int n_tiles = (kv_end + 63) / 64;
  const int my_q = q_base + 32 * wave + (lane & 31);
  const int q_ld = my_q < S ? my_q : S - 1;
  const int wave_q_max = q_base + 32 * wave + 31;
  const float sl2 = LOG2E * rsqrtf((float)D);

  bf16x8_t qf[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const bf16x8_t*>(base + q_ld * rs + 16 * s + 8 * kc);

  f32x16_t o[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  TileMover<D> mk, mv;
  if (n_tiles > 0) {
    mk.load(base + H, rs, 0, S - 1, tid, S);
    mv.load(base + 2 * H, rs, 0, S - 1, tid, S);
    mk.store(smem, tid);
    mv.store(smem + 64 * D, tid);
  }
  __syncthreads();
  for (int it = 0; it < n_tiles; ++it) {
    const int kv0 = it * 64;
    const bf16_t* kt = smem + (it & 1) * 128 * D;
    const bf16_t* vt = kt + 64 * D;
    if (it + 1 < n_tiles) {
      mk.load(base + H, rs, kv0 + 64, S - 1, tid, S);
      mv.load(base + 2 * H, rs, kv0 + 64, S - 1, tid, S);
    }
    if (!sh.causal || kv0 <= wave_q_max) {
      f32x16_t sc[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[i][r] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s)
          sc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(kt, i * 32, s, lane), qf[s], sc[i], 0, 0, 0);
      }
      const bool edge = (kv0 + 64 > kv_len) || (sh.causal && kv0 + 63 > q_base + 32 * wave);
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = sc[i][r] * sl2;
          if (edge) {
            const int kv = kv0 + i * 32 + acc_row(r, lane);
            if (kv >= kv_len || (sh.causal && kv > my_q)) v = -INFINITY;
          }
          sc[i][r] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m - m_safe);
      l *= alpha;
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] *= alpha;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(sc[i][r] - m_safe);
          sc[i][r] = p;
          l += p;
        }
      m = m_new;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const bf16x8_t pf = pack8(sc[i], h);
#pragma unroll
          for (int t = 0; t < NT; ++t)
            o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<D>(vt, i * 32 + 16 * h, t, lane), pf, o[t], 0, 0, 0);
        }
    }
    if (it + 1 < n_tiles) {
      bf16_t* nk = smem + ((it + 1) & 1) * 128 * D;
      mk.store(nk, tid);
      mv.store(nk + 64 * D, tid);
    }
    __syncthreads();
  }
  const float l_tot = l + __shfl_xor(l, 32, 64);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (my_q < S) {
    bf16_t* orow = out + ((int64_t)b * S + my_q) * H + a * D;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16x2(o[t][4 * g] * inv, o[t][4 * g + 1] * inv);
        w.y = pack_bf16x2(o[t][4 * g + 2] * inv, o[t][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(orow + t * 32 + g * 8 + 4 * kc) = w;
      }
    if (kc == 0) lse[((int64_t)b * sh.heads + a) * S + my_q] = l_tot > 0.f ? (m + __log2f(l_tot)) * LN2 : -INFINITY;
  }
}

// ============================ backward: delta = rowsum(dO * O) ===================================
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(AttnShape sh, const T* __restrict__ o,
                                                         const T* __restrict__ dout, float* __restrict__ delta) {
  // 8 lanes per (token, head); each lane D/8 elements
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t item = gid >> 3;
  const int sub = (int)(gid & 7);
  const int64_t total = (int64_t)sh.batch * sh.seq * sh.heads;
  float s = 0.f;
  int64_t tok = 0;
  int a = 0;
  if (item < total) {
    tok = item / sh.heads;
    a = (int)(item % sh.heads);
    const int64_t off = tok * sh.hidden + a * D + sub * (D / 8);
#pragma unroll
    for (int i = 0; i < D / 64; ++i) {
      float x[8], y[8];
      load8(o + off + i * 8, x);
      load8(dout + off + i * 8, y);
#pragma unroll
      for (int j = 0; j < 8; ++j) s += x[j] * y[j];
    }
  }
  s += __shfl_xor(s, 1, 64);
  s += __shfl_xor(s, 2, 64);
  s += __shfl_xor(s, 4, 64);
  if (item < total && sub == 0) {
    const int64_t bb = tok / sh.seq, i = tok % sh.seq;
    delta[(bb * sh.heads + a) * sh.seq + i] = s;
  }
}

// ============================ backward: dK, dV per key tile ======================================
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_bf16_kernel(AttnShape sh, const bf16_t* __restrict__ qkv,
                                                                 const int32_t* __restrict__ seqlens,
                                                                 const bf16_t* __restrict__ dout,
                                                                 const float* __restrict__ lse,
                                                                 const float* __restrict__ delta,
                                                                 bf16_t* __restrict__ dqkv) {
  constexpr int NS = D / 16, NT = D / 32;
  constexpr int STAGE = 128 * D + 256;  // bf16 units: Q tile, dO tile, 64 lse + 64 delta floats
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  const int S = sh.seq, H = sh.hidden;
  const int b = blockIdx.z, a = blockIdx.y, kv_base = blockIdx.x * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kc = lane >> 5;
  const int64_t rs = 3 * (int64_t)H;
  const bf16_t* base = qkv + (int64_t)b * S * rs + a * D;
  const bf16_t* dobase = dout + (int64_t)b * S * H + a * D;
  const float* lse_row = lse + ((int64_t)b * sh.heads + a) * S;
  const float* delta_row = delta + ((int64_t)b * sh.heads + a) * S;
  const int kv_len = visible_keys(sh, seqlens, b);
  const int my_kv = kv_base + 32 * wave + (lane & 31);
  const int kv_ld = my_kv < S ? my_kv : S - 1;
  const int wave_kv_min = kv_base + 32 * wave;
  const float scale = rsqrtf((float)D), sl2 = LOG2E * scale;

  bf16x8_t kf[NS], vf[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    kf[s] = *reinterpret_cast<const bf16x8_t*>(base + H + kv_ld * rs + 16 * s + 8 * kc);
    vf[s] = *reinterpret_cast<const bf16x8_t*>(base + 2 * H + kv_ld * rs + 16 * s + 8 * kc);
  }
  f32x16_t dk[NT], dv[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[t][r] = dv[t][r] = 0.f;

  const int q_first = sh.causal ? (kv_base / 64) : 0;
  const int q_tiles = (kv_base < kv_len) ? (S + 63) / 64 : q_first;  // nothing to do for fully hidden keys
  TileMover<D> mq, md;
  float aux = 0.f;
  auto load_tile = [&](int qt) {
    const int q0 = qt * 64;
    mq.load(base, rs, q0, S - 1, tid, S);
    md.load(dobase, H, q0, S - 1, tid, S);
    if (tid < 128) {
      const int q = q0 + (tid & 63);
      aux = 0.f;
      if (q < S) aux = tid < 64 ? lse_row[q] * LOG2E : delta_row[q];
    }
  };
  auto store_tile = [&](int stage) {
    bf16_t* t0 = smem + stage * STAGE;
    mq.store(t0, tid);
    md.store(t0 + 64 * D, tid);
    if (tid < 128) reinterpret_cast<float*>(t0 + 128 * D)[tid] = aux;
  };
  if (q_first < q_tiles) { load_tile(q_first); store_tile(0); }
  __syncthreads();
  for (int qt = q_first; qt < q_tiles; ++qt) {
    const int stage = (qt - q_first) & 1, q0 = qt * 64;
    const bf16_t* qtile = smem + stage * STAGE;
    const bf16_t* dtile = qtile + 64 * D;
    const float* stats = reinterpret_cast<const float*>(qtile + 128 * D);
    if (qt + 1 < q_tiles) load_tile(qt + 1);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (sh.causal && q0 + i * 32 + 31 < wave_kv_min) continue;  // every query of this sub-tile precedes my keys
      f32x16_t sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = dp[r] = 0.f;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(qtile, i * 32, s, lane), kf[s], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(dtile, i * 32, s, lane), vf[s], dp, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qi = i * 32 + acc_row(r, lane);
        const int q = q0 + qi;
        float p = __builtin_amdgcn_exp2f(sc[r] * sl2 - stats[qi]);
        if (my_kv >= kv_len || q >= S || (sh.causal && my_kv > q)) p = 0.f;
        sc[r] = p;
        dp[r] = p * (dp[r] - stats[64 + qi]);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8_t pf = pack8(sc, h), dsf = pack8(dp, h);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<D>(dtile, i * 32 + 16 * h, t, lane), pf, dv[t], 0, 0, 0);
          dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<D>(qtile, i * 32 + 16 * h, t, lane), dsf, dk[t], 0, 0, 0);
        }
      }
    }
    if (qt + 1 < q_tiles) store_tile(stage ^ 1);
    __syncthreads();
  }
  if (my_kv < S) {
    bf16_t* krow = dqkv + ((int64_t)b * S + my_kv) * rs + H + a * D;
    bf16_t* vrow = krow + H;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16x2(dk[t][4 * g] * scale, dk[t][4 * g + 1] * scale);
        w.y = pack_bf16x2(dk[t][4 * g + 2] * scale, dk[t][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(krow + t * 32 + g * 8 + 4 * kc) = w;
        w.x = pack_bf16x2(dv[t][4 * g], dv[t][4 * g + 1]);
        w.y = pack_bf16x2(dv[t][4 * g + 2], dv[t][4 * g + 3]);
        *reinterpret_cast<uint2*>(vrow + t * 32 + g * 8 + 4 * kc) = w;
      }
  }
}

// ============================ backward: dQ per query tile ========================================
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_bf16_kernel(AttnShape sh, const bf16_t* __restrict__ qkv,
                                                               const int32_t* __restrict__ seqlens,
                                                               const bf16_t* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta,
                                                               bf16_t* __restrict__ dqkv) {
  constexpr int NS = D / 16, NT = D / 32;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];  // [2][K tile | V tile]
  const int S = sh.seq, H = sh.hidden;
  const int b = blockIdx.z, a = blockIdx.y, q_base = blockIdx.x * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kc = lane >> 5;
  const int64_t rs = 3 * (int64_t)H;
  const bf16_t* base = qkv + (int64_t)b * S * rs + a * D;
  const int kv_len = visible_keys(sh, seqlens, b);
  int kv_end = kv_len;
  if (sh.causal && q_base + 128 < kv_end) kv_end = q_base + 128;
  const int n_tiles = (kv_end + 63) / 64;
  const int my_q = q_base + 32 * wave + (lane & 31);
  const int q_ld = my_q < S ? my_q : S - 1;
  const int wave_q_max = q_base + 32 * wave + 31;
  const float scale = rsqrtf((float)D), sl2 = LOG2E * scale;

  bf16x8_t qf[NS], df[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    qf[s] = *reinterpret_cast<const bf16x8_t*>(base + q_ld * rs + 16 * s + 8 * kc);
    df[s] = *reinterpret_cast<const bf16x8_t*>(dout + ((int64_t)b * S + q_ld) * H + a * D + 16 * s + 8 * kc);
  }
  const float my_lse2 = lse[((int64_t)b * sh.heads + a) * S + q_ld] * LOG2E;
  const float my_delta = delta[((int64_t)b * sh.heads + a) * S + q_ld];
  f32x16_t dq[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[t][r] = 0.f;

  TileMover<D> mk, mv;
  if (n_tiles > 0) {
    mk.load(base + H, rs, 0, S - 1, tid, S);
    mv.load(base + 2 * H, rs, 0, S - 1, tid, S);
    mk.store(smem, tid);
    mv.store(smem + 64 * D, tid);
  }
  __syncthreads();
  for (int it = 0; it < n_tiles; ++it) {
    const int kv0 = it * 64;
    const bf16_t* kt = smem + (it & 1) * 128 * D;
    const bf16_t* vt = kt + 64 * D;
    if (it + 1 < n_tiles) {
      mk.load(base + H, rs, kv0 + 64, S - 1, tid, S);
      mv.load(base + 2 * H, rs, kv0 + 64, S - 1, tid, S);
    }
    if (!sh.causal || kv0 <= wave_q_max) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        f32x16_t sc, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = dp[r] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(kt, i * 32, s, lane), qf[s], sc, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(vt, i * 32, s, lane), df[s], dp, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + i * 32 + acc_row(r, lane);
          float p = __builtin_amdgcn_exp2f(sc[r] * sl2 - my_lse2);
          if (kv >= kv_len || (sh.causal && kv > my_q)) p = 0.f;
          dp[r] = p * (dp[r] - my_delta);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const bf16x8_t dsf = pack8(dp, h);
#pragma unroll
          for (int t = 0; t < NT; ++t)
            dq[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<D>(kt, i * 32 + 16 * h, t, lane), dsf, dq[t], 0, 0, 0);
        }
      }
    }
    if (it + 1 < n_tiles) {
      bf16_t* nk = smem + ((it + 1) & 1) * 128 * D;
      mk.store(nk, tid);
      mv.store(nk + 64 * D, tid);
    }
    __syncthreads();
  }
  if (my_q < S) {
    bf16_t* qrow = dqkv + ((int64_t)b * S + my_q) * rs + a * D;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16x2(dq[t][4 * g] * scale, dq[t][4 * g + 1] * scale);
        w.y = pack_bf16x2(dq[t][4 * g + 2] * scale, dq[t][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(qrow + t * 32 + g * 8 + 4 * kc) = w;
      }
  }
}

// =================================== fp32 / generic simple kernels ===============================
// One wavefront per query row; lane <-> key for the scores, lane <-> head-dim column for the output.
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_fwd_simple_kernel(AttnShape sh, const T* __restrict__ qkv,
                                                              const int32_t* __restrict__ seqlens,
                                                              T* __restrict__ out, float* __restrict__ lse) {
  extern __shared__ float fsm[];  // per wave: q[D], p[S]
  const int S = sh.seq, H = sh.hidden, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, a = blockIdx.y, i = blockIdx.x * 4 + wave;
  float* qs = fsm + wave * (D + S);
  float* ps = qs + D;
  if (i >= S) return;  // no block-wide barrier below
  const int64_t rs = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)b * S * rs + a * D;
  int kv_end = visible_keys(sh, seqlens, b);
  if (sh.causal && i + 1 < kv_end) kv_end = i + 1;
  const float scale = rsqrtf((float)D);
  for (int dd = lane; dd < D; dd += 64) qs[dd] = to_f32(base[i * rs + dd]);
  __builtin_amdgcn_wave_barrier();
  float mx = -INFINITY;
  for (int j = lane; j < kv_end; j += 64) {
    const T* kr = base + H + j * rs;
    float s = 0.f;
    for (int dd = 0; dd < D; ++dd) s = fmaf(qs[dd], to_f32(kr[dd]), s);
    s *= scale;
    ps[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < kv_end; j += 64) { const float p = __expf(ps[j] - mx); ps[j] = p; sum += p; }
  sum = wave_sum(sum);
  __builtin_amdgcn_wave_barrier();
  const float inv = sum > 0.f ? 1.f / sum : 0.f;
  for (int dd = lane; dd < D; dd += 64) {
    float acc = 0.f;
    for (int j = 0; j < kv_end; ++j) acc = fmaf(ps[j], to_f32(base[2 * H + j * rs + dd]), acc);
    from_f32(out[((int64_t)b * S + i) * H + a * D + dd], acc * inv);
  }
  if (lane == 0) lse[((int64_t)b * sh.heads + a) * S + i] = sum > 0.f ? mx + __logf(sum) : -INFINITY;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple_kernel(AttnShape sh, const T* __restrict__ qkv,
                                                                 const int32_t* __restrict__ seqlens,
                                                                 const T* __restrict__ dout,
                                                                 const float* __restrict__ lse,
                                                                 const float* __restrict__ delta,
                                                                 T* __restrict__ dqkv) {
  extern __shared__ float fsm[];  // per wave: q[D], do[D], ds[S]
  const int S = sh.seq, H = sh.hidden, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, a = blockIdx.y, i = blockIdx.x * 4 + wave;
  float* qs = fsm + wave * (2 * D + S);
  float* dos = qs + D;
  float* ds = dos + D;
  if (i >= S) return;
  const int64_t rs = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)b * S * rs + a * D;
  int kv_end = visible_keys(sh, seqlens, b);
  if (sh.causal && i + 1 < kv_end) kv_end = i + 1;
  const float scale = rsqrtf((float)D);
  const float my_lse = lse[((int64_t)b * sh.heads + a) * S + i], my_delta = delta[((int64_t)b * sh.heads + a) * S + i];
  for (int dd = lane; dd < D; dd += 64) {
    qs[dd] = to_f32(base[i * rs + dd]);
    dos[dd] = to_f32(dout[((int64_t)b * S + i) * H + a * D + dd]);
  }
  __builtin_amdgcn_wave_barrier();
  for (int j = lane; j < kv_end; j += 64) {
    const T* kr = base + H + j * rs;
    const T* vr = base + 2 * H + j * rs;
    float s = 0.f, dp = 0.f;
    for (int dd = 0; dd < D; ++dd) { s = fmaf(qs[dd], to_f32(kr[dd]), s); dp = fmaf(dos[dd], to_f32(vr[dd]), dp); }
    const float p = __expf(s * scale - my_lse);
    ds[j] = p * (dp - my_delta);
  }
  __builtin_amdgcn_wave_barrier();
  for (int dd = lane; dd < D; dd += 64) {
    float acc = 0.f;
    for (int j = 0; j < kv_end; ++j) acc = fmaf(ds[j], to_f32(base[H + j * rs + dd]), acc);
    from_f32(dqkv[((int64_t)b * S + i) * rs + a * D + dd], acc * scale);
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_simple_kernel(AttnShape sh, const T* __restrict__ qkv,
                                                                   const int32_t* __restrict__ seqlens,
                                                                   const T* __restrict__ dout,
                                                                   const float* __restrict__ lse,
                                                                   const float* __restrict__ delta,
                                                                   T* __restrict__ dqkv) {
  extern __shared__ float fsm[];  // per wave: k[D], v[D], p[S], ds[S]
  const int S = sh.seq, H = sh.hidden, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.z, a = blockIdx.y, j = blockIdx.x * 4 + wave;
  float* ks = fsm + wave * (2 * D + 2 * S);
  float* vs = ks + D;
  float* ps = vs + D;
  float* ds = ps + S;
  if (j >= S) return;
  const int64_t rs = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)b * S * rs + a * D;
  const int kv_len = visible_keys(sh, seqlens, b);
  const float scale = rsqrtf((float)D);
  const int i_first = (j >= kv_len) ? S : (sh.causal ? j : 0);  // hidden key: no query sees it
  for (int dd = lane; dd < D; dd += 64) { ks[dd] = to_f32(base[H + j * rs + dd]); vs[dd] = to_f32(base[2 * H + j * rs + dd]); }
  __builtin_amdgcn_wave_barrier();
  for (int i = i_first + lane; i < S; i += 64) {
    const T* qr = base + i * rs;
    const T* dr = dout + ((int64_t)b * S + i) * H + a * D;
    float s = 0.f, dp = 0.f;
    for (int dd = 0; dd < D; ++dd) { s = fmaf(to_f32(qr[dd]), ks[dd], s); dp = fmaf(to_f32(dr[dd]), vs[dd], dp); }
    const float p = __expf(s * scale - lse[((int64_t)b * sh.heads + a) * S + i]);
    ps[i] = p;
    ds[i] = p * (dp - delta[((int64_t)b * sh.heads + a) * S + i]);
  }
  __builtin_amdgcn_wave_barrier();
  for (int dd = lane; dd < D; dd += 64) {
    float dk = 0.f, dv = 0.f;
    for (int i = i_first; i < S; ++i) {
      dk = fmaf(ds[i], to_f32(base[i * rs + dd]), dk);
      dv = fmaf(ps[i], to_f32(dout[((int64_t)b * S + i) * H + a * D + dd]), dv);
    }
    from_f32(dqkv[((int64_t)b * S + j) * rs + H + a * D + dd], dk * scale);
    from_f32(dqkv[((int64_t)b * S + j) * rs + 2 * H + a * D + dd], dv);
  }
}

// =================================== launchers ===================================================
template <int D>
static void fwd_bf16(const AttnShape& s, const void* qkv, const int32_t* seqlens, void* out, float* lse, hipStream_t st) {
  const size_t lds = (size_t)2 * 128 * D * sizeof(bf16_t);
  auto kern = attn_fwd_bf16_kernel<D>;
  (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3((s.seq + 127) / 128, s.heads, s.batch), dim3(256), lds, st, s, (const bf16_t*)qkv,
                     seqlens, (bf16_t*)out, lse);
}
template <int D>
static void fwd_f32(const AttnShape& s, const void* qkv, const int32_t* seqlens, void* out, float* lse, hipStream_t st) {
  const size_t lds = (size_t)4 * (D + s.seq) * sizeof(float);
  auto kern = attn_fwd_simple_kernel<float, D>;
  (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3((s.seq + 3) / 4, s.heads, s.batch), dim3(256), lds, st, s, (const float*)qkv, seqlens,
                     (float*)out, lse);
}

void launch_attn_fwd(int dtype_fp32, const AttnShape& s, const void* qkv, const int32_t* seqlens, void* out,
                     float* lse, hipStream_t st) {
  const int D = s.hidden / s.heads;
  if (dtype_fp32) { if (D == 64) fwd_f32<64>(s, qkv, seqlens, out, lse, st); else fwd_f32<128>(s, qkv, seqlens, out, lse, st); }
  else { if (D == 64) fwd_bf16<64>(s, qkv, seqlens, out, lse, st); else fwd_bf16<128>(s, qkv, seqlens, out, lse, st); }
}

template <int D>
static void bwd_bf16(const AttnShape& s, const void* qkv, const int32_t* seqlens, const void* out, const void* dout,
                     const float* lse, float* delta, void* dqkv, hipStream_t st) {
  const int64_t items = (int64_t)s.batch * s.seq * s.heads * 8;
  hipLaunchKernelGGL((attn_delta_kernel<bf16_t, D>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, s,
                     (const bf16_t*)out, (const bf16_t*)dout, delta);
  dim3 grid((s.seq + 127) / 128, s.heads, s.batch);
  {
    const size_t lds = (size_t)2 * (128 * D + 256) * sizeof(bf16_t);
    auto kern = attn_bwd_dkdv_bf16_kernel<D>;
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, s, (const bf16_t*)qkv, seqlens, (const bf16_t*)dout, lse,
                       (const float*)delta, (bf16_t*)dqkv);
  }
  {
    const size_t lds = (size_t)2 * 128 * D * sizeof(bf16_t);
    auto kern = attn_bwd_dq_bf16_kernel<D>;
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, s, (const bf16_t*)qkv, seqlens, (const bf16_t*)dout, lse,
                       (const float*)delta, (bf16_t*)dqkv);
  }
}
template <int D>
static void bwd_f32(const AttnShape& s, const void* qkv, const int32_t* seqlens, const void* out, const void* dout,
                    const float* lse, float* delta, void* dqkv, hipStream_t st) {
  const int64_t items = (int64_t)s.batch * s.seq * s.heads * 8;
  hipLaunchKernelGGL((attn_delta_kernel<float, D>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, s,
                     (const float*)out, (const float*)dout, delta);
  dim3 grid((s.seq + 3) / 4, s.heads, s.batch);
  {
    const size_t lds = (size_t)4 * (2 * D + s.seq) * sizeof(float);
    auto kern = attn_bwd_dq_simple_kernel<float, D>;
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, s, (const float*)qkv, seqlens, (const float*)dout, lse,
                       (const float*)delta, (float*)dqkv);
  }
  {
    const size_t lds = (size_t)4 * (2 * D + 2 * s.seq) * sizeof(float);
    auto kern = attn_bwd_dkdv_simple_kernel<float, D>;
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, s, (const float*)qkv, seqlens, (const float*)dout, lse,
                       (const float*)delta, (float*)dqkv);
  }
}

void launch_attn_bwd(int dtype_fp32, const AttnShape& s, const void* qkv, const int32_t* seqlens, const void* out,
                     const void* dout, const float* lse, float* delta, void* dqkv, hipStream_t st) {
  const int D = s.hidden / s.heads;
  if (dtype_fp32) {
    if (D == 64) bwd_f32<64>(s, qkv, seqlens, out, dout, lse, delta, dqkv, st);
    else bwd_f32<128>(s, qkv, seqlens, out, dout, lse, delta, dqkv, st);
  } else {
    if (D == 64) bwd_bf16<64>(s, qkv, seqlens, out, dout, lse, delta, dqkv, st);
    else bwd_bf16<128>(s, qkv, seqlens, out, dout, lse, delta, dqkv, st);
  }
}

}  // namespace slapo
