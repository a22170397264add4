// HBM-bound row kernels: the fused bias + dropout + residual + LayerNorm pattern of the scheduled
// layer (paper section 2.2 and the appendix schedule's "LNResidual" fusion), its hand-derived
// backward, and the deterministic two-stage column reductions for bias / gamma / beta gradients.
//
// One wavefront owns one row of H elements at a time: lane l holds the 8-element chunks l, l+64, ...
// of the row in registers, so every tensor is read and written exactly once with 16-byte accesses
// and the row statistics are plain 64-lane reductions. The dropout decision of a chunk comes from
// one Philox4x32-10 call on the chunk's index, so nothing about the mask is ever stored.
#include "common.h"
#include "kernels.h"

namespace slapo {

template <typename T, int NCH, bool BDR, bool LN, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void bdrln_fwd_kernel(
    int64_t rows, int H, const T* __restrict__ r, const T* __restrict__ bias, const T* __restrict__ res,
    const T* __restrict__ gamma, const T* __restrict__ beta, T* __restrict__ z_out, T* __restrict__ out,
    float* __restrict__ mu_out, float* __restrict__ rstd_out, DropoutParams dp, float eps, int rms) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nchunk = H >> 3;
  const float inv_h = 1.0f / (float)H;
  for (int64_t row = (int64_t)blockIdx.x * WAVES + wave; row < rows; row += (int64_t)gridDim.x * WAVES) {
    const int64_t base = row * H;
    float v[NCH][8];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        load8(res + base + c * 8, v[i]);
        if (BDR) {
          float a[8], b[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          load8(r + base + c * 8, a);
          if (bias) load8(bias + c * 8, b);
          const uint32_t keep = dropout_keep8(dp, (uint64_t)(base >> 3) + (uint64_t)c);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float t = (a[j] + b[j]) * dp.scale;
            v[i][j] += ((keep >> j) & 1u) ? t : 0.f;
          }
          if (z_out) {
            store8(z_out + base + c * 8, v[i]);
            if (LN && sizeof(T) == 2) {
              // statistics are taken of the stored (rounded) sum, the value backward will read
#pragma unroll
              for (int j = 0; j < 8; ++j) { T h; from_f32(h, v[i][j]); v[i][j] = to_f32(h); }
            }
          }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += v[i][j];
      }
    }
    if (!LN) continue;
    const float mean = rms ? 0.f : wave_sum(sum) * inv_h;   // RMSNorm: second moment about zero
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (lane + 64 * i < nchunk) {
#pragma unroll
        for (int j = 0; j < 8; ++j) { const float d = v[i][j] - mean; sq += d * d; }
      }
    }
    const float rstd = rsqrtf(wave_sum(sq) * inv_h + eps);
    if (lane == 0) { if (mu_out) mu_out[row] = mean; rstd_out[row] = rstd; }
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        float g[8], b[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, y[8];
        load8(gamma + c * 8, g);
        if (beta) load8(beta + c * 8, b);
#pragma unroll
        for (int j = 0; j < 8; ++j) y[j] = (v[i][j] - mean) * rstd * g[j] + b[j];
        store8(out + base + c * 8, y);
      }
    }
  }
}

// Replaces eight fp32 values by what they read back as after a store in the element type: a kernel that
// goes on from them then computes exactly what a separate kernel reading the stored array would.
template <typename T>
__device__ __forceinline__ void round_as(float (&v)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    T h;
    from_f32(h, v[j]);
    v[j] = to_f32(h);
  }
}

// Backward of out = LN(z), z = res + keep*(r+bias)*scale.  See slapo_bdrln_bwd for the contract.
// dr_from_stored: the branch gradient dr is derived from dz as stored (rounded to T) rather than from the
// fp32 value, i.e. dz_out and dr_out are those of two kernels in a row (dz first, then dr from the stored dz).
template <typename T, int NCH, bool LN, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void bdrln_bwd_kernel(
    int64_t rows, int H, const T* __restrict__ dout, const T* __restrict__ z, const float* __restrict__ mu,
    const float* __restrict__ rstd, const T* __restrict__ gamma, const T* __restrict__ dres_in,
    T* __restrict__ dz_out, T* __restrict__ dr_out, float* __restrict__ partials, DropoutParams dp, int dr_from_stored) {
  extern __shared__ float red[];  // [WAVES/2][3][H]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nchunk = H >> 3;
  const float inv_h = 1.0f / (float)H;
  float pg[NCH][8], pb[NCH][8], pd[NCH][8];
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) pg[i][j] = pb[i][j] = pd[i][j] = 0.f;

  const int64_t stride = (int64_t)gridDim.x * WAVES;
  Raw8<T> ndy[NCH], nz[NCH], nres[NCH];
  float nm = 0.f, nrs = 0.f;
  auto fetch = [&](int64_t r) {
    const int64_t base = r * H;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        ndy[i].load(dout + base + c * 8);
        if (LN) nz[i].load(z + base + c * 8);
        if (dres_in) nres[i].load(dres_in + base + c * 8);
      }
    }
    if (LN) { nm = mu ? mu[r] : 0.f; nrs = rstd[r]; }   // no mu: RMSNorm
  };
  // (issuing the next row's loads ahead of the reductions was measured and made no difference)
  for (int64_t row = (int64_t)blockIdx.x * WAVES + wave; row < rows; row += stride) {
    fetch(row);
    const int64_t base = row * H;
    float dy[NCH][8], xh[NCH][8], res[NCH][8];
    float s1 = 0.f, s2 = 0.f;
    const float m = nm, rs = nrs;
    Raw8<T> cz[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (lane + 64 * i < nchunk) {
        ndy[i].get(dy[i]);
        cz[i] = nz[i];
        if (dres_in) nres[i].get(res[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        if (LN) {
          float zz[8], g[8];
          cz[i].get(zz);
          load8(gamma + c * 8, g);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            xh[i][j] = (zz[j] - m) * rs;
            pg[i][j] += dy[i][j] * xh[i][j];
            pb[i][j] += dy[i][j];
            dy[i][j] *= g[j];  // from here on dy holds g = dout * gamma
            s1 += dy[i][j];
            s2 += dy[i][j] * xh[i][j];
          }
        }
      }
    }
    if (LN) { s1 = mu ? wave_sum(s1) * inv_h : 0.f; s2 = wave_sum(s2) * inv_h; }
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        float dz[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) dz[j] = LN ? rs * (dy[i][j] - s1 - xh[i][j] * s2) : dy[i][j];
        if (dres_in) {
#pragma unroll
          for (int j = 0; j < 8; ++j) dz[j] += res[i][j];
        }
        if (dz_out) store8(dz_out + base + c * 8, dz);
        if (dr_out) {
          if (dr_from_stored) round_as<T>(dz);
          const uint32_t keep = dropout_keep8(dp, (uint64_t)(base >> 3) + (uint64_t)c);
          float dr[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            dr[j] = ((keep >> j) & 1u) ? dz[j] * dp.scale : 0.f;
            pd[i][j] += dr[j];
          }
          store8(dr_out + base + c * 8, dr);
        }
      }
    }
  }
  // fixed-order tree over the waves of the block, then one partial row per block
  for (int s = WAVES / 2; s >= 1; s >>= 1) {
    if (wave >= s && wave < 2 * s) {
      float* slot = red + (size_t)(wave - s) * 3 * H;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunk) {
          store8(slot + c * 8, pg[i]);
          store8(slot + H + c * 8, pb[i]);
          store8(slot + 2 * H + c * 8, pd[i]);
        }
      }
    }
    __syncthreads();
    if (wave < s) {
      const float* slot = red + (size_t)wave * 3 * H;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunk) {
          float a[8], b[8], d[8];
          load8(slot + c * 8, a);
          load8(slot + H + c * 8, b);
          load8(slot + 2 * H + c * 8, d);
#pragma unroll
          for (int j = 0; j < 8; ++j) { pg[i][j] += a[j]; pb[i][j] += b[j]; pd[i][j] += d[j]; }
        }
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
    float* prow = partials + (size_t)blockIdx.x * 3 * H;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        store8(prow + c * 8, pg[i]);
        store8(prow + H + c * 8, pb[i]);
        store8(prow + 2 * H + c * 8, pd[i]);
      }
    }
  }
}

// The same backward for rows of 512 elements and more. The kernel above keeps a whole row and three column
// accumulators per lane, which stops fitting the register file from H = 2048 on, and it has one row per wavefront
// in flight. Here a block is G groups of NW wavefronts; inside a group thread c owns the 8 columns of chunk c for
// every row the group visits, so the column sums never leave their lane while the rows go by; the two per-row
// sums cross the group's wavefronts through LDS (one barrier per step, added in wave order). A step handles R rows
// per group, G * R consecutive rows per block, and the loads of the next step are issued before the arithmetic
// of the current one (the barrier is a bare s_barrier: it does not wait for them), so that the block always has
// two steps' worth of rows on their way from memory: with one block per CU (the partial sums it leaves are
// [blocks, 3, H] floats, which bounds the block count) that is what keeps the memory pipeline full. At the end
// the groups' column sums are added in group order through LDS: one partial row per block, as above.
template <typename T, bool LN, int R, int MAXT, bool ONE = false>
__global__ __launch_bounds__(MAXT) void bdrln_bwd_wide_kernel(
    int64_t rows, int H, const T* __restrict__ dout, const T* __restrict__ z, const float* __restrict__ mu,
    const float* __restrict__ rstd, const T* __restrict__ gamma, const T* __restrict__ dres_in,
    T* __restrict__ dz_out, T* __restrict__ dr_out, float* __restrict__ partials, DropoutParams dp, int dr_from_stored,
    int NW, int G) {
  extern __shared__ __attribute__((aligned(16))) float wsm[];   // per-row sums [2][G][R][NW][2]; at the end column sums [G-1][3][H]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int group = wave / NW, gw = wave - group * NW;
  const int c = gw * 64 + lane;
  const bool active = c < (H >> 3);
  const float inv_h = 1.0f / (float)H;
  float pg[8], pb[8], pd[8], g[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { pg[e] = pb[e] = pd[e] = 0.f; g[e] = 0.f; }
  if (LN && active) load8(gamma + c * 8, g);
  const int64_t per_step = (int64_t)gridDim.x * G * R;
  // (ONE: the launch covers all rows in one step; nothing is prefetched, which leaves registers for a third row)
  const int64_t n_steps = ONE ? 1 : (rows + per_step - 1) / per_step;   // the same for every group: they share the barrier
  auto first_row = [&](int64_t step) { return ((step * gridDim.x + blockIdx.x) * G + group) * R; };
  Raw8<T> ndy[R], nz[R], nres[R];
  float nm[R], nrs[R];
  auto fetch = [&](int64_t step) {   // all loads of a step go out before anything waits
    const int64_t row0 = first_row(step);
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int64_t row = row0 + j;
      nm[j] = 0.f; nrs[j] = 0.f;
      if (row < rows) {
        if (active) {
          ndy[j].load(dout + row * H + c * 8);
          if (LN) nz[j].load(z + row * H + c * 8);
          if (dres_in) nres[j].load(dres_in + row * H + c * 8);
        }
        if (LN) { nm[j] = mu ? mu[row] : 0.f; nrs[j] = rstd[row]; }   // no mu: RMSNorm
      }
    }
  };
  if (n_steps > 0) fetch(0);
  int par = 0;
  for (int64_t step = 0; step < n_steps; ++step, par ^= 1) {
    const int64_t row0 = first_row(step);
    float dy[R][8], xh[R][8], s1[R], s2[R], m[R], rs[R];
    Raw8<T> cres[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      s1[j] = 0.f; s2[j] = 0.f; m[j] = nm[j]; rs[j] = nrs[j];
      if (row0 + j < rows && active) {
        ndy[j].get(dy[j]);
        if (dres_in) cres[j] = nres[j];
        if (LN) {
          float zz[8];
          nz[j].get(zz);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            xh[j][e] = (zz[e] - m[j]) * rs[j];
            pg[e] += dy[j][e] * xh[j][e];
            pb[e] += dy[j][e];
            dy[j][e] *= g[e];   // from here on dy holds dout * gamma
            s1[j] += dy[j][e];
            s2[j] += dy[j][e] * xh[j][e];
          }
        }
      }
    }
    if (step + 1 < n_steps) fetch(step + 1);   // on their way during the rest of this step
    if (LN) {
      float* xs = wsm + (size_t)((par * G + group) * R) * NW * 2;
#pragma unroll
      for (int j = 0; j < R; ++j) {
        const float a = wave_sum(s1[j]), b = wave_sum(s2[j]);
        if (lane == 0) { xs[(j * NW + gw) * 2] = a; xs[(j * NW + gw) * 2 + 1] = b; }
      }
      wait_loads_and_lds<63>();   // the LDS writes are done; the loads just issued stay in flight
      block_barrier();            // (the other parity is written next time round: no second barrier needed)
#pragma unroll
      for (int j = 0; j < R; ++j) {
        float a = 0.f, b = 0.f;
        for (int w = 0; w < NW; ++w) { a += xs[(j * NW + w) * 2]; b += xs[(j * NW + w) * 2 + 1]; }
        s1[j] = mu ? a * inv_h : 0.f;
        s2[j] = b * inv_h;
      }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int64_t row = row0 + j;
      if (row < rows && active) {
        const int64_t base = row * H;
        float dz[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) dz[e] = LN ? rs[j] * (dy[j][e] - s1[j] - xh[j][e] * s2[j]) : dy[j][e];
        if (dres_in) {
          float res[8];
          cres[j].get(res);
#pragma unroll
          for (int e = 0; e < 8; ++e) dz[e] += res[e];
        }
        if (dz_out) store8(dz_out + base + c * 8, dz);
        if (dr_out) {
          if (dr_from_stored) round_as<T>(dz);
          const uint32_t keep = dropout_keep8(dp, (uint64_t)(base >> 3) + (uint64_t)c);
          float dr[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            dr[e] = ((keep >> e) & 1u) ? dz[e] * dp.scale : 0.f;
            pd[e] += dr[e];
          }
          store8(dr_out + base + c * 8, dr);
        }
      }
    }
  }
  // column sums of the groups, added in group order
  __syncthreads();   // the per-row sums in LDS have been read by everybody
  if (group > 0 && active) {
    float* slot = wsm + (size_t)(group - 1) * 3 * H;
    store8(slot + c * 8, pg);
    store8(slot + H + c * 8, pb);
    store8(slot + 2 * H + c * 8, pd);
  }
  __syncthreads();
  if (group == 0 && active) {
    for (int gg = 1; gg < G; ++gg) {
      const float* slot = wsm + (size_t)(gg - 1) * 3 * H;
      float a[8], b[8], d[8];
      load8(slot + c * 8, a);
      load8(slot + H + c * 8, b);
      load8(slot + 2 * H + c * 8, d);
#pragma unroll
      for (int e = 0; e < 8; ++e) { pg[e] += a[e]; pb[e] += b[e]; pd[e] += d[e]; }
    }
    float* prow = partials + (size_t)blockIdx.x * 3 * H;
    store8(prow + c * 8, pg);
    store8(prow + H + c * 8, pb);
    store8(prow + 2 * H + c * 8, pd);
  }
}

// stage 1 of a column sum: block (bx, by) sums rows of slab by for the 32 chunks of column group bx
template <typename T>
__global__ __launch_bounds__(256) void colsum_partials_kernel(int64_t rows, int64_t N, const T* __restrict__ a,
                                                              float* __restrict__ partials) {
  __shared__ __attribute__((aligned(16))) float red[8][32][8];
  const int cx = threadIdx.x & 31, ry = threadIdx.x >> 5;
  const int64_t chunk = (int64_t)blockIdx.x * 32 + cx;
  const int64_t per = (rows + gridDim.y - 1) / gridDim.y;
  const int64_t r0 = (int64_t)blockIdx.y * per, r1 = (r0 + per < rows) ? r0 + per : rows;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (chunk * 8 < N) {
    // eight rows' loads go out before the first is added (one load in flight per thread left the kernel bound by
    // memory latency: 92 us for 134 MB); the rows are added in the order of the plain loop, so the sums keep their bits
    constexpr int U = 8;
    const T* p = a + chunk * 8;
    int64_t rr = r0 + ry;
    for (; rr + 8 * (U - 1) < r1; rr += 8 * U) {
      Raw8<T> raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) raw[u].load(p + (rr + 8 * u) * N);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float v[8];
        raw[u].get(v);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += v[j];
      }
    }
    for (; rr < r1; rr += 8) {
      float v[8];
      load8(p + rr * N, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += v[j];
    }
  }
  store8(&red[ry][cx][0], acc);
  __syncthreads();
  if (ry == 0 && chunk * 8 < N) {
#pragma unroll
    for (int k = 1; k < 8; ++k) {
      float v[8];
      load8(&red[k][cx][0], v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += v[j];
    }
    store8(partials + (int64_t)blockIdx.y * N + chunk * 8, acc);
  }
}

// stage 2: out[n] = sum_i partials[i*stride + n]. A block owns 64 columns; its RW wavefronts each sum a
// contiguous share of the rows with eight loads in flight at once, then the shares are added in wave order.
// Four wavefronts per block: these kernels run between the GEMMs of the backward pass, whose workgroups leave a
// CU room for a few more wavefronts but never for a block of sixteen (which waited for a CU to fall idle: 84 us
// in the step against 4 us alone).
constexpr int RW = 4;
template <typename T>
__global__ __launch_bounds__(RW * 64) void colreduce_partials_kernel(int64_t nblk, int64_t stride, int64_t N,
                                                                  const float* __restrict__ partials,
                                                                  T* __restrict__ out, int accumulate) {
  __shared__ float red[RW][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t n = (int64_t)blockIdx.x * 64 + lane;
  const int64_t per = (nblk + RW - 1) / RW;
  const int64_t i0 = wave * per, i1 = (i0 + per < nblk) ? i0 + per : nblk;
  float s = 0.f;
  if (n < N) {
    int64_t i = i0;
    for (; i + 8 <= i1; i += 8) {
      float v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = partials[(i + k) * stride + n];
#pragma unroll
      for (int k = 0; k < 8; ++k) s += v[k];
    }
    for (; i < i1; ++i) s += partials[i * stride + n];
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && n < N) {
    float t = red[0][lane];
#pragma unroll
    for (int w = 1; w < RW; ++w) t += red[w][lane];
    if (accumulate) t += to_f32(out[n]);
    from_f32(out[n], t);
  }
}

__global__ __launch_bounds__(256) void dropout_mask_kernel(int64_t nblocks8, uint8_t* __restrict__ mask,
                                                           DropoutParams dp) {
  const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (b >= nblocks8) return;
  const uint32_t keep = dropout_keep8(dp, (uint64_t)b);
  uint2 w;
  w.x = (keep & 1u) | ((keep >> 1 & 1u) << 8) | ((keep >> 2 & 1u) << 16) | ((keep >> 3 & 1u) << 24);
  w.y = (keep >> 4 & 1u) | ((keep >> 5 & 1u) << 8) | ((keep >> 6 & 1u) << 16) | ((keep >> 7 & 1u) << 24);
  *reinterpret_cast<uint2*>(mask + b * 8) = w;
}

// ---- host launchers -----------------------------------------------------------------------------

// chunks of 8 columns per lane of the row-per-wavefront kernels (H <= 8192)
static int nch_for(int H) {
  const int n = (H / 8 + 63) / 64;
  return n <= 1 ? 1 : n <= 2 ? 2 : n <= 4 ? 4 : n <= 5 ? 5 : n <= 8 ? 8 : n <= 10 ? 10 : 16;
}

template <typename T, bool BDR, bool LN>
static void launch_fwd(int64_t rows, int H, const void* r, const void* bias, const void* res, const void* gamma,
                       const void* beta, void* z_out, void* out, float* mu, float* rstd, const DropoutParams& dp,
                       float eps, int rms, hipStream_t st) {
  constexpr int WAVES = 4;
  int64_t blocks = (rows + WAVES - 1) / WAVES;
  if (blocks > 4096) blocks = 4096;
#define SLAPO_FWD(N)                                                                                          \
  hipLaunchKernelGGL((bdrln_fwd_kernel<T, N, BDR, LN, WAVES>), dim3((unsigned)blocks), dim3(WAVES * 64), 0, st, \
                     rows, H, (const T*)r, (const T*)bias, (const T*)res, (const T*)gamma, (const T*)beta,    \
                     (T*)z_out, (T*)out, mu, rstd, dp, eps, rms)
  switch (nch_for(H)) {
    case 1: SLAPO_FWD(1); break;
    case 2: SLAPO_FWD(2); break;
    case 4: SLAPO_FWD(4); break;
    case 5: SLAPO_FWD(5); break;
    case 8: SLAPO_FWD(8); break;
    case 10: SLAPO_FWD(10); break;
    default: SLAPO_FWD(16); break;
  }
#undef SLAPO_FWD
}

void launch_bdrln_fwd(int dtype, int64_t rows, int H, const void* r, const void* bias, const void* res,
                      const void* gamma, const void* beta, void* z_out, void* out, float* mu, float* rstd,
                      const DropoutParams& dp, float eps, int rms, hipStream_t st) {
  const bool bdr = r != nullptr, ln = gamma != nullptr;
  if (rms) { beta = nullptr; mu = nullptr; }
#define SLAPO_PICK(T)                                                                                   \
  if (bdr && ln) launch_fwd<T, true, true>(rows, H, r, bias, res, gamma, beta, z_out, out, mu, rstd, dp, eps, rms, st); \
  else if (bdr) launch_fwd<T, true, false>(rows, H, r, bias, res, gamma, beta, z_out, out, mu, rstd, dp, eps, rms, st); \
  else launch_fwd<T, false, true>(rows, H, r, bias, res, gamma, beta, z_out, out, mu, rstd, dp, eps, rms, st)
  if (dtype == DT_FP32) { SLAPO_PICK(float); } else if (dtype == DT_FP16) { SLAPO_PICK(f16_t); } else { SLAPO_PICK(bf16_t); }
#undef SLAPO_PICK
}

int bdrln_bwd_blocks(int64_t rows) {
  int64_t b = (rows + 7) / 8;
  return (int)(b > 256 ? 256 : (b < 1 ? 1 : b));
}

template <typename T, bool LN>
static void launch_bwd(int64_t rows, int H, const void* dout, const void* z, const float* mu, const float* rstd,
                       const void* gamma, const void* dres_in, void* dz_out, void* dr_out, float* partials,
                       const DropoutParams& dp, int dr_from_stored, hipStream_t st) {
  const int blocks = bdrln_bwd_blocks(rows);
  if (H >= 512) {
    // Groups of NW wavefronts that split the columns. Up to hidden 3072 as many groups as fit 12 wavefronts (the
    // register budget of three wavefronts per SIMD holds two rows per group and their prefetch without spilling);
    // wider rows fill the block with one group, four rows at a time up to 4096, one above.
    const int nw = (H / 8 + 63) / 64;
    const int groups = nw <= 6 ? (12 / nw > 8 ? 8 : 12 / nw) : 1;
    const int rows_per_group = nw <= 6 ? 2 : nw <= 8 ? 4 : 1;
    const size_t xs_bytes = (size_t)2 * groups * (rows_per_group == 2 ? 3 : rows_per_group) * nw * 2 * sizeof(float);
    const size_t col_bytes = (size_t)(groups - 1) * 3 * H * sizeof(float);
    const size_t lds = xs_bytes > col_bytes ? xs_bytes : col_bytes;
#define SLAPO_WIDE(R, MAXT, ...)                                                                                     \
  do {                                                                                                               \
    auto kern = bdrln_bwd_wide_kernel<T, LN, R, MAXT, ##__VA_ARGS__>;                                                \
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);             \
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(groups * nw * 64), lds, st, rows, H, (const T*)dout, (const T*)z, mu, \
                       rstd, (const T*)gamma, (const T*)dres_in, (T*)dz_out, (T*)dr_out, partials, dp,              \
                       dr_from_stored, nw, groups);                                                                  \
  } while (0)
    // (three rows per group where that takes all rows in ONE step instead of a full and a thin one: 4096 rows of 1024)
    if (nw <= 6 && rows > (int64_t)blocks * groups * 2 && rows <= (int64_t)blocks * groups * 3) SLAPO_WIDE(3, 768, true);
    else if (nw <= 6) SLAPO_WIDE(2, 768);
    else if (nw <= 8) SLAPO_WIDE(4, 512);
    else SLAPO_WIDE(1, 1024);
#undef SLAPO_WIDE
    return;
  }
#define SLAPO_BWD(N, W)                                                                                      \
  do {                                                                                                       \
    auto kern = bdrln_bwd_kernel<T, N, LN, W>;                                                               \
    const size_t lds = (size_t)(W / 2) * 3 * H * 4;                                                          \
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);     \
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(W * 64), lds, st, rows, H, (const T*)dout, (const T*)z, mu,  \
                       rstd, (const T*)gamma, (const T*)dres_in, (T*)dz_out, (T*)dr_out, partials, dp,       \
                       dr_from_stored);                                                                      \
  } while (0)
  switch (nch_for(H)) {
    case 1: SLAPO_BWD(1, 8); break;
    default: SLAPO_BWD(2, 8); break;
  }
#undef SLAPO_BWD
}

void launch_bdrln_bwd(int dtype, int64_t rows, int H, const void* dout, const void* z, const float* mu,
                      const float* rstd, const void* gamma, const void* dres_in, void* dz_out, void* dr_out,
                      float* partials, const DropoutParams& dp, int rms, hipStream_t st, int dr_from_stored) {
  if (rms) mu = nullptr;   // the kernel reads a missing mean as RMSNorm (mean 0, no mean-of-gradient term)
  const bool ln = gamma != nullptr;
#define SLAPO_PICK(T)                                                                                          \
  if (ln) launch_bwd<T, true>(rows, H, dout, z, mu, rstd, gamma, dres_in, dz_out, dr_out, partials, dp, dr_from_stored, st); \
  else launch_bwd<T, false>(rows, H, dout, z, mu, rstd, gamma, dres_in, dz_out, dr_out, partials, dp, dr_from_stored, st)
  if (dtype == DT_FP32) { SLAPO_PICK(float); } else if (dtype == DT_FP16) { SLAPO_PICK(f16_t); } else { SLAPO_PICK(bf16_t); }
#undef SLAPO_PICK
}

int colsum_blocks(int64_t rows) {
  int64_t b = (rows + 31) / 32;
  return (int)(b > 64 ? 64 : (b < 1 ? 1 : b));
}

void launch_colsum_partials(int dtype, int64_t rows, int64_t N, const void* a, float* partials,
                            hipStream_t st) {
  dim3 grid((unsigned)((N / 8 + 31) / 32), (unsigned)colsum_blocks(rows));
  if (dtype == DT_FP32) hipLaunchKernelGGL(colsum_partials_kernel<float>, grid, dim3(256), 0, st, rows, N, (const float*)a, partials);
  else if (dtype == DT_FP16) hipLaunchKernelGGL(colsum_partials_kernel<f16_t>, grid, dim3(256), 0, st, rows, N, (const f16_t*)a, partials);
  else hipLaunchKernelGGL(colsum_partials_kernel<bf16_t>, grid, dim3(256), 0, st, rows, N, (const bf16_t*)a, partials);
}

void launch_colreduce_partials(int dtype, int64_t nblk, int64_t stride, int64_t N, const float* partials,
                               void* out, int accumulate, hipStream_t st) {
  dim3 grid((unsigned)((N + 63) / 64));
  if (dtype == DT_FP32) hipLaunchKernelGGL(colreduce_partials_kernel<float>, grid, dim3(RW * 64), 0, st, nblk, stride, N, partials, (float*)out, accumulate);
  else if (dtype == DT_FP16) hipLaunchKernelGGL(colreduce_partials_kernel<f16_t>, grid, dim3(RW * 64), 0, st, nblk, stride, N, partials, (f16_t*)out, accumulate);
  else hipLaunchKernelGGL(colreduce_partials_kernel<bf16_t>, grid, dim3(RW * 64), 0, st, nblk, stride, N, partials, (bf16_t*)out, accumulate);
}

// the three partial rows (dgamma, dbeta, dbias) of the fused backward kernel in one launch
template <typename T>
__global__ __launch_bounds__(RW * 64) void colreduce3_kernel(int64_t nblk, int H, const float* __restrict__ partials,
                                                          T* out0, T* out1, T* out2, int accumulate) {
  __shared__ float red[RW][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, which = blockIdx.y;
  T* out = which == 0 ? out0 : (which == 1 ? out1 : out2);
  if (out == nullptr) return;   // uniform for the block
  const int64_t n = (int64_t)blockIdx.x * 64 + lane;
  const int64_t per = (nblk + RW - 1) / RW;
  const int64_t i0 = wave * per, i1 = (i0 + per < nblk) ? i0 + per : nblk;
  const float* src = partials + (int64_t)which * H;
  const int64_t stride = 3 * (int64_t)H;
  float s = 0.f;
  if (n < H) {
    int64_t i = i0;
    for (; i + 8 <= i1; i += 8) {
      float v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = src[(i + k) * stride + n];
#pragma unroll
      for (int k = 0; k < 8; ++k) s += v[k];
    }
    for (; i < i1; ++i) s += src[i * stride + n];
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && n < H) {
    float t = red[0][lane];
#pragma unroll
    for (int w = 1; w < RW; ++w) t += red[w][lane];
    if (accumulate) t += to_f32(out[n]);
    from_f32(out[n], t);
  }
}

void launch_colreduce3(int dtype, int64_t nblk, int H, const float* partials, void* out0, void* out1, void* out2,
                       int accumulate, hipStream_t st) {
  dim3 grid((unsigned)((H + 63) / 64), 3);
  if (dtype == DT_FP32) hipLaunchKernelGGL(colreduce3_kernel<float>, grid, dim3(RW * 64), 0, st, nblk, H, partials, (float*)out0, (float*)out1, (float*)out2, accumulate);
  else if (dtype == DT_FP16) hipLaunchKernelGGL(colreduce3_kernel<f16_t>, grid, dim3(RW * 64), 0, st, nblk, H, partials, (f16_t*)out0, (f16_t*)out1, (f16_t*)out2, accumulate);
  else hipLaunchKernelGGL(colreduce3_kernel<bf16_t>, grid, dim3(RW * 64), 0, st, nblk, H, partials, (bf16_t*)out0, (bf16_t*)out1, (bf16_t*)out2, accumulate);
}

void launch_dropout_mask(int64_t n_elements, uint8_t* mask, const DropoutParams& dp, hipStream_t st) {
  const int64_t nb = n_elements / 8;
  hipLaunchKernelGGL(dropout_mask_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, nb, mask, dp);
}

// ---- rotary position embedding ---------------------------------------------------------------------
// (cos, sin) of position m, pair j, for the angle m * base^(-j / half) (= m * base^(-2j/d)). Evaluated in
// double precision: positions reach thousands of radians, where an fp32 angle alone would cost 1e-4.
__global__ __launch_bounds__(256) void rope_table_kernel(int seq, int half, double log_base, float2* __restrict__ table) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= seq * half) return;
  const int m = idx / half, j = idx % half;
  const double angle = (double)m * exp(-log_base * (double)j / (double)half);
  double sn, cs;
  sincos(angle, &sn, &cs);
  table[idx] = make_float2((float)cs, (float)sn);
}

// One thread turns the four adjacent pairs of 8 consecutive columns of the Q or K part of one row, in place.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(int64_t rows, int seq, int H, int d, const float2* __restrict__ table,
                                                   T* qkv, int inverse) {
  const int64_t per_row = (2 * (int64_t)H) >> 3;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * per_row) return;
  const int64_t t = idx / per_row;
  const int n = (int)(idx - t * per_row) * 8;
  const int pos = (int)(t % seq), half = d >> 1;
  const float4* tb = reinterpret_cast<const float4*>(table + (int64_t)pos * half + ((n % d) >> 1));
  const float4 t0 = tb[0], t1 = tb[1];
  const float cs[4] = {t0.x, t0.z, t1.x, t1.z};
  const float sn[4] = {t0.y, t0.w, t1.y, t1.w};
  T* p = qkv + t * 3 * H + n;
  float v[8];
  load8(p, v);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float s = inverse ? -sn[e] : sn[e], a = v[2 * e], b = v[2 * e + 1];
    v[2 * e] = a * cs[e] - b * s;
    v[2 * e + 1] = a * s + b * cs[e];
  }
  store8(p, v);
}

void launch_rope_table(int seq, int d, float base, float* table, hipStream_t st) {
  const int n = seq * (d / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, seq, d / 2,
                     log((double)base), reinterpret_cast<float2*>(table));
}

void launch_rope(int dtype, int64_t rows, int seq, int H, int d, const float* table, void* qkv, int inverse,
                 hipStream_t st) {
  const int64_t n = rows * (2 * (int64_t)H / 8);
  const dim3 grid((unsigned)((n + 255) / 256));
  const float2* tb = reinterpret_cast<const float2*>(table);
  if (dtype == DT_FP32) hipLaunchKernelGGL(rope_kernel<float>, grid, dim3(256), 0, st, rows, seq, H, d, tb, (float*)qkv, inverse);
  else if (dtype == DT_FP16) hipLaunchKernelGGL(rope_kernel<f16_t>, grid, dim3(256), 0, st, rows, seq, H, d, tb, (f16_t*)qkv, inverse);
  else hipLaunchKernelGGL(rope_kernel<bf16_t>, grid, dim3(256), 0, st, rows, seq, H, d, tb, (bf16_t*)qkv, inverse);
}

}  // namespace slapo
