// Host-side launch interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.h"

namespace slapo {

enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };
enum { EPI_NONE = 0, EPI_BIAS = 1, EPI_BIAS_ACT = 2, EPI_DACT = 3, EPI_ADD = 4 };

void launch_gemm(int dtype, int layout, int epi, int act, int M, int N, int K, const void* A, const void* B,
                 void* C, const void* bias, const void* aux_in, void* aux_out, hipStream_t st);

struct AttnShape {
  int batch, seq, hidden, heads, causal;
  // dropout on the attention probabilities (site 2; element ((b*heads + a)*seq + i)*seq + j); thr == 0: none
  DropoutParams drop = {0u, 0u, 2u, 0u, 0u, 1.0f};
};
void launch_attn_fwd(int dtype, const AttnShape& s, const void* qkv, const int32_t* seqlens, void* out,
                     float* lse, hipStream_t st);
void launch_attn_bwd(int dtype, const AttnShape& s, const void* qkv, const int32_t* seqlens, const void* out,
                     const void* dout, const float* lse, float* delta, void* dqkv, hipStream_t st);

void launch_bdrln_fwd(int dtype, int64_t rows, int H, const void* r, const void* bias, const void* res,
                      const void* gamma, const void* beta, void* z_out, void* out, float* mu, float* rstd,
                      const DropoutParams& dp, float eps, hipStream_t st);
int bdrln_bwd_blocks(int64_t rows);
void launch_bdrln_bwd(int dtype, int64_t rows, int H, const void* dout, const void* z, const float* mu,
                      const float* rstd, const void* gamma, const void* dres_in, void* dz_out, void* dr_out,
                      float* partials, const DropoutParams& dp, hipStream_t st);
int colsum_blocks(int64_t rows);
void launch_colsum_partials(int dtype, int64_t rows, int64_t N, const void* a, float* partials,
                            hipStream_t st);
void launch_colreduce_partials(int dtype, int64_t nblk, int64_t stride, int64_t N, const float* partials,
                               void* out, int accumulate, hipStream_t st);
// out_k[n] (+)= sum_i partials[(i*3 + k)*H + n] for k = 0..2 in one launch; null outputs are skipped
void launch_colreduce3(int dtype, int64_t nblk, int H, const float* partials, void* out0, void* out1, void* out2,
                       int accumulate, hipStream_t st);
void launch_dropout_mask(int64_t n_elements, uint8_t* mask, const DropoutParams& dp, hipStream_t st);

}  // namespace slapo
