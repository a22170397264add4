// Host-side launch interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.h"

namespace slapo {

// true if `name` is listed in the SLAPO_DEBUG environment variable (comma-separated debugging / A-B switches)
bool debug_flag(const char* name);

enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };
// EPI_GATE: the product's columns are (gate, up) pairs; C [M,N/2] = silu(gate) * up, aux_out [M,N] = the pair
//   (up * silu'(gate), silu(gate)), the two factors backward multiplies the gradient of C with.
// EPI_DGATE: the product is that gradient [M,N]; C [M,2N] = (acc * aux_in[m,2n], acc * aux_in[m,2n+1]).
// EPI_SPLITK (internal to the weight-gradient path): the workgroup covers one of `act` K ranges of its tile and
//   writes the fp32 accumulators to aux_out (a float workspace [splits][M][N]); splitk_reduce sums them.
enum { EPI_NONE = 0, EPI_BIAS = 1, EPI_BIAS_ACT = 2, EPI_DACT = 3, EPI_ADD = 4, EPI_GATE = 5, EPI_DGATE = 6, EPI_SPLITK = 7 };

// solo: nothing else runs beside this GEMM (it may then pick tiles by round count, see launch_bf16)
// ws / ws_bytes: optional fp32 workspace (gemm_ws_bytes says how much a shape can use; 0: none). With it, a grid
//   of 256x256 tiles that would end in a thin last round computes its last tiles in several K ranges instead.
void launch_gemm(int dtype, int layout, int epi, int act, int M, int N, int K, const void* A, const void* B,
                 void* C, const void* bias, const void* aux_in, void* aux_out, hipStream_t st, bool solo = false,
                 float* ws = nullptr, size_t ws_bytes = 0);
size_t gemm_ws_bytes(int dtype, int epi, int M, int N, int K);
void describe_gemm(int dtype, int layout, int epi, int M, int N, int K, bool solo, bool weight_grad, bool with_ws,
                   char* buf, size_t len);
// Weight gradient C[M,N] (+)= A[K,M]^T B[K,N] (accumulate: add to C). Outputs with too few tiles to fill the
// chip are computed in several K ranges at once (fp32 partial tiles in `ws`, summed in range order by a second
// kernel: deterministic), outputs whose tile grid ends in a thin round have their last tiles cut into K ranges
// (launch_gemm); weight_grad_ws_bytes says how much workspace a shape wants (0: none, plain GEMM).
size_t weight_grad_ws_bytes(int dtype, int M, int N, int K);
void launch_weight_grad(int dtype, int accumulate, int M, int N, int K, const void* A, const void* B, void* C,
                        float* ws, hipStream_t st, bool solo = false);

struct AttnShape {
  int batch, seq, hidden, heads, causal;
  int lpt_heads = 0;   // causal block order: heads per longest-first group (set by the launchers; 0 = head by head)
  // dropout on the attention probabilities (site 2; element ((b*heads + a)*seq + i)*seq + j); thr == 0: none
  DropoutParams drop = {0u, 0u, 2u, 0u, 0u, 1.0f};
};
void launch_attn_fwd(int dtype, const AttnShape& s, const void* qkv, const int32_t* seqlens, void* out,
                     float* lse, hipStream_t st);
void launch_attn_bwd(int dtype, const AttnShape& s, const void* qkv, const int32_t* seqlens, const void* out,
                     const void* dout, const float* lse, float* delta, void* dqkv, hipStream_t st);

// rms: the normalisation is RMSNorm (no mean subtraction, no offset; beta, mu unused). bias may be null.
void launch_bdrln_fwd(int dtype, int64_t rows, int H, const void* r, const void* bias, const void* res,
                      const void* gamma, const void* beta, void* z_out, void* out, float* mu, float* rstd,
                      const DropoutParams& dp, float eps, int rms, hipStream_t st);
int bdrln_bwd_blocks(int64_t rows);
void launch_bdrln_bwd(int dtype, int64_t rows, int H, const void* dout, const void* z, const float* mu,
                      const float* rstd, const void* gamma, const void* dres_in, void* dz_out, void* dr_out,
                      float* partials, const DropoutParams& dp, int rms, hipStream_t st, int dr_from_stored = 0);
// Rotary embedding on the Q and K parts of a packed [rows, 3H] array, in place: inside every head of width d
// the adjacent pair (2j, 2j+1) of row t is turned by the angle of table entry (t % seq, j) (negated when
// `inverse`). table: [seq, d/2] (cos, sin) pairs in fp32, written by launch_rope_table (angle m * base^(-2j/d),
// evaluated in double precision).
void launch_rope_table(int seq, int d, float base, float* table, hipStream_t st);
void launch_rope(int dtype, int64_t rows, int seq, int H, int d, const float* table, void* qkv, int inverse,
                 hipStream_t st);
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
