/*
 * slapo_mi355x -- one transformer layer's training step (forward + backward) in the form a Slapo
 * schedule rewrites it to, as hand-written HIP kernels for gfx950 behind a C ABI.
 *
 * The scheduled layer (paper section 2.2 and the appendix schedule) consists of
 *   - one linear producing the concatenated Q,K,V (three nn.Linear fused into one),
 *   - a fused softmax-attention kernel working block by block (flash attention),
 *   - the output and second FFN linears with their bias "decomposed" out of the matmul,
 *   - F.gelu(bias + x) fused into the first FFN linear,
 *   - LayerNorm(dropout(bias + x) + residual) fused into one kernel after both blocks,
 * and the backward of all of these, which the paper leaves to autograd and this library derives
 * by hand.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, 16-byte aligned, row-major with
 *     the last index contiguous. The descriptor and the pointer tables are HOST structs.
 *   - Weights use the nn.Linear layout [out_features, in_features] (paper Fig. 3 caption).
 *   - `stream` is a hipStream_t passed as void*; all work is ordered after what was enqueued there
 *     before the call and before what is enqueued there afterwards; nothing synchronises with the host,
 *     no device memory is allocated or freed, no pointer is kept after the call returns.
 *     slapo_layer_bwd issues its weight-gradient GEMMs on one internal helper stream per device, created
 *     on first use and kept for the life of the process, forked from and joined back into `stream` with
 *     events (capturable in a HIP graph like any fork/join). This helper stream and its events are the only
 *     state the library holds besides the fixed scratch array of slapo_weight_grad_static.
 *   - Threads: every entry point may be called from several host threads at once, also on one device; calls
 *     touch only their own arguments. Backward calls of different threads on the same device share that
 *     device's helper stream: each event record and the stream wait that consumes it are issued under a
 *     per-device lock, so every call waits for its own records, and the weight-gradient work of concurrent
 *     calls queues up on the one helper stream in issue order (correct, but not concurrent with each other).
 *     Two calls that are given the same `scratch` or `saved` buffer must be ordered by the caller as usual.
 *   - SLAPO_DEBUG in the environment, read once at first use, is a comma-separated list of debugging / A-B
 *     timing switches: "single-stream" keeps all of backward on `stream`; "no-splitk" computes every weight
 *     gradient as one plain GEMM and "no-hybrid" every thin last round of tiles in one piece (both shrink the
 *     workspace sizes reported accordingly). Nothing else in the environment changes what the library does.
 *   - Return value: SLAPO_OK (0) or a negative slapo_status. Argument checks run before the first
 *     HIP call, so they behave the same on a host without a GPU. Nothing throws or aborts.
 *   - Same inputs and seed give bitwise identical outputs (no floating-point atomics anywhere).
 *   - Element type: SLAPO_BF16 or SLAPO_FP16 (16-bit storage, fp32 accumulation and fp32 elementwise math;
 *     the same kernels) or SLAPO_FP32 (fp32 everywhere; a correctness mode with simple kernels, not a tuned one).
 */
#ifndef SLAPO_MI355X_H
#define SLAPO_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SLAPO_OK = 0,
  SLAPO_ERR_NULL = -1,        /* a required pointer is NULL                                   */
  SLAPO_ERR_SHAPE = -2,       /* non-positive size, hidden % heads != 0, dropout_p not in [0,1) */
  SLAPO_ERR_UNSUPPORTED = -3, /* head dim not 64/128, hidden > 8192, fp32 seq limit, bad enum  */
  SLAPO_ERR_ALIGN = -4,       /* pointer not 16-byte aligned / size not a multiple of 8        */
  SLAPO_ERR_WORKSPACE = -5,   /* the shape needs more workspace than a fixed-size buffer of the library holds */
  SLAPO_ERR_HIP = -6          /* a kernel launch reported an error                             */
} slapo_status;

enum { SLAPO_BF16 = 0, SLAPO_FP32 = 1, SLAPO_FP16 = 2 };   /* FP16: IEEE half storage, fp32 accumulation, same kernels */
enum { SLAPO_GELU_ERF = 0, SLAPO_RELU = 1 };
/* Layer family. CLASSIC: the LayerNorm / bias / GeLU-or-ReLU layer described above (BERT, GPT, OPT ...).
 * LLAMA: the decoder layer of the LLaMA models the paper also evaluates (section 5.2), i.e. the classic
 * pre-norm layer with RMSNorm (y = z / sqrt(mean(z^2) + eps) * g) in place of LayerNorm, rotary position
 * embedding on queries and keys (adjacent pairs (2j, 2j+1) of every head turned by position * base^(-2j/d),
 * positions counted from 0 in every sequence), a SwiGLU feed-forward block (silu(n Wgate^T) * (n Wup^T)) W2^T
 * and no bias anywhere. */
enum { SLAPO_ARCH_CLASSIC = 0, SLAPO_ARCH_LLAMA = 1 };

/* Layer description (host struct). The head dim (hidden/heads, or attn_dim/heads) must be 64 or 128; hidden,
 * ffn multiples of 8; hidden <= 8192; in the fp32 mode seq <= 5056 (d = 64) / 4992 (d = 128). */
typedef struct {
  int32_t batch, seq, hidden, heads, ffn;
  int32_t causal;           /* 1: query i sees keys j <= i                                     */
  float dropout_p;          /* probability of dropping, in [0,1); applied at the two fused
                               bias+dropout+residual sites (attention probabilities: see below) */
  uint64_t seed;            /* dropout seed (Philox key)                                       */
  int32_t dtype;            /* SLAPO_BF16 | SLAPO_FP32 | SLAPO_FP16: activations, weights, gradients */
  int32_t act;              /* SLAPO_GELU_ERF (0.5 u (1 + erf(u/sqrt 2))) | SLAPO_RELU         */
  int32_t pre_ln;           /* 0: y = LN(x + f(x)) (BERT); 1: y = x + f(LN(x)) (GPT/OPT)       */
  int32_t layer_id;         /* mixed into the dropout counter so stacked layers differ         */
  float ln_eps;             /* LayerNorm epsilon (inside the square root)                      */
  int32_t accumulate_grads; /* 0: overwrite parameter gradients, 1: add to them                */
  int32_t checkpoint;       /* 1: activation checkpointing (the third optimisation the paper's schedules apply,
                               section 2.2): forward keeps nothing, backward recomputes the
                               forward from x first. No `saved` buffer exists (size 0, the argument is
                               ignored and may be NULL); `scratch` is larger instead. The regenerated
                               dropout masks make the recomputation exact: gradients are bit for bit
                               those of checkpoint = 0.                                          */
  float attn_dropout_p;     /* dropout on the attention probabilities, in [0,1): the
                               dropout(softmax(attn), p) of the attention listing in section 2.2 step 2,
                               applied inside the fused attention kernels (mask stream: site 2, element
                               ((b*heads + a)*seq + i)*seq + j; needs seq % 8 == 0). 0 = none.     */
  int32_t arch;             /* SLAPO_ARCH_CLASSIC | SLAPO_ARCH_LLAMA (needs pre_ln = 1; act is ignored) */
  float rope_base;          /* LLAMA: base of the rotary frequencies (10000 in the published models), > 1 */
  int32_t attn_dim;         /* width W = heads * head dim of each of Q, K, V when it differs from hidden; 0 = hidden.
                               W/heads must be 64 or 128. With W != hidden, wqkv is [3W,hidden], bqkv [3W], wo
                               [hidden,W], and every "[.., 3H]" / attention "[.., H]" shape below reads 3W / W.
                               This is one rank's share of a layer whose fused QKV and output projections are
                               sharded along the heads (section 2.2 step 3): heads/tp heads, W = hidden/tp, and
                               ffn = F/tp for the feed-forward shards; the all-reduces between the shares are the
                               caller's (the output is then this rank's partial layer, biases included).      */
} slapo_layer_desc;

/* Parameters: wqkv [3H,H] = [Wq;Wk;Wv] stacked on the output dim, bqkv [3H], wo [H,H], bo [H],
 * ln1_g/ln1_b [H], w1 [F,H], b1 [F], w2 [H,F], b2 [H], ln2_g/ln2_b [H].
 * Post-LN: ln1 follows the attention block, ln2 follows the FFN block.
 * Pre-LN:  ln1 precedes the attention block, ln2 precedes the FFN block.
 * SLAPO_ARCH_LLAMA uses wqkv, wo, ln1_g, w1, w2, ln2_g only (the other entries are ignored and may be NULL;
 * no gradient is written for them). Its w1 is [2F,H] and holds the gate and up projections interleaved by
 * rows: row 2c = gate row c, row 2c+1 = up row c, so that one product yields both and a (gate, up) pair
 * lands in adjacent columns; its gradient has the same layout. */
typedef struct {
  const void *wqkv, *bqkv, *wo, *bo, *ln1_g, *ln1_b, *w1, *b1, *w2, *b2, *ln2_g, *ln2_b;
} slapo_layer_params;
typedef struct {
  void *wqkv, *bqkv, *wo, *bo, *ln1_g, *ln1_b, *w1, *b1, *w2, *b2, *ln2_g, *ln2_b;
} slapo_layer_grads;

/* Sizes in bytes of the two caller-provided device buffers: `saved` carries activations from
 * slapo_layer_fwd to slapo_layer_bwd (QKV, attention output, logsumexp, pre-norm sums, LayerNorm
 * statistics, FFN activation and activation derivative) and must stay untouched in between; `scratch` is
 * free for reuse as soon as a call's work has completed on the stream (so one scratch buffer can serve
 * every layer of a stack). With desc->checkpoint = 1, saved_bytes is 0. */
int slapo_layer_workspace(const slapo_layer_desc *desc, size_t *saved_bytes, size_t *scratch_bytes);

/* Named regions inside `saved`, for tests and tools. Writes byte offset and byte length; returns
 * SLAPO_ERR_UNSUPPORTED if the region does not exist for this wiring. Names: "qkv" [T,3H], "attn"
 * [T,H], "lse" [B,heads,S] fp32, "z1" [T,H], "n1" (pre-LN) [T,H], "y1" (post-LN) / "n2" (pre-LN)
 * [T,H], "dact" [T,F] (act'(u) of the FFN pre-activation u; GeLU layers only, a ReLU layer reads its gate
 * off "g"), "g" [T,F], "z2" (post-LN) [T,H], "mu1","rstd1","mu2","rstd2" [T] fp32.
 * SLAPO_ARCH_LLAMA: "qkv" holds the rotated queries and keys, "dgate" [T,2F] replaces "dact" (column 2c:
 * up_c * silu'(gate_c), column 2c+1: silu(gate_c)), "mu1"/"mu2" are unused. */
int slapo_layer_saved_region(const slapo_layer_desc *desc, const char *name, size_t *offset, size_t *bytes);

/* Forward of the scheduled layer (section 2.2 steps 1-2, appendix schedule):
 *   post-LN: QKV = x Wqkv^T + bqkv; A = attention(QKV); Z1 = x + drop0(A Wo^T + bo); Y1 = LN1(Z1);
 *            G = act(Y1 W1^T + b1); Z2 = Y1 + drop1(G W2^T + b2); y = LN2(Z2)
 *   pre-LN:  N1 = LN1(x); QKV from N1; Z1 = x + drop0(A Wo^T + bo); N2 = LN2(Z1);
 *            G = act(N2 W1^T + b1); y = Z1 + drop1(G W2^T + b2)
 *   LLAMA:   N1 = RMSNorm1(x); QKV = rotate(N1 Wqkv^T); Z1 = x + drop0(A Wo^T); N2 = RMSNorm2(Z1);
 *            (gate, up) = N2 W1^T; G = silu(gate) * up; y = Z1 + drop1(G W2^T)
 * x, y: [B,S,H]. seqlens: device int32 [B] with 1 <= seqlens[b] <= S (keys j >= seqlens[b] are
 * hidden from every query of sample b), or NULL for no padding mask; may be combined with causal. */
int slapo_layer_fwd(const slapo_layer_desc *desc, const slapo_layer_params *params, const void *x,
                    const int32_t *seqlens, void *y, void *saved, void *scratch, void *stream);

/* Backward: given dy = dL/dy [B,S,H] and the `saved` buffer of the matching forward, writes
 * dx [B,S,H] and the parameter gradients (twelve; six for SLAPO_ARCH_LLAMA; same shapes and element type as
 * the parameters).
 * The dropout masks are regenerated from (seed, layer_id, site, element index), never stored. */
int slapo_layer_bwd(const slapo_layer_desc *desc, const slapo_layer_params *params, const void *x,
                    const int32_t *seqlens, const void *dy, const void *saved, void *dx,
                    const slapo_layer_grads *grads, void *scratch, void *stream);

/* A stack of n_layers layers of one shape (the evaluation's encoder stacks, section 5): layer l runs with
 * layer_id = desc->layer_id + l (so its dropout masks differ), parameters params[l] and gradients grads[l]
 * (host arrays of n_layers pointer tables). Forward feeds x through the layers into y; backward takes
 * dy = dL/dy at the top and produces every layer's parameter gradients and dx = dL/dx at the bottom.
 *   acts:    device, (n_layers-1) x [B,S,H]: the outputs of layers 0..n_layers-2, kept from forward to backward
 *            (may be NULL for one layer)
 *   saved:   device, n_layers x the `saved` buffer of one layer (size 0 / ignored with desc->checkpoint: then
 *            acts and x are all that survives the forward pass)
 *   scratch: device, one layer's scratch plus two (pre-LN: four) [B,S,H] gradient buffers; free between calls
 * Pre-LN stacks fuse across the layer boundary: the last forward kernel of a layer also writes the first
 * LayerNorm of the layer above, the last backward kernel of a layer also writes the first gradient of the
 * layer below. Results are bit for bit those of the layers called one at a time.
 * Sizes come from slapo_stack_workspace. Errors as for the layer calls (every layer's tables are checked
 * before the first launch); n_layers <= 0 is SLAPO_ERR_SHAPE. */
int slapo_stack_workspace(const slapo_layer_desc *desc, int32_t n_layers, size_t *acts_bytes, size_t *saved_bytes,
                          size_t *scratch_bytes);
int slapo_stack_fwd(const slapo_layer_desc *desc, int32_t n_layers, const slapo_layer_params *params, const void *x,
                    const int32_t *seqlens, void *y, void *acts, void *saved, void *scratch, void *stream);
int slapo_stack_bwd(const slapo_layer_desc *desc, int32_t n_layers, const slapo_layer_params *params, const void *x,
                    const int32_t *seqlens, const void *dy, const void *acts, const void *saved, void *dx,
                    const slapo_layer_grads *grads, void *scratch, void *stream);

const char *slapo_status_string(int status);

/* ---- building blocks, exported for per-kernel tests and measurement ---------------------------- */

/* GEMM C[M,N] = op(A) op(B) with fp32 accumulation and a fused epilogue.
 *   layout 0 (NT): A [M,K], B [N,K]   -- forward linears x W^T (fused QKV, output, FFN)
 *   layout 1 (NN): A [M,K], B [K,N]   -- input gradients dY W
 *   layout 2 (TN): A [K,M], B [K,N]   -- weight gradients dY^T X
 *   epilogue 0: C = acc                       1: C = acc + bias[n]
 *            2: u = acc + bias[n]; C = act(u), aux_out = act'(u)   (F.gelu(bias + x), appendix schedule;
 *               the derivative is all that backward needs of u, and its terms are at hand here; with
 *               act = SLAPO_RELU aux_out may be NULL: the derivative [u > 0] equals [C > 0])
 *            3: GeLU: C = acc * aux_in[m,n] (aux_in = the aux_out of epilogue 2); ReLU: C = acc * [aux_in[m,n] > 0]
 *               (aux_in = the C or the aux_out of epilogue 2)   4: C = acc + aux_in[m,n]  (aux_in may alias C)
 *            5: columns are (gate, up) pairs (N % 16 == 0): C [M,N/2] = silu(gate) * up,
 *               aux_out [M,N] = (up * silu'(gate), silu(gate)) per pair            (SwiGLU forward)
 *            6: C [M,2N] = (acc * aux_in[m,2n], acc * aux_in[m,2n+1]), aux_in [M,2N] = the aux_out of
 *               epilogue 5: the gradient of the gated values turned into (gate, up) gradient pairs
 * M, N, K > 0; K-contiguous operands need K % 8 == 0, M/N-contiguous ones M % 8 / N % 8 == 0;
 * N % 8 == 0. */
int slapo_gemm(int dtype, int layout, int epilogue, int act, int64_t M, int64_t N, int64_t K,
               const void *A, const void *B, void *C, const void *bias, const void *aux_in,
               void *aux_out, void *stream);

/* slapo_gemm with options, as the layer calls use the kernels.
 *   flags: SLAPO_GEMM_SHARED selects tiles as slapo_layer_bwd does for the GEMMs of its data-gradient chain while the
 *          helper stream's weight gradients share the chip (slapo_gemm, like the forward pass, selects for a GEMM that
 *          runs alone: it may take 128x128 tiles where a grid of 256x256 tiles would end in a thin last round).
 *   ws, ws_bytes: optional device workspace (16-byte aligned; free again when the call's work is done). With it, a
 *          plain or add-epilogue GEMM (epilogue 0 or 4) whose grid of 256x256 tiles is not a multiple of the 256 CUs
 *          and whose K is long computes the tiles beyond the last full round in several K ranges (fp32 partial tiles
 *          in ws, added in range order by a second kernel: bitwise reproducible), so that the last round is short
 *          instead of thin. slapo_gemm_workspace writes the bytes a shape can use (0: it runs as slapo_gemm would);
 *          a non-NULL ws smaller than that is refused with SLAPO_ERR_WORKSPACE. The layer calls do the same with a
 *          region of their scratch buffer. */
enum { SLAPO_GEMM_SHARED = 1 };
int slapo_gemm_workspace(int dtype, int layout, int epilogue, int64_t M, int64_t N, int64_t K, size_t *ws_bytes);
int slapo_gemm_ex(int dtype, int layout, int epilogue, int act, int64_t M, int64_t N, int64_t K,
                  const void *A, const void *B, void *C, const void *bias, const void *aux_in,
                  void *aux_out, int flags, void *ws, size_t ws_bytes, void *stream);
/* Writes the kernel instance a GEMM of this shape is launched as into buf (NUL-terminated, truncated to len), spelt
 * as a profiler prints the symbol. flags as for slapo_gemm_ex; with_ws != 0: as launched with a sufficient
 * workspace; weight_grad != 0 (layout 2 only): the selection of slapo_weight_grad, K ranges included. Host-only. */
int slapo_gemm_kernel_name(int dtype, int layout, int epilogue, int64_t M, int64_t N, int64_t K, int flags,
                           int weight_grad, int with_ws, char *buf, size_t len);

/* Weight gradient C[M,N] (+)= A[K,M]^T B[K,N] (layout 2 with K = tokens; accumulate != 0 adds to C). When the
 * output has too few 128x128 tiles to fill the chip and K is a long multiple of 256 (at least 6144), the product is
 * computed in up to 8 K ranges at once, as fp32 partial tiles in `ws` that a second kernel adds in range order (bitwise
 * reproducible); an output with many tiles whose grid ends in a thin round uses `ws` as slapo_gemm_ex does.
 * slapo_weight_grad_workspace writes the bytes of `ws` a shape wants (0: the plain GEMM is used
 * and ws may be NULL; also for SLAPO_FP32). ws: device, 16-byte aligned, free again when the call's work is done.
 * slapo_layer_bwd uses this path for its four weight gradients with a region of its scratch buffer. */
int slapo_weight_grad_workspace(int dtype, int64_t M, int64_t N, int64_t K, size_t *ws_bytes);
int slapo_weight_grad(int dtype, int accumulate, int64_t M, int64_t N, int64_t K, const void *A, const void *B,
                      void *C, void *ws, void *stream);

/* slapo_weight_grad for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving / training loops, harnesses that forbid allocation. Same arguments without `ws`, same
 * results bit for bit. The fp32 partial tiles of the K-range path live in a fixed 16 MiB array in device memory that
 * is part of the library's code object (one copy per GPU the library runs on, held until the process ends); the call
 * allocates and frees nothing. A shape whose partial tiles would not fit returns SLAPO_ERR_WORKSPACE before anything
 * is launched (with the current rule - at most 256 partial tiles of 128x128 - every shape fits; the check guards the
 * array). The array keeps the last call's contents and nothing in it needs clearing: every partial tile a call reads
 * it has written itself. All calls on one GPU share the array, so two calls whose work may overlap in time on one GPU
 * (different streams, different host threads) race on it: order them, or use slapo_weight_grad with a workspace each.
 * The device address of the array is looked up on the first call on each device; make that call outside any graph
 * capture. At most 16 devices per process. */
int slapo_weight_grad_static(int dtype, int accumulate, int64_t M, int64_t N, int64_t K, const void *A, const void *B,
                             void *C, void *stream);

/* Fused softmax attention over the packed projection qkv [B,S,3H] (Q | K | V on the last axis,
 * head a owning columns a*d..a*d+d-1 of each): out [B,S,H], lse [B,heads,S] fp32 holding
 * log sum_j exp(q_i.k_j/sqrt(d)) over the visible keys (natural log). Uses desc->batch, seq, hidden,
 * heads, causal, dtype. The S x S matrix never reaches memory (section 2.2 step 2). */
int slapo_attn_fwd(const slapo_layer_desc *desc, const void *qkv, const int32_t *seqlens, void *out,
                   float *lse, void *stream);

/* Backward of slapo_attn_fwd: recomputes probabilities from lse; delta [B,heads,S] fp32 is scratch
 * for rowsum(dout*out). Writes the packed dqkv [B,S,3H]. */
int slapo_attn_bwd(const slapo_layer_desc *desc, const void *qkv, const int32_t *seqlens,
                   const void *out, const void *dout, const float *lse, float *delta, void *dqkv,
                   void *stream);

/* z = res + keep * (r + bias) / (1 - p)   (bias, dropout, residual; skipped if r == NULL, then z := res)
 * out = LayerNorm(z; gamma, beta), mu/rstd [T] fp32   (skipped if gamma == NULL)
 * With desc->arch == SLAPO_ARCH_LLAMA the normalisation is RMSNorm (beta and mu are ignored and may be NULL;
 * rstd = 1/sqrt(mean(z^2) + eps)) and bias may be NULL (= 0); the same holds for slapo_bdrln_bwd (mu ignored).
 * T rows of H elements. z_out may be NULL when only `out` is wanted (r == NULL case).
 * site selects the dropout stream (0 after attention, 1 after the FFN). */
int slapo_bdrln_fwd(const slapo_layer_desc *desc, int site, int64_t T, const void *r, const void *bias,
                    const void *res, const void *gamma, const void *beta, void *z_out, void *out,
                    float *mu, float *rstd, void *stream);

/* Backward of the fused pattern. With gamma != NULL: dz = dres_in + LayerNorm'(dout; z, mu, rstd, gamma)
 * and partial sums of dgamma = sum_t dout*xhat, dbeta = sum_t dout; with gamma == NULL: dz = dout
 * (+ dres_in). If dr_out != NULL: dr = dz * keep / (1-p) (mask regenerated) and partial sums of
 * dbias = sum_t dr. dz_out may be NULL. partials: fp32 [nblk, 3, H] (rows: dgamma, dbeta, dbias) with
 * nblk = slapo_bdrln_bwd_blocks(T); reduce them with slapo_colreduce_partials. */
int slapo_bdrln_bwd(const slapo_layer_desc *desc, int site, int64_t T, const void *dout, const void *z,
                    const float *mu, const float *rstd, const void *gamma, const void *dres_in,
                    void *dz_out, void *dr_out, float *partials, void *stream);
int slapo_bdrln_bwd_blocks(int64_t T);

/* Rotary embedding (SLAPO_ARCH_LLAMA descriptors only), in place on the Q and K parts of a packed [B,S,3H] array:
 * pair (2j, 2j+1) of every head at position m is turned by m * rope_base^(-2j/d), by the negative angle if
 * `inverse` (the transpose, which maps gradients w.r.t. rotated vectors back). table: device scratch of
 * seq * d/2 * 8 bytes that receives the (cos, sin) pairs. */
int slapo_rope(const slapo_layer_desc *desc, void *qkv, float *table, int inverse, void *stream);

/* Column sums of a [T,N] matrix in two deterministic stages: partials fp32 [nblk,N] with
 * nblk = slapo_colsum_blocks(T), then slapo_colreduce_partials. */
int slapo_colsum_partials(int dtype, int64_t T, int64_t N, const void *a, float *partials, void *stream);
int slapo_colsum_blocks(int64_t T);
/* out[n] (element type dtype) = (accumulate ? out[n] : 0) + sum_i partials[i*stride + n], i < nblk. */
int slapo_colreduce_partials(int dtype, int64_t nblk, int64_t stride, int64_t N, const float *partials,
                             void *out, int accumulate, void *stream);

/* Writes the keep decisions (1 = kept, 0 = dropped) of one dropout site as bytes [T*H]:
 * element e = t*H + c uses Philox4x32-10 with counter (lo32(e>>3), hi32(e>>3), site, layer_id),
 * key (lo32(seed), hi32(seed)), 16-bit draw (out[(e&7)>>1] >> 16*(e&1)) & 0xffff, kept iff
 * draw >= round(p * 65536). */
int slapo_dropout_mask(const slapo_layer_desc *desc, int site, int64_t T, uint8_t *mask, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SLAPO_MI355X_H */
