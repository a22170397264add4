// C ABI of the library: argument validation, layout of the `saved` / `scratch` buffers and the
// sequence of kernel launches that makes up one layer forward / backward. Host code only.
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/slapo.h"
#include "kernels.h"

using namespace slapo;

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// width of each of Q, K, V (heads * head dim): the hidden size unless the descriptor says otherwise
inline int attn_width(const slapo_layer_desc* d) { return d->attn_dim > 0 ? d->attn_dim : d->hidden; }

int check_desc(const slapo_layer_desc* d) {
  if (!d) return SLAPO_ERR_NULL;
  if (d->batch <= 0 || d->seq <= 0 || d->hidden <= 0 || d->heads <= 0 || d->ffn <= 0 || d->attn_dim < 0) return SLAPO_ERR_SHAPE;
  if (attn_width(d) % d->heads != 0) return SLAPO_ERR_SHAPE;
  if (!(d->dropout_p >= 0.f && d->dropout_p < 1.f)) return SLAPO_ERR_SHAPE;
  if (!(d->ln_eps > 0.f)) return SLAPO_ERR_SHAPE;
  if (d->hidden % 8 != 0 || d->ffn % 8 != 0) return SLAPO_ERR_ALIGN;
  const int hd = attn_width(d) / d->heads;
  if (hd != 64 && hd != 128) return SLAPO_ERR_UNSUPPORTED;
  if (d->hidden > 8192) return SLAPO_ERR_UNSUPPORTED;   // the row kernels hold a row per wavefront / per block
  // the fp32 (correctness-mode) attention keeps two score rows per wavefront in LDS: 16 (2 d + 2 seq) bytes per block
  if (d->dtype == SLAPO_FP32 && (int64_t)16 * (2 * hd + 2 * (int64_t)d->seq) > 160 * 1024) return SLAPO_ERR_UNSUPPORTED;
  if (d->dtype != SLAPO_BF16 && d->dtype != SLAPO_FP32 && d->dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (d->act != SLAPO_GELU_ERF && d->act != SLAPO_RELU) return SLAPO_ERR_UNSUPPORTED;
  if ((d->causal != 0 && d->causal != 1) || (d->pre_ln != 0 && d->pre_ln != 1)) return SLAPO_ERR_UNSUPPORTED;
  if (d->checkpoint != 0 && d->checkpoint != 1) return SLAPO_ERR_UNSUPPORTED;
  if (!(d->attn_dropout_p >= 0.f && d->attn_dropout_p < 1.f)) return SLAPO_ERR_SHAPE;
  if (d->attn_dropout_p > 0.f && d->seq % 8 != 0) return SLAPO_ERR_ALIGN;   // a mask block of 8 keys stays inside one query row
  if ((int64_t)d->batch * d->seq * 3 * d->hidden >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  if ((int64_t)d->batch * d->seq * 3 * attn_width(d) >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  if ((int64_t)d->batch * d->seq * d->ffn >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  if (d->arch != SLAPO_ARCH_CLASSIC && d->arch != SLAPO_ARCH_LLAMA) return SLAPO_ERR_UNSUPPORTED;
  if (d->arch == SLAPO_ARCH_LLAMA) {
    if (!d->pre_ln) return SLAPO_ERR_UNSUPPORTED;                    // the family is pre-norm by definition
    if (!(d->rope_base > 1.f)) return SLAPO_ERR_SHAPE;
    if ((int64_t)d->batch * d->seq * 2 * d->ffn >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  }
  return SLAPO_OK;
}

inline bool is_llama(const slapo_layer_desc* d) { return d->arch == SLAPO_ARCH_LLAMA; }
inline bool keeps_dact(const slapo_layer_desc* d) { return is_llama(d) || d->act != SLAPO_RELU; }
// The pointer tables list weight, bias (or gain, offset) alternately; the LLaMA-style layer has the six
// weights and gains only, i.e. the even entries.
inline bool param_needed(const slapo_layer_desc* d, int index) { return !is_llama(d) || index % 2 == 0; }
int check_tables(const slapo_layer_desc* d, const void* const (&ps)[12]) {
  for (int i = 0; i < 12; ++i) {
    if (!param_needed(d, i)) continue;
    if (!ps[i]) return SLAPO_ERR_NULL;
    if (misaligned(ps[i])) return SLAPO_ERR_ALIGN;
  }
  return SLAPO_OK;
}

}  // namespace

namespace slapo {
// SLAPO_DEBUG in the environment: a comma-separated list of switches for debugging and A/B timing, read once.
//   single-stream  backward keeps all of its work on the caller's stream (no helper stream)
//   no-splitk      weight gradients always run as one plain GEMM (no K ranges; also shrinks the workspace sizes
//                  the *_workspace calls report, so set it before the first call, not between size query and use)
bool debug_flag(const char* name) {
  const char* env = getenv("SLAPO_DEBUG");
  if (!env) return false;
  const size_t n = strlen(name);
  for (const char* p = env; *p;) {
    const char* e = strchr(p, ',');
    const size_t len = e ? (size_t)(e - p) : strlen(p);
    if (len == n && !strncmp(p, name, n)) return true;
    p += len + (e ? 1 : 0);
  }
  return false;
}
}  // namespace slapo

namespace {

DropoutParams make_dropout(const slapo_layer_desc* d, int site) {
  DropoutParams dp;
  dp.key0 = (uint32_t)(d->seed & 0xffffffffu);
  dp.key1 = (uint32_t)(d->seed >> 32);
  dp.site = (uint32_t)site;
  dp.layer = (uint32_t)d->layer_id;
  dp.thr = (uint32_t)llround((double)d->dropout_p * 65536.0);
  dp.scale = 1.0f / (1.0f - d->dropout_p);
  return dp;
}

AttnShape make_attn_shape(const slapo_layer_desc* d) {
  AttnShape as = {d->batch, d->seq, attn_width(d), d->heads, d->causal};
  as.drop.key0 = (uint32_t)(d->seed & 0xffffffffu);
  as.drop.key1 = (uint32_t)(d->seed >> 32);
  as.drop.site = 2u;
  as.drop.layer = (uint32_t)d->layer_id;
  as.drop.thr = (uint32_t)llround((double)d->attn_dropout_p * 65536.0);
  as.drop.scale = 1.0f / (1.0f - d->attn_dropout_p);
  return as;
}

// A launch that failed leaves its error in the runtime's per-thread "last error". Every entry point samples that
// slot before its first launch (entry_error) and again after its last one (finish): an error that was already
// there belongs to somebody else and is neither reported as ours nor cleared; one that appeared in between is
// ours, is reported as SLAPO_ERR_HIP and cleared.
thread_local hipError_t g_error_at_entry = hipSuccess;
void entry_error() { g_error_at_entry = hipPeekAtLastError(); }
int finish() {
  if (g_error_at_entry != hipSuccess) return SLAPO_OK;   // cannot tell ours from the stale one: leave it to its owner
  return hipGetLastError() == hipSuccess ? SLAPO_OK : SLAPO_ERR_HIP;
}

// The weight-gradient GEMMs of the backward pass do not feed the data-gradient chain, and most kernels of
// the chain leave half of each CU's LDS and wave slots free (one 128x128 tile per CU). They are therefore
// issued on a helper stream that forks from and joins back into the caller's stream with events, so the
// two kinds of GEMM share the CUs. One helper stream and a few events per device are created on first use
// and kept for the life of the process (the only state the library holds). Host threads that call into the
// library on the same device share them: every event record and the stream wait that consumes it are issued
// under the device's mutex, so a wait always captures the record of its own call (a wait refers to the
// record that precedes it at the time it is issued), and the calls' helper-stream work simply queues up
// behind each other. "single-stream" in SLAPO_DEBUG turns the helper stream off.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork[4] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t join = nullptr;
  int state = 0;   // 0 untried, 1 ready, -1 unavailable
  std::mutex pair_mu;   // held across each (record, wait) pair
  // everything issued on `from` so far happens before what is issued on `to` from now on
  void order(hipEvent_t ev, hipStream_t from, hipStream_t to) {
    std::lock_guard<std::mutex> lock(pair_mu);
    (void)hipEventRecord(ev, from);
    (void)hipStreamWaitEvent(to, ev, 0);
  }
};
SideStream* side_stream() {
  static SideStream table[16];
  static std::mutex mu;
  static const bool disabled = debug_flag("single-stream");
  if (disabled) return nullptr;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  SideStream& s = table[dev];
  if (s.state == 0) {
    bool ok = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess;
    // the events order work of two streams of ONE device: no timing, and no system-scope fence at the record
    // (the host and other devices never look at what they guard; the fence cost ~7 us of idle stream per fork)
    const unsigned flags = hipEventDisableTiming | hipEventDisableSystemFence;
    for (int i = 0; ok && i < 4; ++i) ok = hipEventCreateWithFlags(&s.fork[i], flags) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&s.join, flags) == hipSuccess;
    s.state = ok ? 1 : -1;
    if (!ok) (void)hipGetLastError();
  }
  return s.state == 1 ? &s : nullptr;
}

// byte offsets of the regions of `saved`
struct SavedLayout {
  size_t qkv, attn, lse, z1, n1, y1, u, g, z2, mu1, rstd1, mu2, rstd2, total;
};
SavedLayout saved_layout(const slapo_layer_desc* d) {
  const size_t eb = d->dtype == SLAPO_FP32 ? 4 : 2;
  const size_t T = (size_t)d->batch * d->seq, H = d->hidden, F = d->ffn, A = attn_width(d);
  SavedLayout L;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align256(o + bytes); return at; };
  L.qkv = take(T * 3 * A * eb);
  L.attn = take(T * A * eb);
  L.lse = take((size_t)d->batch * d->heads * d->seq * 4);
  L.z1 = take(T * H * eb);
  L.n1 = d->pre_ln ? take(T * H * eb) : (size_t)-1;
  L.y1 = take(T * H * eb);  // post-LN: LN1 output; pre-LN: LN2 output ("n2")
  // act'(u) of a GeLU layer, or the (gate, up) factor pairs [T,2F]; a ReLU layer keeps nothing here: its
  // derivative is [g > 0], read off the activation output it keeps anyway
  L.u = keeps_dact(d) ? take(T * F * eb * (is_llama(d) ? 2 : 1)) : (size_t)-1;
  L.g = take(T * F * eb);
  L.z2 = d->pre_ln ? (size_t)-1 : take(T * H * eb);
  L.mu1 = take(T * 4);
  L.rstd1 = take(T * 4);
  L.mu2 = take(T * 4);
  L.rstd2 = take(T * 4);
  L.total = o;
  return L;
}

struct ScratchLayout {
  size_t t0, t1, t2, t3, du, dqkv, delta, part_row, part_col, part_col2, rope, splitk, gemm_ws, gemm_ws_bytes, splitk_bytes, acts, total;
};
ScratchLayout scratch_layout(const slapo_layer_desc* d) {
  const size_t eb = d->dtype == SLAPO_FP32 ? 4 : 2;
  const size_t T = (size_t)d->batch * d->seq, H = d->hidden, F = d->ffn, A = attn_width(d);
  ScratchLayout L;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align256(o + bytes); return at; };
  L.t0 = take(T * (H > A ? H : A) * eb);   // also holds the gradient of the attention output [T,A]
  L.t1 = take(T * H * eb);
  L.t2 = take(T * H * eb);
  L.t3 = take(T * H * eb);
  L.du = take(T * F * eb * (is_llama(d) ? 2 : 1));
  L.dqkv = take(T * 3 * A * eb);
  L.delta = take((size_t)d->batch * d->heads * d->seq * 4);
  L.part_row = take((size_t)bdrln_bwd_blocks((int64_t)T) * 3 * H * 4);
  const size_t widest = F > 3 * A ? F : 3 * A;
  L.part_col = take((size_t)colsum_blocks((int64_t)T) * widest * 4);
  L.part_col2 = take((size_t)colsum_blocks((int64_t)T) * widest * 4);   // the two streams of backward each own one
  L.rope = is_llama(d) ? take((size_t)d->seq * (A / d->heads / 2) * 8) : 0;   // (cos, sin) table
  // fp32 partial tiles of the weight gradients that are computed in several K ranges (one at a time: all of them
  // run on the helper stream); 0 for shapes that fill the chip with plain tiles
  {
    const int Ti = (int)T, Hi = (int)H, Fi = (int)F, Ai = (int)A, F1 = is_llama(d) ? 2 * Fi : Fi;
    size_t w = weight_grad_ws_bytes(d->dtype, Hi, Fi, Ti);
    const size_t w1 = weight_grad_ws_bytes(d->dtype, F1, Hi, Ti), wo = weight_grad_ws_bytes(d->dtype, Hi, Ai, Ti);
    const size_t wq = weight_grad_ws_bytes(d->dtype, 3 * Ai, Hi, Ti);
    w = w > w1 ? w : w1; w = w > wo ? w : wo; w = w > wq ? w : wq;
    L.splitk = w ? take(w) : 0;
    L.splitk_bytes = w;
    // the same kind of workspace for the GEMMs of the forward pass and of the data-gradient chain whose tile grid
    // would end in a thin round (their last tiles are then computed in K ranges); a region of its own, because
    // the chain runs while the helper stream's weight gradients use the one above
    size_t g = gemm_ws_bytes(d->dtype, EPI_NONE, Ti, Hi, Ai);                       // attention output projection
    auto upto = [&](size_t v) { g = g > v ? g : v; };
    upto(gemm_ws_bytes(d->dtype, EPI_NONE, Ti, Hi, Fi));                             // second FFN product
    upto(gemm_ws_bytes(d->dtype, EPI_NONE, Ti, Hi, F1));                             // gradient of the FFN input
    upto(gemm_ws_bytes(d->dtype, EPI_NONE, Ti, Ai, Hi));                             // gradient of the attention output
    upto(gemm_ws_bytes(d->dtype, EPI_NONE, Ti, Hi, 3 * Ai));                         // gradient of the attention input
    L.gemm_ws = g ? take(g) : 0;
    L.gemm_ws_bytes = g;
  }
  // checkpoint mode: the activations that forward would hand to backward live here instead, for the
  // duration of one call only (backward recomputes them), so the caller keeps nothing per layer but x
  L.acts = d->checkpoint ? take(saved_layout(d).total) : 0;
  L.total = o;
  return L;
}

}  // namespace

extern "C" {

const char* slapo_status_string(int status) {
  switch (status) {
    case SLAPO_OK: return "ok";
    case SLAPO_ERR_NULL: return "a required pointer is NULL";
    case SLAPO_ERR_SHAPE: return "invalid shape or scalar argument";
    case SLAPO_ERR_UNSUPPORTED: return "unsupported configuration";
    case SLAPO_ERR_ALIGN: return "pointer not 16-byte aligned or size not a multiple of 8";
    case SLAPO_ERR_WORKSPACE: return "shape needs more workspace than the library's fixed-size buffer holds";
    case SLAPO_ERR_HIP: return "HIP reported an error";
    default: return "unknown status";
  }
}

int slapo_layer_workspace(const slapo_layer_desc* desc, size_t* saved_bytes, size_t* scratch_bytes) {
  if (!saved_bytes || !scratch_bytes) return SLAPO_ERR_NULL;
  const int rc = check_desc(desc);
  if (rc) return rc;
  *saved_bytes = desc->checkpoint ? 0 : saved_layout(desc).total;
  *scratch_bytes = scratch_layout(desc).total;
  return SLAPO_OK;
}

int slapo_layer_saved_region(const slapo_layer_desc* desc, const char* name, size_t* offset, size_t* bytes) {
  if (!name || !offset || !bytes) return SLAPO_ERR_NULL;
  const int rc = check_desc(desc);
  if (rc) return rc;
  const SavedLayout L = saved_layout(desc);
  const size_t eb = desc->dtype == SLAPO_FP32 ? 4 : 2;
  const size_t T = (size_t)desc->batch * desc->seq, H = desc->hidden, F = desc->ffn, A = attn_width(desc);
  size_t off = (size_t)-1, len = 0;
  if (!strcmp(name, "qkv")) { off = L.qkv; len = T * 3 * A * eb; }
  else if (!strcmp(name, "attn")) { off = L.attn; len = T * A * eb; }
  else if (!strcmp(name, "lse")) { off = L.lse; len = (size_t)desc->batch * desc->heads * desc->seq * 4; }
  else if (!strcmp(name, "z1")) { off = L.z1; len = T * H * eb; }
  else if (!strcmp(name, "n1")) { off = L.n1; len = T * H * eb; }
  else if (!strcmp(name, "y1") && !desc->pre_ln) { off = L.y1; len = T * H * eb; }
  else if (!strcmp(name, "n2") && desc->pre_ln) { off = L.y1; len = T * H * eb; }
  else if (!strcmp(name, "dact") && !is_llama(desc) && keeps_dact(desc)) { off = L.u; len = T * F * eb; }
  else if (!strcmp(name, "dgate") && is_llama(desc)) { off = L.u; len = 2 * T * F * eb; }
  else if (!strcmp(name, "g")) { off = L.g; len = T * F * eb; }
  else if (!strcmp(name, "z2")) { off = L.z2; len = T * H * eb; }
  else if (!strcmp(name, "mu1")) { off = L.mu1; len = T * 4; }
  else if (!strcmp(name, "rstd1")) { off = L.rstd1; len = T * 4; }
  else if (!strcmp(name, "mu2")) { off = L.mu2; len = T * 4; }
  else if (!strcmp(name, "rstd2")) { off = L.rstd2; len = T * 4; }
  if (off == (size_t)-1) return SLAPO_ERR_UNSUPPORTED;
  *offset = off;
  *bytes = len;
  return SLAPO_OK;
}

// In a stack of pre-LN layers the LayerNorm that opens layer l+1 reads what the last kernel of layer l has
// just written, so that kernel produces it on the way: the pattern (sum out, its LayerNorm out) is the one
// the layer already uses between its attention and feed-forward blocks, and one pass over [T,H] per layer
// boundary goes away. The normalised values are computed from the stored (rounded) sum, exactly as the
// separate kernel would, so a layer run on its own reproduces them bit for bit.
struct ForwardLink {
  bool ln1_done = false;                       // the layer below has filled n1, mu1, rstd1 of `saved`
  const slapo_layer_params* above = nullptr;   // the layer above: its first LayerNorm rides on my last kernel
  void* above_saved = nullptr;                 // ... and lands in the n1, mu1, rstd1 regions of its `saved`
};

// The forward launch sequence; `saved` receives the activations. Also the first half of a checkpointed
// backward (`for_backward`), which is why it is a function of its own.
static void run_forward(const slapo_layer_desc* d, const slapo_layer_params* p, const void* x, const int32_t* seqlens,
                        void* y, void* saved, void* scratch, hipStream_t st, bool for_backward = false,
                        const ForwardLink* link = nullptr) {
  const int dt = d->dtype;   // SLAPO_* element types are the launch interface's DT_* values
  const int T = d->batch * d->seq, H = d->hidden, F = d->ffn, A = attn_width(d);
  const SavedLayout L = saved_layout(d);
  const ScratchLayout W = scratch_layout(d);
  char* sv = (char*)saved;
  char* sc = (char*)scratch;
  void *qkv = sv + L.qkv, *attn = sv + L.attn, *z1 = sv + L.z1, *y1 = sv + L.y1, *g = sv + L.g;
  void* u = keeps_dact(d) ? sv + L.u : nullptr;
  float *lse = (float*)(sv + L.lse), *mu1 = (float*)(sv + L.mu1), *rstd1 = (float*)(sv + L.rstd1);
  float *mu2 = (float*)(sv + L.mu2), *rstd2 = (float*)(sv + L.rstd2);
  void* r = sc + W.t0;
  const AttnShape as = make_attn_shape(d);
  const DropoutParams dp0 = make_dropout(d, 0), dp1 = make_dropout(d, 1);

  const bool llama = is_llama(d);
  const int rms = llama ? 1 : 0;
  const void* attn_in = x;
  if (d->pre_ln) {
    void* n1 = sv + L.n1;
    if (!(link && link->ln1_done))
      launch_bdrln_fwd(dt, T, H, nullptr, nullptr, x, p->ln1_g, p->ln1_b, nullptr, n1, mu1, rstd1, dp0, d->ln_eps, rms, st);
    attn_in = n1;
  }
  if (llama) {
    // no biases; queries and keys are rotated in place by their position before the attention reads them
    float* table = (float*)(sc + W.rope);
    launch_rope_table(d->seq, A / d->heads, d->rope_base, table, st);
    launch_gemm(dt, GEMM_NT, EPI_NONE, d->act, T, 3 * A, H, attn_in, p->wqkv, qkv, nullptr, nullptr, nullptr, st, true);
    launch_rope(dt, T, d->seq, A, A / d->heads, table, qkv, 0, st);
  } else {
    launch_gemm(dt, GEMM_NT, EPI_BIAS, d->act, T, 3 * A, H, attn_in, p->wqkv, qkv, p->bqkv, nullptr, nullptr, st, true);
  }
  launch_attn_fwd(dt, as, qkv, seqlens, attn, lse, st);
  float* gws = W.gemm_ws_bytes ? (float*)(sc + W.gemm_ws) : nullptr;   // for GEMMs whose tile grid ends in a thin round
  launch_gemm(dt, GEMM_NT, EPI_NONE, d->act, T, H, A, attn, p->wo, r, nullptr, nullptr, nullptr, st, true, gws, W.gemm_ws_bytes);
  const void* bo = llama ? nullptr : p->bo;
  const void* b2 = llama ? nullptr : p->b2;
  if (d->pre_ln) launch_bdrln_fwd(dt, T, H, r, bo, x, p->ln2_g, p->ln2_b, z1, y1, mu2, rstd2, dp0, d->ln_eps, rms, st);
  else launch_bdrln_fwd(dt, T, H, r, bo, x, p->ln1_g, p->ln1_b, z1, y1, mu1, rstd1, dp0, d->ln_eps, rms, st);
  if (llama)   // w1 holds (gate, up) row pairs: one product, gated in the epilogue; `u` keeps the backward factors
    launch_gemm(dt, GEMM_NT, EPI_GATE, d->act, T, 2 * F, H, y1, p->w1, g, nullptr, nullptr, u, st, true);
  else
    launch_gemm(dt, GEMM_NT, EPI_BIAS_ACT, d->act, T, F, H, y1, p->w1, g, p->b1, nullptr, u, st, true);
  // Backward of a pre-LN layer reads nothing downstream of the activation output (its last step has no
  // LayerNorm whose input would have to be kept), so a recomputation stops here: one GEMM in six less.
  if (for_backward && d->pre_ln) return;
  launch_gemm(dt, GEMM_NT, EPI_NONE, d->act, T, H, F, g, p->w2, r, nullptr, nullptr, nullptr, st, true, gws, W.gemm_ws_bytes);
  if (d->pre_ln && link && link->above) {
    char* up = (char*)link->above_saved;
    launch_bdrln_fwd(dt, T, H, r, b2, z1, link->above->ln1_g, llama ? nullptr : link->above->ln1_b, y, up + L.n1,
                     (float*)(up + L.mu1), (float*)(up + L.rstd1), dp1, d->ln_eps, rms, st);
  } else if (d->pre_ln) {
    launch_bdrln_fwd(dt, T, H, r, b2, z1, nullptr, nullptr, y, nullptr, nullptr, nullptr, dp1, d->ln_eps, rms, st);
  } else {
    void* z2 = sv + L.z2;
    launch_bdrln_fwd(dt, T, H, r, b2, y1, p->ln2_g, p->ln2_b, z2, y, mu2, rstd2, dp1, d->ln_eps, rms, st);
  }
}

static int check_forward_args(const slapo_layer_desc* d, const slapo_layer_params* p, const void* x, const void* y,
                              const void* saved, const void* scratch) {
  int rc = check_desc(d);
  if (rc) return rc;
  if (!p || !x || !y || !scratch || (!saved && !d->checkpoint)) return SLAPO_ERR_NULL;
  const void* const ps[12] = {p->wqkv, p->bqkv, p->wo, p->bo, p->ln1_g, p->ln1_b, p->w1, p->b1, p->w2, p->b2, p->ln2_g, p->ln2_b};
  if ((rc = check_tables(d, ps))) return rc;
  if (misaligned(x) || misaligned(y) || misaligned(scratch) || (!d->checkpoint && misaligned(saved))) return SLAPO_ERR_ALIGN;
  return SLAPO_OK;
}

int slapo_layer_fwd(const slapo_layer_desc* d, const slapo_layer_params* p, const void* x, const int32_t* seqlens,
                    void* y, void* saved, void* scratch, void* stream) {
  const int rc = check_forward_args(d, p, x, y, saved, scratch);
  if (rc) return rc;
  entry_error();
  if (d->checkpoint) saved = (char*)scratch + scratch_layout(d).acts;   // transient: nothing is kept for backward
  run_forward(d, p, x, seqlens, y, saved, scratch, (hipStream_t)stream);
  return finish();
}

static int check_backward_args(const slapo_layer_desc* d, const slapo_layer_params* p, const void* x, const void* dy,
                               const void* saved, const void* dx, const slapo_layer_grads* gr, const void* scratch) {
  int rc = check_desc(d);
  if (rc) return rc;
  if (!p || !x || !dy || !dx || !gr || !scratch || (!saved && !d->checkpoint)) return SLAPO_ERR_NULL;
  const void* const ps[12] = {p->wqkv, p->bqkv, p->wo, p->bo, p->ln1_g, p->ln1_b, p->w1, p->b1, p->w2, p->b2, p->ln2_g, p->ln2_b};
  const void* const gs[12] = {gr->wqkv, gr->bqkv, gr->wo, gr->bo, gr->ln1_g, gr->ln1_b, gr->w1, gr->b1, gr->w2, gr->b2, gr->ln2_g, gr->ln2_b};
  if ((rc = check_tables(d, ps)) || (rc = check_tables(d, gs))) return rc;
  if (misaligned(x) || misaligned(dy) || misaligned(dx) || misaligned(scratch) || (!d->checkpoint && misaligned(saved))) return SLAPO_ERR_ALIGN;
  return SLAPO_OK;
}

// The backward counterpart of ForwardLink: the last kernel of a pre-LN layer's backward (LayerNorm backward
// plus the residual gradient -> dx) is also where the layer below would start (dx -> its dropped-out branch
// gradient dR2 and the row sums behind its b2 gradient), so in a stack the upper layer's kernel writes both
// and the lower layer starts at its first GEMM.
struct BackwardLink {
  const void* dr2_in = nullptr;   // my dR2, already produced (with my b2 gradient) by the layer above
  void* dr2_below = nullptr;      // where the dR2 of the layer below goes ...
  DropoutParams dp_below;         // ... its mask stream (site 1 of that layer)
  void* db2_below = nullptr;      // ... and its b2 gradient (NULL: the family has no biases)
};

static int run_backward(const slapo_layer_desc* d, const slapo_layer_params* p, const void* x, const int32_t* seqlens,
                        const void* dy, const void* saved, void* dx, const slapo_layer_grads* gr, void* scratch,
                        hipStream_t st, const BackwardLink* link = nullptr) {
  const int dt = d->dtype, acc = d->accumulate_grads ? 1 : 0;
  const int T = d->batch * d->seq, H = d->hidden, F = d->ffn, A = attn_width(d);
  const SavedLayout L = saved_layout(d);
  const ScratchLayout W = scratch_layout(d);
  if (d->checkpoint) {
    // Activation checkpointing (section 2.2, the paper's third optimisation): nothing but x was kept, so run
    // the forward again into the transient region. The dropout masks are a pure function of (seed, layer,
    // site, element), so the recomputed activations are bit for bit those of the original forward. The layer
    // output lands in a gradient buffer that backward overwrites later.
    char* acts = (char*)scratch + W.acts;
    run_forward(d, p, x, seqlens, (char*)scratch + W.t1, acts, scratch, st, true);
    saved = acts;
  }
  const char* sv = (const char*)saved;
  char* sc = (char*)scratch;
  const void *qkv = sv + L.qkv, *attn = sv + L.attn, *z1 = sv + L.z1, *y1 = sv + L.y1, *g = sv + L.g;
  const void* u = keeps_dact(d) ? sv + L.u : g;   // ReLU: the gate [g > 0] comes from the activation output
  const float *lse = (const float*)(sv + L.lse), *mu1 = (const float*)(sv + L.mu1), *rstd1 = (const float*)(sv + L.rstd1);
  const float *mu2 = (const float*)(sv + L.mu2), *rstd2 = (const float*)(sv + L.rstd2);
  void *t0 = sc + W.t0, *t1 = sc + W.t1, *t2 = sc + W.t2, *t3 = sc + W.t3, *du = sc + W.du, *dqkv = sc + W.dqkv;
  float *delta = (float*)(sc + W.delta), *prow = (float*)(sc + W.part_row), *pcol = (float*)(sc + W.part_col), *pcol2 = (float*)(sc + W.part_col2);
  const AttnShape as = make_attn_shape(d);
  const DropoutParams dp0 = make_dropout(d, 0), dp1 = make_dropout(d, 1);
  const int nrow = bdrln_bwd_blocks(T), ncol = colsum_blocks(T);
  // `st` carries the data-gradient chain; `ws` the weight / bias gradients that hang off it
  SideStream* side = side_stream();
  const bool solo = side == nullptr;   // one stream: every GEMM has the chip to itself
  hipStream_t ws = side ? side->stream : st;
  auto fork = [&](int i) {   // everything issued on st so far happens before what follows on ws
    if (side) side->order(side->fork[i], st, ws);
  };
  // weight gradient: C (+)= A^T B
  float* splitk_ws = W.splitk_bytes ? (float*)(sc + W.splitk) : nullptr;
  float* gws = W.gemm_ws_bytes ? (float*)(sc + W.gemm_ws) : nullptr;
  const size_t gwb = W.gemm_ws_bytes;
  auto dweight = [&](int M, int N, const void* a, const void* b, void* c) {
    launch_weight_grad(dt, acc, M, N, T, a, b, c, splitk_ws, ws, solo);
  };
  auto colsum = [&](const void* a, int N, void* out, hipStream_t s) {
    float* part = s == st ? pcol2 : pcol;   // per stream, so that the two sums may run at the same time
    launch_colsum_partials(dt, T, N, a, part, s);
    launch_colreduce_partials(dt, ncol, N, N, part, out, acc, s);
  };
  auto reduce_rows = [&](void* dgamma, void* dbeta, void* dbias) {
    launch_colreduce3(dt, nrow, H, prow, dgamma, dbeta, dbias, acc, st);
  };
  // Buffers: t0 dZ2 -> dY1/dN2 -> dA -> dN1; t1 dR2 (kept for dW2); t2 dZ1; t3 dR1 (kept for dWo).

  const bool llama = is_llama(d);
  const int rms = llama ? 1 : 0;
  // the LLaMA-style layer has no bias or offset gradients: those outputs are simply not produced
  void *g_b2 = llama ? nullptr : gr->b2, *g_bo = llama ? nullptr : gr->bo;
  void *g_ln1_b = llama ? nullptr : gr->ln1_b, *g_ln2_b = llama ? nullptr : gr->ln2_b;

  // ---- FFN block ----
  const void* dr2 = t1;
  if (d->pre_ln && link && link->dr2_in) {
    dr2 = link->dr2_in;
  } else if (d->pre_ln) {
    launch_bdrln_bwd(dt, T, H, dy, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, t1, prow, dp1, rms, st);
    if (!llama) reduce_rows(nullptr, nullptr, g_b2);
  } else {
    launch_bdrln_bwd(dt, T, H, dy, sv + L.z2, mu2, rstd2, p->ln2_g, nullptr, t0, t1, prow, dp1, rms, st);
    reduce_rows(gr->ln2_g, g_ln2_b, g_b2);
  }
  fork(0);
  dweight(H, F, dr2, g, gr->w2);
  if (llama) {
    // dG = dR2 W2, turned into the (gate, up) gradient pairs [T,2F] by the two saved factors in the epilogue
    launch_gemm(dt, GEMM_NN, EPI_DGATE, d->act, T, F, H, dr2, p->w2, du, nullptr, u, nullptr, st, solo);
    fork(1);
    dweight(2 * F, H, du, y1, gr->w1);
    launch_gemm(dt, GEMM_NN, EPI_NONE, d->act, T, H, 2 * F, du, p->w1, t0, nullptr, nullptr, nullptr, st, solo, gws, gwb);
  } else {
    launch_gemm(dt, GEMM_NN, EPI_DACT, d->act, T, F, H, dr2, p->w2, du, nullptr, u, nullptr, st, solo);
    fork(1);
    colsum(du, F, gr->b1, ws);
    dweight(F, H, du, y1, gr->w1);
    if (d->pre_ln) launch_gemm(dt, GEMM_NN, EPI_NONE, d->act, T, H, F, du, p->w1, t0, nullptr, nullptr, nullptr, st, solo, gws, gwb);
    else launch_gemm(dt, GEMM_NN, EPI_ADD, d->act, T, H, F, du, p->w1, t0, nullptr, t0, nullptr, st, solo, gws, gwb);
  }
  // ---- attention block ----
  if (d->pre_ln) {
    launch_bdrln_bwd(dt, T, H, t0, z1, mu2, rstd2, p->ln2_g, dy, t2, t3, prow, dp0, rms, st);
    reduce_rows(gr->ln2_g, g_ln2_b, g_bo);
  } else {
    launch_bdrln_bwd(dt, T, H, t0, z1, mu1, rstd1, p->ln1_g, nullptr, t2, t3, prow, dp0, rms, st);
    reduce_rows(gr->ln1_g, g_ln1_b, g_bo);
  }
  fork(2);
  dweight(H, A, t3, attn, gr->wo);
  launch_gemm(dt, GEMM_NN, EPI_NONE, d->act, T, A, H, t3, p->wo, t0, nullptr, nullptr, nullptr, st, solo, gws, gwb);
  launch_attn_bwd(dt, as, qkv, seqlens, attn, t0, lse, delta, dqkv, st);
  if (llama) {
    // the attention gradients are w.r.t. the rotated queries and keys: turn them back (the rotation's transpose)
    float* table = (float*)(sc + W.rope);
    if (!d->checkpoint) launch_rope_table(d->seq, A / d->heads, d->rope_base, table, st);   // else the recomputed forward just wrote it
    launch_rope(dt, T, d->seq, A, A / d->heads, table, dqkv, 1, st);
  }
  fork(3);
  if (d->pre_ln) {
    dweight(3 * A, H, dqkv, sv + L.n1, gr->wqkv);
    launch_gemm(dt, GEMM_NN, EPI_NONE, d->act, T, H, 3 * A, dqkv, p->wqkv, t0, nullptr, nullptr, nullptr, st, solo, gws, gwb);
    if (link && link->dr2_below) {
      // (from the stored dx, so that the layer below sees what it would compute from dx itself, bit for bit)
      launch_bdrln_bwd(dt, T, H, t0, x, mu1, rstd1, p->ln1_g, t2, dx, link->dr2_below, prow, link->dp_below, rms, st, 1);
      reduce_rows(gr->ln1_g, g_ln1_b, link->db2_below);
    } else {
      launch_bdrln_bwd(dt, T, H, t0, x, mu1, rstd1, p->ln1_g, t2, dx, nullptr, prow, dp0, rms, st);
      reduce_rows(gr->ln1_g, g_ln1_b, nullptr);
    }
  } else {
    dweight(3 * A, H, dqkv, x, gr->wqkv);
    launch_gemm(dt, GEMM_NN, EPI_ADD, d->act, T, H, 3 * A, dqkv, p->wqkv, dx, nullptr, t2, nullptr, st, solo, gws, gwb);
  }
  // the last bias gradient goes behind the data gradient on the caller's stream: the helper stream's last
  // product is the longer one, and this way the two streams end at about the same time
  if (!llama) colsum(dqkv, 3 * A, gr->bqkv, st);
  if (side) side->order(side->join, ws, st);   // join: the caller's stream continues only after the weight gradients are complete
  return finish();
}

int slapo_layer_bwd(const slapo_layer_desc* d, const slapo_layer_params* p, const void* x, const int32_t* seqlens,
                    const void* dy, const void* saved, void* dx, const slapo_layer_grads* gr, void* scratch,
                    void* stream) {
  const int rc = check_backward_args(d, p, x, dy, saved, dx, gr, scratch);
  if (rc) return rc;
  entry_error();
  return run_backward(d, p, x, seqlens, dy, saved, dx, gr, scratch, (hipStream_t)stream);
}

// ---- a stack of layers of one shape ------------------------------------------------------------------
static size_t stack_act_bytes(const slapo_layer_desc* d) {
  return (size_t)d->batch * d->seq * d->hidden * (d->dtype == SLAPO_FP32 ? 4 : 2);
}

int slapo_stack_workspace(const slapo_layer_desc* desc, int32_t n_layers, size_t* acts_bytes, size_t* saved_bytes,
                          size_t* scratch_bytes) {
  if (!acts_bytes || !saved_bytes || !scratch_bytes) return SLAPO_ERR_NULL;
  const int rc = check_desc(desc);
  if (rc) return rc;
  if (n_layers <= 0) return SLAPO_ERR_SHAPE;
  *acts_bytes = (size_t)(n_layers - 1) * stack_act_bytes(desc);
  *saved_bytes = desc->checkpoint ? 0 : (size_t)n_layers * saved_layout(desc).total;
  // behind the layer's own scratch: two alternating buffers for the gradient that flows down the stack and,
  // for pre-LN layers, two for the branch gradient that each layer's last kernel prepares for the layer below
  *scratch_bytes = scratch_layout(desc).total + (desc->pre_ln ? 4 : 2) * align256(stack_act_bytes(desc));
  return SLAPO_OK;
}

int slapo_stack_fwd(const slapo_layer_desc* desc, int32_t n_layers, const slapo_layer_params* params, const void* x,
                    const int32_t* seqlens, void* y, void* acts, void* saved, void* scratch, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (n_layers <= 0) return SLAPO_ERR_SHAPE;
  if (!params || !x || !y || !scratch || (n_layers > 1 && !acts) || (!saved && !desc->checkpoint)) return SLAPO_ERR_NULL;
  const size_t ab = stack_act_bytes(desc), sb = desc->checkpoint ? 0 : saved_layout(desc).total;
  slapo_layer_desc d = *desc;
  // every layer is checked before the first launch, so that a bad table leaves nothing half done
  for (int l = 0; l < n_layers; ++l) {
    const void* in = l == 0 ? x : (const char*)acts + (size_t)(l - 1) * ab;
    void* out = l == n_layers - 1 ? y : (char*)acts + (size_t)l * ab;
    if ((rc = check_forward_args(&d, params + l, in, out, saved, scratch))) return rc;
  }
  entry_error();
  // with checkpointing every layer works in the same transient region, whose contents die with the layer
  char* transient = (char*)scratch + scratch_layout(desc).acts;
  auto saved_of = [&](int l) -> void* { return desc->checkpoint ? transient : (char*)saved + (size_t)l * sb; };
  for (int l = 0; l < n_layers; ++l) {
    d.layer_id = desc->layer_id + l;
    const void* in = l == 0 ? x : (const char*)acts + (size_t)(l - 1) * ab;
    void* out = l == n_layers - 1 ? y : (char*)acts + (size_t)l * ab;
    ForwardLink link;
    if (d.pre_ln) {   // the first LayerNorm of layer l+1 rides on the last kernel of layer l
      link.ln1_done = l > 0;
      if (l + 1 < n_layers) { link.above = params + l + 1; link.above_saved = saved_of(l + 1); }
    }
    run_forward(&d, params + l, in, seqlens, out, saved_of(l), scratch, (hipStream_t)stream, false, &link);
  }
  return finish();
}

int slapo_stack_bwd(const slapo_layer_desc* desc, int32_t n_layers, const slapo_layer_params* params, const void* x,
                    const int32_t* seqlens, const void* dy, const void* acts, const void* saved, void* dx,
                    const slapo_layer_grads* grads, void* scratch, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (n_layers <= 0) return SLAPO_ERR_SHAPE;
  if (!params || !grads || !x || !dy || !dx || !scratch || (n_layers > 1 && !acts) || (!saved && !desc->checkpoint))
    return SLAPO_ERR_NULL;
  const size_t ab = stack_act_bytes(desc), sb = desc->checkpoint ? 0 : saved_layout(desc).total;
  char* pong = (char*)scratch + scratch_layout(desc).total;   // two gradient buffers behind the layer's own scratch
  char* carry = pong + 2 * align256(ab);                      // (pre-LN) two branch-gradient buffers behind those
  slapo_layer_desc d = *desc;
  for (int l = 0; l < n_layers; ++l) {   // every layer is checked before the first launch
    const void* in = l == 0 ? x : (const char*)acts + (size_t)(l - 1) * ab;
    if ((rc = check_backward_args(&d, params + l, in, dy, saved, dx, grads + l, scratch))) return rc;
  }
  entry_error();
  const void* gin = dy;
  for (int l = n_layers - 1; l >= 0; --l) {
    d.layer_id = desc->layer_id + l;
    const void* in = l == 0 ? x : (const char*)acts + (size_t)(l - 1) * ab;
    void* gout = l == 0 ? dx : pong + (size_t)(l & 1) * align256(ab);
    BackwardLink link;
    if (d.pre_ln) {
      // Layer l reads buffer l&1 (on both streams) and writes the other one; that one was last read by the
      // weight gradient of layer l+1, which the join at the end of that layer's backward has waited for.
      if (l + 1 < n_layers) link.dr2_in = carry + (size_t)(l & 1) * align256(ab);
      if (l > 0) {
        slapo_layer_desc below = d;
        below.layer_id = d.layer_id - 1;
        link.dr2_below = carry + (size_t)((l - 1) & 1) * align256(ab);
        link.dp_below = make_dropout(&below, 1);
        link.db2_below = is_llama(desc) ? nullptr : grads[l - 1].b2;
      }
    }
    rc = run_backward(&d, params + l, in, seqlens, gin, saved ? (const char*)saved + (size_t)l * sb : nullptr, gout,
                      grads + l, scratch, (hipStream_t)stream, &link);
    if (rc) return rc;
    gin = gout;
  }
  return SLAPO_OK;
}

static int gemm_entry(int dtype, int layout, int epilogue, int act, int64_t M, int64_t N, int64_t K, const void* A,
                      const void* B, void* C, const void* bias, const void* aux_in, void* aux_out, void* stream, bool solo,
                      void* ws, size_t ws_bytes) {
  if (dtype != SLAPO_BF16 && dtype != SLAPO_FP32 && dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (layout < GEMM_NT || layout > GEMM_TN || epilogue < EPI_NONE || epilogue > EPI_DGATE) return SLAPO_ERR_UNSUPPORTED;
  if (act != SLAPO_GELU_ERF && act != SLAPO_RELU) return SLAPO_ERR_UNSUPPORTED;
  if (M <= 0 || N <= 0 || K <= 0) return SLAPO_ERR_SHAPE;
  if (M * N >= ((int64_t)1 << 31) || M * K >= ((int64_t)1 << 31) || N * K >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  if (!A || !B || !C) return SLAPO_ERR_NULL;
  if ((epilogue == EPI_BIAS || epilogue == EPI_BIAS_ACT) && !bias) return SLAPO_ERR_NULL;
  if (((epilogue == EPI_BIAS_ACT && act != SLAPO_RELU) || epilogue == EPI_GATE) && !aux_out) return SLAPO_ERR_NULL;
  if ((epilogue == EPI_DACT || epilogue == EPI_ADD || epilogue == EPI_DGATE) && !aux_in) return SLAPO_ERR_NULL;
  if (epilogue == EPI_DGATE && 2 * M * N >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  if (N % 8 || (epilogue == EPI_GATE && N % 16)) return SLAPO_ERR_ALIGN;
  if (layout == GEMM_TN ? (M % 8) : (K % 8)) return SLAPO_ERR_ALIGN;   // A's contiguous dimension
  if (layout == GEMM_NT && (K % 8)) return SLAPO_ERR_ALIGN;
  if (misaligned(A) || misaligned(B) || misaligned(C) || misaligned(ws)) return SLAPO_ERR_ALIGN;
  // a workspace is all or nothing: one that is too small for what the shape can use is refused, not half used
  if (ws && ws_bytes < gemm_ws_bytes(dtype, epilogue, (int)M, (int)N, (int)K)) return SLAPO_ERR_WORKSPACE;
  entry_error();
  launch_gemm(dtype, layout, epilogue, act, (int)M, (int)N, (int)K, A, B, C, bias, aux_in, aux_out,
              (hipStream_t)stream, solo, (float*)ws, ws ? ws_bytes : 0);
  return finish();
}

int slapo_gemm(int dtype, int layout, int epilogue, int act, int64_t M, int64_t N, int64_t K, const void* A,
               const void* B, void* C, const void* bias, const void* aux_in, void* aux_out, void* stream) {
  return gemm_entry(dtype, layout, epilogue, act, M, N, K, A, B, C, bias, aux_in, aux_out, stream, true, nullptr, 0);
}

int slapo_gemm_workspace(int dtype, int layout, int epilogue, int64_t M, int64_t N, int64_t K, size_t* ws_bytes) {
  if (!ws_bytes) return SLAPO_ERR_NULL;
  if (dtype != SLAPO_BF16 && dtype != SLAPO_FP32 && dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (layout < GEMM_NT || layout > GEMM_TN || epilogue < EPI_NONE || epilogue > EPI_DGATE) return SLAPO_ERR_UNSUPPORTED;
  if (M <= 0 || N <= 0 || K <= 0) return SLAPO_ERR_SHAPE;
  if (M * N >= ((int64_t)1 << 31) || M * K >= ((int64_t)1 << 31) || N * K >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  *ws_bytes = gemm_ws_bytes(dtype, epilogue, (int)M, (int)N, (int)K);
  return SLAPO_OK;
}

int slapo_gemm_ex(int dtype, int layout, int epilogue, int act, int64_t M, int64_t N, int64_t K, const void* A,
                  const void* B, void* C, const void* bias, const void* aux_in, void* aux_out, int flags, void* ws,
                  size_t ws_bytes, void* stream) {
  if (flags & ~SLAPO_GEMM_SHARED) return SLAPO_ERR_UNSUPPORTED;
  return gemm_entry(dtype, layout, epilogue, act, M, N, K, A, B, C, bias, aux_in, aux_out, stream,
                    !(flags & SLAPO_GEMM_SHARED), ws, ws_bytes);
}

int slapo_gemm_kernel_name(int dtype, int layout, int epilogue, int64_t M, int64_t N, int64_t K, int flags,
                           int weight_grad, int with_ws, char* buf, size_t len) {
  if (!buf || len == 0) return SLAPO_ERR_NULL;
  if (dtype != SLAPO_BF16 && dtype != SLAPO_FP32 && dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (layout < GEMM_NT || layout > GEMM_TN || epilogue < EPI_NONE || epilogue > EPI_DGATE) return SLAPO_ERR_UNSUPPORTED;
  if (flags & ~SLAPO_GEMM_SHARED) return SLAPO_ERR_UNSUPPORTED;
  if (M <= 0 || N <= 0 || K <= 0 || M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31) || K >= ((int64_t)1 << 31)) return SLAPO_ERR_SHAPE;
  if (weight_grad && layout != GEMM_TN) return SLAPO_ERR_UNSUPPORTED;
  describe_gemm(dtype, layout, epilogue, (int)M, (int)N, (int)K, !(flags & SLAPO_GEMM_SHARED), weight_grad != 0, with_ws != 0, buf, len);
  return SLAPO_OK;
}

static int check_weight_grad_shape(int dtype, int64_t M, int64_t N, int64_t K) {
  if (dtype != SLAPO_BF16 && dtype != SLAPO_FP32 && dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (M <= 0 || N <= 0 || K <= 0) return SLAPO_ERR_SHAPE;
  if (M * N >= ((int64_t)1 << 31) || M * K >= ((int64_t)1 << 31) || N * K >= ((int64_t)1 << 31)) return SLAPO_ERR_UNSUPPORTED;
  if (M % 8 || N % 8) return SLAPO_ERR_ALIGN;
  return SLAPO_OK;
}

int slapo_weight_grad_workspace(int dtype, int64_t M, int64_t N, int64_t K, size_t* ws_bytes) {
  if (!ws_bytes) return SLAPO_ERR_NULL;
  const int rc = check_weight_grad_shape(dtype, M, N, K);
  if (rc) return rc;
  *ws_bytes = weight_grad_ws_bytes(dtype, (int)M, (int)N, (int)K);
  return SLAPO_OK;
}

int slapo_weight_grad(int dtype, int accumulate, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
                      void* ws, void* stream) {
  const int rc = check_weight_grad_shape(dtype, M, N, K);
  if (rc) return rc;
  if (!A || !B || !C) return SLAPO_ERR_NULL;
  if (!ws && weight_grad_ws_bytes(dtype, (int)M, (int)N, (int)K)) return SLAPO_ERR_NULL;
  if (misaligned(A) || misaligned(B) || misaligned(C) || misaligned(ws)) return SLAPO_ERR_ALIGN;
  entry_error();
  launch_weight_grad(dtype, accumulate ? 1 : 0, (int)M, (int)N, (int)K, A, B, C, (float*)ws, (hipStream_t)stream);
  return finish();
}

// ---- the weight gradient for callers that cannot allocate ---------------------------------------------
// Same computation as slapo_weight_grad, with the fp32 partial tiles of the K-range path in a fixed array in
// device memory that belongs to the library instead of a caller-provided workspace. The array's name is only a
// host-side handle: its device address is looked up once per device (with that device current) and kept, and
// that pointer is what the kernels are given.
}  // extern "C"

namespace {
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[STATIC_SCRATCH_BYTES];

// device address of this device's copy of g_static_scratch, or nullptr (with *status set) if it cannot be had
float* static_scratch(int* status) {
  static void* table[16] = {};
  static std::mutex mu;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { *status = SLAPO_ERR_HIP; return nullptr; }
  if (dev < 0 || dev >= 16) { *status = SLAPO_ERR_UNSUPPORTED; return nullptr; }
  std::lock_guard<std::mutex> lock(mu);
  if (!table[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      *status = SLAPO_ERR_HIP;
      return nullptr;
    }
    table[dev] = ptr;
  }
  return (float*)table[dev];
}
}  // namespace

extern "C" {

int slapo_weight_grad_static(int dtype, int accumulate, int64_t M, int64_t N, int64_t K, const void* A, const void* B,
                             void* C, void* stream) {
  const int rc = check_weight_grad_shape(dtype, M, N, K);
  if (rc) return rc;
  if (!A || !B || !C) return SLAPO_ERR_NULL;
  if (misaligned(A) || misaligned(B) || misaligned(C)) return SLAPO_ERR_ALIGN;
  const size_t need = weight_grad_ws_bytes(dtype, (int)M, (int)N, (int)K);
  if (need > STATIC_SCRATCH_BYTES) return SLAPO_ERR_WORKSPACE;
  float* ws = nullptr;
  if (need) {   // shapes that run as one plain GEMM touch no scratch at all
    int st = SLAPO_OK;
    ws = static_scratch(&st);
    if (!ws) return st;
  }
  entry_error();
  launch_weight_grad(dtype, accumulate ? 1 : 0, (int)M, (int)N, (int)K, A, B, C, ws, (hipStream_t)stream);
  return finish();
}

int slapo_attn_fwd(const slapo_layer_desc* d, const void* qkv, const int32_t* seqlens, void* out, float* lse,
                   void* stream) {
  const int rc = check_desc(d);
  if (rc) return rc;
  if (!qkv || !out || !lse) return SLAPO_ERR_NULL;
  if (misaligned(qkv) || misaligned(out)) return SLAPO_ERR_ALIGN;
  const AttnShape as = make_attn_shape(d);
  entry_error();
  launch_attn_fwd(d->dtype, as, qkv, seqlens, out, lse, (hipStream_t)stream);
  return finish();
}

int slapo_attn_bwd(const slapo_layer_desc* d, const void* qkv, const int32_t* seqlens, const void* out,
                   const void* dout, const float* lse, float* delta, void* dqkv, void* stream) {
  const int rc = check_desc(d);
  if (rc) return rc;
  if (!qkv || !out || !dout || !lse || !delta || !dqkv) return SLAPO_ERR_NULL;
  if (misaligned(qkv) || misaligned(out) || misaligned(dout) || misaligned(dqkv)) return SLAPO_ERR_ALIGN;
  const AttnShape as = make_attn_shape(d);
  entry_error();
  launch_attn_bwd(d->dtype, as, qkv, seqlens, out, dout, lse, delta, dqkv, (hipStream_t)stream);
  return finish();
}

int slapo_bdrln_fwd(const slapo_layer_desc* d, int site, int64_t T, const void* r, const void* bias, const void* res,
                    const void* gamma, const void* beta, void* z_out, void* out, float* mu, float* rstd,
                    void* stream) {
  const int rc = check_desc(d);
  if (rc) return rc;
  if (T <= 0 || site < 0 || site > 1) return SLAPO_ERR_SHAPE;
  const bool llama = is_llama(d);   // RMSNorm: no offset, no mean; no biases
  if (!res) return SLAPO_ERR_NULL;
  if (r && ((!bias && !llama) || !z_out)) return SLAPO_ERR_NULL;
  if (gamma && (!out || !rstd || (!llama && (!beta || !mu)))) return SLAPO_ERR_NULL;
  if (!r && !gamma) return SLAPO_ERR_NULL;
  if (misaligned(r) || misaligned(bias) || misaligned(res) || misaligned(gamma) || misaligned(beta) ||
      misaligned(z_out) || misaligned(out)) return SLAPO_ERR_ALIGN;
  entry_error();
  launch_bdrln_fwd(d->dtype, T, d->hidden, r, bias, res, gamma, beta, z_out, out, mu, rstd,
                   make_dropout(d, site), d->ln_eps, llama ? 1 : 0, (hipStream_t)stream);
  return finish();
}

int slapo_bdrln_bwd_blocks(int64_t T) { return bdrln_bwd_blocks(T); }

int slapo_bdrln_bwd(const slapo_layer_desc* d, int site, int64_t T, const void* dout, const void* z, const float* mu,
                    const float* rstd, const void* gamma, const void* dres_in, void* dz_out, void* dr_out,
                    float* partials, void* stream) {
  const int rc = check_desc(d);
  if (rc) return rc;
  if (T <= 0 || site < 0 || site > 1) return SLAPO_ERR_SHAPE;
  if (!dout || !partials) return SLAPO_ERR_NULL;
  if (gamma && (!z || !rstd || (!mu && !is_llama(d)))) return SLAPO_ERR_NULL;
  if (!dz_out && !dr_out) return SLAPO_ERR_NULL;
  if (misaligned(dout) || misaligned(z) || misaligned(gamma) || misaligned(dres_in) || misaligned(dz_out) ||
      misaligned(dr_out) || misaligned(partials)) return SLAPO_ERR_ALIGN;
  entry_error();
  launch_bdrln_bwd(d->dtype, T, d->hidden, dout, z, mu, rstd, gamma, dres_in, dz_out, dr_out, partials,
                   make_dropout(d, site), is_llama(d) ? 1 : 0, (hipStream_t)stream);
  return finish();
}

int slapo_rope(const slapo_layer_desc* d, void* qkv, float* table, int inverse, void* stream) {
  const int rc = check_desc(d);
  if (rc) return rc;
  if (!is_llama(d)) return SLAPO_ERR_UNSUPPORTED;
  if (!qkv || !table) return SLAPO_ERR_NULL;
  if (misaligned(qkv) || misaligned(table)) return SLAPO_ERR_ALIGN;
  const int hd = attn_width(d) / d->heads;
  entry_error();
  launch_rope_table(d->seq, hd, d->rope_base, table, (hipStream_t)stream);
  launch_rope(d->dtype, (int64_t)d->batch * d->seq, d->seq, attn_width(d), hd, table, qkv, inverse ? 1 : 0, (hipStream_t)stream);
  return finish();
}

int slapo_colsum_blocks(int64_t T) { return colsum_blocks(T); }

int slapo_colsum_partials(int dtype, int64_t T, int64_t N, const void* a, float* partials, void* stream) {
  if (dtype != SLAPO_BF16 && dtype != SLAPO_FP32 && dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (T <= 0 || N <= 0) return SLAPO_ERR_SHAPE;
  if (!a || !partials) return SLAPO_ERR_NULL;
  if (N % 8 || misaligned(a) || misaligned(partials)) return SLAPO_ERR_ALIGN;
  entry_error();
  launch_colsum_partials(dtype, T, N, a, partials, (hipStream_t)stream);
  return finish();
}

int slapo_colreduce_partials(int dtype, int64_t nblk, int64_t stride, int64_t N, const float* partials, void* out,
                             int accumulate, void* stream) {
  if (dtype != SLAPO_BF16 && dtype != SLAPO_FP32 && dtype != SLAPO_FP16) return SLAPO_ERR_UNSUPPORTED;
  if (nblk <= 0 || N <= 0 || stride < N) return SLAPO_ERR_SHAPE;
  if (!partials || !out) return SLAPO_ERR_NULL;
  entry_error();
  launch_colreduce_partials(dtype, nblk, stride, N, partials, out, accumulate, (hipStream_t)stream);
  return finish();
}

int slapo_dropout_mask(const slapo_layer_desc* d, int site, int64_t T, uint8_t* mask, void* stream) {
  const int rc = check_desc(d);
  if (rc) return rc;
  if (T <= 0 || site < 0 || site > 1) return SLAPO_ERR_SHAPE;
  if (!mask) return SLAPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(mask) & 7u) != 0) return SLAPO_ERR_ALIGN;
  entry_error();
  launch_dropout_mask(T * d->hidden, mask, make_dropout(d, site), (hipStream_t)stream);
  return finish();
}

}  // extern "C"
