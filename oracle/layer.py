"""fp64 definition of one transformer layer's training step (forward and hand-derived backward).

TEST INFRASTRUCTURE ONLY: the plain, unfused definition the HIP path is compared with. The full
S x S attention matrix is materialised, nothing is blocked or fused, every value is IEEE double.

What is computed follows the paper's description of the scheduled layer: one linear producing the
concatenated Q, K, V (section 2.2, step 1), softmax(Q K^T / sqrt(d)) V attention (section 2.2, step 2),
the output projection whose bias is moved into the following fused pattern, F.gelu(bias + x) in the
feed-forward block and LayerNorm(dropout(bias + x) + residual) after both blocks (appendix schedule).
The paper gives no equations; each op is the textbook one. Readings taken where the paper is silent:
score scale 1/sqrt(head dim); dropout on the attention probabilities (the dropout(softmax(attn), p) of
the listing in section 2.2 step 2) only when cfg.attn_dropout_p > 0, with its own mask stream (site 2, element
index ((b*heads + a)*S + i)*S + j); exact erf GeLU; biased
variance and eps inside the square root for LayerNorm; key-padding mask hides keys j >= len_b from
every query row; [Wq; Wk; Wv] stacked on the output dimension; pre-LN layers normalise the block
inputs and have no LayerNorm after the second residual. The attention width heads * d may differ from the
hidden size (cfg.attn_width): that is what one rank holds when the query/key/value and output projections are
sharded along the heads (section 2.2 step 3); the packed projection is then [T, 3*width] and wo is [H, width].

Tensors: x [B,S,H]; weights in [out, in] layout (Fig. 3 caption). Backward is derived by hand from
these definitions and pinned by finite differences in the tests.
"""
import numpy as np
from scipy.special import erf

from . import philox

GELU, RELU = 0, 1


def _act(u, kind):
    if kind == GELU:
        return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))
    return np.where(u > 0.0, u, 0.0)


def _act_grad(u, kind):
    if kind == GELU:
        cdf = 0.5 * (1.0 + erf(u / np.sqrt(2.0)))
        pdf = np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)
        return cdf + u * pdf
    return (u > 0.0).astype(np.float64)


def layer_norm(z, g, b, eps):
    mu = z.mean(axis=-1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mu) * rstd
    return xhat * g + b, mu[..., 0], rstd[..., 0]


def layer_norm_bwd(dy, z, mu, rstd, g):
    """Returns (dz, dgamma, dbeta) for y = (z-mu)*rstd*g + b over the last axis; z is [T,H]."""
    xhat = (z - mu[:, None]) * rstd[:, None]
    gg = dy * g
    dz = rstd[:, None] * (gg - gg.mean(axis=-1, keepdims=True) - xhat * (gg * xhat).mean(axis=-1, keepdims=True))
    return dz, (dy * xhat).sum(axis=0), dy.sum(axis=0)


def score_mask(cfg, seqlens, b):
    """Boolean [S,S] matrix, True where query i may attend key j in sample b."""
    S = cfg.seq
    ok = np.ones((S, S), dtype=bool)
    if cfg.causal:
        ok &= np.tril(np.ones((S, S), dtype=bool))
    if seqlens is not None:
        ok &= (np.arange(S) < int(seqlens[b]))[None, :]
    return ok


def attention_keep(cfg):
    """[B,h,S,S] array of 0/1 keep decisions for the attention probabilities (dropout site 2), or None."""
    if not cfg.attn_dropout_p > 0:
        return None
    B, S, h = cfg.batch, cfg.seq, cfg.heads
    return philox.keep_mask(B * h * S * S, cfg.attn_dropout_p, cfg.seed, 2, cfg.layer_id).reshape(B, h, S, S).astype(np.float64)


def attention_fwd(cfg, qkv, seqlens):
    """qkv [T,3H] -> (A [T,H], P [B,h,S,S], LSE [B,h,S]). P is the softmax before dropout; A uses the dropped P."""
    B, S, H, h = cfg.batch, cfg.seq, cfg.attn_width, cfg.heads   # H: width of each of Q, K, V
    d = H // h
    keep = attention_keep(cfg)
    A = np.zeros((B * S, H))
    P = np.zeros((B, h, S, S))
    LSE = np.zeros((B, h, S))
    for b in range(B):
        ok = score_mask(cfg, seqlens, b)
        rows = slice(b * S, (b + 1) * S)
        for a in range(h):
            q = qkv[rows, a * d:(a + 1) * d]
            k = qkv[rows, H + a * d:H + (a + 1) * d]
            v = qkv[rows, 2 * H + a * d:2 * H + (a + 1) * d]
            sc = (q @ k.T) / np.sqrt(d)
            sc = np.where(ok, sc, -np.inf)
            m = sc.max(axis=-1, keepdims=True)
            ex = np.exp(sc - m)
            den = ex.sum(axis=-1, keepdims=True)
            p = ex / den
            P[b, a] = p
            LSE[b, a] = (m + np.log(den))[:, 0]
            if keep is not None:
                p = p * keep[b, a] / (1.0 - cfg.attn_dropout_p)
            A[rows, a * d:(a + 1) * d] = p @ v
    return A, P, LSE


def attention_bwd(cfg, qkv, P, dA):
    """Gradient of attention_fwd's A w.r.t. the packed qkv."""
    B, S, H, h = cfg.batch, cfg.seq, cfg.attn_width, cfg.heads   # H: width of each of Q, K, V
    d = H // h
    dqkv = np.zeros_like(qkv)
    keep = attention_keep(cfg)
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for a in range(h):
            q = qkv[rows, a * d:(a + 1) * d]
            k = qkv[rows, H + a * d:H + (a + 1) * d]
            v = qkv[rows, 2 * H + a * d:2 * H + (a + 1) * d]
            p = P[b, a]
            da = dA[rows, a * d:(a + 1) * d]
            if keep is None:
                dv = p.T @ da
                dp = da @ v.T
            else:                               # A = (P * keep / (1 - pd)) V
                w = keep[b, a] / (1.0 - cfg.attn_dropout_p)
                dv = (p * w).T @ da
                dp = (da @ v.T) * w
            dsc = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
            dqkv[rows, a * d:(a + 1) * d] = (dsc @ k) / np.sqrt(d)
            dqkv[rows, H + a * d:H + (a + 1) * d] = (dsc.T @ q) / np.sqrt(d)
            dqkv[rows, 2 * H + a * d:2 * H + (a + 1) * d] = dv
    return dqkv


def dropout_keep(cfg, site):
    """[T,H] array of 0/1 keep decisions of dropout site 0 (after attention) or 1 (after the FFN)."""
    T, H = cfg.batch * cfg.seq, cfg.hidden
    return philox.keep_mask(T * H, cfg.dropout_p, cfg.seed, site, cfg.layer_id).reshape(T, H).astype(np.float64)


def layer_forward(cfg, params, x, seqlens=None):
    """Forward of one layer. Returns a dict with the output ``y`` [B,S,H] and every intermediate."""
    p = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    T, H = cfg.batch * cfg.seq, cfg.hidden
    X = np.asarray(x, dtype=np.float64).reshape(T, H)
    scale = 1.0 / (1.0 - cfg.dropout_p)
    c = {"X": X}
    c["M1"], c["M2"] = dropout_keep(cfg, 0), dropout_keep(cfg, 1)
    if cfg.pre_ln:
        c["N1"], c["mu1"], c["rstd1"] = layer_norm(X, p["ln1_g"], p["ln1_b"], cfg.ln_eps)
        attn_in = c["N1"]
    else:
        attn_in = X
    c["QKV"] = attn_in @ p["wqkv"].T + p["bqkv"]
    c["A"], c["P"], c["LSE"] = attention_fwd(cfg, c["QKV"], seqlens)
    c["R1"] = c["A"] @ p["wo"].T
    c["Z1"] = X + c["M1"] * (c["R1"] + p["bo"]) * scale
    if cfg.pre_ln:
        c["N2"], c["mu2"], c["rstd2"] = layer_norm(c["Z1"], p["ln2_g"], p["ln2_b"], cfg.ln_eps)
        ffn_in = c["N2"]
    else:
        c["Y1"], c["mu1"], c["rstd1"] = layer_norm(c["Z1"], p["ln1_g"], p["ln1_b"], cfg.ln_eps)
        ffn_in = c["Y1"]
    c["U"] = ffn_in @ p["w1"].T + p["b1"]
    c["G"] = _act(c["U"], cfg.act)
    c["R2"] = c["G"] @ p["w2"].T
    if cfg.pre_ln:
        Y = c["Z1"] + c["M2"] * (c["R2"] + p["b2"]) * scale
    else:
        c["Z2"] = ffn_in + c["M2"] * (c["R2"] + p["b2"]) * scale
        Y, c["mu2"], c["rstd2"] = layer_norm(c["Z2"], p["ln2_g"], p["ln2_b"], cfg.ln_eps)
    c["y"] = Y.reshape(cfg.batch, cfg.seq, H)
    return c


def layer_backward(cfg, params, c, dy):
    """Backward of one layer given the forward dict ``c`` and dL/dy. Returns {'dx', 'wqkv', 'bqkv', ...}."""
    p = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    T, H = cfg.batch * cfg.seq, cfg.hidden
    dY = np.asarray(dy, dtype=np.float64).reshape(T, H)
    scale = 1.0 / (1.0 - cfg.dropout_p)
    g = {}
    if cfg.pre_ln:
        dZ1 = dY.copy()                       # residual branch of y = Z1 + drop(R2 + b2)
        dR2 = dY * c["M2"] * scale
        ffn_in = c["N2"]
    else:
        dZ2, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dY, c["Z2"], c["mu2"], c["rstd2"], p["ln2_g"])
        dffn_in = dZ2.copy()                  # residual branch of Z2 = Y1 + drop(R2 + b2)
        dR2 = dZ2 * c["M2"] * scale
        ffn_in = c["Y1"]
    g["b2"] = dR2.sum(axis=0)
    g["w2"] = dR2.T @ c["G"]
    dU = (dR2 @ p["w2"]) * _act_grad(c["U"], cfg.act)
    g["b1"] = dU.sum(axis=0)
    g["w1"] = dU.T @ ffn_in
    if cfg.pre_ln:
        dN2 = dU @ p["w1"]
        d, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dN2, c["Z1"], c["mu2"], c["rstd2"], p["ln2_g"])
        dZ1 = dZ1 + d
        attn_in = c["N1"]
    else:
        dffn_in = dffn_in + dU @ p["w1"]
        dZ1, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(dffn_in, c["Z1"], c["mu1"], c["rstd1"], p["ln1_g"])
        attn_in = c["X"]
    dX = dZ1.copy()                           # residual branch of Z1 = X + drop(R1 + bo)
    dR1 = dZ1 * c["M1"] * scale
    g["bo"] = dR1.sum(axis=0)
    g["wo"] = dR1.T @ c["A"]
    dA = dR1 @ p["wo"]
    dQKV = attention_bwd(cfg, c["QKV"], c["P"], dA)
    g["bqkv"] = dQKV.sum(axis=0)
    g["wqkv"] = dQKV.T @ attn_in
    dattn_in = dQKV @ p["wqkv"]
    if cfg.pre_ln:
        d, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(dattn_in, c["X"], c["mu1"], c["rstd1"], p["ln1_g"])
        dX = dX + d
    else:
        dX = dX + dattn_in
    g["dx"] = dX.reshape(cfg.batch, cfg.seq, H)
    g["_dQKV"], g["_dA"], g["_dU"], g["_dR1"], g["_dR2"] = dQKV, dA, dU, dR1, dR2
    return g


def max_rel_err(got, ref):
    """Per-tensor error metric: max |got - ref| / max |ref|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    num = np.abs(got - ref).max() if ref.size else 0.0
    return float(num / den) if den > 0 else float(num)
