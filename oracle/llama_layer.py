"""fp64 definition of the training step of a LLaMA-style decoder layer (forward and hand-derived backward).

TEST INFRASTRUCTURE ONLY: the plain, unfused definition the HIP path's second layer family is compared
with; nothing is blocked or fused, every value is IEEE double.

The paper evaluates its schedules on LLaMA-7B beside the GPT/BERT families (section 5.2) without restating
that model; the layer is the one of the LLaMA report (Touvron et al. 2023, section 2.1), whose three changes
to the classic pre-norm decoder layer are taken from the publications it cites:
  * RMSNorm in front of both blocks (Zhang & Sennrich 2019, eq. 4): y = z / sqrt(mean(z^2) + eps) * g,
    no mean subtraction, no offset;
  * rotary position embedding on queries and keys (Su et al. 2021, eq. 34): inside every head the adjacent
    pair (2j, 2j+1) of the vector at position m is rotated by the angle m * base^(-2j/d);
  * SwiGLU feed-forward (Shazeer 2020, eq. 6): (silu(n W_gate^T) * (n W_up^T)) W_down^T, silu(u) = u * sigmoid(u);
and no linear layer has a bias. Attention itself (causal softmax(Q K^T / sqrt(d)) V) and the dropout sites on
the two residual branches are the classic layer's and are taken from there.

Readings: eps sits inside the square root; the pair convention is the adjacent one of the equation (the
split-half convention some libraries use differs by a fixed permutation of the weight rows); positions count
from 0 inside each sequence; gate and up projections are stored as ONE matrix w1 [2F, H] whose row 2c is
gate row c and row 2c+1 is up row c (so that one product yields both and a (gate, up) pair sits in adjacent
columns); dropout (off in the LLaMA workload) keeps the classic layer's two sites and mask streams.

Parameters: wqkv [3W,H], wo [H,W], ln1_g [H], w1 [2F,H], w2 [H,F], ln2_g [H], with W = heads * d the attention
width (= H unless the projections are sharded along the heads, cfg.attn_width).
"""
import numpy as np

from .layer import attention_bwd, attention_fwd, dropout_keep


def rms_norm(z, g, eps):
    """Returns (z * r * g, r) with r = 1/sqrt(mean(z^2) + eps) over the last axis; r is [T]."""
    r = 1.0 / np.sqrt((z * z).mean(axis=-1, keepdims=True) + eps)
    return z * r * g, r[..., 0]


def rms_norm_bwd(dy, z, r, g):
    """Returns (dz, dgamma) for y = z*r*g. With zhat = z*r: dz = r * (g*dy - zhat * mean(g*dy*zhat))."""
    zhat = z * r[:, None]
    gg = dy * g
    dz = r[:, None] * (gg - zhat * (gg * zhat).mean(axis=-1, keepdims=True))
    return dz, (dy * zhat).sum(axis=0)


def rope_angles(cfg):
    """[S, d/2] rotation angles: position m, pair j -> m * base^(-2j/d)."""
    d = cfg.attn_width // cfg.heads
    theta = cfg.rope_base ** (-2.0 * np.arange(d // 2) / d)
    return np.arange(cfg.seq, dtype=np.float64)[:, None] * theta[None, :]


def rope_apply(cfg, qkv, inverse=False):
    """Rotates the adjacent pairs of the Q and K parts of a packed [T,3H] array; V is copied.

    ``inverse`` rotates by the negative angle: the transpose of the rotation, which is what carries a
    gradient w.r.t. the rotated vectors back to the unrotated ones.
    """
    B, S, H, h = cfg.batch, cfg.seq, cfg.attn_width, cfg.heads   # H: width of each of Q, K, V
    d = H // h
    ang = rope_angles(cfg)
    c, s = np.cos(ang), np.sin(ang)
    if inverse:
        s = -s
    c, s = c[None, :, None, :], s[None, :, None, :]            # broadcast over batch and the 2h heads of Q, K
    qk = np.ascontiguousarray(qkv[:, :2 * H]).reshape(B, S, 2 * h, d // 2, 2)
    even, odd = qk[..., 0], qk[..., 1]
    rot = np.stack([even * c - odd * s, even * s + odd * c], axis=-1)
    out = np.array(qkv, dtype=np.float64, copy=True)
    out[:, :2 * H] = rot.reshape(B * S, 2 * H)
    return out


def silu(u):
    return u / (1.0 + np.exp(-u))


def silu_grad(u):
    sg = 1.0 / (1.0 + np.exp(-u))
    return sg * (1.0 + u * (1.0 - sg))


def layer_forward(cfg, params, x, seqlens=None):
    """Forward of one layer. Returns a dict with the output ``y`` [B,S,H] and every intermediate."""
    p = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    T, H = cfg.batch * cfg.seq, cfg.hidden
    X = np.asarray(x, dtype=np.float64).reshape(T, H)
    scale = 1.0 / (1.0 - cfg.dropout_p)
    c = {"X": X, "M1": dropout_keep(cfg, 0), "M2": dropout_keep(cfg, 1)}
    c["N1"], c["r1"] = rms_norm(X, p["ln1_g"], cfg.ln_eps)
    c["QKV0"] = c["N1"] @ p["wqkv"].T
    c["QKV"] = rope_apply(cfg, c["QKV0"])
    c["A"], c["P"], c["LSE"] = attention_fwd(cfg, c["QKV"], seqlens)
    c["R1"] = c["A"] @ p["wo"].T
    c["Z1"] = X + c["M1"] * c["R1"] * scale
    c["N2"], c["r2"] = rms_norm(c["Z1"], p["ln2_g"], cfg.ln_eps)
    c["UV"] = c["N2"] @ p["w1"].T                     # [T,2F]: gate in the even columns, up in the odd ones
    U, V = c["UV"][:, 0::2], c["UV"][:, 1::2]
    c["G"] = silu(U) * V
    c["R2"] = c["G"] @ p["w2"].T
    c["y"] = (c["Z1"] + c["M2"] * c["R2"] * scale).reshape(cfg.batch, cfg.seq, H)
    return c


def layer_backward(cfg, params, c, dy):
    """Backward of one layer given the forward dict ``c`` and dL/dy. Returns {'dx', 'wqkv', 'wo', ...}."""
    p = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    T, H = cfg.batch * cfg.seq, cfg.hidden
    dY = np.asarray(dy, dtype=np.float64).reshape(T, H)
    scale = 1.0 / (1.0 - cfg.dropout_p)
    g = {}
    dZ1 = dY.copy()                                   # residual branch of y = Z1 + drop(R2)
    dR2 = dY * c["M2"] * scale
    g["w2"] = dR2.T @ c["G"]
    dG = dR2 @ p["w2"]
    U, V = c["UV"][:, 0::2], c["UV"][:, 1::2]
    dUV = np.empty_like(c["UV"])
    dUV[:, 0::2] = dG * V * silu_grad(U)
    dUV[:, 1::2] = dG * silu(U)
    g["w1"] = dUV.T @ c["N2"]
    d, g["ln2_g"] = rms_norm_bwd(dUV @ p["w1"], c["Z1"], c["r2"], p["ln2_g"])
    dZ1 = dZ1 + d
    dX = dZ1.copy()                                   # residual branch of Z1 = X + drop(R1)
    dR1 = dZ1 * c["M1"] * scale
    g["wo"] = dR1.T @ c["A"]
    dA = dR1 @ p["wo"]
    dQKV = attention_bwd(cfg, c["QKV"], c["P"], dA)   # w.r.t. the rotated queries and keys
    dQKV0 = rope_apply(cfg, dQKV, inverse=True)
    g["wqkv"] = dQKV0.T @ c["N1"]
    d, g["ln1_g"] = rms_norm_bwd(dQKV0 @ p["wqkv"], c["X"], c["r1"], p["ln1_g"])
    g["dx"] = (dX + d).reshape(cfg.batch, cfg.seq, H)
    g["_dQKV"], g["_dQKV0"], g["_dUV"], g["_dG"] = dQKV, dQKV0, dUV, dG
    return g
