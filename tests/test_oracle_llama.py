"""Pins for the fp64 oracle of the LLaMA-style layer (CPU only): finite differences, a torch fp64 autograd
rebuild from library ops in a different formulation (complex multiplication for the rotary embedding,
F.rms_norm, F.silu, F.scaled_dot_product_attention), and what the published definitions fix by themselves."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as W
from oracle import layer as L
from oracle import llama_layer as LL

VARIANTS = [dict(dropout_p=0.0), dict(dropout_p=0.25), dict(dropout_p=0.25, len_lo=2, len_hi=6),
            dict(dropout_p=0.0, heads=1), dict(dropout_p=0.1, attn_dropout_p=0.3, seq=8),
            dict(dropout_p=0.0, heads=1, attn_dim=4), dict(dropout_p=0.25, heads=3, attn_dim=12)]   # attention width != hidden


def _setup(**kw):
    base = dict(arch=W.LLAMA, pre_ln=1, causal=1, ln_eps=1e-6)
    base.update(kw)
    cfg = W.small_config(**base)
    params = {k: v.astype(np.float64) for k, v in W.make_params(cfg, perturbed=True).items()}
    for k in ("wqkv", "wo", "w1", "w2"):    # larger than the benchmark init: every path carries a visible signal
        params[k] = params[k] * 15.0
    x, dy, sl = W.make_inputs(cfg)
    return cfg, params, x.astype(np.float64), dy.astype(np.float64), sl


@pytest.mark.parametrize("variant", VARIANTS)
def test_backward_matches_central_finite_differences(variant):
    cfg, params, x, dy, sl = _setup(**variant)
    g = LL.layer_backward(cfg, params, LL.layer_forward(cfg, params, x, sl), dy)

    def loss():
        return float((LL.layer_forward(cfg, params, x, sl)["y"] * dy).sum())

    h = 1e-6
    for name in ("x",) + W.param_names(cfg):
        base = x if name == "x" else params[name]
        grad = g["dx"] if name == "x" else g[name]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = base[idx]
            base[idx] = old + h
            lp = loss()
            base[idx] = old - h
            lm = loss()
            base[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.abs(num - grad).max() / max(np.abs(num).max(), 1e-12)
        assert err < 1e-6, (name, err)


def _torch_layer(cfg, tp, x, sl, M1, M2, MA):
    """The same layer from torch CPU fp64 library ops; rotary embedding as a complex multiplication."""
    B, S, H, h, AW = cfg.batch, cfg.seq, cfg.hidden, cfg.heads, cfg.attn_width
    d = AW // h
    scale = 1.0 / (1.0 - cfg.dropout_p)
    inv_freq = 1.0 / (cfg.rope_base ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
    phase = torch.polar(torch.ones(S, d // 2, dtype=torch.float64), torch.outer(torch.arange(S, dtype=torch.float64), inv_freq))

    def rotate(t):   # t [B,S,h,d] -> same, adjacent pairs read as complex numbers
        tc = torch.view_as_complex(t.reshape(B, S, h, d // 2, 2))
        return torch.view_as_real(tc * phase[None, :, None, :]).reshape(B, S, h, d)

    ok = torch.tril(torch.ones(S, S, dtype=torch.bool))[None, None]
    if sl is not None:
        ok = ok & (torch.arange(S)[None, :] < torch.tensor(sl)[:, None])[:, None, None, :]
    n1 = F.rms_norm(x, (H,), tp["ln1_g"], cfg.ln_eps)
    q, k, v = F.linear(n1, tp["wqkv"]).split(AW, dim=-1)
    q = rotate(q.reshape(B, S, h, d)).transpose(1, 2)
    k = rotate(k.reshape(B, S, h, d)).transpose(1, 2)
    v = v.reshape(B, S, h, d).transpose(1, 2)
    if MA is None:
        A = F.scaled_dot_product_attention(q, k, v, attn_mask=ok)
    else:
        pr = torch.softmax(((q @ k.transpose(-1, -2)) / d ** 0.5).masked_fill(~ok, float("-inf")), dim=-1)
        A = (pr * MA / (1.0 - cfg.attn_dropout_p)) @ v
    A = A.transpose(1, 2).reshape(B, S, AW)
    z1 = x + M1 * F.linear(A, tp["wo"]) * scale
    n2 = F.rms_norm(z1, (H,), tp["ln2_g"], cfg.ln_eps)
    gate, up = F.linear(n2, tp["w1"][0::2]), F.linear(n2, tp["w1"][1::2])
    return z1 + M2 * F.linear(F.silu(gate) * up, tp["w2"]) * scale


@pytest.mark.parametrize("variant", VARIANTS)
def test_matches_torch_fp64_library_ops_and_autograd(variant):
    cfg, params, x, dy, sl = _setup(**variant)
    c = LL.layer_forward(cfg, params, x, sl)
    g = LL.layer_backward(cfg, params, c, dy)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    shape = (cfg.batch, cfg.seq, cfg.hidden)
    MA = L.attention_keep(cfg)
    y = _torch_layer(cfg, tp, tx, sl, torch.tensor(c["M1"]).reshape(shape), torch.tensor(c["M2"]).reshape(shape),
                     None if MA is None else torch.tensor(MA))
    assert L.max_rel_err(c["y"], y.detach().numpy()) < 1e-12
    y.backward(torch.tensor(dy))
    assert L.max_rel_err(g["dx"], tx.grad.numpy()) < 1e-11
    for name in W.param_names(cfg):
        assert L.max_rel_err(g[name], tp[name].grad.numpy()) < 1e-11, name


def test_rotary_embedding_properties():
    """What eq. 34 of the rotary-embedding paper fixes: values at small positions, isometry, and that a
    query-key product depends on the positions only through their difference."""
    cfg = W.small_config(arch=W.LLAMA, batch=1, seq=16, hidden=16, heads=2, causal=1)
    H, d = cfg.hidden, cfg.hidden // cfg.heads
    rng = np.random.default_rng(5)
    qkv = rng.standard_normal((cfg.seq, 3 * H))
    rot = LL.rope_apply(cfg, qkv)
    assert np.array_equal(rot[:, 2 * H:], qkv[:, 2 * H:])                      # values untouched
    assert np.allclose(rot[0], qkv[0], rtol=0, atol=0)                        # position 0: identity
    # pair 0 turns by one radian per position, pair j by base^(-2j/d) radians
    e = np.zeros((cfg.seq, 3 * H)); e[:, 0] = 1.0; e[:, 2] = 1.0
    r = LL.rope_apply(cfg, e)
    for m in (1, 2, 7):
        assert np.allclose(r[m, 0:2], [np.cos(m), np.sin(m)], atol=1e-15)
        th = cfg.rope_base ** (-2.0 / d)
        assert np.allclose(r[m, 2:4], [np.cos(m * th), np.sin(m * th)], atol=1e-15)
    # the same frequencies restart in every head and in K
    e2 = np.zeros((cfg.seq, 3 * H)); e2[:, d + 1] = 1.0; e2[:, H + 1] = 1.0
    r2 = LL.rope_apply(cfg, e2)
    assert np.allclose(r2[3, d:d + 2], [-np.sin(3.0), np.cos(3.0)], atol=1e-15)
    assert np.allclose(r2[3, H:H + 2], [-np.sin(3.0), np.cos(3.0)], atol=1e-15)
    # isometry per head, and inverse = transpose
    for a in range(2 * cfg.heads):
        assert np.allclose(np.linalg.norm(rot[:, a * d:(a + 1) * d], axis=1), np.linalg.norm(qkv[:, a * d:(a + 1) * d], axis=1))
    assert np.allclose(LL.rope_apply(cfg, rot, inverse=True), qkv, atol=1e-14)
    u, v = rng.standard_normal((cfg.seq, 3 * H)), rng.standard_normal((cfg.seq, 3 * H))
    assert abs((LL.rope_apply(cfg, u) * v).sum() - (u * LL.rope_apply(cfg, v, inverse=True)).sum()) < 1e-12
    # relative-position property: the same q and k placed at (m, n) and at (m + 5, n + 5) give the same product
    q0, k0 = rng.standard_normal(d), rng.standard_normal(d)
    def prod(m, n):
        t = np.zeros((cfg.seq, 3 * H)); t[m, :d] = q0; t[n, H:H + d] = k0
        rr = LL.rope_apply(cfg, t)
        return rr[m, :d] @ rr[n, H:H + d]
    assert abs(prod(3, 1) - prod(8, 6)) < 1e-13 and abs(prod(3, 1) - prod(10, 8)) < 1e-13
    assert abs(prod(3, 1) - prod(4, 1)) > 1e-3                                 # and does change with the distance


def test_rms_norm_definition_and_special_cases():
    rng = np.random.default_rng(9)
    z = rng.standard_normal((7, 32)) * 3.0
    g = 1.0 + 0.1 * rng.standard_normal(32)
    y, r = LL.rms_norm(z, g, 0.0)
    assert np.allclose(((y / g) ** 2).mean(axis=1), 1.0)                        # unit mean square before the gain
    y2, _ = LL.rms_norm(5.0 * z, g, 0.0)
    assert np.allclose(y, y2)                                                  # invariant to the input's scale
    # on rows of zero mean it is LayerNorm without offset (the routine pinned elsewhere)
    zc = z - z.mean(axis=1, keepdims=True)
    yl, _, rstd = L.layer_norm(zc, g, np.zeros(32), 1e-5)
    yr, r = LL.rms_norm(zc, g, 1e-5)
    assert np.allclose(yl, yr, atol=1e-14) and np.allclose(r, rstd)
    # eps inside the root: a zero row gives zero output and r = eps^-1/2
    y0, r0 = LL.rms_norm(np.zeros((1, 32)), g, 1e-6)
    assert np.all(y0 == 0.0) and np.allclose(r0, 1e3)
    # backward: the input gradient is orthogonal to z when eps = 0 (the output does not change along z)
    dy = rng.standard_normal((7, 32))
    dz, dg = LL.rms_norm_bwd(dy, z, LL.rms_norm(z, g, 0.0)[1], g)
    assert np.abs((dz * z).sum(axis=1)).max() < 1e-12
    assert np.allclose(dg, (dy * z * LL.rms_norm(z, g, 0.0)[1][:, None]).sum(axis=0))


def test_silu_and_gated_ffn_special_cases():
    u = np.linspace(-6, 6, 25)
    assert LL.silu(np.array([0.0]))[0] == 0.0 and LL.silu_grad(np.array([0.0]))[0] == 0.5
    assert np.allclose(LL.silu(u) - LL.silu(-u), u)                            # u*s(u) - (-u)*s(-u) = u
    assert np.allclose(LL.silu(u), u * 0.5 * (1.0 + np.tanh(0.5 * u)))         # sigmoid via tanh
    h = 1e-6
    assert np.allclose(LL.silu_grad(u), (LL.silu(u + h) - LL.silu(u - h)) / (2 * h), atol=1e-9)
    # the layer's feed-forward block, rebuilt from the two halves of w1 taken apart
    cfg, params, x, dy, sl = _setup(dropout_p=0.0)
    c = LL.layer_forward(cfg, params, x, sl)
    U, V = c["N2"] @ params["w1"][0::2].T, c["N2"] @ params["w1"][1::2].T
    assert np.allclose(c["G"], U / (1 + np.exp(-U)) * V)
    assert np.allclose(c["y"].reshape(-1, cfg.hidden), c["Z1"] + c["G"] @ params["w2"].T)


def test_zero_output_projections_make_the_layer_the_identity():
    cfg, params, x, dy, sl = _setup(dropout_p=0.25)
    params["wo"][:] = 0.0
    params["w2"][:] = 0.0
    c = LL.layer_forward(cfg, params, x, sl)
    assert np.array_equal(c["y"], x)
    g = LL.layer_backward(cfg, params, c, dy)
    assert np.array_equal(g["dx"], dy)
    for k in ("wqkv", "w1", "ln1_g", "ln2_g"):
        assert np.all(g[k] == 0.0), k


def test_positions_restart_in_every_sequence_and_causality_holds():
    cfg, params, x, dy, sl = _setup(dropout_p=0.0, batch=2)
    x[1] = x[0]                                      # same content in both sequences -> same output
    c = LL.layer_forward(cfg, params, x, None)
    assert np.allclose(c["y"][0], c["y"][1], atol=1e-13)
    x2 = x.copy(); x2[0, 4:] += 1.0                  # changing later tokens leaves earlier outputs alone
    c2 = LL.layer_forward(cfg, params, x2, None)
    assert np.array_equal(c["y"][0, :4], c2["y"][0, :4]) and not np.allclose(c["y"][0, 4:], c2["y"][0, 4:])
