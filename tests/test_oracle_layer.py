"""Pins for the fp64 layer oracle (CPU only): finite differences, a torch fp64 autograd rebuild from
library ops, and the invariants the definitions imply."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as W
from oracle import layer as L

VARIANTS = [dict(pre_ln=pl, act=act, causal=ca, len_hi=lh, len_lo=(2 if lh else 0))
            for pl, act, ca, lh in [(0, W.GELU, 0, 0), (0, W.GELU, 0, 6), (1, W.RELU, 1, 0),
                                    (1, W.GELU, 1, 6), (0, W.RELU, 1, 0), (1, W.GELU, 0, 5)]]
# with dropout on the attention probabilities (section 2.2 step 2 listing): padded encoder, causal pre-LN decoder
VARIANTS += [dict(pre_ln=0, act=W.GELU, causal=0, len_hi=6, len_lo=3, attn_dropout_p=0.3, seq=8),
             dict(pre_ln=1, act=W.GELU, causal=1, len_hi=0, len_lo=0, attn_dropout_p=0.4, seq=8)]
# attention width different from the hidden size (one rank's heads of a head-sharded layer; a wider inner width)
VARIANTS += [dict(pre_ln=0, act=W.GELU, causal=0, len_hi=6, len_lo=2, heads=1, attn_dim=4),
             dict(pre_ln=1, act=W.RELU, causal=1, len_hi=0, len_lo=0, heads=3, attn_dim=12)]


def _setup(**kw):
    cfg = W.small_config(**kw)
    params = {k: v.astype(np.float64) for k, v in W.make_params(cfg, perturbed=True).items()}
    # larger weights than the benchmark init so that every path carries a visible signal
    for k in ("wqkv", "wo", "w1", "w2"):
        params[k] = params[k] * 15.0
    x, dy, sl = W.make_inputs(cfg)
    return cfg, params, x.astype(np.float64), dy.astype(np.float64), sl


@pytest.mark.parametrize("variant", VARIANTS)
def test_backward_matches_central_finite_differences(variant):
    cfg, params, x, dy, sl = _setup(**variant)
    c = L.layer_forward(cfg, params, x, sl)
    g = L.layer_backward(cfg, params, c, dy)

    def loss(pp, xx):
        return float((L.layer_forward(cfg, pp, xx, sl)["y"] * dy).sum())

    h = 1e-6
    worst = 0.0
    for name in ("x",) + W.PARAM_NAMES:
        base = x if name == "x" else params[name]
        grad = g["dx"] if name == "x" else g[name]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = base[idx]
            base[idx] = old + h
            lp = loss(params, x)
            base[idx] = old - h
            lm = loss(params, x)
            base[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.abs(num - grad).max() / max(np.abs(num).max(), 1e-12)
        worst = max(worst, err)
        assert err < 1e-6, (name, err)
    assert worst < 1e-6


def _torch_layer(cfg, tp, x, sl, M1, M2, MA=None):
    """The same layer built only from torch CPU fp64 library ops, the dropout masks entering as constants."""
    B, S, H, h, AW = cfg.batch, cfg.seq, cfg.hidden, cfg.heads, cfg.attn_width
    d = AW // h
    scale = 1.0 / (1.0 - cfg.dropout_p)
    ok = torch.ones(B, 1, S, S, dtype=torch.bool)
    if cfg.causal:
        ok = ok & torch.tril(torch.ones(S, S, dtype=torch.bool))
    if sl is not None:
        ok = ok & (torch.arange(S)[None, :] < torch.tensor(sl)[:, None])[:, None, None, :]
    ln = lambda z, k: F.layer_norm(z, (H,), tp[k + "_g"], tp[k + "_b"], cfg.ln_eps)
    act = F.gelu if cfg.act == W.GELU else F.relu
    a_in = ln(x, "ln1") if cfg.pre_ln else x
    q, k, v = F.linear(a_in, tp["wqkv"], tp["bqkv"]).split(AW, dim=-1)
    heads = lambda t: t.reshape(B, S, h, d).transpose(1, 2)
    if MA is None:
        A = F.scaled_dot_product_attention(heads(q), heads(k), heads(v), attn_mask=ok)
    else:   # dropout(softmax(scores), p) @ v with the keep decisions given
        sc = (heads(q) @ heads(k).transpose(-1, -2)) / d ** 0.5
        pr = torch.softmax(sc.masked_fill(~ok, float("-inf")), dim=-1)
        A = (pr * MA / (1.0 - cfg.attn_dropout_p)) @ heads(v)
    A = A.transpose(1, 2).reshape(B, S, AW)
    z1 = x + M1 * (F.linear(A, tp["wo"]) + tp["bo"]) * scale
    f_in = ln(z1, "ln2") if cfg.pre_ln else ln(z1, "ln1")
    r2 = F.linear(act(F.linear(f_in, tp["w1"], tp["b1"])), tp["w2"])
    if cfg.pre_ln:
        return z1 + M2 * (r2 + tp["b2"]) * scale
    return ln(f_in + M2 * (r2 + tp["b2"]) * scale, "ln2")


@pytest.mark.parametrize("variant", VARIANTS)
def test_matches_torch_fp64_library_ops_and_autograd(variant):
    cfg, params, x, dy, sl = _setup(**variant)
    c = L.layer_forward(cfg, params, x, sl)
    g = L.layer_backward(cfg, params, c, dy)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    shape = (cfg.batch, cfg.seq, cfg.hidden)
    MA = L.attention_keep(cfg)
    y = _torch_layer(cfg, tp, tx, sl, torch.tensor(c["M1"]).reshape(shape), torch.tensor(c["M2"]).reshape(shape),
                     None if MA is None else torch.tensor(MA))
    assert L.max_rel_err(c["y"], y.detach().numpy()) < 1e-12
    y.backward(torch.tensor(dy))
    assert L.max_rel_err(g["dx"], tx.grad.numpy()) < 1e-11
    for name in W.PARAM_NAMES:
        assert L.max_rel_err(g[name], tp[name].grad.numpy()) < 1e-11, name


def test_softmax_rows_and_masks():
    cfg, params, x, dy, sl = _setup(causal=1, len_lo=3, len_hi=6)
    c = L.layer_forward(cfg, params, x, sl)
    P = c["P"]
    assert np.abs(P.sum(-1) - 1.0).max() < 1e-12
    S = cfg.seq
    for b in range(cfg.batch):
        for i in range(S):
            for j in range(S):
                if j > i or j >= sl[b]:
                    assert (P[b, :, i, j] == 0.0).all()
    # the saved logsumexp reproduces the probabilities from the raw scores
    H, d = cfg.hidden, cfg.head_dim
    for b in range(cfg.batch):
        for a in range(cfg.heads):
            rows = slice(b * S, (b + 1) * S)
            q = c["QKV"][rows, a * d:(a + 1) * d]
            k = c["QKV"][rows, H + a * d:H + (a + 1) * d]
            sc = q @ k.T / np.sqrt(d)
            ok = L.score_mask(cfg, sl, b)
            naive = np.log(np.where(ok, np.exp(sc), 0.0).sum(-1))
            assert np.abs(naive - c["LSE"][b, a]).max() < 1e-12
            assert np.abs(np.where(ok, np.exp(sc - c["LSE"][b, a][:, None]), 0.0) - P[b, a]).max() < 1e-12


def test_layernorm_moments():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((7, 32)) * 3 + 2
    y, mu, rstd = L.layer_norm(z, np.ones(32), np.zeros(32), 1e-5)
    assert np.abs(y.mean(-1)).max() < 1e-12
    var = z.var(-1)
    assert np.abs(y.var(-1) - var / (var + 1e-5)).max() < 1e-12
    assert np.abs(y.var(-1) - 1.0).max() < 1e-4


@pytest.mark.parametrize("pre_ln", [0, 1])
def test_causal_layer_ignores_future_tokens(pre_ln):
    cfg, params, x, dy, sl = _setup(causal=1, pre_ln=pre_ln)
    y0 = L.layer_forward(cfg, params, x, None)["y"]
    x2 = x.copy()
    i = 3
    x2[:, i + 1:, :] += np.random.default_rng(1).standard_normal(x2[:, i + 1:, :].shape)
    y1 = L.layer_forward(cfg, params, x2, None)["y"]
    assert np.array_equal(y0[:, :i + 1], y1[:, :i + 1])
    assert not np.array_equal(y0[:, i + 1:], y1[:, i + 1:])


def test_padding_mask():
    cfg, params, x, dy, _ = _setup()
    sl = np.array([4, 6], dtype=np.int32)
    c0 = L.layer_forward(cfg, params, x, sl)
    x2 = x.copy()
    x2[0, 4:, :] += 1.0                       # padded keys of sample 0
    c1 = L.layer_forward(cfg, params, x2, sl)
    S = cfg.seq
    assert np.array_equal(c0["A"][0:4], c1["A"][0:4])          # valid rows of sample 0
    assert np.array_equal(c0["A"][S:2 * S], c1["A"][S:2 * S])  # sample 1 untouched
    full = L.layer_forward(cfg, params, x, np.array([S, S], dtype=np.int32))
    none = L.layer_forward(cfg, params, x, None)
    assert np.array_equal(full["y"], none["y"])


def test_fused_qkv_equals_three_linears():
    cfg, params, x, dy, sl = _setup()
    c = L.layer_forward(cfg, params, x, sl)
    H = cfg.hidden
    X = x.reshape(-1, H)
    for i in range(3):
        w, b = params["wqkv"][i * H:(i + 1) * H], params["bqkv"][i * H:(i + 1) * H]
        assert np.abs(c["QKV"][:, i * H:(i + 1) * H] - (X @ w.T + b)).max() < 1e-13


def test_tensor_parallel_identity():
    """f(XA)B = f(XA1)B1 + f(XA2)B2 (section 2.2, step 3): heads split in two halves."""
    cfg, params, x, dy, sl = _setup(heads=2)
    c = L.layer_forward(cfg, params, x, sl)
    H, d = cfg.hidden, cfg.head_dim
    total = np.zeros_like(c["R1"])
    for a in range(cfg.heads):
        total += c["A"][:, a * d:(a + 1) * d] @ params["wo"][:, a * d:(a + 1) * d].T
    assert np.abs(total - c["R1"]).max() < 1e-13
    F_ = cfg.ffn
    halves = [slice(0, F_ // 2), slice(F_ // 2, F_)]
    r2 = sum(c["G"][:, s] @ params["w2"][:, s].T for s in halves)
    assert np.abs(r2 - c["R2"]).max() < 1e-13


def test_zero_dropout_is_identity_and_masked_positions_are_dropped():
    cfg, params, x, dy, sl = _setup(dropout_p=0.0)
    c = L.layer_forward(cfg, params, x, sl)
    assert c["M1"].all() and c["M2"].all()
    assert np.array_equal(c["Z1"], c["X"] + (c["R1"] + params["bo"]))
    cfg, params, x, dy, sl = _setup(dropout_p=0.5)
    c = L.layer_forward(cfg, params, x, sl)
    dropped = c["M1"] == 0
    assert dropped.any() and (~dropped).any()
    assert np.array_equal(c["Z1"][dropped], c["X"][dropped])
    assert np.allclose(c["Z1"][~dropped], (c["X"] + 2.0 * (c["R1"] + params["bo"]))[~dropped], rtol=0, atol=1e-13)


def test_attention_dropout_mask_stream_and_effect():
    """Site 2: element ((b*heads + a)*S + i)*S + j of the Philox stream; dropped probabilities leave A, kept ones
    are scaled by 1/(1-p); p = 0 is the plain attention bit for bit."""
    from test_oracle_philox import _keep_scalar
    cfg, params, x, dy, sl = _setup(attn_dropout_p=0.3, seq=8, len_hi=7, len_lo=4)
    cfg = cfg.replace(seed=0x0123456789ABCDEF, layer_id=3)
    keep = L.attention_keep(cfg)
    B, h, S = cfg.batch, cfg.heads, cfg.seq
    assert keep.shape == (B, h, S, S) and set(np.unique(keep)) <= {0.0, 1.0}
    for (b, a, i, j) in [(0, 0, 0, 0), (0, 0, 0, 7), (0, 1, 3, 5), (1, 0, 7, 7), (1, 1, 2, 1), (1, 1, 7, 6)]:
        e = ((b * h + a) * S + i) * S + j
        assert bool(keep[b, a, i, j]) == _keep_scalar(e, 0.3, cfg.seed, 2, cfg.layer_id), (b, a, i, j)
    # a different stream from the two residual sites
    assert not np.array_equal(keep.reshape(-1)[:B * S * cfg.hidden],
                              L.dropout_keep(cfg, 0).reshape(-1)[:keep.size][:B * S * cfg.hidden])
    # effect on A, written out by hand for one (sample, head, query row)
    qkv = L.layer_forward(cfg, params, x, sl)["QKV"]
    A, P, _ = L.attention_fwd(cfg, qkv, sl)
    H, d = cfg.hidden, cfg.hidden // cfg.heads
    b, a, i = 1, 1, 5
    v = qkv[b * S:(b + 1) * S, 2 * H + a * d:2 * H + (a + 1) * d]
    want = sum(P[b, a, i, j] * keep[b, a, i, j] / 0.7 * v[j] for j in range(S))
    assert np.allclose(A[b * S + i, a * d:(a + 1) * d], want, rtol=1e-13, atol=1e-15)
    assert np.allclose(P[b, a].sum(axis=-1), 1.0)          # P itself stays the undropped softmax
    A0, _, _ = L.attention_fwd(cfg.replace(attn_dropout_p=0.0), qkv, sl)
    assert np.array_equal(A0[b * S + i, a * d:(a + 1) * d], (P[b, a] @ v)[i])


def test_head_sharded_attention_blocks_sum_to_the_full_block():
    """Section 2.2 step 3: with the fused QKV and the output projection sharded along the heads, every rank runs
    the attention block at width H/tp and the partial outputs add up to the unsharded block's."""
    cfg, params, x, dy, sl = _setup(heads=4, hidden=8, causal=1, len_lo=3, len_hi=6)
    full = L.layer_forward(cfg, params, x, sl)
    H, h, d = cfg.hidden, cfg.heads, cfg.head_dim
    for tp in (2, 4):
        share = cfg.replace(heads=h // tp, attn_dim=H // tp)
        assert share.head_dim == d and share.attn_width == H // tp
        total = 0.0
        for r in range(tp):
            cols = np.arange(r * H // tp, (r + 1) * H // tp)                 # this rank's heads
            rows = np.concatenate([cols, H + cols, 2 * H + cols])            # their Q, K and V rows of wqkv
            qkv_r = full["X"] @ params["wqkv"][rows].T + params["bqkv"][rows]
            a_r, _, lse_r = L.attention_fwd(share, qkv_r, sl)
            assert np.array_equal(a_r, full["A"][:, cols]) and np.array_equal(lse_r, full["LSE"][:, r * h // tp:(r + 1) * h // tp])
            total = total + a_r @ params["wo"][:, cols].T
        assert np.abs(total - full["R1"]).max() < 1e-13
