"""GPU parity of the LLaMA-style layer family: the gated GEMM epilogues, the rotary kernel, RMSNorm in the fused
row kernels and the whole layer step, each against the fp64 oracle."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import llama_layer as LL
from oracle import philox
from paper_2302_08005_amd import binding as B
from gpu_util import DEV, TOL, err, store, tdtype, to_dev, to_np

pytestmark = pytest.mark.gpu


# the shapes reach the 256x256-tile kernel, the 128x128 kernel fed by loader wavefronts and the general kernel
@pytest.mark.parametrize("dtype", [W.BF16, W.FP32, W.FP16])
@pytest.mark.parametrize("M,F,K", [(2048, 6144, 128), (1664, 1664, 512), (296, 136, 200)])
def test_gated_epilogues(dtype, M, F, K):
    rng = np.random.default_rng(M + F)
    a = store(rng.standard_normal((M, K)), dtype)
    w = store(rng.standard_normal((2 * F, K)) * (2.0 / np.sqrt(K)), dtype)     # rows: gate_0, up_0, gate_1, ...
    uv = a.astype(np.float64) @ w.astype(np.float64).T
    U, V = uv[:, 0::2], uv[:, 1::2]
    g_ref = LL.silu(U) * V
    f_ref = np.empty_like(uv)
    f_ref[:, 0::2] = V * LL.silu_grad(U)
    f_ref[:, 1::2] = LL.silu(U)
    dt, tol = tdtype(dtype), TOL[dtype]
    A, Wt = to_dev(a, dtype), to_dev(w, dtype)
    G = torch.empty(M, F, dtype=dt, device=DEV)
    Fa = torch.empty(M, 2 * F, dtype=dt, device=DEV)
    B.slapo_gemm(dtype, B.NT, B.EPI_GATE, 0, M, 2 * F, K, A, Wt, G, aux_out=Fa)
    assert err(G, g_ref) <= tol and err(Fa, f_ref) <= tol

    # backward epilogue: the gradient of the gated values (itself a product, [M,F]) times the two stored factors
    K2 = 264 if K % 64 else 256
    dr = store(rng.standard_normal((M, K2)), dtype)
    w2 = store(rng.standard_normal((K2, F)) * (1.0 / np.sqrt(K2)), dtype)
    fac = store(rng.standard_normal((M, 2 * F)), dtype)
    dg = dr.astype(np.float64) @ w2.astype(np.float64)
    duv_ref = np.repeat(dg, 2, axis=1) * fac
    DUV = torch.empty(M, 2 * F, dtype=dt, device=DEV)
    B.slapo_gemm(dtype, B.NN, B.EPI_DGATE, 0, M, F, K2, to_dev(dr, dtype), to_dev(w2, dtype), DUV, aux_in=to_dev(fac, dtype))
    assert err(DUV, duv_ref) <= tol


@pytest.mark.parametrize("dtype", [W.FP32, W.BF16, W.FP16])
@pytest.mark.parametrize("batch,seq,heads,d", [(2, 200, 3, 64), (1, 2048, 1, 128), (3, 64, 2, 128)])
def test_rotary_kernel(dtype, batch, seq, heads, d):
    cfg = W.LayerConfig("rope", batch, seq, heads * d, heads, 64, causal=1, dtype=dtype, arch=W.LLAMA, pre_ln=1)
    desc = B.make_desc(cfg)
    rng = np.random.default_rng(seq)
    qkv = store(rng.standard_normal((batch * seq, 3 * heads * d)), dtype)
    table = torch.empty(seq * (d // 2) * 2, dtype=torch.float32, device=DEV)
    t = to_dev(qkv, dtype)
    B.slapo_rope(desc, t, table, 0)
    ref = LL.rope_apply(cfg, qkv.astype(np.float64))
    tol = {W.FP32: 2e-6, W.BF16: 2.0 ** -8, W.FP16: 2.0 ** -11}[dtype]    # one rounding of the output
    assert err(t, ref) <= tol
    assert torch.equal(t[:, 2 * heads * d:], to_dev(qkv, dtype)[:, 2 * heads * d:])          # V untouched
    ang = LL.rope_angles(cfg)
    tab = to_np(table).reshape(seq, d // 2, 2)
    assert np.abs(tab[..., 0] - np.cos(ang)).max() <= 1.2e-7 and np.abs(tab[..., 1] - np.sin(ang)).max() <= 1.2e-7
    t2 = to_dev(qkv, dtype)
    B.slapo_rope(desc, t2, table, 1)
    assert err(t2, LL.rope_apply(cfg, qkv.astype(np.float64), inverse=True)) <= tol


@pytest.mark.parametrize("dtype", [W.FP32, W.BF16, W.FP16])
@pytest.mark.parametrize("T,H", [(37, 256), (515, 1024), (64, 4096)])
def test_rmsnorm_in_the_fused_row_kernels(dtype, T, H):
    rng = np.random.default_rng(T + H)
    p, seed, site, layer = 0.1, 3, 0, 2
    d = B.make_desc(batch=1, seq=T, hidden=H, heads=H // 64, ffn=64, dropout_p=p, seed=seed, layer_id=layer, dtype=dtype,
                    arch=B.LLAMA, pre_ln=1, ln_eps=1e-6)
    dt, tol = tdtype(dtype), TOL[dtype]
    r, res, dy, dres = (store(rng.standard_normal((T, H)), dtype) for _ in range(4))
    res = store(res + 0.5, dtype)                        # a row mean that RMSNorm must NOT remove
    gamma = store(1.0 + rng.standard_normal(H) * 0.1, dtype)
    keep = philox.keep_mask(T * H, p, seed, site, layer).reshape(T, H).astype(np.float64)
    z_ref = res.astype(np.float64) + keep * r.astype(np.float64) / (1 - p)
    y_ref, r_ref = LL.rms_norm(z_ref, gamma.astype(np.float64), 1e-6)
    z = torch.empty(T, H, dtype=dt, device=DEV)
    y = torch.empty_like(z)
    rstd = torch.empty(T, dtype=torch.float32, device=DEV)
    B.slapo_bdrln_fwd(d, site, T, to_dev(r, dtype), None, to_dev(res, dtype), to_dev(gamma, dtype), None, z, y, None, rstd)
    assert err(z, z_ref) <= tol and err(y, y_ref) <= tol and err(rstd, r_ref) <= tol

    zs = store(z_ref, dtype)
    _, rs = LL.rms_norm(zs.astype(np.float64), gamma.astype(np.float64), 1e-6)
    dz_ref, dg_ref = LL.rms_norm_bwd(dy.astype(np.float64), zs.astype(np.float64), rs, gamma.astype(np.float64))
    dz_ref = dz_ref + dres
    dr_ref = dz_ref * keep / (1 - p)
    nblk = B.slapo_bdrln_bwd_blocks(T)
    part = torch.empty(nblk, 3, H, dtype=torch.float32, device=DEV)
    dz = torch.empty_like(z)
    drr = torch.empty_like(z)
    B.slapo_bdrln_bwd(d, site, T, to_dev(dy, dtype), to_dev(zs, dtype), None, torch.from_numpy(rs.astype(np.float32)).to(DEV),
                      to_dev(gamma, dtype), to_dev(dres, dtype), dz, drr, part)
    assert err(dz, dz_ref) <= tol and err(drr, dr_ref) <= tol
    assert err(part.sum(0)[0], dg_ref) <= max(tol, 1e-5)


SMALL = [
    W.LayerConfig("llama-fp32", 2, 128, 256, 4, 344, causal=1, dropout_p=0.0, dtype=W.FP32, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, config_id=21),
    W.LayerConfig("llama-fp32-dropout-padding-d128", 2, 96, 256, 2, 520, causal=1, dropout_p=0.2, dtype=W.FP32, pre_ln=1,
                  ln_eps=1e-6, arch=W.LLAMA, len_lo=40, len_hi=96, layer_id=3, config_id=22),
    W.LayerConfig("llama-bf16", 3, 200, 384, 6, 1000, causal=1, dropout_p=0.0, dtype=W.BF16, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, config_id=23),
    W.LayerConfig("llama-bf16-d128-dropouts", 2, 264, 512, 4, 1376, causal=1, dropout_p=0.1, attn_dropout_p=0.1, dtype=W.BF16,
                  pre_ln=1, ln_eps=1e-6, arch=W.LLAMA, config_id=24),
    W.LayerConfig("llama-fp16", 2, 264, 512, 4, 1376, causal=1, dropout_p=0.0, dtype=W.FP16, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, config_id=25),
    W.LayerConfig("llama-bf16-bidirectional-base500", 2, 128, 256, 4, 512, causal=0, dropout_p=0.0, dtype=W.BF16, pre_ln=1,
                  ln_eps=1e-5, arch=W.LLAMA, rope_base=500.0, config_id=26),
    # one of four ranks of a head-sharded layer: 2 of 8 heads, a quarter of the FFN
    W.LayerConfig("llama-bf16-tp4-share", 2, 128, 512, 2, 344, causal=1, dropout_p=0.0, dtype=W.BF16, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, attn_dim=128, config_id=27),
]
SAVED = {"qkv": "QKV", "attn": "A", "z1": "Z1", "n1": "N1", "n2": "N2", "g": "G", "lse": "LSE", "rstd1": "r1", "rstd2": "r2"}


def run_case(cfg, perturbed=True, check_saved=True, **layer_kw):
    params = W.make_params(cfg, perturbed=perturbed)
    x, dy, sl = W.make_inputs(cfg)
    ref = LL.layer_forward(cfg, params, x, sl)
    gref = LL.layer_backward(cfg, params, ref, dy)
    layer = B.Layer(cfg, params, **layer_kw)
    xd, dyd = layer.to_device(x), layer.to_device(dy)
    sld = None if sl is None else torch.from_numpy(sl).to(DEV)
    y = layer.forward(xd, sld)
    dx = layer.backward(xd, sld, dyd)
    torch.cuda.synchronize()
    errs = {"y": err(y, ref["y"]), "dx": err(dx, gref["dx"])}
    for k in W.param_names(cfg):
        errs["d" + k] = err(layer.grads[k], gref[k])
    if check_saved and layer.saved is not None:
        for k, rk in SAVED.items():
            errs["saved." + k] = err(layer.saved_tensor(k).reshape(-1), ref[rk].reshape(-1))
        U, V = ref["UV"][:, 0::2], ref["UV"][:, 1::2]
        fac = np.empty_like(ref["UV"])
        fac[:, 0::2], fac[:, 1::2] = V * LL.silu_grad(U), LL.silu(U)
        errs["saved.dgate"] = err(layer.saved_tensor("dgate").reshape(-1), fac.reshape(-1))
    return errs, layer, (xd, sld, dyd, y, dx)


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_llama_layer_parity_small(cfg):
    errs, _, _ = run_case(cfg)
    tol = TOL[cfg.dtype]
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (bad, errs)


@pytest.mark.parametrize("idx", [1, 3])
def test_llama_checkpoint_mode_and_determinism(idx):
    cfg = SMALL[idx]
    errs, layer, (xd, sld, dyd, y, dx) = run_case(cfg, check_saved=False)
    g1 = {k: v.clone() for k, v in layer.grads.items()}
    y2 = layer.forward(xd, sld)
    dx2 = layer.backward(xd, sld, dyd)
    assert torch.equal(y, y2) and torch.equal(dx, dx2)
    ck = B.Layer(cfg, W.make_params(cfg, perturbed=True), checkpoint=1)
    assert ck.saved is None
    y3 = ck.forward(xd, sld)
    ck.scratch.fill_(0xAB)                       # nothing may survive from forward to backward
    dx3 = ck.backward(xd, sld, dyd)
    torch.cuda.synchronize()
    assert torch.equal(y, y3) and torch.equal(dx, dx3)
    for k in W.param_names(cfg):
        assert torch.equal(g1[k], ck.grads[k]), k
    layer.desc.accumulate_grads = 1
    layer.backward(xd, sld, dyd)
    for k in W.param_names(cfg):
        assert err(layer.grads[k], 2 * to_np(g1[k])) <= 1e-2, k


def test_llama_layer_parity_full_size():
    """The LLaMA-7B-shaped layer in the launch configuration bench.py times."""
    cfg = W.CONFIGS["C6"]
    errs, _, _ = run_case(cfg, perturbed=False, check_saved=False)
    bad = {k: v for k, v in errs.items() if not v <= TOL[cfg.dtype]}
    assert not bad, (bad, errs)


@pytest.mark.parametrize("cfg", [
    W.LayerConfig("llama-one-token-fp32", 1, 1, 64, 1, 8, causal=1, dropout_p=0.0, dtype=W.FP32, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, config_id=41),
    W.LayerConfig("llama-three-tokens-bf16", 2, 3, 128, 1, 8, causal=1, dropout_p=0.1, dtype=W.BF16, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, len_lo=1, len_hi=3, config_id=42),
    # the widest rows the RMSNorm kernels take (narrow attention and FFN keep the oracle quick)
    W.LayerConfig("llama-widest-hidden-bf16", 1, 72, 8192, 8, 256, causal=1, dropout_p=0.0, dtype=W.BF16, pre_ln=1, ln_eps=1e-6,
                  arch=W.LLAMA, attn_dim=1024, config_id=43),
], ids=lambda c: c.name)
def test_llama_layer_parity_degenerate_sizes(cfg):
    errs, _, _ = run_case(cfg, check_saved=cfg.hidden <= 4096)   # (intermediates: see the classic layer's test)
    bad = {k: v for k, v in errs.items() if not v <= TOL[cfg.dtype]}
    assert not bad, (bad, errs)
