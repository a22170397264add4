"""GPU parity: dropout mask (bit-exact), fused bias+dropout+residual+LayerNorm forward / backward,
column reductions -- HIP path through the C ABI vs the fp64 oracle."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import layer as L
from oracle import philox
from paper_2302_08005_amd import binding as B
from gpu_util import DEV, TOL, err, store, tdtype, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,H,p,seed,site,layer", [(256, 256, 0.1, 0, 0, 0), (1000, 1024, 0.1, 0x1234567890ABCDEF, 1, 23),
                                                   (4096, 2560, 0.5, 7, 1, 3), (64, 64, 0.0, 1, 0, 0)])
def test_dropout_mask_bit_exact(T, H, p, seed, site, layer):
    d = B.make_desc(batch=1, seq=T, hidden=H, heads=H // 64, ffn=64, dropout_p=p, seed=seed, layer_id=layer)
    m = torch.empty(T * H, dtype=torch.uint8, device=DEV)
    B.slapo_dropout_mask(d, site, T, m)
    ref = philox.keep_mask(T * H, p, seed, site, layer)
    assert np.array_equal(m.cpu().numpy().astype(bool), ref)


def _ref_fwd(r, bias, res, gamma, beta, keep, p, eps):
    z = res + keep * (r + bias) / (1.0 - p) if r is not None else res
    if gamma is None:
        return z, None, None, None
    y, mu, rstd = L.layer_norm(z, gamma, beta, eps)
    return z, y, mu, rstd


@pytest.mark.parametrize("dtype", [W.FP32, W.BF16, W.FP16])
@pytest.mark.parametrize("T,H", [(37, 256), (515, 1024), (130, 2560), (64, 4096), (9, 64), (70, 5120), (35, 8192)])
def test_bdrln_forward_and_backward(dtype, T, H):
    rng = np.random.default_rng(T * 7 + H)
    p, seed, site, layer = 0.1, 11, 1, 5
    d = B.make_desc(batch=1, seq=T, hidden=H, heads=H // 64, ffn=64, dropout_p=p, seed=seed, layer_id=layer, dtype=dtype)
    dt = tdtype(dtype)
    r, res, dy, dres = (store(rng.standard_normal((T, H)), dtype) for _ in range(4))
    bias, beta = (store(rng.standard_normal(H) * 0.1, dtype) for _ in range(2))
    gamma = store(1.0 + rng.standard_normal(H) * 0.1, dtype)
    keep = philox.keep_mask(T * H, p, seed, site, layer).reshape(T, H).astype(np.float64)
    z_ref, y_ref, mu_ref, rstd_ref = _ref_fwd(r.astype(np.float64), bias, res.astype(np.float64), gamma, beta, keep, p, 1e-5)

    z = torch.empty(T, H, dtype=dt, device=DEV)
    y = torch.empty_like(z)
    mu = torch.empty(T, dtype=torch.float32, device=DEV)
    rstd = torch.empty_like(mu)
    B.slapo_bdrln_fwd(d, site, T, to_dev(r, dtype), to_dev(bias, dtype), to_dev(res, dtype), to_dev(gamma, dtype),
                      to_dev(beta, dtype), z, y, mu, rstd)
    tol = TOL[dtype]
    assert err(z, z_ref) <= tol and err(y, y_ref) <= tol
    assert err(mu, mu_ref) <= tol and err(rstd, rstd_ref) <= tol
    if dtype != W.FP32:
        # a 16-bit output carries two roundings (the stored sum, the output): a few units of the type's own
        # precision, so half storage must be about 8 times closer than bf16 (a rounding through the wrong
        # 16-bit type anywhere in the kernel fails this)
        unit = 2.0 ** (-8 if dtype == W.BF16 else -11)
        assert err(z, z_ref) <= unit and err(y, y_ref) <= 4 * unit, (err(z, z_ref), err(y, y_ref), unit)
    # dropped positions carry the residual exactly (no bias leak)
    assert np.array_equal(to_np(z)[keep == 0], res.astype(np.float64)[keep == 0])

    # LN only, and bias+dropout+residual only
    y2 = torch.empty_like(z)
    B.slapo_bdrln_fwd(d, site, T, None, None, to_dev(res, dtype), to_dev(gamma, dtype), to_dev(beta, dtype), None, y2, mu, rstd)
    assert err(y2, L.layer_norm(res.astype(np.float64), gamma, beta, 1e-5)[0]) <= tol
    z3 = torch.empty_like(z)
    B.slapo_bdrln_fwd(d, site, T, to_dev(r, dtype), to_dev(bias, dtype), to_dev(res, dtype), None, None, z3, None, None, None)
    assert err(z3, z_ref) <= tol

    # backward, on the oracle's own forward values so that only the backward arithmetic is compared
    zs = store(z_ref, dtype)
    _, _, mu_s, rstd_s = _ref_fwd(None, None, zs.astype(np.float64), gamma, beta, keep, p, 1e-5)
    dz_ref, dg_ref, db_ref = L.layer_norm_bwd(dy.astype(np.float64), zs.astype(np.float64), mu_s, rstd_s, gamma.astype(np.float64))
    dz_ref = dz_ref + dres
    dr_ref = dz_ref * keep / (1.0 - p)
    nblk = B.slapo_bdrln_bwd_blocks(T)
    part = torch.empty(nblk, 3, H, dtype=torch.float32, device=DEV)
    dz = torch.empty_like(z)
    dr = torch.empty_like(z)
    B.slapo_bdrln_bwd(d, site, T, to_dev(dy, dtype), to_dev(zs, dtype), torch.from_numpy(mu_s.astype(np.float32)).to(DEV),
                      torch.from_numpy(rstd_s.astype(np.float32)).to(DEV), to_dev(gamma, dtype), to_dev(dres, dtype), dz, dr, part)
    assert err(dz, dz_ref) <= tol and err(dr, dr_ref) <= tol
    outs = []
    for which in range(3):
        o = torch.empty(H, dtype=dt, device=DEV)
        B.slapo_colreduce_partials(dtype, nblk, 3 * H, H, part.view(-1)[which * H:], o, 0)
        outs.append(o)
    assert err(outs[0], dg_ref) <= tol and err(outs[1], db_ref) <= tol and err(outs[2], dr_ref.sum(0)) <= tol
    # no LayerNorm: dz = dout (+ dres), dr masked
    B.slapo_bdrln_bwd(d, site, T, to_dev(dy, dtype), None, None, None, None, None, None, dr, part)
    assert err(dr, dy.astype(np.float64) * keep / (1.0 - p)) <= tol


@pytest.mark.parametrize("dtype", [W.FP32, W.BF16, W.FP16])
@pytest.mark.parametrize("T,N", [(100, 264), (4096, 3072), (33, 8)])
def test_column_sums(dtype, T, N):
    rng = np.random.default_rng(3)
    a = store(rng.standard_normal((T, N)), dtype)
    nblk = B.slapo_colsum_blocks(T)
    part = torch.empty(nblk, N, dtype=torch.float32, device=DEV)
    dt = tdtype(dtype)
    out = torch.ones(N, dtype=dt, device=DEV)
    B.slapo_colsum_partials(dtype, T, N, to_dev(a, dtype), part)
    B.slapo_colreduce_partials(dtype, nblk, N, N, part, out, 0)
    assert err(out, a.astype(np.float64).sum(0)) <= TOL[dtype]
    B.slapo_colreduce_partials(dtype, nblk, N, N, part, out, 1)     # accumulate on top
    assert err(out, 2 * a.astype(np.float64).sum(0)) <= 2 * TOL[dtype]
