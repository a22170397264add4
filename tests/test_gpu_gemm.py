"""GPU parity of the GEMMs and their fused epilogues vs fp64 products of the same stored inputs."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import layer as L
from paper_2302_08005_amd import binding as B
from gpu_util import DEV, TOL, err, store, to_dev, to_np

pytestmark = pytest.mark.gpu


# the activation and its derivative are the oracle's own (pinned in tests/test_oracle_layer.py), not a second copy
_act, _dact = L._act, L._act_grad


# the last three reach the direct-load kernels with ragged edge tiles: 128x128 tiles fed by loader wavefronts
# (long K, one round of tiles), 256x256 tiles, and 128x64 tiles (long K, few tiles)
SHAPES = [(256, 256, 128), (296, 264, 200), (128, 128, 64), (1024, 768, 512), (520, 136, 72), (4096, 1024, 1024),
          (1664, 1672, 2048), (3592, 3336, 256), (520, 136, 2048)]


@pytest.mark.parametrize("dtype", [W.BF16, W.FP32, W.FP16])
@pytest.mark.parametrize("layout", [B.NT, B.NN, B.TN])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_layouts(dtype, layout, M, N, K):
    rng = np.random.default_rng(M + 3 * N + 7 * K + layout)
    a = store(rng.standard_normal((M, K)), dtype)
    b = store(rng.standard_normal((K, N)) * 0.1, dtype)
    ref = a.astype(np.float64) @ b.astype(np.float64)
    A = to_dev(a if layout != B.TN else a.T.copy(), dtype)
    Bm = to_dev(b.T.copy() if layout == B.NT else b, dtype)
    Cout = torch.empty(M, N, dtype=A.dtype, device=DEV)
    B.slapo_gemm(dtype, layout, B.EPI_NONE, 0, M, N, K, A, Bm, Cout)
    assert err(Cout, ref) <= {W.BF16: 5e-3, W.FP16: 1e-3}.get(dtype, 1e-5)


@pytest.mark.parametrize("dtype", [W.BF16, W.FP32, W.FP16])
@pytest.mark.parametrize("act", [W.GELU, W.RELU])
def test_gemm_epilogues(dtype, act):
    M, N, K = 392, 520, 256
    rng = np.random.default_rng(5)
    a = store(rng.standard_normal((M, K)), dtype)
    w = store(rng.standard_normal((N, K)) * 0.1, dtype)
    bias = store(rng.standard_normal(N), dtype)
    aux = store(rng.standard_normal((M, N)), dtype)
    acc = a.astype(np.float64) @ w.astype(np.float64).T
    A, Wt, bd, auxd = to_dev(a, dtype), to_dev(w, dtype), to_dev(bias, dtype), to_dev(aux, dtype)
    tol = TOL[dtype]
    Cout = torch.empty(M, N, dtype=A.dtype, device=DEV)
    U = torch.empty_like(Cout)
    B.slapo_gemm(dtype, B.NT, B.EPI_BIAS, act, M, N, K, A, Wt, Cout, bias=bd)
    assert err(Cout, acc + bias) <= tol
    B.slapo_gemm(dtype, B.NT, B.EPI_BIAS_ACT, act, M, N, K, A, Wt, Cout, bias=bd, aux_out=U)   # U receives act'(pre)
    if act == W.GELU:   # (the ReLU gate is a 0/1 decision at pre = 0 +- rounding: compared where it is decided)
        assert err(U, _dact(acc + bias, act)) <= tol
    else:
        clear = np.abs(acc + bias) > 1e-2
        assert np.array_equal(to_np(U)[clear], _dact(acc + bias, act)[clear])
    assert err(Cout, _act(acc + bias, act)) <= tol
    if act == W.RELU:   # the derivative store is optional: the gate can be read off the output
        C0 = torch.empty_like(Cout)
        B.slapo_gemm(dtype, B.NT, B.EPI_BIAS_ACT, act, M, N, K, A, Wt, C0, bias=bd)
        assert torch.equal(C0, Cout)
    B.slapo_gemm(dtype, B.NT, B.EPI_DACT, act, M, N, K, A, Wt, Cout, aux_in=auxd)
    # GeLU: C = acc * aux_in; ReLU: C = acc * [aux_in > 0], the same for aux_in = relu(u) and aux_in = relu'(u)
    assert err(Cout, acc * (aux > 0 if act == W.RELU else aux.astype(np.float64))) <= tol
    B.slapo_gemm(dtype, B.NT, B.EPI_ADD, act, M, N, K, A, Wt, Cout, aux_in=auxd)
    assert err(Cout, acc + aux) <= tol
    C2 = auxd.clone()                          # in-place accumulate (aux_in aliases C)
    B.slapo_gemm(dtype, B.NT, B.EPI_ADD, act, M, N, K, A, Wt, C2, aux_in=C2)
    assert err(C2, acc + aux) <= tol


# (M, N, K): tile-starved weight gradients that take the several-K-ranges path (4, 2 and 8 ranges, ragged edges),
# and two that must not (K too short to cut up, enough tiles)
@pytest.mark.parametrize("dtype", [W.BF16, W.FP16, W.FP32])
@pytest.mark.parametrize("M,N,K,split", [(1024, 1024, 16384, True), (136, 264, 8192, True), (264, 136, 24576, True),
                                         (1024, 1024, 4096, False), (2048, 1536, 1024, False)])
def test_weight_gradient_in_k_ranges(dtype, M, N, K, split):
    rng = np.random.default_rng(M + K)
    a = store(rng.standard_normal((K, M)), dtype)
    b = store(rng.standard_normal((K, N)) * 0.05, dtype)
    c0 = store(rng.standard_normal((M, N)), dtype)
    ref = a.astype(np.float64).T @ b.astype(np.float64)
    nbytes = B.slapo_weight_grad_workspace(dtype, M, N, K)
    assert (nbytes > 0) == (split and dtype != W.FP32)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV)
    A, Bt = to_dev(a, dtype), to_dev(b, dtype)
    out = torch.empty(M, N, dtype=A.dtype, device=DEV)
    B.slapo_weight_grad(dtype, 0, M, N, K, A, Bt, out, ws)
    tol = TOL[dtype]
    assert err(out, ref) <= tol
    ws.fill_(0x7F)                                   # stale workspace contents must not matter
    out2 = torch.empty_like(out)
    B.slapo_weight_grad(dtype, 0, M, N, K, A, Bt, out2, ws)
    assert torch.equal(out, out2)                    # bit for bit, whichever workgroup finishes first
    acc = to_dev(c0, dtype)
    B.slapo_weight_grad(dtype, 1, M, N, K, A, Bt, acc, ws)
    assert err(acc, ref + c0) <= tol
    plain = torch.empty_like(out)                    # the one-range kernel: same product, other summation order
    B.slapo_gemm(dtype, B.TN, B.EPI_NONE, 0, M, N, K, A, Bt, plain)
    assert err(plain, to_np(out)) <= tol


# Grids of 256x256 tiles that end in a thin round (272 and 289 tiles on 256 CUs, ragged edges in the second case):
# with a workspace the tiles beyond the full round are computed in several K ranges and added by a second kernel.
@pytest.mark.parametrize("dtype", [W.BF16, W.FP16])
@pytest.mark.parametrize("layout", [B.NT, B.NN, B.TN])
@pytest.mark.parametrize("M,N,K", [(4352, 4096, 2048), (4296, 4200, 3072)])
def test_thin_last_round_in_k_ranges(dtype, layout, M, N, K):
    nbytes = B.slapo_gemm_workspace(dtype, layout, B.EPI_NONE, M, N, K)
    assert nbytes > 0 and nbytes == B.slapo_gemm_workspace(dtype, layout, B.EPI_ADD, M, N, K)
    assert B.slapo_gemm_workspace(dtype, layout, B.EPI_BIAS, M, N, K) == 0          # plain and add epilogues only
    assert B.slapo_gemm_workspace(dtype, layout, B.EPI_NONE, 4096, 4096, K) == 0     # a full round: nothing to do
    assert "K ranges" in B.slapo_gemm_kernel_name(dtype, layout, B.EPI_NONE, M, N, K, flags=B.GEMM_SHARED, with_ws=1)
    rng = np.random.default_rng(M + N + K + layout)
    a = store(rng.standard_normal((M, K)), dtype)
    b = store(rng.standard_normal((K, N)) * 0.1, dtype)
    aux = store(rng.standard_normal((M, N)), dtype)
    ref = a.astype(np.float64) @ b.astype(np.float64)
    A = to_dev(a if layout != B.TN else a.T.copy(), dtype)
    Bm = to_dev(b.T.copy() if layout == B.NT else b, dtype)
    auxd = to_dev(aux, dtype)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out = torch.empty(M, N, dtype=A.dtype, device=DEV)
    B.slapo_gemm_ex(dtype, layout, B.EPI_NONE, 0, M, N, K, A, Bm, out, ws=ws, flags=B.GEMM_SHARED)
    tol = {W.BF16: 5e-3, W.FP16: 1e-3}[dtype]
    assert err(out, ref) <= tol
    ws.fill_(0x7F)                                   # stale workspace contents must not matter
    out2 = torch.empty_like(out)
    B.slapo_gemm_ex(dtype, layout, B.EPI_NONE, 0, M, N, K, A, Bm, out2, ws=ws, flags=B.GEMM_SHARED)
    assert torch.equal(out, out2)                    # bit for bit, whichever workgroup finishes first
    plain = torch.empty_like(out)                    # without a workspace: every tile in one piece
    B.slapo_gemm(dtype, layout, B.EPI_NONE, 0, M, N, K, A, Bm, plain)
    assert err(plain, to_np(out)) <= tol and not torch.equal(plain, out)   # (the tail tiles sum in another order)
    acc = auxd.clone()                               # add epilogue, in place
    B.slapo_gemm_ex(dtype, layout, B.EPI_ADD, 0, M, N, K, A, Bm, acc, aux_in=acc, ws=ws, flags=B.GEMM_SHARED)
    assert err(acc, ref + aux) <= tol
    with pytest.raises(B.SlapoError) as e:           # a workspace that is too small is refused, not half used
        B.slapo_gemm_ex(dtype, layout, B.EPI_NONE, 0, M, N, K, A, Bm, out, ws=ws[:nbytes // 2])
    assert e.value.status == -5
