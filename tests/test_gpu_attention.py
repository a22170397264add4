"""GPU parity of the fused attention forward / backward vs the oracle's materialised S x S attention."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import layer as L
from paper_2302_08005_amd import binding as B
from gpu_util import DEV, TOL, err, store, to_dev

pytestmark = pytest.mark.gpu

CASES = [
    # batch, seq, heads, d, causal, seqlens, q_scale
    (2, 128, 2, 64, 0, None, 1.0),
    (2, 200, 2, 64, 1, None, 1.0),            # ragged: not a multiple of the 128-row tile
    (3, 320, 2, 64, 0, [320, 1, 130], 1.0),   # padding mask incl. a single visible key
    (2, 256, 3, 64, 1, [256, 77], 8.0),       # causal + padding, large scores (online-softmax rescaling)
    (1, 384, 2, 128, 1, None, 1.0),
    (2, 136, 1, 128, 0, [100, 136], 4.0),
    # d = 128 with mask-free and boundary tiles side by side (the dK/dV kernel pipelines the mask-free ones by hand):
    # ragged length, causal + padding; and a bidirectional one whose tiles are all mask-free
    (2, 456, 2, 128, 1, [456, 300], 2.0),
    (2, 320, 1, 128, 0, None, 1.0),
    # a long sequence (65 key tiles), ragged, causal + padding
    (1, 4160, 1, 64, 1, [3000], 1.0),
    # with dropout on the attention probabilities (last entry): plain, causal + padding, d = 128 causal, padding
    (2, 128, 2, 64, 0, None, 1.0, 0.2),
    (2, 256, 3, 64, 1, [256, 77], 4.0, 0.1),
    (1, 384, 2, 128, 1, None, 1.0, 0.3),
    (3, 320, 2, 64, 0, [320, 8, 130], 1.0, 0.25),
]


@pytest.mark.parametrize("dtype", [W.BF16, W.FP32, W.FP16])
@pytest.mark.parametrize("case", CASES)
def test_attention_fwd_bwd(dtype, case):
    Bt, S, h, d, causal, sl, qs = case[:7]
    pd = case[7] if len(case) > 7 else 0.0
    H = h * d
    cfg = W.LayerConfig("t", Bt, S, H, h, 64, causal=causal, dtype=dtype, attn_dropout_p=pd,
                        seed=0x5EED0000ABCD1234 if pd else 0, layer_id=3 if pd else 0)
    rng = np.random.default_rng(S + d + causal)
    qkv = rng.standard_normal((Bt * S, 3 * H))
    qkv[:, :H] *= qs
    qkv = store(qkv, dtype)
    dout = store(rng.standard_normal((Bt * S, H)), dtype)
    sl_np = None if sl is None else np.array(sl, dtype=np.int32)
    A_ref, P, LSE_ref = L.attention_fwd(cfg, qkv.astype(np.float64), sl_np)
    desc = B.make_desc(cfg)
    sl_d = None if sl is None else torch.from_numpy(sl_np).to(DEV)
    qkv_d = to_dev(qkv, dtype)
    out = torch.empty(Bt * S, H, dtype=qkv_d.dtype, device=DEV)
    lse = torch.empty(Bt, h, S, dtype=torch.float32, device=DEV)
    B.slapo_attn_fwd(desc, qkv_d, sl_d, out, lse)
    tol = TOL[dtype]
    assert err(out, A_ref) <= tol
    assert err(lse, LSE_ref) <= (1e-5 if dtype == W.FP32 else 2e-3)
    # backward on the oracle's (stored) forward output
    A_s = store(A_ref, dtype)
    dqkv_ref = L.attention_bwd(cfg, qkv.astype(np.float64), P, dout.astype(np.float64))
    delta = torch.empty(Bt, h, S, dtype=torch.float32, device=DEV)
    dqkv = torch.full((Bt * S, 3 * H), float("nan"), dtype=qkv_d.dtype, device=DEV)
    B.slapo_attn_bwd(desc, qkv_d, sl_d, to_dev(A_s, dtype), to_dev(dout, dtype),
                     torch.from_numpy(LSE_ref.astype(np.float32)).to(DEV), delta, dqkv)
    for i, name in enumerate(("dq", "dk", "dv")):
        assert err(dqkv[:, i * H:(i + 1) * H], dqkv_ref[:, i * H:(i + 1) * H]) <= tol, name


@pytest.mark.parametrize("dtype", [W.BF16, W.FP32, W.FP16])
@pytest.mark.parametrize("causal", [0, 1])
def test_sample_without_visible_keys_yields_zeros_not_nans(dtype, causal):
    """Outside the documented precondition (len >= 1) the kernels still behave: a sample whose length is 0 gets
    zero output, -inf logsumexp and zero gradients, and leaves its neighbours untouched."""
    Bt, S, h, d = 3, 136, 2, 64
    H = h * d
    cfg = W.LayerConfig("t", Bt, S, H, h, 64, causal=causal, dtype=dtype)
    rng = np.random.default_rng(11)
    qkv = store(rng.standard_normal((Bt * S, 3 * H)), dtype)
    dout = store(rng.standard_normal((Bt * S, H)), dtype)
    sl = np.array([S, 0, 70], dtype=np.int32)
    desc = B.make_desc(cfg)
    qkv_d, sl_d = to_dev(qkv, dtype), torch.from_numpy(sl).to(DEV)
    out = torch.full((Bt * S, H), float("nan"), dtype=qkv_d.dtype, device=DEV)
    lse = torch.full((Bt, h, S), float("nan"), dtype=torch.float32, device=DEV)
    B.slapo_attn_fwd(desc, qkv_d, sl_d, out, lse)
    assert torch.isfinite(out).all() and (out[S:2 * S] == 0).all() and torch.isneginf(lse[1]).all()
    # the other two samples equal a run in which the empty one is given a length
    ok = np.array([S, 5, 70], dtype=np.int32)
    A_ref, P, LSE_ref = L.attention_fwd(cfg, qkv.astype(np.float64), ok)
    keep = np.r_[0:S, 2 * S:3 * S]
    assert err(out[keep], A_ref[keep]) <= TOL[dtype]
    delta = torch.empty(Bt, h, S, dtype=torch.float32, device=DEV)
    dqkv = torch.full((Bt * S, 3 * H), float("nan"), dtype=qkv_d.dtype, device=DEV)
    B.slapo_attn_bwd(desc, qkv_d, sl_d, out, to_dev(dout, dtype), lse, delta, dqkv)
    assert torch.isfinite(dqkv).all() and (dqkv[S:2 * S] == 0).all()
    dqkv_ref = L.attention_bwd(cfg, qkv.astype(np.float64), P, dout.astype(np.float64))
    assert err(dqkv[keep], dqkv_ref[keep]) <= TOL[dtype]
