"""The allocation-free weight gradient (slapo_weight_grad_static) against slapo_weight_grad with a workspace.

Both run the same kernels; the only difference is where the fp32 partial tiles of the K-range path live (a fixed
array inside the library instead of the caller's workspace), so the outputs must agree bit for bit. Two calls in
a row, the second on a smaller shape, so that what the first call left in the array lies under and beside what
the second one uses; then a shape that runs as one plain GEMM and touches no scratch. The workspace variant is
itself compared with the fp64 product here (and in test_gpu_gemm.py).
"""
import numpy as np
import pytest
import torch

import workloads as W
from paper_2302_08005_amd import binding as B
from gpu_util import DEV, TOL, err, store, to_dev

pytestmark = pytest.mark.gpu

# (M, N, K, K ranges expected): 4 ranges x 4 MiB, then 2 ranges of a small ragged shape, then no ranges
CALLS = [(1024, 1024, 16384, True), (136, 264, 8192, True), (2048, 1536, 1024, False)]


@pytest.mark.parametrize("dtype", [W.BF16, W.FP16])
def test_static_scratch_weight_gradient_matches_workspace_variant(dtype):
    for accumulate in (0, 1):
        for (M, N, K, split) in CALLS:
            rng = np.random.default_rng(M + K + accumulate)
            a = store(rng.standard_normal((K, M)), dtype)
            b = store(rng.standard_normal((K, N)) * 0.05, dtype)
            c0 = store(rng.standard_normal((M, N)), dtype)
            A, Bt = to_dev(a, dtype), to_dev(b, dtype)
            nbytes = B.slapo_weight_grad_workspace(dtype, M, N, K)
            assert (nbytes > 0) == split and nbytes <= 16 << 20
            ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV)
            want = to_dev(c0, dtype)
            B.slapo_weight_grad(dtype, accumulate, M, N, K, A, Bt, want, ws)
            got = to_dev(c0, dtype)
            B.slapo_weight_grad_static(dtype, accumulate, M, N, K, A, Bt, got)
            torch.cuda.synchronize()
            assert torch.equal(got, want), (accumulate, M, N, K)
            ref = a.astype(np.float64).T @ b.astype(np.float64) + (c0 if accumulate else 0.0)
            assert err(got, ref) <= TOL[dtype], (accumulate, M, N, K)
