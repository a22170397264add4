"""Host-only checks of the C ABI: the library loads, exports what the header declares, and rejects
bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2302_08005_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "slapo.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(slapo_[a-z0-9_]+)\s*\(", header))
    assert {"slapo_layer_fwd", "slapo_layer_bwd", "slapo_layer_workspace", "slapo_gemm", "slapo_attn_fwd",
            "slapo_attn_bwd", "slapo_bdrln_fwd", "slapo_bdrln_bwd", "slapo_dropout_mask"} <= names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_descriptor_validation():
    ok = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024)
    saved, scratch = B.slapo_layer_workspace(ok)
    assert saved > 0 and scratch > 0
    ck_saved, ck_scratch = B.slapo_layer_workspace(B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024, checkpoint=1))
    assert ck_saved == 0 and scratch + saved <= ck_scratch <= scratch + saved + 256   # the activations move into scratch
    bad = [
        (dict(checkpoint=2), -3), (dict(heads=5), -2), (dict(batch=0), -2), (dict(dropout_p=1.0), -2), (dict(dropout_p=-0.1), -2),
        (dict(hidden=256, heads=8), -3), (dict(hidden=16384, heads=128), -3), (dict(dtype=B.FP32, seq=5120), -3), (dict(dtype=7), -3), (dict(act=3), -3),
        (dict(ffn=1001), -4), (dict(ln_eps=0.0), -2),
    ]
    for kw, code in bad:
        base = dict(batch=2, seq=128, hidden=256, heads=4, ffn=1024)
        base.update(kw)
        with pytest.raises(B.SlapoError) as e:
            B.slapo_layer_workspace(B.make_desc(**base))
        assert e.value.status == code, (kw, e.value.status)


def test_null_and_alignment_errors_come_before_any_device_work():
    d = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024)
    lib = B.lib()
    params = B._Ptrs(**{n: 4096 for n in B.PARAM_NAMES})
    assert lib.slapo_layer_fwd(C.byref(d), C.byref(params), None, None, 4096, 4096, 4096, None) == -1
    assert lib.slapo_layer_fwd(C.byref(d), C.byref(params), 4096 + 4, None, 4096, 4096, 4096, None) == -4
    ck = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024, checkpoint=1)
    assert lib.slapo_layer_fwd(C.byref(d), C.byref(params), 4096, None, 4096, None, 4096, None) == -1    # saved is required ...
    assert lib.slapo_layer_fwd(C.byref(ck), C.byref(params), 4096 + 4, None, 4096, None, 4096, None) == -4  # ... but not when checkpointing
    params.wo = None
    assert lib.slapo_layer_fwd(C.byref(d), C.byref(params), 4096, None, 4096, 4096, 4096, None) == -1
    assert lib.slapo_gemm(0, 0, 0, 0, 128, 128, 0, 4096, 4096, 4096, None, None, None, None) == -2
    assert lib.slapo_gemm(0, 0, 1, 0, 128, 128, 64, 4096, 4096, 4096, None, None, None, None) == -1
    assert lib.slapo_gemm(0, 0, 0, 0, 128, 132, 64, 4096, 4096, 4096, None, None, None, None) == -4
    assert lib.slapo_gemm(0, 5, 0, 0, 128, 128, 64, 4096, 4096, 4096, None, None, None, None) == -3   # unknown layout
    assert lib.slapo_dropout_mask(C.byref(d), 2, 256, 4096, None) == -2
    assert B.status_string(-6).startswith("HIP")


def test_saved_regions_are_disjoint_and_inside_the_buffer():
    for pre_ln in (0, 1):
        d = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024, pre_ln=pre_ln)
        saved, _ = B.slapo_layer_workspace(d)
        names = ["qkv", "attn", "lse", "z1", "dact", "g", "mu1", "rstd1", "mu2", "rstd2"]
        names += ["n1", "n2"] if pre_ln else ["y1", "z2"]
        spans = sorted(B.slapo_layer_saved_region(d, n) for n in names)
        for (o0, b0), (o1, _) in zip(spans, spans[1:]):
            assert o0 + b0 <= o1
        assert spans[-1][0] + spans[-1][1] <= saved
        with pytest.raises(B.SlapoError):
            B.slapo_layer_saved_region(d, "y1" if pre_ln else "n1")
        # a ReLU layer keeps no derivative of its activation: [relu(u) > 0] is read off "g"
        r = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024, pre_ln=pre_ln, act=B.RELU)
        assert B.slapo_layer_workspace(r)[0] == saved - 2 * 128 * 1024 * 2
        with pytest.raises(B.SlapoError):
            B.slapo_layer_saved_region(r, "dact")


def test_stack_workspace_and_argument_checks():
    d = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024)
    saved, scratch = B.slapo_layer_workspace(d)
    acts, ssaved, sscratch = B.slapo_stack_workspace(d, 24)
    act = 2 * 128 * 256 * 2
    assert acts == 23 * act and ssaved == 24 * saved and scratch + 2 * act <= sscratch <= scratch + 2 * act + 512
    assert B.slapo_stack_workspace(d, 1)[0] == 0
    # pre-LN stacks hand the branch gradient from each layer to the one below through two more buffers
    pre = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024, pre_ln=1)
    pscratch = B.slapo_layer_workspace(pre)[1]
    assert pscratch + 4 * act <= B.slapo_stack_workspace(pre, 24)[2] <= pscratch + 4 * act + 1024
    with pytest.raises(B.SlapoError) as e:
        B.slapo_stack_workspace(d, 0)
    assert e.value.status == -2
    ck = B.make_desc(batch=2, seq=128, hidden=256, heads=4, ffn=1024, checkpoint=1)
    assert B.slapo_stack_workspace(ck, 24)[1] == 0
    lib = B.lib()
    tabs = (B._Ptrs * 2)()
    assert lib.slapo_stack_fwd(C.byref(d), 2, tabs, 4096, None, 4096, None, 4096, 4096, None) == -1   # acts missing
    assert lib.slapo_stack_fwd(C.byref(d), 2, tabs, 4096, None, 4096, 4096, 4096, 4096, None) == -1   # NULL parameters
    assert lib.slapo_stack_bwd(C.byref(d), 0, tabs, 4096, None, 4096, 4096, 4096, 4096, tabs, 4096, None) == -2


def test_llama_family_descriptor_and_pointer_checks():
    base = dict(batch=2, seq=128, hidden=256, heads=4, ffn=1024, pre_ln=1, arch=B.LLAMA)
    d = B.make_desc(**base)
    saved, scratch = B.slapo_layer_workspace(d)
    csaved, cscratch = B.slapo_layer_workspace(B.make_desc(**dict(base, arch=B.CLASSIC)))
    T, F = 2 * 128, 1024
    assert saved == csaved + T * F * 2                      # the factor pairs [T,2F] where the classic layer keeps act'(u) [T,F]
    assert scratch >= cscratch + T * F * 2 + 128 * 32 * 8   # gradient pairs [T,2F] and the (cos, sin) table
    for kw, code in [(dict(pre_ln=0), -3), (dict(rope_base=1.0), -2), (dict(rope_base=-5.0), -2), (dict(arch=2), -3)]:
        with pytest.raises(B.SlapoError) as e:
            B.slapo_layer_workspace(B.make_desc(**dict(base, **kw)))
        assert e.value.status == code, (kw, e.value.status)
    assert B.slapo_layer_saved_region(d, "dgate")[1] == 2 * T * F * 2
    with pytest.raises(B.SlapoError):
        B.slapo_layer_saved_region(d, "dact")
    lib = B.lib()
    # only the six weights and gains are required ...
    params = B._Ptrs(**{n: (4096 if n in ("wqkv", "wo", "ln1_g", "w1", "w2", "ln2_g") else None) for n in B.PARAM_NAMES})
    assert lib.slapo_layer_fwd(C.byref(d), C.byref(params), 4096 + 4, None, 4096, 4096, 4096, None) == -4   # got past the NULL checks
    params.w2 = None
    assert lib.slapo_layer_fwd(C.byref(d), C.byref(params), 4096, None, 4096, 4096, 4096, None) == -1
    # ... and the classic layer still wants all twelve
    params.w2 = 4096
    assert lib.slapo_layer_fwd(C.byref(B.make_desc(**dict(base, arch=B.CLASSIC))), C.byref(params), 4096, None, 4096, 4096, 4096, None) == -1
    # gated epilogues: the pair layout needs N % 16 == 0 and its auxiliary buffer; rotary needs a LLaMA descriptor
    assert lib.slapo_gemm(0, 0, 5, 0, 128, 136, 64, 4096, 4096, 4096, None, None, 4096, None) == -4
    assert lib.slapo_gemm(0, 0, 5, 0, 128, 128, 64, 4096, 4096, 4096, None, None, None, None) == -1
    assert lib.slapo_gemm(0, 1, 6, 0, 128, 128, 64, 4096, 4096, 4096, None, None, None, None) == -1
    assert lib.slapo_gemm(0, 0, 7, 0, 128, 128, 64, 4096, 4096, 4096, None, None, None, None) == -3
    assert lib.slapo_rope(C.byref(B.make_desc(**dict(base, arch=B.CLASSIC))), 4096, 4096, 0, None) == -3
    assert lib.slapo_rope(C.byref(d), 4096, None, 0, None) == -1


def test_attention_width_other_than_hidden():
    base = dict(batch=2, seq=128, hidden=512, heads=4, ffn=1024)
    full = B.slapo_layer_workspace(B.make_desc(**base))
    share = B.slapo_layer_workspace(B.make_desc(**dict(base, heads=2, attn_dim=256)))     # half the heads of width 128
    T = 2 * 128
    assert full[0] - share[0] == T * (3 + 1) * 256 * 2 + T * 2 * 4   # packed projection, attention output, and the lse of two heads
    d = B.make_desc(**dict(base, heads=2, attn_dim=256))
    assert B.slapo_layer_saved_region(d, "qkv")[1] == T * 3 * 256 * 2 and B.slapo_layer_saved_region(d, "attn")[1] == T * 256 * 2
    wide = B.slapo_layer_workspace(B.make_desc(**dict(base, heads=6, attn_dim=768)))
    assert wide[0] > full[0] and wide[1] > full[1]
    for kw, code in [(dict(heads=3, attn_dim=256), -2), (dict(heads=2, attn_dim=64), -3), (dict(attn_dim=-8), -2)]:
        with pytest.raises(B.SlapoError) as e:
            B.slapo_layer_workspace(B.make_desc(**dict(base, **kw)))
        assert e.value.status == code, (kw, e.value.status)


def test_weight_gradient_workspace_rule():
    assert B.slapo_weight_grad_workspace(B.BF16, 1024, 1024, 16384) == 4 * 1024 * 1024 * 4     # 64 tiles -> 4 K ranges
    assert B.slapo_weight_grad_workspace(B.BF16, 1024, 1024, 8192) == 2 * 1024 * 1024 * 4      # ranges of at least 48 slabs
    assert B.slapo_weight_grad_workspace(B.BF16, 1024, 1024, 4096) == 0                         # too short to cut up
    assert B.slapo_weight_grad_workspace(B.BF16, 128, 128, 65536) == 8 * 128 * 128 * 4          # never more than 8
    assert B.slapo_weight_grad_workspace(B.BF16, 1024, 4096, 4096) == 0                         # a full round of tiles
    assert B.slapo_weight_grad_workspace(B.BF16, 1024, 1024, 4000) == 0                         # K no multiple of 256
    assert B.slapo_weight_grad_workspace(B.FP32, 1024, 1024, 4096) == 0
    lib = B.lib()
    assert lib.slapo_weight_grad(0, 0, 1024, 1024, 16384, 4096, 4096, 4096, None, None) == -1   # wants a workspace
    assert lib.slapo_weight_grad(0, 0, 1024, 1028, 16384, 4096, 4096, 4096, 4096, None) == -4
    assert lib.slapo_weight_grad(0, 0, 0, 1024, 4096, 4096, 4096, 4096, 4096, None) == -2


def test_static_scratch_bound_and_argument_checks():
    """slapo_weight_grad_static keeps its partial tiles in a fixed 16 MiB array: the K-range rule never asks for more
    (at most 256 partial tiles of 128 x 128 floats), and its argument checks come before any device work."""
    lib = B.lib()
    worst = 0
    for M in (8, 136, 1024, 1536, 2048, 2560, 4096, 12288):
        for N in (8, 264, 1024, 1280, 2560, 4096):
            for K in (256, 4096, 8192, 16384, 65536):
                if M * K < 2 ** 31 and N * K < 2 ** 31:
                    worst = max(worst, B.slapo_weight_grad_workspace(B.BF16, M, N, K))
    assert 0 < worst <= 16 << 20
    assert lib.slapo_weight_grad_static(0, 0, 1024, 1024, 16384, None, 4096, 4096, None) == -1
    assert lib.slapo_weight_grad_static(0, 0, 1024, 1024, 16384, 4096 + 2, 4096, 4096, None) == -4
    assert lib.slapo_weight_grad_static(0, 0, 1024, 1020, 16384, 4096, 4096, 4096, None) == -4
    assert lib.slapo_weight_grad_static(0, 0, 0, 1024, 16384, 4096, 4096, 4096, None) == -2
    assert lib.slapo_weight_grad_static(9, 0, 1024, 1024, 16384, 4096, 4096, 4096, None) == -3


def test_gemm_workspace_rules_on_the_host():
    """The K-range treatment of thin last rounds: which shapes ask for a workspace, and the too-small refusal."""
    lib = B.lib()
    # 8192 x 2560 outputs are 320 tiles of 256 x 256: 64 tail tiles in 4 K ranges when K is long ...
    assert B.slapo_gemm_workspace(B.BF16, B.NN, B.EPI_NONE, 8192, 2560, 10240) == 64 * 4 * 256 * 256 * 4
    assert "256 tiles + 64 tiles in 4 K ranges" in B.slapo_gemm_kernel_name(B.BF16, B.NN, B.EPI_NONE, 8192, 2560, 10240, flags=B.GEMM_SHARED, with_ws=1)
    # ... nothing for short K (the partial tiles would cost more than the thin round), full rounds, other epilogues, fp32
    assert B.slapo_gemm_workspace(B.BF16, B.NN, B.EPI_NONE, 8192, 2560, 1024) == 0
    assert B.slapo_gemm_workspace(B.BF16, B.NT, B.EPI_NONE, 8192, 2048, 8192) == 0
    assert B.slapo_gemm_workspace(B.BF16, B.NT, B.EPI_BIAS_ACT, 8192, 2560, 10240) == 0
    assert B.slapo_gemm_workspace(B.FP32, B.NN, B.EPI_NONE, 8192, 2560, 10240) == 0
    need = B.slapo_gemm_workspace(B.BF16, B.NN, B.EPI_NONE, 8192, 2560, 10240)
    args = (0, 1, 0, 0, 8192, 2560, 10240, 4096, 4096, 4096, None, None, None, 0)
    assert lib.slapo_gemm_ex(*args, 4096, need - 16, None) == -5      # before any device work
    assert lib.slapo_gemm_ex(*args, 4096 + 8, need, None) == -4
    assert lib.slapo_gemm_ex(*args[:13], 2, 4096, need, None) == -3   # unknown flag
    assert B.status_string(-5).startswith("shape needs more workspace")


def test_debug_switches_shrink_the_reported_workspaces():
    """SLAPO_DEBUG is read once per process: a child with the switches set reports no K-range workspaces."""
    import subprocess
    import sys
    code = ("from paper_2302_08005_amd import binding as B; import workloads as W; "
            "print(B.slapo_weight_grad_workspace(W.BF16, 1024, 1024, 16384), "
            "B.slapo_gemm_workspace(W.BF16, B.NN, B.EPI_NONE, 4352, 4096, 2048))")
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    def run(debug):
        env = dict(os.environ, SLAPO_DEBUG=debug)
        out = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, check=True)
        return [int(x) for x in out.stdout.split()]
    wg, hyb = run("")
    assert wg > 0 and hyb > 0
    assert run("no-splitk,no-hybrid") == [0, 0]
    assert run("no-splitk") == [0, hyb]
