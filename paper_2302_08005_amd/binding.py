"""ctypes binding of libslapo_mi355x.so: same entry-point names as include/slapo.h, arguments
marshalled from torch tensors (used for device memory and streams only). No arithmetic here."""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SLAPO_LIB", os.path.join(HERE, "libslapo_mi355x.so"))

BF16, FP32, FP16 = 0, 1, 2
GELU, RELU = 0, 1
NT, NN, TN = 0, 1, 2
EPI_NONE, EPI_BIAS, EPI_BIAS_ACT, EPI_DACT, EPI_ADD, EPI_GATE, EPI_DGATE = 0, 1, 2, 3, 4, 5, 6
CLASSIC, LLAMA = 0, 1
PARAM_NAMES = ("wqkv", "bqkv", "wo", "bo", "ln1_g", "ln1_b", "w1", "b1", "w2", "b2", "ln2_g", "ln2_b")


class LayerDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32),
                ("ffn", C.c_int32), ("causal", C.c_int32), ("dropout_p", C.c_float), ("seed", C.c_uint64),
                ("dtype", C.c_int32), ("act", C.c_int32), ("pre_ln", C.c_int32), ("layer_id", C.c_int32),
                ("ln_eps", C.c_float), ("accumulate_grads", C.c_int32), ("checkpoint", C.c_int32), ("attn_dropout_p", C.c_float),
                ("arch", C.c_int32), ("rope_base", C.c_float), ("attn_dim", C.c_int32)]


class _Ptrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class SlapoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib():
    """Loads the HIP library; there is no fallback if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        L.slapo_status_string.restype = C.c_char_p
        L.slapo_status_string.argtypes = [C.c_int]
        vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
        dp = C.POINTER(LayerDesc)
        sigs = {
            "slapo_layer_workspace": [dp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)],
            "slapo_layer_saved_region": [dp, C.c_char_p, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)],
            "slapo_layer_fwd": [dp, C.POINTER(_Ptrs), vp, vp, vp, vp, vp, vp],
            "slapo_layer_bwd": [dp, C.POINTER(_Ptrs), vp, vp, vp, vp, vp, C.POINTER(_Ptrs), vp, vp],
            "slapo_stack_workspace": [dp, i32, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)],
            "slapo_stack_fwd": [dp, i32, C.POINTER(_Ptrs), vp, vp, vp, vp, vp, vp, vp],
            "slapo_stack_bwd": [dp, i32, C.POINTER(_Ptrs), vp, vp, vp, vp, vp, vp, C.POINTER(_Ptrs), vp, vp],
            "slapo_gemm": [i32, i32, i32, i32, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp],
            "slapo_gemm_ex": [i32, i32, i32, i32, i64, i64, i64, vp, vp, vp, vp, vp, vp, i32, vp, C.c_size_t, vp],
            "slapo_gemm_workspace": [i32, i32, i32, i64, i64, i64, C.POINTER(C.c_size_t)],
            "slapo_gemm_kernel_name": [i32, i32, i32, i64, i64, i64, i32, i32, i32, C.c_char_p, C.c_size_t],
            "slapo_attn_fwd": [dp, vp, vp, vp, vp, vp],
            "slapo_attn_bwd": [dp, vp, vp, vp, vp, vp, vp, vp, vp],
            "slapo_bdrln_fwd": [dp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp],
            "slapo_bdrln_bwd": [dp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp],
            "slapo_bdrln_bwd_blocks": [i64],
            "slapo_colsum_partials": [i32, i64, i64, vp, vp, vp],
            "slapo_colsum_blocks": [i64],
            "slapo_colreduce_partials": [i32, i64, i64, i64, vp, vp, i32, vp],
            "slapo_dropout_mask": [dp, i32, i64, vp, vp],
            "slapo_rope": [dp, vp, vp, i32, vp],
            "slapo_weight_grad_workspace": [i32, i64, i64, i64, C.POINTER(C.c_size_t)],
            "slapo_weight_grad": [i32, i32, i64, i64, i64, vp, vp, vp, vp, vp],
            "slapo_weight_grad_static": [i32, i32, i64, i64, i64, vp, vp, vp, vp],
        }
        for name, args in sigs.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().slapo_status_string(int(status)).decode()


def _check(rc, where):
    if rc != 0:
        raise SlapoError(rc, where)


def _p(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def make_desc(cfg=None, **kw) -> LayerDesc:
    """Builds a descriptor from a workloads.LayerConfig-like object and/or keyword overrides."""
    vals = dict(batch=1, seq=1, hidden=64, heads=1, ffn=64, causal=0, dropout_p=0.0, seed=0, dtype=BF16, act=GELU,
                pre_ln=0, layer_id=0, ln_eps=1e-5, accumulate_grads=0, checkpoint=0, attn_dropout_p=0.0,
                arch=CLASSIC, rope_base=10000.0, attn_dim=0)
    if cfg is not None:
        for k in vals:
            if hasattr(cfg, k):
                vals[k] = getattr(cfg, k)
    vals.update(kw)
    return LayerDesc(**vals)


def torch_dtype(desc: LayerDesc):
    return {FP32: torch.float32, FP16: torch.float16}.get(desc.dtype, torch.bfloat16)


def slapo_layer_workspace(desc: LayerDesc):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib().slapo_layer_workspace(C.byref(desc), C.byref(a), C.byref(b)), "slapo_layer_workspace")
    return a.value, b.value


def slapo_layer_saved_region(desc: LayerDesc, name: str):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib().slapo_layer_saved_region(C.byref(desc), name.encode(), C.byref(a), C.byref(b)),
           "slapo_layer_saved_region")
    return a.value, b.value


def _ptr_table(tensors: dict) -> _Ptrs:
    return _Ptrs(**{n: _p(tensors.get(n)) for n in PARAM_NAMES})   # entries a layer family does not have stay NULL


def slapo_layer_fwd(desc, params: dict, x, seqlens, y, saved, scratch, stream=None):
    pt = _ptr_table(params)
    _check(lib().slapo_layer_fwd(C.byref(desc), C.byref(pt), _p(x), _p(seqlens), _p(y), _p(saved), _p(scratch),
                                 _stream(stream)), "slapo_layer_fwd")


def slapo_layer_bwd(desc, params: dict, x, seqlens, dy, saved, dx, grads: dict, scratch, stream=None):
    pt, gt = _ptr_table(params), _ptr_table(grads)
    _check(lib().slapo_layer_bwd(C.byref(desc), C.byref(pt), _p(x), _p(seqlens), _p(dy), _p(saved), _p(dx),
                                 C.byref(gt), _p(scratch), _stream(stream)), "slapo_layer_bwd")


def slapo_gemm(dtype, layout, epilogue, act, M, N, K, A, B, Cout, bias=None, aux_in=None, aux_out=None, stream=None):
    _check(lib().slapo_gemm(dtype, layout, epilogue, act, M, N, K, _p(A), _p(B), _p(Cout), _p(bias), _p(aux_in),
                            _p(aux_out), _stream(stream)), "slapo_gemm")


GEMM_SHARED = 1


def slapo_gemm_workspace(dtype, layout, epilogue, M, N, K) -> int:
    a = C.c_size_t(0)
    _check(lib().slapo_gemm_workspace(dtype, layout, epilogue, M, N, K, C.byref(a)), "slapo_gemm_workspace")
    return a.value


def slapo_gemm_ex(dtype, layout, epilogue, act, M, N, K, A, B, Cout, bias=None, aux_in=None, aux_out=None, flags=0, ws=None,
                  stream=None):
    _check(lib().slapo_gemm_ex(dtype, layout, epilogue, act, M, N, K, _p(A), _p(B), _p(Cout), _p(bias), _p(aux_in),
                               _p(aux_out), flags, _p(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                               _stream(stream)), "slapo_gemm_ex")


def slapo_gemm_kernel_name(dtype, layout, epilogue, M, N, K, flags=0, weight_grad=0, with_ws=0) -> str:
    buf = C.create_string_buffer(320)
    _check(lib().slapo_gemm_kernel_name(dtype, layout, epilogue, M, N, K, flags, weight_grad, with_ws, buf, len(buf)),
           "slapo_gemm_kernel_name")
    return buf.value.decode()


def slapo_weight_grad_workspace(dtype, M, N, K) -> int:
    a = C.c_size_t(0)
    _check(lib().slapo_weight_grad_workspace(dtype, M, N, K, C.byref(a)), "slapo_weight_grad_workspace")
    return a.value


def slapo_weight_grad(dtype, accumulate, M, N, K, A, B, Cout, ws=None, stream=None):
    _check(lib().slapo_weight_grad(dtype, accumulate, M, N, K, _p(A), _p(B), _p(Cout), _p(ws), _stream(stream)),
           "slapo_weight_grad")


def slapo_weight_grad_static(dtype, accumulate, M, N, K, A, B, Cout, stream=None):
    _check(lib().slapo_weight_grad_static(dtype, accumulate, M, N, K, _p(A), _p(B), _p(Cout), _stream(stream)),
           "slapo_weight_grad_static")


def slapo_attn_fwd(desc, qkv, seqlens, out, lse, stream=None):
    _check(lib().slapo_attn_fwd(C.byref(desc), _p(qkv), _p(seqlens), _p(out), _p(lse), _stream(stream)),
           "slapo_attn_fwd")


def slapo_attn_bwd(desc, qkv, seqlens, out, dout, lse, delta, dqkv, stream=None):
    _check(lib().slapo_attn_bwd(C.byref(desc), _p(qkv), _p(seqlens), _p(out), _p(dout), _p(lse), _p(delta),
                                _p(dqkv), _stream(stream)), "slapo_attn_bwd")


def slapo_bdrln_fwd(desc, site, T, r, bias, res, gamma, beta, z_out, out, mu, rstd, stream=None):
    _check(lib().slapo_bdrln_fwd(C.byref(desc), site, T, _p(r), _p(bias), _p(res), _p(gamma), _p(beta), _p(z_out),
                                 _p(out), _p(mu), _p(rstd), _stream(stream)), "slapo_bdrln_fwd")


def slapo_bdrln_bwd_blocks(T) -> int:
    return lib().slapo_bdrln_bwd_blocks(T)


def slapo_bdrln_bwd(desc, site, T, dout, z, mu, rstd, gamma, dres_in, dz_out, dr_out, partials, stream=None):
    _check(lib().slapo_bdrln_bwd(C.byref(desc), site, T, _p(dout), _p(z), _p(mu), _p(rstd), _p(gamma), _p(dres_in),
                                 _p(dz_out), _p(dr_out), _p(partials), _stream(stream)), "slapo_bdrln_bwd")


def slapo_colsum_blocks(T) -> int:
    return lib().slapo_colsum_blocks(T)


def slapo_colsum_partials(dtype, T, N, a, partials, stream=None):
    _check(lib().slapo_colsum_partials(dtype, T, N, _p(a), _p(partials), _stream(stream)), "slapo_colsum_partials")


def slapo_colreduce_partials(dtype, nblk, stride, N, partials, out, accumulate=0, stream=None):
    _check(lib().slapo_colreduce_partials(dtype, nblk, stride, N, _p(partials), _p(out), accumulate,
                                          _stream(stream)), "slapo_colreduce_partials")


def slapo_dropout_mask(desc, site, T, mask, stream=None):
    _check(lib().slapo_dropout_mask(C.byref(desc), site, T, _p(mask), _stream(stream)), "slapo_dropout_mask")


def slapo_rope(desc, qkv, table, inverse=0, stream=None):
    _check(lib().slapo_rope(C.byref(desc), _p(qkv), _p(table), inverse, _stream(stream)), "slapo_rope")


def slapo_stack_workspace(desc: LayerDesc, n_layers: int):
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(lib().slapo_stack_workspace(C.byref(desc), n_layers, C.byref(a), C.byref(b), C.byref(c)),
           "slapo_stack_workspace")
    return a.value, b.value, c.value


def _ptr_tables(layers: list):
    arr = (_Ptrs * len(layers))()
    for i, t in enumerate(layers):
        arr[i] = _ptr_table(t)
    return arr


def slapo_stack_fwd(desc, params: list, x, seqlens, y, acts, saved, scratch, stream=None):
    _check(lib().slapo_stack_fwd(C.byref(desc), len(params), _ptr_tables(params), _p(x), _p(seqlens), _p(y), _p(acts),
                                 _p(saved), _p(scratch), _stream(stream)), "slapo_stack_fwd")


def slapo_stack_bwd(desc, params: list, x, seqlens, dy, acts, saved, dx, grads: list, scratch, stream=None):
    _check(lib().slapo_stack_bwd(C.byref(desc), len(params), _ptr_tables(params), _p(x), _p(seqlens), _p(dy), _p(acts),
                                 _p(saved), _p(dx), _ptr_tables(grads), _p(scratch), _stream(stream)), "slapo_stack_bwd")


class Stack:
    """Convenience holder for a stack of layers of one shape: per-layer parameters and gradients, shared workspaces."""

    def __init__(self, cfg, params_np: list, device="cuda:0", **desc_kw):
        self.desc = make_desc(cfg, **desc_kw)
        self.device = torch.device(device)
        self.dt = torch_dtype(self.desc)
        self.params = [{k: torch.from_numpy(v).to(self.device).to(self.dt).contiguous() for k, v in p.items()}
                       for p in params_np]
        self.grads = [{k: torch.zeros_like(v) for k, v in p.items()} for p in self.params]
        ab, sb, wb = slapo_stack_workspace(self.desc, len(self.params))
        mk = lambda n: torch.empty(n, dtype=torch.uint8, device=self.device) if n else None
        self.acts, self.saved, self.scratch = mk(ab), mk(sb), mk(wb)

    def to_device(self, a_np):
        return torch.from_numpy(a_np).to(self.device).to(self.dt).contiguous()

    def forward(self, x, seqlens=None):
        y = torch.empty_like(x)
        slapo_stack_fwd(self.desc, self.params, x, seqlens, y, self.acts, self.saved, self.scratch)
        return y

    def backward(self, x, seqlens, dy):
        dx = torch.empty_like(x)
        slapo_stack_bwd(self.desc, self.params, x, seqlens, dy, self.acts, self.saved, dx, self.grads, self.scratch)
        return dx


class Layer:
    """Convenience holder: device parameters, gradients and the two workspaces of one layer."""

    def __init__(self, cfg, params_np: dict, device="cuda:0", **desc_kw):
        self.desc = make_desc(cfg, **desc_kw)
        self.device = torch.device(device)
        self.dt = torch_dtype(self.desc)
        self.params = {k: torch.from_numpy(v).to(self.device).to(self.dt).contiguous() for k, v in params_np.items()}
        self.grads = {k: torch.zeros_like(v) for k, v in self.params.items()}
        sb, wb = slapo_layer_workspace(self.desc)
        self.saved = torch.empty(sb, dtype=torch.uint8, device=self.device) if sb else None   # None: checkpoint mode
        self.scratch = torch.empty(wb, dtype=torch.uint8, device=self.device)

    def to_device(self, a_np):
        return torch.from_numpy(a_np).to(self.device).to(self.dt).contiguous()

    def forward(self, x, seqlens=None):
        y = torch.empty_like(x)
        slapo_layer_fwd(self.desc, self.params, x, seqlens, y, self.saved, self.scratch)
        return y

    def backward(self, x, seqlens, dy):
        dx = torch.empty_like(x)
        slapo_layer_bwd(self.desc, self.params, x, seqlens, dy, self.saved, dx, self.grads, self.scratch)
        return dx

    def saved_tensor(self, name):
        off, nbytes = slapo_layer_saved_region(self.desc, name)
        raw = self.saved[off:off + nbytes]
        if name in ("lse", "mu1", "rstd1", "mu2", "rstd2"):
            return raw.view(torch.float32)
        return raw.view(self.dt)
