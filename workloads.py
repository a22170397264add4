"""Seeded synthetic workloads shared by the tests, the benchmark and the CPU oracle's callers.

This module holds the layer shapes the measurements are quoted on and the random-input recipe.
It contains none of the layer's arithmetic: it only draws numbers and rounds them to the storage
type, so that the fp64 oracle and the HIP path can be fed the very same values.

Shapes follow the models the paper evaluates (BERT-large, OPT, GPT-Neo style layers; Table 3 and
section 5); weights and activations are synthetic stand-ins for the trained models and datasets.
"""
from __future__ import annotations

import dataclasses
import numpy as np

GELU, RELU = 0, 1
BF16, FP32, FP16 = 0, 1, 2
CLASSIC, LLAMA = 0, 1   # layer family: LayerNorm/bias/GeLU-or-ReLU layer, or RMSNorm + rotary + SwiGLU without biases


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    batch: int
    seq: int
    hidden: int
    heads: int
    ffn: int
    causal: int = 0
    dropout_p: float = 0.1
    attn_dropout_p: float = 0.0   # dropout on the attention probabilities (0 = off, the benchmark configurations)
    seed: int = 0
    dtype: int = BF16
    act: int = GELU
    pre_ln: int = 0
    layer_id: int = 0
    ln_eps: float = 1e-5
    # key-padding mask: per-sample valid length drawn uniformly in [len_lo, len_hi]; 0 = no padding mask
    len_lo: int = 0
    len_hi: int = 0
    config_id: int = 0
    n_layers: int = 1
    arch: int = CLASSIC
    attn_dim: int = 0             # heads * head_dim when it differs from hidden (one tensor-parallel rank's heads); 0 = hidden
    rope_base: float = 10000.0    # rotary base (LLAMA layers only)

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    @property
    def attn_width(self) -> int:
        return self.attn_dim or self.hidden

    @property
    def head_dim(self) -> int:
        return self.attn_width // self.heads

    def replace(self, **kw) -> "LayerConfig":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    # small fp32 encoder layer: the correctness configuration
    "C1": LayerConfig("C1-encoder-fp32", 2, 128, 256, 4, 1024, causal=0, dropout_p=0.1, dtype=FP32,
                      act=GELU, pre_ln=0, config_id=1),
    # BERT-large-shaped encoder layer, key-padding mask
    "C2": LayerConfig("C2-bert-large-layer-bf16", 8, 512, 1024, 16, 4096, causal=0, dropout_p=0.1,
                      dtype=BF16, act=GELU, pre_ln=0, len_lo=256, len_hi=512, config_id=2),
    # OPT-1.3B-shaped causal decoder layer
    "C3": LayerConfig("C3-opt-1.3b-layer-bf16", 8, 1024, 2048, 32, 8192, causal=1, dropout_p=0.1,
                      dtype=BF16, act=RELU, pre_ln=1, config_id=3),
    # GPT-Neo-2.7B-shaped causal decoder layer
    "C4": LayerConfig("C4-gptneo-2.7b-layer-bf16", 4, 2048, 2560, 20, 10240, causal=1, dropout_p=0.0,
                      dtype=BF16, act=GELU, pre_ln=1, config_id=4),
    # 24-layer BERT-large-shaped stack
    "C5": LayerConfig("C5-bert-large-24-layer-bf16", 32, 512, 1024, 16, 4096, causal=0, dropout_p=0.1,
                      dtype=BF16, act=GELU, pre_ln=0, len_lo=128, len_hi=512, config_id=5, n_layers=24),
    # LLaMA-7B-shaped decoder layer (RMSNorm, rotary, SwiGLU, no biases, no dropout), sequence length of the paper's run
    "C6": LayerConfig("C6-llama-7b-layer-bf16", 4, 1024, 4096, 32, 11008, causal=1, dropout_p=0.0,
                      dtype=BF16, pre_ln=1, ln_eps=1e-6, config_id=6, arch=LLAMA),
}

PARAM_NAMES = ("wqkv", "bqkv", "wo", "bo", "ln1_g", "ln1_b", "w1", "b1", "w2", "b2", "ln2_g", "ln2_b")
_TENSOR_IDS = {n: i for i, n in enumerate(("x", "dy", "seqlens") + PARAM_NAMES)}


LLAMA_PARAM_NAMES = ("wqkv", "wo", "ln1_g", "w1", "w2", "ln2_g")


def param_names(cfg: LayerConfig) -> tuple:
    return LLAMA_PARAM_NAMES if cfg.arch == LLAMA else PARAM_NAMES


def param_shapes(cfg: LayerConfig) -> dict:
    H, F, A = cfg.hidden, cfg.ffn, cfg.attn_width
    if cfg.arch == LLAMA:   # w1 holds gate (even rows) and up (odd rows) projections
        return {"wqkv": (3 * A, H), "wo": (H, A), "ln1_g": (H,), "w1": (2 * F, H), "w2": (H, F), "ln2_g": (H,)}
    return {"wqkv": (3 * A, H), "bqkv": (3 * A,), "wo": (H, A), "bo": (H,), "ln1_g": (H,), "ln1_b": (H,),
            "w1": (F, H), "b1": (F,), "w2": (H, F), "b2": (H,), "ln2_g": (H,), "ln2_b": (H,)}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that are already exactly representable in bf16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _rng(cfg: LayerConfig, layer_id: int, name: str) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([cfg.config_id, layer_id, _TENSOR_IDS[name]]))


def _store(cfg: LayerConfig, a: np.ndarray) -> np.ndarray:
    a = a.astype(np.float32)
    if cfg.dtype == BF16:
        a = round_to_bf16(a)
    elif cfg.dtype == FP16:
        a = a.astype(np.float16).astype(np.float32)   # IEEE half, round to nearest even
    return a


def make_params(cfg: LayerConfig, layer_id: int = 0, perturbed: bool = False) -> dict:
    """Weights ~ N(0, 0.02^2), biases 0, gamma 1, beta 0 (benchmark initialisation).

    With ``perturbed`` the biases and beta are drawn ~ N(0, 0.02^2) and gamma ~ 1 + N(0, 0.02^2), so
    that a wrong bias or gain path cannot hide behind the neutral initial values.
    Values are fp32 arrays already rounded to the storage type of ``cfg``.
    """
    out = {}
    for name, shape in param_shapes(cfg).items():
        g = _rng(cfg, layer_id, name)
        n = g.standard_normal(shape) * 0.02
        if name.startswith("w"):
            v = n
        elif name.endswith("_g"):
            v = 1.0 + n if perturbed else np.ones(shape)
        else:
            v = n if perturbed else np.zeros(shape)
        out[name] = _store(cfg, v)
    return out


def make_inputs(cfg: LayerConfig, layer_id: int = 0, q_scale: float = 1.0):
    """Returns (x, dy, seqlens): x, dy ~ N(0,1) as fp32 arrays in storage precision; seqlens int32 or None."""
    x = _store(cfg, _rng(cfg, layer_id, "x").standard_normal((cfg.batch, cfg.seq, cfg.hidden)) * q_scale)
    dy = _store(cfg, _rng(cfg, layer_id, "dy").standard_normal((cfg.batch, cfg.seq, cfg.hidden)))
    seqlens = None
    if cfg.len_hi > 0:
        seqlens = _rng(cfg, 0, "seqlens").integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.batch).astype(np.int32)
    return x, dy, seqlens


def small_config(**kw) -> LayerConfig:
    base = dict(name="small", batch=2, seq=6, hidden=8, heads=2, ffn=16, causal=0, dropout_p=0.25,
                dtype=FP32, act=GELU, pre_ln=0, config_id=99)
    base.update(kw)
    return LayerConfig(**base)
