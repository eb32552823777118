"""Seeded synthetic inputs for the Transformer-encoder-layer workloads.

This module only produces data (shapes, value distributions, rounding of the
inputs to the storage type).  It holds none of the layer's arithmetic and is
imported by the tests and the benchmark, never by the oracle or the HIP
binding, which both take plain arrays.

The workloads stand in for the BERT-like, ASR-Transformer and ViT rows of the
paper's performance table (Section 5.1.2, Table 3): the paper states neither
layer dimensions nor sequence lengths, so the shapes are the five synthetic
configurations listed below.

Draw order for a seed (fixed so that every consumer sees the same arrays):
X, Wq, Wk, Wv, Wo, W1, W2, lengths, dY, then -- only for ``nontrivial=True``
-- bqkv, bo, b1, b2, ln1_g, ln1_b, ln2_g, ln2_b.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

PARAM_NAMES = ("Wqkv", "bqkv", "Wo", "bo", "W1", "b1", "W2", "b2",
               "ln1_g", "ln1_b", "ln2_g", "ln2_b")


@dataclass(frozen=True)
class LayerConfig:
    name: str
    B: int
    T: int
    D: int          # d_model
    H: int          # heads
    F: int          # d_ffn
    act: str        # "relu" | "gelu"
    norm: str       # "post" | "pre"
    dtype: str      # "f32" | "bf16" (bf16 storage, fp32 accumulate)
    init: str       # "xavier" | "normal0.02"
    len_lo: int = 0  # key-padding lengths uniform integers in [len_lo, len_hi]; 0 = no mask
    len_hi: int = 0
    layers: int = 1
    eps: float = 1e-5
    causal: bool = False   # query i attends to keys j <= i only (autoregressive variant)

    @property
    def M(self) -> int:
        return self.B * self.T

    @property
    def dh(self) -> int:
        return self.D // self.H

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


CONFIGS = {
    "cfg1_tiny_f32": LayerConfig("cfg1_tiny_f32", 2, 16, 64, 4, 256, "relu", "post", "f32", "xavier"),
    "cfg2_small_f32": LayerConfig("cfg2_small_f32", 8, 128, 256, 4, 1024, "relu", "post", "f32", "xavier"),
    "cfg3_bert_base_bf16": LayerConfig("cfg3_bert_base_bf16", 32, 128, 768, 12, 3072, "gelu", "post",
                                       "bf16", "normal0.02", 64, 128),
    "cfg4_speech_bf16": LayerConfig("cfg4_speech_bf16", 8, 1000, 768, 4, 3072, "relu", "post",
                                    "bf16", "normal0.02", 500, 1000),
    "cfg5_vit_b16_bf16": LayerConfig("cfg5_vit_b16_bf16", 64, 197, 768, 12, 3072, "gelu", "pre",
                                     "bf16", "normal0.02", 0, 0, layers=12),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already exactly representable in bf16."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def _weight(rng, cfg: LayerConfig, fan_out: int, fan_in: int) -> np.ndarray:
    if cfg.init == "xavier":
        a = np.sqrt(6.0 / (fan_in + fan_out))
        return rng.uniform(-a, a, size=(fan_out, fan_in)).astype(np.float32)
    return (0.02 * rng.standard_normal((fan_out, fan_in))).astype(np.float32)


def make_layer_params(rng, cfg: LayerConfig) -> dict:
    """The seven weight draws of one layer, in the fixed order; trivial biases / LayerNorm affine."""
    D, F = cfg.D, cfg.F
    Wq = _weight(rng, cfg, D, D)
    Wk = _weight(rng, cfg, D, D)
    Wv = _weight(rng, cfg, D, D)
    p = {
        "Wqkv": np.concatenate([Wq, Wk, Wv], axis=0),
        "Wo": _weight(rng, cfg, D, D),
        "W1": _weight(rng, cfg, F, D),
        "W2": _weight(rng, cfg, D, F),
        "bqkv": np.zeros(3 * D, np.float32), "bo": np.zeros(D, np.float32),
        "b1": np.zeros(F, np.float32), "b2": np.zeros(D, np.float32),
        "ln1_g": np.ones(D, np.float32), "ln1_b": np.zeros(D, np.float32),
        "ln2_g": np.ones(D, np.float32), "ln2_b": np.zeros(D, np.float32),
    }
    return p


def _nontrivial_affine(rng, cfg: LayerConfig, p: dict) -> None:
    D, F = cfg.D, cfg.F
    p["bqkv"] = (0.02 * rng.standard_normal(3 * D)).astype(np.float32)
    p["bo"] = (0.02 * rng.standard_normal(D)).astype(np.float32)
    p["b1"] = (0.02 * rng.standard_normal(F)).astype(np.float32)
    p["b2"] = (0.02 * rng.standard_normal(D)).astype(np.float32)
    p["ln1_g"] = (1.0 + 0.1 * rng.standard_normal(D)).astype(np.float32)
    p["ln1_b"] = (0.1 * rng.standard_normal(D)).astype(np.float32)
    p["ln2_g"] = (1.0 + 0.1 * rng.standard_normal(D)).astype(np.float32)
    p["ln2_b"] = (0.1 * rng.standard_normal(D)).astype(np.float32)


def make_inputs(cfg: LayerConfig, seed: int = 0, nontrivial: bool = False) -> dict:
    """Inputs of a single-layer workload.

    Returns float32 arrays ``X`` [B,T,D], ``dY`` [B,T,D], ``params`` (dict of
    the 12 parameter arrays), and ``lengths`` (int32 [B]) or None.  For bf16
    configurations every floating-point array is rounded to bf16 first, so the
    oracle and the GPU path consume identical values.
    """
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((cfg.B, cfg.T, cfg.D)).astype(np.float32)
    p = make_layer_params(rng, cfg)
    lengths = None
    if cfg.len_hi > 0:
        lengths = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
    dY = rng.standard_normal((cfg.B, cfg.T, cfg.D)).astype(np.float32)
    if nontrivial:
        _nontrivial_affine(rng, cfg, p)
    if cfg.dtype == "bf16":
        X, dY = round_to_bf16(X), round_to_bf16(dY)
        p = {k: round_to_bf16(v) for k, v in p.items()}
    return {"X": X, "dY": dY, "params": p, "lengths": lengths}


def make_stack_inputs(cfg: LayerConfig, seed: int = 0, nontrivial: bool = False) -> dict:
    """Inputs of an L-layer stack: X, then L parameter sets in layer order, then dY."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((cfg.B, cfg.T, cfg.D)).astype(np.float32)
    plist = []
    for _ in range(cfg.layers):
        p = make_layer_params(rng, cfg)
        if nontrivial:
            _nontrivial_affine(rng, cfg, p)
        plist.append(p)
    lengths = None
    if cfg.len_hi > 0:
        lengths = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
    dY = rng.standard_normal((cfg.B, cfg.T, cfg.D)).astype(np.float32)
    if cfg.dtype == "bf16":
        X, dY = round_to_bf16(X), round_to_bf16(dY)
        plist = [{k: round_to_bf16(v) for k, v in p.items()} for p in plist]
    return {"X": X, "dY": dY, "params": plist, "lengths": lengths}


def layer_flops(cfg: LayerConfig, lengths=None) -> dict:
    """Algorithmic flop counts of one layer (multiply-add = 2 flops).

    Linear part forward: M(8D^2 + 4DF).  Attention forward: 4*D*(number of
    (query, allowed key) pairs): sum_b T*len_b, or with the causal mask
    sum_b sum_i min(len_b, i+1).  Forward+backward is three times the forward count.
    """
    M, D, F = cfg.M, cfg.D, cfg.F
    lin = M * (8 * D * D + 4 * D * F)
    lens = np.full(cfg.B, cfg.T, np.int64) if lengths is None else np.asarray(lengths, np.int64)
    if cfg.causal:
        pairs = int(sum(np.minimum(n, np.arange(1, cfg.T + 1)).sum() for n in lens))
    else:
        pairs = int(cfg.T * lens.sum())
    attn = 4 * D * pairs
    return {"fwd_linear": lin, "fwd_attn": attn, "fwd": lin + attn, "fwd_bwd": 3 * (lin + attn)}
