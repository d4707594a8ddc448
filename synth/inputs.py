"""Seeded synthetic inputs for the decoder-layer training step.

This module only draws random numbers and rounds them to bf16; it contains none
of the layer's arithmetic.  Both the fp64 oracle and the GPU tests consume the
bf16 values produced here (the oracle upcasts them to fp64, which is exact).

Recipe: NumPy Generator(PCG64(seed)), tensors drawn as fp32 in a fixed order
(x, dy, g_attn, wq, wk, wv, wo, g_mlp, w_gate, w_up, w_down), each rounded to
bf16 with round-to-nearest-even.  Activations and upstream gradient ~N(0,1),
projection weights ~N(0, 0.02^2), norm gains 1 + 0.02*N(0,1).  These tensors
stand in for tokenised web text and trained weights, which dense kernels do not
depend on for throughput and which parity against the oracle does not need.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict, replace

import numpy as np

VOCAB_8B = 128256


@dataclass(frozen=True)
class LayerConfig:
    batch: int
    seq: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    rope_layout: int = 0  # 0: pairs (i, i + dh/2); 1: pairs (2i, 2i+1)
    recompute: int = 0    # library option (which activations the backward rebuilds); no effect on the mathematics

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)

    def asdict(self):
        return asdict(self)


# The five workload shapes: tiny, small, 1B-scale, 8B-shaped, and the layer of
# the 8B-shaped 4-layer stack (batch 1).
CONFIGS = {
    "tiny": LayerConfig(1, 128, 128, 4, 4, 32, 384, 1e-5, 10000.0),
    "small": LayerConfig(8, 1024, 768, 12, 12, 64, 2048, 1e-5, 10000.0),
    "1b": LayerConfig(4, 2048, 2048, 16, 8, 128, 5632, 1e-5, 10000.0),
    "8b": LayerConfig(2, 8192, 4096, 32, 8, 128, 14336, 1e-5, 500000.0),
    "8b_stack_layer": LayerConfig(1, 8192, 4096, 32, 8, 128, 14336, 1e-5, 500000.0),
    # not one of the five workloads: a layer twice as wide (70B-like proportions), for timing only
    "70b_width": LayerConfig(1, 8192, 8192, 64, 8, 128, 28672, 1e-5, 500000.0),
}

WEIGHT_NAMES = ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")


def weight_shapes(cfg: LayerConfig) -> dict:
    D, F = cfg.d_model, cfg.d_ff
    nq, nkv = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    return {
        "g_attn": (D,), "wq": (nq, D), "wk": (nkv, D), "wv": (nkv, D), "wo": (D, nq),
        "g_mlp": (D,), "w_gate": (F, D), "w_up": (F, D), "w_down": (D, F),
    }


def layer_param_count(cfg: LayerConfig) -> int:
    return int(sum(int(np.prod(s)) for s in weight_shapes(cfg).values()))


# --------------------------------------------------------------------------
# bf16 <-> float helpers (storage format only: 1-8-7 bits, the top half of fp32)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _normal_bf16(rng, shape, mean=0.0, std=1.0, chunk=1 << 24) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        z = rng.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            z *= np.float32(std)
        if mean != 0.0:
            z += np.float32(mean)
        out[lo:hi] = f32_to_bf16_bits(z)
    return out.reshape(shape)


def draw_layer_weights(rng, cfg: LayerConfig, w_std: float = 0.02) -> dict:
    shapes = weight_shapes(cfg)
    w = {}
    for name in WEIGHT_NAMES:
        if name.startswith("g_"):
            w[name] = _normal_bf16(rng, shapes[name], mean=1.0, std=0.02)
        else:
            w[name] = _normal_bf16(rng, shapes[name], std=w_std)
    return w


def make_layer_inputs(cfg: LayerConfig, seed: int = 0, w_std: float = 0.02,
                      x_std: float = 1.0) -> dict:
    """x, dy [B,S,D] and the nine weight tensors, all as bf16 bit patterns (uint16)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    shape = (cfg.batch, cfg.seq, cfg.d_model)
    out = {"x": _normal_bf16(rng, shape, std=x_std), "dy": _normal_bf16(rng, shape)}
    out.update(draw_layer_weights(rng, cfg, w_std))
    return out


def make_stack_inputs(cfg: LayerConfig, n_layers: int, vocab: int, seed: int = 0) -> dict:
    """ids, targets (int64, iid uniform in [0, vocab)), embedding table E [V,D], per-layer
    weights, final gain g_final, LM head w_lm [V,D] (untied), all bf16 bit patterns.
    Uniform ids stand in for tokenised text (which is Zipfian; that only changes the
    contention pattern of the embedding-gradient scatter-add)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    T = cfg.tokens
    out = {
        "ids": rng.integers(0, vocab, size=(cfg.batch, cfg.seq), dtype=np.int64),
        "targets": rng.integers(0, vocab, size=(cfg.batch, cfg.seq), dtype=np.int64),
        "embed": _normal_bf16(rng, (vocab, cfg.d_model), std=0.02),
        "layers": [draw_layer_weights(rng, cfg) for _ in range(n_layers)],
        "g_final": _normal_bf16(rng, (cfg.d_model,), mean=1.0, std=0.02),
        "w_lm": _normal_bf16(rng, (vocab, cfg.d_model), std=0.02),
    }
    assert out["ids"].size == T
    return out


def to_f64(tree):
    """Upcast every uint16 (bf16 bits) array in a dict/list tree to float64."""
    if isinstance(tree, dict):
        return {k: to_f64(v) for k, v in tree.items()}
    if isinstance(tree, (list, tuple)):
        return [to_f64(v) for v in tree]
    if isinstance(tree, np.ndarray) and tree.dtype == np.uint16:
        return bf16_bits_to_f64(tree)
    return tree


# --------------------------------------------------------------------------
# FLOP accounting used by the benchmark: algorithmic, fwd+bwd = 3 x fwd, causal
# attention counted as half of the dense S^2 products, no credit for recompute.
# --------------------------------------------------------------------------
def layer_fwd_flops(cfg: LayerConfig) -> float:
    T, D, F = cfg.tokens, cfg.d_model, cfg.d_ff
    hq, hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    qkv = 2.0 * T * D * (hq + 2 * hkv) * dh
    o = 2.0 * T * hq * dh * D
    mlp = 6.0 * T * D * F
    attn = 2.0 * cfg.batch * hq * float(cfg.seq) ** 2 * dh
    return qkv + o + mlp + attn


def layer_fwd_bwd_flops(cfg: LayerConfig) -> float:
    return 3.0 * layer_fwd_flops(cfg)
