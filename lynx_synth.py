"""Seeded synthetic inputs and the named workload shapes.

This module serves both the CPU oracle and the HIP path.  It holds none of the
method's arithmetic: it only names layer shapes, draws normally distributed
tensors from fixed seeds and rounds them once to the configuration's storage
type.  Both sides then consume the very same rounded arrays.

Recipe (stands in for the language-model batches the paper trains on; no
kernel on this path has data-dependent cost):
  X, dOUT ~ N(0, 1); weights and biases ~ N(0, 0.02); LayerNorm gamma = 1,
  beta = 0; data seed 1 for X, 2 for dOUT, 3 + k for the k-th parameter.
Arrays are float32 numpy arrays; for bf16 configurations every value is
already representable in bf16 (round-to-nearest-even applied once here).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np

F32 = 0
BF16 = 1

PARAM_NAMES = ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2",
               "g1", "be1", "g2", "be2")


@dataclass(frozen=True)
class LayerConfig:
    """Shape and constants of one tensor-parallel shard of a GPT block."""
    dtype: int            # F32 or BF16: storage type of activations/params
    hidden: int           # h
    local_heads: int      # a
    head_dim: int         # d
    local_ffn: int        # f
    seq: int              # s
    micro_batch: int      # b
    tp_size: int = 1
    tp_rank: int = 0
    causal: int = 1
    dropout_p: float = 0.1
    ln_eps: float = 1e-5
    seed: int = 0         # dropout generator key
    layer_id: int = 0
    flags: int = 0        # 1: attention without the seq x seq tensors where the policy allows

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq

    @property
    def proj(self) -> int:
        return self.local_heads * self.head_dim

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


# The five workloads (tiny fp32 block; GPT-1.3B TP=1; 7B TP=4; 13B TP=8;
# 23B TP=8 six-layer slice).
CONFIGS: Dict[str, LayerConfig] = {
    "C1": LayerConfig(F32, 256, 4, 64, 1024, 128, 2, tp_size=1),
    "C2": LayerConfig(BF16, 2048, 16, 128, 8192, 2048, 4, tp_size=1),
    "C3": LayerConfig(BF16, 4096, 8, 128, 4096, 2048, 4, tp_size=4),
    "C4": LayerConfig(BF16, 5120, 5, 128, 2560, 2048, 8, tp_size=8),
    "C5": LayerConfig(BF16, 6144, 6, 128, 3072, 2048, 4, tp_size=8),
}
C5_LAYERS = 6


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


def _store(x: np.ndarray, dtype: int) -> np.ndarray:
    x = x.astype(np.float32)
    return round_to_bf16(x) if dtype == BF16 else x


def _normal(seed: int, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed))
    return rng.standard_normal(shape, dtype=np.float64) * std


def param_shapes(cfg: LayerConfig) -> Dict[str, tuple]:
    h, p, f = cfg.hidden, cfg.proj, cfg.local_ffn
    return {
        "wqkv": (3 * p, h), "bqkv": (3 * p,),
        "wo": (h, p), "bo": (h,),
        "w1": (f, h), "b1": (f,),
        "w2": (h, f), "b2": (h,),
        "g1": (h,), "be1": (h,), "g2": (h,), "be2": (h,),
    }


def make_params(cfg: LayerConfig, seed_base: int = 3, random_ln: bool = False
                ) -> Dict[str, np.ndarray]:
    """Layer parameters.  With random_ln the LayerNorm affine terms are drawn
    too (gamma ~ 1 + N(0, 0.1), beta ~ N(0, 0.1)) so tests exercise them."""
    out = {}
    for k, (name, shape) in enumerate(param_shapes(cfg).items()):
        seed = seed_base + k + 1000 * cfg.layer_id
        if name in ("g1", "g2"):
            v = np.ones(shape) + (_normal(seed, shape, 0.1) if random_ln else 0.0)
        elif name in ("be1", "be2"):
            v = _normal(seed, shape, 0.1) if random_ln else np.zeros(shape)
        else:
            v = _normal(seed, shape, 0.02)
        out[name] = _store(v, cfg.dtype)
    return out


def make_x(cfg: LayerConfig, seed: int = 1) -> np.ndarray:
    return _store(_normal(seed, (cfg.tokens, cfg.hidden), 1.0), cfg.dtype)


def make_dout(cfg: LayerConfig, seed: int = 2) -> np.ndarray:
    return _store(_normal(seed, (cfg.tokens, cfg.hidden), 1.0), cfg.dtype)


def c5_retain_masks(policy_seed: int = 0, layers: int = C5_LAYERS):
    """Per-layer retain masks of the six-layer slice: bits 1..13 drawn from a
    seeded generator, bit 0 (the layer input, always the checkpoint) set."""
    rng = np.random.Generator(np.random.Philox(1_000_003 + policy_seed))
    return [int(m) | 1 for m in rng.integers(0, 1 << 14, size=layers)]
