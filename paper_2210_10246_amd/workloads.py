"""Seeded synthetic inputs with the shapes of BERT / GPT-2 / RoBERTa encoder layers.

This module only draws random tensors: it holds none of the layers' arithmetic, imports
neither the HIP binding nor the CPU checker, and serves both.  Values are drawn in float64
from one numpy PCG64 stream per (config, tensor), then rounded to the storage dtype, so
every consumer sees identical bits.

The paper trains on English Wikipedia, WikiText and MRPC; the layers' cost depends only on
shape, dtype and mask structure, so these tensors stand in for those corpora.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

BASE_SEED = 20221010
RNG_SEED_BASE = 0x5EED0000


@dataclass(frozen=True)
class LayerConfig:
    index: int
    name: str
    dtype: str            # "f32" | "bf16": storage dtype of activations
    batch: int
    seq: int
    hidden: int
    heads: int
    eps: float
    gelu_kind: str        # "erf" | "tanh"
    mask: str             # "none" | "padding" | "causal"
    len_lo: int = 0
    len_hi: int = 0
    p: float = 0.1
    outliers: bool = False  # 1 % of entries multiplied by 20

    @property
    def ffn(self) -> int:
        return 4 * self.hidden

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def dropout_seed(self) -> int:
        return RNG_SEED_BASE + self.index


CONFIGS = (
    LayerConfig(0, "bert-base-s128-f32", "f32", 2, 128, 768, 12, 1e-12, "erf", "none"),
    LayerConfig(1, "bert-large-s128-bf16", "bf16", 64, 128, 1024, 16, 1e-12, "erf",
                "padding", 64, 128),
    LayerConfig(2, "bert-large-s512-bf16", "bf16", 16, 512, 1024, 16, 1e-12, "erf",
                "padding", 256, 512),
    LayerConfig(3, "gpt2-small-s1024-bf16", "bf16", 8, 1024, 768, 12, 1e-5, "tanh", "causal"),
    LayerConfig(4, "roberta-large-s512", "bf16", 8, 512, 1024, 16, 1e-12, "erf", "none",
                outliers=True),
)


def config(index: int, *, batch: Optional[int] = None, dtype: Optional[str] = None) -> LayerConfig:
    """Config by index; config 4 is swept over batch (8/16/32/64) and dtype."""
    cfg = CONFIGS[index]
    if batch is not None:
        cfg = replace(cfg, batch=batch)
    if dtype is not None:
        cfg = replace(cfg, dtype=dtype)
    return cfg


_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def torch_dtype(dt: str) -> torch.dtype:
    return _TORCH_DT[dt]


def _rng(cfg: LayerConfig, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([BASE_SEED + cfg.index, stream]))


def _store(a: np.ndarray, dt: str) -> torch.Tensor:
    """float64 draw -> CPU tensor in the storage dtype."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(_TORCH_DT[dt])


def _normal(cfg: LayerConfig, stream: int, shape, scale: float = 1.0) -> np.ndarray:
    g = _rng(cfg, stream)
    a = g.standard_normal(shape)
    if cfg.outliers:
        hit = g.random(shape) < 0.01
        a = np.where(hit, a * 20.0, a)
    return a * scale


def as_f64(t: torch.Tensor) -> np.ndarray:
    """Widen a stored tensor to float64 without changing its value."""
    return t.detach().cpu().to(torch.float64).numpy()


def gelu_inputs(cfg: LayerConfig, rows: Optional[int] = None):
    """x, dy of shape [rows, 4H] (rows defaults to batch*seq)."""
    rows = cfg.tokens if rows is None else rows
    shape = (rows, cfg.ffn)
    return {
        "x": _store(_normal(cfg, 10, shape), cfg.dtype),
        "dy": _store(_rng(cfg, 11).standard_normal(shape), cfg.dtype),
    }


def layernorm_inputs(cfg: LayerConfig, rows: Optional[int] = None):
    """x, dy [rows, H]; gamma = 1 + N(0, 0.1), beta = N(0, 0.1) in float32."""
    rows = cfg.tokens if rows is None else rows
    shape = (rows, cfg.hidden)
    g = _rng(cfg, 22)
    gamma = 1.0 + 0.1 * g.standard_normal(cfg.hidden)
    beta = 0.1 * g.standard_normal(cfg.hidden)
    return {
        "x": _store(_normal(cfg, 20, shape), cfg.dtype),
        "dy": _store(_rng(cfg, 21).standard_normal(shape), cfg.dtype),
        "gamma": _store(gamma, "f32"),
        "beta": _store(beta, "f32"),
    }


def attention_inputs(cfg: LayerConfig, batch: Optional[int] = None):
    """scores [B, A, S, S] ~ N(0,1)/8 (already scaled by 1/sqrt(d)), dout ~ N(0,1),
    key_len [B] int32 for padding masks (uniform in [len_lo, len_hi]) else None."""
    B = cfg.batch if batch is None else batch
    shape = (B, cfg.heads, cfg.seq, cfg.seq)
    key_len = None
    if cfg.mask == "padding":
        kl = _rng(cfg, 32).integers(cfg.len_lo, cfg.len_hi + 1, size=B)
        key_len = torch.from_numpy(kl.astype(np.int32))
    return {
        "scores": _store(_normal(cfg, 30, shape, 0.125), cfg.dtype),
        "dout": _store(_rng(cfg, 31).standard_normal(shape), cfg.dtype),
        "key_len": key_len,
        "causal": cfg.mask == "causal",
    }
