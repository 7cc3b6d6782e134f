"""Synthetic LLM-shaped inputs (weights, calibration maxima, activations).

The paper evaluates on INT8 checkpoints of OPT / Llama2 / Falcon / Mistral and on
activation statistics from a small calibration set (Section 4.1); none of these
exist here, so seeded synthetic tensors of the same shapes stand in for them:

* weights: fp32 ~ N(0, 0.02^2), with 1 % of the rows multiplied by 8 (the paper
  describes weights as small-magnitude with a few outliers, Section 2);
* per-input-channel activation maxima a ~ LogNormal(0, 1) (channel-wise,
  heavy-tailed activation magnitudes, Section 3.2);
* batch-1 activations x ~ N(0, 1) rounded to bf16 for the fused GEMV path.

Only random draws and shapes live here; nothing below rescales, quantises,
prunes or codes anything.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

SEED_BASE = 0x250215443000


@dataclass(frozen=True)
class MatrixSpec:
    name: str
    rows: int  # output features
    cols: int  # input features (contiguous axis)
    index: int  # position m inside its decoder layer (0..6)


def _layer(hidden: int, ffn: int) -> List[MatrixSpec]:
    return [
        MatrixSpec("q_proj", hidden, hidden, 0),
        MatrixSpec("k_proj", hidden, hidden, 1),
        MatrixSpec("v_proj", hidden, hidden, 2),
        MatrixSpec("o_proj", hidden, hidden, 3),
        MatrixSpec("gate_proj", ffn, hidden, 4),
        MatrixSpec("up_proj", ffn, hidden, 5),
        MatrixSpec("down_proj", hidden, ffn, 6),
    ]


LLAMA7B_LAYER = _layer(4096, 11008)
LLAMA13B_LAYER = _layer(5120, 13824)


def layer_specs(kind: str) -> List[MatrixSpec]:
    if kind == "llama7b":
        return LLAMA7B_LAYER
    if kind == "llama13b":
        return LLAMA13B_LAYER
    raise ValueError(f"unknown layer kind {kind!r}")


def matrix_seed(layer: int, m: int) -> int:
    """Seed of matrix m (0..6: q,k,v,o,gate,up,down) of decoder layer `layer`."""
    return SEED_BASE + 16 * layer + m


def gen_weight(rows: int, cols: int, seed: int, outlier_frac: float = 0.01,
               outlier_gain: float = 8.0) -> np.ndarray:
    """fp32 W[rows, cols] ~ N(0, 0.02^2); round(outlier_frac*rows) distinct rows times 8."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.standard_normal((rows, cols), dtype=np.float32)
    w *= np.float32(0.02)
    n_out = int(round(outlier_frac * rows))
    if n_out > 0:
        idx = rng.choice(rows, size=n_out, replace=False)
        w[idx, :] *= np.float32(outlier_gain)
    return w


def gen_act_absmax(cols: int, seed: int) -> np.ndarray:
    """fp32 a[cols] ~ LogNormal(0, 1): stand-in for the calibrated max|X_i| per input channel."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5A5A5A5A))
    return rng.lognormal(mean=0.0, sigma=1.0, size=cols).astype(np.float32)


def gen_activation_bf16(cols: int, seed: int) -> np.ndarray:
    """x[cols] ~ N(0,1) rounded to nearest-even bf16, returned as uint16 bit patterns."""
    rng = np.random.Generator(np.random.PCG64(seed + 8))
    x = rng.standard_normal(cols, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)
