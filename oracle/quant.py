"""CPU oracle for the numeric steps around the codec.  TEST INFRASTRUCTURE ONLY.

Plain numpy, one line per step of the paper's compression stage (Section 3.2):
per-channel scaling (Eqs. 1-2), INT8 quantisation (Eq. 4), pruning of
near-zero quantised weights (the role of Eq. 5), and the two consumers of the
decoded bytes: dequantisation to bf16 and the batch-1 product Y = X' W' (Eq. 1).

Nothing here is imported by the library; nothing of the library is imported here.
"""
from __future__ import annotations

import numpy as np


def channel_scale(act_absmax: np.ndarray, alpha: float) -> np.ndarray:
    """s_j = (max|X_j|)^alpha per input channel j (Eq. 2), evaluated in fp64, stored as fp32."""
    return np.power(act_absmax.astype(np.float64), np.float64(alpha)).astype(np.float32)


def rescale(w: np.ndarray, s: np.ndarray) -> np.ndarray:
    """W' = s * W along the input-channel (column) axis of W[out, in] (Eq. 1), in fp32."""
    assert w.dtype == np.float32 and s.dtype == np.float32 and s.shape == (w.shape[1],)
    return w * s[None, :]


def quantise_rows(w: np.ndarray):
    """Symmetric per-row absmax INT8 (Eq. 4 with the workload's per-row granularity).

    scale_i = max_j |W'_ij| / 127 (fp32 division); q = clip(rint(W'/scale_i), -127, 127) with
    round-half-to-even and a true fp32 division; an all-zero row gets scale 1 and q = 0.
    """
    assert w.dtype == np.float32
    m = np.max(np.abs(w), axis=1)
    scale = (m / np.float32(127.0)).astype(np.float32)
    scale[m == 0] = np.float32(1.0)
    q = np.clip(np.rint(w / scale[:, None]), -127, 127).astype(np.int8)
    return q, scale


def quantise_tensor(w: np.ndarray):
    """Symmetric per-tensor absmax INT8 (Eq. 4 with the paper's own granularity, Section 4.5
    "scaled-tensor"): scale = max |W'| / 127 (fp32), q = clip(rint(W'/scale), -127, 127)."""
    assert w.dtype == np.float32
    m = np.max(np.abs(w))
    scale = np.float32(1.0) if m == 0 else np.float32(m / np.float32(127.0))
    q = np.clip(np.rint(w / scale), -127, 127).astype(np.int8)
    return q, scale


def prune(q: np.ndarray) -> np.ndarray:
    """Quantised weights of magnitude <= 1 become 0 (fixed-threshold form of the score rule, Eq. 5)."""
    out = q.copy()
    out[np.abs(q.astype(np.int16)) <= 1] = 0
    return out


def prune_by_score(q: np.ndarray, act_absmax: np.ndarray, sparsity: float) -> np.ndarray:
    """Paper's rule (Eq. 5): score = ||X_j||_inf * |Q(W')_ij|; the fraction `sparsity` of lowest
    scores is set to zero.  Ties at the threshold are all pruned."""
    score = np.abs(q.astype(np.float64)) * act_absmax.astype(np.float64)[None, :]
    k = int(np.floor(sparsity * score.size))
    if k <= 0:
        return q.copy()
    thr = np.partition(score.ravel(), k - 1)[k - 1]
    out = q.copy()
    out[score <= thr] = 0
    return out


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def dequant_bf16(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """bf16( fp32(q_ij) * scale_i ): one fp32 product (exactly rounded), then one rounding to bf16."""
    prod = q.astype(np.float32) * scale.astype(np.float32)[:, None]
    return bf16_round(prod).reshape(q.shape)


def gemv_ref(q: np.ndarray, scale: np.ndarray, x_bf16: np.ndarray) -> np.ndarray:
    """y_i = scale_i * sum_j q_ij x_j in fp64 (Eq. 1 for one activation row)."""
    x = bf16_to_f64(x_bf16)
    return (q.astype(np.float64) @ x) * scale.astype(np.float64)


def quantise_vector(x: np.ndarray):
    """Symmetric absmax INT8 of one activation row (Eq. 4, "Quant(X')"; Section 4.1: weight and activation
    are both quantised to INT8).  The paper gives no granularity for activations; one scale for the row:
    scale = max |x| / 127 (fp32 division; 1 if x is all zero), xq = clip(rint(x / scale), -127, 127)."""
    assert x.dtype == np.float32 and x.ndim == 1
    m = np.max(np.abs(x)) if x.size else np.float32(0)
    scale = np.float32(1.0) if m == 0 else np.float32(m / np.float32(127.0))
    xq = np.clip(np.rint(x / scale), -127, 127).astype(np.int8)
    return xq, scale


def gemv_w8a8_acc(q: np.ndarray, xq: np.ndarray) -> np.ndarray:
    """acc_i = sum_j q_ij xq_j, exact integers (Eq. 4: the product of the two quantised operands)."""
    return q.astype(np.int64) @ xq.astype(np.int64)


def gemv_w8a8(q: np.ndarray, scale: np.ndarray, xq: np.ndarray, x_scale) -> np.ndarray:
    """y_i = fp32(fp32(acc_i) * scale_i) * x_scale: the integer sum is converted to fp32 (round to nearest
    even), multiplied by the weight scale of the row, then by the activation scale, each product rounded
    once.  The order is fixed so that the result has one right value."""
    acc = gemv_w8a8_acc(q, xq)
    assert np.abs(acc).max(initial=0) < 2 ** 31
    y = acc.astype(np.float32) * scale.astype(np.float32)
    return (y * np.float32(x_scale)).astype(np.float32)
