"""Shared helpers for the tests: workloads built from the seeded generators and the oracle."""
from __future__ import annotations

import functools

import numpy as np

import oracle.codec as oc
import oracle.quant as oq
import synth


@functools.lru_cache(maxsize=40)
def oracle_matrix(rows: int, cols: int, seed: int, rescale: bool):
    """(q int8[rows, cols], row_scale fp32[rows]) by the oracle: generate, (rescale), quantise, prune."""
    w = synth.gen_weight(rows, cols, seed)
    if rescale:
        a = synth.gen_act_absmax(cols, seed)
        w = oq.rescale(w, oq.channel_scale(a, 0.5))
    q, scale = oq.quantise_rows(w)
    return oq.prune(q), scale


def weightlike_bytes(n: int, seed: int) -> np.ndarray:
    """Byte string with chunk-to-chunk varying spread, so chunks differ in gain."""
    r = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.uint8)
    step = 8192
    for i in range(0, n, step):
        sigma = 2.0 + 40.0 * r.random()
        m = min(step, n - i)
        out[i:i + m] = np.clip(np.rint(r.standard_normal(m) * sigma), -127, 127).astype(np.int8).view(np.uint8)
    return out


def lopsided_bytes(n: int, S: int, seed: int) -> np.ndarray:
    """Bytes whose sub-streams use the code very unevenly: the 16-byte groups of stream 0 hold rare
    values (longest codes), those of stream 1 a mix, all others one frequent value (shortest code), and a
    stretch in the middle swaps the roles, so the streams' positions drift far apart and back."""
    r = np.random.default_rng(seed)
    out = np.full(n, 0x00, dtype=np.uint8)
    groups = (n + 15) // 16
    rare = r.integers(1, 256, size=n, dtype=np.uint8)
    for g in range(groups):
        j = g % S
        lo, hi = 16 * g, min(16 * g + 16, n)
        swap = groups // 3 <= g < 2 * groups // 3
        heavy = (j == 0) != swap if S > 1 else (g % 2 == 0)
        if heavy:
            out[lo:hi] = rare[lo:hi]
        elif j == 1:
            out[lo:hi] = np.where(r.random(hi - lo) < 0.5, rare[lo:hi], 0)
    return out
