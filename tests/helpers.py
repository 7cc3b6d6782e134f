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
