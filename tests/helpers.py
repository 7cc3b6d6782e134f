"""Shared helpers for the tests: workloads built from the seeded generators and the oracle."""
from __future__ import annotations

import functools

import numpy as np

import oracle.codec as oc
import oracle.quant as oq
import synth


@functools.lru_cache(maxsize=64)
def oracle_matrix(rows: int, cols: int, seed: int, rescale: bool):
    """(q int8[rows, cols], row_scale fp32[rows]) by the oracle: generate, (rescale), quantise, prune."""
    w = synth.gen_weight(rows, cols, seed)
    if rescale:
        a = synth.gen_act_absmax(cols, seed)
        w = oq.rescale(w, oq.channel_scale(a, 0.5))
    q, scale = oq.quantise_rows(w)
    return oq.prune(q), scale


def gemv_workspace(n_chunks: int):
    """(device tensor, size in bytes) for the workspace argument of the fused product calls, filled with
    all-ones bytes (fp32 NaN), so that a partial sum that is read without having been written shows."""
    import torch

    import paper_2502_15443_amd as dc

    n = dc.decompress_gemv_workspace(n_chunks)
    return torch.full((n,), 0xFF, dtype=torch.uint8, device="cuda"), n


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


def empty_buffer_before_three_codes(data: np.ndarray, S: int):
    """Walk of a decoder that keeps a 64-bit buffer per sub-stream, refills it by 32 bits whenever at most 32
    bits are valid, and decodes each half group of 8 symbols as 3 + 2 + 3 codes: the places (lane, group,
    half, first symbol of the batch) where a batch of three 11-bit codes (33 bits) begins on a buffer that the
    batch before it emptied completely, so that one refill leaves 32 bits.  Code lengths from the oracle."""
    raw = data.size
    ln = oc.code_lengths(np.bincount(data, minlength=256).astype(np.uint64)).astype(int)
    groups = (raw + 15) // 16
    hits = []
    for j in range(min(S, groups)):
        lens = [ln[data[16 * g:16 * g + 16]] for g in range(j, groups, S)]
        size = (int(sum(int(x.sum()) for x in lens)) + 7) // 8
        avail = 64 - 8 * (((-size) % 16) & 3)  # the stream starts pad bytes into its first block
        for gi, gl in enumerate(lens):
            if gl.size < 16:
                break
            for half in (0, 1):
                h = gl[8 * half:8 * half + 8]
                for lo, hi in ((0, 3), (3, 5), (5, 8)):
                    if avail <= 32:
                        if avail == 0 and int(h[lo:hi].sum()) == 33:
                            hits.append((j, gi, half, lo))
                        avail += 32
                    avail -= int(h[lo:hi].sum())
    return hits


def emptied_buffer_bytes(S: int) -> np.ndarray:
    """24 rounds of a chunk in which sub-stream 0 is nearly all rare byte values (10- and 11-bit codes) and
    the other sub-streams are a geometric mix of ten frequent ones; drawn again (seeded) until the walk above
    meets its case."""
    r = np.random.default_rng(1)
    p = np.array([2.0 ** -(k + 1) for k in range(10)])
    for _ in range(50):
        n = 16 * S * 24
        data = r.choice(np.arange(10), size=n, p=p / p.sum()).astype(np.uint8)
        for rd in range(24):
            grp = r.integers(100, 164, 16).astype(np.uint8)
            k = int(r.integers(0, 4))
            grp[r.integers(0, 16, k)] = r.integers(0, 3, k)
            data[16 * rd * S:16 * rd * S + 16] = grp
        if empty_buffer_before_three_codes(data, S):
            return data
    raise AssertionError("no such input found")
