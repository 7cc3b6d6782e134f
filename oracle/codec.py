"""ctypes front end of the plain-C codec oracle (oracle/dc_oracle.c).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dc_oracle.c")
_LIB = os.path.join(_HERE, "libdc_oracle.so")

ALL_HUFF, AUTO, RAW_FRACTION, RAW_MASK, BLOCK_LAST = 0, 1, 2, 3, 4
HUFFMAN, TANS = 0, 1  # the coder of the chunks that are not raw
TANS_L = 2048
RAW_FLAG = 0x80000000

CHUNK_DTYPE = np.dtype([("off", "<u8"), ("comp_bytes", "<u4"), ("raw_bytes_flags", "<u4")])


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None
_lock = threading.Lock()


def lib():
    global _lib
    with _lock:
        if _lib is None:
            build()
            L = C.CDLL(_LIB)
            vp = C.c_void_p
            L.orc_histogram.argtypes = [vp, C.c_uint64, vp]
            L.orc_histogram.restype = None
            L.orc_code_lengths.argtypes = [vp, C.c_int, vp]
            L.orc_code_lengths.restype = C.c_int
            L.orc_canonical_codes.argtypes = [vp, vp]
            L.orc_canonical_codes.restype = None
            L.orc_stream_symbols.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
            L.orc_stream_symbols.restype = C.c_uint32
            L.orc_huff_bound.argtypes = [C.c_uint32, C.c_uint32]
            L.orc_huff_bound.restype = C.c_uint64
            L.orc_encode_chunk.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_int, vp, C.c_uint64]
            L.orc_encode_chunk.restype = C.c_uint64
            L.orc_decode_chunk.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, vp]
            L.orc_decode_chunk.restype = C.c_int
            L.orc_payload_bound.argtypes = [C.c_uint32, C.c_uint32, C.c_int]
            L.orc_payload_bound.restype = C.c_uint64
            L.orc_encode_chunk_codec.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_int, C.c_int, vp, C.c_uint64]
            L.orc_encode_chunk_codec.restype = C.c_uint64
            L.orc_decode_chunk_codec.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int, vp]
            L.orc_decode_chunk_codec.restype = C.c_int
            L.orc_tans_normalise.argtypes = [vp, vp]
            L.orc_tans_normalise.restype = C.c_int
            L.orc_tans_states.argtypes = [vp, vp, vp]
            L.orc_tans_states.restype = C.c_int
            L.orc_chunk_sizes_codec.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int, C.c_uint64,
                                                C.c_uint64, vp]
            L.orc_chunk_sizes_codec.restype = C.c_int
            L.orc_emit_codec.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int, vp, C.c_uint64,
                                         C.c_uint64, vp]
            L.orc_emit_codec.restype = C.c_int
            L.orc_decompress_codec.argtypes = [vp, C.c_uint64, vp, C.c_uint64, C.c_uint64, C.c_uint32,
                                               C.c_uint32, C.c_int, vp]
            L.orc_decompress_codec.restype = C.c_int
            L.orc_num_chunks.argtypes = [C.c_uint64, C.c_uint32]
            L.orc_num_chunks.restype = C.c_uint64
            L.orc_chunk_sizes.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64, vp]
            L.orc_chunk_sizes.restype = C.c_int
            L.orc_select_raw.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint64, C.c_int, C.c_double,
                                         C.c_uint32, vp, vp]
            L.orc_select_raw.restype = C.c_int
            L.orc_layout.argtypes = [vp, vp, C.c_uint64, C.c_uint32, C.c_uint64, vp]
            L.orc_layout.restype = C.c_uint64
            L.orc_emit.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, vp, C.c_uint64, C.c_uint64, vp]
            L.orc_emit.restype = C.c_int
            L.orc_decompress.argtypes = [vp, C.c_uint64, vp, C.c_uint64, C.c_uint64, C.c_uint32,
                                         C.c_uint32, vp]
            L.orc_decompress.restype = C.c_int
            L.orc_close_blob.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int]
            L.orc_close_blob.restype = C.c_int
            L.orc_check_trailer.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int]
            L.orc_check_trailer.restype = C.c_int
            _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _bytes(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(-1)


def histogram(data) -> np.ndarray:
    src = _bytes(data)
    cnt = np.zeros(256, dtype=np.uint64)
    lib().orc_histogram(_ptr(src), src.size, _ptr(cnt))
    return cnt


def code_lengths(cnt, max_len: int = 11) -> np.ndarray:
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    assert cnt.size == 256
    out = np.zeros(256, dtype=np.uint8)
    rc = lib().orc_code_lengths(_ptr(cnt), max_len, _ptr(out))
    if rc != 0:
        raise ValueError(f"orc_code_lengths failed: {rc}")
    return out


def canonical_codes(lengths) -> np.ndarray:
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    out = np.zeros(256, dtype=np.uint16)
    lib().orc_canonical_codes(_ptr(lengths), _ptr(out))
    return out


def stream_symbols(raw_bytes: int, S: int, j: int) -> int:
    return int(lib().orc_stream_symbols(raw_bytes, S, j))


def tans_normalise(cnt) -> np.ndarray:
    """Frequencies normalised to TANS_L by the format's rule."""
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    assert cnt.size == 256
    q = np.zeros(256, dtype=np.uint16)
    rc = lib().orc_tans_normalise(_ptr(cnt), _ptr(q))
    if rc != 0:
        raise ValueError(f"orc_tans_normalise failed: {rc}")
    return q


def tans_states(q):
    """(value_of[x], number_of[x]) for the TANS_L states of normalised frequencies q."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    value_of = np.zeros(TANS_L, dtype=np.uint8)
    number_of = np.zeros(TANS_L, dtype=np.uint16)
    rc = lib().orc_tans_states(_ptr(q), _ptr(value_of), _ptr(number_of))
    if rc != 0:
        raise ValueError(f"orc_tans_states failed: {rc}")
    return value_of, number_of


def encode_chunk(data, S: int, max_len: int = 11, codec: int = HUFFMAN) -> np.ndarray:
    src = _bytes(data)
    cap = int(lib().orc_payload_bound(src.size, S, codec))
    out = np.zeros(cap, dtype=np.uint8)
    n = int(lib().orc_encode_chunk_codec(_ptr(src), src.size, S, codec, max_len, _ptr(out), cap))
    if n == 0:
        raise ValueError("orc_encode_chunk failed")
    return out[:n].copy()


def decode_chunk(payload, raw_bytes: int, S: int, codec: int = HUFFMAN) -> np.ndarray:
    p = _bytes(payload)
    dst = np.zeros(raw_bytes, dtype=np.uint8)
    rc = lib().orc_decode_chunk_codec(_ptr(p), p.size, raw_bytes, S, codec, _ptr(dst))
    if rc != 0:
        raise ValueError(f"orc_decode_chunk failed: {rc}")
    return dst


@dataclass
class Compressed:
    blob: np.ndarray  # uint8
    table: np.ndarray  # CHUNK_DTYPE
    raw_bytes: int
    chunk_bytes: int
    n_streams: int
    codec: int = HUFFMAN

    @property
    def n_chunks(self) -> int:
        return int(self.table.size)

    @property
    def ratio(self) -> float:
        """CR = size before / size after (Section 2), the chunk table counted with the blob."""
        return self.raw_bytes / float(self.blob.size + self.table.nbytes)


def _split(n: int, parts: int):
    parts = max(1, min(parts, n))
    edges = [n * i // parts for i in range(parts + 1)]
    return [(edges[i], edges[i + 1]) for i in range(parts) if edges[i + 1] > edges[i]]


def _run_ranges(fn, n: int, threads: int):
    ranges = _split(n, threads)
    if len(ranges) <= 1:
        for a, b in ranges:
            rc = fn(a, b)
            if rc != 0:
                raise ValueError(f"oracle call failed: {rc}")
        return
    rcs = [0] * len(ranges)

    def work(i, a, b):
        rcs[i] = fn(a, b)

    ts = [threading.Thread(target=work, args=(i, a, b)) for i, (a, b) in enumerate(ranges)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    for rc in rcs:
        if rc != 0:
            raise ValueError(f"oracle call failed: {rc}")


def compress(data, chunk_bytes: int, n_streams: int, policy: int = ALL_HUFF, raw_fraction: float = 0.0,
             block: int = 0, mask: Optional[np.ndarray] = None, threads: int = 1, codec: int = HUFFMAN) -> Compressed:
    """Whole-buffer compression.  `threads` only splits the chunk range; each chunk is coded alone."""
    L = lib()
    src = _bytes(data)
    n = src.size
    nc = int(L.orc_num_chunks(n, chunk_bytes))
    huff = np.zeros(nc, dtype=np.uint32)
    _run_ranges(lambda a, b: L.orc_chunk_sizes_codec(_ptr(src), n, chunk_bytes, n_streams, codec, a, b, _ptr(huff)),
                nc, threads)
    is_raw = np.zeros(nc, dtype=np.uint8)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    # the fraction is a parameter of the method, a 32-bit float at the library's boundary: both sides are
    # given the same value (0.9 as a float is just below 0.9, which matters when f * n_chunks + 1/2 is whole)
    rc = L.orc_select_raw(_ptr(huff), n, chunk_bytes, nc, policy, float(np.float32(raw_fraction)), block,
                          None if m is None else _ptr(m), _ptr(is_raw))
    if rc != 0:
        raise ValueError(f"orc_select_raw failed: {rc}")
    table = np.zeros(nc, dtype=CHUNK_DTYPE)
    total = int(L.orc_layout(_ptr(huff), _ptr(is_raw), n, chunk_bytes, nc, _ptr(table)))
    blob = np.zeros(total, dtype=np.uint8)
    _run_ranges(lambda a, b: L.orc_emit_codec(_ptr(src), n, chunk_bytes, n_streams, codec, _ptr(table), a, b,
                                              _ptr(blob)), nc, threads)
    if L.orc_close_blob(_ptr(blob), total, chunk_bytes, n_streams, codec) != 0:
        raise ValueError("orc_close_blob failed")
    return Compressed(blob, table, n, chunk_bytes, n_streams, codec)


def decompress(blob, table, chunk_bytes: int, n_streams: int, raw_bytes: int, threads: int = 1,
               codec: int = HUFFMAN) -> np.ndarray:
    L = lib()
    b = _bytes(blob)
    t = np.ascontiguousarray(table, dtype=CHUNK_DTYPE)
    # the destination is sized by the caller: the table must describe exactly that many bytes
    sizes = (t["raw_bytes_flags"] & np.uint32(0x7FFFFFFF)).astype(np.int64)
    if t.size == 0 or (sizes[:-1] != chunk_bytes).any() or (t.size - 1) * chunk_bytes + int(sizes[-1]) != raw_bytes:
        raise ValueError("the table does not describe raw_bytes bytes")
    dst = np.zeros(raw_bytes, dtype=np.uint8)
    _run_ranges(lambda a, c: L.orc_decompress_codec(_ptr(b), b.size, _ptr(t), a, c, chunk_bytes, n_streams, codec,
                                                    _ptr(dst)), int(t.size), threads)
    return dst
