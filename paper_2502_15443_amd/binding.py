"""ctypes binding of libdc_mi355x.so: same names as the C entry points, argument marshalling only.

Host buffers are numpy arrays; device buffers are anything with a ``data_ptr()`` (torch tensors) or
plain integer addresses.  Streams are raw hipStream_t handles (``torch.cuda.current_stream().cuda_stream``).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdc_mi355x.so")

POLICY_ALL_HUFF, POLICY_AUTO, POLICY_RAW_FRACTION, POLICY_RAW_MASK, POLICY_BLOCK_LAST = 0, 1, 2, 3, 4
CODEC_HUFFMAN, CODEC_TANS = 0, 1
FORMAT_ID = 5  # DC_FORMAT_ID of include/dc.h
CHUNK_RAW = 0x80000000
STATIC_SCRATCH_BYTES = 16 << 20
TRACE_DECODED, TRACE_COPIED, TRACE_SKIPPED = 0, 1, 2
CHUNK_DTYPE = np.dtype([("off", "<u8"), ("comp_bytes", "<u4"), ("raw_bytes_flags", "<u4")])


class DCError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {version_safe_strerror(code)}")
        self.code = code


class _CParams(C.Structure):
    _fields_ = [("chunk_bytes", C.c_uint32), ("n_streams", C.c_uint32), ("policy", C.c_uint32),
                ("raw_fraction", C.c_float), ("block_chunks", C.c_uint32), ("codec", C.c_uint32),
                ("format", C.c_uint32), ("raw_mask", C.c_void_p)]


class _CMatrix(C.Structure):
    _fields_ = [("first_chunk", C.c_uint64), ("rows", C.c_uint32), ("cols", C.c_uint32),
                ("row_scale_dev", C.c_void_p), ("dst_bf16_dev", C.c_void_p), ("dst_cap_elems", C.c_uint64),
                ("x_bf16_dev", C.c_void_p), ("y_accum_dev", C.c_void_p), ("y_bf16_dev", C.c_void_p),
                ("x_i8_dev", C.c_void_p), ("x_scale", C.c_float)]


@dataclass
class Matrix:
    """One matrix of a whole-layer fused call (dc_matrix): device buffers are tensors or addresses."""
    first_chunk: int
    rows: int
    cols: int
    row_scale_dev: object
    dst_bf16_dev: object = None
    dst_cap_elems: int = 0
    x_bf16_dev: object = None
    y_accum_dev: object = None
    y_bf16_dev: object = None
    x_i8_dev: object = None
    x_scale: float = 0.0


@dataclass
class Params:
    chunk_bytes: int = 65536
    n_streams: int = 32
    policy: int = POLICY_ALL_HUFF
    raw_fraction: float = 0.0
    block_chunks: int = 0
    raw_mask: Optional[np.ndarray] = None
    codec: int = CODEC_HUFFMAN
    format: int = FORMAT_ID

    def _c(self) -> _CParams:
        p = _CParams(self.chunk_bytes, self.n_streams, self.policy, float(self.raw_fraction),
                     self.block_chunks, self.codec, self.format, None)
        if self.raw_mask is not None:
            self._mask_keepalive = np.ascontiguousarray(self.raw_mask, dtype=np.uint8)
            p.raw_mask = self._mask_keepalive.ctypes.data
        return p


def lib_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python paper_2502_15443_amd/build.py` "
            "(there is no fallback path)")
    # Device memory and streams come from PyTorch, so the library must run on the HIP runtime that
    # PyTorch loaded: bring PyTorch in first so that the shared runtime is resolved to its copy.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(_LIB_PATH)
    vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int
    pp = C.POINTER(_CParams)
    pu64 = C.POINTER(C.c_uint64)
    L.dc_version.restype = C.c_char_p
    L.dc_version.argtypes = []
    L.dc_last_hip_error.restype = C.c_char_p
    L.dc_last_hip_error.argtypes = []
    L.dc_strerror.restype = C.c_char_p
    L.dc_strerror.argtypes = [i32]
    L.dc_set_num_threads.restype = i32
    L.dc_set_num_threads.argtypes = [i32]
    L.dc_quantize_rows.restype = i32
    L.dc_quantize_rows.argtypes = [vp, u32, u32, vp, C.c_double, u32, vp, vp, vp]
    L.dc_quantize_tensor.restype = i32
    L.dc_quantize_tensor.argtypes = [vp, u32, u32, vp, C.c_double, C.c_double, vp, vp, vp]
    L.dc_compress_bound.restype = i32
    L.dc_compress_bound.argtypes = [u64, pp, pu64, pu64]
    L.dc_compress_chunks.restype = i32
    L.dc_compress_chunks.argtypes = [vp, u64, pp, vp, u64, pu64, vp, u64, pu64]
    L.dc_compress_chunks_dev_workspace.restype = i32
    L.dc_compress_chunks_dev_workspace.argtypes = [u64, pp, pu64]
    L.dc_compress_chunks_dev.restype = i32
    L.dc_compress_chunks_dev.argtypes = [vp, u64, pp, vp, u64, vp, u64, vp, u64, vp, vp]
    L.dc_compress_chunks_dev_static.restype = i32
    L.dc_compress_chunks_dev_static.argtypes = [vp, u64, pp, vp, u64, vp, u64, vp, vp]
    L.dc_blob_trailer.restype = i32
    L.dc_blob_trailer.argtypes = [vp, pp]
    L.dc_validate.restype = i32
    L.dc_validate.argtypes = [vp, u64, vp, u64, pp, pu64]
    L.dc_decompress_chunks.restype = i32
    L.dc_decompress_chunks.argtypes = [vp, u64, vp, u64, pp, vp, u64, vp]
    L.dc_issue_rate_count.restype = u32
    L.dc_issue_rate_count.argtypes = []
    L.dc_issue_rate_name.restype = C.c_char_p
    L.dc_issue_rate_name.argtypes = [u32]
    L.dc_issue_rate.restype = i32
    L.dc_issue_rate.argtypes = [u32, vp, u64, vp, C.POINTER(C.c_double)]
    L.dc_decompress_chunks_traced.restype = i32
    L.dc_decompress_chunks_traced.argtypes = [vp, u64, vp, u64, pp, vp, u64, vp, vp]
    L.dc_decompress_dequant_bf16.restype = i32
    L.dc_decompress_dequant_bf16.argtypes = [vp, u64, vp, u64, pp, vp, u32, u32, vp, u64, vp]
    L.dc_decompress_gemv.restype = i32
    L.dc_decompress_gemv.argtypes = [vp, u64, vp, u64, pp, vp, u32, u32, vp, vp, vp, vp, u64, vp]
    L.dc_decompress_gemv_workspace.restype = i32
    L.dc_decompress_gemv_workspace.argtypes = [u64, pu64]
    pm = C.POINTER(_CMatrix)
    L.dc_decompress_dequant_bf16_layer.restype = i32
    L.dc_decompress_dequant_bf16_layer.argtypes = [vp, u64, vp, u64, pp, pm, u32, vp]
    L.dc_decompress_gemv_layer.restype = i32
    L.dc_decompress_gemv_layer.argtypes = [vp, u64, vp, u64, pp, pm, u32, vp, u64, vp]
    L.dc_gemv_i8.restype = i32
    L.dc_gemv_i8.argtypes = [vp, vp, u32, u32, vp, vp, vp, vp]
    L.dc_decompress_gemv_w8a8.restype = i32
    L.dc_decompress_gemv_w8a8.argtypes = [vp, u64, vp, u64, pp, vp, u32, u32, vp, C.c_float, vp, vp, vp]
    L.dc_decompress_gemv_w8a8_layer.restype = i32
    L.dc_decompress_gemv_w8a8_layer.argtypes = [vp, u64, vp, u64, pp, pm, u32, vp]
    L.dc_gemv_w8a8.restype = i32
    L.dc_gemv_w8a8.argtypes = [vp, vp, u32, u32, vp, C.c_float, vp, vp, vp]
    L.dc_quantize_vector.restype = i32
    L.dc_quantize_vector.argtypes = [vp, u32, vp, vp]
    L.dc_device_copy.restype = i32
    L.dc_device_copy.argtypes = [vp, vp, u64, vp]
    return L


_L = _load()


def version_safe_strerror(code: int) -> str:
    msg = _L.dc_strerror(code).decode()
    if code == -4:
        msg += " (" + _L.dc_last_hip_error().decode() + ")"
    return msg


def version() -> str:
    return _L.dc_version().decode()


def set_num_threads(n: int) -> int:
    return int(_L.dc_set_num_threads(n))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise DCError(rc, what)


def _dev(t) -> int:
    """Device address of a tensor-like object (or an int address, or None)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _host(a: np.ndarray) -> int:
    return a.ctypes.data


def quantize_rows(w: np.ndarray, act_absmax: Optional[np.ndarray] = None, alpha: float = 0.5,
                  prune_abs: int = 1) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """dc_quantize_rows: fp32 W[rows, cols] -> (int8 q, fp32 row_scale[rows], fp32 col_scale[cols])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    rows, cols = w.shape
    a = None if act_absmax is None else np.ascontiguousarray(act_absmax, dtype=np.float32)
    if a is not None and a.shape != (cols,):
        raise ValueError("act_absmax must have one value per column")
    q = np.empty((rows, cols), dtype=np.int8)
    rs = np.empty(rows, dtype=np.float32)
    cs = np.empty(cols, dtype=np.float32)
    _check(_L.dc_quantize_rows(_host(w), rows, cols, None if a is None else _host(a), float(alpha),
                               int(prune_abs), _host(q), _host(rs), _host(cs)), "dc_quantize_rows")
    return q, rs, cs


def quantize_tensor(w: np.ndarray, act_absmax: Optional[np.ndarray] = None, alpha: float = 0.5,
                    sparsity: float = 0.0) -> Tuple[np.ndarray, float, np.ndarray]:
    """dc_quantize_tensor: fp32 W[rows, cols] -> (int8 q, fp32 tensor scale, fp32 col_scale[cols])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    rows, cols = w.shape
    a = None if act_absmax is None else np.ascontiguousarray(act_absmax, dtype=np.float32)
    if a is not None and a.shape != (cols,):
        raise ValueError("act_absmax must have one value per column")
    q = np.empty((rows, cols), dtype=np.int8)
    ts = np.empty(1, dtype=np.float32)
    cs = np.empty(cols, dtype=np.float32)
    _check(_L.dc_quantize_tensor(_host(w), rows, cols, None if a is None else _host(a), float(alpha),
                                 float(sparsity), _host(q), _host(ts), _host(cs)), "dc_quantize_tensor")
    return q, float(ts[0]), cs


def compress_bound(raw_bytes: int, params: Params) -> Tuple[int, int]:
    cap, nc = C.c_uint64(0), C.c_uint64(0)
    cp = params._c()
    _check(_L.dc_compress_bound(raw_bytes, C.byref(cp), C.byref(cap), C.byref(nc)), "dc_compress_bound")
    return int(cap.value), int(nc.value)


def compress_chunks(src: np.ndarray, params: Params) -> Tuple[np.ndarray, np.ndarray]:
    """dc_compress_chunks: int8/uint8 array -> (blob uint8[blob_bytes], table CHUNK_DTYPE[n_chunks])."""
    s = np.ascontiguousarray(src).view(np.uint8).reshape(-1)
    cap, nc = compress_bound(s.size, params)
    blob = np.empty(cap, dtype=np.uint8)
    table = np.zeros(nc, dtype=CHUNK_DTYPE)
    used, n_out = C.c_uint64(0), C.c_uint64(0)
    cp = params._c()
    _check(_L.dc_compress_chunks(_host(s), s.size, C.byref(cp), _host(blob), cap, C.byref(used), _host(table),
                                 nc, C.byref(n_out)), "dc_compress_chunks")
    return blob[:used.value].copy(), table[:n_out.value]


def compress_chunks_dev_workspace(raw_bytes: int, params: Params) -> int:
    n = C.c_uint64(0)
    cp = params._c()
    _check(_L.dc_compress_chunks_dev_workspace(raw_bytes, C.byref(cp), C.byref(n)), "dc_compress_chunks_dev_workspace")
    return int(n.value)


def compress_chunks_dev(src_dev, raw_bytes: int, params: Params, blob_dev, blob_cap: int, table_dev, table_cap: int,
                        workspace_dev, workspace_bytes: int, result_dev, stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_compress_chunks_dev(_dev(src_dev), raw_bytes, C.byref(cp), _dev(blob_dev), blob_cap, _dev(table_dev),
                                     table_cap, _dev(workspace_dev), workspace_bytes, _dev(result_dev), stream),
           "dc_compress_chunks_dev")


def compress_chunks_dev_static(src_dev, raw_bytes: int, params: Params, blob_dev, blob_cap: int, table_dev,
                               table_cap: int, result_dev, stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_compress_chunks_dev_static(_dev(src_dev), raw_bytes, C.byref(cp), _dev(blob_dev), blob_cap,
                                            _dev(table_dev), table_cap, _dev(result_dev), stream),
           "dc_compress_chunks_dev_static")


def blob_trailer(blob: np.ndarray) -> Params:
    """dc_blob_trailer on the last 16 bytes of a blob in host memory: the parameters a reader needs."""
    t = np.ascontiguousarray(np.asarray(blob, dtype=np.uint8).reshape(-1)[-16:])
    cp = _CParams()
    _check(_L.dc_blob_trailer(_host(t), C.byref(cp)), "dc_blob_trailer")
    return Params(cp.chunk_bytes, cp.n_streams, codec=cp.codec, format=cp.format)


def validate(blob: np.ndarray, table: np.ndarray, params: Params) -> None:
    """dc_validate: raises DCError(DC_E_FORMAT) naming the first bad chunk."""
    b = np.ascontiguousarray(blob, dtype=np.uint8)
    t = np.ascontiguousarray(table, dtype=CHUNK_DTYPE)
    bad = C.c_uint64(0)
    cp = params._c()
    rc = _L.dc_validate(_host(b), b.size, _host(t), t.size, C.byref(cp), C.byref(bad))
    if rc != 0:
        raise DCError(rc, f"dc_validate (chunk {bad.value})")


def decompress_chunks(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, dst_dev,
                      dst_cap: int, stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_decompress_chunks(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp),
                                   _dev(dst_dev), dst_cap, stream), "dc_decompress_chunks")


def issue_rate_names() -> list:
    return [_L.dc_issue_rate_name(i).decode() for i in range(_L.dc_issue_rate_count())]


def issue_rate(which: int, sink_dev, sink_bytes: int, stream: int = 0) -> float:
    """ns from one wavefront instruction to the next on a SIMD, for instruction number `which`."""
    ns = C.c_double(0.0)
    _check(_L.dc_issue_rate(which, _dev(sink_dev), sink_bytes, stream, C.byref(ns)), "dc_issue_rate")
    return ns.value


def decompress_chunks_traced(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, dst_dev,
                             dst_cap: int, trace_dev, stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_decompress_chunks_traced(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp),
                                          _dev(dst_dev), dst_cap, _dev(trace_dev), stream), "dc_decompress_chunks_traced")


def decompress_dequant_bf16(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, row_scale_dev,
                            rows: int, cols: int, dst_bf16_dev, dst_cap_elems: int, stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_decompress_dequant_bf16(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp),
                                         _dev(row_scale_dev), rows, cols, _dev(dst_bf16_dev), dst_cap_elems,
                                         stream), "dc_decompress_dequant_bf16")


def decompress_gemv_workspace(n_chunks: int) -> int:
    n = C.c_uint64(0)
    _check(_L.dc_decompress_gemv_workspace(n_chunks, C.byref(n)), "dc_decompress_gemv_workspace")
    return int(n.value)


def decompress_gemv(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, row_scale_dev,
                    rows: int, cols: int, x_bf16_dev, y_f32_dev, y_bf16_dev, workspace_dev, workspace_bytes: int,
                    stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_decompress_gemv(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp),
                                 _dev(row_scale_dev), rows, cols, _dev(x_bf16_dev), _dev(y_f32_dev),
                                 _dev(y_bf16_dev), _dev(workspace_dev), workspace_bytes, stream), "dc_decompress_gemv")


def _matrices(mats):
    arr = (_CMatrix * len(mats))()
    for i, m in enumerate(mats):
        arr[i] = _CMatrix(m.first_chunk, m.rows, m.cols, _dev(m.row_scale_dev) or None, _dev(m.dst_bf16_dev) or None,
                          m.dst_cap_elems, _dev(m.x_bf16_dev) or None, _dev(m.y_accum_dev) or None,
                          _dev(m.y_bf16_dev) or None, _dev(m.x_i8_dev) or None, float(m.x_scale))
    return arr


def decompress_dequant_bf16_layer(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, mats,
                                  stream: int = 0) -> None:
    cp = params._c()
    arr = _matrices(mats)
    _check(_L.dc_decompress_dequant_bf16_layer(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp),
                                               arr, len(mats), stream), "dc_decompress_dequant_bf16_layer")


def decompress_gemv_layer(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, mats,
                          workspace_dev, workspace_bytes: int, stream: int = 0) -> None:
    cp = params._c()
    arr = _matrices(mats)
    _check(_L.dc_decompress_gemv_layer(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp), arr,
                                       len(mats), _dev(workspace_dev), workspace_bytes, stream),
           "dc_decompress_gemv_layer")


def gemv_i8(q_dev, row_scale_dev, rows: int, cols: int, x_bf16_dev, y_f32_dev, y_bf16_dev=None, stream: int = 0) -> None:
    _check(_L.dc_gemv_i8(_dev(q_dev), _dev(row_scale_dev), rows, cols, _dev(x_bf16_dev), _dev(y_f32_dev),
                         _dev(y_bf16_dev), stream), "dc_gemv_i8")


def decompress_gemv_w8a8(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, row_scale_dev,
                         rows: int, cols: int, x_i8_dev, x_scale: float, y_accum_dev, y_bf16_dev=None,
                         stream: int = 0) -> None:
    cp = params._c()
    _check(_L.dc_decompress_gemv_w8a8(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp),
                                      _dev(row_scale_dev), rows, cols, _dev(x_i8_dev), float(x_scale), _dev(y_accum_dev),
                                      _dev(y_bf16_dev), stream), "dc_decompress_gemv_w8a8")


def decompress_gemv_w8a8_layer(blob_dev, blob_bytes: int, table_dev, n_chunks: int, params: Params, mats,
                               stream: int = 0) -> None:
    cp = params._c()
    arr = _matrices(mats)
    _check(_L.dc_decompress_gemv_w8a8_layer(_dev(blob_dev), blob_bytes, _dev(table_dev), n_chunks, C.byref(cp), arr,
                                            len(mats), stream), "dc_decompress_gemv_w8a8_layer")


def gemv_w8a8(q_dev, row_scale_dev, rows: int, cols: int, x_i8_dev, x_scale: float, y_f32_dev, y_bf16_dev=None,
              stream: int = 0) -> None:
    _check(_L.dc_gemv_w8a8(_dev(q_dev), _dev(row_scale_dev), rows, cols, _dev(x_i8_dev), float(x_scale),
                           _dev(y_f32_dev), _dev(y_bf16_dev), stream), "dc_gemv_w8a8")


def quantize_vector(x: np.ndarray) -> Tuple[np.ndarray, float]:
    """dc_quantize_vector: fp32 x[n] -> (int8 xq[n], fp32 scale)."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    xq = np.empty(x.size, dtype=np.int8)
    sc = np.empty(1, dtype=np.float32)
    _check(_L.dc_quantize_vector(_host(x), x.size, _host(xq), _host(sc)), "dc_quantize_vector")
    return xq, float(sc[0])


def device_copy(src_dev, dst_dev, nbytes: int, stream: int = 0) -> None:
    _check(_L.dc_device_copy(_dev(src_dev), _dev(dst_dev), nbytes, stream), "dc_device_copy")
