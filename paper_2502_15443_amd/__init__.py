"""MI355X-native decode path of the double-compression method (arXiv 2502.15443).

Thin Python binding over the C-ABI library libdc_mi355x.so (see include/dc.h).  Every step of the
path runs inside the library (host C++ for quantise/compress/validate, HIP kernels for the decode
calls); this package only marshals arguments.  There is no CPU fallback: if the library is missing
the import of the binding fails.
"""
from .binding import (  # noqa: F401
    DCError,
    Params,
    CHUNK_DTYPE,
    CODEC_HUFFMAN,
    CODEC_TANS,
    FORMAT_ID,
    POLICY_ALL_HUFF,
    POLICY_AUTO,
    POLICY_RAW_FRACTION,
    POLICY_RAW_MASK,
    POLICY_BLOCK_LAST,
    CHUNK_RAW,
    STATIC_SCRATCH_BYTES,
    lib_path,
    version,
    set_num_threads,
    quantize_rows,
    quantize_tensor,
    compress_bound,
    compress_chunks,
    compress_chunks_dev,
    compress_chunks_dev_workspace,
    compress_chunks_dev_static,
    validate,
    blob_trailer,
    decompress_chunks,
    decompress_dequant_bf16,
    decompress_gemv,
    decompress_gemv_workspace,
    decompress_dequant_bf16_layer,
    decompress_gemv_layer,
    Matrix,
    gemv_i8,
    decompress_gemv_w8a8,
    decompress_gemv_w8a8_layer,
    gemv_w8a8,
    quantize_vector,
    device_copy,
)
