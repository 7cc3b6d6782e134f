"""GPU parity at the full sizes of the workloads, in the launch configurations bench.py times.

Whole outputs are compared with the oracle-quantised bytes (the decode of a lossless code has one
right answer); in addition the oracle decodes sampled chunks of the very blob the GPU decoded.
"""
import numpy as np
import pytest

import oracle.codec as oc
import oracle.quant as oq
import paper_2502_15443_amd as dc
import synth
from tests.helpers import gemv_workspace, oracle_matrix, weightlike_bytes

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).cuda()


def stream():
    return torch.cuda.current_stream().cuda_stream


def oracle_layer(kind: str, layer: int, rescale: bool):
    """[(spec, q int8[rows, cols], row_scale)] of one decoder layer, quantised by the oracle."""
    out = []
    for m in synth.layer_specs(kind):
        q, scale = oracle_matrix(m.rows, m.cols, synth.matrix_seed(layer, m.index), rescale)
        out.append((m, q, scale))
    return out


def compress_concat(qs, params):
    """Library compression matrix by matrix, blobs and tables concatenated (as bench.py does)."""
    blobs, tables, off = [], [], 0
    for q in qs:
        blob, table = dc.compress_chunks(q, params)
        table = table.copy()
        table["off"] += off
        off += blob.size
        blobs.append(blob)
        tables.append(table)
    return np.concatenate(blobs), np.concatenate(tables)


def check_sampled_chunks_with_oracle(blob, table, C, S, flat, ks, codec=oc.HUFFMAN):
    for k in ks:
        t = table[k:k + 1].copy()
        raw = int(t["raw_bytes_flags"][0] & 0x7FFFFFFF)
        ref = oc.decompress(blob, t, C, S, raw, codec=codec)
        assert np.array_equal(ref, flat[k * C:k * C + raw]), k


def gpu_decode(blob, table, params, n):
    blob_d, table_d = dev(blob), dev(table)
    dst = torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, blob.size, table_d, len(table), params, dst, n, stream())
    torch.cuda.synchronize()
    return dst.cpu().numpy()


@pytest.mark.parametrize("S", [256, 64])
def test_config2_llama7b_layer_one_launch(S):
    """The benchmark's launch: 3088 chunks of 64 KiB of the compression-aware quantised layer."""
    print(f"case config 2 S={S}", flush=True)
    layer = oracle_layer("llama7b", 0, True)
    C = 65536
    p = dc.Params(C, S)
    # the library's quantiser must give the oracle's bytes and scales
    m, q_ref, s_ref = layer[4]
    w = synth.gen_weight(m.rows, m.cols, synth.matrix_seed(0, m.index))
    a = synth.gen_act_absmax(m.cols, synth.matrix_seed(0, m.index))
    q_lib, s_lib, _ = dc.quantize_rows(w, a, 0.5, 1)
    assert np.array_equal(q_lib, q_ref) and np.array_equal(s_lib, s_ref)
    blob, table = compress_concat([q for _, q, _ in layer], p)
    flat = np.concatenate([q.reshape(-1) for _, q, _ in layer]).view(np.uint8)
    assert len(table) == 3088 and flat.size == 202375168
    out = gpu_decode(blob, table, p, flat.size)
    assert np.array_equal(out, flat)
    check_sampled_chunks_with_oracle(blob, table, C, S, flat, [0, 255, 256, 1711, 3087])
    # one matrix compressed by the oracle: same bytes, same ratio
    c = oc.compress(layer[0][1], C, S, threads=8)
    b0, t0 = dc.compress_chunks(layer[0][1], p)
    assert np.array_equal(b0, c.blob) and np.array_equal(t0, c.table)


@pytest.mark.parametrize("C,S", [(65536, 256), (262144, 64)])
def test_config2_llama7b_layer_tans_coded(C, S):
    """The same layer through the second coder, in the launches `bench.py` times for it."""
    print(f"case config 2 tANS C={C} S={S}", flush=True)
    layer = oracle_layer("llama7b", 0, True)
    p = dc.Params(C, S, codec=dc.CODEC_TANS)
    blob, table = compress_concat([q for _, q, _ in layer], p)
    flat = np.concatenate([q.reshape(-1) for _, q, _ in layer]).view(np.uint8)
    assert len(table) == 202375168 // C
    out = gpu_decode(blob, table, p, flat.size)
    assert np.array_equal(out, flat)
    check_sampled_chunks_with_oracle(blob, table, C, S, flat, [0, len(table) // 3, len(table) - 1], codec=oc.TANS)
    c = oc.compress(layer[0][1], C, S, threads=8, codec=oc.TANS)
    b0, t0 = dc.compress_chunks(layer[0][1], p)
    assert np.array_equal(b0, c.blob) and np.array_equal(t0, c.table)


@pytest.mark.parametrize("C,S", [(16384, 64), (65536, 64), (262144, 64), (16384, 256), (262144, 256)])
def test_config3_layers_into_one_buffer_chunk_sweep(C, S):
    """Four layers of the 32-layer weight set (the first two and the last two; per-layer seeds, no rescale)
    decoded into one buffer by one launch, for the chunk sizes of the sweep.  (bench.py decodes all 32 in its
    timed launch and compares every byte with the quantised input.)"""
    print(f"case config 3 C={C} S={S}", flush=True)
    qs = []
    for layer in (0, 1, 30, 31):
        qs += [q for _, q, _ in oracle_layer("llama7b", layer, False)]
    p = dc.Params(C, S)
    blob, table = compress_concat(qs, p)
    flat = np.concatenate([q.reshape(-1) for q in qs]).view(np.uint8)
    assert len(table) == 4 * 202375168 // C
    out = gpu_decode(blob, table, p, flat.size)
    assert np.array_equal(out, flat)
    check_sampled_chunks_with_oracle(blob, table, C, S, flat, [0, len(table) // 4, len(table) // 2, len(table) - 1])


@pytest.mark.parametrize("f", [0.0, 0.25, 0.5, 0.75, 1.0])
def test_config4_raw_fraction_on_config1_matrix(f):
    print(f"case config 4 f={f}", flush=True)
    q, _ = oracle_matrix(4096, 4096, synth.matrix_seed(0, 0), False)
    C, S = 65536, 32
    p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, f)
    blob, table = dc.compress_chunks(q, p)
    c = oc.compress(q, C, S, oc.RAW_FRACTION, f, threads=8)
    assert np.array_equal(blob, c.blob) and np.array_equal(table, c.table)
    is_raw = (table["raw_bytes_flags"] & dc.CHUNK_RAW) != 0
    assert int(is_raw.sum()) == int(f * 256)
    # closed form of the ratio: coded payloads + raw chunks + table + closing bytes
    size = int(table["comp_bytes"].sum()) + 64 + table.nbytes
    assert blob.size + table.nbytes == size and int(table["comp_bytes"][is_raw].sum()) == int(is_raw.sum()) * C
    if f == 1.0:
        assert q.size / size < 1.0
    out = gpu_decode(blob, table, p, q.size)
    assert np.array_equal(out, q.view(np.uint8).ravel())


@pytest.mark.parametrize("index", [0, 4, 6])
def test_config5_llama13b_fused_paths(index):
    """q_proj (5120x5120), gate_proj (13824x5120) and down_proj (5120x13824) of the 13B-shaped layer:
    fused GEMV against the fp64 reference on every row, fused bf16 dequantisation bit for bit on every element
    (the oracle's result is uploaded and compared on the device)."""
    print(f"case config 5 matrix {index}", flush=True)
    m = synth.layer_specs("llama13b")[index]
    seed = synth.matrix_seed(0, m.index)
    q, scale = oracle_matrix(m.rows, m.cols, seed, False)
    C, S = 65536, 256
    p = dc.Params(C, S)
    blob, table = dc.compress_chunks(q, p)
    blob_d, table_d, scale_d = dev(blob), dev(table), torch.from_numpy(scale).cuda()
    x = synth.gen_activation_bf16(m.cols, seed)
    x_d = torch.from_numpy(x.view(np.int16)).cuda()
    y32 = torch.empty(m.rows, dtype=torch.float32, device="cuda")
    y16 = torch.empty(m.rows, dtype=torch.int16, device="cuda")
    dc.decompress_gemv(blob_d, blob.size, table_d, len(table), p, scale_d, m.rows, m.cols, x_d, y32, y16,
                       *gemv_workspace(len(table)), stream())
    out16 = torch.empty(q.size, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, blob.size, table_d, len(table), p, scale_d, m.rows, m.cols, out16, q.size,
                               stream())
    torch.cuda.synchronize()
    y_ref = oq.gemv_ref(q, scale, x)
    y = y32.cpu().numpy().astype(np.float64)
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    assert (np.abs(y - y_ref) <= 1e-2 * np.abs(y_ref) + 1e-2 * rms).all()
    yb = oq.bf16_to_f64(y16.cpu().numpy().view(np.uint16))
    assert (np.abs(yb - y_ref) <= 1e-2 * np.abs(y_ref) + 1e-2 * rms).all()
    want = torch.from_numpy(oq.dequant_bf16(q, scale).view(np.int16).reshape(-1)).cuda()
    assert torch.equal(out16, want)


def test_config5_whole_layer_in_one_fused_call():
    """All seven matrices of the 13B-shaped layer through one dc_decompress_gemv_layer and one
    dc_decompress_dequant_bf16_layer call: same results as matrix by matrix."""
    print("case config 5 whole layer", flush=True)
    layer = oracle_layer("llama13b", 0, False)
    C, S = 65536, 256
    p = dc.Params(C, S)
    blob, table = compress_concat([q for _, q, _ in layer], p)
    blob_d, table_d = dev(blob), dev(table)
    mats_g, mats_b, keep = [], [], []
    k0 = 0
    for m, q, scale in layer:
        seed = synth.matrix_seed(0, m.index)
        x = synth.gen_activation_bf16(m.cols, seed)
        x_d = torch.from_numpy(x.view(np.int16)).cuda()
        s_d = torch.from_numpy(scale).cuda()
        y32 = torch.full((m.rows,), 3.0, dtype=torch.float32, device="cuda")
        y16 = torch.zeros(m.rows, dtype=torch.int16, device="cuda")
        o16 = torch.zeros(q.size, dtype=torch.int16, device="cuda")
        mats_g.append(dc.Matrix(k0, m.rows, m.cols, s_d, x_bf16_dev=x_d, y_accum_dev=y32, y_bf16_dev=y16))
        mats_b.append(dc.Matrix(k0, m.rows, m.cols, s_d, dst_bf16_dev=o16, dst_cap_elems=q.size))
        keep.append((m, q, scale, x, y32, y16, o16))
        k0 += q.size // C
    assert k0 == len(table) == 4840
    dc.decompress_gemv_layer(blob_d, blob.size, table_d, len(table), p, mats_g, *gemv_workspace(len(table)), stream())
    dc.decompress_dequant_bf16_layer(blob_d, blob.size, table_d, len(table), p, mats_b, stream())
    torch.cuda.synchronize()
    for m, q, scale, x, y32, y16, o16 in keep:
        y_ref = oq.gemv_ref(q, scale, x)
        rms = float(np.sqrt(np.mean(y_ref ** 2)))
        y = y32.cpu().numpy().astype(np.float64)
        assert (np.abs(y - y_ref) <= 1e-2 * np.abs(y_ref) + 1e-2 * rms).all(), m.name
        assert np.abs(y - y_ref).max() / np.abs(y_ref).max() < 1e-4
        assert np.array_equal(y16.cpu().numpy().view(np.uint16), oq.bf16_round(y32.cpu().numpy()))
        want = torch.from_numpy(oq.dequant_bf16(q, scale).view(np.int16).reshape(-1)).cuda()
        assert torch.equal(o16, want), m.name
    # descriptor errors are caught on the host
    bad = [dc.Matrix(mm.first_chunk + 1, mm.rows, mm.cols, mm.row_scale_dev, x_bf16_dev=mm.x_bf16_dev,
                     y_accum_dev=mm.y_accum_dev) for mm in mats_g]
    with pytest.raises(dc.DCError):
        dc.decompress_gemv_layer(blob_d, blob.size, table_d, len(table), p, bad, *gemv_workspace(len(table)), stream())
    with pytest.raises(dc.DCError):
        dc.decompress_gemv_layer(blob_d, blob.size, table_d, len(table), p, mats_g[:-1], *gemv_workspace(len(table)),
                                 stream())


@pytest.mark.parametrize("codec", [oc.HUFFMAN, oc.TANS])
def test_offsets_beyond_4_gib_in_blob_and_destination(codec):
    """64-bit arithmetic of the launch: 4104 chunks of the largest chunk size (1 MiB) decode into 4.3 GB, from
    a blob whose payloads lie on both sides of the 4 GiB mark.  The table refers to nine payloads the oracle
    wrote (two of them raw, the last one ragged) over and over — the kernel takes every entry on its own —
    and every decoded chunk is compared on the device."""
    C, S = 1 << 20, 256
    n_chunks, tail = 4104, 12345
    print(f"case beyond 4 GiB codec={codec}", flush=True)
    data = weightlike_bytes(8 * C + tail, 9090 + codec)
    mask = np.zeros(9, np.uint8)
    mask[[2, 5]] = 1
    c = oc.compress(data, C, S, oc.RAW_MASK, mask=mask, threads=8, codec=codec)
    assert c.n_chunks == 9 and int(((c.table["raw_bytes_flags"] >> 31) & 1).sum()) == 2
    high = (1 << 32) + 4096
    blob_bytes = high + c.blob.size
    blob_d = torch.zeros(blob_bytes, dtype=torch.uint8, device="cuda")
    table = np.zeros(n_chunks, dtype=c.table.dtype)
    place = {}
    low_end = 0
    for r in range(9):
        off, size = int(c.table["off"][r]), int(c.table["comp_bytes"][r])
        padded = (size + 15) // 16 * 16
        base = low_end if r % 2 == 0 else high + off
        if r % 2 == 0:
            low_end += padded
        blob_d[base:base + size] = torch.from_numpy(c.blob[off:off + size].copy()).cuda()
        place[r] = base
    blob_d[blob_bytes - 64:] = torch.from_numpy(c.blob[-64:].copy()).cuda()  # the closing bytes with the trailer
    for k in range(n_chunks):
        r = 8 if k == n_chunks - 1 else k % 8
        table[k] = (place[r], c.table["comp_bytes"][r], c.table["raw_bytes_flags"][r])
    n = (n_chunks - 1) * C + tail
    assert n > 1 << 32 and max(place.values()) > 1 << 32
    table_d = dev(table.view(np.uint8))
    dst = torch.full((n + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, blob_bytes, table_d, n_chunks, dc.Params(C, S, codec=codec), dst, n, stream())
    torch.cuda.synchronize()
    src_d = torch.from_numpy(data).cuda()
    rows = dst[:(n_chunks - 1) * C].view(n_chunks - 1, C)
    for r in range(8):
        assert bool((rows[r::8] == src_d[r * C:(r + 1) * C]).all()), f"payload {r}"
    assert torch.equal(dst[(n_chunks - 1) * C:n], src_d[8 * C:])
    assert bool((dst[n:] == 0x5A).all())


def test_fused_calls_on_a_matrix_beyond_4_gib():
    """The fused epilogues on a 524 800 x 8192 matrix (4.3 G weights, 8.6 GB of bf16): 4100 chunks of 1 MiB
    whose table refers to eight payloads of the oracle in turn, so the weights repeat every 1024 rows while
    the row scales do not.  Dequantised rows are compared with the oracle on sampled chunks (first, around the
    element 2^32, last); the bf16 product against the fp64 reference and the integer product bit for bit, on
    every row (the references are those of the 1024 distinct rows times each row's scale)."""
    C, S = 1 << 20, 256
    n_chunks, cols = 4100, 8192
    rows, rows_per_chunk = n_chunks * C // cols, C // cols
    print(f"case fused beyond 4 GiB rows={rows} cols={cols}", flush=True)
    data = weightlike_bytes(8 * C, 9191)
    data[data == 0x80] = 0x81            # int8 weights never hold -128
    c = oc.compress(data, C, S, threads=8)
    table = np.zeros(n_chunks, dtype=c.table.dtype)
    for k in range(n_chunks):
        table[k] = c.table[k % 8]
    q8 = data.view(np.int8).reshape(8 * rows_per_chunk, cols)
    scale = (np.random.default_rng(5).random(rows, dtype=np.float32) + np.float32(0.5)) * np.float32(0.01)
    blob_d, table_d, scale_d = dev(c.blob), dev(table.view(np.uint8)), torch.from_numpy(scale).cuda()
    p = dc.Params(C, S)
    n = rows * cols
    assert n > 1 << 32

    out16 = torch.zeros(n, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, n_chunks, p, scale_d, rows, cols, out16, n, stream())
    torch.cuda.synchronize()
    for k in (0, 1, (1 << 32) // C - 1, (1 << 32) // C, (1 << 32) // C + 3, n_chunks - 1):
        r0 = k * rows_per_chunk
        got = out16[k * C:(k + 1) * C].cpu().numpy().view(np.uint16).reshape(rows_per_chunk, cols)
        qk = q8[(k % 8) * rows_per_chunk:(k % 8 + 1) * rows_per_chunk]
        assert np.array_equal(got, oq.dequant_bf16(qk, scale[r0:r0 + rows_per_chunk])), f"chunk {k}"
    del out16

    x = synth.gen_activation_bf16(cols, 321)
    y32 = torch.full((rows + 16,), 7.0, dtype=torch.float32, device="cuda")
    dc.decompress_gemv(blob_d, c.blob.size, table_d, n_chunks, p, scale_d, rows, cols,
                       torch.from_numpy(x.view(np.int16)).cuda(), y32, None, *gemv_workspace(n_chunks), stream())
    xq, sx = oq.quantise_vector(np.random.default_rng(6).standard_normal(cols).astype(np.float32))
    z32 = torch.full((rows + 16,), 7.0, dtype=torch.float32, device="cuda")
    dc.decompress_gemv_w8a8(blob_d, c.blob.size, table_d, n_chunks, p, scale_d, rows, cols,
                            torch.from_numpy(xq).cuda(), float(sx), z32, None, stream())
    torch.cuda.synchronize()
    which = np.arange(rows) % q8.shape[0]
    y_ref = oq.gemv_ref(q8, np.ones(q8.shape[0], np.float32), x)[which] * scale.astype(np.float64)
    y = y32.cpu().numpy()
    err = np.abs(y[:rows].astype(np.float64) - y_ref)
    assert (err <= 1e-2 * np.abs(y_ref) + 1e-2 * float(np.sqrt(np.mean(y_ref ** 2)))).all() and (y[rows:] == 7.0).all()
    acc = oq.gemv_w8a8_acc(q8, xq)[which]
    z_ref = (acc.astype(np.float32) * scale) * np.float32(sx)
    z = z32.cpu().numpy()
    assert np.array_equal(z[:rows].view(np.uint32), z_ref.view(np.uint32)) and (z[rows:] == 7.0).all()
