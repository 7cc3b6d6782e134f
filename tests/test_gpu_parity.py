"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

Bar: decoded int8 bytes and bf16 dequantised values are bit-exact; fused GEMV outputs satisfy
|y - y_ref| <= 1e-2*|y_ref| + 1e-2*rms(y_ref) against the fp64 reference.
"""
import numpy as np
import pytest

import oracle.codec as oc
import oracle.quant as oq
import paper_2502_15443_amd as dc
import synth
from tests.helpers import gemv_workspace, lopsided_bytes, oracle_matrix, weightlike_bytes

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()


def stream():
    return torch.cuda.current_stream().cuda_stream


def gpu_decode(blob, table, params, n, fill=0xAB):
    blob_d, table_d = dev(blob), dev(table)
    dst = torch.full((n,), fill, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, blob.size, table_d, len(table), params, dst, n, stream())
    torch.cuda.synchronize()
    return dst.cpu().numpy()


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("n,C", [(3 * 65536, 65536), (5 * 16384 + 777, 16384), (7 * 4096 + 4095, 4096),
                                 (65536 + 16, 65536), (100, 65536), (1, 4096), (9 * 2048 + 1, 2048),
                                 (2 * 262144 + 12345, 262144)])
def test_decode_matches_oracle_bytes(S, n, C):
    print(f"case S={S} n={n} C={C}", flush=True)
    data = weightlike_bytes(n, 1000 + n % 977 + S)
    c = oc.compress(data, C, S)  # the oracle's blob
    out = gpu_decode(c.blob, c.table, dc.Params(C, S), n)
    assert np.array_equal(out, data)
    assert np.array_equal(out, oc.decompress(c.blob, c.table, C, S, n))


@pytest.mark.parametrize("S", [32, 64, 128, 256])
def test_decode_degenerate_chunks(S):
    print(f"case degenerate S={S}", flush=True)
    C = 4096
    r = np.random.default_rng(0)
    skew = np.clip(np.rint(r.standard_cauchy(C) * 2), -127, 127).astype(np.int8).view(np.uint8)  # 11-bit codes
    data = np.concatenate([np.zeros(C, np.uint8), np.full(C, 0x81, np.uint8), r.integers(0, 256, C, dtype=np.uint8),
                           np.tile(np.array([3, 250], np.uint8), C // 2), np.arange(C, dtype=np.uint32).astype(np.uint8),
                           skew, np.array([7], np.uint8)])
    for policy in (oc.ALL_HUFF, oc.AUTO):
        c = oc.compress(data, C, S, policy)
        out = gpu_decode(c.blob, c.table, dc.Params(C, S), data.size)
        assert np.array_equal(out, data)


@pytest.mark.parametrize("S", [32, 64, 128, 256])
def test_decode_lopsided_streams(S):
    """Sub-streams whose positions drift far apart (one all long codes, most all short codes)."""
    print(f"case lopsided S={S}", flush=True)
    C = 65536
    n = 3 * C + 4096 + 50
    data = lopsided_bytes(n, S, 7 + S)
    c = oc.compress(data, C, S)
    assert np.array_equal(gpu_decode(c.blob, c.table, dc.Params(C, S), n), data)


@pytest.mark.parametrize("S", [32, 64])
@pytest.mark.parametrize("f", [0.0, 0.25, 0.5, 0.75, 1.0])
def test_decode_with_raw_fraction(S, f):
    print(f"case raw fraction S={S} f={f}", flush=True)
    C = 16384
    data = weightlike_bytes(41 * C + 333, 17)
    p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, f)
    blob, table = dc.compress_chunks(data, p)  # the library's compressor ...
    c = oc.compress(data, C, S, oc.RAW_FRACTION, f)
    assert np.array_equal(blob, c.blob) and np.array_equal(table, c.table)  # ... equals the oracle's
    assert np.array_equal(gpu_decode(blob, table, p, data.size), data)


def test_decode_block_last_policy():
    C, S = 8192, 32
    data = weightlike_bytes(23 * C, 19)
    c = oc.compress(data, C, S, oc.BLOCK_LAST, block=5)
    assert np.array_equal(gpu_decode(c.blob, c.table, dc.Params(C, S), data.size), data)


@pytest.mark.parametrize("S", [32, 64])
def test_three_longest_codes_on_a_buffer_that_was_just_emptied(S):
    """Three 11-bit codes need 33 bits, one refill of an empty bit buffer gives 32: the decoder must take a
    second word there.  The input is built so that this happens (checked by a walk over the code lengths);
    every decode mode must still give the oracle's result.  Found by a random sweep: one such case in
    about ten thousand chunks of weight-like data."""
    from tests.helpers import emptied_buffer_bytes, empty_buffer_before_three_codes
    data = emptied_buffer_bytes(S)
    assert empty_buffer_before_three_codes(data, S)
    n, C = data.size, data.size
    c = oc.compress(data, C, S)
    assert np.array_equal(gpu_decode(c.blob, c.table, dc.Params(C, S), n), data)
    cols = 16 * S
    rows = n // cols
    q = data.view(np.int8).reshape(rows, cols)
    scale = np.full(rows, 0.0123, np.float32)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    out16 = torch.zeros(n, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, c.n_chunks, dc.Params(C, S), scale_d, rows, cols, out16, n,
                               stream())
    xq = (np.arange(cols) % 5 - 2).astype(np.int8)
    y32 = torch.zeros(rows, dtype=torch.float32, device="cuda")
    dc.decompress_gemv_w8a8(blob_d, c.blob.size, table_d, c.n_chunks, dc.Params(C, S), scale_d, rows, cols,
                            torch.from_numpy(xq).cuda(), 0.5, y32, None, stream())
    torch.cuda.synchronize()
    assert np.array_equal(out16.cpu().numpy().view(np.uint16).reshape(rows, cols), oq.dequant_bf16(q, scale))
    assert np.array_equal(y32.cpu().numpy().view(np.uint32), oq.gemv_w8a8(q, scale, xq, np.float32(0.5)).view(np.uint32))


def test_decode_a_range_of_chunks_of_a_blob():
    """A layer out of a model: the table pointer advanced to the first chunk wanted, the same blob."""
    C, S, n = 4096, 64, 11 * 4096 + 500
    data = weightlike_bytes(n, 31)
    c = oc.compress(data, C, S, oc.RAW_FRACTION, 0.3)
    blob_d, table_d = dev(c.blob), dev(c.table)
    k0, count = 4, 5
    dst = torch.full((count * C + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, c.blob.size, table_d.data_ptr() + 16 * k0, count, dc.Params(C, S), dst, count * C, stream())
    torch.cuda.synchronize()
    out = dst.cpu().numpy()
    assert np.array_equal(out[:count * C], data[k0 * C:(k0 + count) * C]) and (out[count * C:] == 0x5A).all()


def test_destination_untouched_beyond_decoded_bytes():
    C, S, n = 4096, 32, 3 * 4096 + 100
    data = weightlike_bytes(n, 23)
    c = oc.compress(data, C, S)
    blob_d, table_d = dev(c.blob), dev(c.table)
    dst = torch.full((4 * C,), 0x5A, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, c.blob.size, table_d, 4, dc.Params(C, S), dst, 4 * C, stream())
    torch.cuda.synchronize()
    out = dst.cpu().numpy()
    assert np.array_equal(out[:n], data) and (out[n:] == 0x5A).all()


@pytest.mark.parametrize("S,codec", [(32, oc.HUFFMAN), (256, oc.HUFFMAN), (64, oc.TANS)])
def test_blob_of_another_format_is_not_decoded(S, codec):
    """A blob that a writer of format 3 would have closed (look-ahead 320), one without a trailer, one of
    another coder or sub-stream count than the caller says: every decode call leaves its output untouched
    (the kernels compare the blob's last 16 bytes with what the parameters imply), and a caller that states
    another format id is refused on the host with DC_E_FORMAT."""
    print(f"case other format S={S} codec={codec}", flush=True)
    C, rows, cols = 16384, 64, 1024
    q, scale = oracle_matrix(rows, cols, synth.matrix_seed(7, 2), False)
    n = q.size
    c = oc.compress(q, C, S, codec=codec)
    p = dc.Params(C, S, codec=codec)
    scale_d = torch.from_numpy(scale).cuda()
    x_d = torch.from_numpy(synth.gen_activation_bf16(cols, 5).view(np.int16)).cuda()
    old = c.blob.copy()
    old[-12:-8] = np.frombuffer((3).to_bytes(2, "little") + (320).to_bytes(2, "little"), np.uint8)
    bare = c.blob.copy()
    bare[-16:] = 0
    params_differ = [dc.Params(C, 64 if S != 64 else 128, codec=codec), dc.Params(C, max(S, 64), codec=1 - codec),
                     dc.Params(2 * C, S, codec=codec)]
    cases = [(old, p), (bare, p)] + [(c.blob, pp) for pp in params_differ]
    for blob, pp in cases:
        blob_d, table_d = dev(blob), dev(c.table)
        dst = torch.full((2 * n,), 0x5A, dtype=torch.uint8, device="cuda")
        out16 = torch.full((n,), 0x5A5A, dtype=torch.int16, device="cuda")
        dc.decompress_chunks(blob_d, blob.size, table_d, c.n_chunks, pp, dst, 2 * n, stream())
        if pp.chunk_bytes == C:
            dc.decompress_dequant_bf16(blob_d, blob.size, table_d, c.n_chunks, pp, scale_d, rows, cols, out16, n, stream())
        torch.cuda.synchronize()
        assert (dst.cpu().numpy() == 0x5A).all() and (out16.cpu().numpy() == 0x5A5A).all()
    # the blob as it is decodes
    blob_d, table_d = dev(c.blob), dev(c.table)
    dst = torch.full((n,), 0x5A, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, c.blob.size, table_d, c.n_chunks, p, dst, n, stream())
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy(), q.view(np.uint8).ravel())
    stale = dc.Params(C, S, codec=codec, format=4)
    y32 = torch.zeros(rows, dtype=torch.float32, device="cuda")
    calls = [
        lambda: dc.decompress_chunks(blob_d, c.blob.size, table_d, c.n_chunks, stale, dst, n, stream()),
        lambda: dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, c.n_chunks, stale, scale_d, rows, cols,
                                           torch.zeros(n, dtype=torch.int16, device="cuda"), n, stream()),
        lambda: dc.decompress_gemv(blob_d, c.blob.size, table_d, c.n_chunks, stale, scale_d, rows, cols, x_d, y32, None,
                                   *gemv_workspace(c.n_chunks), stream()),
        lambda: dc.decompress_gemv_w8a8(blob_d, c.blob.size, table_d, c.n_chunks, stale, scale_d, rows, cols,
                                        torch.zeros(cols, dtype=torch.int8, device="cuda"), 1.0, y32, None, stream()),
    ]
    for call in calls:
        with pytest.raises(dc.DCError) as e:
            call()
        assert e.value.code == -3


@pytest.mark.parametrize("S", [32, 256])
def test_corrupt_payloads_and_table_entries_stay_inside_the_buffers(S):
    """Whatever the payloads and the table hold, the kernels read inside the blob and write inside the
    destination (the header of the library promises it; dc_validate is what reports the damage): chunks
    with damaged headers or random payloads give unspecified bytes for those chunks only, chunks with
    impossible table entries are skipped, the others decode, and the guard bytes stay."""
    print(f"case corrupt S={S}", flush=True)
    C = 16384
    n = 12 * C
    rows, cols = 12 * 16, 1024
    q, scale = oracle_matrix(rows, cols, synth.matrix_seed(5, 1), False)
    data = q.view(np.uint8).ravel()
    c = oc.compress(data, C, S)
    blob, table = c.blob.copy(), c.table.copy()
    r = np.random.default_rng(99 + S)
    off = [int(o) for o in table["off"]]
    size = [int(x) for x in table["comp_bytes"]]
    blob[off[1]:off[1] + 128] = r.integers(0, 256, 128, dtype=np.uint8)                  # code lengths
    blob[off[2] + 128:off[2] + 128 + 2 * S] = r.integers(0, 256, 2 * S, dtype=np.uint8)  # blocks and words per stream
    blob[off[3] + 128 + 2 * S:off[3] + 132 + 2 * S] = 0xFF                               # area offset far outside
    blob[off[4]:off[4] + size[4]] = r.integers(0, 256, size[4], dtype=np.uint8)           # everything
    blob[off[5]:off[5] + 128] = 0x11                                                      # 256 codes of one bit
    blob[off[6]:off[6] + 128] = 0                                                         # no code at all
    table["off"][7] += 4                                 # misaligned
    table["comp_bytes"][8] = 1 << 30                     # beyond the blob
    table["raw_bytes_flags"][9] = C + 16                 # longer than a chunk
    table["off"][10] = 1 << 40                           # beyond the blob
    good = [0, 11]
    blob_d, table_d, scale_d = dev(blob), dev(table), torch.from_numpy(scale).cuda()
    p = dc.Params(C, S)

    dst = torch.full((n + 4096,), 0x5A, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, blob.size, table_d, 12, p, dst, n, stream())
    torch.cuda.synchronize()
    out = dst.cpu().numpy()
    assert (out[n:] == 0x5A).all()
    for k in good:
        assert np.array_equal(out[k * C:(k + 1) * C], data[k * C:(k + 1) * C])
    for k in (7, 8, 9, 10):
        assert (out[k * C:(k + 1) * C] == 0x5A).all()  # skipped

    out16 = torch.full((n + 4096,), 0x5A5A, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, blob.size, table_d, 12, p, scale_d, rows, cols, out16, n, stream())
    torch.cuda.synchronize()
    got = out16.cpu().numpy().view(np.uint16)
    assert (got[n:] == 0x5A5A).all()
    want = oq.dequant_bf16(q, scale).ravel()
    for k in good:
        assert np.array_equal(got[k * C:(k + 1) * C], want[k * C:(k + 1) * C])

    x = synth.gen_activation_bf16(cols, 3)
    x_d = torch.from_numpy(x.view(np.int16)).cuda()
    y32 = torch.full((rows + 64,), 7.0, dtype=torch.float32, device="cuda")
    dc.decompress_gemv(blob_d, blob.size, table_d, 12, p, scale_d, rows, cols, x_d, y32, None, *gemv_workspace(12), stream())
    torch.cuda.synchronize()
    y = y32.cpu().numpy()
    assert (y[rows:] == 7.0).all()
    y_ref = oq.gemv_ref(q, scale, x)
    rows_of = lambda k: slice(k * C // cols, (k + 1) * C // cols)
    for k in good:
        gemv_check(y[rows_of(k)], y_ref[rows_of(k)])


def test_host_argument_checks_on_device_entry_points():
    C, S, n = 4096, 32, 2 * 4096
    data = weightlike_bytes(n, 29)
    c = oc.compress(data, C, S)
    blob_d, table_d = dev(c.blob), dev(c.table)
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    with pytest.raises(dc.DCError) as e:
        dc.decompress_chunks(blob_d, c.blob.size, table_d, 2, dc.Params(C, S), dst, C, stream())
    assert e.value.code == -2
    with pytest.raises(dc.DCError) as e:
        dc.decompress_chunks(blob_d, c.blob.size, table_d, 2, dc.Params(C, 48), dst, n, stream())
    assert e.value.code == -1
    with pytest.raises(dc.DCError) as e:
        dc.decompress_chunks(blob_d.data_ptr() + 4, c.blob.size - 4, table_d, 2, dc.Params(C, S), dst, n, stream())
    assert e.value.code == -1


# ------------------------------------------------------------------ matrices: configs at reduced and full size

def matrix_case(rows, cols, seed, rescale, C, S):
    q, scale = oracle_matrix(rows, cols, seed, rescale)
    c = oc.compress(q, C, S, threads=8)
    return q, scale, c


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("rows,cols,rescale", [(160, 1024, False), (96, 2752, True), (33, 5120, False)])
def test_dequant_bf16_bit_exact(S, rows, cols, rescale):
    print(f"case bf16 S={S} {rows}x{cols}", flush=True)
    C = 16384
    q, scale, c = matrix_case(rows, cols, synth.matrix_seed(1, 4), rescale, C, S)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    out = torch.zeros(rows * cols, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, c.n_chunks, dc.Params(C, S), scale_d, rows, cols, out,
                               rows * cols, stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16).reshape(rows, cols)
    assert np.array_equal(got, oq.dequant_bf16(q, scale))


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("rows,cols,C,f", [(1, 16784, 16384, 0.0), (3, 5488, 4096, 0.5), (67, 1040, 65536, 0.0),
                                           (40, 2752, 16384, 1.0)])
def test_dequant_bf16_ragged_ends_and_raw_chunks(S, rows, cols, C, f):
    """Last chunks that end inside a 16-lane row of sub-streams (the lanes of a row and of the next trade
    halves before they store), raw chunks among the coded ones, and nothing written past the matrix."""
    print(f"case bf16 ragged S={S} {rows}x{cols} C={C} f={f}", flush=True)
    q, scale = oracle_matrix(rows, cols, synth.matrix_seed(4, 2), False)
    c = oc.compress(q, C, S, oc.RAW_FRACTION, f)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    n = rows * cols
    out = torch.full((n + 64,), 0x5A5A, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, c.n_chunks, dc.Params(C, S), scale_d, rows, cols, out, n,
                               stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[:n].reshape(rows, cols), oq.dequant_bf16(q, scale))
    assert (got[n:] == 0x5A5A).all()


def gemv_check(y, y_ref):
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    err = np.abs(y.astype(np.float64) - y_ref)
    assert (err <= 1e-2 * np.abs(y_ref) + 1e-2 * rms).all(), float(err.max())
    return float(err.max() / np.abs(y_ref).max())


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("rows,cols,C,f", [(160, 1024, 16384, 0.0), (50, 5120, 65536, 0.0), (37, 13824, 65536, 0.3),
                                           (64, 2752, 16384, 0.5), (24, 8192, 4096, 0.2), (5, 16384, 1024, 0.0),
                                           (2048, 64, 16384, 0.3), (640, 256, 16384, 0.0), (512, 512, 16384, 0.0)])
def test_gemv_within_tolerance(S, rows, cols, C, f):
    print(f"case gemv S={S} {rows}x{cols} C={C} f={f}", flush=True)
    seed = synth.matrix_seed(2, 5)
    q, scale = oracle_matrix(rows, cols, seed, False)
    c = oc.compress(q, C, S, oc.RAW_FRACTION, f)
    x = synth.gen_activation_bf16(cols, seed)
    y_ref = oq.gemv_ref(q, scale, x)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    x_d = torch.from_numpy(x.view(np.int16)).cuda()
    y32 = torch.full((rows,), 7.0, dtype=torch.float32, device="cuda")  # what it holds before the call must not matter
    y16 = torch.zeros(rows, dtype=torch.int16, device="cuda")
    dc.decompress_gemv(blob_d, c.blob.size, table_d, c.n_chunks, dc.Params(C, S), scale_d, rows, cols, x_d, y32, y16,
                       *gemv_workspace(c.n_chunks), stream())
    torch.cuda.synchronize()
    norm_err = gemv_check(y32.cpu().numpy(), y_ref)
    assert norm_err < 1e-4  # fp32 accumulation: far inside the 1e-2 bar
    y16f = oq.bf16_to_f64(y16.cpu().numpy().view(np.uint16))
    gemv_check(y16f, y_ref)
    assert np.array_equal(y16.cpu().numpy().view(np.uint16), oq.bf16_round(y32.cpu().numpy()))


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("codec", [oc.HUFFMAN, oc.TANS])
@pytest.mark.parametrize("rows,cols,C,f", [(50, 5120, 65536, 0.0), (37, 13824, 65536, 0.3), (24, 8192, 4096, 0.2),
                                           (512, 512, 16384, 0.0)])
def test_gemv_same_bits_at_every_run(S, codec, rows, cols, C, f):
    """The fused product adds in a fixed order (a chunk touches at most min(S, 64) rows in these shapes), so
    two runs give the same fp32 bits whatever the workspace held before, and what they give is the sum of
    the workspace's partial sums taken row by row in chunk order."""
    if codec == oc.TANS and S == 32:
        pytest.skip("the tANS payload needs at least 64 sub-streams")
    print(f"case gemv bits S={S} codec={codec} {rows}x{cols} C={C} f={f}", flush=True)
    seed = synth.matrix_seed(4, 1)
    q, scale = oracle_matrix(rows, cols, seed, False)
    c = oc.compress(q, C, S, oc.RAW_FRACTION, f, codec=codec)
    x = synth.gen_activation_bf16(cols, seed)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    x_d = torch.from_numpy(x.view(np.int16)).cuda()
    p = dc.Params(C, S, codec=codec)
    runs = []
    for fill in (0xFF, 0x00, 0x3C):
        ws, ws_bytes = gemv_workspace(c.n_chunks)
        ws.fill_(fill)
        y32 = torch.full((rows + 3,), 7.0, dtype=torch.float32, device="cuda")
        dc.decompress_gemv(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols, x_d, y32, None, ws, ws_bytes,
                           stream())
        torch.cuda.synchronize()
        runs.append((y32.cpu().numpy(), ws.cpu().numpy().view(np.float32).reshape(c.n_chunks, 64)))
    (y0, part), (y1, _), (y2, _) = runs
    assert (y0[rows:] == 7.0).all()
    assert np.array_equal(y0.view(np.uint32), y1.view(np.uint32)) and np.array_equal(y0.view(np.uint32), y2.view(np.uint32))
    gemv_check(y0[:rows], oq.gemv_ref(q, scale, x))
    # the second launch, redone on the host from the partial sums the first one left
    want = np.zeros(rows, np.float32)
    for i in range(rows):
        total = np.float32(0.0)
        for k in range(i * cols // C, ((i + 1) * cols - 1) // C + 1):
            total = np.float32(total + part[k, i - k * C // cols])
        want[i] = np.float32(scale[i] * total)
    assert np.array_equal(want.view(np.uint32), y0[:rows].view(np.uint32))


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("rows,cols,C,f", [(160, 1024, 16384, 0.0), (50, 5120, 65536, 0.0), (37, 13824, 65536, 0.3),
                                           (64, 2752, 16384, 0.5), (3, 16384, 4096, 0.0)])
def test_gemv_w8a8_bit_exact(S, rows, cols, C, f):
    """Weights and activations both INT8: the integer sums are exact and the two scalings have a fixed
    order, so the fused call must give the oracle's fp32 values bit for bit (and their bf16 roundings)."""
    print(f"case gemv w8a8 S={S} {rows}x{cols} C={C} f={f}", flush=True)
    seed = synth.matrix_seed(6, 3)
    q, scale = oracle_matrix(rows, cols, seed, False)
    if rows >= 3:
        q = q.copy()
        q[1] = 0  # a row of zeros gives exactly zero
        q[2] = 127  # and one of the largest sums
    c = oc.compress(q, C, S, oc.RAW_FRACTION, f)
    x = np.random.default_rng(seed & 0xFFFF).standard_normal(cols).astype(np.float32) * np.float32(3.0)
    xq, sx = oq.quantise_vector(x)
    if rows >= 3:
        xq = xq.copy()
        xq[:] = np.where(np.arange(cols) % 7 == 0, xq, 127).astype(np.int8)  # large sums of one sign in row 2
    y_ref = oq.gemv_w8a8(q, scale, xq, sx)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    xq_d = torch.from_numpy(xq).cuda()
    y32 = torch.full((rows + 5,), 7.0, dtype=torch.float32, device="cuda")
    y16 = torch.zeros(rows, dtype=torch.int16, device="cuda")
    dc.decompress_gemv_w8a8(blob_d, c.blob.size, table_d, c.n_chunks, dc.Params(C, S), scale_d, rows, cols, xq_d,
                            float(sx), y32, y16, stream())
    torch.cuda.synchronize()
    y = y32.cpu().numpy()
    assert (y[rows:] == 7.0).all()
    assert np.array_equal(y[:rows].view(np.uint32), y_ref.view(np.uint32))
    assert np.array_equal(y16.cpu().numpy().view(np.uint16), oq.bf16_round(y_ref))
    # the same product on the decoded weights in a buffer
    z32 = torch.full((rows + 5,), 7.0, dtype=torch.float32, device="cuda")
    dc.gemv_w8a8(dev(q), scale_d, rows, cols, xq_d, float(sx), z32, None, stream())
    torch.cuda.synchronize()
    z = z32.cpu().numpy()
    assert (z[rows:] == 7.0).all() and np.array_equal(z[:rows].view(np.uint32), y_ref.view(np.uint32))
    if rows >= 3:
        assert y_ref[1] == 0.0
        if cols >= 2048:
            assert abs(int(oq.gemv_w8a8_acc(q, xq)[2])) > 2 ** 24  # beyond the integers fp32 holds exactly


def test_gemv_w8a8_whole_layer_call_and_argument_checks():
    C, S = 16384, 256
    shapes = [(96, 1024), (40, 2752), (33, 5120)]
    blobs, tables, mats, refs, keep = [], [], [], [], []
    off = k0 = 0
    for i, (rows, cols) in enumerate(shapes):
        q, scale = oracle_matrix(rows, cols, synth.matrix_seed(7, i), False)
        c = oc.compress(q, C, S)
        t = c.table.copy(); t["off"] += off
        blobs.append(c.blob); tables.append(t); off += c.blob.size
        xq, sx = oq.quantise_vector(np.random.default_rng(i).standard_normal(cols).astype(np.float32))
        s_d, x_d = torch.from_numpy(scale).cuda(), torch.from_numpy(xq).cuda()
        y32 = torch.full((rows,), 7.0, dtype=torch.float32, device="cuda")
        mats.append(dc.Matrix(k0, rows, cols, s_d, y_accum_dev=y32, x_i8_dev=x_d, x_scale=float(sx)))
        refs.append((oq.gemv_w8a8(q, scale, xq, sx), y32)); keep += [s_d, x_d]
        k0 += len(t)
    blob, table = np.concatenate(blobs), np.concatenate(tables)
    p = dc.Params(C, S)
    dc.decompress_gemv_w8a8_layer(dev(blob), blob.size, dev(table), len(table), p, mats, stream())
    torch.cuda.synchronize()
    for y_ref, y32 in refs:
        assert np.array_equal(y32.cpu().numpy().view(np.uint32), y_ref.view(np.uint32))
    bad = [dc.Matrix(m.first_chunk, m.rows, m.cols, m.row_scale_dev, y_accum_dev=m.y_accum_dev, x_i8_dev=None)
           for m in mats]
    with pytest.raises(dc.DCError):
        dc.decompress_gemv_w8a8_layer(dev(blob), blob.size, dev(table), len(table), p, bad, stream())


@pytest.mark.parametrize("rows,cols", [(1, 16), (7, 1040), (64, 4096), (37, 13824), (530, 5120)])
def test_gemv_i8_on_decoded_weights(rows, cols):
    """The plain product on weights in the decompression buffer against the fp64 reference."""
    print(f"case gemv_i8 {rows}x{cols}", flush=True)
    seed = synth.matrix_seed(3, 6)
    q, scale = oracle_matrix(rows, cols, seed, False)
    x = synth.gen_activation_bf16(cols, seed)
    y_ref = oq.gemv_ref(q, scale, x)
    q_d, scale_d = dev(q), torch.from_numpy(scale).cuda()
    x_d = torch.from_numpy(x.view(np.int16)).cuda()
    y32 = torch.full((rows + 3,), 7.0, dtype=torch.float32, device="cuda")
    y16 = torch.zeros(rows, dtype=torch.int16, device="cuda")
    dc.gemv_i8(q_d, scale_d, rows, cols, x_d, y32, y16, stream())
    torch.cuda.synchronize()
    y = y32.cpu().numpy()
    assert (y[rows:] == 7.0).all()  # nothing written past the last row
    assert gemv_check(y[:rows], y_ref) < 1e-4
    assert np.array_equal(y16.cpu().numpy().view(np.uint16), oq.bf16_round(y[:rows]))
    with pytest.raises(dc.DCError):
        dc.gemv_i8(q_d, scale_d, rows, cols + 8, x_d, y32, y16, stream())


def test_config1_full_size_bit_exact_and_ratio():
    """4096x4096, 64 KiB chunks, 32 sub-streams, all chunks Huffman coded."""
    q, scale = oracle_matrix(4096, 4096, synth.matrix_seed(0, 0), False)
    p = dc.Params(65536, 32)
    blob, table = dc.compress_chunks(q, p)
    c = oc.compress(q, 65536, 32, threads=8)
    assert np.array_equal(blob, c.blob) and np.array_equal(table, c.table)
    assert q.size / (blob.size + table.nbytes) == c.ratio
    out = gpu_decode(blob, table, p, q.size)
    assert np.array_equal(out, q.view(np.uint8).ravel())
