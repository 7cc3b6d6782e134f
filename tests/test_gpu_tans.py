"""GPU parity of the tANS coder: the decode calls on tANS blobs against the CPU oracle (bytes, bf16 values and the
W8A8 product bit for bit); the library's host compressor against the oracle's blob (the device compressor's is in
tests/test_gpu_compress.py); what the calls say to 32 sub-streams."""
import numpy as np
import pytest

import oracle.codec as oc
import paper_2502_15443_amd as dc
from tests.helpers import gemv_workspace, lopsided_bytes, weightlike_bytes

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()


def stream():
    return torch.cuda.current_stream().cuda_stream


def gpu_decode(blob, table, params, n, fill=0xAB, guard=256):
    blob_d, table_d = dev(blob), dev(table)
    dst = torch.full((n + guard,), fill, dtype=torch.uint8, device="cuda")
    dc.decompress_chunks(blob_d, blob.size, table_d, len(table), params, dst, n, stream())
    torch.cuda.synchronize()
    out = dst.cpu().numpy()
    assert (out[n:] == fill).all()
    return out[:n]


def tans(C, S, policy=dc.POLICY_ALL_HUFF, f=0.0, block=0):
    return dc.Params(C, S, policy, f, block, codec=dc.CODEC_TANS)


@pytest.mark.parametrize("S", [64, 128, 256])
@pytest.mark.parametrize("n,C", [(3 * 65536, 65536), (5 * 16384 + 777, 16384), (7 * 4096 + 4095, 4096),
                                 (65536 + 16, 65536), (100, 65536), (1, 4096), (9 * 2048 + 1, 2048),
                                 (2 * 262144 + 12345, 262144), (1048576 + 5, 1048576)])
def test_decode_matches_oracle_bytes(S, n, C):
    print(f"case tans S={S} n={n} C={C}", flush=True)
    data = weightlike_bytes(n, 2000 + n % 977 + S)
    c = oc.compress(data, C, S, codec=oc.TANS, threads=8)  # the oracle's blob
    out = gpu_decode(c.blob, c.table, tans(C, S), n)
    assert np.array_equal(out, data)


@pytest.mark.parametrize("S", [64, 128, 256])
def test_decode_degenerate_chunks(S):
    """One value only (fields of no bits), two values, all 256 equally often (8 bits each), a long-tailed chunk
    whose rare values have one state (fields of 11 bits), a chunk of one byte."""
    print(f"case tans degenerate S={S}", flush=True)
    C = 4096
    r = np.random.default_rng(0)
    skew = np.clip(np.rint(r.standard_cauchy(C) * 2), -127, 127).astype(np.int8).view(np.uint8)
    data = np.concatenate([np.zeros(C, np.uint8), np.full(C, 0x81, np.uint8), r.integers(0, 256, C, dtype=np.uint8),
                           np.tile(np.array([3, 250], np.uint8), C // 2), np.arange(C, dtype=np.uint32).astype(np.uint8),
                           skew, np.array([7], np.uint8)])
    for policy in (oc.ALL_HUFF, oc.AUTO):
        c = oc.compress(data, C, S, policy, codec=oc.TANS)
        assert np.array_equal(gpu_decode(c.blob, c.table, tans(C, S), data.size), data)


@pytest.mark.parametrize("S", [64, 128, 256])
def test_decode_lopsided_streams(S):
    print(f"case tans lopsided S={S}", flush=True)
    C = 65536
    n = 3 * C + 4096 + 50
    data = lopsided_bytes(n, S, 7 + S)
    c = oc.compress(data, C, S, codec=oc.TANS, threads=8)
    assert np.array_equal(gpu_decode(c.blob, c.table, tans(C, S), n), data)


@pytest.mark.parametrize("S", [64, 256])
@pytest.mark.parametrize("policy,f,block", [(dc.POLICY_RAW_FRACTION, 0.5, 0), (dc.POLICY_BLOCK_LAST, 0.0, 3),
                                            (dc.POLICY_AUTO, 0.0, 0)])
def test_library_compressor_is_the_oracles_and_decodes_with_raw_chunks(S, policy, f, block):
    print(f"case tans compress S={S} policy={policy}", flush=True)
    C = 16384
    n = 23 * C + 333
    data = weightlike_bytes(n, 17 + S)
    data[5 * C:6 * C] = np.random.default_rng(1).integers(0, 256, C, dtype=np.uint8)
    p = tans(C, S, policy, f, block)
    blob, table = dc.compress_chunks(data, p)
    c = oc.compress(data, C, S, policy, f, block=block, codec=oc.TANS, threads=8)
    assert np.array_equal(blob, c.blob) and np.array_equal(table, c.table)
    dc.validate(blob, table, p)
    assert np.array_equal(gpu_decode(blob, table, p, n), data)


@pytest.mark.parametrize("S", [64, 256])
def test_corrupt_payloads_stay_inside_the_buffers(S):
    """Frequencies that do not add up, damaged stream fields, random payloads: unspecified bytes (or none) for
    those chunks only, nothing outside the destination, the other chunks decode."""
    print(f"case tans corrupt S={S}", flush=True)
    C = 16384
    n = 8 * C
    data = weightlike_bytes(n, 31)
    c = oc.compress(data, C, S, codec=oc.TANS)
    blob, table = c.blob.copy(), c.table.copy()
    r = np.random.default_rng(5 + S)
    off = [int(o) for o in table["off"]]
    size = [int(x) for x in table["comp_bytes"]]
    blob[off[1]:off[1] + 384] = r.integers(0, 256, 384, dtype=np.uint8)                    # frequencies
    blob[off[2] + 384:off[2] + 384 + 2 * S] = r.integers(0, 256, 2 * S, dtype=np.uint8)    # blocks per stream
    blob[off[3] + 384 + 2 * S:off[3] + 388 + 2 * S] = 0xFF                                 # area offset far outside
    blob[off[4]:off[4] + size[4]] = r.integers(0, 256, size[4], dtype=np.uint8)             # everything
    blob[off[5]:off[5] + 384] = 0                                                          # no value at all
    blob[off[6] + 600:off[6] + size[6]] ^= r.integers(0, 256, size[6] - 600, dtype=np.uint8)  # every stream bit
    with pytest.raises(dc.DCError):
        dc.validate(blob, table, tans(C, S))
    out = gpu_decode(blob, table, tans(C, S), n, fill=0x5A, guard=4096)
    for k in (0, 7):
        assert np.array_equal(out[k * C:(k + 1) * C], data[k * C:(k + 1) * C])
    for k in (1, 5):
        assert (out[k * C:(k + 1) * C] == 0x5A).all()  # frequencies that do not add up: nothing is written


@pytest.mark.parametrize("S", [64, 128, 256])
@pytest.mark.parametrize("rows,cols,C,policy", [(192, 1024, 16384, dc.POLICY_ALL_HUFF), (77, 1040, 4096, dc.POLICY_RAW_FRACTION),
                                                (1031, 4096, 65536, dc.POLICY_ALL_HUFF)])
def test_fused_calls_on_tans_blobs(S, rows, cols, C, policy):
    """Dequantisation to bf16 and both batch-1 products fused into the tANS decode: the same bars as on Huffman
    blobs (bf16 and the W8A8 product bit for bit, the bf16-activation product within the stated tolerance)."""
    import oracle.quant as oq
    import synth
    from tests.helpers import oracle_matrix
    print(f"case tans fused S={S} rows={rows} cols={cols} C={C} policy={policy}", flush=True)
    q, scale = oracle_matrix(rows, cols, synth.matrix_seed(3, 2), True)
    n = rows * cols
    p = tans(C, S, policy, 0.4)
    c = oc.compress(q, C, S, policy, 0.4, codec=oc.TANS, threads=8)
    blob_d, table_d, scale_d = dev(c.blob), dev(c.table), torch.from_numpy(scale).cuda()
    out16 = torch.full((n + 64,), 0x5A5A, dtype=torch.int16, device="cuda")
    dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols, out16, n, stream())
    x = synth.gen_activation_bf16(cols, 99)
    y32 = torch.full((rows + 8,), 7.0, dtype=torch.float32, device="cuda")
    dc.decompress_gemv(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols,
                       torch.from_numpy(x.view(np.int16)).cuda(), y32, None, *gemv_workspace(c.n_chunks), stream())
    xq = np.random.default_rng(S).integers(-127, 128, cols).astype(np.int8)
    sx = np.float32(0.021)
    z32 = torch.full((rows + 8,), 7.0, dtype=torch.float32, device="cuda")
    dc.decompress_gemv_w8a8(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols, torch.from_numpy(xq).cuda(),
                            float(sx), z32, None, stream())
    torch.cuda.synchronize()
    got = out16.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[:n].reshape(rows, cols), oq.dequant_bf16(q, scale)) and (got[n:] == 0x5A5A).all()
    y, y_ref = y32.cpu().numpy(), oq.gemv_ref(q, scale, x)
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    assert (y[rows:] == 7.0).all() and (np.abs(y[:rows] - y_ref) <= 1e-2 * np.abs(y_ref) + 1e-2 * rms).all()
    z = z32.cpu().numpy()
    assert (z[rows:] == 7.0).all()
    assert np.array_equal(z[:rows].view(np.uint32), oq.gemv_w8a8(q, scale, xq, sx).view(np.uint32))


def test_32_sub_streams_are_refused():
    C, S, n = 16384, 64, 4 * 16384
    data = weightlike_bytes(n, 3)
    p = tans(C, S)
    with pytest.raises(dc.DCError):
        dc.compress_chunks_dev_workspace(n, dc.Params(C, 32, codec=dc.CODEC_TANS))
    blob, table = dc.compress_chunks(data, p)
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    with pytest.raises(dc.DCError):  # 32 sub-streams are half a wavefront: Huffman only
        dc.decompress_chunks(dev(blob), blob.size, dev(table), len(table), dc.Params(C, 32, codec=dc.CODEC_TANS), dst, n, stream())
    with pytest.raises(dc.DCError):
        dc.compress_chunks(data, dc.Params(C, 32, codec=dc.CODEC_TANS))  # tANS needs whole wavefronts of streams
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", [21, 22])
def test_random_valid_inputs(seed):
    r = np.random.default_rng(seed)
    for it in range(60):
        S = int(r.choice([64, 128, 256]))
        C = int(r.choice([16, 48, 512, 4096, 16384, 65536, 262144]))
        n_chunks = int(r.integers(1, 6)) if C >= 65536 else int(r.integers(1, 30))
        n = (n_chunks - 1) * C + int(r.integers(1, C + 1))
        kind = int(r.integers(0, 5))
        if kind == 0:
            data = weightlike_bytes(n, int(r.integers(1 << 30)))
        elif kind == 1:
            data = lopsided_bytes(n, S, int(r.integers(1 << 30)))
        elif kind == 2:
            data = r.integers(0, 256, n, dtype=np.uint8)
        elif kind == 3:
            data = np.full(n, int(r.integers(256)), np.uint8)
        else:
            pz = 1.0 / np.arange(1, 257) ** float(r.uniform(0.7, 1.8))
            data = r.permutation(256).astype(np.uint8)[r.choice(256, size=n, p=pz / pz.sum())]
        policy = int(r.choice([oc.ALL_HUFF, oc.AUTO, oc.RAW_FRACTION, oc.BLOCK_LAST]))
        f = float(r.choice([0.0, 0.2, 0.5, 1.0]))
        block = int(r.integers(1, 5))
        print(f"case tans random seed={seed} it={it} S={S} C={C} n={n} kind={kind} policy={policy}", flush=True)
        c = oc.compress(data, C, S, policy, f, block=block, codec=oc.TANS, threads=8)
        p = tans(C, S, policy, f, block)
        blob, table = dc.compress_chunks(data, p)
        assert np.array_equal(blob, c.blob) and np.array_equal(table, c.table)
        assert np.array_equal(gpu_decode(c.blob, c.table, p, n), data)
        from tests.test_gpu_compress import dev_compress
        dblob, dtable, used, status = dev_compress(data, p)
        assert status == 0 and used == c.blob.size and np.array_equal(dtable, c.table) and np.array_equal(dblob[:used], c.blob)
