"""Seeded random sweep of valid inputs through every device entry point against the CPU oracle: sizes,
chunk sizes, sub-stream counts, data kinds and raw-chunk policies drawn together, so that combinations
nobody listed by hand are met (a sweep like this found a float/double mismatch of the raw fraction and a
zero matrix that did not give exact zeros)."""
import numpy as np
import pytest

import oracle.codec as oc
import oracle.quant as oq
import paper_2502_15443_amd as dc
import synth
from tests.helpers import gemv_workspace, lopsided_bytes, weightlike_bytes

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()


def draw_case(r):
    S = int(r.choice([32, 64, 128, 256]))
    C = int(r.choice([16, 48, 512, 4096, 16384, 65536, 262144]))
    n_chunks = int(r.integers(1, 9)) if C >= 65536 else int(r.integers(1, 40))
    n = (n_chunks - 1) * C + int(r.integers(1, C + 1))
    if r.random() < 0.5:
        n = max(16, n // 16 * 16)  # a whole number of 16-byte groups: the fused calls apply
    kind = int(r.integers(0, 7))
    if kind == 0:
        data = weightlike_bytes(n, int(r.integers(1 << 30)))
    elif kind == 1:
        data = lopsided_bytes(n, S, int(r.integers(1 << 30)))
    elif kind == 2:
        data = r.integers(0, 256, n, dtype=np.uint8)
    elif kind == 3:
        sigma = float(r.choice([0.3, 2, 8, 40]))
        data = np.clip(np.rint(r.standard_normal(n) * sigma), -127, 127).astype(np.int8).view(np.uint8)
    elif kind == 4:
        data = np.full(n, int(r.integers(256)), np.uint8)
    else:  # a wide alphabet with a long tail: many codes at the length limit
        pz = 1.0 / np.arange(1, 257) ** float(r.uniform(0.7, 1.8))
        data = r.permutation(256).astype(np.uint8)[r.choice(256, size=n, p=pz / pz.sum())]
    policy = int(r.choice([oc.ALL_HUFF, oc.AUTO, oc.RAW_FRACTION, oc.BLOCK_LAST]))
    f = float(r.choice([0.0, 0.2, 0.5, 0.9, 1.0]))
    block = int(r.integers(1, 6))
    return S, C, n, data, policy, f, block


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_valid_inputs_all_entry_points(seed):
    st = torch.cuda.current_stream().cuda_stream
    r = np.random.default_rng(seed)
    fused = 0
    for it in range(120):
        S, C, n, data, policy, f, block = draw_case(r)
        print(f"case random seed={seed} it={it} S={S} C={C} n={n} policy={policy} f={f} block={block}", flush=True)
        c = oc.compress(data, C, S, policy, f, block=block, threads=8)
        p = dc.Params(C, S, policy, f, block)
        blob_d, table_d = dev(c.blob), dev(c.table)

        # decode of the oracle's blob
        dst = torch.full((n + 256,), 0x5A, dtype=torch.uint8, device="cuda")
        dc.decompress_chunks(blob_d, c.blob.size, table_d, c.n_chunks, p, dst, n, st)
        torch.cuda.synchronize()
        out = dst.cpu().numpy()
        assert np.array_equal(out[:n], data) and (out[n:] == 0x5A).all()

        # compression on the device: the oracle's blob and table, nothing beyond the capacity
        cap, nc = dc.compress_bound(n, p)
        out_blob = torch.full((cap + 64,), 0xEE, dtype=torch.uint8, device="cuda")
        out_table = torch.zeros(nc * 16, dtype=torch.uint8, device="cuda")
        ws_bytes = dc.compress_chunks_dev_workspace(n, p)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        res = torch.zeros(2, dtype=torch.int64, device="cuda")
        src = torch.zeros((n + 15) // 16 * 16, dtype=torch.uint8, device="cuda")
        src[:n] = torch.from_numpy(data).cuda()
        dc.compress_chunks_dev(src, n, p, out_blob, cap, out_table, nc, ws, ws_bytes, res, st)
        torch.cuda.synchronize()
        used = int(res.cpu()[0])
        assert used == c.blob.size and int(res.cpu()[1]) == 0
        assert np.array_equal(out_blob[:used].cpu().numpy(), c.blob)
        assert np.array_equal(out_table.cpu().numpy().view(dc.CHUNK_DTYPE), c.table)
        assert (out_blob[cap:].cpu().numpy() == 0xEE).all()

        # the fused calls, when the bytes are a matrix of whole 16-byte groups
        if n % 16:
            continue
        cols = 16 * max(d for d in range(1, 1025) if (n // 16) % d == 0)
        rows = n // cols
        fused += 1
        scale = ((r.random(rows) + 0.5) * 0.01).astype(np.float32)
        scale_d = torch.from_numpy(scale).cuda()
        q = data.view(np.int8).reshape(rows, cols)
        out16 = torch.full((n + 64,), 0x5A5A, dtype=torch.int16, device="cuda")
        dc.decompress_dequant_bf16(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols, out16, n, st)
        torch.cuda.synchronize()
        got = out16.cpu().numpy().view(np.uint16)
        assert np.array_equal(got[:n].reshape(rows, cols), oq.dequant_bf16(q, scale)) and (got[n:] == 0x5A5A).all()
        x = synth.gen_activation_bf16(cols, seed * 1000 + it)
        y32 = torch.full((rows + 8,), 7.0, dtype=torch.float32, device="cuda")
        dc.decompress_gemv(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols,
                           torch.from_numpy(x.view(np.int16)).cuda(), y32, None, *gemv_workspace(c.n_chunks), st)
        torch.cuda.synchronize()
        y = y32.cpu().numpy()
        y_ref = oq.gemv_ref(q, scale, x)
        assert (y[rows:] == 7.0).all()
        rms = float(np.sqrt(np.mean(y_ref ** 2)))
        assert (np.abs(y[:rows] - y_ref) <= 1e-2 * np.abs(y_ref) + 1e-2 * rms).all()
        # weights and activations both INT8: exact sums, the oracle's fp32 bits
        xq = r.integers(-127, 128, cols).astype(np.int8)
        sx = np.float32(0.013)
        z32 = torch.full((rows + 8,), 7.0, dtype=torch.float32, device="cuda")
        dc.decompress_gemv_w8a8(blob_d, c.blob.size, table_d, c.n_chunks, p, scale_d, rows, cols,
                                torch.from_numpy(xq).cuda(), float(sx), z32, None, st)
        torch.cuda.synchronize()
        z = z32.cpu().numpy()
        assert (z[rows:] == 7.0).all()
        assert np.array_equal(z[:rows].view(np.uint32), oq.gemv_w8a8(q, scale, xq, sx).view(np.uint32))
    assert fused >= 30


@pytest.mark.parametrize("codec", [dc.CODEC_HUFFMAN, dc.CODEC_TANS])
def test_damaged_blobs_that_still_validate_decode_as_the_oracle_decodes_them(codec):
    """Flipped payload bits that dc_validate lets through (a flip in padding, or one that turns a stream into
    another stream of the same size) give a blob that is valid by the format, so it has one right decode:
    the device and the oracle must agree on it byte for byte, although it is no longer the input."""
    r = np.random.default_rng(70 + codec)
    st = torch.cuda.current_stream().cuda_stream
    accepted = changed = 0
    for it in range(400):
        S = int(r.choice([64, 128, 256]))
        C = int(r.choice([512, 4096, 16384]))
        n = max(1, int(r.integers(1, 6)) * C - int(r.integers(0, C)))
        data = weightlike_bytes(n, int(r.integers(1 << 30)))
        p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, float(r.choice([0, 0.3])), codec=codec)
        blob, table = dc.compress_chunks(data, p)
        b = blob.copy()
        for _ in range(int(r.integers(1, 4))):
            b[r.integers(b.size - 64)] ^= 1 << int(r.integers(8))
        try:
            dc.validate(b, table, p)
        except dc.DCError:
            continue
        accepted += 1
        want = oc.decompress(b, table, C, S, n, codec=codec)
        changed += not np.array_equal(want, data)
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
        dc.decompress_chunks(dev(b), b.size, dev(table.view(np.uint8)), len(table), p, dst, n, st)
        torch.cuda.synchronize()
        assert np.array_equal(dst.cpu().numpy(), want), f"case {it} S={S} C={C} n={n}"
    assert accepted >= 15 and changed >= 5
