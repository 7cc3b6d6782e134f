"""CPU tests of the library: exported symbols, host-side quantiser / compressor / validator against
the oracle.  No GPU call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle.codec as oc
import oracle.quant as oq
import paper_2502_15443_amd as dc
import synth
from tests.helpers import weightlike_bytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dc.h")).read()
    names = set(re.findall(r"\b(dc_[a-z0-9_]+)\s*\(", header))
    assert {"dc_compress_chunks", "dc_decompress_chunks", "dc_decompress_dequant_bf16",
            "dc_decompress_gemv", "dc_quantize_rows", "dc_validate"} <= names
    lib = ctypes.CDLL(dc.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert "gfx950" in dc.version()


@pytest.mark.parametrize("rescale", [False, True])
def test_quantize_rows_matches_oracle_bit_for_bit(rescale):
    rows, cols, seed = 192, 1024, synth.matrix_seed(3, 2)
    w = synth.gen_weight(rows, cols, seed)
    w[5] = 0  # an all-zero row
    a = synth.gen_act_absmax(cols, seed) if rescale else None
    q, rs, cs = dc.quantize_rows(w, a, 0.5, 1)
    w2 = oq.rescale(w, oq.channel_scale(a, 0.5)) if rescale else w
    q_ref, rs_ref = oq.quantise_rows(w2)
    q_ref = oq.prune(q_ref)
    assert np.array_equal(q, q_ref) and np.array_equal(rs, rs_ref)
    if rescale:
        assert np.array_equal(cs, oq.channel_scale(a, 0.5))
    else:
        assert (cs == 1).all()
    q0, _, _ = dc.quantize_rows(w, a, 0.5, 0)  # no pruning
    assert np.array_equal(q0, oq.quantise_rows(w2)[0])


@pytest.mark.parametrize("alpha", [0.0, 0.3, 1.0])
def test_quantize_rows_other_exponents(alpha):
    rows, cols, seed = 64, 512, 99
    w = synth.gen_weight(rows, cols, seed)
    a = synth.gen_act_absmax(cols, seed)
    q, rs, cs = dc.quantize_rows(w, a, alpha, 1)
    s = oq.channel_scale(a, alpha)
    q_ref, rs_ref = oq.quantise_rows(oq.rescale(w, s))
    assert np.array_equal(cs, s) and np.array_equal(q, oq.prune(q_ref)) and np.array_equal(rs, rs_ref)


@pytest.mark.parametrize("alpha", [0.0, 0.5, 1.0])
@pytest.mark.parametrize("sparsity", [0.0, 0.2, 0.4])
def test_quantize_tensor_matches_oracle_bit_for_bit(alpha, sparsity):
    """The paper's own front end: one scale per tensor, pruning by the importance score (Eq. 5)."""
    rows, cols, seed = 160, 768, synth.matrix_seed(4, 1)
    w = synth.gen_weight(rows, cols, seed)
    a = synth.gen_act_absmax(cols, seed)
    q, ts, cs = dc.quantize_tensor(w, a, alpha, sparsity)
    s = oq.channel_scale(a, alpha)
    q_ref, ts_ref = oq.quantise_tensor(oq.rescale(w, s))
    q_ref = oq.prune_by_score(q_ref, a, sparsity)
    assert np.array_equal(cs, s) and np.float32(ts) == ts_ref and np.array_equal(q, q_ref)
    assert np.mean(q == 0) >= sparsity
    # without activation statistics the score is the magnitude
    q1, ts1, cs1 = dc.quantize_tensor(w, None, alpha, sparsity)
    q1_ref, ts1_ref = oq.quantise_tensor(w)
    assert (cs1 == 1).all() and np.float32(ts1) == ts1_ref
    assert np.array_equal(q1, oq.prune_by_score(q1_ref, np.ones(cols, np.float32), sparsity))
    with pytest.raises(dc.DCError):
        dc.quantize_tensor(w, a, alpha, 1.0)


@pytest.mark.parametrize("S", [32, 64, 128, 256])
@pytest.mark.parametrize("n,C", [(5 * 16384 + 777, 16384), (3 * 65536, 65536), (100, 65536), (65536 + 16, 65536),
                                 (7 * 4096 + 4095, 4096)])
def test_compress_is_byte_identical_to_oracle(S, n, C):
    data = weightlike_bytes(n, n + S)
    p = dc.Params(C, S)
    blob, table = dc.compress_chunks(data, p)
    c = oc.compress(data, C, S)
    assert np.array_equal(table, c.table)
    assert np.array_equal(blob, c.blob)
    dc.validate(blob, table, p)
    assert np.array_equal(oc.decompress(blob, table, C, S, n), data)


def test_compress_degenerate_chunks():
    C, S = 4096, 32
    r = np.random.default_rng(0)
    data = np.concatenate([np.zeros(C, np.uint8), np.full(C, 0x81, np.uint8), r.integers(0, 256, C, dtype=np.uint8),
                           np.tile(np.array([3, 250], np.uint8), C // 2), np.arange(C, dtype=np.uint32).astype(np.uint8),
                           np.array([7], np.uint8)])
    for policy in (dc.POLICY_ALL_HUFF, dc.POLICY_AUTO):
        p = dc.Params(C, S, policy)
        blob, table = dc.compress_chunks(data, p)
        c = oc.compress(data, C, S, policy)
        assert np.array_equal(table, c.table) and np.array_equal(blob, c.blob)
        dc.validate(blob, table, p)


@pytest.mark.parametrize("policy,kw", [(dc.POLICY_RAW_FRACTION, dict(raw_fraction=0.0)),
                                       (dc.POLICY_RAW_FRACTION, dict(raw_fraction=0.25)),
                                       (dc.POLICY_RAW_FRACTION, dict(raw_fraction=0.5)),
                                       (dc.POLICY_RAW_FRACTION, dict(raw_fraction=0.75)),
                                       (dc.POLICY_RAW_FRACTION, dict(raw_fraction=1.0)),
                                       (dc.POLICY_AUTO, {}), (dc.POLICY_BLOCK_LAST, dict(block_chunks=5)),
                                       (dc.POLICY_BLOCK_LAST, dict(block_chunks=1))])
def test_raw_policies_match_oracle(policy, kw):
    C, S = 8192, 32
    data = weightlike_bytes(37 * C + 100, 5)
    p = dc.Params(C, S, policy, **kw)
    blob, table = dc.compress_chunks(data, p)
    c = oc.compress(data, C, S, policy, raw_fraction=kw.get("raw_fraction", 0.0), block=kw.get("block_chunks", 0))
    assert np.array_equal(table, c.table) and np.array_equal(blob, c.blob)
    ratio = data.size / (blob.size + table.nbytes)
    assert abs(ratio - c.ratio) < 1e-15  # compression ratio equal to the oracle's
    dc.validate(blob, table, p)


def test_raw_fraction_is_taken_as_a_32_bit_float_on_both_sides():
    """25 chunks at f = 0.9: f * n + 1/2 is 23 exactly in real numbers and just below 23 for the 32-bit
    value of 0.9 that the parameter block carries; the count of raw chunks follows the carried value."""
    C, S = 4096, 32
    data = weightlike_bytes(25 * C, 3)
    p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, 0.9)
    blob, table = dc.compress_chunks(data, p)
    c = oc.compress(data, C, S, oc.RAW_FRACTION, 0.9)
    assert np.array_equal(table, c.table) and np.array_equal(blob, c.blob)
    assert int((table["raw_bytes_flags"] >> 31).sum()) == int(np.float64(np.float32(0.9)) * 25 + 0.5) == 22


def test_raw_mask_policy():
    C, S = 4096, 64
    data = weightlike_bytes(10 * C, 6)
    mask = np.array([1, 0, 0, 1, 1, 0, 1, 0, 0, 1], dtype=np.uint8)
    p = dc.Params(C, S, dc.POLICY_RAW_MASK, raw_mask=mask)
    blob, table = dc.compress_chunks(data, p)
    c = oc.compress(data, C, S, oc.RAW_MASK, mask=mask)
    assert np.array_equal(table, c.table) and np.array_equal(blob, c.blob)


def test_result_independent_of_thread_count():
    data = weightlike_bytes(20 * 16384 + 5, 7)
    p = dc.Params(16384, 32, dc.POLICY_RAW_FRACTION, 0.3)
    prev = dc.set_num_threads(1)
    try:
        b1, t1 = dc.compress_chunks(data, p)
        dc.set_num_threads(5)
        b5, t5 = dc.compress_chunks(data, p)
    finally:
        dc.set_num_threads(prev)
    assert np.array_equal(b1, b5) and np.array_equal(t1, t5)


def test_argument_errors():
    data = weightlike_bytes(4096, 1)
    for bad in (dc.Params(1000, 32), dc.Params(4096, 33), dc.Params(1 << 21, 32), dc.Params(4096, 32, 9),
                dc.Params(4096, 32, dc.POLICY_RAW_FRACTION, 1.5), dc.Params(4096, 32, dc.POLICY_BLOCK_LAST),
                dc.Params(4096, 32, dc.POLICY_RAW_MASK)):
        with pytest.raises(dc.DCError) as e:
            dc.compress_chunks(data, bad)
        assert e.value.code == -1


def test_compress_reports_required_capacity():
    lib = ctypes.CDLL(dc.lib_path())
    data = weightlike_bytes(3 * 4096, 2)
    p = dc.Params(4096, 32)
    blob, table = dc.compress_chunks(data, p)
    used, n = ctypes.c_uint64(0), ctypes.c_uint64(0)
    small = np.zeros(16, np.uint8)
    tab = np.zeros(3, dc.CHUNK_DTYPE)
    cp = p._c()
    rc = lib.dc_compress_chunks(ctypes.c_void_p(data.ctypes.data), ctypes.c_uint64(data.size), ctypes.byref(cp),
                                ctypes.c_void_p(small.ctypes.data), ctypes.c_uint64(16), ctypes.byref(used),
                                ctypes.c_void_p(tab.ctypes.data), ctypes.c_uint64(3), ctypes.byref(n))
    assert rc == -2 and used.value == blob.size and n.value == 3


def test_validate_catches_corruption():
    C, S = 4096, 32
    data = weightlike_bytes(6 * C + 9, 8)
    p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, 0.34)
    blob, table = dc.compress_chunks(data, p)
    dc.validate(blob, table, p)
    huff = [k for k in range(len(table)) if not table["raw_bytes_flags"][k] & dc.CHUNK_RAW]
    k = huff[1]
    o = int(table["off"][k])

    def expect_bad(b, t, chunk):
        with pytest.raises(dc.DCError) as e:
            dc.validate(b, t, p)
        assert e.value.code == -3 and f"chunk {chunk})" in str(e.value)

    b = blob.copy(); b[o] = 0xFF  # code lengths 15
    expect_bad(b, table, k)
    b = blob.copy(); b[o + 3] ^= 0x01  # Kraft sum no longer 1
    expect_bad(b, table, k)
    b = blob.copy(); b[o + 128 + 2 * 5] += 1  # block count of stream 5 one too many
    expect_bad(b, table, k)
    b = blob.copy(); b[o + 128 + 2 * 5] -= 1  # ... one too few: the stream runs out of bits
    expect_bad(b, table, k)
    b = blob.copy(); b[o + 128 + 2 * 5 + 1] ^= 0x10  # bytes of the first block of stream 5 changed
    expect_bad(b, table, k)
    b = blob.copy(); b[o + 128 + 2 * S:o + 128 + 2 * S + 4] = np.frombuffer(np.uint32(1 << 24).tobytes(), np.uint8)
    expect_bad(b, table, k)  # region offset outside the payload
    b = blob.copy(); b[o + 128 + 2 * S] ^= 0x10  # region not right after the header
    expect_bad(b, table, k)
    b = blob.copy(); b[o + 128 + 2 * S + 5] = 1  # header padding not zero
    expect_bad(b, table, k)
    field = np.frombuffer(blob[o + 128:o + 128 + 2 * S].tobytes(), dtype="<u2").astype(int)
    end = o + 144 + 2 * S + 16 * int(((field & 0xFFF) - 1).sum()) + int(((field >> 12) + 1).sum())  # header is 144 + 2 S bytes at S = 32
    if end % 16:  # the area of the one stream set is padded with zeros
        b = blob.copy(); b[end] = 1
        expect_bad(b, table, k)
    t = table.copy(); t["raw_bytes_flags"][2] = (t["raw_bytes_flags"][2] & dc.CHUNK_RAW) | (C + 16)  # too long
    expect_bad(blob, t, 2)
    t = table.copy(); t["off"][3] += 16  # payloads no longer back to back
    expect_bad(blob, t, 3)
    t = table.copy(); t["comp_bytes"][-1] += 1 << 20  # beyond the blob
    expect_bad(blob, t, len(t) - 1)
    expect_bad(blob[:o + 64].copy(), table, len(table))  # truncated blob: it no longer ends in its trailer
    expect_bad(blob[:-1].copy(), table, len(table))
    b = np.concatenate([blob[:-64], blob[-16:]])  # the trailer right behind the last payload: closing bytes incomplete
    expect_bad(b, table, len(table) - 1)


def test_trailer_names_format_and_parameters():
    """The blob's last 16 bytes, spelled out: 'DCBF', format id 5, look-ahead 392, chunk size, sub-streams,
    coder; the same bytes from the oracle; and every host entry point refuses another format id."""
    for C, S, codec in [(4096, 32, dc.CODEC_HUFFMAN), (65536, 256, dc.CODEC_TANS), (1 << 20, 64, dc.CODEC_HUFFMAN)]:
        data = weightlike_bytes(C + 100, 5)
        p = dc.Params(C, S, codec=codec)
        blob, table = dc.compress_chunks(data, p)
        want = b"DCBF" + (5).to_bytes(2, "little") + (392).to_bytes(2, "little") + C.to_bytes(4, "little") \
            + S.to_bytes(2, "little") + codec.to_bytes(2, "little")
        assert blob[-16:].tobytes() == want and not blob[-64:-16].any()
        assert oc.compress(data, C, S, codec=codec).blob[-64:].tobytes() == blob[-64:].tobytes()
        got = dc.blob_trailer(blob)
        assert (got.chunk_bytes, got.n_streams, got.codec, got.format) == (C, S, codec, dc.FORMAT_ID)
    with pytest.raises(dc.DCError) as e:
        dc.blob_trailer(np.zeros(64, np.uint8))  # a blob of the formats before this one ended in zeros
    assert e.value.code == -3


def test_blob_of_another_format_is_refused():
    """A blob as format 3 would have closed it (look-ahead 320), one without a trailer, and one whose trailer
    names other parameters: dc_validate returns DC_E_FORMAT for each, the oracle's decoder refuses them too,
    and a caller that states another format id is refused by every entry point that takes parameters."""
    C, S = 4096, 64
    data = weightlike_bytes(3 * C, 6)
    p = dc.Params(C, S)
    blob, table = dc.compress_chunks(data, p)
    dc.validate(blob, table, p)
    old = blob.copy()
    old[-12:-8] = np.frombuffer((3).to_bytes(2, "little") + (320).to_bytes(2, "little"), np.uint8)
    bare = blob.copy()
    bare[-16:] = 0
    other = blob.copy()
    other[-4] = 128  # says 128 sub-streams
    for b in (old, bare, other):
        with pytest.raises(dc.DCError) as e:
            dc.validate(b, table, p)
        assert e.value.code == -3 and f"chunk {len(table)})" in str(e.value)
        with pytest.raises(ValueError):
            oc.decompress(b, table, C, S, data.size)
    with pytest.raises(dc.DCError) as e:
        dc.blob_trailer(old)
    assert e.value.code == -3
    stale = dc.Params(C, S, format=4)
    for call in (lambda: dc.validate(blob, table, stale), lambda: dc.compress_chunks(data, stale),
                 lambda: dc.compress_bound(data.size, stale), lambda: dc.compress_chunks_dev_workspace(data.size, stale)):
        with pytest.raises(dc.DCError) as e:
            call()
        assert e.value.code == -3


def test_validate_takes_appended_blobs_and_parts_of_a_table():
    """Blobs put one after the other (a layer's matrices, each compressed alone, offsets moved) and a part of
    such a table (one matrix of the layer): both are what the decode calls take, and the validator checks them."""
    C, S = 4096, 64
    p = dc.Params(C, S, dc.POLICY_AUTO)
    parts = [weightlike_bytes(n, 40 + i) for i, n in enumerate((5 * C, 2 * C + 7, 3 * C))]
    blobs, tables, off = [], [], 0
    for d in parts:
        b, t = dc.compress_chunks(d, p)
        t = t.copy()
        t["off"] += off
        off += b.size
        blobs.append(b)
        tables.append(t)
    blob, table = np.concatenate(blobs), np.concatenate(tables)
    with pytest.raises(dc.DCError):  # as one table it is not one byte string: the middle part ends in a short chunk
        dc.validate(blob, table, p)
    k = 0
    for t in tables:  # every part on its own, against the whole blob
        dc.validate(blob, table[k:k + len(t)], p)
        k += len(t)
    whole = [weightlike_bytes(n, 50 + i) for i, n in enumerate((5 * C, 2 * C, 3 * C))]
    blobs, tables, off = [], [], 0
    for d in whole:
        b, t = dc.compress_chunks(d, p)
        t = t.copy()
        t["off"] += off
        off += b.size
        blobs.append(b)
        tables.append(t)
    blob, table = np.concatenate(blobs), np.concatenate(tables)
    dc.validate(blob, table, p)
    assert np.array_equal(oc.decompress(blob, table, C, S, 10 * C), np.concatenate(whole))
    t = table.copy()
    t["off"][6] -= 16  # a payload that begins inside the one before it
    with pytest.raises(dc.DCError) as e:
        dc.validate(blob, t, p)
    assert "chunk 6)" in str(e.value)


def test_compress_bound_holds_on_worst_case():
    C, S = 4096, 128
    r = np.random.default_rng(3)
    # skewed enough to get 11-bit codes, noisy enough to use many of them
    data = np.clip(np.rint(r.standard_cauchy(8 * C) * 2), -127, 127).astype(np.int8).view(np.uint8)
    p = dc.Params(C, S)
    cap, nc = dc.compress_bound(data.size, p)
    blob, table = dc.compress_chunks(data, p)
    assert nc == 8 and blob.size <= cap


def test_quantize_vector_matches_oracle_bit_for_bit():
    r = np.random.default_rng(8)
    for n, mult in [(1, 1.0), (16, 3.0), (4096, 1.0), (13824, 40.0), (5, 1e-20)]:
        x = (r.standard_normal(n) * mult).astype(np.float32)
        x[r.integers(n)] *= 8
        xq, s = dc.quantize_vector(x)
        xq_ref, s_ref = oq.quantise_vector(x)
        assert np.array_equal(xq, xq_ref) and np.float32(s) == s_ref
    xq, s = dc.quantize_vector(np.zeros(9, np.float32))
    assert s == 1.0 and not xq.any()
    halves = (np.arange(-8, 9, dtype=np.float32) + 0.5) * np.float32(127.0 / 127.0)  # ties, scale exactly 1/...
    x = np.concatenate([halves, np.array([127.0], np.float32)])
    xq, s = dc.quantize_vector(x)
    assert np.array_equal(xq, oq.quantise_vector(x)[0])


@pytest.mark.parametrize("seed", [21, 22])
def test_random_inputs_host_compressor_equals_oracle(seed):
    """Seeded random sweep on the CPU: the library's host compressor writes the oracle's blob and table for
    sizes, chunk sizes, sub-stream counts, data kinds and policies drawn together; the validator accepts
    it, the oracle decodes it back, and the independent Python decoder agrees on the small chunks."""
    from tests import pyref
    from tests.helpers import lopsided_bytes
    r = np.random.default_rng(seed)
    for it in range(120):
        S = int(r.choice([32, 64, 128, 256]))
        C = int(r.choice([16, 48, 512, 4096, 16384, 65536]))
        n_chunks = int(r.integers(1, 5)) if C >= 16384 else int(r.integers(1, 30))
        n = (n_chunks - 1) * C + int(r.integers(1, C + 1))
        kind = int(r.integers(0, 4))
        if kind == 0:
            data = weightlike_bytes(n, int(r.integers(1 << 30)))
        elif kind == 1:
            data = lopsided_bytes(n, S, int(r.integers(1 << 30)))
        elif kind == 2:
            data = r.integers(0, 256, n, dtype=np.uint8)
        else:
            data = np.full(n, int(r.integers(256)), np.uint8)
        policy = int(r.choice([dc.POLICY_ALL_HUFF, dc.POLICY_AUTO, dc.POLICY_RAW_FRACTION, dc.POLICY_BLOCK_LAST]))
        f = float(r.choice([0.0, 0.1, 0.3, 0.7, 0.9, 1.0]))
        block = int(r.integers(1, 6))
        p = dc.Params(C, S, policy, f, block)
        blob, table = dc.compress_chunks(data, p)
        c = oc.compress(data, C, S, policy, f, block=block)
        assert np.array_equal(table, c.table) and np.array_equal(blob, c.blob), (seed, it, S, C, n, policy, f, block)
        dc.validate(blob, table, p)
        assert np.array_equal(oc.decompress(blob, table, C, S, n), data)
        if C <= 512:
            k = int(r.integers(len(table)))
            if not table["raw_bytes_flags"][k] & dc.CHUNK_RAW:
                o, size, raw = int(table["off"][k]), int(table["comp_bytes"][k]), int(table["raw_bytes_flags"][k])
                assert pyref.parse_and_decode(blob[o:o + size].tobytes(), raw, S) == data[k * C:k * C + raw].tobytes()


# ------------------------------------------------------------------ the second coder (tANS)

def tans(C, S, policy=dc.POLICY_ALL_HUFF, f=0.0, block=0):
    return dc.Params(C, S, policy, f, block, codec=dc.CODEC_TANS)


@pytest.mark.parametrize("seed", [31, 32])
def test_random_inputs_host_tans_compressor_equals_oracle(seed):
    """The sweep above for tANS blobs: the oracle's blob and table, accepted by the validator, decoded back by
    the oracle, and on small chunks by the independent Python decoder."""
    from tests import pyref
    from tests.helpers import lopsided_bytes
    r = np.random.default_rng(seed)
    for it in range(80):
        S = int(r.choice([64, 128, 256]))
        C = int(r.choice([16, 48, 512, 4096, 16384, 65536]))
        n_chunks = int(r.integers(1, 5)) if C >= 16384 else int(r.integers(1, 30))
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
        else:  # a long tail: many values with a single state
            pz = 1.0 / np.arange(1, 257) ** float(r.uniform(0.7, 1.8))
            data = r.permutation(256).astype(np.uint8)[r.choice(256, size=n, p=pz / pz.sum())]
        policy = int(r.choice([dc.POLICY_ALL_HUFF, dc.POLICY_AUTO, dc.POLICY_RAW_FRACTION, dc.POLICY_BLOCK_LAST]))
        f = float(r.choice([0.0, 0.3, 0.9, 1.0]))
        block = int(r.integers(1, 6))
        p = tans(C, S, policy, f, block)
        blob, table = dc.compress_chunks(data, p)
        c = oc.compress(data, C, S, policy, f, block=block, codec=oc.TANS)
        assert np.array_equal(table, c.table) and np.array_equal(blob, c.blob), (seed, it, S, C, n, policy, f, block)
        cap, nc = dc.compress_bound(n, p)
        assert blob.size <= cap and nc == len(table)
        dc.validate(blob, table, p)
        assert np.array_equal(oc.decompress(blob, table, C, S, n, codec=oc.TANS), data)
        if C <= 512:
            k = int(r.integers(len(table)))
            if not table["raw_bytes_flags"][k] & dc.CHUNK_RAW:
                o, size, raw = int(table["off"][k]), int(table["comp_bytes"][k]), int(table["raw_bytes_flags"][k])
                assert pyref.parse_and_decode(blob[o:o + size].tobytes(), raw, S, tans=True) == data[k * C:k * C + raw].tobytes()


def test_validate_catches_corruption_of_tans_payloads():
    C, S = 4096, 64
    data = weightlike_bytes(5 * C + 9, 8)
    p = tans(C, S)
    blob, table = dc.compress_chunks(data, p)
    dc.validate(blob, table, p)
    k = 2
    o = int(table["off"][k])

    def expect_bad(b, chunk=k):
        with pytest.raises(dc.DCError) as e:
            dc.validate(b, table, p)
        assert e.value.code == -3 and f"chunk {chunk})" in str(e.value)

    b = blob.copy(); b[o] ^= 0x01            # one frequency one off: the sum is no longer 2048
    expect_bad(b)
    b = blob.copy(); b[o:o + 384] = 0        # no value at all
    expect_bad(b)
    # two frequencies changed so that the sum stays 2048: a different, valid table; the streams then walk other
    # states and (almost surely) do not end in state 0 or run out of bits
    bits = int.from_bytes(blob[o:o + 384].tobytes(), "little")
    q = [(bits >> (12 * v)) & 0xFFF for v in range(256)]
    hi = max(range(256), key=lambda v: q[v])
    lo = next(v for v in range(256) if q[v] > 0 and v != hi)
    q[hi] -= 1
    q[lo] += 1
    nbits = sum(x << (12 * v) for v, x in enumerate(q))
    b = blob.copy(); b[o:o + 384] = np.frombuffer(nbits.to_bytes(384, "little"), np.uint8)
    expect_bad(b)
    b = blob.copy(); b[o + 384 + 2 * 5] += 1   # block count of stream 5 one too many
    expect_bad(b)
    b = blob.copy(); b[o + 384 + 2 * S] ^= 0x10  # area not right after the header
    expect_bad(b)
    # a flipped stream bit: caught when the walk has not found its way back to the right states before the stream
    # ends (a field of many bits sets most of the next state, so walks do meet again) or runs out of bits
    hdr = (384 + 2 * S + 4 + 15) // 16 * 16
    caught = 0
    r = np.random.default_rng(2)
    for _ in range(40):
        b = blob.copy()
        b[o + hdr + int(r.integers(int(table["comp_bytes"][k]) - hdr - 16))] ^= 1 << int(r.integers(8))
        try:
            dc.validate(b, table, p)
        except dc.DCError:
            caught += 1
    assert caught >= 10
    # a Huffman blob is not a tANS blob
    hb, ht = dc.compress_chunks(data, dc.Params(C, S))
    with pytest.raises(dc.DCError):
        dc.validate(hb, ht, p)


def test_tans_argument_errors():
    data = weightlike_bytes(4096, 1)
    for bad in (dc.Params(4096, 32, codec=dc.CODEC_TANS), dc.Params(4096, 64, codec=2)):
        with pytest.raises(dc.DCError) as e:
            dc.compress_chunks(data, bad)
        assert e.value.code == -1


@pytest.mark.parametrize("codec", [dc.CODEC_HUFFMAN, dc.CODEC_TANS])
def test_what_the_validator_accepts_the_oracle_decodes(codec):
    """Damaged blobs and tables (flipped bits, overwritten header bytes, changed table fields, truncation): the
    validator rejects most; whatever it accepts, the oracle's decoder, which checks the format on its own, decodes
    without complaint (a flip in bits that nothing reads, or a table field that still describes the blob)."""
    r = np.random.default_rng(40 + codec)
    accepted = rejected = 0
    for it in range(250):
        S = int(r.choice([64, 128, 256]))
        C = int(r.choice([512, 4096, 16384]))
        n = max(1, int(r.integers(1, 6)) * C - int(r.integers(0, C)))
        data = weightlike_bytes(n, int(r.integers(1 << 30)))
        p = dc.Params(C, S, dc.POLICY_RAW_FRACTION, float(r.choice([0, 0.3])), codec=codec)
        blob, table = dc.compress_chunks(data, p)
        b, t = blob.copy(), table.copy()
        what = int(r.integers(0, 4))
        if what == 0:
            for _ in range(int(r.integers(1, 4))):
                b[r.integers(b.size)] ^= 1 << int(r.integers(8))
        elif what == 1:
            k = int(r.integers(len(t)))
            b[int(t["off"][k]) + int(r.integers(0, min(700, int(t["comp_bytes"][k]))))] = int(r.integers(256))
        elif what == 2:
            k = int(r.integers(len(t)))
            f = str(r.choice(["off", "comp_bytes", "raw_bytes_flags"]))
            t[f][k] = int(t[f][k]) ^ (1 << int(r.integers(0, 24)))
        else:
            b = b[:max(1, b.size - int(r.integers(1, 100)))].copy()
        try:
            dc.validate(b, t, p)
        except dc.DCError:
            rejected += 1
            continue
        accepted += 1
        sizes = (t["raw_bytes_flags"] & 0x7FFFFFFF).astype(np.int64)
        oc.decompress(b, t, C, S, int((len(t) - 1) * C + sizes[-1]), codec=codec)
    assert rejected > 150 and accepted > 0
