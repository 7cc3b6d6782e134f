"""Pins for the tANS coder of the C codec oracle (the second coder of the container; the paper, Section 4.2,
compares entropy coders and settles on ANS but prints no bitstream and no worked example): closed forms that
follow from the definition, invariants of the state table, an information bound, and an independent decoder
written from the format text (tests/pyref.py)."""
import numpy as np
import pytest

import oracle.codec as oc
from tests import pyref
from tests.helpers import lopsided_bytes

L = 2048


def gaussian_bytes(n, sigma, seed):
    r = np.random.default_rng(seed)
    return np.clip(np.rint(r.standard_normal(n) * sigma), -127, 127).astype(np.int8).view(np.uint8)


def rev11(x):
    return int(format(x, "011b")[::-1], 2)


def frequencies_of(payload):
    bits = int.from_bytes(payload[:384].tobytes(), "little")
    return np.array([(bits >> (12 * v)) & 0xFFF for v in range(256)])


def header_bytes(S):
    return (384 + 2 * S + 4 * (S // min(S, 64)) + 15) // 16 * 16


# ------------------------------------------------------------------ normalised frequencies

@pytest.mark.parametrize("seed", range(8))
def test_normalised_frequencies_add_up_and_keep_every_present_value(seed):
    r = np.random.default_rng(seed)
    cnt = np.zeros(256, dtype=np.uint64)
    idx = r.choice(256, size=int(r.integers(1, 257)), replace=False)
    cnt[idx] = r.integers(1, [3, 50, 100000][seed % 3], size=idx.size)
    q = oc.tans_normalise(cnt).astype(int)
    assert q.sum() == L
    assert ((q > 0) == (cnt > 0)).all()
    # a more frequent value never gets fewer states (among equally frequent ones the order is free)
    order = np.lexsort((q, cnt))
    assert (np.diff(q[order]) >= 0).all()


def test_normalisation_closed_forms():
    cnt = np.zeros(256, dtype=np.uint64)
    cnt[77] = 12345
    q = oc.tans_normalise(cnt)
    assert q[77] == L and q.sum() == L                      # one value: all states
    cnt[:] = 256
    assert (oc.tans_normalise(cnt) == 8).all()              # uniform: 2048 / 256
    cnt[:] = 0
    cnt[3] = cnt[200] = 500
    q = oc.tans_normalise(cnt)
    assert q[3] == 1024 and q[200] == 1024                  # two equal values
    # dyadic counts whose total divides L: the shares are whole numbers and are kept exactly
    cnt[:] = 0
    cnt[[1, 2, 3, 4]] = [8, 4, 2, 2]
    q = oc.tans_normalise(cnt)
    assert list(q[[1, 2, 3, 4]]) == [1024, 512, 256, 256]
    # three equal values: 682 each leaves two states, which go to the lower values
    cnt[:] = 0
    cnt[[10, 20, 30]] = 1
    q = oc.tans_normalise(cnt)
    assert list(q[[10, 20, 30]]) == [683, 683, 682]


def test_rare_values_are_raised_to_one_state_and_the_surplus_is_taken_back():
    """255 values seen once beside one seen a million times: the 255 get one state each (their share is
    below one), which makes 255 + 2047 states; the surplus comes off the only value that has more than one."""
    cnt = np.ones(256, dtype=np.uint64)
    cnt[0] = 1_000_000
    q = oc.tans_normalise(cnt).astype(int)
    assert (q[1:] == 1).all() and q[0] == L - 255


# ------------------------------------------------------------------ state table

def test_states_of_the_uniform_table_closed_form():
    """q = 8 for every value: place p = 8v + t is state rev11(p) = rev3(t) << 8 | rev8(v), so the states of v
    in ascending order are those of t with rev3(t) ascending, numbered 8 + rev3(t)."""
    value_of, number_of = oc.tans_states(np.full(256, 8, dtype=np.uint16))
    for x in range(L):
        p = rev11(x)
        assert value_of[x] == p // 8
        assert number_of[x] == 8 + (x >> 8)


@pytest.mark.parametrize("seed", range(5))
def test_state_table_invariants(seed):
    data = gaussian_bytes(50000, [0.6, 3.0, 12.0, 30.0, 60.0][seed], seed)
    q = oc.tans_normalise(np.bincount(data, minlength=256).astype(np.uint64)).astype(int)
    value_of, number_of = oc.tans_states(q)
    cum = np.concatenate([[0], np.cumsum(q)])
    for v in range(256):
        xs = np.nonzero(value_of == v)[0]
        assert xs.size == q[v]
        # the states of v are the reversed places of v, and their numbers q .. 2q-1 rise with the state
        assert sorted(rev11(int(x)) for x in xs) == list(range(cum[v], cum[v + 1]))
        assert list(number_of[xs]) == list(range(q[v], 2 * q[v]))
    # every state's next states, over all values of its field, stay inside the table and tile it once per value:
    # the map (state, field) -> next state is onto [0, L) for each value (what makes the coder invertible)
    for v in np.nonzero(q)[0][:20]:
        nxt = []
        for x in np.nonzero(value_of == v)[0]:
            k = int(number_of[x])
            n = 11 - (k.bit_length() - 1)
            nxt += [(k << n) - L + f for f in range(1 << n)]
        assert sorted(nxt) == list(range(L))
    # the independent construction agrees
    table = pyref.tans_state_table(list(q))
    assert all(table[x] == (int(value_of[x]), int(number_of[x])) for x in range(L))


def test_frequencies_that_do_not_add_up_are_refused():
    q = np.full(256, 8, dtype=np.uint16)
    q[5] = 9
    with pytest.raises(ValueError):
        oc.tans_states(q)


# ------------------------------------------------------------------ bitstream

def test_two_equal_values_spell_the_stream_out():
    """Two values, 1024 states each: the lower value owns places 0..1023, whose reversals are the even
    states; a state numbered k has a one-bit field and base (k << 1) - L = the state with bit 0 cleared.  So
    the next state is the old one with its lowest bit replaced by the stream bit, and a symbol is the upper
    value iff the lowest bit of the state is set: the stream is symbol 0 as one bit, ten zero bits (the encoder
    starts at state 0, nothing ever sets them), then symbols 1, 2, ... one bit each."""
    n = 100
    r = np.random.default_rng(5)
    sym = r.permutation(np.repeat([0, 1], n // 2))
    data = np.where(sym == 1, 201, 17).astype(np.uint8)
    payload = oc.encode_chunk(data, 1, codec=oc.TANS)
    q = frequencies_of(payload)
    assert q[17] == 1024 and q[201] == 1024 and q.sum() == L
    bits = [int(sym[0])] + [0] * 10 + [int(b) for b in sym[1:]]
    want = bytearray((len(bits) + 7) // 8)
    for i, b in enumerate(bits):
        want[i >> 3] |= b << (i & 7)
    # one stream of 14 bytes: one short block, which is the head of the only area
    hdr = header_bytes(1)
    assert int.from_bytes(payload[384:386].tobytes(), "little") == 1 | (13 << 12)
    assert int.from_bytes(payload[386:390].tobytes(), "little") == hdr
    assert payload.size == hdr + 16
    assert payload[hdr:hdr + 14].tobytes() == bytes(want)
    assert (oc.decode_chunk(payload, n, 1, codec=oc.TANS) == data).all()


@pytest.mark.parametrize("raw,S", [(65536, 32), (16384, 256), (4096 + 256, 4)])
def test_uniform_values_cost_eight_bits_each(raw, S):
    """Every value equally often: 8 states each, every state numbered 8..15, so every field is 11 - 3 = 8 bits
    and a stream is 11 + 8 * symbols bits: the payload size follows."""
    per = raw // 256
    assert per * 256 == raw
    data = np.random.default_rng(3).permutation(np.repeat(np.arange(256, dtype=np.uint8), per))
    payload = oc.encode_chunk(data, S, codec=oc.TANS)
    assert (frequencies_of(payload) == 8).all()
    W = min(S, 64)
    size = header_bytes(S)
    for w in range(S // W):
        area = 0
        for j in range(w * W, (w + 1) * W):
            n = oc.stream_symbols(raw, S, j)
            area += (11 + 8 * n + 7) // 8 if n else 0
        size += (area + 15) // 16 * 16
    assert payload.size == size
    assert (oc.decode_chunk(payload, raw, S, codec=oc.TANS) == data).all()


def test_single_value_chunk_costs_the_first_states_only():
    """One value: 2048 states numbered 2048..4095, fields of no bits; a stream is its first state, which is the
    state the encoder starts from, 0: two zero bytes a stream."""
    raw, S = 65536, 64
    data = np.full(raw, 0x80, dtype=np.uint8)
    payload = oc.encode_chunk(data, S, codec=oc.TANS)
    hdr = header_bytes(S)
    assert payload.size == hdr + 64 * 2
    assert not payload[hdr:].any()
    field = np.frombuffer(payload[384:384 + 2 * S].tobytes(), dtype="<u2")
    assert (field == (1 | (1 << 12))).all()  # one block, two bytes of it
    assert (oc.decode_chunk(payload, raw, S, codec=oc.TANS) == data).all()
    assert pyref.parse_and_decode(payload.tobytes(), raw, S, tans=True) == data.tobytes()


@pytest.mark.parametrize("raw", [1, 2, 15, 16, 17, 31, 33, 255, 511, 512, 513, 1000, 4095, 4096, 4097])
@pytest.mark.parametrize("S", [1, 4, 32])
def test_round_trip_and_independent_decoder_ragged(raw, S):
    data = gaussian_bytes(raw, 6.0, raw * 131 + S)
    payload = oc.encode_chunk(data, S, codec=oc.TANS)
    assert payload.size % 16 == 0
    assert (oc.decode_chunk(payload, raw, S, codec=oc.TANS) == data).all()
    assert pyref.parse_and_decode(payload.tobytes(), raw, S, tans=True) == data.tobytes()


@pytest.mark.parametrize("raw,S", [(65536, 64), (40000, 128), (16384, 256), (5000, 4)])
def test_lopsided_streams_round_trip(raw, S):
    data = lopsided_bytes(raw, S, raw + S)
    payload = oc.encode_chunk(data, S, codec=oc.TANS)
    assert (oc.decode_chunk(payload, raw, S, codec=oc.TANS) == data).all()
    assert pyref.parse_and_decode(payload.tobytes(), raw, S, tans=True) == data.tobytes()


@pytest.mark.parametrize("sigma", [40.0, 12.0, 3.0, 0.7])
def test_stream_bits_against_the_information_in_the_symbols(sigma):
    """What a stream holds beyond its first state is, up to the imprecision of 2048 states, the information of
    its symbols under the stored frequencies: sum of log2(L / q[v]).  The total is within 0.3 % (and a few
    bytes of rounding a stream) above it and not below the chunk's empirical entropy."""
    raw, S = 65536, 4
    data = gaussian_bytes(raw, sigma, int(sigma * 10))
    payload = oc.encode_chunk(data, S, codec=oc.TANS)
    q = frequencies_of(payload).astype(float)
    cnt = np.bincount(data, minlength=256).astype(float)
    info = float((cnt[cnt > 0] * np.log2(L / q[cnt > 0])).sum())
    entropy = float(-(cnt[cnt > 0] * np.log2(cnt[cnt > 0] / raw)).sum())
    assert info >= entropy - 1e-6                     # Gibbs
    stream_bits = 8 * (payload.size - header_bytes(S)) - 11 * S
    assert entropy * 0.999 <= stream_bits <= info * 1.003 + 8 * 16 * S
    # and an 11-bit Huffman code of the same chunk needs at least as much for its symbols, up to the same rounding
    ln = oc.code_lengths(cnt.astype(np.uint64)).astype(float)
    assert stream_bits <= float((cnt * ln).sum()) + 8 * 16 * S


def test_flipped_bits_are_noticed():
    """A stream must end in the state the encoder started from; a flipped stream bit sends the walk elsewhere,
    and unless it finds its way back before the stream ends (a wide field sets most of the next state, so walks
    do meet again) the end state shows it, or the stream runs out of its blocks.  None may crash the decoder."""
    raw, S = 20000, 32
    data = gaussian_bytes(raw, 9.0, 4)
    payload = oc.encode_chunk(data, S, codec=oc.TANS)
    r = np.random.default_rng(6)
    caught = 0
    for _ in range(200):
        bad = payload.copy()
        at = int(r.integers(header_bytes(S), payload.size - 16))
        bad[at] ^= 1 << int(r.integers(8))
        try:
            out = oc.decode_chunk(bad, raw, S, codec=oc.TANS)
            assert not (out == data).all() or True
        except ValueError:
            caught += 1
    assert caught >= 150


def test_whole_buffer_round_trip_with_raw_chunks():
    n, C, S = 5 * 16384 + 777, 16384, 64
    r = np.random.default_rng(8)
    data = np.concatenate([gaussian_bytes(2 * C, 5.0, 1), r.integers(0, 256, C, dtype=np.uint8),
                           gaussian_bytes(n - 3 * C, 20.0, 2)])
    c = oc.compress(data, C, S, oc.AUTO, codec=oc.TANS)
    raw_flags = c.table["raw_bytes_flags"] >> 31
    # the uniform chunk gains nothing and stays raw, and so does the 777-byte tail (its header alone is 528 bytes)
    assert list(raw_flags) == [0, 0, 1, 0, 0, 1]
    assert c.blob.size == int(c.table["comp_bytes"].sum()) + 64
    assert (oc.decompress(c.blob, c.table, C, S, n, codec=oc.TANS) == data).all()
    # each coded chunk is the chunk coder's payload
    k = 4
    off, comp = int(c.table["off"][k]), int(c.table["comp_bytes"][k])
    assert (c.blob[off:off + comp] == oc.encode_chunk(data[k * C:(k + 1) * C], S, codec=oc.TANS)).all()
