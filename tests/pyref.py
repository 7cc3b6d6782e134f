"""Independent pure-Python references used to pin the C oracle.

Nothing here calls the oracle or the library: a textbook Huffman (heap), an
exhaustive / dynamic-programming optimum for length-limited codes, and a
bit-walking decoder written straight from the format description.
"""
from __future__ import annotations

import heapq
import itertools
import math
from typing import Dict, List, Sequence


def entropy_bits(cnt: Sequence[int]) -> float:
    n = float(sum(cnt))
    return -sum(c / n * math.log2(c / n) for c in cnt if c > 0)


def huffman_lengths(cnt: Sequence[int]) -> List[int]:
    """Unrestricted Huffman code lengths (textbook heap construction)."""
    syms = [i for i, c in enumerate(cnt) if c > 0]
    out = [0] * len(cnt)
    if len(syms) == 1:
        out[syms[0]] = 1
        return out
    heap = [(cnt[i], i, (i,)) for i in syms]
    heapq.heapify(heap)
    tick = len(cnt)
    while len(heap) > 1:
        a = heapq.heappop(heap)
        b = heapq.heappop(heap)
        for s in a[2] + b[2]:
            out[s] += 1
        heapq.heappush(heap, (a[0] + b[0], tick, a[2] + b[2]))
        tick += 1
    return out


def cost(cnt: Sequence[int], lens: Sequence[int]) -> int:
    return sum(int(c) * int(l) for c, l in zip(cnt, lens))


def brute_force_limited_cost(cnt: Sequence[int], max_len: int) -> int:
    """Minimum of sum cnt*len over ALL length vectors in 1..max_len with Kraft sum <= 1."""
    syms = [c for c in cnt if c > 0]
    if len(syms) == 1:
        return syms[0]
    best = None
    for lens in itertools.product(range(1, max_len + 1), repeat=len(syms)):
        if sum(1 << (max_len - l) for l in lens) <= (1 << max_len):
            c = sum(a * b for a, b in zip(syms, lens))
            if best is None or c < best:
                best = c
    return best


def dp_limited_cost(cnt: Sequence[int], max_len: int) -> int:
    """Optimal length-limited cost by dynamic programming over levels.

    In some optimal code lengths do not decrease as counts decrease, so sort counts descending and
    hand out lengths level by level: f[i][k] = least cost of giving the i most frequent symbols
    lengths <= l using k units of 2^-max_len of the Kraft budget.
    """
    c = sorted((int(x) for x in cnt if x > 0), reverse=True)
    n = len(c)
    if n == 1:
        return c[0]
    pre = [0]
    for x in c:
        pre.append(pre[-1] + x)
    full = 1 << max_len
    INF = float("inf")
    f = [[INF] * (full + 1) for _ in range(n + 1)]
    f[0][0] = 0
    for l in range(1, max_len + 1):
        unit = 1 << (max_len - l)
        g = [row[:] for row in f]  # zero symbols at this level
        for i in range(n):
            fi = f[i]
            for k in range(0, full + 1):
                base = fi[k]
                if base == INF:
                    continue
                m = 1
                while i + m <= n and k + m * unit <= full:
                    v = base + l * (pre[i + m] - pre[i])
                    if v < g[i + m][k + m * unit]:
                        g[i + m][k + m * unit] = v
                    m += 1
        f = g
    return int(min(f[n]))


def tans_state_table(q: Sequence[int]):
    """(value, number) of every state of a tANS payload, from the written format alone: the byte values in
    ascending order take q[v] consecutive places each; place p is the state whose 11 bits are those of p
    reversed; the states of a value, sorted, are numbered q[v], q[v] + 1, ..."""
    assert sum(q) == 2048, "frequencies do not add up to the number of states"
    table = [None] * 2048
    place = 0
    for v in range(256):
        states = sorted(int(format(p, "011b")[::-1], 2) for p in range(place, place + q[v]))
        for i, x in enumerate(states):
            table[x] = (v, q[v] + i)
        place += q[v]
    return table


def parse_and_decode(payload: bytes, raw_bytes: int, S: int, tans: bool = False, flight: int = 0) -> bytes:
    """Decode one Huffman (or, with `tans`, tANS) payload by walking bits, from the written format alone.

    header: 128 bytes of 4-bit code lengths (value v in nibble v&1 of byte v>>1), then S little-endian
    u16 (low 12 bits: blocks of the stream; top 4 bits: bytes of its first block that exist, less
    one), then one u32 area offset per stream set (W = min(S, 64) streams a set), padded to 16; stream
    bit i = bit (i%8) of stream byte i/8; codes canonical by (length, value), written most significant
    bit first; bytes of 16-byte group g go to stream g % S.  A stream is a whole number of bytes, cut
    into 16-byte blocks from its end, so that only its first block is short (the bytes missing at its
    front do not exist; positions count from where that block would start).  An area holds the
    16-byte blocks of its streams, all but the first of each, in request order, then the short first
    blocks in stream order: before every half group (8 symbols) of all streams, each stream in turn that
    has blocks left and fewer than 392 placed bits beyond its position takes its next block (its own
    short first block, or the next of the area); the first such step runs five times.

    tANS payload: the front of the header is 384 bytes, the 12-bit frequencies of the 256 byte values as one
    little-endian bit string; a stream is the 11 bits of its first state and then, for every symbol, as many
    bits as the state asks for (fields least significant bit first): the symbol is the state's value, and with
    k the state's number and n = 11 - floor(log2 k) the next state is (k << n) - 2048 + the next n bits.  The
    first state is read after the fourth and before the fifth run of the first step; the last state is 0.

    flight > 0 checks what a decoder may rely on that gets a block `flight` steps after the step that took it
    (the blocks of the first four runs are there when decoding starts): at the start of every half group a
    stream has 215 bits beyond its position among the blocks that have arrived, or all of its blocks have.
    (215 = the 88 bits half a group can use, the 96 a decoder may hold in registers beyond them, 31 of rounding
    to whole words.)
    """
    front = 384 if tans else 128
    book: Dict[tuple, int] = {}
    table = None
    if tans:
        bits = int.from_bytes(payload[:384], "little")
        table = tans_state_table([(bits >> (12 * v)) & 0xFFF for v in range(256)])
    else:
        lens = [(payload[v >> 1] >> (4 * (v & 1))) & 15 for v in range(256)]
        code = 0
        prev = 0
        for l in range(1, 16):
            for v in range(256):
                if lens[v] == l:
                    if prev:
                        code = (code + 1) << (l - prev)
                    book[(l, code)] = v
                    prev = l
    W = min(S, 64)
    field = [int.from_bytes(payload[front + 2 * j:front + 2 + 2 * j], "little") for j in range(S)]
    nb = [x & 0xFFF for x in field]
    first_bytes = [(x >> 12) + 1 if x & 0xFFF else 0 for x in field]
    out = bytearray(raw_bytes)
    groups = (raw_bytes + 15) // 16
    rounds = (groups + S - 1) // S
    for w in range(S // W):
        o = front + 2 * S + 4 * w
        pos = int.from_bytes(payload[o:o + 4], "little")
        # the short first blocks start where the whole blocks of the set end
        whole = sum(nb[w * W + i] - 1 for i in range(W) if nb[w * W + i])
        first_at = []
        at = pos + 16 * whole
        for i in range(W):
            first_at.append(at)
            at += first_bytes[w * W + i]
        assert at <= len(payload), "area runs past the payload"
        data = [bytearray() for _ in range(W)]  # blocks of each stream, in order
        taken_at = [[] for _ in range(W)]       # the step at which each block was taken (-flight: before decoding)
        now = -flight
        # the position starts behind the bytes that the first block lacks
        bit = [8 * (16 - first_bytes[w * W + i]) if nb[w * W + i] else 0 for i in range(W)]

        def step():
            nonlocal pos
            for i in range(W):
                j = w * W + i
                if len(data[i]) < 16 * nb[j] and 8 * len(data[i]) - bit[i] < 392:
                    taken_at[i].append(now)
                    if len(data[i]) > 0:
                        data[i] += payload[pos:pos + 16]
                        pos += 16
                    else:
                        n = first_bytes[j]
                        data[i] += bytes(16 - n) + payload[first_at[i]:first_at[i] + n]

        def take(i, n):
            """the next n bits of stream i, first bit least significant"""
            v = 0
            for b in range(n):
                assert bit[i] < 8 * len(data[i]), "stream ran past its placed blocks"
                v |= ((data[i][bit[i] >> 3] >> (bit[i] & 7)) & 1) << b
                bit[i] += 1
            return v

        state = [0] * W
        for h in range(2 * rounds):
            step()
            if h == 0:
                step()
                step()
                step()
                if tans:
                    for i in range(W):
                        if w * W + i < groups:
                            state[i] = take(i, 11)
                now = 0
                step()
            if flight:
                for i in range(W):
                    arrived = sum(1 for t in taken_at[i] if t <= h - flight)
                    assert arrived == nb[w * W + i] or bit[i] + 215 <= 128 * arrived, (w * W + i, h, bit[i], arrived)
            now = h + 1
            for i in range(W):
                g = w * W + i + (h // 2) * S
                if g >= groups:
                    continue
                lo = 16 * g + 8 * (h % 2)
                for p in range(lo, min(lo + 8, raw_bytes)):
                    if tans:
                        out[p], k = table[state[i]]
                        n = 11 - (k.bit_length() - 1)
                        state[i] = (k << n) - 2048 + take(i, n)
                        continue
                    l = 0
                    c = 0
                    while True:
                        c = (c << 1) | take(i, 1)
                        l += 1
                        if (l, c) in book:
                            out[p] = book[(l, c)]
                            break
                        assert l < 15, "no code matched"
        assert not any(state), "a tANS stream does not end in state 0"
        for i in range(W):
            assert len(data[i]) == 16 * nb[w * W + i], "blocks left unplaced"
        assert pos == first_at[0], "whole blocks left over in the area"
    return bytes(out)
