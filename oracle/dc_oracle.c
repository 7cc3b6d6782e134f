/*
 * CPU oracle for the chunked Huffman codec of INT8 LLM weights.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code, header, table or helper
 * with the library, and only tests, the smoke check and the benchmark's
 * cpu_baseline leg may build or call it.
 *
 * What the paper fixes (Section 3.1, Section 3.3 "Speed Adaptive Partial
 * Compression"): quantised INT8 weights are compressed losslessly, in
 * independently coded data chunks, and only some chunks of every data block are
 * compressed while the others stay raw.  The paper picks an entropy coder
 * (Section 4.2) but describes no bitstream.  The bitstream here is this
 * project's own: a per-chunk canonical Huffman code over the 256 byte values,
 * code length at most 11, each chunk split into S symbol-interleaved
 * sub-bitstreams.  The format, restated:
 *
 *   chunk table entry (16 bytes, little endian)
 *     u64 off          payload offset in the blob, multiple of 16
 *     u32 comp_bytes   payload size including padding, multiple of 16
 *     u32 raw_bytes | RAW<<31
 *   blob              the payloads back to back in chunk order, then 64
 *                     closing bytes: 48 zeros and a trailer of 16 bytes that
 *                     names the format and the parameters (orc_close_blob)
 *   raw payload       raw_bytes bytes, zero padded to 16
 *   Huffman payload
 *     [0,128)          code length of byte value v in nibble (v&1) of byte v>>1
 *                      (0 = value absent, else 1..11)
 *     [128,128+2S)     u16 per sub-stream j: bits 0-11 nb[j], the number of
 *                      16-byte blocks of the stream; bits 12-15 hb[j]-1, where
 *                      hb[j] = 1..16 is the number of bytes of its first block
 *                      that hold stream bits (both 0 for an empty stream)
 *     then             u32 set_off[w], one per stream set: start of the set's
 *                      area from payload start; then zeros to a multiple of
 *                      16.  A stream set is W = min(S,64) consecutive
 *                      sub-streams.
 *     sub-streams      stream j = codes of the bytes of the 16-byte groups
 *                      g = j, j+S, j+2S, ... of the chunk, in increasing
 *                      position, rounded up to whole bytes.  It is cut into
 *                      16-byte blocks from its END: block 0 is short (its
 *                      first pad[j] = 16 - hb[j] bytes do not exist), every
 *                      later block is whole.  Positions in a stream count from
 *                      the start of block 0, so the first code starts at bit
 *                      8*pad[j].
 *     set areas        one per stream set, back to back after the header:
 *                      first the whole blocks (blocks 1, 2, ... of each of the
 *                      set's streams) in the order of the placement rule
 *                      below; then the heads: for the streams of the set in
 *                      ascending order, the hb[j] bytes of block 0; then zeros
 *                      to a multiple of 16
 *   bit order          stream bit i is bit (i mod 8) of stream byte i/8; a code
 *                      is written most significant code bit first
 *   codes              canonical: lengths by package-merge (below), codes
 *                      numbered in order of (length, byte value)
 *
 * Placement rule.  Decoding goes in steps h = 0, 1, ...: step h comes before
 * symbols 8*(h%2) .. 8*(h%2)+7 of group number h/2 of every stream.  With c[j]
 * the stream bits used by the symbols of stream j before step h and f[j] the
 * blocks of stream j placed so far: at a step, for j ascending over the set, if
 * f[j] < nb[j] and 128*f[j] - c[j] < 392 then the stream takes block f[j] and
 * f[j] grows by one: block 0 is the stream's head, any other block is the next
 * one in the area.  Step 0 is carried out five times, every later step once.
 * (c[j] counts from the start of block 0: it is 8*pad[j] before the first
 * symbol, which is why a stream may need a fourth block before it starts.  For
 * a Huffman payload the fifth time changes nothing: c[j] is what it was, and a
 * fifth block would have to start less than 392 bits beyond a position of at
 * most 120.  In a tANS payload the first state is read between the fourth and
 * the fifth time.)
 *
 * Every function is written for a reader to check by eye, not for speed:
 * one bit at a time, explicit item lists, no tables.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_CAP (-2)
#define ORC_E_FORMAT (-3)

#define ORC_RAW_FLAG 0x80000000u
#define ORC_BLOB_TAIL 64
/* format 5 of the container: sub-streams cut to bytes with a short first block, look-ahead of 392
 * bits, and a trailer in the blob's closing bytes that says so */
#define ORC_FORMAT 5
#define ORC_LOOKAHEAD_IN_TRAILER 392

enum { ORC_ALL_HUFF = 0, ORC_AUTO = 1, ORC_RAW_FRACTION = 2, ORC_RAW_MASK = 3, ORC_BLOCK_LAST = 4 };

typedef struct {
    uint64_t off;
    uint32_t comp_bytes;
    uint32_t raw_bytes_flags;
} orc_chunk;

/* ---------------------------------------------------------------- histogram */

/* Counts of each byte value (the int8 weight seen as its two's-complement byte). */
void orc_histogram(const uint8_t *src, uint64_t n, uint64_t *cnt)
{
    memset(cnt, 0, 256 * sizeof(uint64_t));
    for (uint64_t i = 0; i < n; i++)
        cnt[src[i]]++;
}

/* ------------------------------------------------- length-limited code lengths */

/*
 * Package-merge (Larmore & Hirschberg's coin-collector view), written with
 * explicit items.  An item is a weight plus, for every leaf, how many times the
 * leaf is inside it.  Level 1 is the sorted leaves.  Level j is the sorted
 * leaves merged with the packages made of consecutive pairs of level j-1.  The
 * first 2n-2 items of level max_len are bought; a leaf's code length is the
 * number of bought items that contain it, counted with multiplicity.
 *
 * Determinism: leaves are ordered by (count ascending, byte value ascending);
 * when a leaf and a package weigh the same the leaf goes first; packages keep
 * the order they were made in.
 *
 * Values with count 0 get length 0.  A single distinct value gets length 1.
 */
typedef struct {
    uint64_t w;
    uint16_t mult[256]; /* indexed by leaf rank */
} pm_item;

int orc_code_lengths(const uint64_t *cnt, int max_len, uint8_t *len)
{
    int leaf_sym[256];
    int n = 0;
    memset(len, 0, 256);
    if (max_len < 1 || max_len > 15)
        return ORC_E_ARG;
    for (int v = 0; v < 256; v++)
        if (cnt[v] > 0)
            leaf_sym[n++] = v;
    if (n == 0)
        return ORC_E_ARG;
    if (n == 1) {
        len[leaf_sym[0]] = 1;
        return ORC_OK;
    }
    if ((n - 1) >> max_len)
        return ORC_E_ARG; /* more than 2^max_len values cannot be coded */

    /* insertion sort of the leaves by (count, byte value) */
    for (int i = 1; i < n; i++) {
        int s = leaf_sym[i], j = i;
        while (j > 0 && (cnt[leaf_sym[j - 1]] > cnt[s])) {
            leaf_sym[j] = leaf_sym[j - 1];
            j--;
        }
        leaf_sym[j] = s;
    }

    pm_item *prev = calloc(2 * (size_t)n, sizeof(pm_item));
    pm_item *cur = calloc(2 * (size_t)n, sizeof(pm_item));
    pm_item *pk = calloc((size_t)n, sizeof(pm_item));
    if (!prev || !cur || !pk) {
        free(prev); free(cur); free(pk);
        return ORC_E_CAP;
    }
    int n_prev = n;
    for (int i = 0; i < n; i++) {
        prev[i].w = cnt[leaf_sym[i]];
        prev[i].mult[i] = 1;
    }
    for (int level = 2; level <= max_len; level++) {
        int n_pk = n_prev / 2;
        for (int i = 0; i < n_pk; i++) {
            pk[i].w = prev[2 * i].w + prev[2 * i + 1].w;
            for (int r = 0; r < n; r++)
                pk[i].mult[r] = (uint16_t)(prev[2 * i].mult[r] + prev[2 * i + 1].mult[r]);
        }
        int a = 0, b = 0, m = 0;
        while (a < n || b < n_pk) {
            int take_leaf;
            if (a >= n) take_leaf = 0;
            else if (b >= n_pk) take_leaf = 1;
            else take_leaf = (cnt[leaf_sym[a]] <= pk[b].w);
            if (take_leaf) {
                memset(&cur[m], 0, sizeof(pm_item));
                cur[m].w = cnt[leaf_sym[a]];
                cur[m].mult[a] = 1;
                a++;
            } else {
                cur[m] = pk[b];
                b++;
            }
            m++;
        }
        pm_item *t = prev; prev = cur; cur = t;
        n_prev = m;
    }
    int buy = 2 * n - 2;
    int rc = ORC_OK;
    if (n_prev < buy) {
        rc = ORC_E_ARG;
    } else {
        for (int r = 0; r < n; r++) {
            unsigned l = 0;
            for (int i = 0; i < buy; i++)
                l += prev[i].mult[r];
            len[leaf_sym[r]] = (uint8_t)l;
        }
    }
    free(prev); free(cur); free(pk);
    return rc;
}

/* --------------------------------------------------------------- canonical codes */

/*
 * Codes are numbered in order of (length, byte value): the first code of the
 * shortest length is 0, and going to the next code adds one and, when the
 * length grows by d, appends d zero bits.
 */
void orc_canonical_codes(const uint8_t *len, uint16_t *code)
{
    unsigned next = 0;
    int prev_len = 0;
    memset(code, 0, 256 * sizeof(uint16_t));
    for (int l = 1; l <= 15; l++) {
        for (int v = 0; v < 256; v++) {
            if (len[v] != l)
                continue;
            if (prev_len != 0)
                next = (next + 1) << (l - prev_len);
            code[v] = (uint16_t)next;
            prev_len = l;
        }
    }
}

/* ------------------------------------------------------------ sub-stream geometry */

/* Number of symbols of sub-stream j of a chunk of raw_bytes bytes split S ways. */
uint32_t orc_stream_symbols(uint32_t raw_bytes, uint32_t S, uint32_t j)
{
    uint32_t n = 0;
    uint32_t groups = (raw_bytes + 15) / 16;
    for (uint32_t g = j; g < groups; g += S) {
        uint32_t lo = 16 * g;
        uint32_t hi = lo + 16 < raw_bytes ? lo + 16 : raw_bytes;
        n += hi - lo;
    }
    return n;
}

static uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

#define ORC_BLOCK 16u        /* bytes of a block */
#define ORC_LOOKAHEAD 392u   /* bits a stream keeps placed beyond its position */

/* Streams of a set, number of sets, header size. */
static uint32_t set_width(uint32_t S) { return S < 64 ? S : 64; }
static uint32_t header_bytes(uint32_t S)
{
    return (uint32_t)round_up(128 + 2 * (uint64_t)S + 4 * (uint64_t)(S / set_width(S)), 16);
}

/* Upper bound of a Huffman payload: header + 11 bits a symbol + one partial block a stream
 * (more than the padding of the sets can take). */
uint64_t orc_huff_bound(uint32_t raw_bytes, uint32_t S)
{
    return round_up(header_bytes(S) + ((uint64_t)raw_bytes * 11 + 7) / 8 + ORC_BLOCK * (uint64_t)S, 16);
}

/* Number of symbols of stream j that come before step h: all of its groups before group h/2,
 * plus up to 8 symbols of group h/2 when h is odd. */
static uint32_t symbols_before_step(uint32_t raw_bytes, uint32_t S, uint32_t j, uint32_t h)
{
    uint32_t groups = (raw_bytes + 15) / 16;
    uint32_t n = 0;
    uint32_t r = 0;
    for (uint32_t g = j; g < groups; g += S, r++) {
        uint32_t lo = 16 * g;
        uint32_t size = (lo + 16 < raw_bytes ? lo + 16 : raw_bytes) - lo;
        if (r < h / 2)
            n += size;
        else if (r == h / 2 && (h & 1))
            n += size < 8 ? size : 8;
    }
    return n;
}

/* Number of steps of a chunk: two for every round of S groups. */
static uint32_t step_count(uint32_t raw_bytes, uint32_t S)
{
    uint32_t groups = (raw_bytes + 15) / 16;
    return 2 * ((groups + S - 1) / S);
}

/* ----------------------------------------------------------------------- tANS model */

/*
 * The second coder of the container: tabled asymmetric numeral systems with L =
 * 2048 states (the paper, Section 4.2, compares entropy coders and settles on
 * ANS).  Only the front of the chunk header and what a sub-stream holds differ
 * from the Huffman payload:
 *
 *   tANS payload
 *     [0,384)          normalised frequency q[v] of byte value v, 12 bits each:
 *                      bits 12v .. 12v+11 of the 384 bytes read as one bit string
 *                      (bit i of the string = bit i%8 of byte i/8); the q add up
 *                      to L; q[v] = 0 for an absent value
 *     [384,384+2S)     the u16 per sub-stream, then set_off, then padding, as in
 *                      the Huffman payload
 *   states             position p = 0 .. L-1 in the list of byte values in
 *                      ascending order, value v taking q[v] consecutive places, is
 *                      state x = p with its 11 bits reversed.  The states of v
 *                      taken in ascending x are numbered k = q[v] .. 2q[v]-1.
 *                      A state with number k has nb = 11 - floor(log2 k) and
 *                      base = (k << nb) - L.
 *   sub-stream         bit fields, least significant bit first.  Decoder: x = the
 *                      first 11 bits; for every symbol: the symbol is the value of
 *                      state x, then x = base(x) + the next nb(x) bits.  Encoder:
 *                      X = L; for the symbols from the last to the first, v being
 *                      the symbol: nb = the smallest n with (X >> n) < 2q[v]; the
 *                      symbol's field is the low nb bits of X; X = L + the state
 *                      of v with number X >> nb.  The stream is X - L after the
 *                      first symbol, then the fields in symbol order.  (So the
 *                      decoder ends in state 0.)
 *   placement rule     as for Huffman, c[j] counting every bit read; the 11 bits
 *                      of the first state are read after the fourth and before the
 *                      fifth carrying out of step 0.
 *   frequencies        (what the compressor stores) with n the chunk's size:
 *                      q[v] = max(1, floor(count[v]*L/n)) for present values.
 *                      While the sum is below L: add one to the value with the
 *                      largest count[v]/q[v] (as exact fractions; lower value
 *                      among equals).  While the sum is above L: take one from
 *                      the value with q[v] > 1 and the smallest
 *                      count[v]/(q[v]-1) (lower value among equals).
 */
#define ORC_CODEC_HUFFMAN 0
#define ORC_CODEC_TANS 1
#define ORC_TANS_BITS 11
#define ORC_TANS_L 2048u

/* Frequencies normalised to L by the rule above. */
int orc_tans_normalise(const uint64_t *cnt, uint16_t *q)
{
    uint64_t n = 0, sum = 0;
    for (int v = 0; v < 256; v++)
        n += cnt[v];
    if (n == 0)
        return ORC_E_ARG;
    for (int v = 0; v < 256; v++) {
        uint64_t f = cnt[v] * ORC_TANS_L / n;
        q[v] = cnt[v] == 0 ? 0 : (uint16_t)(f < 1 ? 1 : f);
        sum += q[v];
    }
    while (sum < ORC_TANS_L) {
        int best = -1;
        for (int v = 0; v < 256; v++) {
            if (cnt[v] == 0)
                continue;
            /* cnt[v]/q[v] > cnt[best]/q[best] */
            if (best < 0 || cnt[v] * q[best] > cnt[best] * q[v])
                best = v;
        }
        q[best]++;
        sum++;
    }
    while (sum > ORC_TANS_L) {
        int best = -1;
        for (int v = 0; v < 256; v++) {
            if (q[v] < 2)
                continue;
            /* cnt[v]/(q[v]-1) < cnt[best]/(q[best]-1) */
            if (best < 0 || cnt[v] * (uint64_t)(q[best] - 1) < cnt[best] * (uint64_t)(q[v] - 1))
                best = v;
        }
        if (best < 0)
            return ORC_E_ARG; /* more than L present values cannot happen with 256 values */
        q[best]--;
        sum--;
    }
    return ORC_OK;
}

static unsigned reverse_bits(unsigned x, int bits)
{
    unsigned r = 0;
    for (int i = 0; i < bits; i++)
        if ((x >> i) & 1u)
            r |= 1u << (bits - 1 - i);
    return r;
}

/*
 * The states: value_of[x] and number_of[x] for every state x.  Returns
 * ORC_E_FORMAT when the frequencies do not add up to L.
 */
int orc_tans_states(const uint16_t *q, uint8_t *value_of, uint16_t *number_of)
{
    unsigned p = 0, next[256];
    for (int v = 0; v < 256; v++)
        p += q[v];
    if (p != ORC_TANS_L)
        return ORC_E_FORMAT;
    p = 0;
    for (int v = 0; v < 256; v++) {
        for (unsigned i = 0; i < q[v]; i++, p++)
            value_of[reverse_bits(p, ORC_TANS_BITS)] = (uint8_t)v;
        next[v] = q[v];
    }
    for (unsigned x = 0; x < ORC_TANS_L; x++) /* ascending x: q[v], q[v]+1, ... */
        number_of[x] = (uint16_t)next[value_of[x]]++;
    return ORC_OK;
}

static int floor_log2(unsigned k)
{
    int l = 0;
    while (k >> (l + 1))
        l++;
    return l;
}

/* ------------------------------------------------------------- one sub-stream, written */

static void put_bit(uint8_t *st, uint64_t *bit, unsigned b)
{
    if (st && b)
        st[*bit >> 3] |= (uint8_t)(1u << (*bit & 7));
    (*bit)++;
}

/* The positions of the symbols of stream j, in order; returns how many. */
static uint32_t stream_positions(uint32_t raw_bytes, uint32_t S, uint32_t j, uint32_t *pos)
{
    uint32_t groups = (raw_bytes + 15) / 16, n = 0;
    for (uint32_t g = j; g < groups; g += S)
        for (uint32_t p = 16 * g; p < 16 * g + 16 && p < raw_bytes; p++)
            pos[n++] = p;
    return n;
}

/*
 * Huffman: the codes of the stream's symbols from bit `bit` of st on, most
 * significant code bit first.  used[k] = position after the first k symbols.
 * st and used may be NULL (only the end position is wanted).
 */
static uint64_t huff_stream(const uint8_t *src, const uint32_t *pos, uint32_t n, const uint8_t *len,
                            const uint16_t *code, uint8_t *st, uint64_t bit, uint64_t *used)
{
    if (used)
        used[0] = bit;
    for (uint32_t k = 0; k < n; k++) {
        int l = len[src[pos[k]]];
        unsigned c = code[src[pos[k]]];
        for (int b = l - 1; b >= 0; b--)
            put_bit(st, &bit, (c >> b) & 1u);
        if (used)
            used[k + 1] = bit;
    }
    return bit;
}

/*
 * tANS: the first state and then the fields of the stream's symbols from bit
 * `bit` of st on.  state_of[cum[v] + i] is the state of value v with number
 * q[v] + i.  used[k] = position after the state and the first k fields.
 * scratch holds n fields and n widths.
 */
static uint64_t tans_stream(const uint8_t *src, const uint32_t *pos, uint32_t n, const uint16_t *q,
                            const uint16_t *cum, const uint16_t *state_of, uint16_t *field, uint8_t *width,
                            uint8_t *st, uint64_t bit, uint64_t *used)
{
    if (n == 0) {
        if (used)
            used[0] = bit;
        return bit;
    }
    unsigned X = ORC_TANS_L;
    for (uint32_t k = n; k-- > 0;) {
        unsigned v = src[pos[k]], nb = 0;
        while ((X >> nb) >= 2u * q[v])
            nb++;
        field[k] = (uint16_t)(X & ((1u << nb) - 1u));
        width[k] = (uint8_t)nb;
        X = ORC_TANS_L + state_of[cum[v] + ((X >> nb) - q[v])];
    }
    for (int b = 0; b < ORC_TANS_BITS; b++)
        put_bit(st, &bit, ((X - ORC_TANS_L) >> b) & 1u);
    if (used)
        used[0] = bit;
    for (uint32_t k = 0; k < n; k++) {
        for (unsigned b = 0; b < width[k]; b++)
            put_bit(st, &bit, (field[k] >> b) & 1u);
        if (used)
            used[k + 1] = bit;
    }
    return bit;
}

/* ------------------------------------------------------------------ chunk encode */

static uint32_t front_bytes(int codec) { return codec == ORC_CODEC_TANS ? 384u : 128u; }
static uint32_t header_bytes_codec(uint32_t S, int codec)
{
    return (uint32_t)round_up(front_bytes(codec) + 2 * (uint64_t)S + 4 * (uint64_t)(S / set_width(S)), 16);
}

/* Upper bound of a coded payload of either kind: header + 11 bits a symbol + 11 bits and one
 * partial block a stream (more than the padding of the sets can take). */
uint64_t orc_payload_bound(uint32_t raw_bytes, uint32_t S, int codec)
{
    return round_up(header_bytes_codec(S, codec) + ((uint64_t)raw_bytes * 11 + 7) / 8 + (ORC_BLOCK + 2) * (uint64_t)S, 16);
}

/*
 * Encode one chunk as a Huffman (codec 0) or tANS (codec 1) payload.  Returns the
 * payload size (multiple of 16) or 0 on error (capacity too small, bad
 * arguments).  out may be NULL to only measure.  max_len (Huffman only) is 11
 * in the format; tests may pass less.
 */
uint64_t orc_encode_chunk_codec(const uint8_t *src, uint32_t raw_bytes, uint32_t S, int codec, int max_len,
                                uint8_t *out, uint64_t cap)
{
    uint64_t cnt[256];
    uint8_t len[256];
    uint16_t code[256];
    uint16_t q[256], cum[257], number_of[ORC_TANS_L], state_of[ORC_TANS_L];
    uint8_t value_of[ORC_TANS_L];
    if (raw_bytes == 0 || S == 0 || max_len > 11 || S % set_width(S) != 0)
        return 0;
    if (codec != ORC_CODEC_HUFFMAN && codec != ORC_CODEC_TANS)
        return 0;
    orc_histogram(src, raw_bytes, cnt);
    if (codec == ORC_CODEC_HUFFMAN) {
        if (orc_code_lengths(cnt, max_len, len) != ORC_OK)
            return 0;
        orc_canonical_codes(len, code);
    } else {
        if (orc_tans_normalise(cnt, q) != ORC_OK || orc_tans_states(q, value_of, number_of) != ORC_OK)
            return 0;
        cum[0] = 0;
        for (int v = 0; v < 256; v++)
            cum[v + 1] = (uint16_t)(cum[v] + q[v]);
        for (unsigned x = 0; x < ORC_TANS_L; x++)
            state_of[cum[value_of[x]] + (number_of[x] - q[value_of[x]])] = (uint16_t)x;
    }

    /* size: header, then set by set the whole blocks of the streams (all but the first block of
     * each) and the first blocks cut down to the bytes that hold bits, the set padded to 16 */
    uint32_t W = set_width(S), n_sets = S / W, hdr = header_bytes_codec(S, codec), front = front_bytes(codec);
    uint32_t max_sym = 16 * (((raw_bytes + 15) / 16 + S - 1) / S);
    uint64_t *nb = calloc(S, sizeof(uint64_t));
    uint64_t *hb = calloc(S, sizeof(uint64_t));
    uint32_t *pos_of = calloc(max_sym + 1, sizeof(uint32_t));
    uint16_t *field = calloc(max_sym + 1, sizeof(uint16_t));
    uint8_t *width = calloc(max_sym + 1, 1);
    if (!nb || !hb || !pos_of || !field || !width) {
        free(nb); free(hb); free(pos_of); free(field); free(width);
        return 0;
    }
    uint64_t total = hdr;
    for (uint32_t w = 0; w < n_sets; w++) {
        uint64_t area = 0;
        for (uint32_t j = w * W; j < (w + 1) * W; j++) {
            uint32_t nsym = stream_positions(raw_bytes, S, j, pos_of);
            uint64_t bits = codec == ORC_CODEC_HUFFMAN
                                ? huff_stream(src, pos_of, nsym, len, code, NULL, 0, NULL)
                                : tans_stream(src, pos_of, nsym, q, cum, state_of, field, width, NULL, 0, NULL);
            uint64_t bytes = (bits + 7) / 8;
            nb[j] = (bytes + ORC_BLOCK - 1) / ORC_BLOCK;
            hb[j] = nb[j] ? bytes - ORC_BLOCK * (nb[j] - 1) : 0;
            if (nb[j] > 0xFFFu) /* the header keeps 12 bits for it: chunks up to 1 MiB split 32 ways or more fit */
                total = 0;
            area += nb[j] ? (nb[j] - 1) * ORC_BLOCK + hb[j] : 0;
        }
        if (total)
            total += round_up(area, 16);
    }
    if (!out || total == 0 || cap < total) {
        if (out)
            total = 0;
        free(nb); free(hb); free(pos_of); free(field); free(width);
        return total;
    }
    memset(out, 0, total);
    if (codec == ORC_CODEC_HUFFMAN) {
        for (int v = 0; v < 256; v++)
            out[v >> 1] |= (uint8_t)(len[v] << (4 * (v & 1)));
    } else {
        for (int v = 0; v < 256; v++)
            for (int b = 0; b < 12; b++)
                if ((q[v] >> b) & 1u)
                    out[(12 * v + b) >> 3] |= (uint8_t)(1u << ((12 * v + b) & 7));
    }
    for (uint32_t j = 0; j < S; j++) {
        uint16_t n16 = (uint16_t)(nb[j] | (hb[j] ? (hb[j] - 1) << 12 : 0));
        memcpy(out + front + 2 * (uint64_t)j, &n16, 2); /* little-endian host */
    }

    /* every stream written out on its own from where its block 0 would start; start[j] = its first
     * position, used[j][k] = its position after its first k symbols (tANS: and the first state) */
    uint8_t **st = calloc(S, sizeof(uint8_t *));
    uint64_t **used = calloc(S, sizeof(uint64_t *));
    uint64_t *start = calloc(S, sizeof(uint64_t));
    for (uint32_t j = 0; j < S; j++) {
        uint32_t nsym = stream_positions(raw_bytes, S, j, pos_of);
        st[j] = calloc(nb[j] * ORC_BLOCK + 1, 1);
        used[j] = calloc((size_t)nsym + 1, sizeof(uint64_t));
        start[j] = nb[j] ? 8 * (ORC_BLOCK - hb[j]) : 0; /* block 0 begins with bytes that do not exist */
        if (codec == ORC_CODEC_HUFFMAN)
            huff_stream(src, pos_of, nsym, len, code, st[j], start[j], used[j]);
        else
            tans_stream(src, pos_of, nsym, q, cum, state_of, field, width, st[j], start[j], used[j]);
    }

    /* set areas: the placement rule for the whole blocks, then the heads in stream order */
    uint64_t pos = hdr;
    uint32_t steps = step_count(raw_bytes, S);
    for (uint32_t w = 0; w < n_sets; w++) {
        uint32_t off32 = (uint32_t)pos;
        memcpy(out + front + 2 * (uint64_t)S + 4 * (uint64_t)w, &off32, 4);
        uint64_t *f = calloc(W, sizeof(uint64_t));
        for (uint32_t h = 0; h < steps; h++) {
            int times = h == 0 ? 5 : 1;
            for (int t = 0; t < times; t++) {
                for (uint32_t i = 0; i < W; i++) {
                    uint32_t j = w * W + i;
                    /* the first four times of step 0 come before anything of the stream is read */
                    uint64_t c = (h == 0 && t < 4) ? start[j] : used[j][symbols_before_step(raw_bytes, S, j, h)];
                    if (f[i] < nb[j] && 128 * f[i] < c + ORC_LOOKAHEAD) {
                        if (f[i] > 0) { /* block 0 is not stored here */
                            memcpy(out + pos, st[j] + f[i] * ORC_BLOCK, ORC_BLOCK);
                            pos += ORC_BLOCK;
                        }
                        f[i]++;
                    }
                }
            }
        }
        for (uint32_t i = 0; i < W; i++)
            if (f[i] != nb[w * W + i])
                total = 0; /* cannot happen: every block is placed by the last step */
        free(f);
        for (uint32_t j = w * W; j < (w + 1) * W; j++) {
            if (nb[j] == 0)
                continue;
            memcpy(out + pos, st[j] + (ORC_BLOCK - hb[j]), hb[j]);
            pos += hb[j];
        }
        pos = round_up(pos, 16);
    }
    if (pos != total)
        total = 0;
    for (uint32_t j = 0; j < S; j++) {
        free(st[j]);
        free(used[j]);
    }
    free(st); free(used); free(start); free(nb); free(hb); free(pos_of); free(field); free(width);
    return total;
}

uint64_t orc_encode_chunk(const uint8_t *src, uint32_t raw_bytes, uint32_t S, int max_len,
                          uint8_t *out, uint64_t cap)
{
    return orc_encode_chunk_codec(src, raw_bytes, S, ORC_CODEC_HUFFMAN, max_len, out, cap);
}

/* ------------------------------------------------------------------ chunk decode */

/* One stream bit, or -1 when the stream has no block that holds it yet. */
static int stream_bit(const uint8_t *st, uint64_t *bit, uint64_t blocks_held)
{
    if (*bit >= 8 * ORC_BLOCK * blocks_held)
        return -1;
    int b = (st[*bit >> 3] >> (*bit & 7)) & 1;
    (*bit)++;
    return b;
}

/*
 * Decode one payload bit by bit.  Huffman: grow the code one bit at a time and
 * stop when it falls inside the range of codes of its length.  tANS: walk the
 * states.  Symbol counts come from raw_bytes, never from the stream.  The
 * blocks of a stream are collected from its set's region by the placement rule
 * as decoding goes.
 */
int orc_decode_chunk_codec(const uint8_t *payload, uint64_t comp_bytes, uint32_t raw_bytes, uint32_t S,
                           int codec, uint8_t *dst)
{
    uint8_t len[256];
    unsigned count[16] = {0}, first[16] = {0}, base[16] = {0};
    uint8_t sorted[256];
    uint16_t q[256], number_of[ORC_TANS_L];
    uint8_t value_of[ORC_TANS_L];
    if (codec != ORC_CODEC_HUFFMAN && codec != ORC_CODEC_TANS)
        return ORC_E_ARG;
    uint32_t front = front_bytes(codec);
    if (S == 0 || S % set_width(S) != 0 || comp_bytes < header_bytes_codec(S, codec))
        return ORC_E_FORMAT;
    if (codec == ORC_CODEC_HUFFMAN) {
        for (int v = 0; v < 256; v++) {
            len[v] = (payload[v >> 1] >> (4 * (v & 1))) & 15;
            if (len[v] > 11)
                return ORC_E_FORMAT;
            count[len[v]]++;
        }
        count[0] = 0;
        /* symbols in order of (length, byte value); first code and first rank of each length */
        int k = 0;
        unsigned code = 0;
        for (int l = 1; l <= 11; l++) {
            code <<= 1;
            first[l] = code;
            base[l] = (unsigned)k;
            for (int v = 0; v < 256; v++)
                if (len[v] == l)
                    sorted[k++] = (uint8_t)v;
            code += count[l];
        }
        if (k == 0)
            return ORC_E_FORMAT;
    } else {
        for (int v = 0; v < 256; v++) {
            q[v] = 0;
            for (int b = 0; b < 12; b++)
                q[v] |= (uint16_t)(((payload[(12 * v + b) >> 3] >> ((12 * v + b) & 7)) & 1u) << b);
        }
        if (orc_tans_states(q, value_of, number_of) != ORC_OK)
            return ORC_E_FORMAT;
    }
    uint32_t groups = (raw_bytes + 15) / 16;
    uint32_t W = set_width(S), n_sets = S / W;
    uint32_t steps = step_count(raw_bytes, S);
    int rc = ORC_OK;
    for (uint32_t w = 0; w < n_sets && rc == ORC_OK; w++) {
        uint32_t off32;
        memcpy(&off32, payload + front + 2 * (uint64_t)S + 4 * (uint64_t)w, 4);
        uint64_t pos = off32;
        /* per stream of the set: blocks in all, bytes of the first one, where that one lies; its
         * blocks collected so far, bits used; tANS: its state */
        uint8_t **st = calloc(W, sizeof(uint8_t *));
        uint64_t *f = calloc(W, sizeof(uint64_t));
        uint64_t *bit = calloc(W, sizeof(uint64_t));
        uint64_t *nb = calloc(W, sizeof(uint64_t));
        uint64_t *hb = calloc(W, sizeof(uint64_t));
        uint64_t *head = calloc(W, sizeof(uint64_t));
        unsigned *x = calloc(W, sizeof(unsigned));
        uint64_t head_pos = off32;
        for (uint32_t i = 0; i < W; i++) {
            uint16_t n16;
            memcpy(&n16, payload + front + 2 * (uint64_t)(w * W + i), 2);
            nb[i] = n16 & 0xFFFu;
            hb[i] = nb[i] ? (n16 >> 12) + 1u : 0;
            st[i] = calloc((size_t)nb[i] * ORC_BLOCK + 1, 1);
            head_pos += nb[i] ? (nb[i] - 1) * ORC_BLOCK : 0;
        }
        for (uint32_t i = 0; i < W; i++) { /* the heads follow the whole blocks of the set */
            head[i] = head_pos;
            head_pos += hb[i];
            bit[i] = nb[i] ? 8 * (ORC_BLOCK - hb[i]) : 0;
        }
        if (head_pos > comp_bytes)
            rc = ORC_E_FORMAT;
        for (uint32_t h = 0; h < steps && rc == ORC_OK; h++) {
            int times = h == 0 ? 5 : 1;
            for (int t = 0; t < times && rc == ORC_OK; t++) {
                if (codec == ORC_CODEC_TANS && h == 0 && t == 4) {
                    /* the first state of every stream that has symbols */
                    for (uint32_t i = 0; i < W && rc == ORC_OK; i++) {
                        if (w * W + i >= groups)
                            continue;
                        x[i] = 0;
                        for (int b = 0; b < ORC_TANS_BITS; b++) {
                            int v = stream_bit(st[i], &bit[i], f[i]);
                            if (v < 0) {
                                rc = ORC_E_FORMAT;
                                break;
                            }
                            x[i] |= (unsigned)v << b;
                        }
                    }
                    if (rc != ORC_OK)
                        break;
                }
                for (uint32_t i = 0; i < W; i++) {
                    if (f[i] < nb[i] && 128 * f[i] < bit[i] + ORC_LOOKAHEAD) {
                        if (f[i] > 0) {
                            if (pos + ORC_BLOCK > head[0]) { /* more whole blocks asked for than the area has */
                                rc = ORC_E_FORMAT;
                                break;
                            }
                            memcpy(st[i] + f[i] * ORC_BLOCK, payload + pos, ORC_BLOCK);
                            pos += ORC_BLOCK;
                        } else {
                            memcpy(st[i] + (ORC_BLOCK - hb[i]), payload + head[i], hb[i]);
                        }
                        f[i]++;
                    }
                }
            }
            /* the symbols between step h and step h+1: half of group h/2 of every stream */
            for (uint32_t i = 0; i < W && rc == ORC_OK; i++) {
                uint32_t j = w * W + i;
                uint32_t g = j + (h / 2) * S;
                if (g >= groups)
                    continue;
                uint32_t lo = 16 * g + 8 * (h & 1);
                uint32_t hi = 16 * g + 8 * (h & 1) + 8;
                if (hi > raw_bytes)
                    hi = raw_bytes;
                for (uint32_t p = lo; p < hi && rc == ORC_OK; p++) {
                    if (codec == ORC_CODEC_HUFFMAN) {
                        unsigned code = 0;
                        int l = 0, found = 0;
                        while (l < 11) {
                            int v = stream_bit(st[i], &bit[i], f[i]);
                            if (v < 0) {
                                rc = ORC_E_FORMAT;
                                break;
                            }
                            code = (code << 1) | (unsigned)v;
                            l++;
                            if (code >= first[l] && code - first[l] < count[l]) {
                                dst[p] = sorted[base[l] + (code - first[l])];
                                found = 1;
                                break;
                            }
                        }
                        if (!found)
                            rc = ORC_E_FORMAT;
                    } else {
                        unsigned k = number_of[x[i]];
                        int n = ORC_TANS_BITS - floor_log2(k);
                        unsigned field = 0;
                        dst[p] = value_of[x[i]];
                        for (int b = 0; b < n; b++) {
                            int v = stream_bit(st[i], &bit[i], f[i]);
                            if (v < 0) {
                                rc = ORC_E_FORMAT;
                                break;
                            }
                            field |= (unsigned)v << b;
                        }
                        x[i] = (k << n) - ORC_TANS_L + field;
                    }
                }
            }
        }
        if (codec == ORC_CODEC_TANS && rc == ORC_OK)
            for (uint32_t i = 0; i < W; i++)
                if (w * W + i < groups && x[i] != 0)
                    rc = ORC_E_FORMAT; /* the encoder started from state 0 */
        for (uint32_t i = 0; i < W; i++)
            free(st[i]);
        free(st); free(f); free(bit); free(nb); free(hb); free(head); free(x);
    }
    return rc;
}

int orc_decode_chunk(const uint8_t *payload, uint64_t comp_bytes, uint32_t raw_bytes, uint32_t S,
                     uint8_t *dst)
{
    return orc_decode_chunk_codec(payload, comp_bytes, raw_bytes, S, ORC_CODEC_HUFFMAN, dst);
}

/* ------------------------------------------------------- whole-buffer operations */

static uint32_t chunk_raw_bytes(uint64_t n, uint32_t C, uint64_t k)
{
    uint64_t lo = k * C;
    uint64_t hi = lo + C < n ? lo + C : n;
    return (uint32_t)(hi - lo);
}

uint64_t orc_num_chunks(uint64_t n, uint32_t C) { return (n + C - 1) / C; }

/* Coded payload size of chunks k0 <= k < k1 (no output written). */
int orc_chunk_sizes_codec(const uint8_t *src, uint64_t n, uint32_t C, uint32_t S, int codec, uint64_t k0,
                          uint64_t k1, uint32_t *huff_bytes)
{
    for (uint64_t k = k0; k < k1; k++) {
        uint64_t sz = orc_encode_chunk_codec(src + k * C, chunk_raw_bytes(n, C, k), S, codec, 11, NULL, 0);
        if (sz == 0)
            return ORC_E_ARG;
        huff_bytes[k] = (uint32_t)sz;
    }
    return ORC_OK;
}

int orc_chunk_sizes(const uint8_t *src, uint64_t n, uint32_t C, uint32_t S, uint64_t k0, uint64_t k1,
                    uint32_t *huff_bytes)
{
    return orc_chunk_sizes_codec(src, n, C, S, ORC_CODEC_HUFFMAN, k0, k1, huff_bytes);
}

/*
 * Which chunks stay raw.
 *   ALL_HUFF      none (even when coding enlarges the chunk)
 *   AUTO          those whose gain = raw_bytes - huffman_payload_bytes is <= 0
 *   RAW_FRACTION  the floor(f * n_chunks + 1/2) chunks of lowest gain, lower
 *                 index first among equal gains
 *   RAW_MASK      those with mask[k] != 0
 *   BLOCK_LAST    the paper's rule (Section 3.3, "Speed Adaptive Partial
 *                 Compression"): chunks are grouped in blocks of `block`
 *                 consecutive chunks and only the last chunk of each block is
 *                 compressed; a trailing partial block has no compressed chunk
 */
int orc_select_raw(const uint32_t *huff_bytes, uint64_t n, uint32_t C, uint64_t n_chunks, int policy,
                   double raw_fraction, uint32_t block, const uint8_t *mask, uint8_t *is_raw)
{
    memset(is_raw, 0, n_chunks);
    if (policy == ORC_ALL_HUFF)
        return ORC_OK;
    if (policy == ORC_AUTO) {
        for (uint64_t k = 0; k < n_chunks; k++)
            is_raw[k] = (int64_t)chunk_raw_bytes(n, C, k) - (int64_t)huff_bytes[k] <= 0;
        return ORC_OK;
    }
    if (policy == ORC_RAW_MASK) {
        if (!mask) return ORC_E_ARG;
        for (uint64_t k = 0; k < n_chunks; k++)
            is_raw[k] = mask[k] != 0;
        return ORC_OK;
    }
    if (policy == ORC_BLOCK_LAST) {
        if (block == 0) return ORC_E_ARG;
        for (uint64_t k = 0; k < n_chunks; k++)
            is_raw[k] = (k % block) != (uint64_t)(block - 1);
        return ORC_OK;
    }
    if (policy == ORC_RAW_FRACTION) {
        if (!(raw_fraction >= 0.0 && raw_fraction <= 1.0)) return ORC_E_ARG;
        uint64_t n_raw = (uint64_t)(raw_fraction * (double)n_chunks + 0.5);
        if (n_raw > n_chunks) n_raw = n_chunks;
        /* selection by repeated minimum: slow and plain */
        for (uint64_t r = 0; r < n_raw; r++) {
            int64_t best_gain = 0;
            uint64_t best = n_chunks;
            for (uint64_t k = 0; k < n_chunks; k++) {
                if (is_raw[k]) continue;
                int64_t gain = (int64_t)chunk_raw_bytes(n, C, k) - (int64_t)huff_bytes[k];
                if (best == n_chunks || gain < best_gain) {
                    best = k;
                    best_gain = gain;
                }
            }
            is_raw[best] = 1;
        }
        return ORC_OK;
    }
    return ORC_E_ARG;
}

/* Offsets and sizes of every payload, laid out back to back.  Returns the blob size, which
 * includes the 64 bytes that close the blob (orc_close_blob writes them). */
uint64_t orc_layout(const uint32_t *huff_bytes, const uint8_t *is_raw, uint64_t n, uint32_t C,
                    uint64_t n_chunks, orc_chunk *table)
{
    uint64_t off = 0;
    for (uint64_t k = 0; k < n_chunks; k++) {
        uint32_t raw = chunk_raw_bytes(n, C, k);
        table[k].off = off;
        if (is_raw[k]) {
            table[k].comp_bytes = (uint32_t)round_up(raw, 16);
            table[k].raw_bytes_flags = raw | ORC_RAW_FLAG;
        } else {
            table[k].comp_bytes = huff_bytes[k];
            table[k].raw_bytes_flags = raw;
        }
        off += table[k].comp_bytes;
    }
    return off + ORC_BLOB_TAIL;
}

/*
 * The blob's closing bytes: 48 zero bytes, then the trailer of 16 bytes, little endian:
 *   bytes 0-3  'D' 'C' 'B' 'F'
 *   bytes 4-5  format id (5)            bytes 6-7   look-ahead bits of the placement rule (392)
 *   bytes 8-11 chunk size C
 *   bytes 12-13 sub-streams S           bytes 14-15 coder (0 Huffman, 1 tANS)
 * A reader that finds anything else at the end of a blob must not decode it.
 */
static void put_le(uint8_t *at, uint64_t v, int bytes)
{
    for (int i = 0; i < bytes; i++)
        at[i] = (uint8_t)(v >> (8 * i));
}

static void make_trailer(uint32_t C, uint32_t S, int codec, uint8_t *t)
{
    t[0] = 'D'; t[1] = 'C'; t[2] = 'B'; t[3] = 'F';
    put_le(t + 4, ORC_FORMAT, 2);
    put_le(t + 6, ORC_LOOKAHEAD_IN_TRAILER, 2);
    put_le(t + 8, C, 4);
    put_le(t + 12, S, 2);
    put_le(t + 14, (uint64_t)codec, 2);
}

int orc_close_blob(uint8_t *blob, uint64_t blob_bytes, uint32_t C, uint32_t S, int codec)
{
    if (blob_bytes < ORC_BLOB_TAIL)
        return ORC_E_ARG;
    memset(blob + blob_bytes - ORC_BLOB_TAIL, 0, ORC_BLOB_TAIL);
    make_trailer(C, S, codec, blob + blob_bytes - 16);
    return ORC_OK;
}

int orc_check_trailer(const uint8_t *blob, uint64_t blob_bytes, uint32_t C, uint32_t S, int codec)
{
    uint8_t want[16];
    if (blob_bytes < ORC_BLOB_TAIL)
        return ORC_E_FORMAT;
    make_trailer(C, S, codec, want);
    return memcmp(blob + blob_bytes - 16, want, 16) == 0 ? ORC_OK : ORC_E_FORMAT;
}

/* Write the payloads of chunks k0 <= k < k1 at the offsets the table gives. */
int orc_emit_codec(const uint8_t *src, uint64_t n, uint32_t C, uint32_t S, int codec, const orc_chunk *table,
                   uint64_t k0, uint64_t k1, uint8_t *blob)
{
    for (uint64_t k = k0; k < k1; k++) {
        uint32_t raw = table[k].raw_bytes_flags & ~ORC_RAW_FLAG;
        uint8_t *out = blob + table[k].off;
        if (raw != chunk_raw_bytes(n, C, k))
            return ORC_E_ARG;
        if (table[k].raw_bytes_flags & ORC_RAW_FLAG) {
            memset(out, 0, table[k].comp_bytes);
            memcpy(out, src + k * C, raw);
        } else {
            uint64_t sz = orc_encode_chunk_codec(src + k * C, raw, S, codec, 11, out, table[k].comp_bytes);
            if (sz != table[k].comp_bytes)
                return ORC_E_ARG;
        }
    }
    return ORC_OK;
}

int orc_emit(const uint8_t *src, uint64_t n, uint32_t C, uint32_t S, const orc_chunk *table,
             uint64_t k0, uint64_t k1, uint8_t *blob)
{
    return orc_emit_codec(src, n, C, S, ORC_CODEC_HUFFMAN, table, k0, k1, blob);
}

/* Decode chunks k0 <= k < k1: chunk k lands at dst + k*C. */
int orc_decompress_codec(const uint8_t *blob, uint64_t blob_bytes, const orc_chunk *table, uint64_t k0,
                         uint64_t k1, uint32_t C, uint32_t S, int codec, uint8_t *dst)
{
    if (orc_check_trailer(blob, blob_bytes, C, S, codec) != ORC_OK)
        return ORC_E_FORMAT;
    for (uint64_t k = k0; k < k1; k++) {
        uint32_t raw = table[k].raw_bytes_flags & ~ORC_RAW_FLAG;
        if (raw == 0 || raw > C)
            return ORC_E_FORMAT;
        if (table[k].off + table[k].comp_bytes > blob_bytes)
            return ORC_E_FORMAT;
        const uint8_t *in = blob + table[k].off;
        if (table[k].raw_bytes_flags & ORC_RAW_FLAG) {
            if (table[k].comp_bytes < raw)
                return ORC_E_FORMAT;
            memcpy(dst + k * C, in, raw);
        } else {
            int rc = orc_decode_chunk_codec(in, table[k].comp_bytes, raw, S, codec, dst + k * C);
            if (rc != ORC_OK)
                return rc;
        }
    }
    return ORC_OK;
}

int orc_decompress(const uint8_t *blob, uint64_t blob_bytes, const orc_chunk *table, uint64_t k0,
                   uint64_t k1, uint32_t C, uint32_t S, uint8_t *dst)
{
    return orc_decompress_codec(blob, blob_bytes, table, k0, k1, C, S, ORC_CODEC_HUFFMAN, dst);
}
