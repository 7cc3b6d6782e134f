// Host side of libdc_mi355x: quantisation front end, chunk compressor, format checker.
//
// Paper: Section 3.2 (per-channel scaling Eqs. 1-2, INT8 quantisation Eq. 4, pruning around Eq. 5),
// Section 3.1 / 3.3 (lossless compression in chunks, speed-adaptive choice of raw chunks).
// The stored format is described in include/dc.h.
#include "dc.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <memory>
#include <thread>
#include <vector>

namespace {

std::atomic<int> g_threads{0};

int worker_count(uint64_t items)
{
    int n = g_threads.load();
    if (n <= 0) {
        n = (int)std::thread::hardware_concurrency();
        if (n <= 0) n = 1;
    }
    if ((uint64_t)n > items) n = (int)std::max<uint64_t>(items, 1);
    return n;
}

// Static partition of [0, items) over the worker threads.
template <class F> void parallel_ranges(uint64_t items, F &&fn)
{
    const int n = worker_count(items);
    if (n <= 1) {
        fn(0, items);
        return;
    }
    std::vector<std::thread> pool;
    pool.reserve(n);
    for (int t = 0; t < n; t++) {
        const uint64_t a = items * (uint64_t)t / n, b = items * (uint64_t)(t + 1) / n;
        if (b > a) pool.emplace_back([&fn, a, b] { fn(a, b); });
    }
    for (auto &th : pool) th.join();
}

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

bool params_ok(const dc_params *p)
{
    if (!p) return false;
    if (p->chunk_bytes < 16 || p->chunk_bytes > DC_MAX_CHUNK_BYTES || p->chunk_bytes % 16) return false;
    if (p->n_streams != 32 && p->n_streams != 64 && p->n_streams != 128 && p->n_streams != 256) return false;
    if (p->codec != DC_CODEC_HUFFMAN && p->codec != DC_CODEC_TANS) return false;
    if (p->codec == DC_CODEC_TANS && p->n_streams < 64) return false;
    return true;
}

// The 16 bytes that close a blob: magic number, format id and its look-ahead, and the parameters a reader needs.
void write_trailer(uint8_t *at, const dc_params *p)
{
    const uint32_t words[4] = {DC_TRAILER_MAGIC, DC_FORMAT_ID | (uint32_t)DC_LOOKAHEAD_BITS << 16, p->chunk_bytes,
                               p->n_streams | p->codec << 16};
    std::memcpy(at, words, sizeof(words));
}

bool trailer_matches(const uint8_t *at, const dc_params *p)
{
    uint8_t want[DC_TRAILER_BYTES];
    write_trailer(want, p);
    return std::memcmp(at, want, sizeof(want)) == 0;
}

inline uint32_t chunk_len(uint64_t total, uint32_t C, uint64_t k)
{
    const uint64_t lo = k * C;
    return (uint32_t)std::min<uint64_t>(C, total - lo);
}

// ---------------------------------------------------------------------------------------------
// Code construction
// ---------------------------------------------------------------------------------------------

struct CodeBook {
    uint8_t len[256];
    uint16_t rev[256]; // code with its bits reversed: ready to be OR-ed into an LSB-first accumulator
};

// Length-limited optimal code lengths by package-merge, in the "how many leaves are bought at each
// level" form: every level list is the sorted leaves merged with the pairs of the level below
// (a leaf before a package of equal weight); buying the first m items of a level buys a prefix of
// the leaves, plus packages that each stand for two items of the level below.
void limited_lengths(const uint32_t cnt[256], uint8_t len[256])
{
    constexpr int L = DC_MAX_CODE_LEN;
    int order[256];
    int n = 0;
    for (int v = 0; v < 256; v++)
        if (cnt[v]) order[n++] = v;
    std::memset(len, 0, 256);
    if (n == 0) return;
    if (n == 1) {
        len[order[0]] = 1;
        return;
    }
    std::stable_sort(order, order + n, [&](int a, int b) { return cnt[a] < cnt[b]; });
    uint64_t leafw[256];
    for (int i = 0; i < n; i++) leafw[i] = cnt[order[i]];

    // weight[j][i] and leaves_before[j][i] = number of leaves among the first i items of level j
    static thread_local uint64_t weight[L][512];
    static thread_local uint16_t leaves_before[L][513];
    int size[L];
    for (int i = 0; i < n; i++) {
        weight[0][i] = leafw[i];
        leaves_before[0][i] = (uint16_t)i;
    }
    leaves_before[0][n] = (uint16_t)n;
    size[0] = n;
    for (int j = 1; j < L; j++) {
        const int npk = size[j - 1] / 2;
        int a = 0, b = 0, m = 0;
        while (a < n || b < npk) {
            const uint64_t pw = b < npk ? weight[j - 1][2 * b] + weight[j - 1][2 * b + 1] : 0;
            const bool leaf = b >= npk || (a < n && leafw[a] <= pw);
            leaves_before[j][m] = (uint16_t)a;
            if (leaf) weight[j][m] = leafw[a++];
            else { weight[j][m] = pw; b++; }
            m++;
        }
        leaves_before[j][m] = (uint16_t)a;
        size[j] = m;
    }
    int bought = 2 * n - 2;
    int depth[256] = {0};
    for (int j = L - 1; j >= 0 && bought > 0; j--) {
        const int nl = leaves_before[j][bought];
        for (int i = 0; i < nl; i++) depth[i]++;
        bought = 2 * (bought - nl);
    }
    for (int i = 0; i < n; i++) len[order[i]] = (uint8_t)depth[i];
}

inline uint32_t bit_reverse(uint32_t x, int bits)
{
    uint32_t r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

void make_codebook(const uint32_t cnt[256], CodeBook &cb)
{
    limited_lengths(cnt, cb.len);
    uint32_t per_len[DC_MAX_CODE_LEN + 2] = {0};
    for (int v = 0; v < 256; v++) per_len[cb.len[v]]++;
    per_len[0] = 0;
    uint32_t next[DC_MAX_CODE_LEN + 2];
    uint32_t code = 0;
    for (int l = 1; l <= DC_MAX_CODE_LEN; l++) {
        code = (code + per_len[l - 1]) << 1;
        next[l] = code;
    }
    for (int v = 0; v < 256; v++) {
        const int l = cb.len[v];
        cb.rev[v] = l ? (uint16_t)bit_reverse(next[l]++, l) : 0;
    }
}

void histogram256(const uint8_t *p, uint32_t n, uint32_t out[256])
{
    uint32_t h[4][256];
    std::memset(h, 0, sizeof(h));
    uint32_t i = 0;
    for (; i + 4 <= n; i += 4) {
        h[0][p[i]]++;
        h[1][p[i + 1]]++;
        h[2][p[i + 2]]++;
        h[3][p[i + 3]]++;
    }
    for (; i < n; i++) h[0][p[i]]++;
    for (int v = 0; v < 256; v++) out[v] = h[0][v] + h[1][v] + h[2][v] + h[3][v];
}

constexpr uint32_t kBlock = DC_BLOCK_BYTES;
constexpr uint32_t kBlockBits = 8 * DC_BLOCK_BYTES;

inline uint32_t set_width(uint32_t S) { return S < 64 ? S : 64; }
// bytes of the code description at the start of a payload: 256 code lengths, or 256 frequencies of 12 bits
inline uint32_t front_bytes(uint32_t codec) { return codec == DC_CODEC_TANS ? 384u : 128u; }
inline uint32_t header_bytes(uint32_t S, uint32_t codec = DC_CODEC_HUFFMAN)
{
    return (uint32_t)align_up(front_bytes(codec) + 2ull * S + 4ull * (S / set_width(S)), 16);
}

// ---------------------------------------------------------------------------------------------
// tANS model (the format text in dc.h: frequencies, states, numbers)
// ---------------------------------------------------------------------------------------------

constexpr uint32_t kTansBits = DC_TANS_STATE_BITS;
constexpr uint32_t kTansL = 1u << kTansBits;

struct TansModel {
    uint16_t q[256];
    uint16_t cum[257];
    uint16_t state_of[kTansL]; // state of value v with number q[v] + i at cum[v] + i
    uint8_t value_of[kTansL];
    uint16_t number_of[kTansL];
};

// Frequencies normalised to 2048 by the rule of the format.  The rule settles the difference one state at a
// time, each time at the value with the extreme ratio count/q (or count/(q-1)); only that value's ratio changes,
// so the values sit in a heap ordered by the exact ratio (cross products, the lower value first among equals)
// and one state costs one re-insertion.
void tans_normalise(const uint32_t cnt[256], uint32_t n, uint16_t q[256])
{
    uint32_t sum = 0;
    for (int v = 0; v < 256; v++) {
        const uint64_t f = (uint64_t)cnt[v] * kTansL / n;
        q[v] = cnt[v] == 0 ? 0 : (uint16_t)std::max<uint64_t>(f, 1);
        sum += q[v];
    }
    if (sum == kTansL) return;
    const bool grow = sum < kTansL;
    // "a comes after b" in the order in which values are served
    auto later = [&](int a, int b) {
        const uint64_t da = grow ? q[a] : q[a] - 1u, db = grow ? q[b] : q[b] - 1u;
        const uint64_t lhs = (uint64_t)cnt[a] * db, rhs = (uint64_t)cnt[b] * da; // cnt[a]/da against cnt[b]/db
        if (lhs != rhs) return grow ? lhs < rhs : lhs > rhs;
        return a > b;
    };
    std::vector<int> heap;
    for (int v = 0; v < 256; v++)
        if (grow ? cnt[v] != 0 : q[v] > 1) heap.push_back(v);
    std::make_heap(heap.begin(), heap.end(), later);
    while (sum != kTansL) {
        std::pop_heap(heap.begin(), heap.end(), later);
        const int v = heap.back();
        if (grow) {
            q[v]++;
            sum++;
        } else {
            q[v]--;
            sum--;
        }
        if (grow || q[v] > 1) std::push_heap(heap.begin(), heap.end(), later);
        else heap.pop_back();
    }
}

// States, numbers and the encoder's inverse from frequencies that add up to 2048.
void tans_tables(TansModel &m)
{
    m.cum[0] = 0;
    for (int v = 0; v < 256; v++) m.cum[v + 1] = (uint16_t)(m.cum[v] + m.q[v]);
    for (int v = 0; v < 256; v++)
        for (uint32_t p = m.cum[v]; p < m.cum[v + 1]; p++) m.value_of[bit_reverse(p, kTansBits)] = (uint8_t)v;
    uint16_t next[256];
    for (int v = 0; v < 256; v++) next[v] = m.q[v];
    for (uint32_t x = 0; x < kTansL; x++) {
        const uint8_t v = m.value_of[x];
        m.number_of[x] = next[v];
        m.state_of[m.cum[v] + (next[v] - m.q[v])] = (uint16_t)x;
        next[v]++;
    }
}

// One sub-stream coded backwards: field and width of every symbol (in symbol order), the first state, and the
// stream's bits.  pos lists the positions of the stream's n symbols.
struct TansStream {
    std::vector<uint16_t> field;
    std::vector<uint8_t> width;
    uint32_t first_state = 0;
    uint64_t bits = 0;
};

void tans_code_stream(const uint8_t *src, uint32_t raw, uint32_t S, uint32_t j, const TansModel &m, TansStream &ts)
{
    const uint32_t groups = (raw + 15) / 16;
    uint32_t n = 0;
    for (uint32_t g = j; g < groups; g += S) n += std::min(raw, 16 * g + 16) - 16 * g;
    ts.field.resize(n);
    ts.width.resize(n);
    ts.bits = 0;
    ts.first_state = 0;
    if (n == 0) return;
    uint32_t X = kTansL, k = n;
    const uint32_t last_group = j + (groups - 1 - j) / S * S;
    for (uint32_t g = last_group;; g -= S) {
        const uint32_t lo = 16 * g, hi = std::min(raw, lo + 16);
        for (uint32_t p = hi; p-- > lo;) {
            const uint8_t v = src[p];
            const uint32_t q = m.q[v];
            uint32_t nb = 0;
            while ((X >> nb) >= 2 * q) nb++;
            k--;
            ts.field[k] = (uint16_t)(X & ((1u << nb) - 1u));
            ts.width[k] = (uint8_t)nb;
            ts.bits += nb;
            X = kTansL + m.state_of[m.cum[v] + ((X >> nb) - q)];
        }
        if (g == j) break;
    }
    ts.first_state = X - kTansL;
    ts.bits += kTansBits;
}

// Bits of every sub-stream of a chunk under a codebook.
void stream_bits(const uint8_t *src, uint32_t raw, uint32_t S, const CodeBook &cb, uint64_t *bits)
{
    std::fill(bits, bits + S, 0);
    const uint32_t groups = (raw + 15) / 16;
    uint32_t j = 0;
    for (uint32_t g = 0; g < groups; g++) {
        const uint32_t lo = 16 * g, hi = std::min(raw, lo + 16);
        uint32_t b = 0;
        for (uint32_t p = lo; p < hi; p++) b += cb.len[src[p]];
        bits[j] += b;
        if (++j == S) j = 0;
    }
}

// A sub-stream of `bits` bits is cut into blocks from its end: blocks in all, and bytes of the short first block.
inline uint32_t bytes_of(uint64_t bits) { return (uint32_t)((bits + 7) / 8); }
inline uint32_t blocks_of(uint64_t bits) { return (bytes_of(bits) + kBlock - 1) / kBlock; }
inline uint32_t head_bytes_of(uint64_t bits) { return bits ? bytes_of(bits) - kBlock * (blocks_of(bits) - 1) : 0; }

// Header, then per stream set the whole blocks, the short first blocks and padding to 16.
uint32_t coded_payload_bytes(const uint64_t *bits, uint32_t S, uint32_t codec)
{
    const uint32_t W = set_width(S);
    uint64_t pos = header_bytes(S, codec);
    for (uint32_t s0 = 0; s0 < S; s0 += W) {
        uint64_t area = 0;
        for (uint32_t j = s0; j < s0 + W; j++)
            if (bits[j]) area += (uint64_t)(blocks_of(bits[j]) - 1) * kBlock + head_bytes_of(bits[j]);
        pos += align_up(area, 16);
    }
    return (uint32_t)pos;
}

// Writes one coded payload; `out` has comp_bytes bytes.  Every sub-stream is first coded on its
// own (whole blocks; the first one starts with the bytes that the format leaves out) while its position
// before each step is noted; then, stream set by stream set, the blocks but the first of each stream are
// placed in the order of the placement rule of the format and the short first blocks follow.
// cb is the codebook of a Huffman payload, tm the model of a tANS payload.
void write_payload(const uint8_t *src, uint32_t raw, uint32_t S, const CodeBook *cb, const TansModel *tm,
                   const uint64_t *bits, uint8_t *out, uint32_t comp_bytes)
{
    const uint32_t codec = tm ? DC_CODEC_TANS : DC_CODEC_HUFFMAN;
    const uint32_t front = front_bytes(codec);
    std::memset(out, 0, comp_bytes);
    if (tm) {
        for (int v = 0; v < 256; v += 2) { // two 12-bit frequencies in three bytes
            const uint32_t two = tm->q[v] | (uint32_t)tm->q[v + 1] << 12;
            out[3 * (v / 2)] = (uint8_t)two;
            out[3 * (v / 2) + 1] = (uint8_t)(two >> 8);
            out[3 * (v / 2) + 2] = (uint8_t)(two >> 16);
        }
    } else {
        for (int v = 0; v < 256; v++) out[v >> 1] |= (uint8_t)(cb->len[v] << (4 * (v & 1)));
    }
    const uint32_t groups = (raw + 15) / 16;
    const uint32_t rounds = (groups + S - 1) / S;
    const uint32_t steps = 2 * rounds;
    const uint32_t W = set_width(S);

    std::vector<uint32_t> nb(S), first_block(S + 1, 0), start(S);
    for (uint32_t j = 0; j < S; j++) {
        nb[j] = blocks_of(bits[j]);
        first_block[j + 1] = first_block[j] + nb[j];
        const uint32_t hb = head_bytes_of(bits[j]);
        const uint16_t n16 = (uint16_t)(nb[j] | (hb ? (hb - 1) << 12 : 0));
        std::memcpy(out + front + 2 * j, &n16, 2);
    }
    std::vector<uint8_t> coded((size_t)first_block[S] * kBlock + 8, 0);
    std::vector<uint32_t> used((size_t)S * (steps + 1), 0); // used[j*(steps+1) + h]: bits before step h
    TansStream ts;

    for (uint32_t j = 0; j < S; j++) {
        uint32_t *w = reinterpret_cast<uint32_t *>(coded.data() + (size_t)first_block[j] * kBlock);
        uint32_t *u = &used[(size_t)j * (steps + 1)];
        // positions count from the start of block 0, whose first `pad` bytes do not exist
        const uint32_t pad = nb[j] ? kBlock - head_bytes_of(bits[j]) : 0;
        w += pad / 4;
        uint64_t acc = 0;
        int fill = 8 * (pad % 4);
        uint32_t total = 8 * pad, h = 0, k = 0;
        start[j] = total;
        auto put = [&](uint32_t value, uint32_t n) {
            acc |= (uint64_t)value << fill;
            fill += n;
            total += n;
            if (fill >= 32) {
                *w++ = (uint32_t)acc;
                acc >>= 32;
                fill -= 32;
            }
        };
        if (tm) {
            tans_code_stream(src, raw, S, j, *tm, ts);
            if (!ts.field.empty()) put(ts.first_state, kTansBits);
        }
        for (uint32_t g = j; g < groups; g += S) {
            const uint32_t lo = 16 * g, hi = std::min(raw, lo + 16), mid = std::min(hi, lo + 8);
            u[h++] = total;
            for (uint32_t p = lo; p < hi; p++) {
                if (p == mid) u[h++] = total;
                if (tm) {
                    put(ts.field[k], ts.width[k]);
                    k++;
                } else {
                    put(cb->rev[src[p]], cb->len[src[p]]);
                }
            }
            if (mid == hi) u[h++] = total;
        }
        for (; h <= steps; h++) u[h] = total;
        if (fill > 0) *w++ = (uint32_t)acc;
    }

    // Placement.  The rule of the format is a walk through the steps; here it is turned round.  Call the
    // carrying-outs of the rule "times": T = 0..3 come before anything of a stream is read, T = 4 + h is step h
    // (T = 4 is the fifth time of step 0).  A stream's position c(T) does not fall with T, and a stream takes at
    // most one block a time, so block b of a stream is taken at the first time T_b > T_(b-1) with
    // 128 b < c(T_b) + look-ahead: one pass over the stream's positions gives the times of all its blocks.  The
    // region is then the blocks b >= 1 of the set's streams sorted by (time, stream), a counting sort.
    uint32_t pos = header_bytes(S, codec);
    const uint32_t times = steps + 4;
    std::vector<uint32_t> at_time(times + 1);
    std::vector<uint32_t> when; // time of every block b >= 1 of the set's streams, stream after stream
    std::vector<uint32_t> begin(W + 1);
    for (uint32_t s0 = 0, w = 0; s0 < S; s0 += W, w++) {
        std::memcpy(out + front + 2 * S + 4 * w, &pos, 4);
        when.clear();
        std::fill(at_time.begin(), at_time.end(), 0);
        for (uint32_t i = 0; i < W; i++) {
            const uint32_t j = s0 + i;
            begin[i] = (uint32_t)when.size();
            const uint32_t *u = &used[(size_t)j * (steps + 1)];
            uint32_t T = 0; // block 0, the head, is taken at time 0 (0 < c + look-ahead always holds)
            for (uint32_t b = 1; b < nb[j]; b++) {
                T++;
                while (T < times && (uint64_t)kBlockBits * b >= (uint64_t)(T < 4 ? start[j] : u[T - 4]) + DC_LOOKAHEAD_BITS) T++;
                // (every block is placed by the last step: the format's look-ahead guarantees it)
                if (T >= times) T = times - 1;
                when.push_back(T);
                at_time[T + 1]++;
            }
        }
        begin[W] = (uint32_t)when.size();
        for (uint32_t T = 0; T < times; T++) at_time[T + 1] += at_time[T]; // first region slot of every time
        for (uint32_t i = 0; i < W; i++) {
            const uint32_t j = s0 + i;
            for (uint32_t n = begin[i]; n < begin[i + 1]; n++) {
                const uint32_t b = n - begin[i] + 1;
                const uint32_t slot = at_time[when[n]]++; // streams are visited in ascending order: stable
                std::memcpy(out + pos + (size_t)slot * kBlock, coded.data() + ((size_t)first_block[j] + b) * kBlock, kBlock);
            }
        }
        pos += (uint32_t)when.size() * kBlock;
        for (uint32_t j = s0; j < s0 + W; j++) {
            if (nb[j] == 0) continue;
            const uint32_t n = head_bytes_of(bits[j]);
            std::memcpy(out + pos, coded.data() + (size_t)first_block[j] * kBlock + (kBlock - n), n);
            pos += n;
        }
        pos = (uint32_t)align_up(pos, 16);
    }
}

} // namespace

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------

extern "C" const char *dc_version(void) { return "dc_mi355x 0.6 (gfx950; stored format 5: canonical Huffman L11 or tANS 2048, block-interleaved sub-streams, short first blocks, trailer)"; }

extern "C" int dc_blob_trailer(const uint8_t *trailer_host, dc_params *params_out)
{
    if (!trailer_host || !params_out) return DC_E_ARG;
    uint32_t words[4];
    std::memcpy(words, trailer_host, sizeof(words));
    if (words[0] != DC_TRAILER_MAGIC) return DC_E_FORMAT;
    *params_out = dc_params{};
    params_out->format = words[1] & 0xFFFFu;
    params_out->chunk_bytes = words[2];
    params_out->n_streams = words[3] & 0xFFFFu;
    params_out->codec = words[3] >> 16;
    if (params_out->format != DC_FORMAT_ID || (words[1] >> 16) != DC_LOOKAHEAD_BITS) return DC_E_FORMAT;
    return DC_OK;
}

extern "C" const char *dc_strerror(int code)
{
    switch (code) {
    case DC_OK: return "DC_OK";
    case DC_E_ARG: return "DC_E_ARG: bad argument";
    case DC_E_CAP: return "DC_E_CAP: output buffer too small";
    case DC_E_FORMAT: return "DC_E_FORMAT: blob of another stored format, or table or payload violates the format";
    case DC_E_HIP: return "DC_E_HIP: HIP runtime call failed";
    default: return "unknown dc error code";
    }
}

extern "C" int dc_set_num_threads(int n)
{
    return g_threads.exchange(n < 0 ? 0 : n);
}

extern "C" int dc_quantize_rows(const float *w, uint32_t rows, uint32_t cols, const float *act_absmax,
                                double alpha, uint32_t prune_abs, int8_t *q, float *row_scale,
                                float *col_scale_out)
{
    if (!w || !q || !row_scale || rows == 0 || cols == 0) return DC_E_ARG;
    std::vector<float> s;
    if (act_absmax) {
        s.resize(cols);
        for (uint32_t j = 0; j < cols; j++) s[j] = (float)std::pow((double)act_absmax[j], alpha);
    }
    if (col_scale_out) {
        for (uint32_t j = 0; j < cols; j++) col_scale_out[j] = act_absmax ? s[j] : 1.0f;
    }
    const float *sp = act_absmax ? s.data() : nullptr;
    const int thr = (int)std::min<uint32_t>(prune_abs, 127);
    parallel_ranges(rows, [&](uint64_t r0, uint64_t r1) {
        std::vector<float> tmp(cols);
        for (uint64_t i = r0; i < r1; i++) {
            const float *wr = w + i * cols;
            float m = 0.0f;
            if (sp) {
                for (uint32_t j = 0; j < cols; j++) {
                    const float v = wr[j] * sp[j];
                    tmp[j] = v;
                    m = std::max(m, std::fabs(v));
                }
            } else {
                for (uint32_t j = 0; j < cols; j++) {
                    tmp[j] = wr[j];
                    m = std::max(m, std::fabs(wr[j]));
                }
            }
            const float sc = m == 0.0f ? 1.0f : m / 127.0f;
            row_scale[i] = sc;
            int8_t *qr = q + i * cols;
            for (uint32_t j = 0; j < cols; j++) {
                float r = std::nearbyintf(tmp[j] / sc); // round-half-even in the default mode
                r = std::min(127.0f, std::max(-127.0f, r));
                int v = (int)r;
                if (v <= thr && v >= -thr) v = 0;
                qr[j] = (int8_t)v;
            }
        }
    });
    return DC_OK;
}

extern "C" int dc_quantize_vector(const float *x, uint32_t n, int8_t *xq, float *scale)
{
    if (!x || !xq || !scale || n == 0) return DC_E_ARG;
    float m = 0.0f;
    for (uint32_t j = 0; j < n; j++) m = std::max(m, std::fabs(x[j]));
    const float sc = m == 0.0f ? 1.0f : m / 127.0f;
    for (uint32_t j = 0; j < n; j++) {
        float r = std::nearbyintf(x[j] / sc); // round-half-even in the default mode
        r = std::min(127.0f, std::max(-127.0f, r));
        xq[j] = (int8_t)r;
    }
    *scale = sc;
    return DC_OK;
}

extern "C" int dc_quantize_tensor(const float *w, uint32_t rows, uint32_t cols, const float *act_absmax,
                                  double alpha, double sparsity, int8_t *q, float *tensor_scale,
                                  float *col_scale_out)
{
    if (!w || !q || !tensor_scale || rows == 0 || cols == 0 || !(sparsity >= 0.0 && sparsity < 1.0)) return DC_E_ARG;
    std::vector<float> s(cols, 1.0f);
    if (act_absmax)
        for (uint32_t j = 0; j < cols; j++) s[j] = (float)std::pow((double)act_absmax[j], alpha);
    if (col_scale_out) std::copy(s.begin(), s.end(), col_scale_out);
    const uint64_t n = (uint64_t)rows * cols;

    // pass 1: maximum of the rescaled tensor
    std::vector<float> row_max(rows, 0.0f);
    parallel_ranges(rows, [&](uint64_t r0, uint64_t r1) {
        for (uint64_t i = r0; i < r1; i++) {
            const float *wr = w + i * cols;
            float m = 0.0f;
            for (uint32_t j = 0; j < cols; j++) m = std::max(m, std::fabs(wr[j] * s[j]));
            row_max[i] = m;
        }
    });
    float m = 0.0f;
    for (uint32_t i = 0; i < rows; i++) m = std::max(m, row_max[i]);
    const float sc = m == 0.0f ? 1.0f : m / 127.0f;
    *tensor_scale = sc;

    // pass 2: quantise
    parallel_ranges(rows, [&](uint64_t r0, uint64_t r1) {
        for (uint64_t i = r0; i < r1; i++) {
            const float *wr = w + i * cols;
            int8_t *qr = q + i * cols;
            for (uint32_t j = 0; j < cols; j++) {
                float r = std::nearbyintf((wr[j] * s[j]) / sc);
                r = std::min(127.0f, std::max(-127.0f, r));
                qr[j] = (int8_t)(int)r;
            }
        }
    });

    // pass 3: prune the k lowest importance scores (Eq. 5)
    const uint64_t k = (uint64_t)std::floor(sparsity * (double)n);
    if (k == 0) return DC_OK;
    auto score = [&](uint64_t i, uint32_t j) {
        const double mag = (double)std::abs((int)q[i * cols + j]);
        return act_absmax ? mag * (double)act_absmax[j] : mag;
    };
    std::vector<double> all(n);
    parallel_ranges(rows, [&](uint64_t r0, uint64_t r1) {
        for (uint64_t i = r0; i < r1; i++)
            for (uint32_t j = 0; j < cols; j++) all[i * cols + j] = score(i, j);
    });
    std::nth_element(all.begin(), all.begin() + (k - 1), all.end());
    const double thr = all[k - 1];
    std::vector<double>().swap(all);
    parallel_ranges(rows, [&](uint64_t r0, uint64_t r1) {
        for (uint64_t i = r0; i < r1; i++)
            for (uint32_t j = 0; j < cols; j++)
                if (score(i, j) <= thr) q[i * cols + j] = 0;
    });
    return DC_OK;
}

extern "C" int dc_compress_bound(uint64_t raw_bytes, const dc_params *params, uint64_t *max_blob_bytes,
                                 uint64_t *n_chunks)
{
    if (!params_ok(params) || raw_bytes == 0) return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) return DC_E_FORMAT;
    const uint32_t C = params->chunk_bytes, S = params->n_streams;
    const uint64_t nc = (raw_bytes + C - 1) / C;
    // worst Huffman payload: header, 11 bits a byte, one partial block per stream
    // (tANS: 11 bits a byte too, and 11 bits of state per stream)
    const uint64_t per_chunk =
        align_up(header_bytes(S, params->codec) + ((uint64_t)C * DC_MAX_CODE_LEN + 7) / 8 + (uint64_t)(kBlock + 2) * S, 16);
    if (max_blob_bytes) *max_blob_bytes = nc * per_chunk + DC_BLOB_TAIL_BYTES;
    if (n_chunks) *n_chunks = nc;
    return DC_OK;
}

extern "C" int dc_compress_chunks(const int8_t *src_i8, uint64_t raw_bytes, const dc_params *params,
                                  uint8_t *blob, uint64_t blob_cap, uint64_t *blob_bytes, dc_chunk *table,
                                  uint64_t table_cap, uint64_t *n_chunks_out)
{
    if (!params_ok(params) || !src_i8 || raw_bytes == 0 || !blob_bytes || !n_chunks_out) return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) return DC_E_FORMAT;
    const uint8_t *src = reinterpret_cast<const uint8_t *>(src_i8);
    const uint32_t C = params->chunk_bytes, S = params->n_streams;
    const uint64_t nc = (raw_bytes + C - 1) / C;
    const uint32_t policy = params->policy;
    if (policy > DC_POLICY_BLOCK_LAST) return DC_E_ARG;
    if (policy == DC_POLICY_RAW_MASK && !params->raw_mask) return DC_E_ARG;
    if (policy == DC_POLICY_BLOCK_LAST && params->block_chunks == 0) return DC_E_ARG;
    if (policy == DC_POLICY_RAW_FRACTION && !(params->raw_fraction >= 0.0f && params->raw_fraction <= 1.0f))
        return DC_E_ARG;

    // pass 1: codebook (or frequencies), per-stream bits and coded payload size of every chunk
    const bool tans = params->codec == DC_CODEC_TANS;
    std::vector<CodeBook> books(tans ? 0 : nc);
    std::vector<uint16_t> freqs(tans ? nc * 256 : 0);
    std::vector<uint64_t> bits(nc * S);
    std::vector<uint32_t> huff(nc);
    parallel_ranges(nc, [&](uint64_t k0, uint64_t k1) {
        uint32_t cnt[256];
        std::unique_ptr<TansModel> tm(tans ? new TansModel : nullptr);
        TansStream ts;
        for (uint64_t k = k0; k < k1; k++) {
            const uint32_t raw = chunk_len(raw_bytes, C, k);
            histogram256(src + k * C, raw, cnt);
            if (tans) {
                tans_normalise(cnt, raw, tm->q);
                tans_tables(*tm);
                std::memcpy(&freqs[k * 256], tm->q, sizeof(tm->q));
                for (uint32_t j = 0; j < S; j++) {
                    tans_code_stream(src + k * C, raw, S, j, *tm, ts);
                    bits[k * S + j] = ts.bits;
                }
            } else {
                make_codebook(cnt, books[k]);
                stream_bits(src + k * C, raw, S, books[k], &bits[k * S]);
            }
            huff[k] = coded_payload_bytes(&bits[k * S], S, params->codec);
        }
    });

    // raw selection
    std::vector<uint8_t> is_raw(nc, 0);
    auto gain = [&](uint64_t k) { return (int64_t)chunk_len(raw_bytes, C, k) - (int64_t)huff[k]; };
    switch (policy) {
    case DC_POLICY_ALL_HUFF: break;
    case DC_POLICY_AUTO:
        for (uint64_t k = 0; k < nc; k++) is_raw[k] = gain(k) <= 0;
        break;
    case DC_POLICY_RAW_MASK:
        for (uint64_t k = 0; k < nc; k++) is_raw[k] = params->raw_mask[k] != 0;
        break;
    case DC_POLICY_BLOCK_LAST:
        for (uint64_t k = 0; k < nc; k++) is_raw[k] = (k % params->block_chunks) != params->block_chunks - 1;
        break;
    case DC_POLICY_RAW_FRACTION: {
        uint64_t n_raw = (uint64_t)((double)params->raw_fraction * (double)nc + 0.5);
        n_raw = std::min(n_raw, nc);
        std::vector<uint64_t> idx(nc);
        for (uint64_t k = 0; k < nc; k++) idx[k] = k;
        std::stable_sort(idx.begin(), idx.end(), [&](uint64_t a, uint64_t b) { return gain(a) < gain(b); });
        for (uint64_t r = 0; r < n_raw; r++) is_raw[idx[r]] = 1;
        break;
    }
    }

    // layout
    uint64_t total = 0;
    for (uint64_t k = 0; k < nc; k++)
        total += is_raw[k] ? align_up(chunk_len(raw_bytes, C, k), 16) : huff[k];
    total += DC_BLOB_TAIL_BYTES;
    *blob_bytes = total;
    *n_chunks_out = nc;
    if (!blob || !table || blob_cap < total || table_cap < nc) return DC_E_CAP;
    uint64_t off = 0;
    for (uint64_t k = 0; k < nc; k++) {
        const uint32_t raw = chunk_len(raw_bytes, C, k);
        table[k].off = off;
        table[k].comp_bytes = is_raw[k] ? (uint32_t)align_up(raw, 16) : huff[k];
        table[k].raw_bytes_flags = raw | (is_raw[k] ? DC_CHUNK_RAW : 0u);
        off += table[k].comp_bytes;
    }

    std::memset(blob + off, 0, DC_BLOB_TAIL_BYTES);
    write_trailer(blob + off + DC_BLOB_TAIL_BYTES - DC_TRAILER_BYTES, params);

    // pass 2: emit
    parallel_ranges(nc, [&](uint64_t k0, uint64_t k1) {
        std::unique_ptr<TansModel> tm(tans ? new TansModel : nullptr);
        for (uint64_t k = k0; k < k1; k++) {
            const uint32_t raw = chunk_len(raw_bytes, C, k);
            uint8_t *out = blob + table[k].off;
            if (is_raw[k]) {
                std::memcpy(out, src + k * C, raw);
                std::memset(out + raw, 0, table[k].comp_bytes - raw);
            } else if (tans) {
                std::memcpy(tm->q, &freqs[k * 256], sizeof(tm->q));
                tans_tables(*tm);
                write_payload(src + k * C, raw, S, nullptr, tm.get(), &bits[k * S], out, table[k].comp_bytes);
            } else {
                write_payload(src + k * C, raw, S, &books[k], nullptr, &bits[k * S], out, table[k].comp_bytes);
            }
        }
    });
    return DC_OK;
}

namespace {

// Checks one coded payload completely: header, code completeness (Huffman) or frequencies that add up
// (tANS), region extents, and that each sub-stream decodes its symbol count from the blocks the placement
// rule has given it by then; a tANS stream must also end in state 0.
bool coded_payload_ok(const uint8_t *p, uint32_t comp, uint32_t raw, uint32_t S, uint32_t codec)
{
    const bool tans = codec == DC_CODEC_TANS;
    const uint32_t front = front_bytes(codec);
    const uint32_t hdr = header_bytes(S, codec);
    const uint32_t W = set_width(S), n_sets = S / W;
    if (comp < hdr) return false;

    // Huffman: length of the code that starts with the next 11 stream bits
    std::vector<uint8_t> peek_len;
    std::unique_ptr<TansModel> tm;
    if (tans) {
        tm.reset(new TansModel);
        uint32_t sum = 0;
        for (int v = 0; v < 256; v += 2) {
            const uint32_t two = p[3 * (v / 2)] | (uint32_t)p[3 * (v / 2) + 1] << 8 | (uint32_t)p[3 * (v / 2) + 2] << 16;
            tm->q[v] = (uint16_t)(two & 0xFFFu);
            tm->q[v + 1] = (uint16_t)(two >> 12);
            sum += tm->q[v] + tm->q[v + 1];
            if (sum > kTansL) return false;
        }
        if (sum != kTansL) return false;
        tans_tables(*tm);
    } else {
        uint8_t len[256];
        uint32_t per_len[16] = {0};
        int used = 0;
        for (int v = 0; v < 256; v++) {
            len[v] = (p[v >> 1] >> (4 * (v & 1))) & 15;
            if (len[v] > DC_MAX_CODE_LEN) return false;
            if (len[v]) { per_len[len[v]]++; used++; }
        }
        if (used == 0) return false;
        uint32_t kraft = 0;
        for (int l = 1; l <= DC_MAX_CODE_LEN; l++) kraft += per_len[l] << (DC_MAX_CODE_LEN - l);
        if (used == 1) { if (per_len[1] != 1) return false; }
        else if (kraft != (1u << DC_MAX_CODE_LEN)) return false;
        peek_len.assign(1u << DC_MAX_CODE_LEN, 0);
        uint32_t next[16], code = 0;
        per_len[0] = 0;
        for (int l = 1; l <= DC_MAX_CODE_LEN; l++) { code = (code + per_len[l - 1]) << 1; next[l] = code; }
        for (int v = 0; v < 256; v++) {
            const int l = len[v];
            if (!l) continue;
            const uint32_t r = bit_reverse(next[l]++, l);
            for (uint32_t i = r; i < (1u << DC_MAX_CODE_LEN); i += 1u << l) peek_len[i] = (uint8_t)l;
        }
    }
    for (uint32_t i = front + 2 * S + 4 * n_sets; i < hdr; i++)
        if (p[i]) return false;

    const uint32_t groups = (raw + 15) / 16;
    const uint32_t steps = 2 * ((groups + S - 1) / S);
    uint32_t region = hdr;
    for (uint32_t w = 0; w < n_sets; w++) {
        uint32_t off;
        std::memcpy(&off, p + front + 2 * S + 4 * w, 4);
        if (off != region) return false;
        std::vector<uint32_t> nb(W), hb(W), head_at(W), f(W, 0), state(W, 0);
        std::vector<uint64_t> bit(W, 0), have(W, 0);
        std::vector<std::vector<uint32_t>> where(W); // payload offset of each block taken
        uint64_t whole = 0, head_bytes = 0;
        for (uint32_t i = 0; i < W; i++) {
            uint16_t n16;
            std::memcpy(&n16, p + front + 2 * (w * W + i), 2);
            nb[i] = n16 & 0xFFFu;
            hb[i] = nb[i] ? (n16 >> 12) + 1u : 0;
            if (nb[i] == 0 && n16 != 0) return false;
            whole += nb[i] ? nb[i] - 1 : 0;
            head_bytes += hb[i];
            bit[i] = nb[i] ? 8 * (kBlock - hb[i]) : 0; // the position starts behind the bytes block 0 lacks
        }
        const uint64_t area = align_up(whole * kBlock + head_bytes, 16);
        if (area > comp - region) return false;
        uint32_t pos = region;
        {
            uint32_t at = region + (uint32_t)(whole * kBlock);
            for (uint32_t i = 0; i < W; i++) {
                head_at[i] = at;
                at += hb[i];
            }
            for (; at < region + area; at++)
                if (p[at]) return false; // padding of the area
        }
        const uint32_t heads_begin = region + (uint32_t)(whole * kBlock);
        region += (uint32_t)area;
        // the next n <= 11 bits of stream i (bits the stream does not have yet read as 0; the caller checks)
        auto window = [&](uint32_t i, int n) {
            uint32_t v = 0;
            for (int b = 0; b < n; b++) {
                const uint64_t x = bit[i] + b;
                if (x < have[i]) {
                    const uint32_t byte = where[i][x / kBlockBits] + (uint32_t)(x % kBlockBits) / 8;
                    v |= (uint32_t)((p[byte] >> (x & 7)) & 1u) << b;
                }
            }
            return v;
        };
        for (uint32_t h = 0; h < steps; h++) {
            for (int t = 0; t < (h == 0 ? 5 : 1); t++) {
                if (tans && h == 0 && t == 4) { // the first states are read before the fifth time
                    for (uint32_t i = 0; i < W; i++) {
                        if (w * W + i >= groups) continue;
                        if (bit[i] + kTansBits > have[i]) return false;
                        state[i] = window(i, kTansBits);
                        bit[i] += kTansBits;
                    }
                }
                for (uint32_t i = 0; i < W; i++)
                    if (f[i] < nb[i] && (uint64_t)kBlockBits * f[i] < bit[i] + DC_LOOKAHEAD_BITS) {
                        if (f[i] > 0) {
                            if (pos + kBlock > heads_begin) return false;
                            where[i].push_back(pos);
                            pos += kBlock;
                        } else {
                            where[i].push_back(head_at[i] - (kBlock - hb[i])); // where block 0 would start
                        }
                        have[i] += kBlockBits;
                        f[i]++;
                    }
            }
            for (uint32_t i = 0; i < W; i++) {
                const uint32_t g = w * W + i + (h / 2) * S;
                if (g >= groups) continue;
                const uint32_t lo = 16 * g + 8 * (h & 1);
                const uint32_t hi = std::min(raw, lo + 8);
                for (uint32_t q = lo; q < hi; q++) {
                    if (tans) {
                        const uint32_t k = tm->number_of[state[i]];
                        const int n = (int)kTansBits - (31 - __builtin_clz(k));
                        if (bit[i] + n > have[i]) return false;
                        state[i] = (k << n) - kTansL + window(i, n);
                        bit[i] += n;
                    } else {
                        const int l = peek_len[window(i, DC_MAX_CODE_LEN)];
                        if (l == 0 || bit[i] + l > have[i]) return false;
                        bit[i] += l;
                    }
                }
            }
        }
        for (uint32_t i = 0; i < W; i++)
            if (f[i] != nb[i] || (bit[i] + 7) / 8 != (uint64_t)kBlock * nb[i] || state[i] != 0) return false;
        if (pos != heads_begin) return false;
    }
    return region == comp;
}

} // namespace

extern "C" int dc_validate(const uint8_t *blob, uint64_t blob_bytes, const dc_chunk *table, uint64_t n_chunks,
                           const dc_params *params, uint64_t *bad_chunk)
{
    if (!params_ok(params) || !blob || !table || n_chunks == 0) return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) {
        if (bad_chunk) *bad_chunk = n_chunks;
        return DC_E_FORMAT;
    }
    const uint32_t C = params->chunk_bytes, S = params->n_streams;
    // the blob ends with the trailer of this format and of these parameters
    if (blob_bytes < DC_BLOB_TAIL_BYTES || !trailer_matches(blob + blob_bytes - DC_TRAILER_BYTES, params)) {
        if (bad_chunk) *bad_chunk = n_chunks;
        return DC_E_FORMAT;
    }
    {
        // the blob must extend DC_BLOB_TAIL_BYTES beyond the last payload
        const dc_chunk &last = table[n_chunks - 1];
        if (last.off > blob_bytes || last.comp_bytes > blob_bytes - last.off ||
            blob_bytes - last.off - last.comp_bytes < DC_BLOB_TAIL_BYTES) {
            if (bad_chunk) *bad_chunk = n_chunks - 1;
            return DC_E_FORMAT;
        }
    }
    std::atomic<uint64_t> first_bad{UINT64_MAX};
    parallel_ranges(n_chunks, [&](uint64_t k0, uint64_t k1) {
        for (uint64_t k = k0; k < k1; k++) {
            const dc_chunk &e = table[k];
            const uint32_t raw = e.raw_bytes_flags & ~DC_CHUNK_RAW;
            bool ok = raw >= 1 && raw <= C && (k + 1 == n_chunks || raw == C) && e.off % 16 == 0 &&
                      e.comp_bytes % 16 == 0 && e.off <= blob_bytes && e.comp_bytes <= blob_bytes - e.off;
            // in chunk order, not overlapping; what lies between two payloads (the closing bytes of a blob
            // that another was appended to) is not a payload's business
            if (ok && k > 0) ok = e.off >= table[k - 1].off && e.off - table[k - 1].off >= table[k - 1].comp_bytes;
            if (ok) {
                if (e.raw_bytes_flags & DC_CHUNK_RAW) ok = e.comp_bytes == align_up(raw, 16);
                else ok = coded_payload_ok(blob + e.off, e.comp_bytes, raw, S, params->codec);
            }
            if (!ok) {
                uint64_t cur = first_bad.load();
                while (k < cur && !first_bad.compare_exchange_weak(cur, k)) {}
            }
        }
    });
    if (first_bad.load() != UINT64_MAX) {
        if (bad_chunk) *bad_chunk = first_bad.load();
        return DC_E_FORMAT;
    }
    return DC_OK;
}
