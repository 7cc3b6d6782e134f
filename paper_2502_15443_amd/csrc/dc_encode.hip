// Device side of libdc_mi355x: chunk compression on the GPU (the compression stage of Section 3.1 of
// the paper; Section 4.2 also reports compression speed).  Three launches:
//   dc_codes_kernel   one workgroup per chunk: byte histogram, length-limited code lengths by
//                     package-merge (same ordering rules as the host compressor, so the lengths are
//                     identical), bits of every sub-stream, size of the Huffman payload;
//   dc_layout_kernel  one workgroup: which chunks stay raw, payload offsets (prefix sum), chunk table;
//   dc_emit_kernel    one workgroup per chunk: header, canonical codes, and the sub-streams written as
//                     16-byte blocks in the order of the format's placement rule.
// For the container's second coder (tANS) dc_tans_model_kernel takes the place of dc_codes_kernel: byte
// histogram, frequencies normalised to 2048 by the format's rule, the states of every value, and every
// sub-stream coded backwards once, which leaves one 16-bit item (field and width) per byte in the
// workspace; dc_emit_kernel then writes those items forwards where it would write codes.
// The stored format is in include/dc.h.
#include <hip/hip_runtime.h>

#include <mutex>

#include "dc.h"
#include "dc_device.h"

using namespace dcdev;

namespace {

constexpr int kL = DC_MAX_CODE_LEN;
constexpr uint32_t kBlockBits = 8 * DC_BLOCK_BYTES;

struct EncArgs {
    const uint8_t *src;
    uint64_t raw_bytes;
    uint64_t n_chunks;
    uint32_t chunk_bytes;
    uint32_t S;
    uint32_t policy;
    uint32_t block_chunks;
    uint64_t n_raw; // DC_POLICY_RAW_FRACTION: chunks that stay raw
    uint32_t codec;
    // workspace
    uint8_t *lens;  // [n_chunks][256] code lengths (Huffman)
    uint32_t *bits; // [n_chunks][S] bits of every sub-stream
    uint32_t *comp; // [n_chunks] bytes of the coded payload
    uint16_t *freq;  // tANS: [n_chunks][256] normalised frequencies
    uint16_t *first; // tANS: [n_chunks][S] first state of every sub-stream
    uint16_t *items; // tANS: [n_chunks * chunk_bytes] per byte: field | width << 12
    // results
    uint8_t *blob;
    uint64_t blob_cap;
    dc_chunk *table;
    uint64_t *result; // [0] blob bytes needed, [1] 0 or DC_E_CAP as an unsigned value
};

__device__ __forceinline__ uint32_t set_width(uint32_t S) { return S < 64 ? S : 64; }
// bytes of the code description at the start of a payload: 256 code lengths, or 256 frequencies of 12 bits
__device__ __forceinline__ uint32_t front_bytes(uint32_t codec) { return codec == DC_CODEC_TANS ? 384u : 128u; }
__device__ __forceinline__ uint32_t header_bytes(uint32_t S, uint32_t codec = DC_CODEC_HUFFMAN)
{
    return (front_bytes(codec) + 2 * S + 4 * (S / set_width(S)) + 15) / 16 * 16;
}
// A sub-stream of `bits` bits is cut into blocks from its end: bytes, 16-byte blocks, and bytes of the short first block.
__device__ __forceinline__ uint32_t bytes_of(uint32_t bits) { return (bits + 7) / 8; }
__device__ __forceinline__ uint32_t blocks_of(uint32_t bits) { return (bytes_of(bits) + DC_BLOCK_BYTES - 1) / DC_BLOCK_BYTES; }
__device__ __forceinline__ uint32_t head_bytes_of(uint32_t bits) { return bits ? bytes_of(bits) - DC_BLOCK_BYTES * (blocks_of(bits) - 1) : 0; }
__device__ __forceinline__ uint32_t chunk_len(const EncArgs &a, uint64_t k)
{
    const uint64_t lo = k * a.chunk_bytes;
    const uint64_t left = a.raw_bytes - lo;
    return left < a.chunk_bytes ? (uint32_t)left : a.chunk_bytes;
}

// Byte histogram of a chunk by 256 threads.  arena: 4096 words of LDS.  Column c = t mod 32 holds, for every
// pair of byte values (2p, 2p+1), two 16-bit counts in the word arena[32 p + c] (one column per LDS bank, so the
// lanes of one update never meet in a bank); a column sees at most raw / 32 <= 32768 bytes, so the low count
// never carries.  Ends with hist[v] valid for all threads.
__device__ __forceinline__ void chunk_histogram(const uint8_t *src, uint32_t raw, uint32_t *arena, uint32_t *hist)
{
    const uint32_t t = threadIdx.x;
    for (uint32_t i = t; i < 4096; i += 256) arena[i] = 0;
    __syncthreads();
    uint32_t *column = arena + (t & 31u);
    auto count = [&](uint32_t b) { atomicAdd(column + ((b >> 1) << 5), 1u << ((b & 1u) << 4)); };
    const uint32_t n16 = raw / 16;
    for (uint32_t i = t; i < n16; i += 256) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(src + 16 * (size_t)i);
#pragma unroll
        for (int w = 0; w < 4; w++)
#pragma unroll
            for (int b = 0; b < 4; b++) count((v[w] >> (8 * b)) & 0xFFu);
    }
    for (uint32_t i = n16 * 16 + t; i < raw; i += 256) count(src[i]);
    __syncthreads();
    {
        // byte value t: its row is 32 words; start at column t so that the threads of a wave spread over the banks
        uint32_t sum = 0;
        for (uint32_t i = 0; i < 32; i++) sum += (arena[((t >> 1) << 5) + ((t + i) & 31u)] >> ((t & 1u) << 4)) & 0xFFFFu;
        hist[t] = sum;
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void dc_codes_kernel(EncArgs a)
{
    // 16 KiB used twice: first the histogram columns, then the tables of the package-merge.
    __shared__ uint32_t arena[4112];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t key[256];    // count << 8 | byte value, ascending after the sort; absent values last
    __shared__ uint32_t bought_leaves[kL];
    __shared__ uint8_t len_of[256];
    __shared__ uint32_t sbits[256];
    __shared__ uint32_t area_bytes[4]; // per stream set: whole blocks and short first blocks
    uint32_t(*level)[512] = reinterpret_cast<uint32_t(*)[512]>(arena);              // weights of the items of the previous / current level
    uint32_t *pack = arena + 1024;                                                    // [256] packages made of the previous level
    uint16_t(*leaves_before)[514] = reinterpret_cast<uint16_t(*)[514]>(arena + 1280); // [kL][514]

    const uint32_t t = threadIdx.x;
    const uint64_t k = blockIdx.x;
    const uint32_t raw = chunk_len(a, k);
    const uint8_t *src = a.src + k * a.chunk_bytes;

    sbits[t] = 0;
    len_of[t] = 0;
    if (t < 4) area_bytes[t] = 0;
    chunk_histogram(src, raw, arena, hist);

    const uint32_t cnt = hist[t];
    key[t] = cnt ? (cnt << 8 | t) : 0xFFFFFFFFu;
    const uint32_t n = (uint32_t)__syncthreads_count(cnt != 0);
    // bitonic sort, ascending: leaves in order of (count, byte value)
    for (uint32_t size = 2; size <= 256; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            const uint32_t partner = t ^ stride;
            if (partner > t) {
                const bool up = (t & size) == 0;
                const uint32_t x = key[t], y = key[partner];
                if ((x > y) == up) {
                    key[t] = y;
                    key[partner] = x;
                }
            }
        }
    }
    __syncthreads();

    if (n == 1) {
        if (t == 0) len_of[key[0] & 0xFFu] = 1;
    } else if (n >= 2) {
        // Package-merge: level 0 is the sorted leaves; level j is the leaves merged with the pairs of
        // level j-1, a leaf before a package of equal weight.  leaves_before[j][m] = leaves among the
        // first m items of level j.
        const uint32_t lw = t < n ? key[t] >> 8 : 0;
        if (t < n) level[0][t] = lw;
        for (uint32_t m = t; m < 514; m += 256) leaves_before[0][m] = (uint16_t)(m < n ? m : n);
        uint32_t size_prev = n, cur = 0;
        for (int j = 1; j < kL; j++) {
            __syncthreads();
            const uint32_t npk = size_prev / 2;
            if (t < npk) pack[t] = level[cur][2 * t] + level[cur][2 * t + 1];
            __syncthreads();
            // A leaf goes after the packages lighter than it, a package after the leaves not heavier
            // than it.  Both counts come from one 9-step search over an ascending array of at most 256
            // entries, the two searches side by side so that their LDS reads overlap.
            const uint32_t pw = t < npk ? pack[t] : 0;
            uint32_t packs_below = 0, leaves_upto = 0;
#pragma unroll
            for (uint32_t step = 256; step > 0; step >>= 1) {
                const uint32_t ip = packs_below + step - 1, il = leaves_upto + step - 1;
                const uint32_t yp = pack[ip < npk ? ip : 0], yl = key[il < n ? il : 0] >> 8;
                if (ip < npk && yp < lw) packs_below += step;
                if (il < n && yl <= pw) leaves_upto += step;
            }
            if (t < n) {
                level[cur ^ 1][t + packs_below] = lw;
                leaves_before[j][t + packs_below] = (uint16_t)t;
            }
            if (t < npk) {
                level[cur ^ 1][t + leaves_upto] = pw;
                leaves_before[j][t + leaves_upto] = (uint16_t)leaves_upto;
            }
            if (t == 0) leaves_before[j][n + npk] = (uint16_t)n;
            size_prev = n + npk;
            cur ^= 1;
        }
        __syncthreads();
        if (t == 0) {
            uint32_t bought = 2 * n - 2;
            for (int j = kL - 1; j >= 0; j--) {
                uint32_t nl = 0;
                if (bought > 0) {
                    nl = leaves_before[j][bought];
                    bought = 2 * (bought - nl);
                }
                bought_leaves[j] = nl;
            }
        }
        __syncthreads();
        if (t < n) {
            uint32_t depth = 0;
#pragma unroll
            for (int j = 0; j < kL; j++) depth += t < bought_leaves[j];
            len_of[key[t] & 0xFFu] = (uint8_t)depth;
        }
    }
    __syncthreads();
    a.lens[k * 256 + t] = len_of[t];

    // bits of every sub-stream: thread t sees the 16-byte groups t, t + 256, ... which all belong to
    // sub-stream t mod S (S divides 256)
    const uint32_t groups = (raw + 15) / 16;
    uint32_t mine = 0;
    for (uint32_t g = t; g < groups; g += 256) {
        const uint32_t lo = 16 * g, hi = lo + 16 < raw ? lo + 16 : raw;
        if (hi - lo == 16) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(src + lo);
#pragma unroll
            for (int w = 0; w < 4; w++)
#pragma unroll
                for (int b = 0; b < 4; b++) mine += len_of[(v[w] >> (8 * b)) & 0xFFu];
        } else {
            for (uint32_t p = lo; p < hi; p++) mine += len_of[src[p]];
        }
    }
    if (mine) atomicAdd(&sbits[t % a.S], mine);
    __syncthreads();
    if (t < a.S) {
        a.bits[k * a.S + t] = sbits[t];
        if (sbits[t]) atomicAdd(&area_bytes[t / set_width(a.S)], DC_BLOCK_BYTES * (blocks_of(sbits[t]) - 1) + head_bytes_of(sbits[t]));
    }
    __syncthreads();
    if (t == 0) {
        uint32_t size = header_bytes(a.S);
        for (uint32_t w = 0; w < a.S / set_width(a.S); w++) size += (area_bytes[w] + 15u) & ~15u;
        a.comp[k] = size;
    }
}


// ---------------------------------------------------------------------------------------------
// tANS: frequencies, states, and every sub-stream coded backwards once
// ---------------------------------------------------------------------------------------------

constexpr uint32_t kTansBits = DC_TANS_STATE_BITS;
constexpr uint32_t kTansL = 1u << kTansBits;

// A candidate of the normalisation rule: value v with count c and the divisor d its ratio c/d is taken with
// (d = 0: no candidate).
struct Cand {
    uint32_t c, d, v;
};
// larger ratio first, the lower value among equal ratios (c * d fits 32 bits: c <= 2^20, d <= 2^11)
__device__ __forceinline__ bool larger(const Cand &x, const Cand &y)
{
    if (x.d == 0 || y.d == 0) return x.d != 0 && y.d == 0;
    const uint32_t l = x.c * y.d, r = y.c * x.d;
    return l > r || (l == r && x.v < y.v);
}
__device__ __forceinline__ bool smaller(const Cand &x, const Cand &y)
{
    if (x.d == 0 || y.d == 0) return x.d != 0 && y.d == 0;
    const uint32_t l = x.c * y.d, r = y.c * x.d;
    return l < r || (l == r && x.v < y.v);
}
template <bool LARGEST> __device__ __forceinline__ Cand wave_best(Cand best)
{
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        Cand o;
        o.c = (uint32_t)__shfl_xor((int)best.c, m);
        o.d = (uint32_t)__shfl_xor((int)best.d, m);
        o.v = (uint32_t)__shfl_xor((int)best.v, m);
        if (LARGEST ? larger(o, best) : smaller(o, best)) best = o;
    }
    return best;
}

__global__ __launch_bounds__(256) void dc_tans_model_kernel(EncArgs a)
{
    __shared__ uint32_t arena[4096];   // histogram columns; then marks (u16[2048]) and state_of (u16[2048])
    __shared__ uint32_t hist[256];
    __shared__ uint32_t nq[256];       // normalised frequencies
    __shared__ uint32_t cumq[256];     // first place | frequency << 16
    __shared__ uint32_t wave_sum[4];
    __shared__ uint32_t sbits[256];
    __shared__ uint32_t area_bytes[4];
    uint16_t *marks = reinterpret_cast<uint16_t *>(arena);
    uint16_t *state_of = reinterpret_cast<uint16_t *>(arena + 1024); // state of value v numbered q + i at cum[v] + i

    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint64_t k = blockIdx.x;
    const uint32_t raw = chunk_len(a, k);
    const uint8_t *src = a.src + k * a.chunk_bytes;
    const uint32_t S = a.S;

    sbits[t] = 0;
    if (t < 4) area_bytes[t] = 0;
    chunk_histogram(src, raw, arena, hist);

    // ---- frequencies: floor shares, at least one state for a present value, then the difference to 2048
    // settled one state at a time (largest count / frequency gains one; smallest count / (frequency - 1)
    // among frequencies above one loses one; the lower value among equals)
    {
        const uint32_t cnt = hist[t];
        const uint32_t share = (uint32_t)(((uint64_t)cnt << kTansBits) / raw);
        const uint32_t q0 = cnt ? (share ? share : 1u) : 0u;
        nq[t] = q0;
        const uint32_t incl = lanes_prefix_sum<false>(q0);
        if (lane == 63) wave_sum[wave] = incl;
    }
    __syncthreads();
    if (wave == 0) {
        int32_t diff = (int32_t)kTansL - (int32_t)(wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3]);
        uint32_t c[4], q[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            c[i] = hist[lane + 64 * i];
            q[i] = nq[lane + 64 * i];
        }
        for (; diff > 0; diff--) {
            Cand best = {0, 0, 0};
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const Cand x = {c[i], c[i] ? q[i] : 0u, lane + 64u * i};
                if (larger(x, best)) best = x;
            }
            best = wave_best<true>(best);
#pragma unroll
            for (int i = 0; i < 4; i++)
                if (best.v == lane + 64u * i) q[i]++;
        }
        for (; diff < 0; diff++) {
            Cand best = {0, 0, 0};
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const Cand x = {c[i], q[i] >= 2 ? q[i] - 1 : 0u, lane + 64u * i};
                if (smaller(x, best)) best = x;
            }
            best = wave_best<false>(best);
#pragma unroll
            for (int i = 0; i < 4; i++)
                if (best.v == lane + 64u * i) q[i]--;
        }
#pragma unroll
        for (int i = 0; i < 4; i++) nq[lane + 64 * i] = q[i];
    }
    for (uint32_t i = t; i < 1024; i += 256) arena[i] = 0; // the marks
    __syncthreads();

    // ---- places: value v owns places cum[v] .. cum[v] + q[v] - 1 of the 2048
    const uint32_t qv = nq[t];
    {
        const uint32_t incl = lanes_prefix_sum<false>(qv);
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        uint32_t cum = incl - qv;
        for (uint32_t w = 0; w < wave; w++) cum += wave_sum[w];
        cumq[t] = cum | qv << 16;
        a.freq[k * 256 + t] = (uint16_t)qv;
        if (qv) {
            marks[cum] = (uint16_t)(t + 1);
            // also at the first place of every later wave of the pass below that the value reaches into
            for (uint32_t p = (cum / 512 + 1) * 512; p < cum + qv; p += 512) marks[p] = (uint16_t)(t + 1);
        }
    }
    __syncthreads();
    // ---- states: place p is state rev11(p); the states of a value in ascending order are numbered q, q + 1, ...
    // Thread t takes places 8t .. 8t + 7; the number of place p among the places a .. a + q - 1 of its value is q
    // plus, for every set bit i of p, the places of the value that agree with p below bit i and have bit i
    // clear: (q + M - 1 - ((p - a - 2^i) mod M)) div M with M = 2^(i+1).
    {
        const uint4 m4 = *reinterpret_cast<const uint4 *>(marks + 8 * t);
        const uint32_t w16[4] = {m4.x, m4.y, m4.z, m4.w};
        uint32_t tail = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint32_t lo = w16[i] & 0xFFFFu, hi = w16[i] >> 16;
            tail = lo ? lo : tail;
            tail = hi ? hi : tail;
        }
        uint32_t cur = lanes_last_nonzero_below<false>(tail);
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const uint32_t m = (i & 1) ? w16[i / 2] >> 16 : w16[i / 2] & 0xFFFFu;
            cur = m ? m : cur;
            const uint32_t cq = cumq[(cur - 1) & 255u];
            const uint32_t first = cq & 0xFFFFu, q = cq >> 16;
            const uint32_t p = 8 * t + i, off = p - first;
            uint32_t rank = 0;
#pragma unroll
            for (uint32_t b = 0; b < kTansBits; b++) {
                const uint32_t M = 2u << b;
                const uint32_t n = (q + M - 1 - ((off - (1u << b)) & (M - 1))) >> (b + 1);
                rank += ((p >> b) & 1u) ? n : 0u;
            }
            state_of[(first + rank) & (kTansL - 1)] = (uint16_t)(__brev(p) >> (32 - kTansBits));
        }
    }
    __syncthreads();

    // ---- every sub-stream coded from its last symbol to its first: X = 2048; per symbol the smallest n with
    // (X >> n) < 2q, the field X mod 2^n, then X = 2048 + the state of the value numbered X >> n.  The items
    // (field | n << 12) land in the workspace at the positions of their bytes.
    const uint32_t groups = (raw + 15) / 16;
    if (t < S) {
        const uint32_t my_groups = t < groups ? (groups - t + S - 1) / S : 0;
        uint32_t X = kTansL, bits = 0;
        for (uint32_t r = my_groups; r-- > 0;) {
            const uint32_t lo = 16 * (t + r * S);
            const uint32_t n = raw - lo < 16 ? raw - lo : 16;
            uint32_t w[4] = {0, 0, 0, 0};
            if (n == 16) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(src + lo);
                w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
            } else {
                for (uint32_t i = 0; i < n; i++) w[i >> 2] |= (uint32_t)src[lo + i] << (8 * (i & 3u));
            }
            uint32_t it[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int i = 15; i >= 0; i--) {
                if ((uint32_t)i < n) {
                    const uint32_t v = (w[i >> 2] >> (8 * (i & 3))) & 0xFFu;
                    const uint32_t cq = cumq[v];
                    const uint32_t first = cq & 0xFFFFu, q = cq >> 16;
                    uint32_t nb = (uint32_t)__builtin_clz(2 * q - 1) - (31 - kTansBits); // 12 - bit length of 2q - 1
                    nb += (X >> nb) >= 2 * q;
                    it[i >> 1] |= ((nb << 12) | (X & ((1u << nb) - 1u))) << (16 * (i & 1));
                    X = kTansL + state_of[(first + (X >> nb) - q) & (kTansL - 1)];
                    bits += nb;
                }
            }
            uint16_t *dst = a.items + (k * a.chunk_bytes + lo);
            if (n == 16) {
                const u32x4 v0 = {it[0], it[1], it[2], it[3]}, v1 = {it[4], it[5], it[6], it[7]};
                reinterpret_cast<u32x4 *>(dst)[0] = v0;
                reinterpret_cast<u32x4 *>(dst)[1] = v1;
            } else {
                for (uint32_t i = 0; i < n; i++) dst[i] = (uint16_t)(it[i >> 1] >> (16 * (i & 1u)));
            }
        }
        if (my_groups) bits += kTansBits;
        a.first[k * S + t] = (uint16_t)(X - kTansL);
        a.bits[k * S + t] = bits;
        if (bits) atomicAdd(&area_bytes[t / set_width(S)], DC_BLOCK_BYTES * (blocks_of(bits) - 1) + head_bytes_of(bits));
    }
    __syncthreads();
    if (t == 0) {
        uint32_t size = header_bytes(S, DC_CODEC_TANS);
        for (uint32_t w = 0; w < S / set_width(S); w++) size += (area_bytes[w] + 15u) & ~15u;
        a.comp[k] = size;
    }
}

// Gain of Huffman coding a chunk (raw size less Huffman payload size) as an unsigned key in the same order.
__device__ __forceinline__ uint32_t gain_key(const EncArgs &a, uint64_t k)
{
    return (uint32_t)((int64_t)chunk_len(a, k) - (int64_t)a.comp[k] + (int64_t)0x80000000ll);
}

// Which chunks stay raw.  DC_POLICY_RAW_FRACTION: the n_raw chunks of lowest gain, lower index first
// among equal gains, i.e. the chunks with key < threshold and the first `equal_raw` chunks with
// key == threshold.
struct RawRule {
    uint32_t threshold;
    uint32_t equal_raw;
};

__device__ __forceinline__ bool stays_raw(const EncArgs &a, const RawRule &r, uint64_t k, uint32_t &equal_seen)
{
    if (a.policy == DC_POLICY_AUTO) return gain_key(a, k) <= 0x80000000u;
    if (a.policy == DC_POLICY_BLOCK_LAST) return (k % a.block_chunks) != a.block_chunks - 1;
    if (a.policy == DC_POLICY_RAW_FRACTION) {
        const uint32_t key = gain_key(a, k);
        if (key != r.threshold) return key < r.threshold;
        return equal_seen++ < r.equal_raw;
    }
    return false;
}

// One workgroup; thread t looks after the chunks [t * per, (t + 1) * per).
__global__ __launch_bounds__(256) void dc_layout_kernel(EncArgs a)
{
    __shared__ uint64_t part[256];
    __shared__ uint32_t digit_count[256];
    __shared__ uint32_t equal_part[256];
    __shared__ uint32_t sel_prefix, sel_rank;
    const uint32_t t = threadIdx.x;
    const uint64_t per = (a.n_chunks + 255) / 256;
    const uint64_t k0 = t * per < a.n_chunks ? t * per : a.n_chunks, k1 = k0 + per < a.n_chunks ? k0 + per : a.n_chunks;

    RawRule rule = {0, 0};
    uint32_t equal_before = 0; // chunks before k0 whose key is the threshold
    if (a.policy == DC_POLICY_RAW_FRACTION && a.n_raw > 0) {
        // Radix select, most significant byte first: the key of rank n_raw - 1 in ascending order.
        if (t == 0) {
            sel_prefix = 0;
            sel_rank = (uint32_t)(a.n_raw - 1);
        }
        for (int shift = 24; shift >= 0; shift -= 8) {
            digit_count[t] = 0;
            __syncthreads();
            const uint32_t prefix = sel_prefix;
            for (uint64_t k = k0; k < k1; k++) {
                const uint32_t key = gain_key(a, k);
                if (shift == 24 || ((key ^ prefix) >> (shift + 8)) == 0) atomicAdd(&digit_count[(key >> shift) & 0xFFu], 1u);
            }
            __syncthreads();
            if (t == 0) {
                uint32_t rank = sel_rank, d = 0;
                while (d < 255 && rank >= digit_count[d]) rank -= digit_count[d++]; // the rank lies among the counted keys
                sel_prefix = prefix | (d << shift);
                sel_rank = rank;
            }
            __syncthreads();
        }
        rule.threshold = sel_prefix;
        rule.equal_raw = sel_rank + 1;
        uint32_t mine = 0;
        for (uint64_t k = k0; k < k1; k++) mine += gain_key(a, k) == rule.threshold;
        equal_part[t] = mine;
        __syncthreads();
        for (uint32_t i = 0; i < t; i++) equal_before += equal_part[i];
    }

    uint64_t sum = 0;
    uint32_t equal_seen = equal_before;
    for (uint64_t k = k0; k < k1; k++) {
        const uint32_t raw = chunk_len(a, k);
        sum += stays_raw(a, rule, k, equal_seen) ? (raw + 15u) & ~15u : a.comp[k];
    }
    part[t] = sum;
    __syncthreads();
    if (t == 0) {
        uint64_t run = 0;
        for (int i = 0; i < 256; i++) {
            const uint64_t s = part[i];
            part[i] = run;
            run += s;
        }
        a.result[0] = run + DC_BLOB_TAIL_BYTES;
        a.result[1] = run + DC_BLOB_TAIL_BYTES > a.blob_cap ? (uint64_t)(int64_t)DC_E_CAP : 0;
        if (run + DC_BLOB_TAIL_BYTES <= a.blob_cap) {
            // the closing bytes: zeros, then the trailer (magic number, format id and look-ahead, chunk size,
            // sub-streams and coder); the blob is 16-byte aligned and so is `run`
            uint32_t *closing = reinterpret_cast<uint32_t *>(a.blob + run);
            for (int i = 0; i < (DC_BLOB_TAIL_BYTES - DC_TRAILER_BYTES) / 4; i++) closing[i] = 0;
            uint32_t *trailer = closing + (DC_BLOB_TAIL_BYTES - DC_TRAILER_BYTES) / 4;
            trailer[0] = DC_TRAILER_MAGIC;
            trailer[1] = DC_FORMAT_ID | (uint32_t)DC_LOOKAHEAD_BITS << 16;
            trailer[2] = a.chunk_bytes;
            trailer[3] = a.S | a.codec << 16;
        }
    }
    __syncthreads();
    uint64_t off = part[t];
    equal_seen = equal_before;
    for (uint64_t k = k0; k < k1; k++) {
        const uint32_t raw = chunk_len(a, k);
        const bool is_raw = stays_raw(a, rule, k, equal_seen);
        const uint32_t size = is_raw ? (raw + 15u) & ~15u : a.comp[k];
        dc_chunk e;
        e.off = off;
        e.comp_bytes = size;
        e.raw_bytes_flags = raw | (is_raw ? DC_CHUNK_RAW : 0u);
        a.table[k] = e;
        off += size;
    }
}

// One sub-stream while it is written: the coder runs ahead of the position a decoder would have at
// the current step, only as far as the next block it must hand over.
struct Coder {
    uint64_t acc;       // bits not yet in the ring
    uint32_t nbits;     // valid bits in acc
    uint32_t words;     // words put into the ring so far
    uint32_t next_half; // next half group to code
    uint64_t bytes;     // its bytes, loaded ahead of use
    u32x4 items;        // tANS: their items (field | width << 12, 16 bits each) instead
    uint32_t n;         // how many of them exist
};

template <int THREADS, int CODEC> __global__ __launch_bounds__(THREADS) void dc_emit_kernel(EncArgs a)
{
    constexpr int WAVES = THREADS / 64;
    constexpr bool TANS = CODEC == DC_CODEC_TANS;
    constexpr uint32_t kFront = TANS ? 384 : 128; // code description at the start of a payload
    __shared__ __attribute__((aligned(4096))) uint32_t ring[WAVES * 16 * 64]; // 16 words a lane, as in the decoder
    __shared__ uint32_t book[256];                                            // bit-reversed code | length << 16
    __shared__ uint8_t len_of[256];
    __shared__ uint32_t set_bytes[WAVES];
    __shared__ uint32_t len_count[4][kL + 1]; // [64 byte values][code length]

    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint64_t k = blockIdx.x;
    const uint32_t S = a.S;
    const dc_chunk ent = a.table[k];
    const uint32_t raw = ent.raw_bytes_flags & ~DC_CHUNK_RAW;
    if (ent.off + ent.comp_bytes + DC_BLOB_TAIL_BYTES > a.blob_cap) return; // the caller's blob is too small
    const uint8_t *src = a.src + k * a.chunk_bytes;
    uint8_t *out = a.blob + ent.off;

    if (ent.raw_bytes_flags & DC_CHUNK_RAW) {
        const uint32_t n16 = raw / 16;
        for (uint32_t i = t; i < n16; i += THREADS)
            *reinterpret_cast<u32x4 *>(out + 16 * (size_t)i) = *reinterpret_cast<const u32x4 *>(src + 16 * (size_t)i);
        if (t < 16 && n16 * 16 < raw) out[n16 * 16 + t] = n16 * 16 + t < raw ? src[n16 * 16 + t] : 0;
        return;
    }

    // ---- header: code lengths (tANS: frequencies, two of 12 bits in three bytes), blocks of every sub-stream,
    // region offsets
    if (TANS) {
        for (uint32_t i = t; i < 128; i += THREADS) {
            const uint32_t two = a.freq[k * 256 + 2 * i] | (uint32_t)a.freq[k * 256 + 2 * i + 1] << 12;
            out[3 * i] = (uint8_t)two;
            out[3 * i + 1] = (uint8_t)(two >> 8);
            out[3 * i + 2] = (uint8_t)(two >> 16);
        }
    } else {
        for (uint32_t v = t; v < 256; v += THREADS) len_of[v] = a.lens[k * 256 + v];
        __syncthreads();
        for (uint32_t i = t; i < 128; i += THREADS) out[i] = (uint8_t)(len_of[2 * i] | (len_of[2 * i + 1] << 4));
    }
    const bool has_stream = t < S;
    const uint32_t stream_bits = has_stream ? a.bits[k * S + t] : 0;
    const uint32_t nb = blocks_of(stream_bits), hb = head_bytes_of(stream_bits);
    const uint32_t pad = nb ? DC_BLOCK_BYTES - hb : 0; // bytes that block 0 of the stream lacks at its front
    if (has_stream) reinterpret_cast<uint16_t *>(out + kFront)[t] = (uint16_t)(nb | (hb ? (hb - 1) << 12 : 0));
    // the area of a stream set: its whole blocks, then the short first blocks, lane after lane
    const uint32_t whole_incl = lanes_prefix_sum<false>(nb ? nb - 1 : 0);
    const uint32_t heads_incl = lanes_prefix_sum<false>(hb);
    const uint32_t whole_total = (uint32_t)__builtin_amdgcn_readlane((int)whole_incl, 63);
    const uint32_t heads_total = (uint32_t)__builtin_amdgcn_readlane((int)heads_incl, 63);
    if (lane == 63) set_bytes[wave] = (DC_BLOCK_BYTES * whole_total + heads_total + 15u) & ~15u;
    __syncthreads();
    const uint32_t hdr = header_bytes(S, CODEC);
    const uint32_t n_sets = S / set_width(S);
    uint32_t region = hdr; // first byte of this wave's area
    for (uint32_t w = 0; w < wave; w++) region += set_bytes[w];
    if (lane == 0 && wave < n_sets) reinterpret_cast<uint32_t *>(out + kFront + 2 * S)[wave] = region;
    const uint32_t heads_at = region + DC_BLOCK_BYTES * whole_total;                  // the heads of the set, padded to 16 ...
    const uint32_t heads_padded = set_bytes[wave] - DC_BLOCK_BYTES * whole_total; // ... take this many bytes
    for (uint32_t i = kFront + 2 * S + 4 * n_sets + t; i < hdr; i += THREADS) out[i] = 0;

    // ---- canonical codes: numbered in order of (length, byte value).  A wave looks at 64 consecutive
    // byte values at a time: rank = values of the same length before this one within the 64.
    for (uint32_t v = t; v < 256 && !TANS; v += THREADS) {
        const uint32_t l = len_of[v];
        uint32_t rank = 0;
        for (uint32_t l2 = 1; l2 <= (uint32_t)kL; l2++) {
            const uint64_t m = __ballot(l == l2);
            if (l == l2) rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            if (lane == 0) len_count[v >> 6][l2] = (uint32_t)__popcll(m);
        }
        book[v] = rank;
    }
    __syncthreads();
    for (uint32_t v = t; v < 256 && !TANS; v += THREADS) {
        const uint32_t l = len_of[v];
        uint32_t entry = 0;
        if (l) {
            // every shorter code of length m stands for 2^(l - m) codes of length l that come first
            uint32_t code = book[v];
            for (uint32_t m = 1; m < l; m++)
                code += (len_count[0][m] + len_count[1][m] + len_count[2][m] + len_count[3][m]) << (l - m);
            for (uint32_t b = 0; b < (v >> 6); b++) code += len_count[b][l];
            entry = (__brev(code) >> (32 - l)) | (l << 16);
        }
        book[v] = entry;
    }
    __syncthreads();
    if (!has_stream) return;

    // ---- the sub-stream of this lane
    const uint32_t groups = (raw + 15) / 16;
    const uint32_t rounds = (groups + S - 1) / S;
    const uint32_t my_groups = t < groups ? (groups - t + S - 1) / S : 0;
    const uint32_t ring_lane = lds_address(ring + wave * (16 * 64) + lane);
    uint32_t taken = 0, used = 8 * pad; // positions count from where block 0 would start
    u32x4 head_blk = {0, 0, 0, 0};
    uint32_t next_block = region / DC_BLOCK_BYTES;
    const uint64_t set_lanes = S < 64 ? (1ull << S) - 1 : ~0ull;

    // bytes [lo, lo + n) of the chunk, n <= 8, as a 64-bit word (missing bytes zero)
    auto half_group = [&](uint32_t h, uint32_t &n) -> uint64_t {
        const uint32_t g = t + (h >> 1) * S;
        const uint32_t lo = 16 * g + 8 * (h & 1);
        n = lo < raw ? (raw - lo < 8 ? raw - lo : 8) : 0;
        if (n == 8) return *reinterpret_cast<const uint64_t *>(src + lo);
        uint64_t v = 0;
        for (uint32_t i = 0; i < n; i++) v |= (uint64_t)src[lo + i] << (8 * i);
        return v;
    };

    // tANS: the items of those bytes, 8 of 16 bits (missing ones zero)
    const uint16_t *items = TANS ? a.items + k * a.chunk_bytes : nullptr;
    auto half_group_items = [&](uint32_t h, uint32_t &n) -> u32x4 {
        const uint32_t g = t + (h >> 1) * S;
        const uint32_t lo = 16 * g + 8 * (h & 1);
        n = lo < raw ? (raw - lo < 8 ? raw - lo : 8) : 0;
        if (n == 8) return *reinterpret_cast<const u32x4 *>(items + lo);
        u32x4 v = {0, 0, 0, 0};
        for (uint32_t i = 0; i < n; i++) v[i >> 1] |= (uint32_t)items[lo + i] << (16 * (i & 1u));
        return v;
    };

    // the coder starts behind the `pad` bytes that block 0 lacks (zeros in the ring, never stored)
    Coder c = {0, 8 * (pad & 3u), pad >> 2, 0, 0, {0, 0, 0, 0}, 0};
    for (uint32_t i = 0; i < (pad >> 2); i++) *(lds_u32 *)(uintptr_t)(ring_lane + (i << 8)) = 0;
    if (TANS && my_groups) {
        // a tANS stream opens with its first state
        c.acc = (uint64_t)a.first[k * S + t] << c.nbits;
        c.nbits += DC_TANS_STATE_BITS;
        if (c.nbits >= 32) {
            *(lds_u32 *)(uintptr_t)(ring_lane + ((c.words & 15u) << 8)) = (uint32_t)c.acc;
            c.words++;
            c.acc >>= 32;
            c.nbits -= 32;
        }
    }
    if (my_groups) {
        if (TANS) c.items = half_group_items(0, c.n);
        else c.bytes = half_group(0, c.n);
    }
    // codes the next half group into the ring: at most 88 bits on top of fewer than 32, so at most
    // three words
    auto code_half = [&]() {
        const uint64_t bytes = c.bytes;
        const u32x4 its = c.items;
        const uint32_t n = c.n;
        c.next_half++;
        if (c.next_half < 2 * my_groups) {
            if (TANS) c.items = half_group_items(c.next_half, c.n);
            else c.bytes = half_group(c.next_half, c.n);
        }
        auto flush = [&]() {
            if (c.nbits >= 32) {
                *(lds_u32 *)(uintptr_t)(ring_lane + ((c.words & 15u) << 8)) = (uint32_t)c.acc;
                c.words++;
                c.acc >>= 32;
                c.nbits -= 32;
            }
        };
        if (TANS) {
            // two items at a time: at most 22 bits on top of fewer than 32 (absent items are zero: no bits)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint32_t w0 = (its[i] >> 12) & 15u, w1 = its[i] >> 28;
                const uint32_t two = (its[i] & 0xFFFu) | ((its[i] >> 16) & 0xFFFu) << w0;
                c.acc |= (uint64_t)two << c.nbits;
                c.nbits += w0 + w1;
                flush();
            }
        } else if (n == 8) {
            // the table reads do not depend on each other; the bit buffer takes two codes (at most 22
            // bits on top of fewer than 32) between checks
            uint32_t e[8];
#pragma unroll
            for (int i = 0; i < 8; i++) e[i] = book[(bytes >> (8 * i)) & 0xFFu];
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                const uint32_t l0 = e[i] >> 16;
                const uint32_t two = (e[i] & 0xFFFFu) | (e[i + 1] & 0xFFFFu) << l0;
                c.acc |= (uint64_t)two << c.nbits;
                c.nbits += l0 + (e[i + 1] >> 16);
                flush();
            }
        } else {
            for (uint32_t i = 0; i < n; i++) { // the ragged end of the chunk
                const uint32_t e = book[(bytes >> (8 * i)) & 0xFFu];
                c.acc |= (uint64_t)(e & 0xFFFFu) << c.nbits;
                c.nbits += e >> 16;
                flush();
            }
        }
    };
    // bits that the items of a half group take
    auto bits_of_items = [&](const u32x4 &its) -> uint32_t {
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) sum += ((its[i] >> 12) & 15u) + (its[i] >> 28);
        return sum;
    };
    // bits that the codes of a half group take
    auto bits_of = [&](uint64_t bytes, uint32_t n) -> uint32_t {
        uint32_t sum = 0;
        if (n == 8) {
#pragma unroll
            for (int i = 0; i < 8; i++) sum += book[(bytes >> (8 * i)) & 0xFFu] >> 16;
        } else {
            for (uint32_t i = 0; i < n; i++) sum += book[(bytes >> (8 * i)) & 0xFFu] >> 16;
        }
        return sum;
    };

    for (uint32_t h = 0; h < 2 * rounds; h++) {
        // the half group a decoder consumes at this step (needed after the blocks of the step)
        uint32_t step_n = 0;
        uint64_t step_bytes = 0;
        u32x4 step_items = {0, 0, 0, 0};
        if ((h >> 1) < my_groups) {
            if (TANS) step_items = half_group_items(h, step_n);
            else step_bytes = half_group(h, step_n);
        }
        // All lanes code one half group ahead together while the ring has room for it (the words of
        // block `taken` onwards are still in the ring, 16 words in all), so that the loop below, where
        // lanes diverge, rarely has anything left to do.
        if (c.next_half < 2 * my_groups && c.words + 3 <= 4 * taken + 16) code_half();
        // step 0 is carried out four times (a fifth changes nothing for Huffman codes); a tANS stream has read its
        // first state before the fifth
        for (int pass = 0; pass < (h == 0 ? (TANS ? 5 : 4) : 1); pass++) {
            if (TANS && h == 0 && pass == 4 && my_groups) used += DC_TANS_STATE_BITS;
            const bool want = taken < nb && kBlockBits * taken < used + DC_LOOKAHEAD_BITS;
            if (want) {
                // code on until block `taken` is complete (or the stream ends, then pad with zeros)
                while (c.words < 4 * (taken + 1)) {
                    if (c.next_half < 2 * my_groups) {
                        code_half();
                    } else {
                        *(lds_u32 *)(uintptr_t)(ring_lane + ((c.words & 15u) << 8)) = (uint32_t)c.acc;
                        c.words++;
                        c.acc = 0;
                        c.nbits = 0;
                    }
                }
            }
            const bool head = taken == 0; // block 0 goes to the heads, without the bytes it lacks
            const uint64_t m = __ballot(want && !head) & set_lanes;
            if (want) {
                const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                u32x4 blk;
#pragma unroll
                for (int i = 0; i < 4; i++) blk[i] = lds_load32(ring_lane + (((4 * taken + i) & 15u) << 8));
                if (!head) *reinterpret_cast<u32x4 *>(out + (size_t)(next_block + rank) * DC_BLOCK_BYTES) = blk;
                else head_blk = blk; // written with the other heads of the set, below
                taken++;
            }
            next_block += (uint32_t)__popcll(m);
        }
        // the decoder's position after half group h
        used += TANS ? bits_of_items(step_items) : bits_of(step_bytes, step_n);
    }

    // ---- the heads of the set: put together in the wave's ring, which is free now (the lanes of a wave
    // leave the loop together), then written with whole 16-byte stores, the padding of the area included
    uint8_t *stage = reinterpret_cast<uint8_t *>(ring + wave * (16 * 64));
    if (lane == 0)
        for (uint32_t p = heads_total; p < heads_padded; p++) stage[p] = 0;
    for (uint32_t i = pad; i < DC_BLOCK_BYTES && nb; i++)
        stage[heads_incl - hb + i - pad] = (uint8_t)((i < 8 ? (i < 4 ? head_blk[0] : head_blk[1]) : (i < 12 ? head_blk[2] : head_blk[3])) >> (8 * (i & 3u)));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (uint32_t o = DC_BLOCK_BYTES * lane; o < heads_padded; o += DC_BLOCK_BYTES * 64)
        *reinterpret_cast<u32x4 *>(out + heads_at + o) = *reinterpret_cast<const u32x4 *>(stage + o);
}

template <int THREADS> void launch_emit(const EncArgs &a, hipStream_t stream)
{
    if (a.codec == DC_CODEC_TANS)
        hipLaunchKernelGGL((dc_emit_kernel<THREADS, DC_CODEC_TANS>), dim3((uint32_t)a.n_chunks), dim3(THREADS), 0, stream, a);
    else
        hipLaunchKernelGGL((dc_emit_kernel<THREADS, DC_CODEC_HUFFMAN>), dim3((uint32_t)a.n_chunks), dim3(THREADS), 0, stream, a);
}

bool enc_params_ok(const dc_params *p)
{
    if (!p) return false;
    if (p->chunk_bytes < 16 || p->chunk_bytes > DC_MAX_CHUNK_BYTES || p->chunk_bytes % 16) return false;
    if (p->n_streams != 32 && p->n_streams != 64 && p->n_streams != 128 && p->n_streams != 256) return false;
    if (p->codec == DC_CODEC_TANS ? p->n_streams < 64 : p->codec != DC_CODEC_HUFFMAN) return false;
    if (p->policy == DC_POLICY_BLOCK_LAST) return p->block_chunks != 0;
    if (p->policy == DC_POLICY_RAW_FRACTION) return p->raw_fraction >= 0.0f && p->raw_fraction <= 1.0f;
    return p->policy == DC_POLICY_ALL_HUFF || p->policy == DC_POLICY_AUTO;
}

uint64_t align256(uint64_t x) { return (x + 255) & ~255ull; }

} // namespace

extern "C" int dc_compress_chunks_dev_workspace(uint64_t raw_bytes, const dc_params *params, uint64_t *workspace_bytes)
{
    if (!enc_params_ok(params) || raw_bytes == 0 || !workspace_bytes) return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) return DC_E_FORMAT;
    const uint64_t nc = (raw_bytes + params->chunk_bytes - 1) / params->chunk_bytes;
    *workspace_bytes = align256(nc * 256) + align256(nc * params->n_streams * 4) + align256(nc * 4);
    // tANS: the frequencies, the first states and one 16-bit item per byte besides
    if (params->codec == DC_CODEC_TANS)
        *workspace_bytes += align256(nc * 512) + align256(nc * params->n_streams * 2) + align256(nc * params->chunk_bytes * 2);
    return DC_OK;
}

namespace {

// The three launches of the compression, with the workspace (code lengths, sub-stream sizes and payload
// sizes between them) wherever the caller of this function has it.
int compress_chunks_on_stream(const int8_t *src_dev, uint64_t raw_bytes, const dc_params *params, uint8_t *blob_dev,
                              uint64_t blob_cap, dc_chunk *table_dev, uint64_t table_cap, void *workspace_dev,
                              uint64_t workspace_bytes, uint64_t *result_dev, void *hip_stream)
{
    uint64_t need = 0;
    if (const int rc = dc_compress_chunks_dev_workspace(raw_bytes, params, &need)) return rc;
    if (!src_dev || !blob_dev || !table_dev || !workspace_dev || !result_dev) return DC_E_ARG;
    if ((reinterpret_cast<uintptr_t>(src_dev) & 15u) || (reinterpret_cast<uintptr_t>(blob_dev) & 15u) ||
        (reinterpret_cast<uintptr_t>(table_dev) & 7u) || (reinterpret_cast<uintptr_t>(workspace_dev) & 15u) ||
        (reinterpret_cast<uintptr_t>(result_dev) & 7u))
        return DC_E_ARG;
    const uint64_t nc = (raw_bytes + params->chunk_bytes - 1) / params->chunk_bytes;
    if (nc > 0x7FFFFFFFull) return DC_E_ARG;
    if (workspace_bytes < need || table_cap < nc) return DC_E_CAP;
    EncArgs a = {};
    a.src = reinterpret_cast<const uint8_t *>(src_dev);
    a.raw_bytes = raw_bytes;
    a.n_chunks = nc;
    a.chunk_bytes = params->chunk_bytes;
    a.S = params->n_streams;
    a.policy = params->policy;
    a.block_chunks = params->block_chunks;
    a.n_raw = 0;
    if (params->policy == DC_POLICY_RAW_FRACTION) {
        a.n_raw = (uint64_t)((double)params->raw_fraction * (double)nc + 0.5);
        if (a.n_raw > nc) a.n_raw = nc;
    }
    uint8_t *ws = static_cast<uint8_t *>(workspace_dev);
    a.lens = ws;
    a.bits = reinterpret_cast<uint32_t *>(ws + align256(nc * 256));
    a.comp = reinterpret_cast<uint32_t *>(ws + align256(nc * 256) + align256(nc * a.S * 4));
    a.codec = params->codec;
    if (a.codec == DC_CODEC_TANS) {
        uint8_t *more = ws + align256(nc * 256) + align256(nc * a.S * 4) + align256(nc * 4);
        a.freq = reinterpret_cast<uint16_t *>(more);
        a.first = reinterpret_cast<uint16_t *>(more + align256(nc * 512));
        a.items = reinterpret_cast<uint16_t *>(more + align256(nc * 512) + align256(nc * a.S * 2));
    }
    a.blob = blob_dev;
    a.blob_cap = blob_cap;
    a.table = table_dev;
    a.result = result_dev;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (a.codec == DC_CODEC_TANS) hipLaunchKernelGGL(dc_tans_model_kernel, dim3((uint32_t)nc), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(dc_codes_kernel, dim3((uint32_t)nc), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(dc_layout_kernel, dim3(1), dim3(256), 0, stream, a);
    switch (a.S) {
    case 32:
    case 64: launch_emit<64>(a, stream); break;
    case 128: launch_emit<128>(a, stream); break;
    default: launch_emit<256>(a, stream); break;
    }
    return dc_launch_status();
}

} // namespace

extern "C" int dc_compress_chunks_dev(const int8_t *src_dev, uint64_t raw_bytes, const dc_params *params,
                                      uint8_t *blob_dev, uint64_t blob_cap, dc_chunk *table_dev, uint64_t table_cap,
                                      void *workspace_dev, uint64_t workspace_bytes, uint64_t *result_dev,
                                      void *hip_stream)
{
    return compress_chunks_on_stream(src_dev, raw_bytes, params, blob_dev, blob_cap, table_dev, table_cap, workspace_dev,
                                     workspace_bytes, result_dev, hip_stream);
}

// ---- the same call for callers that cannot allocate: the workspace is a fixed array in device memory

// Workspace of dc_compress_chunks_dev_static.  One copy per GPU that runs the library, held until the
// process ends.  In host code this name only stands for the array: its address on the current device comes
// from hipGetSymbolAddress (static_scratch below), and only that address is handed to kernels.
static __device__ __align__(256) uint8_t scratch[DC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_of_device[kMaxDevices]; // address of `scratch` on every device that has asked for it

// Address of the workspace array on the current device (looked up once per device), or null with the HIP
// status noted for dc_last_hip_error().
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        dc_launch_status();
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_of_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            dc_launch_status();
            return nullptr;
        }
        g_scratch_of_device[dev] = p;
    }
    return g_scratch_of_device[dev];
}

} // namespace

extern "C" int dc_compress_chunks_dev_static(const int8_t *src_dev, uint64_t raw_bytes, const dc_params *params,
                                             uint8_t *blob_dev, uint64_t blob_cap, dc_chunk *table_dev,
                                             uint64_t table_cap, uint64_t *result_dev, void *hip_stream)
{
    uint64_t need = 0;
    if (const int rc = dc_compress_chunks_dev_workspace(raw_bytes, params, &need)) return rc;
    if (need > DC_STATIC_SCRATCH_BYTES) return DC_E_CAP; // the input is beyond what the fixed workspace serves
    void *ws = static_scratch();
    if (!ws) return DC_E_HIP;
    return compress_chunks_on_stream(src_dev, raw_bytes, params, blob_dev, blob_cap, table_dev, table_cap, ws,
                                     DC_STATIC_SCRATCH_BYTES, result_dev, hip_stream);
}
