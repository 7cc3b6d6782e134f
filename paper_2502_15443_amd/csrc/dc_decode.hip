// Device side of libdc_mi355x: chunk decode kernels for gfx950 (CDNA4, wave64).
//
// Paper: Section 3.3 ("Inference Process", "Throughput Analysis"): compressed chunks resident in GPU
// memory are decompressed by the GPU into a decompression buffer; "Speed Adaptive Partial
// Compression": some chunks are raw and only need a copy.  The stored format is in include/dc.h.
//
// Work decomposition: a lane owns one sub-stream, a wavefront owns one stream set (64 sub-streams
// whose 16-byte blocks are stored interleaved in the order the wavefront asks for them), a workgroup
// owns one chunk (S/64 wavefronts; with S = 32 one wavefront owns two chunks, lanes 0-31 / 32-63).
// Per chunk the LDS holds the decode table (2048 x u16: symbol << 8 | length - 1, indexed by the next
// 11 stream bits).  Per wavefront the LDS holds a ring of 16 stream words per lane.  Before every
// half group of 8 symbols the lanes that are short of look-ahead each take the next block of the
// wavefront's region (consecutive lanes, consecutive blocks: one coalesced load, and the region is
// read front to back exactly once); the block goes into the ring two steps later (the look-ahead of
// DC_LOOKAHEAD_BITS bits in the format allows for it), so the per-symbol loop does not wait on memory.  A lane packs 16 decoded bytes and writes them with one 128-bit
// store; the lanes of a chunk write S*16 contiguous bytes per round.
//
// The container's second coder (tANS, 2048 states; Section 4.2 of the paper settles on ANS) runs through the
// same kernel with another table and another symbol step: the table holds one 32-bit entry per state
// (build_tans_table), the lane carries the state, and a symbol costs one table read and the state's field
// of stream bits (tans_symbols).  Rings, block placement, refills, stores and the fused epilogues are shared.
#include <hip/hip_runtime.h>

#include "dc.h"
#include "dc_device.h"

using namespace dcdev;

namespace {

constexpr int kPeekBits = DC_MAX_CODE_LEN;
constexpr int kTableEntries = 1 << kPeekBits;
constexpr int kRingWords = 16;                 // per lane
constexpr uint32_t kBlockBytes = DC_BLOCK_BYTES; // bitstream fetch granule

// kModeGemv adds the partial sums in a fixed order (per wave in registers, per chunk through LDS, per row in
// dc_gemv_ordered_finish_kernel); kModeGemvAtomic is the same product with one atomic per run of lanes, for
// shapes with more rows to a chunk than a wave has lanes.
enum Mode { kModeI8 = 0, kModeBf16 = 1, kModeGemv = 2, kModeGemvW8A8 = 3, kModeGemvAtomic = 4 };
constexpr uint32_t kPartialSlots = 64; // fp32 partial sums a chunk leaves in the workspace of the ordered product

template <int S> struct Geometry {
    static constexpr int kLanesPerChunk = S < 64 ? S : 64;       // lanes of one wave that serve a chunk
    static constexpr int kChunksPerWave = 64 / kLanesPerChunk;   // 2 when S = 32
    static constexpr int kWaves = S <= 64 ? 1 : S / 64;          // wavefronts of the workgroup
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kThreadsPerChunk = S < 64 ? S : kThreads;
    static constexpr int kSymbolsPerLane = 256 / kThreadsPerChunk; // header values a thread ranks in the table build
};

// One matrix of a fused call: its chunks are table entries [first_chunk, next matrix's first_chunk).
struct MatrixArgs {
    uint64_t first_chunk;
    uint32_t rows, cols;
    const float *row_scale;
    void *dst;              // kModeBf16: bf16 [rows][cols]
    const uint16_t *x_bf16; // kModeGemv
    float *y_accum;         // kModeGemv; kModeGemvW8A8: int32 sums until the finish kernel has run
    uint16_t *y_bf16;       // both products, may be null
    const int8_t *x_i8;     // kModeGemvW8A8
    float x_scale;          // kModeGemvW8A8
};

struct DecodeArgs {
    const uint8_t *blob;
    uint64_t blob_bytes;
    const dc_chunk *table;
    uint64_t n_chunks;
    uint32_t chunk_bytes;
    uint32_t trailer[4]; // what the blob's last 16 bytes must be for this launch to decode it
    uint64_t *trace;     // traced launches: four words per workgroup (see dc_decompress_chunks_traced), else null
    // kModeI8: all chunks decode into one buffer of dst_cap bytes
    void *dst;
    uint64_t dst_cap;
    // kModeGemv: kPartialSlots sums per chunk (slot r: the chunk's share of the r-th row it touches)
    float *partial;
    // fused modes: the matrices, in table order
    uint32_t n_mats;
    MatrixArgs mats[DC_MAX_MATRICES];
};

// Sums `val` (float or int32) over runs of consecutive lanes with equal `key` (keys do not decrease with
// the lane; key 0xFFFFFFFF = lane takes no part) and adds each run's sum to y[key] with one atomic,
// issued by the last lane of the run.
template <bool HALVES, typename T> __device__ __forceinline__ void lanes_add_by_key(T *__restrict__ y, uint32_t key, T val)
{
    static_assert(sizeof(T) == 4, "one register");
#define DC_SEG_STEP(CTRL, MASK)                                                                              \
    {                                                                                                        \
        const uint32_t k2 = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)key, CTRL, MASK, 0xF, false);     \
        const T v2 = __builtin_bit_cast(T, dpp_or_zero<CTRL, MASK>(__builtin_bit_cast(uint32_t, val)));      \
        val += k2 == key ? v2 : T(0);                                                                        \
    }
    DC_SEG_STEP(0x111, 0xF)
    DC_SEG_STEP(0x112, 0xF)
    DC_SEG_STEP(0x114, 0xF)
    DC_SEG_STEP(0x118, 0xF)
    DC_SEG_STEP(0x142, 0xA)
    if (!HALVES) DC_SEG_STEP(0x143, 0xC)
#undef DC_SEG_STEP
    // 0x130: the value of the lane above (lane 63 reads the fill value)
    uint32_t above = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)key, 0x130, 0xF, 0xF, false);
    if (HALVES && (threadIdx.x & 31u) == 31u) above = 0xFFFFFFFFu;
    if (key != 0xFFFFFFFFu && above != key) atomicAdd(y + key, val);
}

// The same sums, kept in the wave: the sum of every run goes to the lane whose number is the run's `slot`
// (slot < 64, the same for all lanes of a run), where it is added to `mine`.  Runs are taken in lane order and
// each lane adds at most one value per call, so the result does not depend on timing.
template <bool HALVES> __device__ __forceinline__ void lanes_add_runs_to_slots(float &mine, uint32_t key, uint32_t slot, float val)
{
    if (!HALVES) {
        // the usual case with rows of some kilobytes: all 64 lanes hold the same row (or none): one plain sum
        const uint32_t first = (uint32_t)__builtin_amdgcn_readfirstlane((int)key);
        if (__all(key == first)) {
            if (first != 0xFFFFFFFFu) {
                const float total = lanes_sum(val); // in lane 63
                const float v = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(total), 63));
                const uint32_t to = (uint32_t)__builtin_amdgcn_readfirstlane((int)slot) & 63u;
                mine += (threadIdx.x & 63u) == to ? v : 0.0f;
            }
            return;
        }
    }
#define DC_SEG_STEP(CTRL, MASK)                                                                              \
    {                                                                                                        \
        const uint32_t k2 = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)key, CTRL, MASK, 0xF, false);     \
        const float v2 = __uint_as_float(dpp_or_zero<CTRL, MASK>(__float_as_uint(val)));                     \
        val += k2 == key ? v2 : 0.0f;                                                                        \
    }
    DC_SEG_STEP(0x111, 0xF)
    DC_SEG_STEP(0x112, 0xF)
    DC_SEG_STEP(0x114, 0xF)
    DC_SEG_STEP(0x118, 0xF)
    DC_SEG_STEP(0x142, 0xA)
    if (!HALVES) DC_SEG_STEP(0x143, 0xC)
#undef DC_SEG_STEP
    uint32_t above = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)key, 0x130, 0xF, 0xF, false);
    if (HALVES && (threadIdx.x & 31u) == 31u) above = 0xFFFFFFFFu;
    uint64_t ends = __ballot(key != 0xFFFFFFFFu && above != key); // the last lane of every run
    const uint32_t lane = threadIdx.x & 63u;
    while (ends) {
        const uint32_t from = (uint32_t)__builtin_ctzll(ends);
        const uint32_t to = (uint32_t)__builtin_amdgcn_readlane((int)slot, from) & 63u;
        const float v = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(val), from));
        mine += lane == to ? v : 0.0f;
        ends &= ends - 1;
    }
}

// One sub-stream as its lane sees it.  Stream words travel memory -> blk -> LDS ring -> next -> buf.
// The ring of a wave is 4 KiB, 4 KiB aligned; ring word j of the lane sits at byte
// (j % 16) * 256 + lane * 4 of it, so the lanes of a wave never collide on a bank and the slot bits
// (0xF00) can be OR-ed into the lane's base address.
struct Stream {
    uint64_t buf;   // LSB-first bit buffer
    uint32_t state; // 256 * (words taken out of the ring) + (valid bits in buf, at most 64)
    uint32_t next;  // the word that follows buf
    uint32_t tk10;  // 1024 * (blocks asked for so far, f of the placement rule)
    uint32_t nb10;  // 1024 * (blocks of the stream)
    uint32_t npend[2]; // -1024: blk[p] holds a block asked for at the last step of parity p, not yet in the ring; else 0
    uint32_t x4;      // tANS: 4 * state = byte offset of the state's table entry
    u32x4 blk[2];     // a block travels for two steps: asked for at step h, put into the ring at step h + 2
};

// What the lanes of one stream set share: where the block region of the set's area stands.
struct Region {
    const uint8_t *payload8;
    uint32_t next_block; // in 16-byte units from the payload start
    uint32_t max_off;    // last payload offset 20 bytes may be loaded from without leaving the blob
    uint64_t lanes;      // the lanes of the wave that belong to the set
};

// 16 bytes at an address that is a multiple of 4 only
typedef uint32_t u32x4_align4 __attribute__((ext_vector_type(4), aligned(4)));

// Block number b of a stream goes to ring words 4b .. 4b+3.
__device__ __forceinline__ void push_block(uint32_t block10, const u32x4 &blk, uint32_t ring_lane)
{
    lds_u32 *w = (lds_u32 *)(uintptr_t)((block10 & 0xF00u) | ring_lane);
    w[0] = blk[0];
    w[64] = blk[1];
    w[128] = blk[2];
    w[192] = blk[3];
}

__device__ __forceinline__ uint32_t ring_word(uint32_t state, uint32_t ring_lane)
{
    return lds_load32((state & 0xF00u) | ring_lane);
}

// The lanes with `want` each take the next block of the region, in lane order.
template <bool UNIFORM>
__device__ __forceinline__ void take_blocks(Stream &s, Region &rg, bool want, u32x4 &dst)
{
    const uint64_t m = __ballot(want) & rg.lanes;
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (want) {
        uint32_t off = (rg.next_block + rank) * kBlockBytes;
        const uint32_t limit = rg.max_off & ~15u;
        off = off < limit ? off : limit;
        dst = *reinterpret_cast<const u32x4 *>(rg.payload8 + off);
        s.tk10 += 1024;
    }
    rg.next_block += (uint32_t)__popcll(m);
    if (UNIFORM) rg.next_block = __builtin_amdgcn_readfirstlane(rg.next_block);
}

// The same inside the decode loop: every lane loads; a lane without `want` loads, and drops, a block that a
// lane below it asks for, or the one after the last asked for (the address is inside the payload in any case).
// A load that is always issued lets the wait for an earlier load be exact (it counts the loads issued
// since), so a block can stay in flight across the next step's load.  npend = -1024 where the lane asked.
template <bool UNIFORM>
__device__ __forceinline__ void take_blocks_all_load(Stream &s, Region &rg, bool want, u32x4 &dst, uint32_t &npend)
{
    const uint64_t m = __ballot(want) & rg.lanes;
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    uint32_t off = (rg.next_block + rank) * kBlockBytes;
    const uint32_t limit = rg.max_off & ~15u;
    off = off < limit ? off : limit;
    dst = *reinterpret_cast<const u32x4 *>(rg.payload8 + off);
    npend = want ? 0xFFFFFC00u : 0u;
    s.tk10 -= npend;
    rg.next_block += (uint32_t)__popcll(m);
    if (UNIFORM) rg.next_block = __builtin_amdgcn_readfirstlane(rg.next_block);
}

// One step of the placement rule (before every half group; P = the step's parity): the block asked for two
// steps before goes into the ring, then the lanes short of look-ahead ask for their next block.  With
// used = 32*(words taken) - 32 - avail stream bits used so far, the rule's
// 128*f - used < DC_LOOKAHEAD_BITS reads, times 8, tk10 < state + 8*(DC_LOOKAHEAD_BITS - 32) - 9*avail.
// Why two steps are safe: before its decision at a step a stream has at least DC_LOOKAHEAD_BITS - 88 bits
// placed beyond its position, at least DC_LOOKAHEAD_BITS - 48 if it asked at the step before; the blocks
// asked for at this step and the one before are the only ones not in the ring, so at least
// DC_LOOKAHEAD_BITS - 176 = 216 bits are, and half a group reads at most 88 + 96 + 31 = 215 bits ahead.
template <bool UNIFORM, int P>
__device__ __forceinline__ void stream_step(Stream &s, Region &rg, uint32_t ring_lane)
{
    if (s.npend[P]) push_block(s.tk10 - 1024 + s.npend[1 - P], s.blk[P], ring_lane);
    const uint32_t avail = s.state & 0xFFu;
    // tk10 below both bounds: the look-ahead's (at least 2368, so no wrap) and the stream's blocks
    const uint32_t bound = s.state + 8u * (DC_LOOKAHEAD_BITS - 32) + (uint32_t)__mul24((int)avail, -9);
    const bool want = s.tk10 < (bound < s.nb10 ? bound : s.nb10);
    take_blocks_all_load<UNIFORM>(s, rg, want, s.blk[P], s.npend[P]);
}

// Start of a sub-stream.  Block 0 of a stream is short: its first pad = 16 - hb bytes do not exist and
// its hb bytes lie among the heads, which follow the whole blocks of the set in lane order.  The lane
// loads the 20 bytes from the 4-byte boundary at or before the place where block 0 would start and
// shifts them down, so the ring holds block 0 with foreign bytes in front, and starts reading behind
// them.  Then step 0 of the rule runs for the three further times (a stream takes a block while it
// has blocks left and fewer than DC_LOOKAHEAD_BITS bits beyond its position 8*pad), and buf and next
// are loaded.  (The step at the head of the decode loop is the fifth time; a tANS stream has read its
// first state by then.)
// What stream_fetch has asked memory for and stream_start puts into the ring.
struct StreamFetch {
    u32x4_align4 v; // the 20 bytes around the head of the stream
    uint32_t v4;
    uint32_t shift; // bytes to shift them down by
    uint32_t pad;   // bytes that block 0 lacks
    bool has_head;
    u32x4 b[3];     // up to three further blocks
    bool got[3];
};

// First half of the set-up: loads only, so that it can run before the decode table is built (the rings share
// their LDS with the scratch of the table build).
template <bool UNIFORM>
__device__ __forceinline__ void stream_fetch(Stream &s, Region &rg, uint32_t field, StreamFetch &f)
{
    // header field of the stream: blocks in all, and the bytes of block 0 less one
    const uint32_t nb = field & 0xFFFu;
    const uint32_t hb = nb ? ((field >> 12) & 15u) + 1 : 0;
    const uint32_t pad = nb ? kBlockBytes - hb : 0;
    const uint32_t whole_incl = lanes_prefix_sum<!UNIFORM>(nb ? nb - 1 : 0);
    const uint32_t heads_incl = lanes_prefix_sum<!UNIFORM>(hb);
    uint32_t whole_total = (uint32_t)__builtin_amdgcn_readlane((int)whole_incl, 63);
    if (!UNIFORM) {
        const uint32_t lower = (uint32_t)__builtin_amdgcn_readlane((int)whole_incl, 31);
        whole_total = (threadIdx.x & 32u) ? whole_total : lower;
    }
    s.nb10 = nb << 10;
    s.tk10 = 0;
    s.npend[0] = s.npend[1] = 0;
    f.pad = pad;
    f.has_head = nb != 0;
    f.shift = 0;
    if (nb) {
        uint32_t at = (rg.next_block + whole_total) * kBlockBytes + (heads_incl - hb) - pad; // the header lies before it
        at = at < rg.max_off ? at : rg.max_off;
        const uint8_t *p = rg.payload8 + (at & ~3u);
        f.v = *reinterpret_cast<const u32x4_align4 *>(p);
        f.v4 = *reinterpret_cast<const uint32_t *>(p + 16);
        f.shift = at & 3u;
        s.tk10 = 1024;
    }
#pragma unroll
    for (int t = 0; t < 3; t++) {
        f.got[t] = s.tk10 < s.nb10 && s.tk10 < ((8u * pad + DC_LOOKAHEAD_BITS) << 3); // 128 f < c + look-ahead, times 8
        take_blocks<UNIFORM>(s, rg, f.got[t], f.b[t]);
    }
}

// Second half: block 0 shifted into place and the further blocks go into the ring, and buf and next are loaded.
__device__ __forceinline__ void stream_start(Stream &s, const StreamFetch &f, uint32_t ring_lane)
{
    if (f.has_head) {
        const u32x4 b0 = {__builtin_amdgcn_alignbyte(f.v[1], f.v[0], f.shift), __builtin_amdgcn_alignbyte(f.v[2], f.v[1], f.shift),
                          __builtin_amdgcn_alignbyte(f.v[3], f.v[2], f.shift), __builtin_amdgcn_alignbyte(f.v4, f.v[3], f.shift)};
        push_block(0, b0, ring_lane);
    }
#pragma unroll
    for (int t = 0; t < 3; t++)
        if (f.got[t]) push_block((t + 1) << 10, f.b[t], ring_lane);
    // the stream begins `pad` bytes into block 0
    const uint32_t skip = f.pad >> 2, bits = 8u * (f.pad & 3u);
    const uint32_t lo = ring_word(skip << 8, ring_lane);
    const uint32_t hi = ring_word((skip + 1) << 8, ring_lane);
    s.buf = ((uint64_t)lo | ((uint64_t)hi << 32)) >> bits;
    s.next = ring_word((skip + 2) << 8, ring_lane);
    s.state = ((skip + 3) << 8) + 64 - bits;
}

// Takes the look-ahead word into the buffer when at most 32 bits are valid.  After it at least 32 bits
// are valid, and exactly 32 only if the buffer was empty: enough for two codes of 11 bits.
__device__ __forceinline__ void refill(Stream &s, uint32_t ring_lane)
{
    if ((s.state & 0xFFu) <= 32) {
        s.buf |= (uint64_t)s.next << (s.state & 63u);
        s.next = ring_word(s.state, ring_lane);
        s.state += 256 + 32;
    }
}

// Three codes of 11 bits need 33 bits.  A buffer that was empty holds 32 after one refill (the three codes
// before it used all 33 bits it had: rare, but it happens); the second call then takes one more word.
__device__ __forceinline__ void refill33(Stream &s, uint32_t ring_lane)
{
    refill(s, ring_lane);
    refill(s, ring_lane);
}

// Table entry = (length - 1) | symbol << 8: the field a 32-bit shift reads (its low 5 bits) is the
// amount that turns "the next 11 bits, times 2" (the byte offset of the next table entry) into a
// single shift and mask.
__device__ __forceinline__ uint32_t table_entry(uint32_t tbl, uint32_t window_times_2)
{
    return lds_load16(tbl + (window_times_2 & (2 * kTableEntries - 2)));
}

// The next N (2 or 3) symbols; at least 11*N bits are valid in buf.  With m_i = length_i - 1:
// the offsets of the three entries are (lo << 1), (lo >> m_0) and (buf >> (m_0 + m_1 + 1)), each masked
// to 0xFFE; the bits used are sum(m_i) + N.
template <int N> __device__ __forceinline__ void symbols(Stream &s, uint32_t tbl, uint32_t *e)
{
    const uint32_t lo = (uint32_t)s.buf, hi = (uint32_t)(s.buf >> 32);
    e[0] = table_entry(tbl, lo << 1);
    e[1] = table_entry(tbl, lo >> (e[0] & 31u));
    uint32_t used = e[0] + e[1] + 1;
    if (N == 3) {
        e[2] = table_entry(tbl, __builtin_amdgcn_alignbit(hi, lo, used));
        used += e[2] + 1;
    }
    used += 1;
    s.buf >>= (used & 63u);
    s.state -= used & 0xFFu;
}

// tANS.  Table entry of a state = nb | value << 8 | (4 * base) << 16, where nb is the width of the state's
// field and base the next state before the field is added; bits 4-7 are 0, so that the low five bits of an
// entry (and of a sum of two) can be used as a field width or offset as they are, and the low byte of a sum
// of three is the number of bits used.  The next N (2 or 3) symbols; at least 11*N bits are valid in buf.
template <int N> __device__ __forceinline__ void tans_symbols(Stream &s, uint32_t tbl, uint32_t *e)
{
    const uint32_t lo = (uint32_t)s.buf, hi = (uint32_t)(s.buf >> 32);
    e[0] = lds_load32(tbl + s.x4);
    uint32_t x4 = (e[0] >> 16) + (__builtin_amdgcn_ubfe(lo, 0u, e[0]) << 2);
    e[1] = lds_load32(tbl + x4);
    x4 = (e[1] >> 16) + (__builtin_amdgcn_ubfe(lo, e[0], e[1]) << 2);
    uint32_t used = e[0] + e[1];
    if (N == 3) {
        e[2] = lds_load32(tbl + x4);
        x4 = (e[2] >> 16) + (__builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(hi, lo, used), 0u, e[2]) << 2);
        used += e[2];
    }
    s.x4 = x4;
    s.buf >>= (used & 63u);
    s.state -= used & 0xFFu;
}

// One tANS symbol at a time, for the ragged end of a chunk.
__device__ __forceinline__ uint32_t tans_decode1(Stream &s, uint32_t tbl, uint32_t ring_lane)
{
    refill(s, ring_lane);
    const uint32_t e = lds_load32(tbl + s.x4);
    const uint32_t nb = e & 15u;
    s.x4 = (e >> 16) + (__builtin_amdgcn_ubfe((uint32_t)s.buf, 0u, nb) << 2);
    s.buf >>= nb;
    s.state -= nb;
    return (e >> 8) & 0xFFu;
}

// bytes 1 of four entries -> one little-endian word of four symbols
__device__ __forceinline__ uint32_t pack4(uint32_t e0, uint32_t e1, uint32_t e2, uint32_t e3)
{
    const uint32_t lo = __builtin_amdgcn_perm(e1, e0, 0x0c0c0501u);
    const uint32_t hi = __builtin_amdgcn_perm(e3, e2, 0x0c0c0501u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Symbols [8*HALF, 8*HALF + 8) of a group: 3 + 2 + 3 symbols.  Only the first batch can meet an empty buffer
// (the batch before it, the last of the half group before, may have used all 33 bits it had) and needs the second
// refill; the two symbols leave at least 10 of the 32 bits their refill guarantees, so one refill gives the
// last three their 33.
template <int HALF, int CODEC>
__device__ __forceinline__ void decode8(Stream &s, uint32_t tbl, uint32_t ring_lane, uint32_t out[4])
{
    uint32_t e[8];
    refill33(s, ring_lane);
    if (CODEC == DC_CODEC_TANS) tans_symbols<3>(s, tbl, e); else symbols<3>(s, tbl, e);
    refill(s, ring_lane);
    if (CODEC == DC_CODEC_TANS) tans_symbols<2>(s, tbl, e + 3); else symbols<2>(s, tbl, e + 3);
    refill(s, ring_lane);
    if (CODEC == DC_CODEC_TANS) tans_symbols<3>(s, tbl, e + 5); else symbols<3>(s, tbl, e + 5);
    out[2 * HALF] = pack4(e[0], e[1], e[2], e[3]);
    out[2 * HALF + 1] = pack4(e[4], e[5], e[6], e[7]);
}

// One whole group of 16 symbols with the two steps of the placement rule that precede its halves.
template <bool UNIFORM, int CODEC = DC_CODEC_HUFFMAN>
__device__ __forceinline__ void decode16(Stream &s, Region &rg, uint32_t tbl, uint32_t ring_lane, bool has_group,
                                         uint32_t out[4])
{
    stream_step<UNIFORM, 0>(s, rg, ring_lane);
    if (has_group) decode8<0, CODEC>(s, tbl, ring_lane, out);
    stream_step<UNIFORM, 1>(s, rg, ring_lane);
    if (has_group) decode8<1, CODEC>(s, tbl, ring_lane, out);
}

// One symbol at a time, for the ragged end of a chunk.
__device__ __forceinline__ uint32_t decode1(Stream &s, uint32_t tbl, uint32_t ring_lane)
{
    refill(s, ring_lane);
    const uint32_t e = table_entry(tbl, (uint32_t)s.buf << 1);
    const uint32_t used = (e & 15u) + 1;
    s.buf >>= used;
    s.state -= used;
    return e >> 8;
}

__device__ __forceinline__ uint32_t bf16x2(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}

// acc + a.lo * b.lo + a.hi * b.hi for two pairs of bf16 values
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "v"(a), "v"(b));
    return acc;
}

// int8 value number N of a word as fp32: one v_cvt_f32_i32 whose operand selects the byte and sign-extends it
template <int N> __device__ __forceinline__ float byte_f32(uint32_t w) { return (float)(int)(int8_t)(w >> (8 * N)); }

// Four int8 values in a word -> fp32, times the row scale (one rounding, as the dequantisation is defined).
__device__ __forceinline__ void word_to_scaled_f32(uint32_t w, float s, float f[4])
{
    f[0] = byte_f32<0>(w) * s;
    f[1] = byte_f32<1>(w) * s;
    f[2] = byte_f32<2>(w) * s;
    f[3] = byte_f32<3>(w) * s;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }


// The tANS table of a chunk (S >= 64: the workgroup's threads are the chunk's).  front: 4 KiB of LDS not yet
// in use (the rings); table32: the 2048 entries; cumq: 256 words; wave_sum: one word per wave.  The threads
// read the 256 frequencies, take their prefix sums (value v owns places cum[v] .. cum[v] + q[v] - 1) and mark
// the first place of every value; then every thread takes 2048/threads consecutive places, finds each
// place's value, and numbers the place among the places of its value by the order of the states (the places
// with their 11 bits reversed): place p of a value with places a .. a+q-1 has as many states below it as there are
// places p' of the value whose reversal is smaller, that is, for every set bit i of p, the places of the value
// that agree with p below bit i and have bit i clear: (q + M - 1 - ((p - a - 2^i) mod M)) div M of them, M = 2^(i+1).
// Returns false (for every thread alike) when the frequencies do not add up to 2048; nothing is decoded then.
template <int S>
__device__ __forceinline__ bool build_tans_table(const uint8_t *payload8, uint32_t ct, uint32_t lane, uint32_t wave,
                                                 uint32_t *front, uint32_t *table32, uint32_t *cumq, uint32_t *wave_sum)
{
    using G = Geometry<S>;
    constexpr int WAVES = G::kWaves;
    constexpr int TPC = G::kThreadsPerChunk;
    constexpr int SPL = G::kSymbolsPerLane;
    constexpr int EPT = kTableEntries / TPC;
    constexpr uint32_t L = kTableEntries;
    uint16_t *marks = reinterpret_cast<uint16_t *>(front);
    {
        uint4 *z = reinterpret_cast<uint4 *>(marks);
        for (uint32_t i = ct; i < kTableEntries * 2 / 16; i += TPC) z[i] = make_uint4(0, 0, 0, 0);
    }
    uint32_t q[SPL], mine = 0;
#pragma unroll
    for (int s = 0; s < SPL; s++) {
        const uint32_t v = ct * SPL + s;
        const uint8_t *g = payload8 + 3 * (v >> 1); // two 12-bit frequencies in three bytes
        q[s] = (v & 1u) ? ((uint32_t)g[1] >> 4 | (uint32_t)g[2] << 4) : ((uint32_t)g[0] | ((uint32_t)g[1] & 15u) << 8);
        mine += q[s];
    }
    const uint32_t incl = lanes_prefix_sum<false>(mine);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t cum = incl - mine, total = 0;
#pragma unroll
    for (int w = 0; w < WAVES; w++) {
        const uint32_t c = wave_sum[w];
        if ((uint32_t)w < wave) cum += c;
        total += c;
    }
    if (total != L) return false;
#pragma unroll
    for (int s = 0; s < SPL; s++) {
        const uint32_t v = ct * SPL + s;
        cumq[v] = cum | q[s] << 16;
        if (q[s]) {
            marks[cum] = (uint16_t)(v + 1);
            // also at the first place of every later wave that the value reaches into
            for (uint32_t p = (cum / (L / WAVES) + 1) * (L / WAVES); p < cum + q[s]; p += L / WAVES) marks[p] = (uint16_t)(v + 1);
        }
        cum += q[s];
    }
    __syncthreads();
    uint32_t w16[EPT / 2];
    {
        const uint4 *m4 = reinterpret_cast<const uint4 *>(marks + EPT * ct);
#pragma unroll
        for (int i = 0; i < EPT / 8; i++) {
            const uint4 v = m4[i];
            w16[4 * i] = v.x; w16[4 * i + 1] = v.y; w16[4 * i + 2] = v.z; w16[4 * i + 3] = v.w;
        }
    }
    uint32_t tail = 0; // last mark among this thread's places
#pragma unroll
    for (int i = 0; i < EPT / 2; i++) {
        const uint32_t lo = w16[i] & 0xFFFFu, hi = w16[i] >> 16;
        tail = lo ? lo : tail;
        tail = hi ? hi : tail;
    }
    uint32_t cur = lanes_last_nonzero_below<false>(tail);
    const uint32_t tbl = lds_address(table32);
#pragma unroll
    for (int i = 0; i < EPT; i++) {
        const uint32_t m = (i & 1) ? w16[i / 2] >> 16 : w16[i / 2] & 0xFFFFu;
        cur = m ? m : cur;
        const uint32_t v = cur - 1;
        const uint32_t cq = cumq[v & 255u];
        const uint32_t a = cq & 0xFFFFu, qv = cq >> 16;
        const uint32_t p = EPT * ct + i, t = p - a;
        uint32_t k = qv;
#pragma unroll
        for (int b = 0; b < kPeekBits; b++) {
            const uint32_t M = 2u << b;
            const uint32_t n = (qv + M - 1 - ((t - (1u << b)) & (M - 1))) >> (b + 1);
            k += ((p >> b) & 1u) ? n : 0u;
        }
        const uint32_t nb = (uint32_t)__builtin_clz(k | 1u) - (31 - kPeekBits);
        const uint32_t base = ((k << nb) - L) & (L - 1);
        *(lds_u32 *)(uintptr_t)(tbl + 4 * (__brev(p) >> (32 - kPeekBits))) = nb | (v & 255u) << 8 | base << 18;
    }
    __syncthreads();
    return true;
}

template <int S, int MODE, int CODEC, bool TRACE = false>
__global__ __launch_bounds__(Geometry<S>::kThreads) void dc_decode_kernel(DecodeArgs a)
{
    using G = Geometry<S>;
    // traced launches: when the workgroup began and ended (ticks of the constant 100 MHz clock), where it ran (the
    // HW_ID register, the XCC_ID register above it) and what it did with its chunk
    const uint64_t began = TRACE ? wall_clock64() : 0;
    auto leave_record = [&](uint32_t did) {
        if (TRACE && threadIdx.x == 0) {
            uint64_t *r = a.trace + 4 * (size_t)blockIdx.x;
            r[0] = began;
            r[1] = wall_clock64();
            r[2] = (uint64_t)(uint32_t)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 4) |
                   (uint64_t)(uint32_t)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 20) << 32;
            r[3] = did;
        }
    };
    constexpr int LPC = G::kLanesPerChunk;
    constexpr int CPW = G::kChunksPerWave;
    constexpr int WAVES = G::kWaves;
    constexpr int TPC = G::kThreadsPerChunk;
    constexpr int SPL = G::kSymbolsPerLane;
    static_assert(CODEC == DC_CODEC_HUFFMAN || S >= 64, "tANS: the workgroup's threads are the chunk's");
    constexpr uint32_t kFront = CODEC == DC_CODEC_TANS ? 384 : 128; // code description at the start of a payload
    constexpr uint32_t kHeader = (kFront + 2 * S + 4 * (S / Geometry<S>::kLanesPerChunk) + 15) / 16 * 16;

    // One block of LDS: the rings (4 KiB a wave, 4 KiB aligned) and then the decode tables.  While
    // the tables are built, before any ring is used, the front part holds the slot markers (one
    // u16 per table slot in code order, 4 KiB a chunk) and the start of the table part holds the
    // first codes of the lengths and the per-wave length counts.
    constexpr int kFrontWords = (WAVES > CPW ? WAVES : CPW) * kRingWords * 64;
    // (tANS: 2048 entries of 32 bits, then 256 words of (first place, frequency) and a word per wave)
    constexpr int kTableWords = CODEC == DC_CODEC_TANS ? kTableEntries + 256 + 16 : CPW * kTableEntries / 2;
    __shared__ __attribute__((aligned(4096))) uint32_t lds_all[kFrontWords + kTableWords];
    uint16_t(*lds_table)[kTableEntries] = reinterpret_cast<uint16_t(*)[kTableEntries]>(lds_all + kFrontWords);
    uint32_t(*lds_first)[16] = reinterpret_cast<uint32_t(*)[16]>(lds_all + kFrontWords); // [wave * CPW + sub][length]
    uint32_t(*lds_counts)[4] = reinterpret_cast<uint32_t(*)[4]>(lds_all + kFrontWords + 16 * WAVES * CPW); // [wave]

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t sub = lane / LPC;
    const uint32_t cl = lane % LPC;              // lane inside the chunk's share of the wave
    const uint32_t ct = wave * 64 + cl;          // thread inside the chunk = sub-stream number
    const uint64_t k = (uint64_t)blockIdx.x * CPW + sub;

    // ---- the blob's trailer: a blob of another format, or of other parameters, is left undecoded
    const uint32_t *closing = reinterpret_cast<const uint32_t *>(a.blob + a.blob_bytes - DC_TRAILER_BYTES);
    const bool readable = closing[0] == a.trailer[0] && closing[1] == a.trailer[1] && closing[2] == a.trailer[2] &&
                          closing[3] == a.trailer[3];
    // ---- chunk table entry, checked so that nothing below can leave the blob or the destination
    bool active = readable && k < a.n_chunks;
    dc_chunk ent = {0, 0, 0};
    if (active) ent = a.table[k];
    const uint32_t raw = ent.raw_bytes_flags & ~DC_CHUNK_RAW;
    const bool is_raw = (ent.raw_bytes_flags & DC_CHUNK_RAW) != 0;
    // fused modes: the matrix the chunk belongs to, and the chunk's number inside it
    uint32_t mi = 0;
    if (MODE != kModeI8)
        for (uint32_t i = 1; i < a.n_mats; i++)
            if (k >= a.mats[i].first_chunk) mi = i;
    const MatrixArgs &mat = a.mats[mi];
    const uint64_t dst_cap = MODE == kModeI8 ? a.dst_cap : (uint64_t)mat.rows * mat.cols;
    // first decoded byte of the chunk (in the buffer, or in its matrix)
    const uint64_t dst_pos = (MODE == kModeI8 ? k : k - mat.first_chunk) * (uint64_t)a.chunk_bytes;
    active = active && raw >= 1 && raw <= a.chunk_bytes && (ent.off & 15) == 0 && ent.off <= a.blob_bytes &&
             ent.comp_bytes <= a.blob_bytes - ent.off && ent.comp_bytes >= 16 && dst_pos + raw <= dst_cap &&
             (is_raw ? ent.comp_bytes >= ((raw + 15u) & ~15u) : ent.comp_bytes >= kHeader);
    const uint8_t *payload8 = a.blob + (active ? ent.off : 0);
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(payload8);
    const bool huff = active && !is_raw;

    uint16_t *tbl = lds_table[sub];
    const uint32_t tbl_addr = lds_address(tbl);
    const uint32_t ring_lane = lds_address(lds_all + wave * (kRingWords * 64) + lane);
    constexpr bool UNI = CPW == 1; // all lanes of the wave belong to one stream set

    // ---- raw chunks: the threads of the chunk copy it, eight 16-byte loads in flight per thread
    if (MODE == kModeI8 && CPW == 2) {
        // S = 32: the wavefront's two chunks one after the other, each copied by all 64 lanes with sixteen loads in
        // flight per lane (a wavefront alone on its SIMD has nothing but its own loads to hide a trip to memory behind)
        for (uint32_t h = 0; h < 2; h++) {
            const int from = 32 * (int)h;
            if (!__shfl((int)(active && is_raw), from)) continue;
            const uint64_t off_h = (uint64_t)(uint32_t)__shfl((int)(uint32_t)ent.off, from) |
                                   (uint64_t)(uint32_t)__shfl((int)(uint32_t)(ent.off >> 32), from) << 32;
            const uint32_t raw_h = (uint32_t)__shfl((int)raw, from);
            const uint8_t *p8 = a.blob + off_h;
            uint8_t *d8 = static_cast<uint8_t *>(a.dst) + ((uint64_t)blockIdx.x * CPW + h) * (uint64_t)a.chunk_bytes;
            const uint32_t n16 = raw_h / 16;
            for (uint32_t base = lane; base < n16; base += 16 * 64) {
                u32x4 v[16];
#pragma unroll
                for (int j = 0; j < 16; j++)
                    if (base + j * 64 < n16) v[j] = load16_stream(p8 + 16 * (size_t)(base + j * 64));
#pragma unroll
                for (int j = 0; j < 16; j++)
                    if (base + j * 64 < n16)
                        __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4 *>(d8 + 16 * (size_t)(base + j * 64)));
            }
            for (uint32_t i = n16 * 16 + lane; i < raw_h; i += 64) d8[i] = p8[i];
        }
    } else if (MODE == kModeI8 && active && is_raw) {
        uint8_t *d8 = static_cast<uint8_t *>(a.dst) + dst_pos;
        const uint32_t n16 = raw / 16;
        for (uint32_t base = ct; base < n16; base += 8 * TPC) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (base + j * TPC < n16) v[j] = load16_stream(payload8 + 16 * (size_t)(base + j * TPC));
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (base + j * TPC < n16)
                    __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4 *>(d8 + 16 * (size_t)(base + j * TPC)));
        }
        for (uint32_t i = n16 * 16 + ct; i < raw; i += TPC) d8[i] = payload8[i];
    }
    if (MODE != kModeI8 && !(active)) return;
    if (MODE == kModeI8 && !huff) {
        leave_record(active ? DC_TRACE_COPIED : DC_TRACE_SKIPPED);
        return;
    }

    // The table is only needed where a chunk of the workgroup is Huffman coded; the condition is the
    // same for every thread that is still here, so the barriers inside are reached together.
    // ---- the code lengths of the header are asked for first, so that they travel while the sub-streams are set up
    uint32_t nib_word = 0;
    if (CODEC == DC_CODEC_HUFFMAN && huff) {
        if (SPL == 8) nib_word = payload[ct];
        else if (SPL == 4) nib_word = reinterpret_cast<const uint16_t *>(payload8)[ct];
        else if (SPL == 2) nib_word = payload8[ct];
        else nib_word = payload8[ct >> 1];
    }

    // ---- sub-stream set-up, first half: the loads (all lanes of a stream set are here together or not at all)
    Region rg;
    Stream st;
    StreamFetch sf;
    if (huff) {
        rg.payload8 = payload8;
        // a 20-byte load may begin in the last bytes of the payload; the blob goes on for DC_BLOB_TAIL_BYTES
        const uint64_t room = a.blob_bytes - ent.off - 20;
        rg.max_off = room < 0xFFFFFFE0ull ? (uint32_t)room : 0xFFFFFFE0u;
        rg.lanes = CPW == 1 ? ~0ull : (sub ? 0xFFFFFFFF00000000ull : 0x00000000FFFFFFFFull);
        rg.next_block = payload[(kFront + 2 * S) / 4 + (CPW == 1 ? wave : 0)] / kBlockBytes;
        if (UNI) rg.next_block = __builtin_amdgcn_readfirstlane(rg.next_block);
        stream_fetch<UNI>(st, rg, reinterpret_cast<const uint16_t *>(payload8)[kFront / 2 + ct], sf);
    }

    const bool build_table = CODEC == DC_CODEC_TANS ? false : CPW == 1 ? huff : (bool)__any(huff);
    if (CODEC == DC_CODEC_TANS && huff) { // (one chunk per workgroup: the same for all of its threads)
        uint32_t *table32 = lds_all + kFrontWords;
        if (!build_tans_table<S>(payload8, ct, lane, wave, lds_all, table32, table32 + kTableEntries,
                                 table32 + kTableEntries + 256))
            return;
    }

    // ---- decode table.  Slot p of the table in code order (p = the next 11 stream bits, first bit
    // most significant) belongs to the code that covers p; codes in canonical order cover
    // consecutive runs of 2^(11-length) slots.  (1) The threads of the chunk rank the 256 code
    // lengths (packed per-length counters, prefix sum over lanes and waves) and every symbol marks
    // the first slot of its run with its table entry.  (2) Every thread takes 2048/threads
    // consecutive slots, extends the marks forward over them, and writes the entries to the table
    // at the bit-reversed slot numbers (the stream is read least significant bit first).
    if (build_table) {
        constexpr int EPT = kTableEntries / TPC; // slots a thread fills
        uint16_t *marks = reinterpret_cast<uint16_t *>(lds_all) + sub * kTableEntries;
        {
            uint4 *z = reinterpret_cast<uint4 *>(marks);
            for (uint32_t i = ct; i < kTableEntries * 2 / 16; i += TPC) z[i] = make_uint4(0, 0, 0, 0);
        }
        // this thread's SPL code lengths, values v = ct*SPL + s (asked for above, with the rest of the header)
        const uint32_t nib = SPL == 1 ? (nib_word >> (4 * (ct & 1))) & 15u : nib_word;
        // counts per length, packed three 10-bit fields a register: length l in reg (l-1)/3
        uint32_t mine[4] = {0, 0, 0, 0};
        uint32_t len_of[SPL];
#pragma unroll
        for (int s = 0; s < SPL; s++) {
            uint32_t l = (nib >> (4 * s)) & 15u;
            if (l > DC_MAX_CODE_LEN) l = 0;
            len_of[s] = l;
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (l != 0 && (l - 1) / 3 == (uint32_t)r) mine[r] += 1u << (10 * ((l - 1) % 3));
        }
        uint32_t before[4], total[4];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const uint32_t incl = lanes_prefix_sum<CPW == 2>(mine[r]);
            before[r] = incl - mine[r];
            if (WAVES > 1) {
                if (lane == 63) lds_counts[wave][r] = incl;
            } else if (CPW == 1) {
                total[r] = __builtin_amdgcn_readlane(incl, 63);
            } else {
                total[r] = __shfl(incl, LPC - 1, LPC);
            }
        }
        __syncthreads();
        if (WAVES > 1) {
#pragma unroll
            for (int r = 0; r < 4; r++) {
                total[r] = 0;
#pragma unroll
                for (int w = 0; w < WAVES; w++) {
                    const uint32_t c = lds_counts[w][r];
                    if ((uint32_t)w < wave) before[r] += c;
                    total[r] += c;
                }
            }
        }
        // left-aligned (11-bit) first code of every length, once per wave and chunk
        uint32_t *first_of = lds_first[wave * CPW + sub];
        if (cl == 0) {
            uint32_t first = 0;
#pragma unroll
            for (int l = 1; l <= DC_MAX_CODE_LEN; l++) {
                first_of[l] = first;
                const uint32_t c = (total[(l - 1) / 3] >> (10 * ((l - 1) % 3))) & 1023u;
                first += c << (kPeekBits - l);
            }
        }
#pragma unroll
        for (int s = 0; s < SPL; s++) {
            const uint32_t l = len_of[s];
            if (l != 0) {
                const uint32_t r = (l - 1) / 3, sh = 10 * ((l - 1) % 3);
                const uint32_t packed = r == 0 ? before[0] : r == 1 ? before[1] : r == 2 ? before[2] : before[3];
                const uint32_t rank = (packed >> sh) & 1023u;
#pragma unroll
                for (int q = 0; q < 4; q++)
                    if (r == (uint32_t)q) before[q] += 1u << sh;
                const uint32_t run = 1u << (kPeekBits - l);
                const uint32_t start = first_of[l] + rank * run;
                const uint16_t entry = (uint16_t)((l - 1) | ((ct * SPL + s) << 8));
                // also at the first slot of every later wave that the run reaches into, so that no
                // wave needs a mark from another wave's slots
                // (marks hold entry + 1, so that 0 means "no mark")
                for (uint32_t p = start; p < start + run && p < (uint32_t)kTableEntries; p += kTableEntries / WAVES)
                    marks[p] = (uint16_t)(entry + 1);
            }
        }
        __syncthreads();
        uint32_t w[EPT / 2];
        {
            const uint4 *m4 = reinterpret_cast<const uint4 *>(marks + EPT * ct);
#pragma unroll
            for (int i = 0; i < EPT / 8; i++) {
                const uint4 v = m4[i];
                w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
            }
        }
        uint32_t tail = 0; // last mark among this thread's slots
#pragma unroll
        for (int i = 0; i < EPT / 2; i++) {
            const uint32_t lo = w[i] & 0xFFFFu, hi = w[i] >> 16;
            tail = lo ? lo : tail;
            tail = hi ? hi : tail;
        }
        uint32_t cur = lanes_last_nonzero_below<CPW == 2>(tail);
        // slot EPT*ct + j in code order = slot bitrev(j) << (11-e) | bitrev(ct) in stream order, EPT = 2^e
        constexpr int E = EPT == 64 ? 6 : EPT == 32 ? 5 : EPT == 16 ? 4 : 3;
        const uint32_t out = lds_address(lds_table[sub]) + 2 * (__brev(ct) >> (32 - (kPeekBits - E)));
#pragma unroll
        for (int i = 0; i < EPT / 2; i++) {
            const uint32_t lo = w[i] & 0xFFFFu, hi = w[i] >> 16;
            cur = lo ? lo : cur;
            *(lds_u16 *)(uintptr_t)(out + 2 * ((__brev((uint32_t)(2 * i)) >> (32 - E)) << (kPeekBits - E))) = (uint16_t)(cur - 1);
            cur = hi ? hi : cur;
            *(lds_u16 *)(uintptr_t)(out + 2 * ((__brev((uint32_t)(2 * i + 1)) >> (32 - E)) << (kPeekBits - E))) = (uint16_t)(cur - 1);
        }
        __syncthreads();
    }

    // ---- sub-stream set-up, second half: the ring is free now
    if (huff) {
        stream_start(st, sf, ring_lane);
        if (CODEC == DC_CODEC_TANS) {
            // the first state: the stream's first 11 bits (at least 40 bits are valid after the set-up)
            st.x4 = ((uint32_t)st.buf & (kTableEntries - 1)) << 2;
            st.buf >>= kPeekBits;
            st.state -= kPeekBits;
        }
    }

    const uint32_t round_bytes = 16 * S;
    const uint32_t full_rounds = raw / round_bytes;
    const uint32_t rem = raw - full_rounds * round_bytes;

    if (MODE == kModeI8) {
        uint8_t *d8 = static_cast<uint8_t *>(a.dst) + dst_pos + ct * 16;
        for (uint32_t r = 0; r < full_rounds; r++) {
            uint32_t w[4];
            decode16<UNI, CODEC>(st, rg, tbl_addr, ring_lane, true, w);
            store16_stream(d8 + (size_t)r * round_bytes, w[0], w[1], w[2], w[3]);
        }
        if (rem) {
            // last, partial round: lanes hold 16, fewer or no symbols; bytes are written one by one
            const uint32_t start = ct * 16;
            const uint32_t n = rem > start ? (rem - start < 16 ? rem - start : 16) : 0;
            uint8_t *d = d8 + (size_t)full_rounds * round_bytes;
            stream_step<UNI, 0>(st, rg, ring_lane);
            for (uint32_t i = 0; i < (n < 8 ? n : 8); i++)
                d[i] = (uint8_t)(CODEC == DC_CODEC_TANS ? tans_decode1(st, tbl_addr, ring_lane) : decode1(st, tbl_addr, ring_lane));
            stream_step<UNI, 1>(st, rg, ring_lane);
            for (uint32_t i = 8; i < n; i++)
                d[i] = (uint8_t)(CODEC == DC_CODEC_TANS ? tans_decode1(st, tbl_addr, ring_lane) : decode1(st, tbl_addr, ring_lane));
        }
        leave_record(DC_TRACE_DECODED);
        return;
    }

    // ---- fused consumers walk the matrix: group position -> (row, column)
    const uint32_t cols = mat.cols;
    const uint32_t rounds = full_rounds + (rem ? 1 : 0);
    uint64_t pos = dst_pos + ct * 16;
    uint32_t row = (uint32_t)(pos / cols);
    uint32_t col = (uint32_t)(pos - (uint64_t)row * cols);

    if (MODE == kModeBf16) {
        // A lane's 16 values become 32 bytes, so two 16-byte stores of its own values would each
        // write half of every 128-byte line.  Lanes l and l + 16 (the same chunk) trade eight bytes
        // first: afterwards the first store of the wave covers the groups of lanes 0-15 and 32-47
        // completely and the second store those of lanes 16-31 and 48-63, whole lines both.
        //   lane l     (bit 4 clear): w0 w1 = its bytes 0-7,          w2 w3 = bytes 0-7 of lane l + 16
        //   lane l + 16             : w0 w1 = bytes 8-15 of lane l,   w2 w3 = its bytes 8-15
        uint16_t *out = static_cast<uint16_t *>(mat.dst);
        const uint32_t upper = (ct >> 4) & 1u;
        const uint32_t ct_a = ct & ~16u, ct_b = ct_a + 16; // the groups the first and the second store belong to
        const uint64_t pos_a = dst_pos + ct_a * 16, pos_b = dst_pos + ct_b * 16;
        uint32_t row_a = (uint32_t)(pos_a / cols), row_b = (uint32_t)(pos_b / cols);
        uint32_t col_a = (uint32_t)(pos_a - (uint64_t)row_a * cols), col_b = (uint32_t)(pos_b - (uint64_t)row_b * cols);
        auto scale_of = [&](uint32_t row) { return mat.row_scale[row < mat.rows ? row : 0]; };
        auto next_round = [&]() {
            col_a += round_bytes;
            while (col_a >= cols) { col_a -= cols; row_a++; }
            col_b += round_bytes;
            while (col_b >= cols) { col_b -= cols; row_b++; }
        };
        // the 16 values of a round, traded between the lanes, scaled and stored (CHECK: groups may be absent)
        auto convert_and_store = [&](const uint32_t w[4], float s_a, float s_b, uint32_t r, bool has_a, bool has_b) {
            // rows of 16 lanes: the odd rows of the first operand change places with the even rows of the second
            const auto x02 = __builtin_amdgcn_permlane16_swap(w[0], w[2], false, false);
            const auto x13 = __builtin_amdgcn_permlane16_swap(w[1], w[3], false, false);
            const uint32_t wa[2] = {x02[0], x13[0]}, wb[2] = {x02[1], x13[1]};
            const uint32_t base = r * round_bytes;
            if (has_a) {
                float f[8];
                word_to_scaled_f32(wa[0], s_a, f);
                word_to_scaled_f32(wa[1], s_a, f + 4);
                store16_stream(out + (pos_a + base + 8 * upper), bf16x2(f[0], f[1]), bf16x2(f[2], f[3]), bf16x2(f[4], f[5]),
                               bf16x2(f[6], f[7]));
            }
            if (has_b) {
                float f[8];
                word_to_scaled_f32(wb[0], s_b, f);
                word_to_scaled_f32(wb[1], s_b, f + 4);
                store16_stream(out + (pos_b + base + 8 * upper), bf16x2(f[0], f[1]), bf16x2(f[2], f[3]), bf16x2(f[4], f[5]),
                               bf16x2(f[6], f[7]));
            }
        };
        if (!huff) {
            // raw chunk: the bytes come straight from the payload
            for (uint32_t r = 0; r < rounds; r++) {
                const uint32_t start = r * round_bytes + ct * 16;
                // the matrix size is a multiple of 16, so a group is whole or absent
                const bool whole = raw >= start + 16;
                const float s_a = scale_of(row_a), s_b = scale_of(row_b);
                uint32_t w[4] = {0, 0, 0, 0};
                if (whole) {
                    const u32x4 v = load16_stream(payload8 + start);
                    w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
                }
                const uint32_t base = r * round_bytes;
                convert_and_store(w, s_a, s_b, r, raw >= base + ct_a * 16 + 16, raw >= base + ct_b * 16 + 16);
                next_round();
            }
            return;
        }
        // Coded chunk.  In the whole rounds every memory access is issued by every lane on every path, in a fixed
        // order (block, block, store, store, scale, scale), so that the wait before a block goes into the ring
        // can count exactly how many younger accesses may stay in flight, the stores among them; the scales of a
        // round are asked for at the end of the round before.
        float s_a = scale_of(row_a), s_b = scale_of(row_b);
        for (uint32_t r = 0; r < full_rounds; r++) {
            uint32_t w[4];
            decode16<UNI, CODEC>(st, rg, tbl_addr, ring_lane, true, w);
            convert_and_store(w, s_a, s_b, r, true, true);
            next_round();
            s_a = scale_of(row_a);
            s_b = scale_of(row_b);
        }
        if (rem) {
            const uint32_t base = full_rounds * round_bytes;
            uint32_t w[4] = {0, 0, 0, 0};
            decode16<UNI, CODEC>(st, rg, tbl_addr, ring_lane, raw >= base + ct * 16 + 16, w);
            convert_and_store(w, s_a, s_b, full_rounds, raw >= base + ct_a * 16 + 16, raw >= base + ct_b * 16 + 16);
        }
        return;
    }

    if (MODE == kModeGemv || MODE == kModeGemvAtomic) {
        // Partial dot products of the int8 values with x; the row scale is applied once per row by the finish
        // kernel.  A lane keeps the sum of its groups of one row; when some lane of the wave moves to another
        // row, the wave sums its lanes by row.  kModeGemvAtomic: one atomic on y per row the wave holds.
        // kModeGemv: the sum of the r-th row the chunk touches goes to lane r of the wave (of the chunk's half
        // of it when S = 32), which keeps the wave's total for that row; at the end the waves' totals are
        // added in wave order through LDS and the chunk leaves one sum per row in the workspace.  Every
        // addition then has a fixed place in a fixed order, so the result is the same bits at every run.
        const uint32_t first_row = (uint32_t)(dst_pos / cols);
        float mine = 0.0f; // kModeGemv: this wave's sum for row first_row + cl
        uint32_t cur_row = 0xFFFFFFFFu;
        float acc = 0.0f;
        auto flush = [&]() {
            const uint32_t key = cur_row < mat.rows ? cur_row : 0xFFFFFFFFu;
            if (MODE == kModeGemvAtomic) lanes_add_by_key<CPW == 2, float>(mat.y_accum, key, acc);
            else lanes_add_runs_to_slots<CPW == 2>(mine, key, (cur_row - first_row) % LPC + sub * LPC, acc);
            acc = 0.0f;
            cur_row = 0xFFFFFFFFu;
        };
        for (uint32_t r = 0; r < rounds; r++) {
            const uint32_t start = r * round_bytes + ct * 16;
            const bool whole = raw >= start + 16;
            uint32_t w[4] = {0, 0, 0, 0};
            if (huff) {
                decode16<UNI, CODEC>(st, rg, tbl_addr, ring_lane, whole, w);
            } else if (whole) {
                const u32x4 v = load16_stream(payload8 + start);
                w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
            }
            if (__any(whole && row != cur_row && cur_row != 0xFFFFFFFFu)) flush();
            if (whole) {
                cur_row = row;
                const uint4 *xp = reinterpret_cast<const uint4 *>(mat.x_bf16 + col);
                const uint4 xa = xp[0], xb = xp[1];
                const uint32_t xs[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    // an int8 value is a bf16 value exactly: two of them packed, times two values of x as they lie in
                    // memory, in one instruction (products exact in fp32, summed in fp32)
                    acc = dot2_bf16(bf16x2(byte_f32<0>(w[i]), byte_f32<1>(w[i])), xs[2 * i], acc);
                    acc = dot2_bf16(bf16x2(byte_f32<2>(w[i]), byte_f32<3>(w[i])), xs[2 * i + 1], acc);
                }
            }
            col += round_bytes;
            while (col >= cols) { col -= cols; row++; }
        }
        flush();
        if (MODE == kModeGemv) {
            float total = mine;
            if (WAVES > 1) {
                // a wave's ring is its own, and the wave has read the last of it: the totals go there
                lds_all[wave * (kRingWords * 64) + lane] = __float_as_uint(mine);
                __syncthreads();
                if (wave == 0) {
                    total = 0.0f;
#pragma unroll
                    for (int v = 0; v < WAVES; v++) total += __uint_as_float(lds_all[v * (kRingWords * 64) + lane]);
                }
            }
            const uint32_t last_row = (uint32_t)((dst_pos + raw - 1) / cols);
            if (wave == 0 && cl <= last_row - first_row) a.partial[k * kPartialSlots + cl] = total;
        }
    }

    if (MODE == kModeGemvW8A8) {
        // The same walk with int8 activations (Eq. 4 of the paper): four v_dot4 per group, exact int32
        // sums, integer atomics, so the result does not depend on the order of the additions.
        int32_t *y_sum = reinterpret_cast<int32_t *>(mat.y_accum);
        uint32_t cur_row = 0xFFFFFFFFu;
        int32_t acc = 0;
        for (uint32_t r = 0; r < rounds; r++) {
            const uint32_t start = r * round_bytes + ct * 16;
            const bool whole = raw >= start + 16;
            uint32_t w[4] = {0, 0, 0, 0};
            if (huff) {
                decode16<UNI, CODEC>(st, rg, tbl_addr, ring_lane, whole, w);
            } else if (whole) {
                const u32x4 v = load16_stream(payload8 + start);
                w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
            }
            if (__any(whole && row != cur_row && cur_row != 0xFFFFFFFFu)) {
                lanes_add_by_key<CPW == 2, int32_t>(y_sum, cur_row < mat.rows ? cur_row : 0xFFFFFFFFu, acc);
                acc = 0;
                cur_row = 0xFFFFFFFFu;
            }
            if (whole) {
                cur_row = row;
                const uint4 x = *reinterpret_cast<const uint4 *>(mat.x_i8 + col);
                acc = __builtin_amdgcn_sdot4((int)w[0], (int)x.x, acc, false);
                acc = __builtin_amdgcn_sdot4((int)w[1], (int)x.y, acc, false);
                acc = __builtin_amdgcn_sdot4((int)w[2], (int)x.z, acc, false);
                acc = __builtin_amdgcn_sdot4((int)w[3], (int)x.w, acc, false);
            }
            col += round_bytes;
            while (col >= cols) { col -= cols; row++; }
        }
        lanes_add_by_key<CPW == 2, int32_t>(y_sum, cur_row < mat.rows ? cur_row : 0xFFFFFFFFu, acc);
    }
}

// Blocks of 256 rows of the matrices of a fused GEMV call, matrix after matrix.
struct RowBlocks {
    uint32_t n_mats;
    uint32_t chunk_bytes;
    const float *partial; // the ordered product: kPartialSlots sums per chunk
    uint32_t first_block[DC_MAX_MATRICES + 1];
    MatrixArgs mats[DC_MAX_MATRICES];
};

__global__ __launch_bounds__(256) void dc_gemv_zero_kernel(RowBlocks rb)
{
    uint32_t mi = 0;
    for (uint32_t i = 1; i < rb.n_mats; i++)
        if (blockIdx.x >= rb.first_block[i]) mi = i;
    const uint32_t i = (blockIdx.x - rb.first_block[mi]) * 256 + threadIdx.x;
    if (i < rb.mats[mi].rows) rb.mats[mi].y_accum[i] = 0.0f;
}

// y_i = scale_i * acc_i; W8A8: y_i = (float(sum_i) * scale_i) * x_scale, each step rounded once, in this order
template <bool W8A8> __global__ __launch_bounds__(256) void dc_gemv_finish_kernel(RowBlocks rb)
{
    uint32_t mi = 0;
    for (uint32_t i = 1; i < rb.n_mats; i++)
        if (blockIdx.x >= rb.first_block[i]) mi = i;
    const MatrixArgs &m = rb.mats[mi];
    const uint32_t i = (blockIdx.x - rb.first_block[mi]) * 256 + threadIdx.x;
    if (i < m.rows) {
        float y;
        if (W8A8) y = ((float)reinterpret_cast<const int32_t *>(m.y_accum)[i] * m.row_scale[i]) * m.x_scale;
        else y = m.row_scale[i] * m.y_accum[i];
        m.y_accum[i] = y;
        if (m.y_bf16) m.y_bf16[i] = (uint16_t)(bf16x2(y, 0.0f) & 0xFFFFu);
    }
}

// The ordered product: y_i = scale_i * (sum over the chunks that hold a part of row i, in chunk order, of the
// chunk's sum for the row).  Chunk c of a matrix holds bytes [c*C, c*C + C) of it and keeps the sum of the r-th
// row it touches, row (c*C) div cols + r, in slot r.
__global__ __launch_bounds__(256) void dc_gemv_ordered_finish_kernel(RowBlocks rb)
{
    uint32_t mi = 0;
    for (uint32_t i = 1; i < rb.n_mats; i++)
        if (blockIdx.x >= rb.first_block[i]) mi = i;
    const MatrixArgs &m = rb.mats[mi];
    const uint32_t i = (blockIdx.x - rb.first_block[mi]) * 256 + threadIdx.x;
    if (i < m.rows) {
        const uint64_t C = rb.chunk_bytes;
        const uint64_t begin = (uint64_t)i * m.cols, last = begin + m.cols - 1;
        float sum = 0.0f;
        for (uint64_t c = begin / C; c <= last / C; c++) {
            const uint64_t first_row = c * C / m.cols;
            sum += rb.partial[(m.first_chunk + c) * kPartialSlots + (i - first_row)];
        }
        const float y = m.row_scale[i] * sum;
        m.y_accum[i] = y;
        if (m.y_bf16) m.y_bf16[i] = (uint16_t)(bf16x2(y, 0.0f) & 0xFFFFu);
    }
}

// Batch-1 product on weights that are already decoded: y_i = scale_i * sum_j q_ij x_j, q int8 row-major.
// A workgroup owns kGemvRows consecutive rows; its 256 threads walk the columns 16 bytes a thread
// (4 KiB a workgroup and row), so that x is converted once for all the rows; a weight costs one
// conversion (sign-extending byte select) and one fused multiply-add.
constexpr int kGemvRows = 4;
__global__ __launch_bounds__(256) void dc_gemv_i8_kernel(const uint8_t *__restrict__ q, const float *__restrict__ row_scale,
                                                         uint32_t rows, uint32_t cols, const uint16_t *__restrict__ x_bf16,
                                                         float *__restrict__ y_f32, uint16_t *__restrict__ y_bf16)
{
    __shared__ float part[4][kGemvRows];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t row0 = blockIdx.x * kGemvRows;
    const uint8_t *qr[kGemvRows];
#pragma unroll
    for (int r = 0; r < kGemvRows; r++) {
        const uint32_t row = row0 + r < rows ? row0 + r : rows - 1; // rows past the end repeat the last one
        qr[r] = q + (size_t)row * cols;
    }
    float acc[kGemvRows] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (uint32_t c = threadIdx.x * 16; c < cols; c += 4096) {
        u32x4 w[kGemvRows];
#pragma unroll
        for (int r = 0; r < kGemvRows; r++) w[r] = load16_stream(qr[r] + c);
        const uint4 *xp = reinterpret_cast<const uint4 *>(x_bf16 + c);
        const uint4 xa = xp[0], xb = xp[1];
        const uint32_t xs[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
        float xf[16];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            xf[2 * i] = bf16_bits_to_f32(xs[i] & 0xFFFFu);
            xf[2 * i + 1] = __uint_as_float(xs[i] & 0xFFFF0000u);
        }
#pragma unroll
        for (int r = 0; r < kGemvRows; r++) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                acc[r] = __builtin_fmaf(byte_f32<0>(w[r][i]), xf[4 * i], acc[r]);
                acc[r] = __builtin_fmaf(byte_f32<1>(w[r][i]), xf[4 * i + 1], acc[r]);
                acc[r] = __builtin_fmaf(byte_f32<2>(w[r][i]), xf[4 * i + 2], acc[r]);
                acc[r] = __builtin_fmaf(byte_f32<3>(w[r][i]), xf[4 * i + 3], acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kGemvRows; r++) acc[r] = lanes_sum(acc[r]);
    if (lane == 63) {
#pragma unroll
        for (int r = 0; r < kGemvRows; r++) part[wave][r] = acc[r];
    }
    __syncthreads();
    if (threadIdx.x < kGemvRows && row0 + threadIdx.x < rows) {
        const uint32_t r = threadIdx.x;
        const float total = part[0][r] + part[1][r] + part[2][r] + part[3][r];
        const float y = row_scale[row0 + r] * total;
        y_f32[row0 + r] = y;
        if (y_bf16) y_bf16[row0 + r] = (uint16_t)(bf16x2(y, 0.0f) & 0xFFFFu);
    }
}

// The same product with int8 activations (Eq. 4): y_i = (float(sum_j q_ij xq_j) * scale_i) * x_scale.
// Same decomposition; four v_dot4 per 16 weights, exact int32 sums.
__global__ __launch_bounds__(256) void dc_gemv_w8a8_kernel(const uint8_t *__restrict__ q, const float *__restrict__ row_scale,
                                                           uint32_t rows, uint32_t cols, const int8_t *__restrict__ x_i8,
                                                           float x_scale, float *__restrict__ y_f32,
                                                           uint16_t *__restrict__ y_bf16)
{
    __shared__ int32_t part[4][kGemvRows];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t row0 = blockIdx.x * kGemvRows;
    const uint8_t *qr[kGemvRows];
#pragma unroll
    for (int r = 0; r < kGemvRows; r++) {
        const uint32_t row = row0 + r < rows ? row0 + r : rows - 1; // rows past the end repeat the last one
        qr[r] = q + (size_t)row * cols;
    }
    int32_t acc[kGemvRows] = {0, 0, 0, 0};
    for (uint32_t c = threadIdx.x * 16; c < cols; c += 4096) {
        u32x4 w[kGemvRows];
#pragma unroll
        for (int r = 0; r < kGemvRows; r++) w[r] = load16_stream(qr[r] + c);
        const uint4 x = *reinterpret_cast<const uint4 *>(x_i8 + c);
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int r = 0; r < kGemvRows; r++)
#pragma unroll
            for (int i = 0; i < 4; i++) acc[r] = __builtin_amdgcn_sdot4((int)w[r][i], (int)xs[i], acc[r], false);
    }
#pragma unroll
    for (int r = 0; r < kGemvRows; r++)
        acc[r] = __builtin_bit_cast(int32_t, lanes_prefix_sum<false>(__builtin_bit_cast(uint32_t, acc[r]))); // total in lane 63
    if (lane == 63) {
#pragma unroll
        for (int r = 0; r < kGemvRows; r++) part[wave][r] = acc[r];
    }
    __syncthreads();
    if (threadIdx.x < kGemvRows && row0 + threadIdx.x < rows) {
        const uint32_t r = threadIdx.x;
        const int32_t total = part[0][r] + part[1][r] + part[2][r] + part[3][r];
        const float y = ((float)total * row_scale[row0 + r]) * x_scale;
        y_f32[row0 + r] = y;
        if (y_bf16) y_bf16[row0 + r] = (uint16_t)(bf16x2(y, 0.0f) & 0xFFFFu);
    }
}

__global__ __launch_bounds__(256) void dc_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, uint64_t n16)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

thread_local hipError_t g_last_hip_error = hipSuccess;

int launch_status() { return dc_launch_status(); }

// Kernel arguments every decode launch shares; the trailer is what a blob of these parameters ends with.
void common_args(DecodeArgs &a, const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev, uint64_t n_chunks,
                 const dc_params *p)
{
    a.blob = blob_dev;
    a.blob_bytes = blob_bytes;
    a.table = table_dev;
    a.n_chunks = n_chunks;
    a.chunk_bytes = p->chunk_bytes;
    a.trailer[0] = DC_TRAILER_MAGIC;
    a.trailer[1] = DC_FORMAT_ID | (uint32_t)DC_LOOKAHEAD_BITS << 16;
    a.trailer[2] = p->chunk_bytes;
    a.trailer[3] = p->n_streams | p->codec << 16;
}

bool decode_params_ok(const dc_params *p)
{
    if (!p) return false;
    if (p->chunk_bytes < 16 || p->chunk_bytes > DC_MAX_CHUNK_BYTES || p->chunk_bytes % 16) return false;
    if (p->codec == DC_CODEC_TANS) return p->n_streams == 64 || p->n_streams == 128 || p->n_streams == 256;
    if (p->codec != DC_CODEC_HUFFMAN) return false;
    return p->n_streams == 32 || p->n_streams == 64 || p->n_streams == 128 || p->n_streams == 256;
}

template <int S, int MODE> void launch_one(const DecodeArgs &a, hipStream_t stream)
{
    using G = Geometry<S>;
    const uint32_t grid = (uint32_t)((a.n_chunks + G::kChunksPerWave - 1) / G::kChunksPerWave);
    hipLaunchKernelGGL((dc_decode_kernel<S, MODE, DC_CODEC_HUFFMAN>), dim3(grid), dim3(G::kThreads), 0, stream, a);
}

// tANS payloads: S >= 64, one chunk per workgroup
template <int MODE> int launch_tans(const DecodeArgs &a, uint32_t S, hipStream_t stream)
{
    if (a.n_chunks > 0x7FFFFFFFull) return DC_E_ARG;
    const uint32_t grid = (uint32_t)a.n_chunks;
    switch (S) {
    case 64: hipLaunchKernelGGL((dc_decode_kernel<64, MODE, DC_CODEC_TANS>), dim3(grid), dim3(64), 0, stream, a); break;
    case 128: hipLaunchKernelGGL((dc_decode_kernel<128, MODE, DC_CODEC_TANS>), dim3(grid), dim3(128), 0, stream, a); break;
    case 256: hipLaunchKernelGGL((dc_decode_kernel<256, MODE, DC_CODEC_TANS>), dim3(grid), dim3(256), 0, stream, a); break;
    default: return DC_E_ARG;
    }
    return launch_status();
}

template <int MODE> int launch_decode(const DecodeArgs &a, uint32_t S, hipStream_t stream, uint32_t codec = DC_CODEC_HUFFMAN)
{
    if (codec == DC_CODEC_TANS) return launch_tans<MODE>(a, S, stream);
    if (a.n_chunks > 0x7FFFFFFFull) return DC_E_ARG;
    switch (S) {
    case 32: launch_one<32, MODE>(a, stream); break;
    case 64: launch_one<64, MODE>(a, stream); break;
    case 128: launch_one<128, MODE>(a, stream); break;
    case 256: launch_one<256, MODE>(a, stream); break;
    default: return DC_E_ARG;
    }
    return launch_status();
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

} // namespace

int dc_launch_status()
{
    g_last_hip_error = hipGetLastError();
    return g_last_hip_error == hipSuccess ? DC_OK : DC_E_HIP;
}


extern "C" int dc_decompress_chunks(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                    uint64_t n_chunks, const dc_params *params, int8_t *dst_dev, uint64_t dst_cap,
                                    void *hip_stream)
{
    if (!decode_params_ok(params) || !blob_dev || !table_dev || !dst_dev || n_chunks == 0 ||
        blob_bytes < DC_BLOB_TAIL_BYTES || blob_bytes % 16)
        return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) return DC_E_FORMAT;
    if (!aligned16(blob_dev) || !aligned16(dst_dev) || (reinterpret_cast<uintptr_t>(table_dev) & 7u)) return DC_E_ARG;
    if (dst_cap < (n_chunks - 1) * (uint64_t)params->chunk_bytes + 1) return DC_E_CAP;
    DecodeArgs a = {};
    common_args(a, blob_dev, blob_bytes, table_dev, n_chunks, params);
    a.dst = dst_dev;
    a.dst_cap = dst_cap;
    return launch_decode<kModeI8>(a, params->n_streams, static_cast<hipStream_t>(hip_stream), params->codec);
}

extern "C" int dc_decompress_chunks_traced(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                           uint64_t n_chunks, const dc_params *params, int8_t *dst_dev, uint64_t dst_cap,
                                           uint64_t *trace_dev, void *hip_stream)
{
    if (!decode_params_ok(params) || !blob_dev || !table_dev || !dst_dev || !trace_dev || n_chunks == 0 ||
        n_chunks > 0x7FFFFFFFull || blob_bytes < DC_BLOB_TAIL_BYTES || blob_bytes % 16)
        return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) return DC_E_FORMAT;
    if (params->codec != DC_CODEC_HUFFMAN || params->n_streams != 256) return DC_E_ARG;
    if (!aligned16(blob_dev) || !aligned16(dst_dev) || (reinterpret_cast<uintptr_t>(table_dev) & 7u) ||
        (reinterpret_cast<uintptr_t>(trace_dev) & 7u))
        return DC_E_ARG;
    if (dst_cap < (n_chunks - 1) * (uint64_t)params->chunk_bytes + 1) return DC_E_CAP;
    DecodeArgs a = {};
    common_args(a, blob_dev, blob_bytes, table_dev, n_chunks, params);
    a.dst = dst_dev;
    a.dst_cap = dst_cap;
    a.trace = trace_dev;
    hipLaunchKernelGGL((dc_decode_kernel<256, kModeI8, DC_CODEC_HUFFMAN, true>), dim3((uint32_t)n_chunks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), a);
    return launch_status();
}

namespace {

// Host checks shared by the fused calls, and the kernel arguments built from the matrix list.
int fused_args(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev, uint64_t n_chunks,
               const dc_params *params, const dc_matrix *mats, uint32_t n_mats, int mode, DecodeArgs &a)
{
    if (!decode_params_ok(params) || !blob_dev || !table_dev || !mats || n_mats == 0 || n_mats > DC_MAX_MATRICES ||
        n_chunks == 0 || blob_bytes < DC_BLOB_TAIL_BYTES || blob_bytes % 16)
        return DC_E_ARG;
    if (params->format != DC_FORMAT_ID) return DC_E_FORMAT;
    if (!aligned16(blob_dev) || (reinterpret_cast<uintptr_t>(table_dev) & 7u)) return DC_E_ARG;
    a = DecodeArgs{};
    common_args(a, blob_dev, blob_bytes, table_dev, n_chunks, params);
    a.n_mats = n_mats;
    uint64_t next_chunk = 0;
    for (uint32_t i = 0; i < n_mats; i++) {
        const dc_matrix &m = mats[i];
        if (m.rows == 0 || m.cols == 0 || m.cols % 16 || !m.row_scale_dev) return DC_E_ARG;
        const bool gemv = mode != kModeBf16;
        if (mode == kModeGemv) {
            if (!m.x_bf16_dev || !m.y_accum_dev || m.cols > 16384 || !aligned16(m.x_bf16_dev)) return DC_E_ARG;
        } else if (mode == kModeGemvW8A8) {
            if (!m.x_i8_dev || !m.y_accum_dev || m.cols > 16384 || !aligned16(m.x_i8_dev)) return DC_E_ARG;
        } else {
            if (!m.dst_bf16_dev || !aligned16(m.dst_bf16_dev)) return DC_E_ARG;
        }
        const uint64_t total = (uint64_t)m.rows * m.cols;
        if (!gemv && m.dst_cap_elems < total) return DC_E_CAP;
        // the matrices follow each other in the table, each starting at a chunk of its own
        if (m.first_chunk != next_chunk) return DC_E_ARG;
        next_chunk += (total + params->chunk_bytes - 1) / params->chunk_bytes;
        MatrixArgs &k = a.mats[i];
        k.first_chunk = m.first_chunk;
        k.rows = m.rows;
        k.cols = m.cols;
        k.row_scale = m.row_scale_dev;
        k.dst = m.dst_bf16_dev;
        k.x_bf16 = m.x_bf16_dev;
        k.y_accum = m.y_accum_dev;
        k.y_bf16 = m.y_bf16_dev;
        k.x_i8 = m.x_i8_dev;
        k.x_scale = m.x_scale;
    }
    if (next_chunk != n_chunks) return DC_E_ARG;
    return DC_OK;
}

} // namespace

extern "C" int dc_decompress_dequant_bf16_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                                uint64_t n_chunks, const dc_params *params, const dc_matrix *mats_host,
                                                uint32_t n_mats, void *hip_stream)
{
    DecodeArgs a;
    const int rc = fused_args(blob_dev, blob_bytes, table_dev, n_chunks, params, mats_host, n_mats, kModeBf16, a);
    if (rc != DC_OK) return rc;
    return launch_decode<kModeBf16>(a, params->n_streams, static_cast<hipStream_t>(hip_stream), params->codec);
}

namespace {

// Rows a chunk of chunk_bytes bytes can touch in a matrix with rows of `cols` bytes whose first chunk starts a row.
uint64_t rows_touched_by_a_chunk(uint32_t chunk_bytes, uint32_t cols)
{
    if (chunk_bytes % cols == 0) return chunk_bytes / cols;
    return (chunk_bytes + cols - 1) / cols + 1;
}

// zero y, decode with the product fused in, scale y: three launches
template <int MODE>
int gemv_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev, uint64_t n_chunks,
               const dc_params *params, const dc_matrix *mats_host, uint32_t n_mats, void *workspace_dev,
               uint64_t workspace_bytes, void *hip_stream)
{
    DecodeArgs a;
    int rc = fused_args(blob_dev, blob_bytes, table_dev, n_chunks, params, mats_host, n_mats, MODE, a);
    if (rc != DC_OK) return rc;
    RowBlocks rb = {};
    rb.n_mats = n_mats;
    rb.chunk_bytes = params->chunk_bytes;
    bool ordered = MODE == kModeGemv;
    for (uint32_t i = 0; i < n_mats; i++) {
        rb.mats[i] = a.mats[i];
        rb.first_block[i + 1] = rb.first_block[i] + (a.mats[i].rows + 255) / 256;
        // the ordered product keeps a row's sum in the lane of the row's number inside the chunk
        if (rows_touched_by_a_chunk(params->chunk_bytes, a.mats[i].cols) > (params->n_streams < 64 ? params->n_streams : 64))
            ordered = false;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (ordered) {
        // decode leaves one sum per chunk and row in the workspace, the finish kernel adds them in chunk order
        if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 3u)) return DC_E_ARG;
        if (workspace_bytes / (kPartialSlots * sizeof(float)) < n_chunks) return DC_E_CAP;
        a.partial = static_cast<float *>(workspace_dev);
        rb.partial = a.partial;
        rc = launch_decode<kModeGemv>(a, params->n_streams, stream, params->codec);
        if (rc != DC_OK) return rc;
        hipLaunchKernelGGL(dc_gemv_ordered_finish_kernel, dim3(rb.first_block[n_mats]), dim3(256), 0, stream, rb);
        return launch_status();
    }
    hipLaunchKernelGGL(dc_gemv_zero_kernel, dim3(rb.first_block[n_mats]), dim3(256), 0, stream, rb);
    rc = launch_decode<MODE == kModeGemv ? kModeGemvAtomic : MODE>(a, params->n_streams, stream, params->codec);
    if (rc != DC_OK) return rc;
    hipLaunchKernelGGL(dc_gemv_finish_kernel<MODE == kModeGemvW8A8>, dim3(rb.first_block[n_mats]), dim3(256), 0, stream, rb);
    return launch_status();
}

} // namespace

extern "C" int dc_decompress_gemv_workspace(uint64_t n_chunks, uint64_t *workspace_bytes)
{
    if (!workspace_bytes || n_chunks == 0 || n_chunks > 0x7FFFFFFFull) return DC_E_ARG;
    *workspace_bytes = n_chunks * kPartialSlots * sizeof(float);
    return DC_OK;
}

extern "C" int dc_decompress_gemv_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                        uint64_t n_chunks, const dc_params *params, const dc_matrix *mats_host,
                                        uint32_t n_mats, void *workspace_dev, uint64_t workspace_bytes, void *hip_stream)
{
    return gemv_layer<kModeGemv>(blob_dev, blob_bytes, table_dev, n_chunks, params, mats_host, n_mats, workspace_dev,
                                 workspace_bytes, hip_stream);
}

extern "C" int dc_decompress_gemv_w8a8_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                             uint64_t n_chunks, const dc_params *params, const dc_matrix *mats_host,
                                             uint32_t n_mats, void *hip_stream)
{
    return gemv_layer<kModeGemvW8A8>(blob_dev, blob_bytes, table_dev, n_chunks, params, mats_host, n_mats, nullptr, 0,
                                     hip_stream);
}

extern "C" int dc_decompress_gemv_w8a8(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                       uint64_t n_chunks, const dc_params *params, const float *row_scale_dev,
                                       uint32_t rows, uint32_t cols, const int8_t *x_i8_dev, float x_scale,
                                       float *y_accum_dev, uint16_t *y_bf16_dev, void *hip_stream)
{
    dc_matrix m = {};
    m.rows = rows;
    m.cols = cols;
    m.row_scale_dev = row_scale_dev;
    m.x_i8_dev = x_i8_dev;
    m.x_scale = x_scale;
    m.y_accum_dev = y_accum_dev;
    m.y_bf16_dev = y_bf16_dev;
    return dc_decompress_gemv_w8a8_layer(blob_dev, blob_bytes, table_dev, n_chunks, params, &m, 1, hip_stream);
}

extern "C" int dc_decompress_dequant_bf16(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                          uint64_t n_chunks, const dc_params *params, const float *row_scale_dev,
                                          uint32_t rows, uint32_t cols, uint16_t *dst_bf16_dev, uint64_t dst_cap_elems,
                                          void *hip_stream)
{
    dc_matrix m = {};
    m.rows = rows;
    m.cols = cols;
    m.row_scale_dev = row_scale_dev;
    m.dst_bf16_dev = dst_bf16_dev;
    m.dst_cap_elems = dst_cap_elems;
    return dc_decompress_dequant_bf16_layer(blob_dev, blob_bytes, table_dev, n_chunks, params, &m, 1, hip_stream);
}

extern "C" int dc_decompress_gemv(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                  uint64_t n_chunks, const dc_params *params, const float *row_scale_dev, uint32_t rows,
                                  uint32_t cols, const uint16_t *x_bf16_dev, float *y_f32_dev, uint16_t *y_bf16_dev,
                                  void *workspace_dev, uint64_t workspace_bytes, void *hip_stream)
{
    dc_matrix m = {};
    m.rows = rows;
    m.cols = cols;
    m.row_scale_dev = row_scale_dev;
    m.x_bf16_dev = x_bf16_dev;
    m.y_accum_dev = y_f32_dev;
    m.y_bf16_dev = y_bf16_dev;
    return dc_decompress_gemv_layer(blob_dev, blob_bytes, table_dev, n_chunks, params, &m, 1, workspace_dev,
                                    workspace_bytes, hip_stream);
}

extern "C" const char *dc_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

extern "C" int dc_gemv_w8a8(const int8_t *q_dev, const float *row_scale_dev, uint32_t rows, uint32_t cols,
                            const int8_t *x_i8_dev, float x_scale, float *y_f32_dev, uint16_t *y_bf16_dev, void *hip_stream)
{
    if (!q_dev || !row_scale_dev || !x_i8_dev || !y_f32_dev || rows == 0 || cols == 0 || cols % 16 || cols > 16384)
        return DC_E_ARG;
    if (!aligned16(q_dev) || !aligned16(x_i8_dev)) return DC_E_ARG;
    const uint32_t blocks = (rows + kGemvRows - 1) / kGemvRows;
    hipLaunchKernelGGL(dc_gemv_w8a8_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const uint8_t *>(q_dev), row_scale_dev, rows, cols, x_i8_dev, x_scale, y_f32_dev,
                       y_bf16_dev);
    return launch_status();
}

extern "C" int dc_gemv_i8(const int8_t *q_dev, const float *row_scale_dev, uint32_t rows, uint32_t cols,
                          const uint16_t *x_bf16_dev, float *y_f32_dev, uint16_t *y_bf16_dev, void *hip_stream)
{
    if (!q_dev || !row_scale_dev || !x_bf16_dev || !y_f32_dev || rows == 0 || cols == 0 || cols % 16) return DC_E_ARG;
    if (!aligned16(q_dev) || !aligned16(x_bf16_dev)) return DC_E_ARG;
    const uint32_t blocks = (rows + kGemvRows - 1) / kGemvRows;
    hipLaunchKernelGGL(dc_gemv_i8_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const uint8_t *>(q_dev), row_scale_dev, rows, cols, x_bf16_dev, y_f32_dev,
                       y_bf16_dev);
    return launch_status();
}

extern "C" int dc_device_copy(const void *src_dev, void *dst_dev, uint64_t bytes, void *hip_stream)
{
    if (!src_dev || !dst_dev || bytes == 0 || bytes % 16 || !aligned16(src_dev) || !aligned16(dst_dev)) return DC_E_ARG;
    const uint64_t n16 = bytes / 16;
    // one 16-byte element a thread: measured 6.5 TB/s (read + write) on 6.5 GB, where a grid capped at 32
    // workgroups a compute unit that strides over the buffer reads 4.9
    uint64_t blocks = (n16 + 255) / 256;
    if (blocks > 0x7FFFFFFFull) blocks = 0x7FFFFFFFull;
    hipLaunchKernelGGL(dc_copy_kernel, dim3((uint32_t)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4 *>(src_dev), static_cast<u32x4 *>(dst_dev), n16);
    return launch_status();
}
