/*
 * dc.h - C ABI of the MI355X double-compression decode library (libdc_mi355x.so).
 *
 * The library implements the runtime half of the paper's double-compression
 * method (Section 3.1 overview, Section 3.3 "Inference with DC-Compressed
 * LLMs"): INT8-quantised, pruned LLM weights are stored as independently coded
 * chunks in GPU memory and are decompressed by the GPU, for the layer that is
 * about to be used, into a caller-owned decompression buffer; a speed-adaptive
 * share of the chunks is stored raw.  The lossless coder is a per-chunk
 * canonical Huffman code over the 256 byte values (code length <= 11) with S
 * symbol-interleaved sub-bitstreams per chunk, stored block-interleaved; a
 * tabled ANS coder with 2048 states can take its place in the same container
 * (dc_params.codec).  The layout is given below.
 *
 * Conventions for every entry point
 *   - extern "C", plain pointers and sizes.  "_host" pointers are ordinary
 *     host memory, "_dev" pointers are device memory of the current HIP device.
 *   - The caller owns every buffer.  The library allocates no memory the caller
 *     can see and keeps no state between calls (except dc_set_num_threads).
 *   - Return value: DC_OK (0) or a negative DC_E_* code; dc_strerror() names it.
 *   - Device entry points only enqueue work on `hip_stream` (a hipStream_t, NULL
 *     = the default stream) and never synchronise.  Arguments are checked on the
 *     host before anything is enqueued; device memory contents (table, blob) are
 *     not read by the host.  The kernels never read outside
 *     [blob_dev, blob_dev + blob_bytes) nor write outside the destination's
 *     stated capacity whatever the table or the payloads contain; a corrupt
 *     chunk yields unspecified bytes for that chunk only.  dc_validate() is the
 *     host-side checker that reports corruption.
 *
 * Stored format
 *   chunk table entry (dc_chunk, 16 bytes, little endian)
 *       off              payload offset inside the blob, multiple of 16
 *       comp_bytes       payload size including padding, multiple of 16
 *       raw_bytes_flags  bits 0..30 decoded size of the chunk (1..chunk_bytes),
 *                        bit 31 set = payload is the raw bytes (DC_CHUNK_RAW)
 *     chunk k decodes to bytes [k*chunk_bytes, k*chunk_bytes + raw_bytes) of the
 *     destination; only the last chunk may be shorter than chunk_bytes.
 *   blob                 the payloads back to back in chunk order, followed by DC_BLOB_TAIL_BYTES
 *                        closing bytes; blob_bytes counts them.  The closing bytes are 48 zero bytes
 *                        and the 16-byte trailer, which says how the blob is to be read:
 *                          u32 DC_TRAILER_MAGIC ("DCBF")
 *                          u16 DC_FORMAT_ID          u16 DC_LOOKAHEAD_BITS of that format
 *                          u32 chunk_bytes
 *                          u16 n_streams             u16 codec
 *                        Blobs written with the same parameters can be put one after the other
 *                        (table offsets moved accordingly): the last trailer closes the whole.
 *   format id            DC_FORMAT_ID names this text as a whole.  Part of it is not of the method
 *                        but of the decode kernel it was written with, and changes the bytes of a
 *                        coded payload when it changes: DC_LOOKAHEAD_BITS and the five times of step 0
 *                        (how far ahead of its position a stream's blocks are placed: the kernel
 *                        keeps a block in flight for two steps), steps of half a group of 8 symbols
 *                        (the kernel's unit between two refills of its ring), DC_BLOCK_BYTES (one
 *                        128-bit load) and stream sets of 64 (one wavefront).  Earlier formats
 *                        (look-ahead 320, sub-streams padded to whole blocks, no trailer) had none
 *                        of this written into the blob; a blob without the trailer of this format
 *                        is refused, never decoded: dc_validate and every dc_decompress_* call
 *                        return DC_E_FORMAT when params->format is not DC_FORMAT_ID, dc_validate also
 *                        when the trailer in the blob differs from what params say, and the decode
 *                        kernels leave every chunk undecoded then.
 *   raw payload          the bytes, zero padded to a multiple of 16
 *   Huffman payload
 *       [0,128)          4-bit code length of byte value v in nibble (v & 1) of
 *                        byte v >> 1; 0 = value absent, otherwise 1..11
 *       [128,128+2S)     u16 per sub-stream j < S: bits 0..11 nb[j], the number of 16-byte blocks
 *                        of the stream; bits 12..15 hb[j] - 1, where hb[j] = 1..16 is the number
 *                        of bytes of the stream's first block that exist (both fields 0 for a
 *                        stream without symbols)
 *       [128+2S, +4*S/W) u32 set_off[w]: first byte of the area of stream set w, counted
 *                        from the payload start, multiple of 16; then zero padding to a multiple
 *                        of 16.  A stream set is W = min(S, 64) consecutive sub-streams (the
 *                        streams one wavefront decodes): set w = streams [W*w, W*w + W).
 *       sub-streams      the chunk is cut in 16-byte groups; group g belongs to
 *                        sub-stream g mod S; a sub-stream is the concatenated
 *                        codes of its bytes in increasing position, zero padded
 *                        to a whole byte.  It is cut into 16-byte blocks from its
 *                        end: every block is whole except block 0, whose first
 *                        pad[j] = 16 - hb[j] bytes do not exist.  Positions in a
 *                        stream count from where block 0 would start: the first
 *                        code begins at bit 8*pad[j].  No end marker: symbol
 *                        counts follow from raw_bytes.
 *       bit order        stream bit i is bit (i mod 32) of little-endian u32
 *                        word i / 32; a code is written most significant code
 *                        bit first.
 *       set areas        one per stream set, back to back after the header, each a multiple of
 *                        16 bytes.  An area is a block region, then the heads, then zero
 *                        padding.  The heads are the short blocks 0 of the set's streams, in
 *                        ascending stream order, hb[j] bytes each (so a stream costs its bits
 *                        rounded up to a byte, not to 16 bytes; a reader may load the 20 bytes
 *                        from the 4-byte boundary at or before the place where block 0 would
 *                        start and ignore what is not the head: that place lies inside the
 *                        payload, and DC_BLOB_TAIL_BYTES keep the end of the load inside the
 *                        blob).  The region holds every other block
 *                        of the streams, interleaved in the order in which a decoder
 *                        that works through all streams in step asks for them, so that it
 *                        reads the region front to back.  The order is fixed by this rule.
 *                        Decoding goes in steps h = 0, 1, ...; step h comes before symbols
 *                        8*(h mod 2) .. 8*(h mod 2)+7 of group number (h div 2) of every stream.
 *                        Let c[j] be the position of stream j before step h (8*pad[j] plus the
 *                        bits of its symbols so far), and f[j] the blocks of stream j placed so far.  At a
 *                        step, for j ascending over the set: if f[j] < nb[j] and
 *                        128*f[j] - c[j] < DC_LOOKAHEAD_BITS, the stream takes block f[j] and
 *                        f[j] grows by one; block 0 is the stream's head and takes no place in
 *                        the region, any other block is placed next in the region.  Step 0 is
 *                        carried out five times in a row, every later step once.  (Three blocks
 *                        are 384 - 8*pad[j] bits beyond the first position, hence the fourth
 *                        time; the fifth changes nothing in a Huffman payload, where c[j] is
 *                        still 8*pad[j] <= 120 and a fifth block would start 512 bits on; in a
 *                        tANS payload the first state is read before it.
 *                        Half a group uses at most 88 bits, so after every step a stream
 *                        has at least DC_LOOKAHEAD_BITS bits placed beyond its position, or all
 *                        of its blocks; every block is placed by the last step.)
 *       codes            canonical: lengths from package-merge with limit 11
 *                        (leaves ordered by count then byte value, a leaf before
 *                        a package of equal weight); codes numbered in order of
 *                        (length, byte value), first code 0.
 *   tANS payload (params.codec = DC_CODEC_TANS; the paper's Section 4.2 settles on ANS among the entropy
 *   coders): the same container; only the front of the header and what a sub-stream holds differ.
 *       [0,384)          normalised frequency q[v] of byte value v, 12 bits each: bits 12v .. 12v+11 of
 *                        the 384 bytes read as one little-endian bit string; the q add up to L = 2048;
 *                        q[v] = 0 for an absent value
 *       [384,384+2S)     the u16 per sub-stream, then set_off, then padding, as in the Huffman payload
 *       states           place p = 0 .. L-1 in the list of byte values in ascending order, value v taking
 *                        q[v] consecutive places, is state x = p with its 11 bits reversed.  The states of v
 *                        taken in ascending x are numbered k = q[v] .. 2q[v]-1.  A state numbered k has
 *                        nb = 11 - floor(log2 k) and base = (k << nb) - L.
 *       sub-stream       bit fields, least significant bit first.  Decoder: x = the first 11 bits; for every
 *                        symbol: the symbol is the value of state x, then x = base(x) + the next nb(x) bits.
 *                        Encoder: X = L; for the symbols from the last to the first, v being the symbol:
 *                        nb = the smallest n with (X >> n) < 2q[v]; the symbol's field is the low nb bits of
 *                        X; X = L + the state of v numbered X >> nb.  The stream is X - L after the first
 *                        symbol, then the fields in symbol order; the decoder ends in state 0.  A field has
 *                        at most 11 bits, like a code.
 *       placement rule   as above, c[j] counting every bit read; the 11 bits of the first state are read
 *                        after the fourth and before the fifth carrying out of step 0.
 *       frequencies      what the compressor stores, n being the chunk's size: q[v] = max(1,
 *                        floor(count[v]*L/n)) for present values; while the sum is below L, one more for the
 *                        value with the largest count[v]/q[v] (exact fractions; the lower value among equals);
 *                        while it is above L, one less for the value with q[v] > 1 and the smallest
 *                        count[v]/(q[v]-1) (the lower value among equals).
 */
#ifndef DC_MI355X_H
#define DC_MI355X_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DC_OK 0
#define DC_E_ARG (-1)    /* bad argument: null pointer, misalignment, unsupported parameter */
#define DC_E_CAP (-2)    /* an output buffer is too small; required sizes are written back where stated */
#define DC_E_FORMAT (-3) /* the blob is of another format than this library reads (params->format, trailer);
                            dc_validate: table or payload violates the stored format */
#define DC_E_HIP (-4)    /* a HIP runtime call failed (launch error, no device) */

#define DC_CHUNK_RAW 0x80000000u
#define DC_MAX_CODE_LEN 11
#define DC_MAX_CHUNK_BYTES (1u << 20)
#define DC_BLOB_TAIL_BYTES 64
#define DC_BLOCK_BYTES 16
#define DC_LOOKAHEAD_BITS 392
#define DC_FORMAT_ID 5
#define DC_TRAILER_BYTES 16
#define DC_TRAILER_MAGIC 0x46424344u /* the bytes 'D' 'C' 'B' 'F' */
#define DC_MAX_MATRICES 16
#define DC_TANS_STATE_BITS 11

/* the coder of the chunks that are not raw (Section 4.2 of the paper compares entropy coders) */
#define DC_CODEC_HUFFMAN 0 /* canonical Huffman, code length <= 11 */
#define DC_CODEC_TANS 1    /* tabled asymmetric numeral systems, 2048 states; n_streams 64, 128 or 256
                              (DC_E_ARG otherwise); decoded by every dc_decompress_* call, written by
                              dc_compress_chunks and dc_compress_chunks_dev, checked by dc_validate */

/* which chunks are stored raw (Section 3.3, "Speed Adaptive Partial Compression") */
#define DC_POLICY_ALL_HUFF 0     /* every chunk Huffman coded, even if that enlarges it */
#define DC_POLICY_AUTO 1         /* raw where gain = raw_bytes - huffman payload bytes <= 0 */
#define DC_POLICY_RAW_FRACTION 2 /* the floor(raw_fraction*n_chunks + 1/2) chunks of lowest gain stay raw
                                    (equal gains: lower chunk index first) */
#define DC_POLICY_RAW_MASK 3     /* chunk k raw iff raw_mask[k] != 0 */
#define DC_POLICY_BLOCK_LAST 4   /* the paper's rule: blocks of block_chunks consecutive chunks, only the
                                    last chunk of each block is compressed */

typedef struct {
    uint64_t off;
    uint32_t comp_bytes;
    uint32_t raw_bytes_flags;
} dc_chunk;

typedef struct {
    uint32_t chunk_bytes;   /* decoded bytes per chunk: multiple of 16, 16..DC_MAX_CHUNK_BYTES */
    uint32_t n_streams;     /* S: sub-streams per chunk, one of 32, 64, 128, 256 */
    uint32_t policy;        /* DC_POLICY_*; only the compressor reads it */
    float raw_fraction;     /* DC_POLICY_RAW_FRACTION: share of chunks kept raw, 0..1; the count is
                               floor((double)raw_fraction * n_chunks + 0.5) of this 32-bit value */
    uint32_t block_chunks;  /* DC_POLICY_BLOCK_LAST: chunks per block, >= 1 */
    uint32_t codec;         /* DC_CODEC_*: the coder of the chunks that are not raw */
    uint32_t format;        /* id of the stored format of the blob that is written or read: DC_FORMAT_ID;
                               any other value is refused with DC_E_FORMAT */
    const uint8_t *raw_mask; /* DC_POLICY_RAW_MASK: host array of n_chunks bytes, else NULL */
} dc_params;

/* One matrix of a fused whole-layer call (host struct; the pointers inside are device pointers). */
typedef struct {
    uint64_t first_chunk;         /* table index of the matrix's first chunk; the matrices follow each other
                                     in the table, each starting at a chunk of its own (compressed on its own) */
    uint32_t rows, cols;          /* decoded bytes are int8 q[rows][cols]; cols a multiple of 16 */
    const float *row_scale_dev;   /* fp32 scale per row */
    uint16_t *dst_bf16_dev;       /* dequant: bf16 [rows][cols], 16-byte aligned */
    uint64_t dst_cap_elems;       /* dequant: capacity of dst_bf16_dev in elements */
    const uint16_t *x_bf16_dev;   /* gemv: cols bf16 activations, 16-byte aligned; cols <= 16384 */
    float *y_accum_dev;           /* gemv: rows fp32 results */
    uint16_t *y_bf16_dev;         /* gemv: rows bf16 results, may be NULL */
    const int8_t *x_i8_dev;       /* gemv_w8a8: cols int8 activations, 16-byte aligned; cols <= 16384 */
    float x_scale;                /* gemv_w8a8: scale of the activations (activation = x_i8 * x_scale) */
} dc_matrix;

/* Library identification string (static storage). */
const char *dc_version(void);
/* Name of a DC_E_* code (static storage). */
const char *dc_strerror(int code);
/* Text of the HIP status behind the calling thread's most recent DC_E_HIP (static storage). */
const char *dc_last_hip_error(void);
/* Host worker threads used by dc_quantize_rows / dc_compress_chunks / dc_validate; 0 = all cores.
 * Returns the previous setting. */
int dc_set_num_threads(int n);

/*
 * Compression-aware quantisation (Section 3.2; Eqs. 1, 2, 4 and the pruning step around Eq. 5).
 *   w_host            fp32 W[rows][cols], row-major, cols = input channels
 *   act_absmax_host   fp32 max|X_j| per input channel (cols values), or NULL for no rescale
 *   alpha             exponent of Eq. 2: s_j = act_absmax_j ^ alpha (evaluated in fp64, rounded to fp32)
 *   prune_abs         quantised weights with |q| <= prune_abs become 0 (0 = no pruning)
 *   q_host            out: int8 q[rows][cols]
 *   row_scale_host    out: fp32 scale per row; dequantised weight = q * row_scale
 *   col_scale_host    out, may be NULL: the s_j that were applied (activations must be divided by them)
 * Per row i: W' = W * s (fp32), m = max_j |W'_ij|, scale_i = m / 127 (fp32 division; 1 if m == 0),
 * q_ij = clamp(round-half-even(W'_ij / scale_i), -127, 127).
 * Errors: DC_E_ARG for null pointers or zero sizes.
 */
int dc_quantize_rows(const float *w_host, uint32_t rows, uint32_t cols, const float *act_absmax_host,
                     double alpha, uint32_t prune_abs, int8_t *q_host, float *row_scale_host,
                     float *col_scale_host);

/*
 * The paper's own form of the compression stage (Section 3.2; Section 4.5 "scaled-tensor"): one
 * scale for the whole tensor, and pruning by the importance score of Eq. 5.
 *   W' = W * s with s_j = act_absmax_j ^ alpha (fp32 product; s = 1 when act_absmax_host is NULL),
 *   m = max |W'_ij| over the tensor, scale = m / 127 (fp32; 1 if m == 0),
 *   q_ij = clamp(round-half-even(W'_ij / scale), -127, 127),
 *   score_ij = act_absmax_j * |q_ij| (evaluated in fp64; |q_ij| alone when act_absmax_host is NULL),
 *   k = floor(sparsity * rows * cols); if k > 0 every q_ij whose score is <= the k-th smallest score
 *   becomes 0 (scores equal to the threshold are pruned together).
 *   tensor_scale_host  out: the one fp32 scale; dequantised weight = q * scale
 *   col_scale_host     out, may be NULL: the s_j that were applied
 * Errors: DC_E_ARG for null pointers, zero sizes, sparsity outside [0, 1).
 */
int dc_quantize_tensor(const float *w_host, uint32_t rows, uint32_t cols, const float *act_absmax_host,
                       double alpha, double sparsity, int8_t *q_host, float *tensor_scale_host,
                       float *col_scale_host);

/*
 * Worst-case blob size and number of chunks for raw_bytes input bytes (Section 3.3: the weight
 * data is divided into data chunks).  Either output pointer may be NULL.
 */
int dc_compress_bound(uint64_t raw_bytes, const dc_params *params, uint64_t *max_blob_bytes,
                      uint64_t *n_chunks);

/*
 * Lossless compression of the quantised, pruned weights into a binary blob (last step of the
 * compression stage, Section 3.1; chunk selection per Section 3.3).  Host to host.
 *   src_host    raw_bytes int8 values (a row-major matrix or any byte string)
 *   blob_host   out: payloads back to back in chunk order, blob_cap bytes available
 *   blob_bytes  out: bytes used (on DC_E_CAP: bytes required)
 *   table_host  out: one dc_chunk per chunk, table_cap entries available
 *   n_chunks    out: entries used (on DC_E_CAP: entries required)
 * The result is a function of the input and params alone (not of the thread count).
 * params->codec chooses the coder of the chunks that are not raw; "Huffman" in the names of the
 * policies then reads "coded".
 */
int dc_compress_chunks(const int8_t *src_host, uint64_t raw_bytes, const dc_params *params,
                       uint8_t *blob_host, uint64_t blob_cap, uint64_t *blob_bytes, dc_chunk *table_host,
                       uint64_t table_cap, uint64_t *n_chunks);

/*
 * The same compression on the GPU (Section 3.1; Section 4.2 reports compression speed as well).
 * Device to device, asynchronous on hip_stream, three launches.  The blob and table are byte for
 * byte those of dc_compress_chunks for the same input and params.  Policies: DC_POLICY_ALL_HUFF,
 * DC_POLICY_AUTO, DC_POLICY_RAW_FRACTION, DC_POLICY_BLOCK_LAST (DC_POLICY_RAW_MASK names a mask in
 * host memory: DC_E_ARG).
 *   src_dev         raw_bytes int8 values, 16-byte aligned
 *   blob_dev        out, 16-byte aligned, blob_cap bytes (dc_compress_bound gives a safe size)
 *   table_dev       out, table_cap >= number of chunks entries
 *   workspace_dev   scratch of at least dc_compress_chunks_dev_workspace() bytes, 16-byte aligned,
 *                   owned by the caller; may be reused once the call's work on the stream is done
 *                   (about 260 + 4 n_streams bytes per chunk; with DC_CODEC_TANS two more bytes per
 *                   input byte, because a tANS sub-stream is coded from its end and written from its
 *                   start)
 *   result_dev      out, two u64 in device memory: [0] = blob bytes (needed, when [1] != 0),
 *                   [1] = 0, or DC_E_CAP as a 64-bit value when blob_cap was too small (then the
 *                   blob is incomplete, the table is still written)
 * Errors on the host: DC_E_ARG (null or misaligned pointers, unsupported policy or sizes), DC_E_CAP
 * (workspace or table too small), DC_E_HIP.
 */
int dc_compress_chunks_dev_workspace(uint64_t raw_bytes, const dc_params *params, uint64_t *workspace_bytes);
int dc_compress_chunks_dev(const int8_t *src_dev, uint64_t raw_bytes, const dc_params *params,
                           uint8_t *blob_dev, uint64_t blob_cap, dc_chunk *table_dev, uint64_t table_cap,
                           void *workspace_dev, uint64_t workspace_bytes, uint64_t *result_dev,
                           void *hip_stream);

/*
 * dc_compress_chunks_dev for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc): the workspace is a fixed array of
 * DC_STATIC_SCRATCH_BYTES in device memory that belongs to the library (one per GPU, held until the
 * process ends), and the call allocates nothing.  Same arguments, results and errors as
 * dc_compress_chunks_dev without the workspace; an input whose workspace
 * (dc_compress_chunks_dev_workspace) exceeds DC_STATIC_SCRATCH_BYTES is refused with DC_E_CAP before
 * anything is enqueued (with the default coder and n_streams = 256 the array serves about 13 000 chunks,
 * 850 MB of weights in 64 KiB chunks; with DC_CODEC_TANS about 8 MB of input).  Every call on a GPU
 * uses that GPU's one array: calls whose work overlaps on the same GPU (two streams, two threads) race
 * and must be serialised by the caller.  Nothing in the array has to be cleared between calls.
 */
#define DC_STATIC_SCRATCH_BYTES (16u << 20)
int dc_compress_chunks_dev_static(const int8_t *src_dev, uint64_t raw_bytes, const dc_params *params,
                                  uint8_t *blob_dev, uint64_t blob_cap, dc_chunk *table_dev, uint64_t table_cap,
                                  uint64_t *result_dev, void *hip_stream);

/*
 * Reads the trailer of a blob (its last DC_TRAILER_BYTES bytes, in host memory) into params_out:
 * format, chunk_bytes, n_streams and codec; the other fields are set to 0.  DC_E_FORMAT when the bytes
 * are not a trailer (no magic number) or name a format this library does not read; DC_E_ARG for null
 * pointers.  For a caller who gets a blob from elsewhere and must know how to decode it.
 */
int dc_blob_trailer(const uint8_t *trailer_host, dc_params *params_out);

/*
 * Host-side check of a table and blob against the stored format: the trailer against params, offsets, sizes, alignment, code
 * lengths forming a complete code (tANS: frequencies adding up to 2048), sub-stream extents, and that
 * every sub-stream holds its symbols (tANS: and ends in state 0).
 * Payloads must lie in the blob in chunk order without overlapping; bytes between them (the closing
 * bytes of blobs that were put one after the other) are not looked at, and the table may be a part of a
 * larger one (a layer of a model).  Returns DC_OK or DC_E_FORMAT (first offending chunk index in
 * *bad_chunk when not NULL; n_chunks when it is the trailer that does not fit params).
 */
int dc_validate(const uint8_t *blob_host, uint64_t blob_bytes, const dc_chunk *table_host,
                uint64_t n_chunks, const dc_params *params, uint64_t *bad_chunk);

/*
 * GPU decompression into the decompression buffer (Section 3.3, "Inference Process" and
 * "Throughput Analysis": compressed chunks resident in GPU memory are decompressed by the GPU into
 * a buffer in GPU memory from which inference reads the weights).  One kernel launch.
 *   blob_dev, blob_bytes   the blob, 16-byte aligned, up to and with its closing bytes (blob_bytes a
 *                          multiple of 16); a launch whose blob does not end in the trailer that params
 *                          describe decodes nothing
 *   table_dev, n_chunks    chunk table in device memory
 *   dst_dev, dst_cap       destination, 16-byte aligned; needs (n_chunks-1)*chunk_bytes + last chunk's
 *                          raw_bytes bytes; the host checks dst_cap >= (n_chunks-1)*chunk_bytes + 1 and
 *                          the kernel skips any chunk that would end beyond dst_cap
 * A part of a blob (a layer of a model, say) is decoded by passing table_dev + k0 and the number of
 * chunks wanted with the same blob: offsets in the table count from blob_dev, and chunk k0 + i then
 * decodes to dst_dev + i * chunk_bytes.
 * params->codec names the coder of the blob's coded chunks; DC_CODEC_TANS needs n_streams >= 64
 * (DC_E_ARG otherwise).  A tANS chunk whose frequencies do not add up to 2048 is left undecoded.
 */
int dc_decompress_chunks(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                         uint64_t n_chunks, const dc_params *params, int8_t *dst_dev, uint64_t dst_cap,
                         void *hip_stream);

/*
 * dc_decompress_chunks with a record of every workgroup of the launch, for whoever wants to see how a launch
 * is laid out in time and over the chip (the tail of a short launch, launches that mix raw and coded chunks); not
 * part of the method.  Same arguments, results and errors as dc_decompress_chunks, Huffman coded blobs of 256
 * sub-streams only (DC_E_ARG otherwise), and
 *   trace_dev   4 * n_chunks 64-bit words of device memory, 8-byte aligned, owned by the caller.  Workgroup b
 *               (= chunk b) writes words 4b .. 4b+3 when it ends: [0] and [1] the readings of the constant 100 MHz
 *               clock (wall_clock64) when it began and when it ended; [2] the wavefront's HW_ID register in the
 *               low 32 bits (compute unit in bits 8-11, shader engine from bit 13) and its XCC_ID register in
 *               the high 32 (the XCD in bits 0-3); [3] one of DC_TRACE_*.
 * The record does not change a launch's duration measurably (74.7 us with it and without it on a layer of 3088 chunks).
 */
#define DC_TRACE_DECODED 0u /* a coded chunk, decoded */
#define DC_TRACE_COPIED 1u  /* a raw chunk, copied */
#define DC_TRACE_SKIPPED 2u /* left alone: the table entry or the blob's trailer did not pass the checks */
int dc_decompress_chunks_traced(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                uint64_t n_chunks, const dc_params *params, int8_t *dst_dev, uint64_t dst_cap,
                                uint64_t *trace_dev, void *hip_stream);

/*
 * How fast a SIMD issues one vector-ALU instruction, for whoever wants to know how close a kernel's instruction mix
 * comes to what the chip issues (the decode kernels are bound by instruction issue and the LDS, not by memory); not
 * part of the method.  dc_issue_rate_count() instructions are known, dc_issue_rate_name(which) is the mnemonic of
 * one (NULL beyond the count); names that begin with ds_ are LDS reads of a 4 KiB table with the named pattern of
 * addresses over the lanes (l), whose time is set by the one LDS that the four SIMDs of a compute unit share.  dc_issue_rate(which, ...) runs a chain of that instruction on values in registers
 * with eight wavefronts resident on every SIMD, twice (the second launch is timed with events on the stream), waits
 * for it, and writes to *ns_per_instruction_host the time from one wavefront instruction to the next on a SIMD.
 *   sink_dev, sink_bytes   at least 1024 bytes of device memory that the kernel may overwrite, owned by the caller
 * Returns DC_OK, DC_E_ARG or DC_E_HIP.  A blocking call; allocates nothing on the device.
 */
uint32_t dc_issue_rate_count(void);
const char *dc_issue_rate_name(uint32_t which);
int dc_issue_rate(uint32_t which, uint32_t *sink_dev, uint64_t sink_bytes, void *hip_stream, double *ns_per_instruction_host);

/*
 * Decompression fused with dequantisation to bf16 (replaces the separate conversion of the
 * decompressed memory into tensors that Section 4.6 counts as overhead; dequantisation inverts Eq. 4):
 *   dst[i*cols + j] = bf16_round_nearest_even( float(q_ij) * row_scale[i] ).
 * The decoded bytes are the row-major int8 matrix q[rows][cols]; rows*cols must equal the decoded
 * size, cols must be a multiple of 16.  dst_cap_elems counts bf16 elements.
 */
int dc_decompress_dequant_bf16(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                               uint64_t n_chunks, const dc_params *params, const float *row_scale_dev,
                               uint32_t rows, uint32_t cols, uint16_t *dst_bf16_dev,
                               uint64_t dst_cap_elems, void *hip_stream);

/*
 * Decompression fused with the batch-1 product of Eq. 1, Y = X' W'^T for one activation row:
 *   y_i = row_scale[i] * sum_j q_ij * x_j,   x given as bf16, accumulated in fp32.
 * Nothing decoded is written to memory.  y_f32_dev (rows fp32 values) receives the result; y_bf16_dev
 * (rows bf16 values, may be NULL) receives it rounded to bf16.  cols must be a multiple of 16 and at
 * most 16384.
 *   workspace_dev, workspace_bytes   scratch of at least dc_decompress_gemv_workspace(n_chunks) bytes
 *                                    (256 per chunk), 4-byte aligned, owned by the caller; its contents
 *                                    before the call do not matter and it may be reused once the call's
 *                                    work on the stream is done
 * Two launches: the decode kernel leaves in the workspace one partial sum per chunk and row the chunk
 * touches, added up inside the chunk in a fixed order, and a second kernel adds a row's partial sums in
 * chunk order and scales them.  No atomic operation is involved, so a call returns the same bits every
 * time it runs on the same input.  That holds while a chunk touches at most min(n_streams, 64) rows
 * (chunk_bytes / cols rows if cols divides chunk_bytes, else ceil(chunk_bytes / cols) + 1); for
 * flatter matrices the call falls back to three launches that add with fp32 atomics on y_f32_dev (the
 * workspace is then not used and may be NULL), and results are reproducible to rounding only.
 * Errors: DC_E_ARG, DC_E_CAP (workspace too small), DC_E_HIP.
 */
int dc_decompress_gemv_workspace(uint64_t n_chunks, uint64_t *workspace_bytes);
int dc_decompress_gemv(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                       uint64_t n_chunks, const dc_params *params, const float *row_scale_dev,
                       uint32_t rows, uint32_t cols, const uint16_t *x_bf16_dev, float *y_f32_dev,
                       uint16_t *y_bf16_dev, void *workspace_dev, uint64_t workspace_bytes, void *hip_stream);

/*
 * The two fused calls for all matrices of a layer at once (Section 3.3 lets the decompression
 * granularity be a layer; one launch over all chunks keeps the GPU filled where a single matrix
 * cannot).  mats_host: n_mats <= DC_MAX_MATRICES descriptors in table order; the chunk counts of the
 * matrices must add up to n_chunks.  Same arithmetic, outputs, workspace and errors as the single-matrix
 * calls, which are these calls with one matrix (the ordered product needs every matrix to meet the
 * condition on rows per chunk).
 */
int dc_decompress_dequant_bf16_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                     uint64_t n_chunks, const dc_params *params, const dc_matrix *mats_host,
                                     uint32_t n_mats, void *hip_stream);
int dc_decompress_gemv_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                             uint64_t n_chunks, const dc_params *params, const dc_matrix *mats_host,
                             uint32_t n_mats, void *workspace_dev, uint64_t workspace_bytes, void *hip_stream);

/*
 * Decompression fused with the batch-1 product in the paper's own arithmetic: weights and activations
 * both INT8 (Section 3.2, Eq. 4, Y_INT8 = Quant(X') * Quant(W'); Section 4.1).  Per row i
 *   sum_i = sum_j q_ij * xq_j            exact, 32-bit integers (cols <= 16384 keeps it inside)
 *   y_i   = (float(sum_i) * row_scale[i]) * x_scale   conversion and each product rounded once, in this order
 * so the result has one right value whatever the order of the additions.  x_i8_dev: cols int8 values,
 * 16-byte aligned; x_scale: their scale (dc_quantize_vector makes both).  y_accum_dev: rows fp32 results
 * (it holds the integer sums while the call runs); y_bf16_dev: the same rounded to bf16, may be NULL.
 * Three launches on hip_stream; nothing decoded is written to memory.  Errors as dc_decompress_gemv.
 * The _layer form takes x_i8_dev and x_scale from the matrix descriptors.
 */
int dc_decompress_gemv_w8a8(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                            uint64_t n_chunks, const dc_params *params, const float *row_scale_dev, uint32_t rows,
                            uint32_t cols, const int8_t *x_i8_dev, float x_scale, float *y_accum_dev,
                            uint16_t *y_bf16_dev, void *hip_stream);
int dc_decompress_gemv_w8a8_layer(const uint8_t *blob_dev, uint64_t blob_bytes, const dc_chunk *table_dev,
                                  uint64_t n_chunks, const dc_params *params, const dc_matrix *mats_host,
                                  uint32_t n_mats, void *hip_stream);
/* The same product on weights that are already in the decompression buffer (q_dev and x_i8_dev 16-byte
 * aligned, cols a multiple of 16, at most 16384).  One launch. */
int dc_gemv_w8a8(const int8_t *q_dev, const float *row_scale_dev, uint32_t rows, uint32_t cols,
                 const int8_t *x_i8_dev, float x_scale, float *y_f32_dev, uint16_t *y_bf16_dev, void *hip_stream);
/*
 * INT8 quantisation of one activation row (Eq. 4, "Quant(X')"; the paper states no granularity for
 * activations: one scale for the row).  Host to host.  scale = max |x| / 127 in fp32 (1 if x is all
 * zero), xq_j = clamp(round-half-even(x_j / scale), -127, 127).
 */
int dc_quantize_vector(const float *x_host, uint32_t n, int8_t *xq_host, float *scale_host);

/*
 * Batch-1 product on weights that are already in the decompression buffer: the "model inference
 * computation" that reads the buffer in Section 3.3 (I_gpu of Eq. 12), Eq. 1 for one activation row:
 *   y_i = row_scale[i] * sum_j q_ij * x_j,   q int8 row-major [rows][cols], x bf16, fp32 accumulation.
 * q_dev and x_bf16_dev 16-byte aligned, cols a multiple of 16.  y_f32_dev receives rows fp32 values,
 * y_bf16_dev (may be NULL) the same rounded to bf16.  One launch, asynchronous on hip_stream.
 */
int dc_gemv_i8(const int8_t *q_dev, const float *row_scale_dev, uint32_t rows, uint32_t cols,
               const uint16_t *x_bf16_dev, float *y_f32_dev, uint16_t *y_bf16_dev, void *hip_stream);

/*
 * Plain device copy kernel (reads n bytes, writes n bytes, 16-byte aligned): the denominator for
 * "share of achievable bandwidth" next to the decode kernels (cf. B_gpu in Eq. 11).
 */
int dc_device_copy(const void *src_dev, void *dst_dev, uint64_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DC_MI355X_H */
