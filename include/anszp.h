/*
 * anszp.h -- C ABI of libanszp: inference-time tabled-ANS (tANS) decoding of
 * entropy-coded, zero-point-quantized, mixed-precision network weights on
 * AMD MI355X (gfx950), fused with dequantisation to compute-ready weights.
 *
 * Method (citations are to the paper "Efficient Neural Compression with
 * Inference-time Decoding"):
 *   Sec. II-A    the decoder is a look-up table with one entry per state holding
 *                (symbol, nb_bits, newX); a step emits the symbol, reads nb_bits
 *                bits from the compressed stream and moves to state newX + bits;
 *                transitions that read no bits allow rates below 1 bit/weight.
 *   Sec. III-A   one table per layer.
 *   Sec. III-B   several streams are decoded at once with one shared table and a
 *                vector of states (here: one GPU lane per stream).
 *   Sec. II-B    weights come from a uniform quantizer with a zero-point, so
 *                w = scale * (q - zero_point).
 *
 * General conventions
 *   - Pointers marked [device] are device addresses of the current HIP device;
 *     pointers marked [host] are ordinary host addresses.  The caller owns every
 *     buffer.  The library allocates no device memory and keeps nothing between calls but
 *     three small per-device caches (the device's number of compute units, which kernels have
 *     been given leave to use the whole of a CU's on-chip memory, and the address of the
 *     fixed plan area that anszp_decode_static_plan uses); they are tables of atomics, so
 *     calls from several host threads are safe.  anszp_build_tables allocates and frees
 *     pinned host memory for its upload and waits for the copy.
 *   - `hip_stream` is a hipStream_t (NULL = default stream).  Device work is
 *     enqueued on it and the call returns without waiting, unless stated.
 *   - Return value: 0 on success, a negative ANSZP_E_* code when the host can
 *     see the problem (nothing has been enqueued then).  Problems only the GPU
 *     can see (corrupt stream, descriptor out of range) are OR-ed into the
 *     caller's status words; no device access ever leaves the caller's buffers
 *     because every index is checked or clamped first.
 *   - No exceptions, aborts or prints cross this boundary.
 *
 * Compressed container (all little-endian)
 *   A layer is a flat row-major array of n symbols q_i in [0, 256).  It is cut
 *   into consecutive chunks of `chunk_size` symbols (the last may be short).
 *   Inside a chunk, element j belongs to stream (j mod N) and is that stream's
 *   symbol number (j div N); N = n_streams <= 64.  Each stream is a private run
 *   of 32-bit words: the bits the decoder reads, in the order it reads them,
 *   filling each word from bit 0 upwards, zero-padded to a whole word.  The
 *   nb_bits of one step are read most significant first (bits = 2*bits + next).  A chunk's
 *   payload is its N streams' words back to back in stream order and starts at
 *   a word offset that is a multiple of 4.  Each stream has one 32-bit header:
 *   bits 0..15 the decoder's initial state X (0 <= X < 2^table_log), bits
 *   16..31 the stream's length in words.  The encoder starts every stream in
 *   state X = 0 and runs over its symbols last to first, so a correct decode
 *   ends in state 0 having read exactly the stream's words.
 */
#ifndef ANSZP_H
#define ANSZP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANSZP_ALPHABET        256   /* symbols are bytes; frequency rows have 256 entries     */
#define ANSZP_MAX_TABLE_LOG   12    /* tables have L = 2^table_log states, 1 <= table_log <= 12 */
#define ANSZP_MAX_STREAMS     64    /* streams per chunk = lanes of one wavefront              */
#define ANSZP_TABLE_WORDS_PER_STATE 8 /* a table of L states occupies 8 L 32-bit words           */

/* error codes returned by the functions */
#define ANSZP_OK              0
#define ANSZP_E_NULL         (-1)   /* a required pointer is NULL                              */
#define ANSZP_E_RANGE        (-2)   /* an argument is outside its documented range             */
#define ANSZP_E_FREQ         (-3)   /* a frequency row does not sum to 2^table_log             */
#define ANSZP_E_SYMBOL       (-4)   /* data contains a symbol whose frequency is zero          */
#define ANSZP_E_SPACE        (-5)   /* an output buffer is too small / a stream exceeds 65535 words */
#define ANSZP_E_HIP          (-6)   /* the HIP runtime reported an error                       */
#define ANSZP_E_NOMEM        (-7)   /* host allocation failed                                  */

/* bits OR-ed into status[0] by the decode kernels */
#define ANSZP_ST_BAD_DESC     1u    /* chunk descriptor points outside a buffer; chunk skipped */
#define ANSZP_ST_BAD_STATE    2u    /* a stream did not end in state 0                          */
#define ANSZP_ST_BAD_LENGTH   4u    /* a stream read more or fewer words than its header says   */
#define ANSZP_ST_INTERNAL     8u    /* a hand-over between wavefronts did not complete; chunk abandoned */
#define ANSZP_ST_BAD_FREQ     16u   /* anszp_build_tables_device, anszp_pack_layer_device: a frequency row does not sum to 2^table_log */
#define ANSZP_ST_BAD_SYMBOL   32u   /* anszp_pack_layer_device: the data contain a symbol whose frequency is zero */
#define ANSZP_ST_NO_SPACE     64u   /* anszp_pack_layer_device: payload buffer too small, or a stream longer than 65535 words */

/* output element types */
#define ANSZP_OUT_U8          0     /* decoded symbols, no dequantisation                       */
#define ANSZP_OUT_F32         1     /* IEEE binary32                                            */
#define ANSZP_OUT_BF16        2     /* bfloat16, round-to-nearest-even of the binary32 value    */

/* One chunk (32 bytes).  Arrays of these live in device memory for anszp_decode.  A descriptor
   names everything its chunk touches, so the array may be in any order: workgroups are handed
   out in array order, and a launch whose chunks differ much in size ends sooner when the chunks
   with the most payload words come first. */
typedef struct {
    uint32_t layer_id;        /* selects the table and the anszp_layer_t                       */
    uint32_t n_symbols;       /* symbols in this chunk; stream k holds ceil((n_symbols-k)/N)   */
    uint64_t out_offset;      /* element index of the chunk's first symbol in `out`            */
    uint64_t payload_offset;  /* first word of the chunk in `payload`; multiple of 4           */
    uint32_t payload_words;   /* sum of the chunk's stream lengths                             */
    uint32_t stream_offset;   /* index of stream 0's header in `stream_hdr`                    */
} anszp_chunk_t;

/* One layer's quantizer (32 bytes), Sec. II-B. */
typedef struct {
    float    scale;           /* used when channel_len == 0                                    */
    uint32_t zero_point;      /* z: symbol that decodes to +0.0                                */
    uint32_t bitwidth;        /* informational: symbols are < 2^bitwidth, 1..8                 */
    uint32_t channel_len;     /* 0: one scale per layer; else elements per output channel and
                                 the scale of layer element e is scales[scales_offset + e / channel_len] */
    uint64_t scales_offset;   /* index of the layer's first channel scale in `scales`          */
    uint64_t out_base;        /* element index of the layer's first element in `out`           */
} anszp_layer_t;

/* Arguments of anszp_decode (the struct itself is read on the host). */
typedef struct {
    const uint32_t*      tables;        /* [device] n_tables * 8 * 2^table_log words from anszp_build_tables, 16-byte aligned */
    uint32_t             n_tables;
    uint32_t             table_log;     /* R, 1..12                                             */
    uint32_t             n_streams;     /* N, 1..64                                             */
    uint32_t             out_dtype;     /* ANSZP_OUT_*                                          */
    const anszp_chunk_t* chunks;        /* [device]                                             */
    uint64_t             n_chunks;      /* may be 0 (nothing is enqueued)                       */
    const uint32_t*      stream_hdr;    /* [device] one header per stream                       */
    uint64_t             n_stream_hdr;
    const uint32_t*      payload;       /* [device] 16-byte aligned                             */
    uint64_t             payload_words;
    const anszp_layer_t* layers;        /* [device] n_tables entries                            */
    const float*         scales;        /* [device] per-channel scales, may be NULL if unused   */
    uint64_t             n_scales;
    void*                out;           /* [device] out_elems elements of out_dtype, 16-byte aligned */
    uint64_t             out_elems;
    uint32_t*            status;        /* [device] 2 words: [0] OR of ANSZP_ST_*, [1] number of
                                           failing chunks.  Never cleared by the library: zero it
                                           once, read it after synchronising the stream.        */
} anszp_decode_args_t;

/* Library version (major * 100 + minor). */
int anszp_version(void);

/* Text for an ANSZP_E_* code; never NULL; static storage. */
const char* anszp_strerror(int code);

/* [host only] Turn symbol counts into table frequencies (the paper does not say how):
 * freqs[s] >= 1 exactly when counts[s] > 0 and sum(freqs) == 2^table_log.
 * counts, freqs: [host] 256 entries.  Errors: E_NULL, E_RANGE, E_FREQ (no symbols, or more
 * distinct symbols than states). */
int anszp_normalize_freqs(const uint64_t* counts, int table_log, uint32_t* freqs);

/* [host only] Sec. II-A / III-A: build n_tables decode tables from normalised frequencies.
 * freqs: [host] n_tables rows of 256.  tables: [host] n_tables * ANSZP_TABLE_WORDS_PER_STATE * 2^table_log
 * 32-bit words.  Table t occupies words [t*8L, (t+1)*8L), L = 2^table_log:
 *   words [0, L)     tables of at most 256 states: the byte table of Sec. II-A, 3 L bytes, state X at
 *                    bytes 3X (symbol), 3X+1 (nb_bits), 3X+2 (newX), the rest zero; larger tables: zero
 *   word [2L + X]    the paper's triple for state X:
 *                    bits 0..15 newX      bits 16..23 nb_bits   bits 24..31 symbol
 *   words [4L + 2(2X + b)], [4L + 2(2X + b) + 1]
 *                    the same automaton with up to 8 steps merged and one bit of look-ahead: in state
 *                    X with next stream bit b (peeked, not consumed) the next c-1 symbols are the
 *                    dominant symbol (f > L/2: its zero-bit transitions and at most one of its 1-bit
 *                    transitions, which consumes b), then `symbol` is emitted; T stream bits are
 *                    consumed in all, and with v = the next T+1 stream bits, first bit on top, the
 *                    next entry is number base + v.  A run never passes through state 0 (the step that
 *                    arrives there ends the entry), so a stream ends where an entry ends.
 *                    first word:  bits 0..4 31-T (T <= 12)   bits 9..11 c-1   bits 16..23 symbol
 *                                 bits 24..27 T   bits 28..30 c-1   bit 31 set for X = 0   other bits zero
 *                    second word: 8 * base (two's complement)
 *   words [L, 2L), [3L, 4L)  zero
 * Errors: E_NULL, E_RANGE, E_FREQ. */
int anszp_build_tables_host(const uint32_t* freqs, int n_tables, int table_log, uint32_t* tables);

/* Same, writing the tables to device memory.  tables_dev: [device], 16-byte aligned.  The
 * host-to-device copy is enqueued on hip_stream and waited for before returning.
 * Errors: as above, E_HIP, E_NOMEM. */
int anszp_build_tables(const uint32_t* freqs_host, int n_tables, int table_log,
                       uint32_t* tables_dev, void* hip_stream);

/* Sec. II-A / III-A on the device: the same tables, word for word, from normalised frequencies that
 * are already in device memory (one workgroup per table; nothing passes through the host).
 * freqs_dev: [device] n_tables rows of 256.  tables_dev: [device] n_tables * 8 * 2^table_log words,
 * 16-byte aligned.  status_dev: [device] 2 words as in anszp_decode_args_t, or NULL: a row that
 * does not sum to 2^table_log leaves its table all zero and sets ANSZP_ST_BAD_FREQ (the host cannot
 * see the rows, so this is not a return code).  Asynchronous on hip_stream; both buffers stay owned
 * by the caller.  Errors: E_NULL, E_RANGE, E_HIP. */
int anszp_build_tables_device(const uint32_t* freqs_dev, int n_tables, int table_log,
                              uint32_t* tables_dev, uint32_t* status_dev, void* hip_stream);

/* [host only] Worst-case sizes for anszp_pack_layer: number of chunks and payload words. */
int anszp_pack_bound(uint64_t n_symbols, int table_log, int n_streams, uint32_t chunk_size,
                     uint64_t* n_chunks, uint64_t* payload_words);

/* [host only] Offline compressor (Sec. II-A encoder; container described at the top).
 * Encodes one layer's symbols with the table given by freqs and appends to caller arrays:
 * chunks_out[0..n_chunks), stream_hdr_out[0..n_chunks*N), payload_out[0..*payload_words_used).
 * layer_id / out_offset / payload_word_offset / stream_offset are the positions the layer's
 * first chunk will have in the full container (payload_word_offset must be a multiple of 4).
 * Errors: E_NULL, E_RANGE, E_FREQ, E_SYMBOL, E_SPACE, E_NOMEM. */
int anszp_pack_layer(const uint8_t* symbols, uint64_t n_symbols, const uint32_t* freqs,
                     int table_log, int n_streams, uint32_t chunk_size,
                     uint32_t layer_id, uint64_t out_offset, uint64_t payload_word_offset,
                     uint32_t stream_offset,
                     anszp_chunk_t* chunks_out, uint32_t* stream_hdr_out,
                     uint32_t* payload_out, uint64_t payload_cap_words, uint64_t* payload_words_used);

/* Sec. II-A decoder + Sec. III-B parallel streams + Sec. II-B dequantisation, fused: decode
 * every chunk (one wavefront per chunk, one lane per stream) and write out[out_offset + j] for
 * each of its symbols j, as raw symbols, fp32 or bf16 weights.  One kernel launch on hip_stream.
 * Errors: E_NULL, E_RANGE (table_log, n_streams, out_dtype, n_tables == 0, n_chunks >= 2^31,
 * payload or out not 16-byte aligned). */
int anszp_decode(const anszp_decode_args_t* args, void* hip_stream);

/* The same call with the kernel chosen by hand; results are identical for every variant.
 *   0  automatic (what anszp_decode does)
 *   1  step-wise kernel: one look-up per symbol, exactly the loop of Sec. II-A / III-B; also the
 *      path any chunk takes whose compressed words exceed the on-chip window or whose first
 *      output element is not 16-byte aligned
 *   2  look-ahead kernel: look-ups use the look-ahead entries of the table (entry 2X + b above),
 *      compressed words and decoded symbols are staged in LDS, and the work of a chunk is split
 *      over several wavefronts of its workgroup
 *   3  step-wise kernel with sixteen chunks per workgroup sharing the tables in LDS
 *   4  streaming kernel: one look-up per symbol from compact entries in LDS, each stream's words
 *      fetched 64 bytes at a time through a ring in LDS by wavefronts that only load (what the
 *      automatic choice takes when the chunks are too large for the on-chip window)
 *   5  byte-table kernel: the decoder as Sec. II-A sizes it, for tables of at most 256 states
 *      (table_log <= 8): the 3 l-byte table (one byte each for symbol, nb_bits and newX; 192 bytes for
 *      64 states) in LDS, three byte reads and a log2(l)-bit addition per symbol
 * Errors: as anszp_decode, E_RANGE for an unknown variant or variant 5 with table_log > 8. */
int anszp_decode_variant(const anszp_decode_args_t* args, int variant, void* hip_stream);

/* For tests of the library's failure handling only.  Every wait of one wavefront for another inside the decode
 * kernels is bounded by a number of polls, after which the chunk is abandoned with ANSZP_ST_INTERNAL and its
 * workgroup drains.  polls >= 1: later launches give up after polls - 1 polls (1: at the first wait that is not
 * satisfied at once, which every launch of the look-ahead and streaming kernels has); 0: back to the default
 * (2^22).  Process-wide, not synchronised with launches in flight. */
void anszp_test_set_spin_limit(uint32_t polls);

/* Sec. III-A: the weights of a network are decoded again at every inference, from arrays that do not
 * change.  What every launch of anszp_decode first works out on the device (which chunks of a layer
 * share a workgroup and its on-chip copy of the layer's table, in which order the chip's dies take
 * them) can therefore be prepared once: anszp_plan_decode writes it to plan_dev, anszp_decode_planned
 * decodes with it and gives the same output and status words as anszp_decode.
 *   anszp_plan_bytes    bytes of device memory a plan for n_chunks chunks takes (a record of 128 bytes per
 *                       workgroup of the launch, and as much again to sort them in: the workgroups take the
 *                       units with the longest chains first); 0 for n_chunks >= 2^31.
 *   anszp_plan_decode   args as for anszp_decode (every array already in place; out and status are not
 *                       touched); plan_dev [device, caller's, 16-byte aligned] at least
 *                       anszp_plan_bytes(args->n_chunks) bytes, written on hip_stream.  A launch that
 *                       the automatic choice does not give to the look-ahead kernel needs no plan:
 *                       nothing is written then, and anszp_decode_planned does not read plan_dev.
 *   anszp_decode_planned  the plan must have been written for these very arrays (same pointers'
 *                       contents, same scalar arguments) on this device.  A plan that was made for
 *                       another number of chunks or another kernel is refused on the device
 *                       (ANSZP_ST_BAD_DESC, nothing decoded); one whose descriptors no longer match the
 *                       arrays decodes what it describes, checked against the caller's buffers like any
 *                       descriptor: never out of bounds.
 * Errors: as anszp_decode; E_NULL for a missing plan, E_RANGE for one that is too small or misaligned. */
uint64_t anszp_plan_bytes(uint64_t n_chunks);
int anszp_plan_decode(const anszp_decode_args_t* args, void* plan_dev, uint64_t plan_bytes, void* hip_stream);
int anszp_decode_planned(const anszp_decode_args_t* args, const void* plan_dev, uint64_t plan_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under stream capture, serving loops, harnesses
 * that forbid it): anszp_decode_planned with the plan kept in device memory of the library's own, a
 * fixed array of 1 MiB per device that holds a plan for at most 4096 chunks and stays until the
 * process ends.  Calls no allocating routine.  replan != 0: the plan is written first (as by
 * anszp_plan_decode) and the decode follows on the same stream; replan == 0: the array must still hold
 * the plan an earlier call on this device wrote for these arrays.  Every call on a device shares that
 * device's array: calls that overlap on one device (other streams, other host threads) race unless all
 * of them pass replan == 0 for the same arrays.
 * Errors: as anszp_decode; E_RANGE for more than 4096 chunks; E_HIP if the array's address cannot be found. */
int anszp_decode_static_plan(const anszp_decode_args_t* args, int replan, void* hip_stream);

/* Sec. II-B alone: out[i] = scale * (symbols[i] - zero_point) for i < n, the scale chosen as in
 * anszp_layer_t with the layer starting at element 0.  symbols_dev, scales_dev, out_dev: [device];
 * layer: [host].  out_dtype is ANSZP_OUT_F32 or ANSZP_OUT_BF16.  Errors: E_NULL, E_RANGE. */
int anszp_dequant_zp(const uint8_t* symbols_dev, uint64_t n, const anszp_layer_t* layer,
                     const float* scales_dev, uint64_t n_scales, void* out_dev, int out_dtype,
                     void* hip_stream);

/* The packer on the GPU (Sec. II-A, the encoding direction: a stream's symbols are walked backwards,
 * the state dropping low bits until the symbol's sub-range holds it): anszp_pack_layer for symbols and
 * frequencies that live in device memory, writing the same descriptors, stream headers and payload
 * words, word for word.  symbols_dev [device] n_symbols bytes; freqs_dev [device] 256 frequencies
 * summing to 2^table_log; chunks_dev [device] ceil(n_symbols / chunk_size) descriptors, stream_hdr_dev
 * [device] n_streams headers per chunk, payload_dev [device] payload_cap_words words where this layer's
 * words begin (its chunks' payload_offset fields count from payload_word_offset, a multiple of 4);
 * payload_words_used_dev [device] one 64-bit count; status_dev [device] 2 words as for anszp_decode.
 * Asynchronous on hip_stream; three kernel launches, nothing allocated.  Errors: E_NULL, E_RANGE, E_HIP on
 * the host; in status: ANSZP_ST_BAD_FREQ (nothing is written), ANSZP_ST_BAD_SYMBOL (the layer's output is
 * unspecified), ANSZP_ST_NO_SPACE (chunks that do not fit are not written; *payload_words_used_dev still
 * holds what the layer needs). */
int anszp_pack_layer_device(const uint8_t* symbols_dev, uint64_t n_symbols, const uint32_t* freqs_dev,
                            int table_log, int n_streams, uint32_t chunk_size, uint32_t layer_id,
                            uint64_t out_offset, uint64_t payload_word_offset, uint32_t stream_offset,
                            anszp_chunk_t* chunks_dev, uint32_t* stream_hdr_dev, uint32_t* payload_dev,
                            uint64_t payload_cap_words, uint64_t* payload_words_used_dev,
                            uint32_t* status_dev, void* hip_stream);

/* The same for a whole set of layers in three launches (one workgroup per chunk, so every chunk of every layer is
 * encoded at once).  symbols_dev [device]: the layers' symbols, layer after layer; jobs_dev [device] n_layers
 * entries in layer order; freqs_dev [device] n_layers rows of 256 frequencies summing to 2^table_log each;
 * n_chunks: the sum over the layers of ceil(n_symbols / chunk_size) (anszp_pack_bound gives each term).
 * Layer l becomes layer_id l; its chunks follow those of layer l-1 in chunks_dev and stream_hdr_dev
 * (stream_offset = chunk index * n_streams), its elements start at out_offset = first_symbol, the payload
 * starts at word 0 of payload_dev.  Writes what one anszp_pack_layer call per layer would write (and what the
 * oracle's encoder writes), word for word.  Status bits as anszp_pack_layer_device, and ANSZP_ST_BAD_DESC
 * when the jobs do not account for n_chunks chunks (those chunks get empty descriptors).
 * Errors: E_NULL, E_RANGE (table_log, n_streams, n_chunks >= 2^31 or n_chunks * n_streams >= 2^32), E_HIP. */
typedef struct {
    uint64_t first_symbol;    /* index of the layer's first symbol in symbols_dev = out_offset of its first chunk */
    uint64_t n_symbols;
    uint32_t chunk_size;      /* >= 1 */
    uint32_t first_chunk;     /* number of chunks of all layers before this one */
    uint32_t reserved[2];     /* 0 */
} anszp_pack_job_t;
int anszp_pack_layers_device(const uint8_t* symbols_dev, const anszp_pack_job_t* jobs_dev, uint32_t n_layers,
                             uint64_t n_chunks, const uint32_t* freqs_dev, int table_log, int n_streams,
                             anszp_chunk_t* chunks_dev, uint32_t* stream_hdr_dev, uint32_t* payload_dev,
                             uint64_t payload_cap_words, uint64_t* payload_words_used_dev,
                             uint32_t* status_dev, void* hip_stream);

/* activation layouts of anszp_conv_fused */
#define ANSZP_ACT_NHWC        0     /* [batch][h][w][channels]                                    */
#define ANSZP_ACT_C8          1     /* [batch][channels / 8][h][w][8]: blocks of 8 channels, so that
                                       the 16 pixels a matrix instruction's operand rows come from
                                       are 256 contiguous bytes; channels a multiple of 8          */

/* Arguments of anszp_conv_fused (the struct itself is read on the host).  The container fields
 * mean what they mean in anszp_decode_args_t; `chunks` points at the FIRST chunk of the layer to
 * convolve with, `n_chunks` counts the chunks from there on. */
typedef struct {
    const uint32_t*      tables;         /* [device] as for anszp_decode                          */
    uint32_t             n_tables;
    uint32_t             table_log;
    uint32_t             n_streams;
    uint32_t             layer_id;       /* the layer's table and anszp_layer_t                   */
    const anszp_chunk_t* chunks;         /* [device] the layer's chunks, in order of output channel */
    uint64_t             n_chunks;       /* at least cout / rows_per_chunk                        */
    const uint32_t*      stream_hdr;     /* [device]                                              */
    uint64_t             n_stream_hdr;
    const uint32_t*      payload;        /* [device]                                              */
    uint64_t             payload_words;
    const anszp_layer_t* layers;         /* [device] n_tables entries; channel_len is 0 or kh*kw*cin
                                            (one scale per output channel)                        */
    const float*         scales;         /* [device] may be NULL if unused                        */
    uint64_t             n_scales;
    uint32_t             rows_per_chunk; /* output channels per chunk: 1, 2, 4, 8 or 16; every chunk
                                            holds rows_per_chunk * kh*kw*cin symbols              */
    uint32_t             batch, in_h, in_w, cin, cout, kh, kw, stride, pad;
    const uint16_t*      x;              /* [device] bf16 activations in x_layout, batch * in_h * in_w * cin
                                            elements (fewer than 2^32), 16-byte aligned            */
    void*                y;              /* [device] batch * out_h * out_w * cout elements (fewer than 2^32)
                                            of y_dtype in y_layout, out = (in + 2 pad - k) / stride + 1,
                                            16-byte aligned; every element is written              */
    uint32_t             y_dtype;        /* ANSZP_OUT_F32, or ANSZP_OUT_BF16 (the fp32 result rounded
                                            to nearest even)                                      */
    uint32_t             x_layout;       /* ANSZP_ACT_*; ANSZP_ACT_C8 needs cin to be a multiple of 8 */
    uint32_t             y_layout;       /* ANSZP_ACT_*                                            */
    uint32_t*            status;         /* [device] 2 words, as for anszp_decode                 */
} anszp_conv_args_t;

/* Fused decode + convolution (the data are decoded on their way from memory to the compute
 * units, Sec. II; weights w = scale * (q - z), Sec. II-B): y = conv2d(x, w) with zero padding,
 * where the layer's symbols q, in the order [cout][kh][kw][cin], are decoded (Sec. II-A, one
 * stream per lane as in Sec. III-B) into on-chip memory and multiplied there with the activations
 * by bf16 matrix instructions with fp32 accumulation; the decoded weights are never written to
 * device memory.  q - z is exact in bf16; the scale multiplies the fp32 sums.
 * Limits: cout a multiple of 16; kh*kw*cin <= 4608; batch*out_h*out_w < 2^31.  Asynchronous on
 * hip_stream; the buffers stay the caller's.  Errors: E_NULL, E_RANGE (a limit above, misaligned
 * x or y, too few chunks), E_HIP; a chunk whose descriptor does not fit the layer, a stream that
 * ends in the wrong state or length: ANSZP_ST_* bits in status, as for anszp_decode (the outputs
 * of the affected output channels are then unspecified but finite sums of finite values).
 * The kernel reads the look-ahead entries of the layer's table (anszp_build_tables*).  The first
 * call of each of its kernels on a device gives that kernel leave to use all of a CU's on-chip
 * memory (a function attribute) and must not be part of a stream capture; later calls may be
 * captured into a graph and replayed. */
int anszp_conv_fused(const anszp_conv_args_t* args, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ANSZP_H */
