// Fused decode + convolution for gfx950: a conv layer's entropy-coded weights are decoded into LDS
// and consumed there by bf16 MFMA instructions; the decoded weights never reach global memory
// (Sec. II: the weights are to be decoded on their way from memory to the compute units).
//
// The convolution is an implicit GEMM  Y[n, o] = sum_k A[o, k] * B[k, n]  with
//   o = output channel, n = (image, output row, output column), k = (kernel row, kernel column,
//   input channel), input channel innermost,
//   A[o, k] = q - z, the decoded symbol minus the layer's zero-point (Sec. II-B): an integer of at
//   most 8 bits and therefore exact in bf16; the scale multiplies the fp32 sums at the end,
//   B[k, n] = the bf16 activation under kernel tap (r, s) of output pixel n, zero outside the image.
// Activations and outputs are NHWC or in blocks of 8 channels ([batch][channels / 8][h][w][8]); in both
// the 8 consecutive k one lane feeds into an MFMA are 16 contiguous bytes of the activation tensor.  In
// the blocked layout the 16 lanes that hold the same 8 k of 16 neighbouring pixels read 256 contiguous
// bytes, where NHWC makes them read 16 pieces a whole pixel apart.
//
// One workgroup owns a panel of 16 * MR output channels (MR = 4, 2 or 1 row tiles of
// v_mfma_f32_16x16x32_bf16: as many as fit in LDS) and a range of output pixels.  Phase 1: its twelve
// wavefronts decode the chunks that hold those weight rows, one lane per stream (Sec. II-A, III-B),
// through the table's look-ahead entries (one look-up per run of up to eight symbols) into a
// [16 * MR][K] panel in LDS: symbols as bytes, or, for short rows, the bf16 values q - z.  Phase 2, by
// kind of layer (see the enumeration in front of the kernel): 1 x 1 kernels read their activation
// vectors from global memory through a ring of hand-issued loads; kernels three taps wide load the
// three taps of a kernel row and 32 channels together, so that the L1 serves what they share; 3 x 3
// kernels of stride 1 with long rows (K > 1152) stage the activations under all nine taps of a round
// of pixels in LDS once per 32 input channels; layers like the first one (3 channels) stage whole
// image rows in LDS and gather from there; other shapes use loops the compiler schedules.  fp32
// accumulators; one store of four consecutive output channels per lane, row tile and column tile.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <type_traits>
#include <utility>

#include <cstdint>

#include "anszp.h"
#include "anszp_layout.h"

namespace {

constexpr uint32_t kWave = 64;
constexpr uint32_t kThreads = 768;
constexpr uint32_t kWaves = kThreads / kWave;
constexpr uint32_t kRows = 16;              // output channels per MFMA row tile
constexpr uint32_t kRowPad = 8;             // bytes between panel rows: rows start two LDS banks apart
constexpr uint32_t kStageWords = 384;       // per wavefront: LDS room for one chunk's compressed words (2.6 bit per
                                            // weight at 4608 symbols; a larger chunk is read from global memory)
constexpr uint32_t kWidenPieces = 7;        // 16-byte pieces of a byte panel one thread widens to bf16
constexpr uint32_t kPatchTaps = 9;          // kTapsPatch: a 3 x 3 kernel
constexpr uint32_t kPatchPieces = 4;        // kTapsPatch: 16-byte pieces of a patch per thread
constexpr uint32_t kMaxMine = (4u * kRows + kWaves - 1u) / kWaves;   // chunks of a panel one wavefront may have to decode

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) uint32_t words4;
typedef __attribute__((ext_vector_type(2))) uint32_t words2;

struct ConvParams {
    const uint32_t* tables;
    const anszp_chunk_t* chunks;        // the layer's first chunk
    const uint32_t* stream_hdr;
    const uint32_t* payload;
    const anszp_layer_t* layers;
    const float* scales;
    const uint16_t* x;
    void* y;
    uint32_t* status;
    uint64_t n_stream_hdr, payload_words, n_scales;
    uint32_t layer_id, table_log, n_streams, rows_per_chunk, chunks_per_panel;
    uint32_t in_h, in_w, cin, cout, kh, kw, stride, pad, out_h, out_w;
    // element strides that tell the two activation layouts apart (see anszp_conv_args_t):
    //   x element (image b, pixel i, channel c) = b * in_h*in_w*cin + i * x_pixel + (c / 8) * x_block + c % 8
    //   y element (image b, pixel i, channel o) = b * out_h*out_w*cout + i * y_pixel + (o / 8) * y_block + o % 8
    // NHWC: pixel = channels, block = 8;  blocks of 8 channels: pixel = 8, block = 8 * pixels per image
    uint32_t x_pixel, x_block, y_pixel, y_block;
    uint32_t y_bf16, K, row_stride, n_pixels, n_mtiles;   // n_mtiles: panels of 16 * MR rows
    uint32_t k_magic;                                     // floor(2^32 / K) + 1: i / K = mulhi(i, k_magic) for i * K < 2^32
    uint32_t panel_off;                                   // first byte of the panel in LDS (behind the table and the staging room)
    uint32_t wave_pixels, patch_off, patch_plane;         // kTapsPatch: pixels per wavefront and round (16..64); first byte of the
                                                          // patch; bytes of one of its four planes
    uint32_t row_pitch;                                   // kGenericPatch: bytes from one staged image row to the next
    uint32_t pixels_per_split, block_pixels;              // multiples of 16: the pixels of a workgroup; of one block (<= 64)
};

__device__ __forceinline__ void report(uint32_t* status, uint32_t bits) {
    atomicOr(&status[0], bits);
    atomicAdd(&status[1], 1u);
}

__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
#pragma unroll
    for (int d = 1; d < int(kWave); d <<= 1) v |= __shfl_xor(v, d, kWave);
    return v;
}

// Exclusive prefix sum over the 64 lanes of a wavefront; *total receives the sum.  Data-parallel-primitive
// moves: within rows of 16 lanes by 1, 2, 4 and 8 (lanes without a source add zero), then lane 15 of rows 0
// and 2 to the rows after them, then lane 31 to the upper half.
__device__ __forceinline__ uint32_t wave_exclusive_sum(uint32_t v, uint32_t* total) {
    int x = static_cast<int>(v);
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);      // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);      // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);      // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);      // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);     // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);     // row_bcast:31 into rows 2 and 3
    *total = static_cast<uint32_t>(__builtin_amdgcn_readlane(x, kWave - 1));
    return static_cast<uint32_t>(x) - v;
}

// What a wavefront fetches of a chunk before it decodes it: the stream headers (lane k: stream k), the chunk's
// words as two 16-byte pieces per lane (kStageWords words in all) and the up to three words behind the last
// whole piece.
struct ChunkData {
    uint32_t hdr;
    words4 q0, q1;
    uint32_t tail;
};

// A chunk's descriptor as the wavefront uses it (uniform values), checked against the layer and the buffers.
struct ChunkDesc {
    uint32_t n_symbols, payload_words, stream_offset;
    uint64_t payload_offset;
    bool ok, staged;             // staged: the chunk's words (and two zero words behind them) fit the wavefront's LDS room
};

// One chunk into the LDS panel: symbol i of the chunk belongs to panel row i / K, column i % K.  One lane per
// stream (Sec. III-B) walks the automaton of Sec. II-A through the table's look-ahead entries (anszp_layout.h):
// one look-up stands for up to eight symbols, all but the last the layer's dominant symbol, which the panel
// already holds everywhere (the caller fills it), so a look-up writes one panel element.  The entry of index
// 2X + b and the two stream words around the lane's bit position are read together; with T the bits the entry
// consumes, the next index is base + (the next T + 1 stream bits, first bit most significant) and the bit
// position moves on by T.  Returns the lane's error bits.
// The chunk's words were fetched into `d` (16-byte loads issued long before) and go to `stage` (LDS, this
// wavefront's own) when they fit, so that the loop waits for no global load; a larger chunk is read word by word
// in place.  P16: the panel holds bf16 values q - z (two bytes per weight) instead of the symbols q.
template <bool P16>
__device__ uint32_t decode_chunk_to_panel(const ConvParams& p, const ChunkDesc& c, const ChunkData& d, const uint8_t* ahead,
                                          uint32_t ahead_mask, uint32_t* stage, uint8_t* rows, uint32_t lane, int32_t zero_point) {
    const uint32_t N = p.n_streams;
    const uint32_t L = 1u << p.table_log;
    const uint32_t X0 = d.hdr & (L - 1u);
    const uint32_t n_words = d.hdr >> 16;
    uint32_t total_words;
    const uint32_t first_word = wave_exclusive_sum(n_words, &total_words);
    uint32_t err = (total_words != c.payload_words) ? ANSZP_ST_BAD_DESC : 0u;

    const uint32_t* words = p.payload + c.payload_offset;
    const uint32_t word_limit = c.payload_words;      // reads beyond the chunk see zeros
    if (c.staged) {
        const uint32_t quads = word_limit >> 2;
        if (lane < quads) *reinterpret_cast<words4*>(stage + 4u * lane) = d.q0;
        if (lane + kWave < quads) *reinterpret_cast<words4*>(stage + 4u * (lane + kWave)) = d.q1;
        const uint32_t tail_at = (quads << 2) + lane;
        if (lane < 3u && tail_at < word_limit) stage[tail_at] = d.tail;
        if (lane < 2u) stage[word_limit + lane] = 0u;                // what a stream reads beyond the chunk
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");       // LDS serves a wavefront's accesses in order
        __builtin_amdgcn_wave_barrier();
    }
    const uint32_t n = lane < N ? c.n_symbols : 0u;   // a lane without a stream never runs
    const uint32_t first_bit = first_word << 5;
    uint32_t bit = first_bit;
    uint32_t elem = lane;                             // the chunk element of the lane's next symbol
    // A chunk of one panel row needs no division to find a symbol's row.  An entry that would carry a stream
    // past its end (corrupt data only: a valid stream ends where an entry ends) writes the chunk's last element.
    const uint32_t last_elem = c.n_symbols - 1u;
    constexpr uint32_t kElem = P16 ? 2u : 1u;
    const uint32_t row_gap_bytes = (p.row_stride - p.K) * kElem;
    auto walk = [&](auto word_at, auto one_row) {
        uint32_t at = ((2u * X0 + (word_at(min(first_word, word_limit)) & 1u)) * 8u) & ahead_mask;   // entry 2 X0 + first stream bit
        bool active = elem < n;
        if (__ballot(active) != 0) {
            do {
                if (active) {
                    const uint32_t wi = min(bit >> 5, word_limit);
                    const uint32_t w0 = word_at(wi), w1 = word_at(wi + 1u);
                    const words2 e = *reinterpret_cast<const words2*>(ahead + at);
                    const uint32_t window = __builtin_amdgcn_alignbit(w1, w0, bit);
                    const uint32_t v = __brev(window) >> (e.x & 31u);       // the next T + 1 stream bits
                    at = (e.y + 8u * v) & ahead_mask;
                    bit += (e.x >> 24) & 15u;
                    elem = __umul24((e.x >> 28) & 7u, N) + elem;            // past the entry's dominant symbols
                    const uint32_t el = min(elem, last_elem);
                    uint32_t where = el * kElem;                            // byte of the panel rows
                    if constexpr (!decltype(one_row)::value)
                        where = __umul24(p.K > 1u ? __umulhi(el, p.k_magic) : el, row_gap_bytes) + where;   // both factors below 2^24
                    const uint32_t sym = (e.x >> 16) & 0xFFu;
                    if constexpr (P16) {              // an integer of at most 8 bits: the upper half of its binary32 form is exact
                        const float w = static_cast<float>(int32_t(sym) - zero_point);
                        *reinterpret_cast<uint16_t*>(rows + where) = static_cast<uint16_t>(__float_as_uint(w) >> 16);
                    } else {
                        rows[where] = static_cast<uint8_t>(sym);
                    }
                    elem += N;
                    active = elem < n;
                }
            } while (__ballot(active) != 0);
        }
        // a stream ends where an entry ends, in state 0 (the index of the next entry is 2 X + peeked bit),
        // having read exactly its words
        if (lane < N) {
            // the lane's elements are lane, lane + N, ...: it has produced exactly its symbols if it stands on the
            // first of them that is no element of the chunk
            if (elem - c.n_symbols >= N) err |= ANSZP_ST_BAD_LENGTH;
            if ((at >> 4) != 0u) err |= ANSZP_ST_BAD_STATE;
            if (((bit - first_bit) + 31u) >> 5 != n_words) err |= ANSZP_ST_BAD_LENGTH;
        }
    };
    if (c.staged) {
        if (p.rows_per_chunk == 1u) walk([&](uint32_t i) { return stage[i]; }, std::true_type{});
        else walk([&](uint32_t i) { return stage[i]; }, std::false_type{});
    } else {
        walk([&](uint32_t i) { return i < word_limit ? words[i] : 0u; }, std::false_type{});
    }
    return err;                                       // this lane's
}

// Eight symbols -> eight bf16 values q - z.  |q - z| <= 255 has at most 8 significant bits, so the
// upper half of its binary32 form is the exact bf16 value.
__device__ __forceinline__ bf16x8 weights_of(words2 q, float z) {
    auto byte = [](uint32_t w, uint32_t i) { return static_cast<float>((w >> (8u * i)) & 0xFFu); };   // v_cvt_f32_ubyte<i>
    const float f0 = byte(q.x, 0) - z, f1 = byte(q.x, 1) - z, f2 = byte(q.x, 2) - z, f3 = byte(q.x, 3) - z;
    const float f4 = byte(q.y, 0) - z, f5 = byte(q.y, 1) - z, f6 = byte(q.y, 2) - z, f7 = byte(q.y, 3) - z;
    auto pack = [](float lo, float hi) {              // upper halves of two binary32 values, lo in bits 0..15
        return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
    };
    words4 w = {pack(f0, f1), pack(f2, f3), pack(f4, f5), pack(f6, f7)};
    return __builtin_bit_cast(bf16x8, w);
}

// The accumulators of one block of up to 64 pixels times the scale(s), to y.  D operand layout: lane holds
// column lane % 16, rows 4 * (lane / 16) + 0..3 of each row tile: four consecutive output channels.
template <uint32_t MR>
__device__ __forceinline__ void store_tiles(const ConvParams& p, const anszp_layer_t& lay, uint32_t mtile, uint32_t kg,
                                            const floatx4 (&acc)[MR][4], const bool (&valid)[4], const uint32_t (&out_at)[4]) {
    const bool per_channel = lay.channel_len != 0;
#pragma unroll
    for (uint32_t m = 0; m < MR; ++m) {
        const uint32_t o = (mtile * MR + m) * kRows + 4u * kg;
        float sc[4];
#pragma unroll
        for (uint32_t i = 0; i < 4; ++i) {
            sc[i] = lay.scale;
            if (per_channel) {
                const uint64_t ch = lay.scales_offset + o + i;
                sc[i] = ch < p.n_scales ? p.scales[ch] : 0.0f;
            }
        }
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            if (valid[q]) {
                const floatx4 out = {acc[m][q][0] * sc[0], acc[m][q][1] * sc[1], acc[m][q][2] * sc[2], acc[m][q][3] * sc[3]};
                const uint32_t at = out_at[q] + (o >> 3) * p.y_block + (o & 7u);
                if (p.y_bf16) {                                   // round to nearest even (v_cvt_pk_bf16_f32)
                    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                    const bf16x4 r = {static_cast<__bf16>(out[0]), static_cast<__bf16>(out[1]),
                                      static_cast<__bf16>(out[2]), static_cast<__bf16>(out[3])};
                    *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(p.y) + at) = r;
                } else {
                    *reinterpret_cast<floatx4*>(static_cast<float*>(p.y) + at) = out;
                }
            }
        }
    }
}

// What a kernel tap outside the image reads (kTapsRing: every load is unconditional).
__device__ __attribute__((aligned(64))) const uint32_t zero_page[16] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};

// kPointwiseRing, kTapsRing: the loads of one ring slot (QT activation vectors) issued by hand, and the wait for them.  When a
// slot is used, LATER loads have been asked for after its own, so the wait is for all but LATER loads; it names the
// slot's registers as its results, so that nothing which uses them can be moved ahead of it.  (The compiler, left
// to count loads that cross the loop's back edge, waits for every load at the head of the loop.)
template <uint32_t QT>
__device__ __forceinline__ void ring_request(words4 (&slot)[QT], const uint16_t* const (&px)[QT], uint32_t element_offset) {
#pragma unroll
    for (uint32_t q = 0; q < QT; ++q) {
        const uint16_t* from = px[q] + element_offset;
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(slot[q]) : "v"(from) : "memory");
    }
}
template <uint32_t QT, uint32_t LATER>
__device__ __forceinline__ void ring_arrived(words4 (&slot)[QT]) {
    static_assert(QT >= 1 && QT <= 4 && LATER < 64, "one to four vectors per slot; the counter has six bits");
    if constexpr (QT == 1) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(slot[0]) : "n"(LATER) : "memory");
    if constexpr (QT == 2) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(slot[0]), "+v"(slot[1]) : "n"(LATER) : "memory");
    if constexpr (QT == 3) asm volatile("s_waitcnt vmcnt(%3)" : "+v"(slot[0]), "+v"(slot[1]), "+v"(slot[2]) : "n"(LATER) : "memory");
    if constexpr (QT == 4) asm volatile("s_waitcnt vmcnt(%4)" : "+v"(slot[0]), "+v"(slot[1]), "+v"(slot[2]), "+v"(slot[3]) : "n"(LATER) : "memory");
}

// MR: MFMA row tiles per workgroup.  Every wavefront multiplies all 16 * MR panel rows with its columns, so
// an activation vector loaded once feeds MR MFMAs.
// P16: the panel is kept as bf16 (short rows: K <= 576), so that the contraction reads its A operands as they are.
// KIND: how the contraction addresses the activations.
enum { kTaps = 0,        // input channels a multiple of 8: a lane's 8 consecutive k lie under one kernel tap
       kPointwise = 1,   // as kTaps with a 1 x 1 kernel and no padding: one pixel per column, nothing outside the image
       kGeneric = 2,     // any number of input channels (NHWC): every activation is addressed on its own
       kPointwiseRing = 3,     // as kPointwise with input channels a multiple of 32 * D: D steps' activations in flight
       kTapsPatch = 4,         // as kTaps with input channels a multiple of 32: the activations under all kernel taps of a
                               // round of pixels are staged in LDS once per 32 input channels
       kTapsRing = 5,          // as kTaps with input channels a multiple of 32 * D: D steps' activations in flight
       kGenericPatch = 6,      // as kGeneric when whole image rows are multiples of 16 bytes: the image rows under a round
                               // of pixels are staged in LDS, zero padding included, and gathered from there
       kTapsRows = 7 };        // as kTapsRing for kernels three taps wide: the three taps of a kernel row and 32 channels
                               // are loaded together, so that the L1 serves what they share
// D (kPointwiseRing only): steps of 32 input channels whose activation loads are in flight at any time.
template <int KIND, uint32_t MR, bool P16, uint32_t D>
__global__ __launch_bounds__(kThreads) void conv_fused_kernel(ConvParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t L = 1u << p.table_log;
    const uint32_t ahead_bytes = 16u * L;                         // 2 L look-ahead entries of two words
    uint8_t* ahead = lds;
    uint32_t* stage = reinterpret_cast<uint32_t*>(lds + ahead_bytes);
    uint8_t* panel = lds + p.panel_off;
    constexpr uint32_t kElem = P16 ? 2u : 1u;                     // bytes per panel element
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // The chip hands consecutive workgroups to its eight dies in turn and every die has its own L2: workgroup
    // blockIdx.x is the (blockIdx.x / 8)-th of die blockIdx.x % 8.  Numbering the workgroups die after die, the
    // panels of one range of pixels follow each other on one die, whose L2 then fetches those activations once
    // for all of them.  (Any one-to-one numbering is correct; this one is for the cache.)
    constexpr uint32_t kDies = 8;
    const uint32_t per_die = gridDim.x / kDies, extra = gridDim.x % kDies, die = blockIdx.x % kDies;
    const uint32_t unit = die * per_die + min(die, extra) + blockIdx.x / kDies;
    const uint32_t mtile = unit % p.n_mtiles, split = unit / p.n_mtiles;

    // ---- phase 1: the layer's look-ahead entries into LDS, then this workgroup's 16 * MR weight rows.
    // Every global read that depends only on the kernel's arguments is issued before any is waited for: the
    // descriptors of this wavefront's chunks (lane i: its i-th chunk, panel chunk wave + i * kWaves), the layer's
    // quantizer, the triple of the last state (it carries the layer's dominant symbol if there is one), the
    // table (one 16-byte row per state: the entries for both values of the peeked bit; up to six rows per thread).
    const uint32_t cpp = p.chunks_per_panel;
    const anszp_chunk_t* panel_chunks = p.chunks + uint64_t(mtile) * cpp;
    const anszp_chunk_t held = panel_chunks[min(wave + min(lane, kMaxMine - 1u) * kWaves, cpp - 1u)];
    const uint32_t* table_src = p.tables + p.layer_id * table_stride_words(p.table_log);
    const anszp_layer_t lay = p.layers[p.layer_id];
    const uint32_t top = table_src[table_triples_offset(p.table_log) + L - 1u];
    constexpr uint32_t kTableLoads = ((1u << ANSZP_MAX_TABLE_LOG) + kThreads - 1u) / kThreads;
    const words4* tsrc = reinterpret_cast<const words4*>(table_src + table_lookahead_offset(p.table_log));
    words4 tv[kTableLoads];
#pragma unroll
    for (uint32_t u = 0; u < kTableLoads; ++u) tv[u] = tsrc[min(tid + u * kThreads, L - 1u)];

    auto desc_of = [&](uint32_t i) {                              // this wavefront's i-th chunk (i uniform)
        ChunkDesc c;
        const uint32_t layer_id = __builtin_amdgcn_readlane(held.layer_id, i);
        c.n_symbols = __builtin_amdgcn_readlane(held.n_symbols, i);
        c.payload_words = __builtin_amdgcn_readlane(held.payload_words, i);
        c.stream_offset = __builtin_amdgcn_readlane(held.stream_offset, i);
        c.payload_offset = uint64_t(uint32_t(__builtin_amdgcn_readlane(uint32_t(held.payload_offset), i))) |
                           uint64_t(uint32_t(__builtin_amdgcn_readlane(uint32_t(held.payload_offset >> 32), i))) << 32;
        c.ok = layer_id == p.layer_id && c.n_symbols == p.rows_per_chunk * p.K && (c.payload_offset & 3u) == 0 &&
               c.payload_offset <= p.payload_words && c.payload_words <= p.payload_words - c.payload_offset &&
               uint64_t(c.stream_offset) + p.n_streams <= p.n_stream_hdr;
        c.staged = c.payload_words + 2u <= kStageWords;           // two zero words behind the chunk's own
        return c;
    };
    auto fetch = [&](const ChunkDesc& c, ChunkData& d) {          // from clamped, always valid addresses
        d.hdr = 0u;
        d.q0 = d.q1 = words4{0u, 0u, 0u, 0u};
        d.tail = 0u;
        if (!c.ok) return;                                        // uniform
        if (lane < p.n_streams) d.hdr = p.stream_hdr[c.stream_offset + lane];
        const uint32_t quads = c.payload_words >> 2;
        if (c.staged && c.payload_words) {
            const uint32_t* words = p.payload + c.payload_offset;
            if (quads) {
                d.q0 = reinterpret_cast<const words4*>(words)[min(lane, quads - 1u)];
                d.q1 = reinterpret_cast<const words4*>(words)[min(lane + kWave, quads - 1u)];
            }
            const uint32_t tail_at = (quads << 2) + lane;
            if (lane < 3u && tail_at < c.payload_words) d.tail = words[tail_at];
        }
    };
    const uint32_t n_mine = wave < cpp ? (cpp - wave + kWaves - 1u) / kWaves : 0u;
    ChunkDesc cur{};
    ChunkData cur_data{};
    if (n_mine) {
        cur = desc_of(0u);
        fetch(cur, cur_data);
    }
    {
        // (done while the table is still on its way: only the quantizer and the last state's triple are needed)
        // The panel starts as the layer's dominant symbol everywhere (decoding writes only the other symbols);
        // also the columns from K to a row's end and the 64 bytes behind the last row, which the contraction
        // reads (the last 32 k of a row tile or of a kernel tap) against activations that are zero: as bf16
        // values they must be finite, whatever an earlier kernel left in LDS.
        const uint32_t dominant = top >> 24;
        uint32_t fill = dominant * 0x01010101u;
        if constexpr (P16) {
            const uint32_t h = __float_as_uint(static_cast<float>(int32_t(dominant) - int32_t(lay.zero_point))) >> 16;
            fill = h | h << 16;
        }
        const uint32_t panel_quads = (kRows * MR * p.row_stride * kElem + 64u) / 16u;
        for (uint32_t i = tid; i < panel_quads; i += kThreads) reinterpret_cast<words4*>(panel)[i] = words4{fill, fill, fill, fill};
    }
#pragma unroll
    for (uint32_t u = 0; u < kTableLoads; ++u)
        if (tid + u * kThreads < L) reinterpret_cast<words4*>(ahead)[tid + u * kThreads] = tv[u];
    __syncthreads();
    uint32_t err = (lay.channel_len != 0 && lay.channel_len != p.K) ? ANSZP_ST_BAD_DESC : 0u;   // scales per output channel only
    for (uint32_t i = 0; i < n_mine; ++i) {
        // the next chunk's words are asked for before this one is decoded
        ChunkDesc nxt{};
        ChunkData nxt_data{};
        if (i + 1u < n_mine) {
            nxt = desc_of(i + 1u);
            fetch(nxt, nxt_data);
        }
        const uint32_t j = wave + i * kWaves;
        if (!cur.ok) err |= ANSZP_ST_BAD_DESC;                    // its rows stay the dominant symbol
        else err |= decode_chunk_to_panel<P16>(p, cur, cur_data, ahead, ahead_bytes - 8u, stage + wave * kStageWords,
                                               panel + j * p.rows_per_chunk * p.row_stride * kElem, lane, int32_t(lay.zero_point));
        cur = nxt;
        cur_data = nxt_data;
    }
    err = wave_or(err);
    if (err && lane == 0) report(p.status, err);
    __syncthreads();
    // kGeneric: what every k of the reduction means, worked out once (the table and the staging room are free now):
    // two words per k, the offset of its activation from the one under the first tap's first channel, and its
    // kernel row | kernel column << 8 (a column no image has for the k beyond K)
    [[maybe_unused]] uint32_t* k_table = reinterpret_cast<uint32_t*>(lds);
    if constexpr (KIND == kGeneric) {
        for (uint32_t k = tid; k < ((p.K + 31u) & ~31u); k += kThreads) {
            const uint32_t tap = k / p.cin, c = k % p.cin;
            const uint32_t r = tap / p.kw, sx = tap % p.kw;
            k_table[2u * k] = (r * p.in_w + sx) * p.cin + c;
            k_table[2u * k + 1u] = k < p.K ? (r | sx << 8) : 0xFFFFFF00u;
        }
        __syncthreads();
    }

    // kPointwiseRing, kTapsRing (which need no other LDS in phase 2): a panel of symbol bytes is first widened in
    // place to bf16 values q - z (the table and the staging room are free now and the widened panel starts at the
    // beginning of LDS): every thread takes its 16-byte pieces into registers, all wait, then every piece is
    // written back as 32 bytes.  Returns where the bf16 panel starts.
    [[maybe_unused]] auto widened_panel = [&]() -> const uint8_t* {
        if constexpr (P16) {
            return panel;
        } else {
            const uint32_t n_pieces = (kRows * MR * p.row_stride + 64u) / 16u;     // the host made sure: <= kWidenPieces * kThreads
            const float zf = static_cast<float>(lay.zero_point);
            words4 held_q[kWidenPieces];
#pragma unroll
            for (uint32_t u = 0; u < kWidenPieces; ++u)
                held_q[u] = reinterpret_cast<const words4*>(panel)[min(tid + u * kThreads, n_pieces - 1u)];
            __syncthreads();
#pragma unroll
            for (uint32_t u = 0; u < kWidenPieces; ++u) {
                const uint32_t i = tid + u * kThreads;
                if (i < n_pieces) {
                    bf16x8* dst = reinterpret_cast<bf16x8*>(lds + 32u * i);
                    dst[0] = weights_of(words2{held_q[u].x, held_q[u].y}, zf);
                    dst[1] = weights_of(words2{held_q[u].z, held_q[u].w}, zf);
                }
            }
            __syncthreads();
            return lds;
        }
    };
    if constexpr (KIND == kPointwiseRing) {
        // ---- phase 2 for 1 x 1 kernels without padding whose input channels are a multiple of 32 * D.
        const uint8_t* a_base = widened_panel();
        const uint32_t col = lane & 15u, kg = lane >> 4;          // MFMA operand layout: row or column, group of 8 k
        const uint8_t* a_row = a_base + (col * p.row_stride + 8u * kg) * 2u;
        const uint32_t tile_stride = kRows * p.row_stride * 2u;
        const uint32_t n_steps = p.cin / 32u;                     // a multiple of D
        const uint32_t step_elems = 4u * p.x_block;               // from one step's activation vector to the next's
        const uint32_t split_begin = split * p.pixels_per_split;
        const uint32_t split_end = min(split_begin + p.pixels_per_split, p.n_pixels);
        // The workgroup's column tiles of 16 pixels are dealt out in rounds of at most 4 * kWaves, and a round's tiles
        // evenly over the wavefronts: every wavefront has one to four neighbouring tiles (as many loads in flight
        // on as many SIMDs as possible: the loop is bound by the activations' way from the L2).
        const uint32_t tiles = (split_end - split_begin + 15u) / 16u;
        const uint32_t n_rounds = (tiles + 4u * kWaves - 1u) / (4u * kWaves);
        const uint32_t round_tiles = n_rounds ? (tiles + n_rounds - 1u) / n_rounds : 0u;
        auto block = [&](uint32_t pix0, uint32_t block_end, auto tiles_here) {
            constexpr uint32_t QT = decltype(tiles_here)::value;
            // B: lane holds column lane % 16 of each of the block's QT column tiles; a column beyond the block
            // reads the block's first pixel (every load is unconditional) and is not stored
            bool valid[4] = {false, false, false, false};
            uint32_t out_at[4] = {0u, 0u, 0u, 0u};
            const uint16_t* px[QT];
#pragma unroll
            for (uint32_t q = 0; q < QT; ++q) {
                const uint32_t pix = pix0 + q * 16u + col;
                valid[q] = pix < block_end;
                const uint32_t n = valid[q] ? pix : pix0;
                const uint32_t wo = n % p.out_w, t = n / p.out_w;
                const uint32_t ho = t % p.out_h, b = t / p.out_h;
                px[q] = p.x + (b * p.in_h * p.in_w * p.cin + (ho * p.stride * p.in_w + wo * p.stride) * p.x_pixel + kg * p.x_block);
                out_at[q] = b * p.out_h * p.out_w * p.cout + (ho * p.out_w + wo) * p.y_pixel;
            }
            floatx4 acc[MR][4];
#pragma unroll
            for (uint32_t m = 0; m < MR; ++m)
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) acc[m][q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
            // A ring of D steps' activation vectors: a step's slot is refilled, for the step D later, as soon as its
            // MFMAs are issued (ring_request / ring_arrived: by hand).
            words4 ring[D][QT];
            auto multiply = [&](uint32_t step, uint32_t d) {
#pragma unroll
                for (uint32_t m = 0; m < MR; ++m) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_row + m * tile_stride + step * 64u);
#pragma unroll
                    for (uint32_t q = 0; q < QT; ++q)
                        acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, ring[d][q]), acc[m][q], 0, 0, 0);
                }
            };
#pragma unroll
            for (uint32_t d = 0; d < D; ++d) ring_request<QT>(ring[d], px, d * step_elems);
            uint32_t base = 0;
            for (; base + D < n_steps; base += D) {               // every group of D steps but the last
#pragma unroll
                for (uint32_t d = 0; d < D; ++d) {
                    ring_arrived<QT, (D - 1u) * QT>(ring[d]);
                    multiply(base + d, d);
                    ring_request<QT>(ring[d], px, (base + d + D) * step_elems);
                }
            }
            // the last group: nothing is asked for any more, so fewer loads follow a slot's own
            static_assert(D == 2 || D == 4, "written out for two and four slots");
            if constexpr (D == 2) {
                ring_arrived<QT, QT>(ring[0]);
                multiply(base, 0u);
                ring_arrived<QT, 0u>(ring[1]);
                multiply(base + 1u, 1u);
            } else {
                ring_arrived<QT, 3u * QT>(ring[0]);
                multiply(base, 0u);
                ring_arrived<QT, 2u * QT>(ring[1]);
                multiply(base + 1u, 1u);
                ring_arrived<QT, QT>(ring[2]);
                multiply(base + 2u, 2u);
                ring_arrived<QT, 0u>(ring[3]);
                multiply(base + 3u, 3u);
            }
            store_tiles<MR>(p, lay, mtile, kg, acc, valid, out_at);
        };
        for (uint32_t round = 0; round < n_rounds; ++round) {
            const uint32_t t0 = round * round_tiles;
            if (t0 >= tiles) break;
            const uint32_t tn = min(round_tiles, tiles - t0);
            const uint32_t w_begin = t0 + tn * wave / kWaves, w_end = t0 + tn * (wave + 1u) / kWaves;   // this wavefront's tiles
            const uint32_t pix0 = split_begin + 16u * w_begin, block_end = min(split_begin + 16u * w_end, split_end);
            switch (w_end - w_begin) {                            // uniform
                case 1: block(pix0, block_end, std::integral_constant<uint32_t, 1>{}); break;
                case 2: block(pix0, block_end, std::integral_constant<uint32_t, 2>{}); break;
                case 3: block(pix0, block_end, std::integral_constant<uint32_t, 3>{}); break;
                case 4: block(pix0, block_end, std::integral_constant<uint32_t, 4>{}); break;
                default: break;
            }
        }
        return;
    }

    if constexpr (KIND == kGenericPatch) {
        // ---- phase 2 for any number of input channels (NHWC) when an image row is a multiple of 16 bytes: the
        // workgroup's column tiles are taken in rounds (dealt out as for kPointwiseRing); the image rows under a
        // round's pixels go to LDS as they are, 16 bytes at a time, each behind 32 bytes whose upper part is the
        // left zero padding, followed by the right one; rows above and below an image are zeros.  A lane then
        // gathers its 8 k per column from LDS: the pixel's place plus an offset per k that is worked out once (a
        // table in LDS in front of the rows).  Nothing tests for the image's border.
        const uint32_t col = lane & 15u, kg = lane >> 4;          // MFMA operand layout: row or column, group of 8 k
        const uint8_t* a_row = panel + (col * p.row_stride + 8u * kg) * kElem;
        const uint32_t tile_stride = kRows * p.row_stride * kElem;
        const float zf = static_cast<float>(lay.zero_point);
        const uint32_t S = p.stride, Hp = p.in_h + 2u * p.pad;
        const uint32_t Kp = (p.K + 31u) & ~31u;
        const uint32_t row_bytes = p.in_w * p.cin * 2u, pieces_per_row = row_bytes / 16u;
        const uint32_t edge_pieces = 2u + (p.row_pitch - 32u - row_bytes) / 16u;   // the 16-byte pieces of a row that hold no image
        uint32_t* k_offset = reinterpret_cast<uint32_t*>(lds);    // [Kp]: bytes from a pixel's first tap, first channel, to k's activation
        uint8_t* rows_at = lds + p.patch_off;
        for (uint32_t k = tid; k < Kp; k += kThreads) {
            const uint32_t tap = k / p.cin, c = k % p.cin;
            const uint32_t r = tap / p.kw, sx = tap % p.kw;
            k_offset[k] = k < p.K ? r * p.row_pitch + (sx * p.cin + c) * 2u : 0u;
        }
        const uint32_t split_begin = split * p.pixels_per_split;
        const uint32_t split_end = min(split_begin + p.pixels_per_split, p.n_pixels);
        const uint32_t tiles = (split_end - split_begin + 15u) / 16u;
        const uint32_t n_rounds = (tiles + 4u * kWaves - 1u) / (4u * kWaves);
        const uint32_t round_tiles = n_rounds ? (tiles + n_rounds - 1u) / n_rounds : 0u;
        constexpr uint32_t kPieces = kPatchPieces;
        for (uint32_t round = 0; round < n_rounds; ++round) {
            const uint32_t t0 = round * round_tiles;
            if (t0 >= tiles) break;
            const uint32_t tn = min(round_tiles, tiles - t0);
            const uint32_t round0 = split_begin + 16u * t0, round_end = min(round0 + 16u * tn, split_end);
            // the staged rows: flat index b * Hp + padded row, from the first pixel's first tap to the last pixel's last
            const uint32_t first_row = round0 / p.out_w, last_row = (round_end - 1u) / p.out_w;   // flat output rows b * out_h + ho
            const uint32_t pr0 = (first_row / p.out_h) * Hp + (first_row % p.out_h) * S;
            const uint32_t pr_last = (last_row / p.out_h) * Hp + (last_row % p.out_h) * S + p.kh - 1u;
            const uint32_t n_rows = pr_last - pr0 + 1u;
            const uint32_t n_pieces = n_rows * pieces_per_row;
            if (n_pieces > kPieces * kThreads) {                  // the host sized the rounds so that this cannot happen
                if (tid == 0) report(p.status, ANSZP_ST_INTERNAL);
                return;                                           // uniform
            }
            __syncthreads();                                      // the previous round's rows have been read (and k_offset written)
            words4 held_x[kPieces];
            uint32_t dst[kPieces];
#pragma unroll
            for (uint32_t u = 0; u < kPieces; ++u) {
                const uint32_t i = tid + u * kThreads;
                held_x[u] = words4{0u, 0u, 0u, 0u};
                dst[u] = 0xFFFFFFFFu;
                if (i < n_pieces) {
                    const uint32_t piece = i % pieces_per_row, row = i / pieces_per_row;
                    const uint32_t pra = pr0 + row;
                    const uint32_t b = pra / Hp, h = pra % Hp - p.pad;                      // unsigned: above the image wraps around
                    dst[u] = row * p.row_pitch + 32u + piece * 16u;
                    if (h < p.in_h) held_x[u] = reinterpret_cast<const words4*>(p.x + (b * p.in_h + h) * p.in_w * p.cin)[piece];
                }
            }
            for (uint32_t i = tid; i < n_rows * edge_pieces; i += kThreads) {
                const uint32_t e = i % edge_pieces, row = i / edge_pieces;
                const uint32_t at = row * p.row_pitch + (e < 2u ? e * 16u : 32u + row_bytes + (e - 2u) * 16u);
                *reinterpret_cast<words4*>(rows_at + at) = words4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (uint32_t u = 0; u < kPieces; ++u)
                if (dst[u] != 0xFFFFFFFFu) *reinterpret_cast<words4*>(rows_at + dst[u]) = held_x[u];
            __syncthreads();

            const uint32_t w_begin = t0 + tn * wave / kWaves, w_end = t0 + tn * (wave + 1u) / kWaves;   // this wavefront's tiles
            const uint32_t pix0 = split_begin + 16u * w_begin, block_end = min(split_begin + 16u * w_end, split_end);
            auto block = [&](auto tiles_here) {
                constexpr uint32_t QT = decltype(tiles_here)::value;
                bool valid[4] = {false, false, false, false};
                uint32_t out_at[4] = {0u, 0u, 0u, 0u};
                uint32_t at_rows[QT];                             // byte of the pixel's first tap, first channel (may lie in the left padding)
#pragma unroll
                for (uint32_t q = 0; q < QT; ++q) {
                    const uint32_t pix = pix0 + q * 16u + col;
                    valid[q] = pix < block_end;
                    const uint32_t n = valid[q] ? pix : pix0;     // a column beyond the block stands on its first pixel
                    const uint32_t wo = n % p.out_w, t = n / p.out_w;
                    const uint32_t ho = t % p.out_h, b = t / p.out_h;
                    at_rows[q] = (b * Hp + ho * S - pr0) * p.row_pitch + 32u + (wo * S * p.cin) * 2u - p.pad * p.cin * 2u;
                    out_at[q] = b * p.out_h * p.out_w * p.cout + (ho * p.out_w + wo) * p.y_pixel;
                }
                floatx4 acc[MR][4];
#pragma unroll
                for (uint32_t m = 0; m < MR; ++m)
#pragma unroll
                    for (uint32_t q = 0; q < 4; ++q) acc[m][q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
                for (uint32_t k0 = 0; k0 < Kp; k0 += 32u) {
                    const uint32_t kbase = k0 + 8u * kg;
                    const words4 off_lo = *reinterpret_cast<const words4*>(k_offset + kbase);
                    const words4 off_hi = *reinterpret_cast<const words4*>(k_offset + kbase + 4u);
                    const uint32_t off[8] = {off_lo.x, off_lo.y, off_lo.z, off_lo.w, off_hi.x, off_hi.y, off_hi.z, off_hi.w};
                    words4 b[QT];
#pragma unroll
                    for (uint32_t q = 0; q < QT; ++q) {
                        uint32_t v[8];
#pragma unroll
                        for (uint32_t j = 0; j < 8; ++j) {
                            v[j] = *reinterpret_cast<const uint16_t*>(rows_at + at_rows[q] + off[j]);
                            if (kbase + j >= p.K) v[j] = 0u;      // beyond the reduction (the last step only)
                        }
                        b[q] = words4{v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16};
                    }
#pragma unroll
                    for (uint32_t m = 0; m < MR; ++m) {
                        bf16x8 a;
                        if constexpr (P16) a = *reinterpret_cast<const bf16x8*>(a_row + m * tile_stride + k0 * 2u);
                        else a = weights_of(*reinterpret_cast<const words2*>(a_row + m * tile_stride + k0), zf);
#pragma unroll
                        for (uint32_t q = 0; q < QT; ++q)
                            acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b[q]), acc[m][q], 0, 0, 0);
                    }
                }
                store_tiles<MR>(p, lay, mtile, kg, acc, valid, out_at);
            };
            switch (w_end - w_begin) {                            // uniform
                case 1: block(std::integral_constant<uint32_t, 1>{}); break;
                case 2: block(std::integral_constant<uint32_t, 2>{}); break;
                case 3: block(std::integral_constant<uint32_t, 3>{}); break;
                case 4: block(std::integral_constant<uint32_t, 4>{}); break;
                default: break;
            }
        }
        return;
    }

    if constexpr (KIND == kTapsRows) {
        // ---- phase 2 for kernels three taps wide whose input channels are a multiple of 64 (and that stage no patch).
        // A step is a kernel row, 32 input channels and the row's three taps; two steps' activation vectors are in
        // flight (hand-issued loads as for kPointwiseRing, each tap of a step waited for on its own).  Kernel rows
        // outermost, channels next, the three taps innermost: the taps of a row read the same pixels shifted by one
        // (stride 1) or alternate halves of the same lines (stride 2), and asked for together they cost the L1 one
        // fetch of a line instead of up to three.  A column whose pixel lies outside the image under a tap reads
        // zero_page with a step stride of zero.
        const uint32_t col = lane & 15u, kg = lane >> 4;          // MFMA operand layout: row or column, group of 8 k
        const uint8_t* a_row = widened_panel() + (col * p.row_stride + 8u * kg) * 2u;
        const uint32_t tile_stride = kRows * p.row_stride * 2u;
        const uint32_t steps_per_row = p.cin / 32u;               // even
        const uint32_t n_steps = p.kh * steps_per_row;
        const uint32_t split_begin = split * p.pixels_per_split;
        const uint32_t split_end = min(split_begin + p.pixels_per_split, p.n_pixels);
        const uint32_t tiles = (split_end - split_begin + 15u) / 16u;
        constexpr uint32_t kTilesMost = MR == 4 ? 2u : 3u;        // column tiles per wavefront and round: what the registers hold
        const uint32_t n_rounds = (tiles + kTilesMost * kWaves - 1u) / (kTilesMost * kWaves);
        const uint32_t round_tiles = n_rounds ? (tiles + n_rounds - 1u) / n_rounds : 0u;
        const uint16_t* zeros = reinterpret_cast<const uint16_t*>(zero_page);
        auto block = [&](uint32_t pix0, uint32_t block_end, auto tiles_here) {
            constexpr uint32_t QT = decltype(tiles_here)::value;
            bool valid[4] = {false, false, false, false};
            uint32_t out_at[4] = {0u, 0u, 0u, 0u};
            int32_t h0[QT], w0[QT];
            uint32_t img[QT];
#pragma unroll
            for (uint32_t q = 0; q < QT; ++q) {
                const uint32_t pix = pix0 + q * 16u + col;
                valid[q] = pix < block_end;
                const uint32_t n = valid[q] ? pix : pix0;         // a column beyond the block stands on its first pixel
                const uint32_t wo = n % p.out_w, t = n / p.out_w;
                const uint32_t ho = t % p.out_h, b = t / p.out_h;
                h0[q] = int32_t(ho * p.stride) - int32_t(p.pad);
                w0[q] = int32_t(wo * p.stride) - int32_t(p.pad);
                img[q] = b * p.in_h * p.in_w * p.cin;
                out_at[q] = b * p.out_h * p.out_w * p.cout + (ho * p.out_w + wo) * p.y_pixel;
            }
            floatx4 acc[MR][4];
#pragma unroll
            for (uint32_t m = 0; m < MR; ++m)
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) acc[m][q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
            // where the requests of the kernel row being asked for read, per tap and column
            const uint16_t* tap_ptr[3][QT];
            uint32_t tap_step[3][QT];
            auto enter_row = [&](uint32_t r) {
#pragma unroll
                for (uint32_t q = 0; q < QT; ++q) {
                    const int32_t h = h0[q] + int32_t(r);
                    const bool row_inside = uint32_t(h) < p.in_h;
#pragma unroll
                    for (uint32_t sx = 0; sx < 3; ++sx) {
                        const int32_t w = w0[q] + int32_t(sx);
                        const bool inside = row_inside && uint32_t(w) < p.in_w;
                        tap_ptr[sx][q] = inside ? p.x + (img[q] + (uint32_t(h) * p.in_w + uint32_t(w)) * p.x_pixel + kg * p.x_block) : zeros;
                        tap_step[sx][q] = inside ? 4u * p.x_block : 0u;
                    }
                }
            };
            words4 ring[2][3][QT];
            auto request = [&](uint32_t slot, uint32_t step_in_row) {
#pragma unroll
                for (uint32_t sx = 0; sx < 3; ++sx) {
                    const uint16_t* from[QT];
#pragma unroll
                    for (uint32_t q = 0; q < QT; ++q) from[q] = tap_ptr[sx][q] + __umul24(step_in_row, tap_step[sx][q]);
                    ring_request<QT>(ring[slot][sx], from, 0u);
                }
            };
            auto multiply = [&](uint32_t k_first, const words4 (&b)[QT]) {   // k_first: the step's first k under this tap (its panel column)
#pragma unroll
                for (uint32_t m = 0; m < MR; ++m) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_row + m * tile_stride + k_first * 2u);
#pragma unroll
                    for (uint32_t q = 0; q < QT; ++q)
                        acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b[q]), acc[m][q], 0, 0, 0);
                }
            };
            // the cursor of the requests runs two steps ahead of the cursor of the multiplications
            uint32_t req_row = 0, req_step = 0;
            auto request_next = [&](uint32_t slot) {
                request(slot, req_step);
                if (++req_step == steps_per_row) {                // uniform
                    req_step = 0;
                    ++req_row;
                    if (req_row < p.kh) enter_row(req_row);
                }
            };
            enter_row(0u);
            request_next(0u);
            request_next(1u);
            uint32_t row = 0, step = 0;                           // of the step being multiplied
            auto use = [&](uint32_t slot, auto other_slot_pending) {
                constexpr uint32_t kOther = decltype(other_slot_pending)::value ? 3u * QT : 0u;   // loads asked for after this slot's
                const uint32_t k_row = row * 3u * p.cin + step * 32u;
                ring_arrived<QT, 2u * QT + kOther>(ring[slot][0]);
                multiply(k_row, ring[slot][0]);
                ring_arrived<QT, QT + kOther>(ring[slot][1]);
                multiply(k_row + p.cin, ring[slot][1]);
                ring_arrived<QT, kOther>(ring[slot][2]);
                multiply(k_row + 2u * p.cin, ring[slot][2]);
                if (++step == steps_per_row) { step = 0; ++row; }
            };
            for (uint32_t t = 0; t + 2u < n_steps; t += 2u) {     // every pair of steps but the last
                use(0u, std::true_type{});
                request_next(0u);
                use(1u, std::true_type{});
                request_next(1u);
            }
            use(0u, std::true_type{});
            use(1u, std::false_type{});
            store_tiles<MR>(p, lay, mtile, kg, acc, valid, out_at);
        };
        for (uint32_t round = 0; round < n_rounds; ++round) {
            const uint32_t t0 = round * round_tiles;
            if (t0 >= tiles) break;
            const uint32_t tn = min(round_tiles, tiles - t0);
            const uint32_t w_begin = t0 + tn * wave / kWaves, w_end = t0 + tn * (wave + 1u) / kWaves;   // this wavefront's tiles
            const uint32_t pix0 = split_begin + 16u * w_begin, block_end = min(split_begin + 16u * w_end, split_end);
            switch (w_end - w_begin) {                            // uniform
                case 1: block(pix0, block_end, std::integral_constant<uint32_t, 1>{}); break;
                case 2: block(pix0, block_end, std::integral_constant<uint32_t, 2>{}); break;
                case 3: if constexpr (kTilesMost >= 3) block(pix0, block_end, std::integral_constant<uint32_t, 3>{}); break;
                default: break;
            }
        }
        return;
    }

    if constexpr (KIND == kTapsRing) {
        // ---- phase 2 for kernels of several taps whose input channels are a multiple of 32 * D: steps of 32 k, kernel
        // taps outermost, in groups of D steps that never straddle a tap; tiles dealt out and loads issued as for
        // kPointwiseRing.  A column whose pixel lies outside the image under a tap reads zero_page for that tap (with a
        // step stride of zero), so every load is unconditional.
        const uint32_t col = lane & 15u, kg = lane >> 4;          // MFMA operand layout: row or column, group of 8 k
        const uint8_t* a_row = widened_panel() + (col * p.row_stride + 8u * kg) * 2u;   // (the host keeps this kind for panels that can be widened)
        const uint32_t tile_stride = kRows * p.row_stride * 2u;
        const uint32_t groups_per_tap = p.cin / (32u * D);
        const uint32_t n_groups = p.kh * p.kw * groups_per_tap;
        const uint32_t split_begin = split * p.pixels_per_split;
        const uint32_t split_end = min(split_begin + p.pixels_per_split, p.n_pixels);
        const uint32_t tiles = (split_end - split_begin + 15u) / 16u;
        const uint32_t n_rounds = (tiles + 4u * kWaves - 1u) / (4u * kWaves);
        const uint32_t round_tiles = n_rounds ? (tiles + n_rounds - 1u) / n_rounds : 0u;
        const uint16_t* zeros = reinterpret_cast<const uint16_t*>(zero_page);
        auto block = [&](uint32_t pix0, uint32_t block_end, auto tiles_here) {
            constexpr uint32_t QT = decltype(tiles_here)::value;
            bool valid[4] = {false, false, false, false};
            uint32_t out_at[4] = {0u, 0u, 0u, 0u};
            int32_t h0[QT], w0[QT];
            uint32_t img[QT];
#pragma unroll
            for (uint32_t q = 0; q < QT; ++q) {
                const uint32_t pix = pix0 + q * 16u + col;
                valid[q] = pix < block_end;
                const uint32_t n = valid[q] ? pix : pix0;         // a column beyond the block stands on its first pixel
                const uint32_t wo = n % p.out_w, t = n / p.out_w;
                const uint32_t ho = t % p.out_h, b = t / p.out_h;
                h0[q] = int32_t(ho * p.stride) - int32_t(p.pad);
                w0[q] = int32_t(wo * p.stride) - int32_t(p.pad);
                img[q] = b * p.in_h * p.in_w * p.cin;
                out_at[q] = b * p.out_h * p.out_w * p.cout + (ho * p.out_w + wo) * p.y_pixel;
            }
            floatx4 acc[MR][4];
#pragma unroll
            for (uint32_t m = 0; m < MR; ++m)
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) acc[m][q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
            // where the requests of the group being asked for read: the tap's pixel of every column, and how far it
            // is from one step's vector to the next's (nothing, on the zero page)
            const uint16_t* tap_ptr[QT];
            uint32_t tap_step[QT];
            auto enter_tap = [&](uint32_t tap) {
                const uint32_t r = tap / p.kw, sx = tap % p.kw;
#pragma unroll
                for (uint32_t q = 0; q < QT; ++q) {
                    const int32_t h = h0[q] + int32_t(r), w = w0[q] + int32_t(sx);
                    const bool inside = uint32_t(h) < p.in_h && uint32_t(w) < p.in_w;
                    tap_ptr[q] = inside ? p.x + (img[q] + (uint32_t(h) * p.in_w + uint32_t(w)) * p.x_pixel + kg * p.x_block) : zeros;
                    tap_step[q] = inside ? 4u * p.x_block : 0u;
                }
            };
            words4 ring[D][QT];
            auto request = [&](uint32_t d, uint32_t step_in_tap) {
                const uint16_t* from[QT];
#pragma unroll
                for (uint32_t q = 0; q < QT; ++q) from[q] = tap_ptr[q] + __umul24(step_in_tap, tap_step[q]);
                ring_request<QT>(ring[d], from, 0u);
            };
            auto multiply = [&](uint32_t k_first, uint32_t d) {   // k_first: the step's first k (its panel column)
#pragma unroll
                for (uint32_t m = 0; m < MR; ++m) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_row + m * tile_stride + k_first * 2u);
#pragma unroll
                    for (uint32_t q = 0; q < QT; ++q)
                        acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, ring[d][q]), acc[m][q], 0, 0, 0);
                }
            };
            enter_tap(0u);
#pragma unroll
            for (uint32_t d = 0; d < D; ++d) request(d, d);
            uint32_t tap = 0, group_in_tap = 0;                   // of the group being multiplied
            for (uint32_t g = 0; g + 1u < n_groups; ++g) {        // every group but the last
                uint32_t next_tap = tap, next_in_tap = group_in_tap + 1u;
                if (next_in_tap == groups_per_tap) {              // uniform
                    next_in_tap = 0;
                    ++next_tap;
                    enter_tap(next_tap);
                }
                const uint32_t k_group = tap * p.cin + group_in_tap * (32u * D);
#pragma unroll
                for (uint32_t d = 0; d < D; ++d) {
                    ring_arrived<QT, (D - 1u) * QT>(ring[d]);
                    multiply(k_group + 32u * d, d);
                    request(d, next_in_tap * D + d);
                }
                tap = next_tap;
                group_in_tap = next_in_tap;
            }
            const uint32_t k_group = tap * p.cin + group_in_tap * (32u * D);
            static_assert(D == 2 || D == 4, "written out for two and four slots");
            if constexpr (D == 2) {
                ring_arrived<QT, QT>(ring[0]);
                multiply(k_group, 0u);
                ring_arrived<QT, 0u>(ring[1]);
                multiply(k_group + 32u, 1u);
            } else {
                ring_arrived<QT, 3u * QT>(ring[0]);
                multiply(k_group, 0u);
                ring_arrived<QT, 2u * QT>(ring[1]);
                multiply(k_group + 32u, 1u);
                ring_arrived<QT, QT>(ring[2]);
                multiply(k_group + 64u, 2u);
                ring_arrived<QT, 0u>(ring[3]);
                multiply(k_group + 96u, 3u);
            }
            store_tiles<MR>(p, lay, mtile, kg, acc, valid, out_at);
        };
        for (uint32_t round = 0; round < n_rounds; ++round) {
            const uint32_t t0 = round * round_tiles;
            if (t0 >= tiles) break;
            const uint32_t tn = min(round_tiles, tiles - t0);
            const uint32_t w_begin = t0 + tn * wave / kWaves, w_end = t0 + tn * (wave + 1u) / kWaves;   // this wavefront's tiles
            const uint32_t pix0 = split_begin + 16u * w_begin, block_end = min(split_begin + 16u * w_end, split_end);
            switch (w_end - w_begin) {                            // uniform
                case 1: block(pix0, block_end, std::integral_constant<uint32_t, 1>{}); break;
                case 2: block(pix0, block_end, std::integral_constant<uint32_t, 2>{}); break;
                case 3: block(pix0, block_end, std::integral_constant<uint32_t, 3>{}); break;
                case 4: block(pix0, block_end, std::integral_constant<uint32_t, 4>{}); break;
                default: break;
            }
        }
        return;
    }

    if constexpr (KIND == kTapsPatch) {
        // ---- phase 2 for kernels of several taps whose input channels are a multiple of 32.
        // The workgroup's pixels are taken in rounds of kWaves * wave_pixels; for a round and 32 input channels
        // the activations under every kernel tap of every pixel of the round (the "patch": the rows of the
        // zero-padded input images from the first pixel's first tap to the last pixel's last, each row with its
        // padding columns) are copied to LDS once, zeros included, and every tap's B operands are read from
        // there: a lane's address is its pixel's place in the patch plus an offset that only depends on the tap,
        // and nothing in the loop tests for the image's border.  The patch is four planes, one per block of 8 of
        // the 32 channels; patch element (row pr, column pc) is the 16 bytes number
        // (pr * stride + pc % stride) * Wh + pc / stride of each plane, Wh = ceil(padded width / stride): the 16
        // lanes that read the same 8 channels of a column tile's 16 pixels read 256 consecutive bytes for every
        // tap and stride (no two of them the same LDS bank).
        // A panel of symbol bytes is widened, 32 input channels of every tap at a time, into a slab of bf16
        // values beside the patch.  The next 32 channels' activations are on their way (in registers) while
        // the current ones are multiplied.
        const uint32_t S = p.stride, Hp = p.in_h + 2u * p.pad, Wp = p.in_w + 2u * p.pad, Wh = (Wp + S - 1u) / S;
        constexpr uint32_t taps = kPatchTaps;                     // 3 x 3 kernels only (the host sees to it)
        constexpr uint32_t slab_row = taps * 64u + 16u;           // bytes; rows start four banks apart
        uint8_t* slab = lds;
        uint8_t* patch = lds + p.patch_off;
        const uint32_t col = lane & 15u, kg = lane >> 4;          // MFMA operand layout: row or column, group of 8 k
        uint32_t tap_off[taps];                                   // from a pixel's place in the patch to what lies under a tap
#pragma unroll
        for (uint32_t tap = 0; tap < taps; ++tap) {
            const uint32_t r = tap / 3u, sx = tap % 3u;
            tap_off[tap] = ((r * S + sx % S) * Wh + sx / S) * 16u;
        }
        // A: lane holds row lane % 16 of a row tile, k = 8 * (lane / 16) + 0..7 of a step
        const uint8_t* a_lane = P16 ? panel + (col * p.row_stride + 8u * kg) * 2u : slab + col * slab_row + kg * 16u;
        const float zf = static_cast<float>(lay.zero_point);
        const uint32_t split_begin = split * p.pixels_per_split;
        const uint32_t split_end = min(split_begin + p.pixels_per_split, p.n_pixels);
        constexpr uint32_t kPieces = kPatchPieces;                // 16-byte pieces of a patch one thread may have to copy
        for (uint32_t round0 = split_begin; round0 < split_end; round0 += kWaves * p.wave_pixels) {
            const uint32_t round_end = min(round0 + kWaves * p.wave_pixels, split_end);
            // the patch's rows: flat index b * Hp + padded row
            const uint32_t first_row = round0 / p.out_w, last_row = (round_end - 1u) / p.out_w;   // flat output rows b * out_h + ho
            const uint32_t pr0 = (first_row / p.out_h) * Hp + (first_row % p.out_h) * S;
            const uint32_t pr_last = (last_row / p.out_h) * Hp + (last_row % p.out_h) * S + p.kh - 1u;
            const uint32_t n_pieces = (pr_last - pr0 + 1u) * 4u * Wp;
            if (n_pieces > kPieces * kThreads) {                  // the host sized the rounds so that this cannot happen
                if (tid == 0) report(p.status, ANSZP_ST_INTERNAL);
                return;                                           // uniform
            }
            uint32_t src[kPieces], dst[kPieces];                  // element of x (none: zeros), byte of the patch (none: no piece)
#pragma unroll
            for (uint32_t u = 0; u < kPieces; ++u) {
                const uint32_t i = tid + u * kThreads;            // piece (row, block of 8 channels, column), column fastest
                src[u] = dst[u] = 0xFFFFFFFFu;
                if (i < n_pieces) {
                    const uint32_t pc = i % Wp, t = i / Wp;
                    const uint32_t j = t & 3u, prl = t >> 2;
                    const uint32_t pra = pr0 + prl;
                    const uint32_t b = pra / Hp, h = pra % Hp - p.pad, w = pc - p.pad;   // unsigned: outside the image wraps around
                    if (h < p.in_h && w < p.in_w) src[u] = b * p.in_h * p.in_w * p.cin + (h * p.in_w + w) * p.x_pixel + j * p.x_block;
                    dst[u] = ((prl * S + pc % S) * Wh + pc / S) * 16u + j * p.patch_plane;
                }
            }
            // this wavefront's pixels: up to four column tiles; a column beyond them stands on the round's first pixel
            const uint32_t mine_begin = round0 + wave * p.wave_pixels;
            const uint32_t mine_end = min(mine_begin + p.wave_pixels, round_end);
            const uint32_t qt = mine_begin < mine_end ? (mine_end - mine_begin + 15u) / 16u : 0u;   // uniform
            bool valid[4];
            uint32_t out_at[4], at_patch[4];
            valid[3] = false;                                     // at most three column tiles (48 pixels) per wavefront and round
            out_at[3] = at_patch[3] = 0u;
#pragma unroll
            for (uint32_t q = 0; q < 3; ++q) {
                const uint32_t pix = mine_begin + q * 16u + col;
                valid[q] = pix < mine_end;
                const uint32_t n = valid[q] ? pix : round0;
                const uint32_t wo = n % p.out_w, t = n / p.out_w;
                const uint32_t ho = t % p.out_h, b = t / p.out_h;
                at_patch[q] = (((b * Hp + ho * S - pr0) * S) * Wh + wo) * 16u + kg * p.patch_plane;
                out_at[q] = b * p.out_h * p.out_w * p.cout + (ho * p.out_w + wo) * p.y_pixel;
            }
            floatx4 acc[MR][4];
#pragma unroll
            for (uint32_t m = 0; m < MR; ++m)
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) acc[m][q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

            words4 held_x[kPieces];
            auto fetch_x = [&](uint32_t c0) {                     // the pieces of input channels c0 .. c0 + 31
#pragma unroll
                for (uint32_t u = 0; u < kPieces; ++u) {
                    held_x[u] = words4{0u, 0u, 0u, 0u};
                    if (src[u] != 0xFFFFFFFFu) held_x[u] = *reinterpret_cast<const words4*>(p.x + src[u] + (c0 >> 3) * p.x_block);
                }
            };
            fetch_x(0u);
            for (uint32_t c0 = 0; c0 < p.cin; c0 += 32u) {
                __syncthreads();                                  // the previous step's patch and slab have been read
#pragma unroll
                for (uint32_t u = 0; u < kPieces; ++u)
                    if (dst[u] != 0xFFFFFFFFu) *reinterpret_cast<words4*>(patch + dst[u]) = held_x[u];
                if constexpr (!P16) {
                    // slab[row][tap][32] = bf16(panel[row][tap * cin + c0 + 0..31] - z), 16 symbols per piece
                    const uint32_t n_quads = kRows * MR * taps * 2u;
                    for (uint32_t i = tid; i < n_quads; i += kThreads) {
                        const uint32_t half = i & 1u, t = i >> 1;
                        const uint32_t tap = t % taps, row = t / taps;
                        const uint8_t* from = panel + row * p.row_stride + tap * p.cin + c0 + half * 16u;
                        bf16x8* to = reinterpret_cast<bf16x8*>(slab + row * slab_row + tap * 64u + half * 32u);
                        to[0] = weights_of(*reinterpret_cast<const words2*>(from), zf);
                        to[1] = weights_of(*reinterpret_cast<const words2*>(from + 8), zf);
                    }
                }
                if (c0 + 32u < p.cin) fetch_x(c0 + 32u);
                __syncthreads();
                // the nine taps, unrolled, with as many column tiles as this wavefront has (uniform)
                auto multiply = [&](auto tiles) {
                    constexpr uint32_t QT = decltype(tiles)::value;
#pragma unroll
                    for (uint32_t tap = 0; tap < kPatchTaps; ++tap) {
                        bf16x8 a[MR];
#pragma unroll
                        for (uint32_t m = 0; m < MR; ++m) {
                            if constexpr (P16) a[m] = *reinterpret_cast<const bf16x8*>(a_lane + (m * kRows * p.row_stride + tap * p.cin + c0) * 2u);
                            else a[m] = *reinterpret_cast<const bf16x8*>(a_lane + m * kRows * slab_row + tap * 64u);
                        }
#pragma unroll
                        for (uint32_t q = 0; q < QT; ++q) {
                            const bf16x8 b = *reinterpret_cast<const bf16x8*>(patch + at_patch[q] + tap_off[tap]);
#pragma unroll
                            for (uint32_t m = 0; m < MR; ++m)
                                acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], b, acc[m][q], 0, 0, 0);
                        }
                    }
                };
                if (qt == 3u) multiply(std::integral_constant<uint32_t, 3>{});
                else if (qt == 2u) multiply(std::integral_constant<uint32_t, 2>{});
                else if (qt == 1u) multiply(std::integral_constant<uint32_t, 1>{});
            }
            store_tiles<MR>(p, lay, mtile, kg, acc, valid, out_at);
        }
        return;
    }

    // ---- phase 2: the panel times the activations
    const uint32_t col = lane & 15u, kg = lane >> 4;              // MFMA operand layout: row or column, group of 8 k
    const uint8_t* a_row = panel + (col * p.row_stride + 8u * kg) * kElem;  // A: lane holds row lane % 16 of a row tile, k = 8 * (lane / 16) + 0..7
    const uint32_t tile_stride = kRows * p.row_stride * kElem;
    const float zf = static_cast<float>(lay.zero_point);
    auto a_operand = [&](const uint8_t* at) {                     // 8 consecutive k of this lane's row
        if constexpr (P16) return *reinterpret_cast<const bf16x8*>(at);
        else return weights_of(*reinterpret_cast<const words2*>(at), zf);
    };
    const uint32_t Kp = (p.K + 31u) & ~31u;
    // The workgroup's pixels are dealt out to its wavefronts in blocks of block_pixels, round robin, so that at
    // any time the wavefronts work on neighbouring pixels (kernel taps of neighbours share input rows).  A block
    // is 64 pixels unless the workgroup has fewer than 64 per wavefront: then it is narrower and the column
    // tiles beyond it are switched off, rather than wavefronts left without work.
    const uint32_t split_end = min((split + 1u) * p.pixels_per_split, p.n_pixels);

    for (uint32_t pix0 = split * p.pixels_per_split + wave * p.block_pixels; pix0 < split_end; pix0 += kWaves * p.block_pixels) {
        const uint32_t block_end = min(pix0 + p.block_pixels, split_end);
        // B: lane holds column lane % 16 of each of the block's four column tiles
        uint32_t pix[4];
        int32_t h0[4], w0[4];
        uint32_t img[4], out_at[4];                              // first element of the image in x; of the pixel in y
        bool valid[4];
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            pix[q] = pix0 + q * 16u + col;
            valid[q] = pix[q] < block_end;
            const uint32_t n = valid[q] ? pix[q] : 0u;
            const uint32_t wo = n % p.out_w, t = n / p.out_w;
            const uint32_t ho = t % p.out_h, b = t / p.out_h;
            h0[q] = int32_t(ho * p.stride) - int32_t(p.pad);
            w0[q] = int32_t(wo * p.stride) - int32_t(p.pad);
            img[q] = b * p.in_h * p.in_w * p.cin;
            out_at[q] = b * p.out_h * p.out_w * p.cout + (ho * p.out_w + wo) * p.y_pixel;
        }
        floatx4 acc[MR][4];
#pragma unroll
        for (uint32_t m = 0; m < MR; ++m)
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) acc[m][q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

        if constexpr (KIND == kPointwise) {
            // One pixel per column for the whole reduction: a step of 32 input channels is one address
            // addition per column.  The next step's activation vectors are requested before this step's MFMAs.
            const uint32_t n_steps = (p.cin + 31u) / 32u;
            const uint16_t* px[4];
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                px[q] = p.x + (valid[q] ? img[q] + (uint32_t(h0[q]) * p.in_w + uint32_t(w0[q])) * p.x_pixel : 0u) + kg * p.x_block;
            auto load_step = [&](uint32_t step, words4 (&b)[4]) {
                const bool live = step < n_steps && step * 32u + 8u * kg < p.cin;   // the last step may be partly beyond the channels
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    b[q] = words4{0u, 0u, 0u, 0u};
                    if (live && valid[q]) b[q] = *reinterpret_cast<const words4*>(px[q] + step * 4u * p.x_block);
                }
            };
            words4 cur[4], nxt[4];
            load_step(0u, cur);
            for (uint32_t step = 0; step < n_steps; ++step) {
                load_step(step + 1u, nxt);
#pragma unroll
                for (uint32_t m = 0; m < MR; ++m) {
                    const bf16x8 a = a_operand(a_row + m * tile_stride + step * 32u * kElem);
#pragma unroll
                    for (uint32_t q = 0; q < 4; ++q)
                        acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, cur[q]), acc[m][q], 0, 0, 0);
                }
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) cur[q] = nxt[q];
            }
        } else if constexpr (KIND == kTaps) {
            // Steps of 32 k: kernel taps outermost, 32 input channels at a time inside a tap.
            const uint32_t steps_per_tap = (p.cin + 31u) / 32u;
            const uint32_t n_steps = p.kh * p.kw * steps_per_tap;
            struct Cursor { uint32_t r, s, c0, a_off; };          // a_off: the step's first k (its panel column)
            auto advance = [&](Cursor& c) {
                c.c0 += 32u;
                if (c.c0 >= p.cin) {
                    c.c0 = 0;
                    c.a_off += p.cin;
                    if (++c.s == p.kw) { c.s = 0; ++c.r; }
                }
            };
            // where each column's pixel under the load cursor's kernel tap lies (recomputed when the cursor
            // enters a tap), so that a step costs one address addition per column
            const uint16_t* tap_ptr[4];
            bool tap_inside[4];
            auto enter_tap = [&](const Cursor& c) {
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    const int32_t h = h0[q] + int32_t(c.r), w = w0[q] + int32_t(c.s);
                    tap_inside[q] = valid[q] && uint32_t(h) < p.in_h && uint32_t(w) < p.in_w;
                    const uint32_t at = tap_inside[q] ? img[q] + (uint32_t(h) * p.in_w + uint32_t(w)) * p.x_pixel : 0u;
                    tap_ptr[q] = p.x + at + kg * p.x_block;           // this lane's block of 8 channels of the step's first 32
                }
            };
            auto load_step = [&](const Cursor& c, bool in_range, words4 (&b)[4]) {
                if (c.c0 == 0) enter_tap(c);                            // wavefront-uniform
                const bool live = in_range && c.c0 + 8u * kg < p.cin;   // the last 32 k of a tap may be partly beyond it
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    b[q] = words4{0u, 0u, 0u, 0u};
                    if (live && tap_inside[q]) b[q] = *reinterpret_cast<const words4*>(tap_ptr[q] + (c.c0 >> 3) * p.x_block);
                }
            };
            // a ring of kDepth steps' activation vectors: a step's slot is refilled, for the step kDepth
            // later, as soon as its MFMAs are issued.  Two steps: a deeper ring buys nothing as long as the
            // compiler waits for all outstanding loads before a step's MFMAs, and its registers are better
            // spent on a third wavefront per SIMD.
            constexpr uint32_t kDepth = 2;
            words4 ring[kDepth][4];
            Cursor ld{0u, 0u, 0u, 0u}, use{0u, 0u, 0u, 0u};
#pragma unroll
            for (uint32_t d = 0; d < kDepth; ++d) { load_step(ld, d < n_steps, ring[d]); advance(ld); }
            for (uint32_t base = 0; base < n_steps; base += kDepth) {
#pragma unroll
                for (uint32_t d = 0; d < kDepth; ++d) {
                    if (base + d < n_steps) {
#pragma unroll
                        for (uint32_t m = 0; m < MR; ++m) {
                            const bf16x8 a = a_operand(a_row + m * tile_stride + (use.a_off + use.c0) * kElem);
#pragma unroll
                            for (uint32_t q = 0; q < 4; ++q)
                                acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, ring[d][q]), acc[m][q], 0, 0, 0);
                        }
                    }
                    advance(use);
                    load_step(ld, base + d + kDepth < n_steps, ring[d]);
                    advance(ld);
                }
            }
        } else {
            // where each column's pixel lies under the first kernel tap (possibly outside the image: only used
            // together with a tap that is inside)
            uint32_t corner[4];
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) corner[q] = img[q] + uint32_t((h0[q] * int32_t(p.in_w) + w0[q]) * int32_t(p.cin));
            for (uint32_t k0 = 0; k0 < Kp; k0 += 32u) {
                const uint32_t kbase = k0 + 8u * kg;
                uint16_t bv[4][8];
                words2 kt[8];                                     // this lane's 8 k of the step: offset, kernel row and column
#pragma unroll
                for (uint32_t j = 0; j < 8; j += 2) {
                    const words4 two = *reinterpret_cast<const words4*>(k_table + 2u * (kbase + j));
                    kt[j] = words2{two.x, two.y};
                    kt[j + 1] = words2{two.z, two.w};
                }
#pragma unroll
                for (uint32_t j = 0; j < 8; ++j) {
                    const uint32_t r = kt[j].y & 0xFFu, s = kt[j].y >> 8;          // s = 0xFFFFFF beyond K: outside every image
#pragma unroll
                    for (uint32_t q = 0; q < 4; ++q) {
                        const int32_t h = h0[q] + int32_t(r), w = w0[q] + int32_t(s);
                        const bool inside = valid[q] && uint32_t(h) < p.in_h && uint32_t(w) < p.in_w;
                        bv[q][j] = inside ? p.x[corner[q] + kt[j].x] : uint16_t(0);   // NHWC only
                    }
                }
                words4 b[4];
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q)
                    b[q] = words4{uint32_t(bv[q][0]) | uint32_t(bv[q][1]) << 16, uint32_t(bv[q][2]) | uint32_t(bv[q][3]) << 16,
                                  uint32_t(bv[q][4]) | uint32_t(bv[q][5]) << 16, uint32_t(bv[q][6]) | uint32_t(bv[q][7]) << 16};
#pragma unroll
                for (uint32_t m = 0; m < MR; ++m) {
                    const bf16x8 a = a_operand(a_row + m * tile_stride + k0 * kElem);
#pragma unroll
                    for (uint32_t q = 0; q < 4; ++q)
                        acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b[q]), acc[m][q], 0, 0, 0);
                }
            }
        }

        store_tiles<MR>(p, lay, mtile, kg, acc, valid, out_at);
    }
}

constexpr uint32_t kMaxK = 4608;           // reduction length whose 16-row panel (72 KiB) fits LDS beside the table
constexpr uint32_t kLdsLimit = 160u * 1024u;
constexpr uint32_t kMaxK16 = 576;          // up to here 64 rows fit as bf16 (73 KiB), and no conversion is left in the loop

}  // namespace

extern "C" int anszp_conv_fused(const anszp_conv_args_t* a, void* stream) {
    if (!a || !a->tables || !a->chunks || !a->stream_hdr || !a->layers || !a->x || !a->y || !a->status) return ANSZP_E_NULL;
    if (a->payload_words && !a->payload) return ANSZP_E_NULL;
    if (a->table_log < 1 || a->table_log > ANSZP_MAX_TABLE_LOG || a->n_streams < 1 || a->n_streams > 64) return ANSZP_E_RANGE;
    if (a->layer_id >= a->n_tables) return ANSZP_E_RANGE;
    if (a->y_dtype != ANSZP_OUT_F32 && a->y_dtype != ANSZP_OUT_BF16) return ANSZP_E_RANGE;
    if (!a->batch || !a->in_h || !a->in_w || !a->cin || !a->cout || !a->kh || !a->kw || !a->stride) return ANSZP_E_RANGE;
    if (a->in_h > 32768u || a->in_w > 32768u || a->cin > 65536u || a->kh > 64u || a->kw > 64u || a->pad > 64u) return ANSZP_E_RANGE;
    if (a->cout % kRows) return ANSZP_E_RANGE;
    const uint64_t K = uint64_t(a->cin) * a->kh * a->kw;
    if (K > kMaxK) return ANSZP_E_RANGE;
    if (a->in_h + 2u * a->pad < a->kh || a->in_w + 2u * a->pad < a->kw) return ANSZP_E_RANGE;
    const uint32_t R = a->rows_per_chunk;
    if (R == 0 || R > kRows || (kRows % R)) return ANSZP_E_RANGE;
    const uint32_t out_h = (a->in_h + 2u * a->pad - a->kh) / a->stride + 1u;
    const uint32_t out_w = (a->in_w + 2u * a->pad - a->kw) / a->stride + 1u;
    const uint64_t n_pixels = uint64_t(a->batch) * out_h * out_w;
    if (n_pixels >= (1ull << 31) || uint64_t(a->batch) * a->in_h * a->in_w >= (1ull << 31)) return ANSZP_E_RANGE;
    if (uint64_t(a->batch) * a->in_h * a->in_w * a->cin >= (1ull << 32) || n_pixels * a->cout >= (1ull << 32))
        return ANSZP_E_RANGE;                                    // elements of x and y are addressed with 32 bits
    if (a->x_layout > ANSZP_ACT_C8 || a->y_layout > ANSZP_ACT_C8) return ANSZP_E_RANGE;
    if (a->x_layout == ANSZP_ACT_C8 && (a->cin % 8u) != 0) return ANSZP_E_RANGE;
    if (a->n_chunks < a->cout / R) return ANSZP_E_RANGE;
    // Row tiles per workgroup: as many of 4, 2, 1 as divide the output channels and leave the panel room in LDS
    // beside the table and the staging buffers (more rows per activation vector loaded).
    const uint32_t row_stride = ((uint32_t(K) + 31u) & ~31u) + kRowPad;
    const uint32_t table_bytes = 16u << a->table_log;             // the look-ahead entries
    const uint32_t fixed_bytes = table_bytes + kWaves * kStageWords * 4u + 64u;
    const bool p16 = K <= kMaxK16;                              // short rows: the panel as bf16
    const uint32_t elem = p16 ? 2u : 1u;
    uint32_t mr = 4;
    while (mr > 1 && ((a->cout % (kRows * mr)) != 0 || fixed_bytes + kRows * mr * row_stride * elem > kLdsLimit)) mr >>= 1;
    // A 3 x 3 kernel of stride 1 stages its activations in LDS where at most two row tiles fit anyway (K > 1152): with
    // four, the loads of a kernel row's three taps issued together do as well through the L1 (measured), and the
    // accumulators and operands in flight of four row tiles would not fit the patch kernel's registers.
    const bool patch_wanted = (a->cin % 32u) == 0 && a->cin >= 128u && a->kh == 3 && a->kw == 3 && a->stride == 1 && mr <= 2;
    const uint32_t n_mtiles = a->cout / (kRows * mr);
    if ((reinterpret_cast<uintptr_t>(a->x) | reinterpret_cast<uintptr_t>(a->y) | reinterpret_cast<uintptr_t>(a->payload) |
         reinterpret_cast<uintptr_t>(a->tables)) & 15u) return ANSZP_E_RANGE;

    ConvParams p{};
    p.tables = a->tables; p.chunks = a->chunks; p.stream_hdr = a->stream_hdr; p.payload = a->payload;
    p.layers = a->layers; p.scales = a->scales; p.x = a->x; p.y = a->y; p.status = a->status;
    p.y_bf16 = a->y_dtype == ANSZP_OUT_BF16;
    p.n_stream_hdr = a->n_stream_hdr; p.payload_words = a->payload_words; p.n_scales = a->scales ? a->n_scales : 0;
    p.layer_id = a->layer_id; p.table_log = a->table_log; p.n_streams = a->n_streams;
    p.rows_per_chunk = R;
    p.in_h = a->in_h; p.in_w = a->in_w; p.cin = a->cin; p.cout = a->cout; p.kh = a->kh; p.kw = a->kw;
    p.stride = a->stride; p.pad = a->pad; p.out_h = out_h; p.out_w = out_w;
    p.x_pixel = a->x_layout == ANSZP_ACT_C8 ? 8u : a->cin;
    p.x_block = a->x_layout == ANSZP_ACT_C8 ? 8u * a->in_h * a->in_w : 8u;
    p.y_pixel = a->y_layout == ANSZP_ACT_C8 ? 8u : a->cout;
    p.y_block = a->y_layout == ANSZP_ACT_C8 ? 8u * out_h * out_w : 8u;
    p.K = uint32_t(K);
    p.k_magic = uint32_t((uint64_t(1) << 32) / K) + 1u;           // unused for K = 1
    p.row_stride = row_stride;
    p.chunks_per_panel = kRows * mr / R;
    p.n_pixels = uint32_t(n_pixels);
    p.n_mtiles = n_mtiles;

    int device = 0, cus = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return ANSZP_E_HIP;
    // Every workgroup decodes its panel once, so few, long-lived workgroups: as many as are resident at once,
    // which is one per CU (twelve wavefronts of more than 128 VGPRs fill a CU's four SIMDs whatever the LDS
    // would allow).  A panel's pixels are dealt out in column tiles of 16, evenly over the workgroups that
    // share the panel.
    const uint32_t lds_bytes = fixed_bytes + kRows * mr * row_stride * elem;
    const uint32_t n_tiles = uint32_t((n_pixels + 15u) / 16u);
    uint32_t splits = (uint32_t(cus > 0 ? cus : 256) + n_mtiles - 1u) / n_mtiles;
    if (splits > n_tiles) splits = n_tiles;
    if (splits == 0) splits = 1;
    const uint32_t tiles_per_split = (n_tiles + splits - 1u) / splits;
    splits = (n_tiles + tiles_per_split - 1u) / tiles_per_split;
    p.pixels_per_split = 16u * tiles_per_split;
    const uint32_t tiles_per_wave = (tiles_per_split + kWaves - 1u) / kWaves;
    p.block_pixels = 16u * (tiles_per_wave < 4u ? tiles_per_wave : 4u);

    // (fixed_bytes counts 64 bytes beyond the panel: the last 32 k of a kernel tap may reach past the end of the last row)
    const bool generic = (a->cin % 8u) != 0;
    const bool pointwise = !generic && a->kh == 1 && a->kw == 1 && a->pad == 0;
    const uint32_t panel_bytes = kRows * mr * row_stride * elem;
    uint32_t lds_total = lds_bytes;
    // 1 x 1 kernels whose input channels are a multiple of 64: the contraction with several steps' loads in flight;
    // a panel of bytes is widened to bf16 in place first, which needs twice its room from the start of LDS
    bool ring = pointwise && (a->cin % 64u) == 0;
    if (ring && !p16) {
        ring = panel_bytes + 64u <= kWidenPieces * kThreads * 16u && 2u * (panel_bytes + 64u) <= kLdsLimit;
        if (ring && lds_total < 2u * (panel_bytes + 64u)) lds_total = 2u * (panel_bytes + 64u);
    }
    const uint32_t depth = ring ? ((a->cin % 128u) == 0 ? 4u : 2u) : 0u;
    // Kernels of several taps (or with padding) whose input channels are a multiple of 32: the patch in LDS.  The
    // pixels a wavefront takes per round are the most (of 64, 48, 32, 16, and no more than the workgroup's share
    // asks for) whose largest possible patch fits: in pieces per thread, and, with the slab of widened weights,
    // in the LDS below the panel.
    p.panel_off = table_bytes + kWaves * kStageWords * 4u;
    bool patch = patch_wanted;
    if (patch) {
        const uint32_t S = a->stride, Hp = a->in_h + 2u * a->pad, Wp = a->in_w + 2u * a->pad, Wh = (Wp + S - 1u) / S;
        const uint32_t taps = a->kh * a->kw;
        const uint32_t slab_bytes = p16 ? 0u : ((kRows * mr * (taps * 64u + 16u) + 63u) & ~63u);
        const int64_t gap = int64_t(Hp) - int64_t(out_h) * S;     // patch rows between the last output row of an image and the next image's first
        uint32_t wave_pixels = std::min(p.block_pixels, 48u);
        patch = false;
        for (; wave_pixels >= 16u; wave_pixels -= 16u) {
            const uint64_t round = std::min<uint64_t>(uint64_t(kWaves) * wave_pixels, p.pixels_per_split);
            const uint64_t rows_out = (round + out_w - 2u) / out_w + 1u;                   // output rows a round can touch
            const uint64_t crossings = std::min<uint64_t>(a->batch - 1u, (rows_out + out_h - 2u) / out_h);
            const uint64_t rows = (rows_out - 1u) * S + a->kh + crossings * uint64_t(gap > 0 ? gap : 0);
            const uint64_t patch_bytes = rows * S * Wh * 64u;
            const uint64_t below = std::max<uint64_t>(p.panel_off, slab_bytes + patch_bytes);
            if (rows * 4u * Wp <= kPatchPieces * kThreads && below + panel_bytes + 64u <= kLdsLimit) {
                patch = true;
                p.wave_pixels = wave_pixels;
                p.patch_off = slab_bytes;
                p.patch_plane = uint32_t(rows * S * Wh * 16u);
                p.panel_off = uint32_t((below + 15u) & ~uint64_t(15));
                lds_total = p.panel_off + panel_bytes + 64u;
                break;
            }
        }
        if (!patch) p.panel_off = table_bytes + kWaves * kStageWords * 4u;
    }
    bool generic_patch = false;
    if (generic) {
        // image rows that are multiples of 16 bytes (NHWC): the rows under a round of pixels staged in LDS, if the most
        // rows a round can need fit below the panel (after the table of k offsets) and in pieces per thread
        const uint32_t Kp = (uint32_t(K) + 31u) & ~31u;
        const uint64_t row_bytes = uint64_t(a->in_w) * a->cin * 2u;
        const uint64_t row_pitch = (32u + row_bytes + uint64_t(a->pad) * a->cin * 2u + 15u) & ~uint64_t(15);
        if (a->x_layout == ANSZP_ACT_NHWC && row_bytes % 16u == 0 && uint64_t(a->pad) * a->cin * 2u <= 32u && row_pitch < (1u << 20)) {
            const uint32_t S = a->stride, Hp = a->in_h + 2u * a->pad;
            const int64_t gap = int64_t(Hp) - int64_t(out_h) * S;
            const uint64_t tiles = (p.pixels_per_split + 15u) / 16u;
            const uint64_t n_rounds = (tiles + 4u * kWaves - 1u) / (4u * kWaves);
            const uint64_t round = ((tiles + n_rounds - 1u) / n_rounds) * 16u;
            const uint64_t rows_out = (round + out_w - 2u) / out_w + 1u;
            const uint64_t crossings = std::min<uint64_t>(a->batch - 1u, (rows_out + out_h - 2u) / out_h);
            const uint64_t rows = (rows_out - 1u) * S + a->kh + crossings * uint64_t(gap > 0 ? gap : 0);
            const uint64_t k_table_bytes = (uint64_t(Kp) * 4u + 63u) & ~uint64_t(63);
            const uint64_t below = std::max<uint64_t>(p.panel_off, k_table_bytes + rows * row_pitch);
            if (rows * (row_bytes / 16u) <= kPatchPieces * kThreads && below + panel_bytes + 64u <= kLdsLimit) {
                generic_patch = true;
                p.row_pitch = uint32_t(row_pitch);
                p.patch_off = uint32_t(k_table_bytes);
                p.panel_off = uint32_t((below + 15u) & ~uint64_t(15));
                lds_total = p.panel_off + panel_bytes + 64u;
            }
        }
        if (!generic_patch) {                                     // room for the table of the k below the panel
            const uint32_t k_table_bytes = Kp * 8u;
            if (p.panel_off < k_table_bytes) {
                p.panel_off = k_table_bytes;
                lds_total = p.panel_off + panel_bytes + 64u;
                if (lds_total > kLdsLimit) return ANSZP_E_RANGE;
            }
        }
    }
    // other kernels of several taps: the ring of loads, if the channels allow whole groups of steps per tap and a
    // step's stride fits a 24-bit multiplication
    const bool taps_ring = !generic && !pointwise && !patch && (a->cin % 64u) == 0 && 4ull * p.x_block < (1u << 24) &&
                           (p16 || (panel_bytes + 64u <= kWidenPieces * kThreads * 16u && 2u * (panel_bytes + 64u) <= kLdsLimit));
    if (taps_ring && !p16 && lds_total < 2u * (panel_bytes + 64u)) lds_total = 2u * (panel_bytes + 64u);
    const uint32_t taps_depth = taps_ring ? ((a->cin % 128u) == 0 ? 4u : 2u) : 0u;
    const bool taps_rows = taps_ring && a->kw == 3;
    const int kind = generic_patch ? kGenericPatch : generic ? kGeneric : ring ? kPointwiseRing : pointwise ? kPointwise : patch ? kTapsPatch
                   : taps_rows ? kTapsRows : taps_ring ? kTapsRing : kTaps;
    void (*kernel)(ConvParams) = nullptr;
#define ANSZP_CONV_PICK(KIND, D)                                                                                       \
    (p16 ? (mr == 4 ? conv_fused_kernel<KIND, 4, true, D> : mr == 2 ? conv_fused_kernel<KIND, 2, true, D> : conv_fused_kernel<KIND, 1, true, D>) \
         : (mr == 4 ? conv_fused_kernel<KIND, 4, false, D> : mr == 2 ? conv_fused_kernel<KIND, 2, false, D> : conv_fused_kernel<KIND, 1, false, D>))
    kernel = kind == kGeneric ? ANSZP_CONV_PICK(kGeneric, 0) : kind == kPointwise ? ANSZP_CONV_PICK(kPointwise, 0)
           : kind == kTaps ? ANSZP_CONV_PICK(kTaps, 0) : kind == kTapsPatch ? ANSZP_CONV_PICK(kTapsPatch, 0)
           : kind == kGenericPatch ? ANSZP_CONV_PICK(kGenericPatch, 0) : kind == kTapsRows ? ANSZP_CONV_PICK(kTapsRows, 0)
           : kind == kTapsRing ? (taps_depth == 4 ? ANSZP_CONV_PICK(kTapsRing, 4) : ANSZP_CONV_PICK(kTapsRing, 2))
           : depth == 4 ? ANSZP_CONV_PICK(kPointwiseRing, 4) : ANSZP_CONV_PICK(kPointwiseRing, 2);
#undef ANSZP_CONV_PICK
    // the kernels may use all of the CU's LDS: said once per kernel and device (a table of atomics:
    // concurrent callers at worst both say it)
    static std::atomic<bool> lds_allowed[2][10][3][64];
    const uint32_t slot = mr == 4 ? 2u : mr == 2 ? 1u : 0u;
    const uint32_t kernel_no = kind == kPointwiseRing && depth == 4 ? 8u : kind == kTapsRing && taps_depth == 4 ? 9u : uint32_t(kind);
    if (device < 0 || device >= 64) return ANSZP_E_HIP;
    if (!lds_allowed[p16][kernel_no][slot][device].load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                int(kLdsLimit)) != hipSuccess) return ANSZP_E_HIP;
        lds_allowed[p16][kernel_no][slot][device].store(true, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL(kernel, dim3(n_mtiles * splits), dim3(kThreads), lds_total, static_cast<hipStream_t>(stream), p);
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}
