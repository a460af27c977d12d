// Device side of libanszp for gfx950 (MI355X): tANS decode kernels with fused zero-point
// dequantisation, and the stand-alone dequantiser.
//
// Paper sections followed: Sec. II-A (one decode step = table look-up, read nb_bits, state =
// newX + bits; empty-label transitions read no bits), Sec. III-B (a vector of states, one per
// stream, all sharing one table: here a 64-lane wavefront is the vector and a lane is a stream),
// Sec. III-A (one table per layer), Sec. II-B (w = scale * (q - z)).
//
// Code paths, all producing identical results:
//   decode_chunk_stepwise  one look-up per symbol from the paper's triple, words read from global
//                          memory; handles every geometry the ABI allows (kernels decode_stepwise,
//                          one chunk per workgroup, and decode_stepwise_shared, sixteen).
//   decode_streaming       one look-up per symbol for thousands of large chunks: fourteen wavefronts of
//                          a workgroup decode a chunk each from 4-byte LDS entries derived from the
//                          triples and store; two load, 64 bytes at a time, into each stream's ring
//                          of words in LDS.
//   decode_lookahead       look-ups use the look-ahead entries of the table (a run of empty-label
//                          transitions of the dominant symbol, at most one of its 1-bit transitions
//                          and the step that ends them are ONE look-up, indexed by the state and the
//                          next stream bit).  The chunk's compressed words are staged in LDS.  One
//                          wavefront only walks the automaton and logs the entries it passes, eight
//                          per lane and block; two more take the logged blocks in turn and expand
//                          them into symbols in an LDS ring; three or four convert finished slabs
//                          of the ring and store them, 16 bytes per lane.  A workgroup serves one
//                          chunk or two chunks of one layer; which, and in what order the
//                          workgroups take them, is found per launch or read from a prepared plan.
// The look-ahead path needs the chunk's words to fit its LDS window and the chunk's first output
// element to be 16-byte aligned; other chunks take the step-wise path inside the same launch.
#include "anszp.h"
#include "anszp_layout.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstddef>
#include <type_traits>

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 768;                    // twelve wavefronts stage; up to seven per chunk stay for the decode
constexpr uint32_t kSlab = 1024u;              // elements that leave the ring together (two runs of 8 per lane)
constexpr uint32_t kBlockLookups = 8u;         // look-ups a lane makes per block of the look-ahead kernel
constexpr uint32_t kLogSlotBytes = (kBlockLookups + 1u) * kWave * 2u + 2u * kWave * 4u;   // nine rows of 16 bits per lane, two of 32
constexpr uint32_t kExpanders = 2u;            // expanding wavefronts per chunk: they take the logged blocks in turn
constexpr uint32_t kSpinLimit = 1u << 22;       // polls before a hand-over between wavefronts is declared stuck

// LDS geometry of the look-ahead kernel.  The large one takes tables of up to 2^12 states (64 KiB of
// look-ahead entries) and two chunks of a layer per workgroup, one workgroup per CU; the small one (tables
// of up to 2^11 states, shorter windows) leaves room for two workgroups per CU.
struct LargeLds {
    static constexpr uint32_t kTableLog = ANSZP_MAX_TABLE_LOG, kPayloadWords = 4096u, kRingElems = 16u * 1024u;
    static constexpr uint32_t kLogSlots = 8u, kWorkgroupsPerCu = 1u, kTag = 1u;
};
struct SmallLds {
    static constexpr uint32_t kTableLog = 11u, kPayloadWords = 2048u, kRingElems = 8u * 1024u;
    static constexpr uint32_t kLogSlots = 4u, kWorkgroupsPerCu = 2u, kTag = 2u;
};

struct DecodeParams {
    const uint32_t* tables;
    const anszp_chunk_t* chunks;
    const uint32_t* stream_hdr;
    const uint32_t* payload;
    const anszp_layer_t* layers;
    const float* scales;
    void* out;
    uint32_t* status;
    uint64_t n_stream_hdr;
    uint64_t payload_words;
    uint64_t n_scales;
    uint64_t out_elems;
    uint32_t n_tables;
    uint32_t table_log;
    uint32_t n_streams;
    uint32_t n_cus;             // compute units of the device: workgroups n_cus apart tend to share one
    uint32_t n_chunks;
    const uint32_t* plan;       // work assignment prepared by plan_units for these very arrays, or null
    uint32_t spin_limit;        // polls before a hand-over between wavefronts is declared stuck (kSpinLimit unless a test says otherwise)
};

// The chip hands consecutive workgroups to its eight dies (XCDs) in turn, and every die has an L2 of its
// own.  Consecutive units of work (chunks, pairs of chunks) belong to one layer and read one table: with
// workgroup b taking unit b, every die would fetch every large layer's table from memory (measured on
// the ResNet-50-shaped set: 13.0 MB fetched per launch, 5.2 MB when a table is fetched by one or two dies).
// So die x (workgroups b = x mod 8) takes groups of kDieGroup consecutive units, the groups dealt to the
// dies in turn.  The launch is rounded up to whole rounds; workgroups that map beyond the last unit return.
constexpr uint32_t kDies = 8u;
constexpr uint32_t kDieGroup = 4u;
__host__ __device__ __forceinline__ uint32_t mapped_workgroups(uint32_t n_units) {
    return (n_units + kDies * kDieGroup - 1u) / (kDies * kDieGroup) * (kDies * kDieGroup);
}
__device__ __forceinline__ uint32_t unit_of_workgroup(uint32_t b) {
    const uint32_t die = b % kDies, j = b / kDies;
    return ((j / kDieGroup) * kDies + die) * kDieGroup + j % kDieGroup;
}
// The workgroup that takes unit u (the inverse of unit_of_workgroup).
__device__ __forceinline__ uint32_t workgroup_of_unit(uint32_t u) {
    const uint32_t g = u % kDieGroup, t = u / kDieGroup, die = t % kDies, q = t / kDies;
    return (q * kDieGroup + g) * kDies + die;
}

__device__ __forceinline__ uint32_t bf16_rne(float w) {
    uint32_t u = __float_as_uint(w);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float dequant(uint32_t sym, uint32_t z, float scale) {
    return scale * static_cast<float>(static_cast<int>(sym) - static_cast<int>(z));
}

template <int OUT>
__device__ __forceinline__ void store_weight(void* out, uint64_t idx, uint32_t sym, uint32_t z, float scale) {
    if constexpr (OUT == ANSZP_OUT_U8) static_cast<uint8_t*>(out)[idx] = static_cast<uint8_t>(sym);
    else if constexpr (OUT == ANSZP_OUT_F32) static_cast<float*>(out)[idx] = dequant(sym, z, scale);
    else static_cast<uint16_t*>(out)[idx] = static_cast<uint16_t>(bf16_rne(dequant(sym, z, scale)));
}

__device__ __forceinline__ void report(uint32_t* status, uint32_t bits) {
    atomicOr(&status[0], bits);
    atomicAdd(&status[1], 1u);
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

// A word in LDS that another wavefront of the workgroup writes or reads: every access is performed,
// in order, as an LDS instruction.
typedef volatile __attribute__((address_space(3))) uint32_t lds_flag_t;

typedef __attribute__((address_space(3))) uint64_t lds_uint64_t;

// Byte address inside the workgroup's LDS of an object in __shared__ memory.
__device__ __forceinline__ uint32_t lds_address(const void* shared) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) void*)shared));
}

// A value every lane holds alike, moved to a scalar register.
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) v |= __shfl_xor(v, d, kWave);
    return v;
}

// True (for the whole workgroup) when the chunk descriptor stays inside the caller's buffers.
__device__ __forceinline__ bool chunk_in_bounds(const DecodeParams& p, const anszp_chunk_t& c) {
    return c.layer_id < p.n_tables && c.n_symbols <= (1u << 31) &&
           c.out_offset <= p.out_elems && c.n_symbols <= p.out_elems - c.out_offset &&
           (c.payload_offset & 3u) == 0u &&
           c.payload_offset <= p.payload_words && c.payload_words <= p.payload_words - c.payload_offset &&
           uint64_t(c.stream_offset) + p.n_streams <= p.n_stream_hdr;
}

// True when the layer's quantizer covers the chunk: a layer with a scale per output channel needs every
// channel the chunk touches to have one in the caller's array, and the chunk to lie inside the layer.
__device__ __forceinline__ bool scales_in_bounds(const DecodeParams& p, const anszp_layer_t& lay, const anszp_chunk_t& c) {
    if (lay.channel_len == 0u || c.n_symbols == 0u) return true;
    if (c.out_offset < lay.out_base) return false;
    const uint64_t last_channel = (c.out_offset - lay.out_base + c.n_symbols - 1u) / lay.channel_len;
    return lay.scales_offset <= p.n_scales && last_channel < p.n_scales - lay.scales_offset;
}

__device__ __forceinline__ float channel_scale(const DecodeParams& p, const anszp_layer_t& lay, uint64_t layer_elem) {
    const uint64_t ch = lay.scales_offset + layer_elem / lay.channel_len;
    return ch < p.n_scales ? p.scales[ch] : 0.0f;
}

// ---------------------------------------------------------------------------------------------
// One look-up per symbol (Sec. III-B: n look-ups and n small additions for a stream of n
// weights).  Executed by one wavefront; `table` is 2^table_log dwords of LDS holding the
// (newX, nb_bits, symbol) half of the entries.  Returns the chunk's error bits (wave-uniform).
// The triple of state X as one word (newX | nb_bits << 16 | symbol << 24) from a table of such words ...
struct WordTable {
    const uint32_t* words;
    __device__ __forceinline__ uint32_t operator()(uint32_t X) const { return words[X]; }
};
// ... or from the table of Sec. II-A itself, three bytes per state (symbol, nb_bits, newX), which holds
// tables of at most 256 states.
struct ByteTable {
    const uint8_t* bytes;
    __device__ __forceinline__ uint32_t operator()(uint32_t X) const {
        return uint32_t(bytes[3u * X + 2u]) | (uint32_t(bytes[3u * X + 1u]) << 16) | (uint32_t(bytes[3u * X]) << 24);
    }
};

template <int OUT, class TABLE>
__device__ uint32_t decode_chunk_stepwise(const DecodeParams& p, const anszp_chunk_t& c, const anszp_layer_t& lay,
                                          const TABLE table, uint32_t lane) {
    const uint32_t N = p.n_streams;
    const uint32_t L = 1u << p.table_log;
    const uint32_t hdr = lane < N ? p.stream_hdr[c.stream_offset + lane] : 0u;
    uint32_t X = hdr & (L - 1u);
    const uint32_t n_words = hdr >> 16;
    uint32_t total_words;
    const uint32_t first_word = wave_exclusive_sum(n_words, &total_words);
    const uint32_t len = (lane < N && c.n_symbols > lane) ? (c.n_symbols - lane + N - 1u) / N : 0u;
    uint32_t err = (total_words != c.payload_words) ? ANSZP_ST_BAD_DESC : 0u;

    const uint32_t* words = p.payload + c.payload_offset;
    const uint32_t word_limit = c.payload_words;      // reads beyond the chunk see zeros
    auto word_at = [&](uint32_t i) { return i < word_limit ? words[i] : 0u; };
    uint32_t next_word = first_word;                  // words moved into buf so far (plus first_word)
    uint64_t buf = 0;
    uint32_t have = 0;
    uint32_t ahead = word_at(first_word);             // the word after those in buf, requested one refill early
    const uint32_t steps = (c.n_symbols + N - 1u) / N;
    const bool per_channel = lay.channel_len != 0;
    // per-channel scales: channel index and position inside the channel advance by N per step
    const uint64_t elem0 = c.out_offset - lay.out_base + lane;
    uint64_t channel = per_channel ? lay.scales_offset + elem0 / lay.channel_len : 0;
    uint32_t in_channel = per_channel ? static_cast<uint32_t>(elem0 % lay.channel_len) : 0;
    float scale = lay.scale;
    if (per_channel) scale = channel < p.n_scales ? p.scales[channel] : 0.0f;
    for (uint32_t t = 0; t < steps; ++t) {
        if (t < len) {
            const uint32_t e = table(X);
            const uint32_t nb = (e >> 16) & 0xFFu;
            if (have < nb) {
                buf |= uint64_t(ahead) << have;
                have += 32;
                ++next_word;
                ahead = word_at(next_word);
            }
            const uint32_t low = static_cast<uint32_t>(buf) & ((1u << nb) - 1u);
            const uint32_t bits = nb ? __brev(low) >> (32u - nb) : 0u;      // first bit read is the top bit
            buf >>= nb;
            have -= nb;
            X = ((e & 0xFFFFu) + bits) & (L - 1u);
            store_weight<OUT>(p.out, c.out_offset + uint64_t(t) * N + lane, e >> 24, lay.zero_point, scale);
            if (per_channel) {
                in_channel += N;
                if (in_channel >= lay.channel_len) {
                    do { in_channel -= lay.channel_len; ++channel; } while (in_channel >= lay.channel_len);
                    scale = channel < p.n_scales ? p.scales[channel] : 0.0f;
                }
            }
        }
    }
    if (lane < N) {
        if (X != 0) err |= ANSZP_ST_BAD_STATE;
        if (next_word - first_word != n_words) err |= ANSZP_ST_BAD_LENGTH;
    }
    return wave_or(err);
}

template <int OUT>
__global__ __launch_bounds__(kWave) void decode_stepwise(DecodeParams p) {
    __shared__ uint32_t table[1u << ANSZP_MAX_TABLE_LOG];
    const uint32_t lane = threadIdx.x;
    const anszp_chunk_t c = p.chunks[blockIdx.x];
    if (!chunk_in_bounds(p, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const uint32_t* src = p.tables + c.layer_id * table_stride_words(p.table_log) + table_triples_offset(p.table_log);   // the paper's triples
    for (uint32_t i = lane; i < (1u << p.table_log); i += kWave) table[i] = src[i];
    const anszp_layer_t lay = p.layers[c.layer_id];
    __syncthreads();
    if (!scales_in_bounds(p, lay, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, WordTable{table}, lane);
    if (err && lane == 0) report(p.status, err);
}

// The decoder of Sec. II-A as the paper sizes it: the table is 3 l bytes (symbol, nb_bits, newX: one byte
// each), 192 bytes for 64 states, read from LDS; a step is three byte reads, nb_bits bits from the stream and
// an addition of log2(l) bits.  Four wavefronts per workgroup, a chunk and a copy of its layer's table each.
constexpr int kByteWaves = 4;
template <int OUT>
__global__ __launch_bounds__(kByteWaves * kWave) void decode_byte_table(DecodeParams p) {
    __shared__ uint32_t table[kByteWaves][3u * 256u / 4u];
    const uint32_t lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t index = blockIdx.x * kByteWaves + wave;
    if (index >= p.n_chunks) return;
    const anszp_chunk_t c = p.chunks[index];
    if (!chunk_in_bounds(p, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const anszp_layer_t lay = p.layers[c.layer_id];
    if (!scales_in_bounds(p, lay, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const uint32_t* src = p.tables + c.layer_id * table_stride_words(p.table_log) + table_bytes_offset(p.table_log);
    for (uint32_t i = lane; i < (3u << p.table_log) / 4u + 1u && i < 3u * 256u / 4u; i += kWave) table[wave][i] = src[i];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // the wavefront's own copy: LDS serves its accesses in order
    __builtin_amdgcn_wave_barrier();
    const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, ByteTable{reinterpret_cast<const uint8_t*>(table[wave])}, lane);
    if (err && lane == 0) report(p.status, err);
}

// The same loop for launches with many large chunks: sixteen wavefronts, each with a chunk of its own,
// share a workgroup and its LDS tables, so that a SIMD has eight wavefronts to hide each other's memory
// waits behind.  Consecutive chunks belong to at most two layers unless layers are tiny: the tables of the
// first and the last chunk's layers are staged; a chunk of any other layer reads its table from global memory.
constexpr int kSharedWaves = 16;
template <int OUT>
__global__ __launch_bounds__(kSharedWaves * kWave) void decode_stepwise_shared(DecodeParams p, uint32_t n_chunks) {
    __shared__ uint32_t table[2][1u << ANSZP_MAX_TABLE_LOG];
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t first = blockIdx.x * kSharedWaves, last = min(first + kSharedWaves, n_chunks) - 1u;
    const uint32_t L = 1u << p.table_log;
    const uint32_t layer_a = p.chunks[first].layer_id, layer_b = p.chunks[last].layer_id;
    if (layer_a < p.n_tables) {
        const uint32_t* src = p.tables + layer_a * table_stride_words(p.table_log) + table_triples_offset(p.table_log);    // the paper's triples
        for (uint32_t i = tid; i < L; i += kSharedWaves * kWave) table[0][i] = src[i];
    }
    if (layer_b != layer_a && layer_b < p.n_tables) {
        const uint32_t* src = p.tables + layer_b * table_stride_words(p.table_log) + table_triples_offset(p.table_log);
        for (uint32_t i = tid; i < L; i += kSharedWaves * kWave) table[1][i] = src[i];
    }
    __syncthreads();
    if (first + wave > last) return;
    const anszp_chunk_t c = p.chunks[first + wave];
    if (!chunk_in_bounds(p, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const anszp_layer_t lay = p.layers[c.layer_id];
    if (!scales_in_bounds(p, lay, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const uint32_t* mine = c.layer_id == layer_a ? table[0] : c.layer_id == layer_b ? table[1]
                           : p.tables + c.layer_id * table_stride_words(p.table_log) + table_triples_offset(p.table_log);
    const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, WordTable{mine}, lane);
    if (err && lane == 0) report(p.status, err);
}

// ---------------------------------------------------------------------------------------------
// One look-up per symbol for launches with thousands of chunks too large for an LDS window (Sec.
// III-B at scale).  The plain loop above reads a stream's words four bytes at a time; with two
// thousand streams per CU each of those reads brings a whole cache line from HBM again, and the
// launch is bound by re-reading its own input.  Here a stream's words come through a ring of 32
// words in LDS, 64 bytes per fetch, and a lane keeps a window of the stream in registers that it
// reloads from the ring every 8 steps (no per-step refill test: lanes need their refills at
// different steps, so such a test would run its body at nearly every step).
//
// A wavefront that stores a weight per step and also fetches its stream words is held up by its
// fetches far beyond their latency (loads and stores of a wavefront complete in issue order behind
// one counter, and the whole chip is writing).  So the work is split: fourteen wavefronts of a
// workgroup decode one chunk each and only store; two wavefronts only load: each follows the word
// positions seven decoding wavefronts publish in LDS, fetches the next 64 bytes of every stream
// whose ring has room for them, and publishes how far each ring is filled.  LDS accesses of a
// wavefront are performed in order, so a decoding wavefront that reads "filled up to w" before
// its window sees every word below w; no fences.  A decoding wavefront whose ring is not filled
// far enough waits (bounded); that only happens when streams spend several words per 8 steps.
//
// The LDS entries of the two tables a workgroup may need are 4 bytes, derived from the paper's
// triples (Sec. II-A) while staging:
//   bits 0..4   fast form (64 streams per chunk, no state of either table reads zero bits):
//               32 - nb_bits; the window holds the stream most significant bit first,
//               bits = window >> (32 - nb_bits), one funnel shift per window register consumes them
//               plain form: 31 - nb_bits; least significant bit first, every shift written so that
//               nb_bits = 0 works
//   bits 5..17  index, in the workgroup's two tables, of the entry of state newX
//   bits 19..31 weights out: the upper 13 bits of (symbol - zero_point) as fp16 (exact: |.| <= 255
//               leaves the lower 3 bits zero); symbols out: bits 19..26 the symbol
// The split needs the fast form and every wavefront-step inside one output channel (the scale is
// then wavefront-uniform per run of steps and the store address one base plus immediates); other
// chunks are decoded by their wavefront alone, fetches included.
constexpr int kStreamWaves = 16;                // per workgroup
constexpr int kStreamLoaders = 2;               // wavefronts that fetch stream words
constexpr int kStreamDecoders = kStreamWaves - kStreamLoaders;   // wavefronts that decode, one chunk each
constexpr int kStreamServed = kStreamDecoders / kStreamLoaders;  // decoding wavefronts per loading wavefront
constexpr int kStreamBatch = 4;                 // decoders whose fetches a loading wavefront has in flight together
constexpr uint32_t kStreamRingWords = 32u;      // per stream, in LDS
constexpr uint32_t kStreamFetchWords = 16u;     // per fetch from global memory: half a 128-byte line, on a 64-byte boundary
constexpr uint32_t kStreamUrgentWords = 8u;     // a stream this close to the end of its ring makes its wavefront's streams fetch
constexpr uint32_t kStreamNotStarted = 0xFFFFFFFEu, kStreamFinished = 0xFFFFFFFFu;   // in place of a published word position
typedef uint32_t words4 __attribute__((ext_vector_type(4)));            // four consecutive registers
typedef words4 __attribute__((aligned(4))) words4_word_aligned;
typedef uint32_t words2 __attribute__((ext_vector_type(2)));
typedef float floats4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uint32_t lds_uint32_t;
static_assert(kStreamDecoders % kStreamLoaders == 0, "every loading wavefront serves the same number of decoders");

// scale * (q - z) (Sec. II-B) with q - z read as fp16 from the high half of `entry` (lower bits
// cleared): the product is rounded once, like the plain multiplication; the addend -0 keeps the
// sign of a zero product.
__device__ __forceinline__ float scaled_high_half(uint32_t entry, float scale) {
    float w;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(w) : "v"(entry & 0xFFF80000u), "v"(scale), "v"(-0.0f));
    return w;
}
// The same for an entry whose bits 5..18 are already clear (only the high half is read).
__device__ __forceinline__ float scaled_clean_high_half(uint32_t cleared, float scale) {
    float w;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(w) : "v"(cleared), "v"(scale), "v"(-0.0f));
    return w;
}
typedef float floats2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16s2 __attribute__((ext_vector_type(2)));

// Byte offset, from the first of the workgroup's entries, of the entry of state newX + bits (Sec.
// II-A), newX taken from `entry`.  Written out so that the field extraction runs beside the
// extraction of `bits` and one instruction follows both.
__device__ __forceinline__ uint32_t next_entry_offset(uint32_t entry, uint32_t bits) {
    uint32_t index, offset;
    asm("v_bfe_u32 %0, %1, 5, 13" : "=v"(index) : "v"(entry));
    asm("v_add_lshl_u32 %0, %1, %2, 2" : "=v"(offset) : "v"(index), "v"(bits));
    return offset;
}

// First chunk of workgroup g when n chunks are dealt evenly to `groups` workgroups.
__host__ __device__ __forceinline__ uint32_t stream_group_begin(uint32_t g, uint32_t n, uint32_t groups) {
    return static_cast<uint32_t>(uint64_t(g) * n / groups);
}

template <int OUT>
__global__ __launch_bounds__(kStreamWaves * kWave) void decode_streaming(DecodeParams p, uint32_t n_chunks, uint32_t n_groups) {
    constexpr uint32_t kStates = 1u << ANSZP_MAX_TABLE_LOG;
    // one object, the tables first: their entries are then within reach of an LDS instruction's offset field
    struct Lds {
        uint32_t table[2][kStates];
        uint32_t rings[kStreamDecoders][kStreamRingWords + 1u][kWave];   // word s of lane l at [wave][s mod 32][l]; row 32 repeats row 0
        uint32_t position[kStreamDecoders][kWave];                       // word each stream's window starts at, or not started / finished
        uint32_t filled[kStreamDecoders][kWave];                         // words of each stream that are in its ring or before it
        uint32_t gave_up;
    };
    __shared__ Lds lds;
    auto& table = lds.table;
    constexpr uint32_t kThreads = kStreamWaves * kWave;
    constexpr uint32_t kPerThread = (kStates + kThreads - 1u) / kThreads;
    constexpr uint32_t kElemBytes = OUT == ANSZP_OUT_U8 ? 1u : OUT == ANSZP_OUT_F32 ? 4u : 2u;
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t first = stream_group_begin(blockIdx.x, n_chunks, n_groups);
    const uint32_t count = min(stream_group_begin(blockIdx.x + 1u, n_chunks, n_groups) - first, uint32_t(kStreamDecoders));
    if (count == 0u) return;
    const uint32_t last = first + count - 1u;
    const uint32_t L = 1u << p.table_log, N = p.n_streams;
    const uint32_t layer_a = p.chunks[first].layer_id, layer_b = p.chunks[last].layer_id;
    const bool have_a = layer_a < p.n_tables, have_b = layer_b != layer_a && layer_b < p.n_tables;
    lds_flag_t* const gave_up = (lds_flag_t*)&lds.gave_up;
    if (tid < uint32_t(kStreamDecoders) * kWave) ((lds_flag_t*)&lds.position[0][0])[tid] = kStreamNotStarted;
    if (tid == 0) *gave_up = 0u;

    // the paper's triples of both tables, held in registers until the form of the entries is known
    const uint32_t* src_a = p.tables + (have_a ? layer_a : 0u) * table_stride_words(p.table_log) + table_triples_offset(p.table_log);
    const uint32_t* src_b = p.tables + (have_b ? layer_b : 0u) * table_stride_words(p.table_log) + table_triples_offset(p.table_log);
    constexpr uint32_t kNoTriple = 0x00010000u;           // reads one bit
    uint32_t ta0 = kNoTriple, ta1 = kNoTriple, ta2 = kNoTriple, ta3 = kNoTriple;
    uint32_t tb0 = kNoTriple, tb1 = kNoTriple, tb2 = kNoTriple, tb3 = kNoTriple;
    static_assert(kPerThread == 4, "four triples of each table per thread");
    if (have_a) {
        if (tid < L) ta0 = src_a[tid];
        if (tid + kThreads < L) ta1 = src_a[tid + kThreads];
        if (tid + 2u * kThreads < L) ta2 = src_a[tid + 2u * kThreads];
        if (tid + 3u * kThreads < L) ta3 = src_a[tid + 3u * kThreads];
    }
    if (have_b) {
        if (tid < L) tb0 = src_b[tid];
        if (tid + kThreads < L) tb1 = src_b[tid + kThreads];
        if (tid + 2u * kThreads < L) tb2 = src_b[tid + 2u * kThreads];
        if (tid + 3u * kThreads < L) tb3 = src_b[tid + 3u * kThreads];
    }
    auto reads_no_bits = [](uint32_t e) { return ((e >> 16) & 0xFFu) == 0u; };
    const bool some_zero = reads_no_bits(ta0) || reads_no_bits(ta1) || reads_no_bits(ta2) || reads_no_bits(ta3) ||
                           reads_no_bits(tb0) || reads_no_bits(tb1) || reads_no_bits(tb2) || reads_no_bits(tb3);
    const bool fast = !__syncthreads_or(some_zero) && N == kWave;
    auto place = [&](uint32_t e, uint32_t i, uint32_t which, uint32_t z) {
        if (i >= L) return;
        const uint32_t sym = e >> 24, nb = min((e >> 16) & 0xFFu, 31u);
        const int centred = static_cast<int>(sym) - static_cast<int>(z);                       // |.| <= 255
        const uint32_t shift = fast ? (32u - nb) & 31u : 31u - nb;
        const uint32_t upper = OUT == ANSZP_OUT_U8 ? sym << 19
            : static_cast<uint32_t>(__builtin_bit_cast(uint16_t, static_cast<_Float16>(centred))) << 16;
        table[which][i] = shift | ((which * kStates + (e & (L - 1u))) << 5) | upper;
    };
    if (have_a) {
        const uint32_t z = p.layers[layer_a].zero_point;
        place(ta0, tid, 0, z); place(ta1, tid + kThreads, 0, z); place(ta2, tid + 2u * kThreads, 0, z); place(ta3, tid + 3u * kThreads, 0, z);
    }
    if (have_b) {
        const uint32_t z = p.layers[layer_b].zero_point;
        place(tb0, tid, 1, z); place(tb1, tid + kThreads, 1, z); place(tb2, tid + 2u * kThreads, 1, z); place(tb3, tid + 3u * kThreads, 1, z);
    }
    __syncthreads();

    // Where the words of this lane's stream of chunk c are.  Fetches are 64 bytes on 64-byte
    // boundaries (a line is then brought in twice, not once per touched piece), so words are counted
    // from the boundary at or before the stream's first word: the stream starts at word `skew` of
    // the returned pointer, `readable` words from there on are inside the caller's buffer.
    auto locate = [&](const anszp_chunk_t& c, uint32_t& n_words, uint32_t& skew, uint32_t& readable, bool& sums_up) {
        const uint32_t hdr = lane < N ? p.stream_hdr[c.stream_offset + lane] : 0u;
        n_words = hdr >> 16;
        uint32_t total_words;
        const uint32_t first_word = wave_exclusive_sum(n_words, &total_words);
        sums_up = total_words == c.payload_words;
        const uint64_t stream_first = c.payload_offset + uint64_t(min(first_word, c.payload_words));
        const uint32_t ahead_of_boundary = static_cast<uint32_t>((reinterpret_cast<uintptr_t>(p.payload + stream_first) & 63u) >> 2);
        skew = ahead_of_boundary <= stream_first ? ahead_of_boundary : 0u;      // not before the caller's buffer
        const uint64_t base = stream_first - skew;
        const uint64_t after = p.payload_words - base;
        readable = after > 0xFFFFFFF0ull ? 0xFFFFFFF0u : static_cast<uint32_t>(after);
        return p.payload + base;
    };
    // sixteen words of a stream; beyond the caller's buffer they read as zero (beyond the stream
    // they are its neighbours' words, never used)
    struct Fetched { words4 a, b, c, d; };
    auto fetch = [&](const uint32_t* mine, uint32_t readable, uint32_t at, Fetched& f) {
        if (at + kStreamFetchWords <= readable) {
            const words4_word_aligned* q = reinterpret_cast<const words4_word_aligned*>(mine + at);
            f.a = q[0];
            f.b = q[1];
            f.c = q[2];
            f.d = q[3];
        } else {
            auto one = [&](uint32_t i) { return at + i < readable ? mine[at + i] : 0u; };
            f.a = words4{one(0), one(1), one(2), one(3)};
            f.b = words4{one(4), one(5), one(6), one(7)};
            f.c = words4{one(8), one(9), one(10), one(11)};
            f.d = words4{one(12), one(13), one(14), one(15)};
        }
    };
    auto land = [&](uint32_t (*ring)[kWave], uint32_t at, const Fetched& f) {      // at is a multiple of 16: no wrap inside
        const uint32_t s0 = at & (kStreamRingWords - 1u);
        ring[s0][lane] = f.a.x; ring[s0 + 1][lane] = f.a.y; ring[s0 + 2][lane] = f.a.z; ring[s0 + 3][lane] = f.a.w;
        ring[s0 + 4][lane] = f.b.x; ring[s0 + 5][lane] = f.b.y; ring[s0 + 6][lane] = f.b.z; ring[s0 + 7][lane] = f.b.w;
        ring[s0 + 8][lane] = f.c.x; ring[s0 + 9][lane] = f.c.y; ring[s0 + 10][lane] = f.c.z; ring[s0 + 11][lane] = f.c.w;
        ring[s0 + 12][lane] = f.d.x; ring[s0 + 13][lane] = f.d.y; ring[s0 + 14][lane] = f.d.z; ring[s0 + 15][lane] = f.d.w;
        if (s0 == 0u) ring[kStreamRingWords][lane] = f.a.x;              // so that a pair of neighbouring words never wraps
    };

    if (wave >= uint32_t(kStreamDecoders)) {
        // ---- loading wavefront: decoders wave - 14, + 2, + 4, ... (little to issue, and others wait for it: first in line)
        __builtin_amdgcn_s_setprio(3);
        const uint32_t mine_index = wave - uint32_t(kStreamDecoders);
        const uint32_t* where[kStreamServed];             // all indexed by constants once the loops are unrolled
        uint32_t readable[kStreamServed], fetched[kStreamServed];
        bool alive[kStreamServed];
#pragma unroll
        for (int j = 0; j < kStreamServed; ++j) {
            const uint32_t d = mine_index + uint32_t(j * kStreamLoaders);
            where[j] = p.payload;
            readable[j] = 0u;
            fetched[j] = kStreamRingWords;                // the decoding wavefront fills its ring once itself
            alive[j] = false;
            if (d < count) {
                const anszp_chunk_t cj = p.chunks[first + d];
                if (chunk_in_bounds(p, cj) && scales_in_bounds(p, p.layers[cj.layer_id], cj)) {
                    uint32_t n_words, skew;
                    bool sums_up;
                    where[j] = locate(cj, n_words, skew, readable[j], sums_up);
                    alive[j] = true;
                }
            }
        }
        for (uint32_t idle = 0;;) {
            bool any_alive = false, moved = false;
#pragma unroll
            for (int b = 0; b < kStreamServed; b += kStreamBatch) {
                Fetched f[kStreamBatch];
                bool want[kStreamBatch];
#pragma unroll
                for (int i = 0; i < kStreamBatch; ++i) {
                    const int j = b + i;
                    want[i] = false;
                    if (j < kStreamServed && alive[j]) {
                        const uint32_t d = mine_index + uint32_t(j * kStreamLoaders);
                        const uint32_t at = ((lds_flag_t*)lds.position[d])[lane];
                        if (__ballot(at != kStreamFinished) == 0ull) {
                            alive[j] = false;
                        } else {
                            any_alive = true;
                            // A stream with room for sixteen more words (they replace words it has passed) gets
                            // them once some stream of its wavefront is down to kStreamUrgentWords: a load
                            // instruction costs the same for one lane as for sixty-four.
                            const uint32_t ahead = fetched[j] - at;
                            const bool started = at < kStreamNotStarted;
                            if (__ballot(started && ahead <= kStreamUrgentWords) != 0ull) {
                                want[i] = started && ahead <= kStreamRingWords - kStreamFetchWords;
                                if (want[i]) fetch(where[j], readable[j], fetched[j], f[i]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < kStreamBatch; ++i) {
                    const int j = b + i;
                    if (j < kStreamServed) {
                        const uint32_t d = mine_index + uint32_t(j * kStreamLoaders);
                        if (want[i]) {
                            land(lds.rings[d], fetched[j], f[i]);
                            fetched[j] += kStreamFetchWords;
                            asm volatile("" ::: "memory");
                            ((lds_flag_t*)lds.filled[d])[lane] = fetched[j];
                        }
                        if (__ballot(want[i]) != 0ull) moved = true;
                    }
                }
            }
            if (!any_alive) break;
            if (moved) { idle = 0; continue; }
            if (uniform(*gave_up)) break;
            if (++idle > p.spin_limit) {
                if (lane == 0) { *gave_up = 1u; report(p.status, ANSZP_ST_INTERNAL); }
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        return;
    }

    // ---- decoding wavefront
    lds_flag_t* const position = (lds_flag_t*)lds.position[wave];
    lds_flag_t* const filled = (lds_flag_t*)lds.filled[wave];
    auto no_more_positions = [&]() { position[lane] = kStreamFinished; };
    if (wave >= count) { no_more_positions(); return; }
    const anszp_chunk_t c = p.chunks[first + wave];
    if (!chunk_in_bounds(p, c) || !scales_in_bounds(p, p.layers[c.layer_id], c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        no_more_positions();
        return;
    }
    const anszp_layer_t lay = p.layers[c.layer_id];
    const bool per_channel = lay.channel_len != 0;
    const uint64_t chunk_elem0 = c.out_offset - lay.out_base;
    const uint64_t channel0 = per_channel ? chunk_elem0 / lay.channel_len : 0;           // within the layer
    const uint32_t in_channel0 = per_channel ? static_cast<uint32_t>(chunk_elem0 - channel0 * lay.channel_len) : 0;
    auto scale_of = [&](uint64_t channel) {               // channel counted within the chunk
        const uint64_t ch = lay.scales_offset + channel0 + channel;
        float v = ch < p.n_scales ? p.scales[ch] : 0.0f;
        asm volatile("" : "+v"(v));                       // the wait for this load stands here, not at a later write of its register
        return v;
    };
    if (c.layer_id != layer_a && c.layer_id != layer_b) {
        // a third layer in one workgroup: the plain loop, table from global memory
        no_more_positions();
        const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, WordTable{p.tables + c.layer_id * table_stride_words(p.table_log) + table_triples_offset(p.table_log)}, lane);
        if (err && lane == 0) report(p.status, err);
        return;
    }
    uint32_t (*ring)[kWave] = lds.rings[wave];
    const uint32_t entries = lds_address(&table[0][0]);
    auto entry_at = [&](uint32_t offset) { return *reinterpret_cast<const lds_uint32_t*>(static_cast<uintptr_t>(entries + offset)); };

    uint32_t n_words, skew, readable;
    bool sums_up;
    const uint32_t* const mine = locate(c, n_words, skew, readable, sums_up);
    const uint32_t hdr = lane < N ? p.stream_hdr[c.stream_offset + lane] : 0u;
    const uint32_t state0 = c.layer_id == layer_a ? 0u : 4u * kStates;   // byte offset of the entry of state 0
    uint32_t X = state0 + ((hdr & (L - 1u)) << 2);       // byte offset of the current state's entry
    const uint32_t len = (lane < N && c.n_symbols > lane) ? (c.n_symbols - lane + N - 1u) / N : 0u;
    uint32_t err = sums_up ? 0u : ANSZP_ST_BAD_DESC;
    const uint32_t full_steps = c.n_symbols / N;          // steps every stream of the chunk takes

    for (uint32_t at = 0; at < kStreamRingWords; at += kStreamFetchWords) {
        Fetched f;
        fetch(mine, readable, at, f);
        land(ring, at, f);
    }
    uint32_t fetched = kStreamRingWords;                  // words of the stream that are in the ring or before it (when this wavefront fetches itself)

    uint32_t abit = 32u * skew;                           // bit position, counted from the first word fetched
    // the stream's next bits from the ring, bit `abit` of the stream in bit 0 of w0: four words, read as
    // two pairs of neighbouring rows (one instruction each: the rows are 64 words apart)
    const uint32_t my_words = lds_address(&ring[0][lane]);               // word 0 of this lane
    auto pair_addresses = [&](uint32_t& a01, uint32_t& a23) {
        a01 = my_words + (((abit >> 5) & (kStreamRingWords - 1u)) << 8);
        a23 = my_words + ((((abit + 64u) >> 5) & (kStreamRingWords - 1u)) << 8);
    };
    auto shift_window = [&](uint32_t& w0, uint32_t& w1, uint32_t& w2, uint32_t& w3) {
        w0 = __builtin_amdgcn_alignbit(w1, w0, abit);
        w1 = __builtin_amdgcn_alignbit(w2, w1, abit);
        w2 = __builtin_amdgcn_alignbit(w3, w2, abit);
        w3 >>= (abit & 31u);
    };
    auto window = [&](uint32_t& w0, uint32_t& w1, uint32_t& w2, uint32_t& w3) {
        uint32_t a01, a23;
        pair_addresses(a01, a23);
        const lds_uint32_t* const p01 = reinterpret_cast<const lds_uint32_t*>(static_cast<uintptr_t>(a01));
        const lds_uint32_t* const p23 = reinterpret_cast<const lds_uint32_t*>(static_cast<uintptr_t>(a23));
        w0 = p01[0]; w1 = p01[kWave]; w2 = p23[0]; w3 = p23[kWave];
        shift_window(w0, w1, w2, w3);
    };
    // K steps of the fast form from the window w0..w2 (bit `abit` of the stream in bit 0 of w0).
    // A step may read table_log <= 12 bits, so of the 96 bits only those a later step of the K can
    // still reach are kept in place.
    // (`first` gives the entry of the current state: a caller may have asked for it with the window)
    auto steps_fast = [&](auto count_tag, uint32_t w0, uint32_t w1, uint32_t w2, auto&& emit, auto&& first) {
        constexpr int K = static_cast<int>(decltype(count_tag)::value);
        static_assert(K * ANSZP_MAX_TABLE_LOG <= 96, "the window of K steps");
        w0 = __brev(w0); w1 = __brev(w1); w2 = __brev(w2);
        uint32_t sum = 0;                                 // 32 - nb_bits over the K steps, in its low bits
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t e = k == 0 ? first() : entry_at(X);
            const uint32_t bits = w0 >> (e & 31u);                         // first bit read is the top bit
            X = next_entry_offset(e, bits);
            if (k <= K - 2) w0 = __builtin_amdgcn_alignbit(w0, w1, e);
            if (k <= K - 4) w1 = __builtin_amdgcn_alignbit(w1, w2, e);
            if (k <= K - 7) w2 = __builtin_amdgcn_alignbit(w2, 0u, e);
            // one mask serves both uses of the entry that remain: with the index of the next entry cleared, the
            // upper half is the centred symbol as fp16 and the lower bits add up to the bits not read (8 * 31
            // fits below the cleared field, whatever the upper halves add up to)
            const uint32_t cleared = e & 0xFFF8001Fu;
            sum += cleared;
            emit(k, cleared, k == K - 1);
        }
        abit += 32u * K - (sum & 0x7FFFFu);
    };
    // a lane asks for sixteen more words when the ring has room for them (they replace words it has passed)
    auto wants_words = [&]() { return fetched - (abit >> 5) <= kStreamRingWords - kStreamFetchWords; };
    // One block of a wavefront that fetches itself: K steps, with a fetch asked for before them
    // and put into the ring after them.  A block reads at most three words beyond its first one,
    // a lane enters it at least four words ahead.
    auto block_fast = [&](auto count_tag, auto&& emit) {
        const bool fetching = wants_words();
        Fetched f;
        if (fetching) fetch(mine, readable, fetched, f);
        uint32_t w0, w1, w2, w3;
        window(w0, w1, w2, w3);
        steps_fast(count_tag, w0, w1, w2, emit, [&]() { return entry_at(X); });
        if (fetching) {
            land(ring, fetched, f);
            fetched += kStreamFetchWords;
        }
    };

    const bool aligned = !per_channel || (lay.channel_len % kWave == 0u && in_channel0 % kWave == 0u);
    const bool fed = fast && aligned && uint64_t(c.n_symbols) * kElemBytes < (1ull << 31);      // fast: all 64 lanes have a stream
    if (!fed) no_more_positions();
    if (lane < N) {
        if (fed) {
            // every wavefront-step lies inside one channel: one scale per run of steps, weights of
            // step k at chunk_out + at + k * 64 * kElemBytes; the stream words come from a loading wavefront
            filled[lane] = kStreamRingWords;
            position[lane] = abit >> 5;
            char* const chunk_out = static_cast<char*>(p.out) + c.out_offset * kElemBytes;
            uint32_t at = lane * kElemBytes;
            // The scale of a channel comes through the scalar cache: a vector load would have to be waited
            // for behind every store the wavefront has in flight.
            auto uniform_scale = [&](uint32_t channel_in_chunk) {
                const uint64_t ch = lay.scales_offset + channel0 + channel_in_chunk;
                if (ch >= p.n_scales) return 0.0f;
                const uintptr_t q = reinterpret_cast<uintptr_t>(p.scales + ch);
                const uint64_t address = (uint64_t(uniform(static_cast<uint32_t>(q >> 32))) << 32) | uniform(static_cast<uint32_t>(q));
                uint32_t v;
                asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(address) : "memory");
                return __uint_as_float(v);
            };
            float scale = per_channel ? uniform_scale(0) : lay.scale;
            uint32_t channel = 0;                                          // within the chunk
            uint32_t left = uniform(per_channel ? (lay.channel_len - in_channel0) / kWave : 0xFFFFFFFFu);   // steps left under this scale
            const uint32_t steps = uniform(full_steps);
            bool stuck = false;
            // (stores marked non-temporal: the weights are not read again here, and the lines of stream words,
            // which are fetched in two halves some microseconds apart, should outlive them in the L2)
            float held = 0.0f;                                             // the weight of an even step, until its odd neighbour's is there
            auto emit = [&](int k, uint32_t e, bool last) {
                char* const q = chunk_out + at + static_cast<uint32_t>(k) * (kWave * kElemBytes);
                if constexpr (OUT == ANSZP_OUT_U8) __builtin_nontemporal_store(static_cast<uint8_t>(e >> 19), reinterpret_cast<uint8_t*>(q));
                else if constexpr (OUT == ANSZP_OUT_F32) __builtin_nontemporal_store(scaled_clean_high_half(e, scale), reinterpret_cast<float*>(q));
                else {
                    // bf16: two steps' weights are rounded by one instruction and stored from the two halves of its result
                    const float w = scaled_clean_high_half(e, scale);
                    if ((k & 1) == 0 && !last) {
                        held = w;
                    } else if (k & 1) {
                        const bf16s2 both = __builtin_convertvector(floats2{held, w}, bf16s2);
                        __builtin_nontemporal_store(both.x, reinterpret_cast<__bf16*>(q - kWave * kElemBytes));
                        __builtin_nontemporal_store(both.y, reinterpret_cast<__bf16*>(q));
                    } else {
                        __builtin_nontemporal_store(static_cast<__bf16>(w), reinterpret_cast<__bf16*>(q));
                    }
                }
            };
            // K steps from the ring as the loading wavefront fills it: the window's four words must be there
            const uint32_t filled_at = lds_address(&lds.filled[wave][lane]);
            auto block_fed = [&](auto count_tag) {
                uint32_t w0, w1, w2, w3, e0;
                for (uint32_t spins = 0;;) {
                    // how far the ring is filled, read before the words themselves, and the entry of the current
                    // state: all in flight together (left to the compiler, each waits for the one before)
                    uint32_t a01, a23, have;
                    words2 w01, w23;
                    pair_addresses(a01, a23);
                    asm volatile("ds_read_b32 %[have], %[at]\n\t"
                                 "ds_read2st64_b32 %[w01], %[a01] offset1:1\n\t"
                                 "ds_read2st64_b32 %[w23], %[a23] offset1:1\n\t"
                                 "ds_read_b32 %[e0], %[x]\n\t"
                                 "s_waitcnt lgkmcnt(0)"
                                 : [have] "=&v"(have), [w01] "=&v"(w01), [w23] "=&v"(w23), [e0] "=&v"(e0)
                                 : [at] "v"(filled_at), [a01] "v"(a01), [a23] "v"(a23), [x] "v"(entries + X)
                                 : "memory");
                    w0 = w01.x; w1 = w01.y; w2 = w23.x; w3 = w23.y;
                    shift_window(w0, w1, w2, w3);
                    if (__ballot(have - (abit >> 5) < 4u) == 0ull) break;
                    if (uniform(*gave_up) || ++spins > p.spin_limit) { stuck = true; return; }
                    __builtin_amdgcn_s_sleep(1);
                }
                steps_fast(count_tag, w0, w1, w2, emit, [&]() { return e0; });
                position[lane] = abit >> 5;
            };
            // Wavefronts go to the four SIMDs round robin, and a SIMD serves the oldest of its wavefronts
            // first: left alone, the decoders of a workgroup finish in the order of their age, 15 % apart,
            // and the youngest run the end of the launch alone on their SIMDs.  So the decoders of a SIMD
            // take turns at each priority, every 8 blocks.
            const uint32_t sharing = (count - (wave & 3u) + 3u) / 4u;      // decoders on this wavefront's SIMD
            uint32_t turn = 0;
            auto take_turn = [&]() {
                if (sharing < 2u) return;
                switch (((wave >> 2) + (turn >> 3)) % sharing) {
                    case 0: __builtin_amdgcn_s_setprio(0); break;
                    case 1: __builtin_amdgcn_s_setprio(1); break;
                    case 2: __builtin_amdgcn_s_setprio(2); break;
                    default: __builtin_amdgcn_s_setprio(3); break;
                }
            };
            take_turn();
            uint32_t t = 0;
            while (t < steps && !stuck) {
                uint32_t seg = min(steps - t, left);
                t += seg;
                left -= seg;
                for (; seg >= 8u && !stuck; seg -= 8u) {
                    block_fed(std::integral_constant<int, 8>{});
                    at += 8u * kWave * kElemBytes;
                    if ((++turn & 7u) == 0u) take_turn();
                }
                if (seg >= 4u && !stuck) { block_fed(std::integral_constant<int, 4>{}); at += 4u * kWave * kElemBytes; seg -= 4u; }
                for (; seg && !stuck; --seg) { block_fed(std::integral_constant<int, 1>{}); at += kWave * kElemBytes; }
                if (left == 0u) {
                    ++channel;
                    left = uniform(lay.channel_len / kWave);
                    scale = uniform_scale(channel);
                }
            }
            if (len > full_steps && !stuck) block_fed(std::integral_constant<int, 1>{});   // ragged tail: streams 0 .. n mod N - 1
            if (stuck) {
                if (lane == 0) { *gave_up = 1u; report(p.status, ANSZP_ST_INTERNAL); }
                no_more_positions();
                return;
            }
        } else {
            // this wavefront alone: a scale per lane, followed from element to element
            const uint64_t elem0 = chunk_elem0 + lane;
            uint64_t channel = per_channel ? elem0 / lay.channel_len - channel0 : 0;                   // within the chunk
            uint32_t in_channel = per_channel ? static_cast<uint32_t>(elem0 % lay.channel_len) : 0;
            float scale = per_channel ? scale_of(channel) : lay.scale;
            uint64_t out_at = c.out_offset + lane;
            auto emit_one = [&](int, uint32_t e, bool) {
                if constexpr (OUT == ANSZP_OUT_U8) static_cast<uint8_t*>(p.out)[out_at] = static_cast<uint8_t>(e >> 19);
                else if constexpr (OUT == ANSZP_OUT_F32) static_cast<float*>(p.out)[out_at] = scaled_high_half(e, scale);
                else static_cast<__bf16*>(p.out)[out_at] = static_cast<__bf16>(scaled_high_half(e, scale));
                out_at += N;
                if (per_channel) {
                    in_channel += N;
                    if (in_channel >= lay.channel_len) {
                        do { in_channel -= lay.channel_len; ++channel; } while (in_channel >= lay.channel_len);
                        scale = scale_of(channel);                         // beyond the layer's scales: 0, never stored
                    }
                }
            };
            // K steps of the plain form from a window loaded once: K * table_log + 31 bits must fit 128
            auto block_plain = [&](auto count_tag) {
                constexpr int K = static_cast<int>(decltype(count_tag)::value);
                const bool fetching = wants_words();
                Fetched f;
                if (fetching) fetch(mine, readable, fetched, f);
                uint32_t w0, w1, w2, w3;
                window(w0, w1, w2, w3);
                uint32_t sum = 0;                                 // 31 - nb_bits over the K steps
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    const uint32_t e = entry_at(X);
                    const uint32_t bits = (__brev(w0) >> (e & 31u)) >> 1;          // first bit read is the top bit; none: 0
                    X = next_entry_offset(e, bits);
                    const uint32_t nb = ~e;                                        // low five bits
                    w0 = __builtin_amdgcn_alignbit(w1, w0, nb);
                    w1 = __builtin_amdgcn_alignbit(w2, w1, nb);
                    w2 = __builtin_amdgcn_alignbit(w3, w2, nb);
                    w3 >>= (nb & 31u);
                    sum += e & 31u;
                    emit_one(k, e, k == K - 1);
                }
                abit += 31u * K - sum;
                if (fetching) {
                    land(ring, fetched, f);
                    fetched += kStreamFetchWords;
                }
            };
            uint32_t t = 0;
            if (fast) {
                for (; t + 8u <= full_steps; t += 8u) block_fast(std::integral_constant<int, 8>{}, emit_one);
                for (; t < full_steps; ++t) block_fast(std::integral_constant<int, 1>{}, emit_one);
                if (len > full_steps) block_fast(std::integral_constant<int, 1>{}, emit_one);
            } else {
                for (; t + 8u <= full_steps; t += 8u) block_plain(std::integral_constant<int, 8>{});
                for (; t < full_steps; ++t) block_plain(std::integral_constant<int, 1>{});
                if (len > full_steps) block_plain(std::integral_constant<int, 1>{});     // ragged tail: streams 0 .. n mod N - 1
            }
        }
        if (X != state0) err |= ANSZP_ST_BAD_STATE;          // state 0
        if (((abit + 31u) >> 5) != skew + n_words) err |= ANSZP_ST_BAD_LENGTH;
    }
    no_more_positions();
    err = wave_or(err);
    if (err && lane == 0) report(p.status, err);
}

// ---------------------------------------------------------------------------------------------
// Look-ahead path: conversion of decoded symbols on their way from the LDS ring to global memory
// (Sec. II-B: w = scale * (q - z)).
template <int OUT, bool PER_CHANNEL>
struct Flusher {
    static constexpr bool kFolded = (OUT == ANSZP_OUT_BF16 && !PER_CHANNEL);
    // Convert the 8 symbols of one lane (bytes of `s`, elements g .. g+7 of the output) and store them.
    // The stores are marked non-temporal: the weights are not read again by this library (measured
    // on the ResNet-50-shaped set: 30.4 -> 28.0 us per launch, with the same bytes fetched from
    // memory: the gain is in the L2's handling of the stores).
    static __device__ __forceinline__ void store8(const DecodeParams& p, const anszp_layer_t& lay, uint64_t g,
                                                  uint64_t layer_elem, uint2 s) {
        if constexpr (OUT == ANSZP_OUT_U8) {
            __builtin_nontemporal_store(words2{s.x, s.y}, reinterpret_cast<words2*>(static_cast<uint8_t*>(p.out) + g));
        } else {
            uint32_t sym[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { sym[i] = (s.x >> (8 * i)) & 0xFFu; sym[4 + i] = (s.y >> (8 * i)) & 0xFFu; }
            if constexpr (kFolded) {
                // Per-layer scale, bf16 out: float(q) - float(z) is exact, the product is rounded once, and two
                // weights are rounded to bf16 by one instruction.  (A table of the 256 weights in LDS, one look-up
                // per symbol, was slower: the storing wavefronts then wait for LDS, which the decoding and
                // expanding wavefronts keep busy.)
                const float zf = static_cast<float>(lay.zero_point), sc = lay.scale;
                auto weights = [&](uint32_t word, int i) {
                    const float a = sc * (static_cast<float>((word >> (16 * i)) & 0xFFu) - zf);
                    const float b = sc * (static_cast<float>((word >> (16 * i + 8)) & 0xFFu) - zf);
                    return __builtin_bit_cast(uint32_t, __builtin_convertvector(floats2{a, b}, bf16s2));
                };
                (void)sym;
                __builtin_nontemporal_store(words4{weights(s.x, 0), weights(s.x, 1), weights(s.y, 0), weights(s.y, 1)},
                                            reinterpret_cast<words4*>(static_cast<uint16_t*>(p.out) + g));
            } else {
                float v[8];
                if constexpr (PER_CHANNEL) {
                    const uint32_t e0 = static_cast<uint32_t>(layer_elem);
                    const uint32_t left = lay.channel_len - e0 % lay.channel_len;   // elements left in this channel
                    if (left >= 8u) {
                        const float sc = channel_scale(p, lay, layer_elem);
#pragma unroll
                        for (int i = 0; i < 8; ++i) v[i] = dequant(sym[i], lay.zero_point, sc);
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            v[i] = dequant(sym[i], lay.zero_point, channel_scale(p, lay, layer_elem + i));
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = dequant(sym[i], lay.zero_point, lay.scale);
                }
                if constexpr (OUT == ANSZP_OUT_F32) {
                    floats4* dst = reinterpret_cast<floats4*>(static_cast<float*>(p.out) + g);
                    __builtin_nontemporal_store(floats4{v[0], v[1], v[2], v[3]}, dst);
                    __builtin_nontemporal_store(floats4{v[4], v[5], v[6], v[7]}, dst + 1);
                } else {
                    const words4 o = {bf16_rne(v[0]) | (bf16_rne(v[1]) << 16), bf16_rne(v[2]) | (bf16_rne(v[3]) << 16),
                                      bf16_rne(v[4]) | (bf16_rne(v[5]) << 16), bf16_rne(v[6]) | (bf16_rne(v[7]) << 16)};
                    __builtin_nontemporal_store(o, reinterpret_cast<words4*>(static_cast<uint16_t*>(p.out) + g));
                }
            }
        }
    }
    // One element (tail of a chunk).
    static __device__ __forceinline__ void store1(const DecodeParams& p, const anszp_layer_t& lay, uint64_t g,
                                                  uint64_t layer_elem, uint32_t sym) {
        const float sc = PER_CHANNEL ? channel_scale(p, lay, layer_elem) : lay.scale;
        store_weight<OUT>(p.out, g, sym, lay.zero_point, sc);
    }
};

// ---------------------------------------------------------------------------------------------
// Which chunks a workgroup of the look-ahead kernel decodes.  A workgroup that has a CU to itself decodes a
// chunk fastest (its wavefronts get a SIMD each); two consecutive chunks of one layer (chunk numbers 2j and
// 2j+1) can share a workgroup and its LDS copy of the layer's table, each a little slower.  A launch with
// more chunks than the chip holds workgroups at once therefore pairs chunks, the most compressible first
// (few stream words: short chains), and only as many as it takes: of the levels below (stream bits per
// symbol under which a chunk may be paired) the lowest that leaves no more units than `capacity`.  The host
// does not see the descriptors, so every workgroup finds unit number `u` itself: thread t looks at chunks
// t, t + THREADS, ...; per level a 64-bit mask per 64 chunks marks those that start a unit; the masks go
// through LDS and every wavefront counts the levels' units and picks the u-th set bit of the chosen level.
// Launches with more than kPairScanRounds * THREADS chunks do not pair.
constexpr uint32_t kPairScanRounds = 4u;
constexpr uint32_t kPairLevels = 8u;
struct Unit { uint32_t first, count; };          // count 0: no such unit

// level from which a chunk may be paired, by its stream bits per symbol (level 0: nothing is paired; 7: everything)
__device__ __forceinline__ uint32_t pair_level_of(uint32_t payload_words, uint32_t n_symbols) {
    const float bits = 32.0f * static_cast<float>(payload_words), n = static_cast<float>(n_symbols);
    uint32_t level = 7u;
    if (bits < 1.2f * n) level = 6u;
    if (bits < 1.0f * n) level = 5u;
    if (bits < 0.8f * n) level = 4u;
    if (bits < 0.7f * n) level = 3u;
    if (bits < 0.6f * n) level = 2u;
    if (bits < 0.5f * n) level = 1u;
    return level;
}

// A chunk descriptor as two 16-byte words, and back (the scan below keeps the descriptors it has read, so that
// the unit's own need not be fetched again once the unit is known).
struct ChunkWords { uint4 a, b; };
__device__ __forceinline__ anszp_chunk_t chunk_of(const ChunkWords& w) {
    anszp_chunk_t c;
    c.layer_id = uniform(w.a.x); c.n_symbols = uniform(w.a.y);
    c.out_offset = uniform(w.a.z) | (uint64_t(uniform(w.a.w)) << 32);
    c.payload_offset = uniform(w.b.x) | (uint64_t(uniform(w.b.y)) << 32);
    c.payload_words = uniform(w.b.z); c.stream_offset = uniform(w.b.w);
    return c;
}
static_assert(sizeof(anszp_chunk_t) == 32, "two 16-byte words");

template <uint32_t THREADS>
__device__ __forceinline__ Unit find_unit(const DecodeParams& p, uint32_t u, uint32_t capacity, uint32_t pair_words,
                                          uint64_t* masks /* LDS, kPairLevels * (kPairScanRounds * THREADS / 64 + 1) + 8 words of 8 bytes */,
                                          anszp_chunk_t& c0, anszp_chunk_t& c1 /* the unit's chunks (the second repeats the first in a unit of one) */) {
    constexpr uint32_t kWaves = THREADS / kWave;
    constexpr uint32_t kMasks = kPairScanRounds * kWaves;
    static_assert(kMasks <= kWave, "one mask per lane");
    const uint32_t n = p.n_chunks;
    if (n > kPairScanRounds * THREADS || n <= capacity) {
        if (u < n) c0 = c1 = p.chunks[u];
        return Unit{u, u < n ? 1u : 0u};
    }
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = uniform(tid >> 6);
    const uint32_t rounds = (n + THREADS - 1u) / THREADS;
    uint32_t* const units = reinterpret_cast<uint32_t*>(masks + kPairLevels * kMasks);     // units per level
    ChunkWords* const handed = reinterpret_cast<ChunkWords*>(masks + kPairLevels * kMasks + 4u);   // the unit's descriptors
    ChunkWords seen[kPairScanRounds];
    uint32_t layer[kPairScanRounds], words[kPairScanRounds], symbols[kPairScanRounds];
#pragma unroll
    for (uint32_t k = 0; k < kPairScanRounds; ++k) {
        layer[k] = 0u; words[k] = 0u; symbols[k] = 1u;
        if (k < rounds) {
            const uint4* c = reinterpret_cast<const uint4*>(p.chunks + min(k * THREADS + tid, n - 1u));
            seen[k].a = c[0]; seen[k].b = c[1];
            layer[k] = seen[k].a.x; words[k] = seen[k].b.z; symbols[k] = seen[k].a.y;
        }
    }
    if (tid < kPairLevels) units[tid] = 0u;              // (while the loads are in flight)
    __syncthreads();
#pragma unroll
    for (uint32_t k = 0; k < kPairScanRounds; ++k) {
        if (k >= rounds) break;
        const uint32_t i = k * THREADS + tid;
        const uint32_t level = words[k] <= pair_words ? pair_level_of(words[k], symbols[k]) : kPairLevels;   // too long to share: never
        // (chunk i - 1 of an odd i sits in the lane below: blocks of 64 chunks start at even numbers; the
        // shuffles are done by every lane, the even lanes are their sources)
        const uint32_t layer_below = __shfl_up(layer[k], 1, kWave), level_below = __shfl_up(level, 1, kWave);
        // from this level on, chunk i is the second of a pair
        const uint32_t second_from = ((i & 1u) && layer[k] == layer_below) ? max(level, level_below) : kPairLevels;
#pragma unroll
        for (uint32_t j = 0; j < kPairLevels; ++j) {
            const uint64_t starts = __ballot(i < n && !(j >= second_from));
            if (lane == 0) {
                masks[j * kMasks + k * kWaves + wave] = starts;
                atomicAdd(&units[j], static_cast<uint32_t>(__popcll(starts)));
            }
        }
    }
    __syncthreads();
    // the lowest level that leaves no more units than there is room for (the last pairs all it can)
    uint32_t chosen = kPairLevels - 1u, total = 0;
    {
        const uint32_t mine = units[lane % kPairLevels];
        bool picked = false;
#pragma unroll
        for (uint32_t j = 0; j < kPairLevels; ++j) {
            const uint32_t count = __builtin_amdgcn_readlane(mine, j);
            if (!picked && (count <= capacity || j == kPairLevels - 1u)) { picked = true; chosen = j; total = count; }
        }
    }
    chosen = uniform(chosen);
    if (u >= total) return Unit{0u, 0u};
    const uint64_t m = lane < rounds * kWaves ? masks[chosen * kMasks + lane] : 0ull;
    uint32_t unused;
    const uint32_t ahead = wave_exclusive_sum(static_cast<uint32_t>(__popcll(m)), &unused);
    const uint64_t holds = __ballot(lane < kMasks && ahead <= u && u < ahead + static_cast<uint32_t>(__popcll(m)));
    const uint32_t which = static_cast<uint32_t>(__ffsll(static_cast<unsigned long long>(holds))) - 1u;   // exactly one lane
    const uint32_t lo = __shfl(static_cast<uint32_t>(m), which, kWave), hi = __shfl(static_cast<uint32_t>(m >> 32), which, kWave);
    const uint32_t rank = u - __shfl(ahead, which, kWave);            // the rank-th set bit of that mask
    const uint32_t below = __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));   // set bits below this lane's
    const uint64_t mask = (uint64_t(hi) << 32) | lo;
    const uint64_t found = __ballot(((mask >> lane) & 1ull) && below == rank);
    const uint32_t first = which * kWave + static_cast<uint32_t>(__ffsll(static_cast<unsigned long long>(found))) - 1u;
    // the chunk after it belongs to the unit when it starts none
    uint32_t count = 1u;
    if (first + 1u < n) {
        const uint32_t next = first + 1u;
        const uint32_t nlo = __shfl(static_cast<uint32_t>(m), next / kWave, kWave), nhi = __shfl(static_cast<uint32_t>(m >> 32), next / kWave, kWave);
        const uint64_t next_mask = (uint64_t(nhi) << 32) | nlo;
        if (!((next_mask >> (next % kWave)) & 1ull)) count = 2u;
    }
    // the threads that read the unit's descriptors hand them to everybody
#pragma unroll
    for (uint32_t k = 0; k < kPairScanRounds; ++k) {
        if (k >= rounds) break;
        const uint32_t i = k * THREADS + tid;
        if (i == first) handed[0] = seen[k];
        if (i == first + count - 1u) handed[1] = seen[k];
    }
    __syncthreads();
    c0 = chunk_of(handed[0]);
    c1 = chunk_of(handed[1]);
    return Unit{uniform(first), uniform(count)};
}

// ---------------------------------------------------------------------------------------------
// A prepared work assignment (anszp_plan_decode): what workgroup b of the look-ahead kernel would find out for
// itself at the start of every launch (its unit, the unit's chunk descriptors, their layer), written down once
// for arrays that stay as they are from launch to launch, one record of 128 bytes per workgroup.  The
// kernel checks a record's descriptors against the caller's buffers like any other, so a plan that no longer
// fits its arrays cannot make it read or write out of bounds.
struct PlanRecord {
    uint32_t tag, n_chunks, first, count;        // tag: kPlanTag + the geometry's tag
    anszp_chunk_t c0, c1;
    anszp_layer_t lay;                           // of the unit's chunks (zero when neither is in bounds)
    uint32_t dominant;                           // symbol of the layer's last state: the dominant symbol if there is one
    uint32_t chain;                              // look-ups expected of a stream of the unit's longer chunk, times the streams (0: not known)
    uint32_t unused[2];
};
static_assert(sizeof(PlanRecord) == 128, "one record per workgroup, 128 bytes");
constexpr uint32_t kPlanTag = 0x414E5300u;

template <class G>
__global__ __launch_bounds__(kBlock) void plan_units(DecodeParams p, PlanRecord* plan) {
    __shared__ uint64_t masks[kPairLevels * (kPairScanRounds * kBlock / kWave) + 16u];
    anszp_chunk_t c0, c1;
    const Unit unit = find_unit<kBlock>(p, unit_of_workgroup(blockIdx.x), max(p.n_cus, 1u) * G::kWorkgroupsPerCu, G::kPayloadWords, masks, c0, c1);
    const bool ok0 = unit.count != 0u && chunk_in_bounds(p, c0), ok1 = unit.count == 2u && chunk_in_bounds(p, c1);
    const uint32_t layer_id = ok0 ? c0.layer_id : c1.layer_id;
    const uint32_t* const triples = p.tables + size_t(ok0 || ok1 ? layer_id : 0u) * table_stride_words(p.table_log) + table_triples_offset(p.table_log);
    const uint32_t L = 1u << p.table_log;
    // How long a stream's chain of look-ups will be: an entry of the look-ahead table ends with a symbol that is not
    // the dominant one (or with a dominant one that had to read bits), so of n symbols about n * (1 - P(dominant))
    // cost a look-up each.  P(dominant) is the share of the table's states that carry the dominant symbol (Sec. II-A:
    // a symbol's states are its normalised frequency).  The stream words a chunk has say less: a layer of few
    // quantisation levels has short codes and as many look-ups.
    __shared__ uint32_t others;
    if (threadIdx.x == 0) others = 0u;
    __syncthreads();
    if (ok0 || ok1) {
        const uint32_t dominant = triples[L - 1u] >> 24;
        uint32_t mine = 0;
        for (uint32_t i = threadIdx.x; i < L; i += kBlock) mine += (triples[i] >> 24) != dominant ? 1u : 0u;
        if (mine) atomicAdd(&others, mine);
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    PlanRecord r = {};
    r.tag = kPlanTag + G::kTag; r.n_chunks = p.n_chunks; r.first = unit.first; r.count = unit.count;
    if (unit.count != 0u) {
        r.c0 = c0; r.c1 = c1;
        if (ok0 || ok1) {
            r.lay = p.layers[layer_id];
            r.dominant = triples[L - 1u] >> 24;
            const uint32_t longer = max(ok0 ? c0.n_symbols : 0u, ok1 ? c1.n_symbols : 0u);
            r.chain = static_cast<uint32_t>(min((uint64_t(longer) * others) >> p.table_log, uint64_t(0x0FFFFFFFu)));
        }
    }
    plan[gridDim.x + blockIdx.x] = r;              // (the second half of the plan's memory: plan_order puts the records in place)
}

// The records in the order the workgroups should take them: the chip starts workgroups in the order of their
// numbers, over about a microsecond, and the launch ends with its slowest unit, so the units with the longest
// chains (as plan_units expects them; two chunks in one workgroup run slower than one) go first.  Sorted units
// keep the mapping to the dies: units of one layer are alike and stay neighbours.  One workgroup; launches of
// more than kPlanOrderMax workgroups keep the order of the descriptors.
constexpr uint32_t kPlanOrderMax = 8192u;
__global__ __launch_bounds__(1024) void plan_order(PlanRecord* plan, uint32_t n) {
    __shared__ uint32_t cost[kPlanOrderMax];
    const PlanRecord* raw = plan + n;
    const uint32_t tid = threadIdx.x;
    if (n > kPlanOrderMax) {
        for (uint32_t i = tid; i < n; i += 1024u) plan[i] = raw[i];
        return;
    }
    for (uint32_t i = tid; i < n; i += 1024u) {
        const PlanRecord& r = raw[i];
        uint32_t c = 0;
        if (r.count == 1u) c = 4u * r.chain;
        else if (r.count == 2u) c = 5u * r.chain;
        cost[i] = c;
    }
    __syncthreads();
    for (uint32_t i = tid; i < n; i += 1024u) {
        const uint32_t mine = cost[i], unit = unit_of_workgroup(i);
        uint32_t rank = 0;
        for (uint32_t j = 0; j < n; ++j) {
            const uint32_t theirs = cost[j];
            rank += (theirs > mine || (theirs == mine && unit_of_workgroup(j) < unit)) ? 1u : 0u;
        }
        plan[workgroup_of_unit(rank)] = raw[i];
    }
}

// ---------------------------------------------------------------------------------------------
// The look-ahead kernel.  One workgroup = one unit (one or two chunks of a layer), twelve wavefronts:
// all stage, then up to seven per chunk keep a task:
//   decode    (one) lane k walks the automaton of stream k (Sec. III-B: a vector of states sharing one
//             table) through the look-ahead entries, in blocks of 8 look-ups with no per-step checks,
//             and logs 16 bits of every entry it passes and where every lane stands when a block begins;
//   expand    (two, taking the logged blocks in turn) turn logged entries into symbols in the chunk's LDS
//             ring (an entry stands for c symbols: c-1 copies of the dominant symbol, which the ring holds
//             as background, then its own), publish how far every stream has got, and check every stream's
//             end: the entry that holds the stream's last symbol must end with it and arrive in state 0
//             (entries never pass through state 0), having read the stream's words and no more;
//   store     (four for a single chunk, three per chunk of a pair) move finished slabs of the ring to
//             global memory, every fourth or third slab each, 16 bytes per lane and store.
// A lane joins a block while its stream is unfinished and the ring has room for 8 entries of 8 symbols
// (what the storing wavefronts have stored decides); a stream that ends inside a block goes on through
// whatever follows it: the table keeps every index in range, what it reads behind the chunk's words
// stays inside LDS, and symbols beyond the chunk's last land in ring slots nobody reads again.
// Hand-overs go through LDS words; LDS performs a wavefront's accesses in order, so a reader that
// sees a count sees everything written before it.  Every wait is bounded.
template <int OUT, bool PER_CHANNEL, class G>
__device__ __forceinline__ void decode_lookahead(const DecodeParams& p) {
    constexpr uint32_t kTableBytes = 16u << G::kTableLog;          // 2 L entries of 8 bytes
    constexpr uint32_t kRingElems = G::kRingElems;                 // LDS ring of decoded symbols (one byte each), per chunk
    constexpr uint32_t kPayloadWords = G::kPayloadWords;           // LDS window for one chunk's compressed words
    constexpr uint32_t kLogSlots = G::kLogSlots;                   // blocks in flight between decoding and expanding wavefront
    // LDS: 512 bytes not in use | table (where the hand-written look-ups expect it) | SIMD of each wavefront |
    // per chunk: hand-over words, positions, log, compressed words | ring 0 | ring 1 (aligned to the size of both)
    constexpr uint32_t kTableOff = 512u;
    constexpr uint32_t kSimdOff = kTableOff + kTableBytes;
    constexpr uint32_t kPipeOff = kSimdOff + 64u;
    constexpr uint32_t kTailWords = 8u;                             // zero words behind a chunk's last: a window of four words may start at the last
    constexpr uint32_t kWordsBytes = (kPayloadWords + kTailWords) * 4u;
    constexpr uint32_t kCtlOff = 0u;                                // within a chunk's area
    constexpr uint32_t kProgOff = kCtlOff + 64u;
    constexpr uint32_t kLogOff = kProgOff + kExpanders * kWave * 4u;      // (positions: a row per expanding wavefront)
    constexpr uint32_t kWordsOff = kLogOff + kLogSlots * kLogSlotBytes;   // the compressed words come last: a single chunk's
    constexpr uint32_t kPipeBytes = kWordsOff + kWordsBytes;             // may run on through the second chunk's area
    constexpr uint32_t kSoloWords = (kWordsBytes + kPipeBytes) / 4u - kTailWords;
    constexpr uint32_t kRingOff = (kPipeOff + 2u * kPipeBytes + 2u * kRingElems - 1u) / (2u * kRingElems) * (2u * kRingElems);
    constexpr uint32_t kLdsBytes = kRingOff + 2u * kRingElems;
    static_assert((kRingElems & (kRingElems - 1u)) == 0u && kTableOff == 512u, "rings aligned to their size; the table where the hand-written look-ups expect it");
    static_assert(kPipeOff % 16u == 0u && kPipeBytes % 16u == 0u && kCtlOff % 16u == 0u && kWordsOff % 16u == 0u, "LDS layout");
    static_assert(kRingElems % kSlab == 0u, "whole slabs");
    static_assert(G::kWorkgroupsPerCu * kLdsBytes <= 160u * 1024u, "workgroups per CU");
    static_assert(kLdsBytes * 8u < (1u << 22), "bit positions count from the start of LDS");
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLdsBytes];
    // hand-over words of a chunk: 0 blocks logged | 1, 2 the next block each expanding wavefront will take |
    // 3 no more blocks will be logged | 4..7 first element of the next slab each storing wavefront will take
    // (all ones where there is no such wavefront) | 8 a wait gave up
    enum { kLogged = 0, kNext0 = 1, kOver = 3, kStored0 = 4, kGaveUp = 8 };
    constexpr uint32_t kMaxStorers = 4u;
    static_assert(kExpanders == 2u, "hand-over words 1 and 2");
    constexpr uint32_t kElemBytes = OUT == ANSZP_OUT_U8 ? 1u : (OUT == ANSZP_OUT_F32 ? 4u : 2u);
    constexpr uint32_t kTableLoads = ((2u << G::kTableLog) / 2u + kBlock - 1u) / kBlock;          // 16-byte loads per thread
    constexpr uint32_t kWordLoads = (kPayloadWords / 4u + kBlock - 1u) / kBlock;                  // per chunk
    static_assert(kSoloWords <= 2u * kWordLoads * 4u * kBlock, "a single chunk's words are loaded by both chunks' loads");

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & (kWave - 1);
    const uint32_t wave = uniform(tid >> 6);
    const uint32_t N = p.n_streams;
    const uint32_t L = 1u << p.table_log;

    anszp_chunk_t c0, c1;        // descriptors (the second repeats the first when the unit is a single chunk)
    anszp_layer_t planned_lay;
    uint32_t planned_dominant = 0;
    Unit unit;
    if (p.plan) {
        // the unit as prepared: one record, read through the scalar cache
        const PlanRecord& r = reinterpret_cast<const PlanRecord*>(p.plan)[blockIdx.x];
        if (r.tag != kPlanTag + G::kTag || r.n_chunks != p.n_chunks || r.count > 2u) {       // not a plan for this launch
            if (tid == 0) report(p.status, ANSZP_ST_BAD_DESC);
            return;
        }
        unit = Unit{r.first, r.count};
        c0 = r.c0; c1 = r.c1; planned_lay = r.lay; planned_dominant = r.dominant;
    } else {
        unit = find_unit<kBlock>(p, unit_of_workgroup(blockIdx.x), max(p.n_cus, 1u) * G::kWorkgroupsPerCu, kPayloadWords,
                                 reinterpret_cast<uint64_t*>(lds + kPipeOff), c0, c1);
    }
    if (unit.count == 0u) return;
    // What the loads below touch depends on the chunk descriptors alone; whether the layer's scales cover the
    // chunks is looked at once the layer's descriptor has arrived, with everything else already on its way.
    const bool ok0 = chunk_in_bounds(p, c0), ok1 = unit.count == 2u && chunk_in_bounds(p, c1);
    if ((!ok0 && !ok1) || lds_address(lds) != 0u) {
        if (tid == 0) {
            report(p.status, lds_address(lds) != 0u ? ANSZP_ST_INTERNAL : ANSZP_ST_BAD_DESC);   // the hand-written parts address LDS from 0
            if (unit.count == 2u && lds_address(lds) == 0u) report(p.status, ANSZP_ST_BAD_DESC);
        }
        return;
    }
    const uint32_t layer_id = ok0 ? c0.layer_id : c1.layer_id;      // both alike when both are in bounds
    const anszp_layer_t lay = p.plan ? planned_lay : p.layers[layer_id];

    // Issue every global read that depends only on the descriptors before waiting for any of them (the
    // stream headers first: they are used first).
    const uint32_t hdr0 = (ok0 && lane < N) ? p.stream_hdr[c0.stream_offset + lane] : 0u;
    const uint32_t hdr1 = (ok1 && lane < N) ? p.stream_hdr[c1.stream_offset + lane] : 0u;
    const uint32_t* src = p.tables + layer_id * table_stride_words(p.table_log);
    const uint4* tsrc = reinterpret_cast<const uint4*>(src + table_lookahead_offset(p.table_log));   // 2 entries per load
    const uint32_t t_last = L - 1u;
    // (named values rather than arrays: an array that lives across a barrier is kept in scratch memory
    // by the compiler; loads beyond the geometry's count repeat the last row and are dropped)
    static_assert(kTableLoads <= 6u && kWordLoads <= 2u, "loads per thread are written out below");
    const uint4 tv0 = tsrc[min(tid, t_last)], tv1 = tsrc[min(tid + kBlock, t_last)], tv2 = tsrc[min(tid + 2u * kBlock, t_last)];
    uint4 tv3 = tv2, tv4 = tv2, tv5 = tv2;
    if constexpr (kTableLoads > 3u) {
        tv3 = tsrc[min(tid + 3u * kBlock, t_last)]; tv4 = tsrc[min(tid + 4u * kBlock, t_last)]; tv5 = tsrc[min(tid + 5u * kBlock, t_last)];
    }
    // (a single chunk may be longer than a chunk's own window: its words then run on through the second chunk's
    // area, and the second chunk's loads fetch them)
    constexpr uint32_t kRowsPerChunk = kWordLoads * kBlock;       // 16-byte rows of words a chunk's loads cover
    const bool single = unit.count == 1u;
    const uint32_t window0 = single ? kSoloWords : kPayloadWords;
    const uint32_t quads0 = ok0 ? min(c0.payload_words, window0) >> 2 : 0u;
    const uint32_t quads1 = ok1 ? min(c1.payload_words, kPayloadWords) >> 2 : (single && quads0 > kRowsPerChunk ? quads0 - kRowsPerChunk : 0u);
    const uint4* wsrc0 = quads0 ? reinterpret_cast<const uint4*>(p.payload + c0.payload_offset) : tsrc;
    const uint4* wsrc1 = !quads1 ? tsrc : single ? wsrc0 + kRowsPerChunk : reinterpret_cast<const uint4*>(p.payload + c1.payload_offset);
    const uint32_t w_last0 = quads0 ? min(quads0, kRowsPerChunk) - 1u : 0u, w_last1 = quads1 ? quads1 - 1u : 0u;
    const uint4 wv00 = wsrc0[min(tid, w_last0)], wv10 = wsrc1[min(tid, w_last1)];
    uint4 wv01 = wv00, wv11 = wv10;
    if constexpr (kWordLoads > 1u) { wv01 = wsrc0[min(tid + kBlock, w_last0)]; wv11 = wsrc1[min(tid + kBlock, w_last1)]; }
    uint32_t tail0 = 0, tail1 = 0;                        // the words behind the last whole row of four
    if (ok0 && tid < kTailWords && (quads0 << 2) + tid < c0.payload_words && c0.payload_words <= window0)
        tail0 = p.payload[c0.payload_offset + (quads0 << 2) + tid];
    if (ok1 && tid < kTailWords && (quads1 << 2) + tid < c1.payload_words && c1.payload_words <= kPayloadWords)
        tail1 = p.payload[c1.payload_offset + (quads1 << 2) + tid];
    const uint32_t top = src[table_triples_offset(p.table_log) + L - 1u];   // state L-1 carries the dominant symbol if there is one
    const bool in0 = ok0 && scales_in_bounds(p, lay, c0), in1 = ok1 && scales_in_bounds(p, lay, c1);
    if (tid == 0) {
        if (!in0) report(p.status, ANSZP_ST_BAD_DESC);
        if (unit.count == 2u && !in1) report(p.status, ANSZP_ST_BAD_DESC);
    }
    // What staging writes without having loaded anything: hand-over words, the log slots' rows of
    // bit positions, the positions, the rings' background.  With a prepared plan this is done while the loads
    // are in flight (the plan names the dominant symbol); without one the LDS it touches is still in use by
    // the search for the unit, and the dominant symbol is on its way with the table.
    const uint32_t storers = single ? 4u : 3u;           // storing wavefronts per chunk
    auto init_pipes = [&](uint32_t dominant) {
        if (tid < (single ? 16u : 2u * 16u)) {            // hand-over words (of both chunks)
            const uint32_t q = tid / 16u, i = tid % 16u;
            uint32_t v = 0u;
            if (i >= kNext0 && i < kNext0 + kExpanders) v = i - kNext0;
            if (i >= kStored0 && i < kStored0 + kMaxStorers) v = i - kStored0 < storers ? (i - kStored0) * kSlab : 0xFFFFFFFFu;
            reinterpret_cast<uint32_t*>(lds + kPipeOff + q * kPipeBytes + kCtlOff)[i] = v;
        }
        for (uint32_t t = tid; t < (single ? 1u : 2u) * kLogSlots * kWave; t += kBlock) {   // the rows of bit positions: no lane has taken part in any block
            const uint32_t q = t / (kLogSlots * kWave), i = t % (kLogSlots * kWave);
            reinterpret_cast<uint32_t*>(lds + kPipeOff + q * kPipeBytes + kLogOff + (i / kWave) * kLogSlotBytes + (kBlockLookups + 1u) * 2u * kWave)[i % kWave] = 0xFFFFFFFFu;
        }
        if (tid < (single ? 1u : 2u) * kExpanders * kWave) {   // where every stream is: its first element, or nothing to wait for
            const uint32_t q = tid / (kExpanders * kWave), l = tid % kWave;
            const uint32_t n_q = q ? (in1 ? c1.n_symbols : 0u) : (in0 ? c0.n_symbols : 0u);
            reinterpret_cast<uint32_t*>(lds + kPipeOff + q * kPipeBytes + kProgOff)[tid % (kExpanders * kWave)] = (l < N && l < n_q) ? l : 0xFFFFFFF0u;
        }
        const uint32_t fill = dominant * 0x01010101u;
        uint4* rdst = reinterpret_cast<uint4*>(lds + kRingOff);
#pragma unroll
        for (uint32_t k = 0; k < (2u * kRingElems / 16u + kBlock - 1u) / kBlock; ++k)
            if (tid + k * kBlock < 2u * kRingElems / 16u) rdst[tid + k * kBlock] = make_uint4(fill, fill, fill, fill);
    };
    if (p.plan) init_pipes(planned_dominant);
    // While those loads are in flight: where every stream's words begin, and the SIMD every wavefront
    // runs on (HW_ID bits 4..5).
    uint32_t total_words0, total_words1;
    const uint32_t first_word0 = wave_exclusive_sum(hdr0 >> 16, &total_words0), first_word1 = wave_exclusive_sum(hdr1 >> 16, &total_words1);
    uint32_t* const simd_of = reinterpret_cast<uint32_t*>(lds + kSimdOff);
    if (lane == 0) simd_of[wave] = (__builtin_amdgcn_s_getreg((31 << 11) | 4) >> 4) & 3u;
    __syncthreads();
    // Tasks.  A lone wavefront's speed is set by how often its SIMD lets it issue, so the two decoding
    // wavefronts get a SIMD each that they share with nothing but wavefronts that leave after staging;
    // expanding and storing wavefronts share the other two.  The second workgroup of a CU (small
    // geometry) mirrors the choice.
    enum { kDecode = 0, kExpand = 1, kStore = 2, kNoTask = 3 };
    uint32_t task = kNoTask, pipe = 0, sub = 0;          // sub: which of the chunk's expanding or storing wavefronts
    {
        constexpr uint32_t kWaves = kBlock / kWave;
        const uint32_t flip = G::kWorkgroupsPerCu > 1u ? ((blockIdx.x / max(p.n_cus, 1u)) & 1u) * 2u : 0u;
        const uint32_t theirs = lane < kWaves ? simd_of[lane] : 4u;                  // lane w: the SIMD of wavefront w
        const uint32_t my_simd = __builtin_amdgcn_readlane(theirs, wave);
        const uint64_t same = __ballot(theirs == my_simd);
        const uint32_t rank = static_cast<uint32_t>(__popcll(same & ((1ull << wave) - 1ull)));
        const bool even = __popcll(__ballot(theirs == 0u)) == 3 && __popcll(__ballot(theirs == 1u)) == 3 &&
                          __popcll(__ballot(theirs == 2u)) == 3 && __popcll(__ballot(theirs == 3u)) == 3;
        // three wavefronts on every SIMD (s2: the SIMD, r2: which of its three); any other placement: as
        // if wavefront w ran on SIMD w mod 4.
        const uint32_t s2 = even ? my_simd ^ flip : (wave & 3u);
        const uint32_t r2 = even ? rank : (wave >> 2);
        if (unit.count == 1u) {
            // one chunk: SIMD 0 decodes and does nothing else, SIMD 1 and 2 expand and store, SIMD 3 stores twice
            if (r2 == 0u) {
                if (s2 == 0u) task = kDecode;
                else if (s2 < 3u) { task = kExpand; sub = s2 - 1u; }
                else task = kStore;
            } else if (r2 == 1u && s2 != 0u) {
                task = kStore; sub = s2 == 3u ? 1u : s2 + 1u;
            }
        } else if (s2 < 2u) {
            // two chunks.  SIMD 0, 1: decode chunk 0, 1, and one storing wavefront of either chunk;
            // SIMD 2, 3: expand chunk 0, 1 (two wavefronts), and the chunk's third storing wavefront
            if (r2 == 0u) { task = kDecode; pipe = s2; }
            else { task = kStore; sub = (r2 - 1u) ^ s2; pipe = r2 - 1u; }
        } else if (r2 < kExpanders) {
            task = kExpand; pipe = s2 - 2u; sub = r2;
        } else {
            task = kStore; pipe = s2 - 2u; sub = 2u;
        }
    }
    pipe = uniform(pipe);
    task = uniform(task);
    sub = uniform(sub);

    // ---- stage: look-ahead entries, both chunks' compressed words, ring background, hand-over words
    {
        // every thread stores what it loaded, to the clamped index it loaded from (threads past the
        // end repeat the last row)
        uint4* tdst = reinterpret_cast<uint4*>(lds + kTableOff);
        tdst[min(tid, t_last)] = tv0;
        tdst[min(tid + kBlock, t_last)] = tv1;
        tdst[min(tid + 2u * kBlock, t_last)] = tv2;
        if constexpr (kTableLoads > 3u) {
            tdst[min(tid + 3u * kBlock, t_last)] = tv3;
            tdst[min(tid + 4u * kBlock, t_last)] = tv4;
            tdst[min(tid + 5u * kBlock, t_last)] = tv5;
        }
        uint4* wdst0 = reinterpret_cast<uint4*>(lds + kPipeOff + kWordsOff);
        uint4* wdst1 = single ? wdst0 + kRowsPerChunk : reinterpret_cast<uint4*>(lds + kPipeOff + kPipeBytes + kWordsOff);
        if (quads0) { wdst0[min(tid, w_last0)] = wv00; if constexpr (kWordLoads > 1u) wdst0[min(tid + kBlock, w_last0)] = wv01; }
        if (quads1) { wdst1[min(tid, w_last1)] = wv10; if constexpr (kWordLoads > 1u) wdst1[min(tid + kBlock, w_last1)] = wv11; }
        if (tid < kTailWords) {                           // tail words, then zeros for clamped reads
            reinterpret_cast<uint32_t*>(lds + kPipeOff + kWordsOff)[(quads0 << 2) + tid] = tail0;
            if (!single) reinterpret_cast<uint32_t*>(lds + kPipeOff + kPipeBytes + kWordsOff)[(quads1 << 2) + tid] = tail1;
        }
    }
    if (!p.plan) init_pipes(top >> 24);
    const uint32_t bg4 = (p.plan ? planned_dominant : top >> 24) * 0x01010101u;      // the rings' background: the dominant symbol
    __syncthreads();
    if (task == kNoTask || (pipe == 1u && !in1) || (pipe == 0u && !in0)) return;

    // ---- this wavefront's chunk
    const anszp_chunk_t c = pipe ? c1 : c0;
    const uint32_t hdr = pipe ? hdr1 : hdr0;
    const uint32_t pipe_off = kPipeOff + pipe * kPipeBytes;          // the chunk's area
    const uint32_t words_off = pipe_off + kWordsOff;                 // its compressed words
    // (a workgroup with a single chunk uses the space of both rings as one)
    const uint32_t ring_elems = unit.count == 1u ? 2u * kRingElems : kRingElems;
    const uint32_t ring_mask = ring_elems - 1u;
    uint8_t* const ring8 = lds + kRingOff + pipe * kRingElems;
    lds_flag_t* const ctl = (lds_flag_t*)(lds + pipe_off + kCtlOff);
    const uint32_t n = c.n_symbols;
    const uint64_t layer_elem0 = c.out_offset - lay.out_base;
    const uint32_t n_words = hdr >> 16;
    const uint32_t len = (lane < N && n > lane) ? (n - lane + N - 1u) / N : 0u;
    const uint32_t lane_end = lane < N ? lane + len * N : n;         // first element of this lane at or beyond the chunk's end
    const bool merged_ok = p.table_log <= G::kTableLog && c.payload_words <= (single ? kSoloWords : kPayloadWords) &&
                           ((c.out_offset * kElemBytes) & 15u) == 0 && n <= (1u << 24) && PER_CHANNEL == (lay.channel_len != 0) &&
                           (!PER_CHANNEL || layer_elem0 + n < (1ull << 32));
    if (!merged_ok) {                                     // the plain loop of Sec. II-A, table read from global memory
        if (task != kDecode) return;
        const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, WordTable{src + table_triples_offset(p.table_log)}, lane);
        if (err && lane == 0) report(p.status, err);
        return;
    }

    // Slabs of the ring are final once every unfinished lane's next symbol lies beyond them.  A lane
    // takes elements 8*lane .. 8*lane+7 of each half of a slab, so that every store instruction writes
    // one contiguous run; the slots go back to the background value.
    auto store_slab = [&](uint32_t first_elem) {
        uint8_t* q = ring8 + ((first_elem & ring_mask) + lane * 8u);         // the ring is a whole number of slabs
        const uint2 lo = *reinterpret_cast<const uint2*>(q);
        const uint2 hi = *reinterpret_cast<const uint2*>(q + kSlab / 2u);
        *reinterpret_cast<uint2*>(q) = make_uint2(bg4, bg4);
        *reinterpret_cast<uint2*>(q + kSlab / 2u) = make_uint2(bg4, bg4);
        const uint32_t first = first_elem + lane * 8u;
        Flusher<OUT, PER_CHANNEL>::store8(p, lay, c.out_offset + first, layer_elem0 + first, lo);
        Flusher<OUT, PER_CHANNEL>::store8(p, lay, c.out_offset + first + kSlab / 2u, layer_elem0 + first + kSlab / 2u, hi);
    };

    if (task == kStore) {
        // ---- storing wavefronts: wavefront `sub` takes every `storers`-th slab
        uint32_t mine = sub * kSlab, spins = 0;          // first element of the next slab this one takes
        for (;;) {
            uint32_t over_v, next_a, next_b;
            uint2 logged_next;                            // blocks logged, the first expanding wavefront's next block
            uint32_t next_1;
            asm volatile(                                // the flag first, the positions last
                "ds_read_b32 %[ov], %[ctla] offset:12\n"
                "ds_read2_b32 %[ln], %[ctla] offset1:1\n"
                "ds_read_b32 %[n1], %[ctla] offset:8\n"
                "ds_read_b32 %[na], %[pa]\n"
                "ds_read_b32 %[nb], %[pa] offset:256\n"
                "s_waitcnt lgkmcnt(0)\n"
                : [ov] "=&v"(over_v), [ln] "=&v"(logged_next), [n1] "=&v"(next_1), [na] "=&v"(next_a), [nb] "=&v"(next_b)
                : [ctla] "v"(pipe_off + kCtlOff), [pa] "v"(pipe_off + kProgOff + lane * 4u)
                : "memory");
            static_assert(kExpanders == 2u && kWave * 4u == 256u, "two rows of positions, 256 bytes apart");
            // A block is expanded once the wavefront whose turn it was has moved past it: every block below both
            // wavefronts' next one is, and a lane's position after the last of those is the smaller of the two
            // rows (positions only grow).  Once no more blocks will be logged and all have been expanded, every
            // stream is complete (the row of the wavefront that did not expand the last block stays behind).
            const bool last_pass = uniform(over_v) && uniform(logged_next.x) <= min(uniform(logged_next.y), uniform(next_1));
            const uint32_t next = last_pass ? 0xFFFFFFFFu : min(next_a, next_b);
            const uint32_t before = mine;
            while (mine + kSlab <= n && __ballot(next < mine + kSlab) == 0) {
                store_slab(mine);
                mine += storers * kSlab;
            }
            if (mine != before) {
                asm volatile("ds_write_b32 %[wa], %[st]\n" :: [wa] "v"(pipe_off + kCtlOff + 4u * (kStored0 + sub)), [st] "v"(mine) : "memory");
                spins = 0;
            }
            if (last_pass) break;
            if (mine == before) {
                if (uniform(ctl[kGaveUp])) return;
                if (++spins > p.spin_limit) {
                    if (lane == 0) { ctl[kGaveUp] = 1u; report(p.status, ANSZP_ST_INTERNAL); }
                    return;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        // the elements behind the last whole slab, by the wavefront whose turn that slab would have been
        const uint32_t rest = n / kSlab * kSlab;
        if ((rest / kSlab) % storers == sub)
            for (uint32_t j = rest + lane; j < n; j += kWave)
                Flusher<OUT, PER_CHANNEL>::store1(p, lay, c.out_offset + j, layer_elem0 + j, ring8[j & ring_mask]);
        return;
    }

    const uint32_t total_words = pipe ? total_words1 : total_words0, first_word = pipe ? first_word1 : first_word0;
    const uint32_t first_bit = (words_off + 4u * min(first_word, c.payload_words)) << 3;   // counted from the start of LDS

    if (task == kExpand) {
        // ---- expanding wavefronts.  The two of a chunk take the logged blocks in turn (this one: sub, sub + 2,
        // ...); a block's log slot holds all a block needs: the position of every lane when the block began, the
        // entries, where the lane's next look-up starts, and the lane's bit position after the block, tagged with
        // the block's number by the lanes that took part.  Every pass reads the count of logged blocks and, in
        // the same batch of LDS reads, the slot: if the count (read first) says the block is there, what was
        // read after it is the block.
        __builtin_amdgcn_s_setprio(2);                   // ahead of the storing wavefronts
        uint32_t err = (sub == 0u && total_words != c.payload_words) ? ANSZP_ST_BAD_DESC : 0u;
        if (sub == 0u && lane < N && !(lane < n)) {      // no symbols: the initial state must be the final one
            if ((hdr & (L - 1u)) != 0u) err |= ANSZP_ST_BAD_STATE;
            if (n_words != 0u) err |= ANSZP_ST_BAD_LENGTH;
        }
        uint32_t block = sub, spins = 0;
        uint32_t ne = (lane < N && lane < n) ? lane : 0xFFFFFFF0u;          // as staged: after the last block (none yet)
        // the block a lane's stream ends in (of this wavefront's blocks), kept for the checks behind the loop
        uint32_t end_ent[kBlockLookups + 1u] = {}, end_bit_after = 0, end_ne_before = 0;
        bool ended_here = false;
        constexpr uint32_t kBitRow = (kBlockLookups + 1u) * 2u * kWave;      // offset of the row of bit positions in a log slot
        constexpr uint32_t kPosRow = kBitRow + 4u * kWave;                   // and of the row of positions
        typedef __attribute__((address_space(3))) uint8_t lds_uint8_t;
        const uint32_t ring_at = lds_address(ring8);     // a multiple of the ring's size: its bits and an element's index do not overlap
        for (;;) {
            const uint32_t slot = block & (kLogSlots - 1u);
            uint32_t logged_v, ent[kBlockLookups + 1u], bit_after, ne_before;
            asm volatile(
                "ds_read_b32 %[lg], %[ctla]\n"
                "ds_read_u16 %[a0], %[loga]\n"
                "ds_read_u16 %[a1], %[loga] offset:128\n"
                "ds_read_u16 %[a2], %[loga] offset:256\n"
                "ds_read_u16 %[a3], %[loga] offset:384\n"
                "ds_read_u16 %[a4], %[loga] offset:512\n"
                "ds_read_u16 %[a5], %[loga] offset:640\n"
                "ds_read_u16 %[a6], %[loga] offset:768\n"
                "ds_read_u16 %[a7], %[loga] offset:896\n"
                "ds_read_u16 %[a8], %[loga] offset:1024\n"
                "ds_read_b32 %[ba], %[bita] offset:%[bitrow]\n"
                "ds_read_b32 %[nb], %[bita] offset:%[posrow]\n"
                "s_waitcnt lgkmcnt(0)\n"
                : [lg] "=&v"(logged_v), [ba] "=&v"(bit_after), [nb] "=&v"(ne_before),
                  [a0] "=&v"(ent[0]), [a1] "=&v"(ent[1]), [a2] "=&v"(ent[2]), [a3] "=&v"(ent[3]), [a4] "=&v"(ent[4]),
                  [a5] "=&v"(ent[5]), [a6] "=&v"(ent[6]), [a7] "=&v"(ent[7]), [a8] "=&v"(ent[8])
                : [ctla] "v"(pipe_off + kCtlOff),
                  [loga] "v"(pipe_off + kLogOff + slot * kLogSlotBytes + lane * 2u), [bita] "v"(pipe_off + kLogOff + slot * kLogSlotBytes + lane * 4u),
                  [bitrow] "n"(kBitRow), [posrow] "n"(kPosRow)
                : "memory");
            if (uniform(logged_v) <= block) {            // not logged yet
                if (uniform(ctl[kOver])) {               // the count may have moved before the flag was set
                    if (uniform(ctl[kLogged]) <= block) break;
                    continue;
                }
                if (uniform(ctl[kGaveUp])) return;
                if (++spins > p.spin_limit) {
                    if (lane == 0) { ctl[kGaveUp] = 1u; report(p.status, ANSZP_ST_INTERNAL); }
                    return;
                }
                __builtin_amdgcn_s_sleep(1);
                continue;
            }
            spins = 0;
            ne = ne_before;                              // (every lane's, whether it took part or not)
            const bool took_part = (bit_after >> 22) == (block & 0x3FFu) && ne_before < lane_end;   // (a lane that never took part keeps the tag it was staged with)
            if (took_part) {
                // entries 0..7: bits 0..7 symbol | 8..11 T | 12..14 c-1 | 15 entry of state 0; 8: address of the lane's next entry
#pragma unroll
                for (uint32_t k = 0; k < kBlockLookups; ++k) {
                    const uint32_t last = __umul24((ent[k] >> 12) & 7u, N) + ne;
                    *reinterpret_cast<lds_uint8_t*>(static_cast<uintptr_t>((last & ring_mask) | ring_at)) = static_cast<uint8_t>(ent[k]);
                    ne = last + N;
                }
            }
            block += kExpanders;
            // publish the lanes' positions, then the next block, issued after the ring writes above (the slot may
            // be logged over from here on: what follows works on the registers)
            asm volatile("ds_write_b32 %[pa], %[ne]\n"
                         "ds_write_b32 %[nxa], %[nx]\n"
                         :: [pa] "v"(pipe_off + kProgOff + sub * (kWave * 4u) + lane * 4u), [ne] "v"(ne),
                            [nxa] "v"(pipe_off + kCtlOff + 4u * (kNext0 + sub)), [nx] "v"(block)
                         : "memory");
            if (took_part && ne >= lane_end) {           // the stream's last symbol lies in this block: looked at behind the loop
#pragma unroll
                for (uint32_t k = 0; k <= kBlockLookups; ++k) end_ent[k] = ent[k];
                end_bit_after = bit_after;
                end_ne_before = ne_before;
                ended_here = true;
            }
        }
        // Streams that ended in one of this wavefront's blocks (once each, so this waits until no block is held up
        // by it): find the entry the last symbol lies in.
        if (ended_here) {
            uint32_t consumed = 0;
#pragma unroll
            for (uint32_t k = 0; k < kBlockLookups; ++k) consumed += (end_ent[k] >> 8) & 15u;
            uint32_t pos = end_ne_before, bits = (end_bit_after & 0x3FFFFFu) - consumed;     // where the stream stood when the block began
            bool found = false;
#pragma unroll
            for (uint32_t k = 0; k < kBlockLookups; ++k) {
                const uint32_t after = pos + (((end_ent[k] >> 12) & 7u) + 1u) * N;
                bits += (end_ent[k] >> 8) & 15u;
                if (!found && after >= lane_end) {
                    found = true;
                    // it must end with the entry, in state 0, the stream's words read and no more
                    const bool in_state_0 = k + 1u < kBlockLookups ? (end_ent[k + 1u] >> 15) != 0u : end_ent[kBlockLookups] < 16u;
                    if (after != lane_end || !in_state_0) err |= ANSZP_ST_BAD_STATE;
                    if (((bits - first_bit + 31u) >> 5) != n_words) err |= ANSZP_ST_BAD_LENGTH;
                }
                pos = after;
            }
        }
        // the wavefront that expanded the last block knows where every stream stands: at its end
        if (block >= kExpanders && uniform(ctl[kLogged]) == block - kExpanders + 1u && lane < N && ne < lane_end) err |= ANSZP_ST_INTERNAL;
        err = wave_or(err);
        if (err && lane == 0) report(p.status, err);
        return;
    }

    // ---- decoding wavefront
    __builtin_amdgcn_s_setprio(3);
    const uint32_t last_word = words_off + (c.payload_words << 2);       // address of the zero words behind the payload
    const uint32_t* const lds_words = reinterpret_cast<const uint32_t*>(lds + words_off);
    // Look-ahead entries are indexed by 2 * state + the next stream bit (peeked, not yet read).
    const uint32_t index0 = 2u * (hdr & (L - 1u)) + (lds_words[min(first_word, c.payload_words)] & 1u);
    uint2 e = reinterpret_cast<const uint2*>(lds + kTableOff)[index0];
    uint32_t abit = first_bit;                           // bit position, counted from the start of LDS
    uint32_t ne = (lane < N && lane < n) ? lane : lane_end;
    uint32_t logged = 0, spins = 0;
    bool gave_up = false;
    // the first eight hand-over words in two LDS reads
    auto hand_over_words = [&](uint4& stored) {
        uint4 v;
        asm volatile("ds_read_b128 %[v], %[ctla]\n ds_read_b128 %[w], %[ctla] offset:16\n s_waitcnt lgkmcnt(0)\n"
                     : [v] "=&v"(v), [w] "=&v"(stored) : [ctla] "v"(pipe_off + kCtlOff) : "memory");
        return v;
    };
    static_assert(kLogged == 0 && kNext0 == 1 && kExpanders == 2u && kStored0 == 4 && kMaxStorers == 4u, "the hand-over words as the decoding wavefront reads them");
    // A block of 8 look-ups, hand-scheduled.  A look-up costs the LDS round trip plus the two instructions
    // between an entry's arrival and the next read; what else is issued while the wavefront waits for an
    // entry is free (up to a dozen instructions or so):
    //   v = r >> (31 - T)            the next T+1 stream bits, r = the window's first word bit-reversed
    //   address' = 8 v + 8 base      Sec. II-A: newX + bits, plus the peeked bit
    //   e' = table[address'];  log[k] = e (its upper half);  window >>= T (funnel shifts);  r = bitrev(w0)
    //   sum += e                     bits 0..8: 31 - T per look-up; bits 9..15: c - 1 per look-up (sums of up to 16 fit)
    // At the start of a block every lane loads four words of its stream (128 bits, at least 97 of them
    // ahead of its bit position: 8 look-ups use at most 8 * 12 and peek one more).  The window is shifted
    // only as far up as a later look-up of the block can still read: with j look-ups to follow only the
    // first 12 j + 1 bits matter, so register m is shifted while 12 j + 1 > 32 m (a register that is no
    // longer shifted goes stale; what it feeds into its lower neighbour lies beyond that reach).  A block
    // ends by logging where each lane's next look-up starts and the lane's bit position tagged with the
    // block's number (a lane that sat the block out keeps an older tag), reloading the words of the lanes
    // that took part and deciding who may run the next block from the words the other wavefronts publish.
#define ANSZP_SHIFT_W0 "v_alignbit_b32 v28, v29, v28, v35\n"
#define ANSZP_SHIFT_W1 ANSZP_SHIFT_W0 "v_alignbit_b32 v29, v30, v29, v35\n"
#define ANSZP_SHIFT_W2 ANSZP_SHIFT_W1 "v_alignbit_b32 v30, v31, v30, v35\n"
#define ANSZP_LOOKUP(WAIT, ELO, EHI, FB, K, SHIFT, SUM, BESIDE)                         \
        "s_waitcnt lgkmcnt(" WAIT ")\n"                                                \
        "v_lshrrev_b32 v36, " ELO ", v53\n"                                            \
        "v_lshl_add_u32 v36, v36, 3, " EHI "\n"                                        \
        "ds_read_b64 " FB ", v36 offset:512\n"                                         \
        "ds_write_b16_d16_hi v42, " ELO " offset:" K "*128\n"                          \
        "v_not_b32 v35, " ELO "\n"                                                     \
        SHIFT                                                                          \
        "v_bfrev_b32 v53, v28\n"                                                       \
        SUM BESIDE
#define ANSZP_AB(WAIT, K, SHIFT, BESIDE) ANSZP_LOOKUP(WAIT, "v24", "v25", "v[26:27]", K, SHIFT, "v_add_u32 v37, v37, v24\n", BESIDE)
#define ANSZP_BA(WAIT, K, SHIFT, BESIDE) ANSZP_LOOKUP(WAIT, "v26", "v27", "v[24:25]", K, SHIFT, "v_add_u32 v37, v37, v26\n", BESIDE)
    static_assert(ANSZP_MAX_TABLE_LOG <= 12 && kBlockLookups == 8u, "the reach of a look-up assumed by the window shifts");
    static_assert(kLogSlotBytes == 1664u, "log slot: nine rows of 16 bits per lane, then two rows of 32");
    const uint32_t reach = kBlockLookups * kLookaheadMaxSymbols * N;      // a block advances a lane by at most 8 entries of 8 symbols
    if (reach >= ring_elems) {                                            // (the host picks a geometry with room)
        if (lane == 0) { ctl[kGaveUp] = 1u; report(p.status, ANSZP_ST_INTERNAL); }
        return;
    }
    const uint32_t room = ring_elems - reach;
    while (!gave_up) {
        if (__ballot(ne < lane_end) == 0) break;          // every stream has ended
        uint4 slabs;
        const uint4 seen = hand_over_words(slabs);
        const uint32_t stored = min(min(uniform(slabs.x), uniform(slabs.y)), min(uniform(slabs.z), uniform(slabs.w)));
        const uint32_t expanded = min(uniform(seen.y), uniform(seen.z));      // every block below this one has been expanded
        const uint32_t limit = min(lane_end, stored + room);
        if (__ballot(ne < limit) == 0 || logged - expanded >= kLogSlots) {        // ring or log full: wait
            if (uniform(ctl[kGaveUp]) || ++spins > p.spin_limit) gave_up = true;
            __builtin_amdgcn_s_sleep(1);
            continue;
        }
        spins = 0;
        uint32_t logged_v = logged;
        // What the wavefront issues between the last look-up of a block and the first of the next one is what a
        // block costs beyond its eight LDS round trips (there it is bound by what it issues, beside a look-up by
        // the round trip), so only what needs the last entry stands there: the new bit position and the reload
        // of the window, the count of symbols, who may run the next block.  The rest is issued beside the
        // look-ups: the other wavefronts' hand-over words are read beside the fourth (late, so that they are fresh) and reduced
        // to scalars beside the sixth and seventh, the next block's number and log slot beside the second and third, the sums over the
        // first seven entries beside the seventh; a block is published beside the first look-up of the next one.
        asm volatile(
            "v_mov_b32 v24, %[elo]\n v_mov_b32 v25, %[ehi]\n v_mov_b32 v52, %[ab]\n v_mov_b32 v39, %[ne]\n"
            "v_mov_b32 v43, %[ctla]\n"
            "v_readfirstlane_b32 s44, %[logged]\n"
            "s_mov_b64 s[40:41], exec\n"
            "s_lshl_b32 s49, %[nstr], 3\n"
            "v_cmp_gt_u32 vcc, %[lim], v39\n"
            "v_lshrrev_b32 v38, 3, v52\n"
            "v_and_b32 v38, 0x1ffffffc, v38\n"
            "v_min_u32 v38, %[lastw], v38\n"
            "ds_read2_b32 v[28:29], v38 offset1:1\n"
            "ds_read2_b32 v[30:31], v38 offset0:2 offset1:3\n"
            "s_and_b64 s[42:43], s[40:41], vcc\n"      /* lanes that run this block (some do) */
            "s_and_b32 s45, s44, %[slotmask]\n"        /* the block's log slot */
            "s_mul_i32 s46, s45, 1664\n"
            "v_add_u32 v42, s46, %[lanelog]\n"         /* this lane's 16-bit column in the slot */
            "v_add_u32 v47, s46, %[lanebit]\n"         /* and its word in the rows of bit positions and positions */
            "ds_write_b32 v47, v39 offset:%[posrow]\n" /* where every lane stands as the block begins */
            "s_mov_b64 exec, s[42:43]\n"
            "s_waitcnt lgkmcnt(1)\n"
            "s_branch 3f\n"
            "1:\n"
            "ds_write_b32 v47, v39 offset:%[posrow]\n"
            "s_mov_b64 exec, s[42:43]\n"
            "s_waitcnt lgkmcnt(2)\n"                   /* the window words (and the entry the block starts from) */
            "3:\n"
            "v_alignbit_b32 v28, v29, v28, v52\n"
            "v_bfrev_b32 v53, v28\n"
            "v_lshrrev_b32 v36, v24, v53\n"            /* first look-up */
            "v_lshl_add_u32 v36, v36, 3, v25\n"
            "ds_read_b64 v[26:27], v36 offset:512\n"
            "ds_write_b16_d16_hi v42, v24 offset:0\n"
            "v_mov_b32 v41, s44\n"
            "ds_write_b32 v43, v41\n"                  /* publish the block before this one */
            "v_alignbit_b32 v29, v30, v29, v52\n"      /* the rest of the window into place */
            "v_alignbit_b32 v30, v31, v30, v52\n"
            "v_lshrrev_b32 v31, v52, v31\n"
            "v_not_b32 v35, v24\n"
            ANSZP_SHIFT_W2
            "v_bfrev_b32 v53, v28\n"
            "v_mov_b32 v37, v24\n"
            "v_add_u32 v34, 31*8, v52\n"               /* the bit position if the block read no bits */
            ANSZP_BA("2", "1", ANSZP_SHIFT_W2,
                     "v_add_u32 v40, s49, v39\n"       /* the position if every look-up stood for one symbol */
                     "s_lshl_b32 s51, s44, 22\n"       /* this block's number, as the bit positions are tagged with it */
                     "s_add_u32 s44, s44, 1\n")        /* from here on: the next block */
            ANSZP_AB("1", "2", ANSZP_SHIFT_W1,
                     "s_and_b32 s45, s44, %[slotmask]\n"
                     "s_mul_i32 s46, s45, 1664\n")     /* the next block's log slot */
            ANSZP_BA("1", "3", ANSZP_SHIFT_W1,         /* (not earlier: what they say decides who runs the next block) */
                     "ds_read_b128 v[48:51], v43\n"    /* blocks logged, the expanding wavefronts' next blocks */
                     "ds_read_b128 v[54:57], v43 offset:16\n")   /* elements stored (by up to four wavefronts) */
            ANSZP_AB("3", "4", ANSZP_SHIFT_W1, "")
            ANSZP_BA("1", "5", ANSZP_SHIFT_W0,
                     "v_min_u32 v49, v49, v50\n"       /* blocks expanded: every one below the next of either expanding wavefront */
                     "v_min3_u32 v50, v54, v55, v56\n" /* elements stored: every slab below the next one of any storing wavefront */
                     "v_readfirstlane_b32 s47, v49\n"  /* (a lane read must not directly follow the instruction that writes its register) */
                     "v_min_u32 v50, v50, v57\n"
                     "s_nop 0\n"
                     "v_readfirstlane_b32 s48, v50\n"
                     "s_add_u32 s48, s48, %[room]\n"   /* lanes below this position fit the ring, */
                     "s_min_u32 s48, s48, %[nsym]\n")  /* and have not ended (a lane's end is its first position at or beyond the chunk's) */
            ANSZP_AB("1", "6", ANSZP_SHIFT_W0,
                     "s_sub_u32 s45, s44, s47\n"
                     "s_cmp_lt_u32 s45, %[slots]\n"    /* unless the next log slot may still be in use, */
                     "s_cselect_b64 s[52:53], s[40:41], 0\n"   /* every lane may go on that fits the ring */
                     "v_and_b32 v46, 0x1ff, v37\n"
                     "v_sub_u32 v33, v34, v46\n"       /* minus the stream bits seven look-ups consumed */
                     "v_bfe_u32 v46, v37, 9, 7\n"
                     "v_mad_u32_u24 v40, v46, %[nstr], v40\n")   /* plus the symbols seven entries stand for beyond one each */
            "s_waitcnt lgkmcnt(1)\n"                   /* the eighth look-up shifts no window */
            "v_lshrrev_b32 v36, v26, v53\n"
            "v_lshl_add_u32 v45, v36, 3, v27\n"
            "ds_read_b64 v[24:25], v45 offset:512\n"
            "ds_write_b16_d16_hi v42, v26 offset:7*128\n"
            "ds_write_b16 v42, v45 offset:8*128\n"   /* where the next look-up starts: below 16 in state 0 */
            "v_sub_u32_sdwa v52, v33, v26 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0\n"   /* and the eighth: the new bit position */
            "v_lshrrev_b32 v38, 3, v52\n"              /* the block's lanes reload their words (a lane that sat the */
            "v_and_b32 v38, 0x1ffffffc, v38\n"         /* block out has not moved: its words are still in place)    */
            "ds_read2_b32 v[28:29], v38 offset1:1\n"
            "ds_read2_b32 v[30:31], v38 offset0:2 offset1:3\n"
            "v_bfe_u32 v46, v26, 9, 3\n"
            "v_mad_u32_u24 v39, v46, %[nstr], v40\n"   /* the new position */
            "v_or_b32 v46, s51, v52\n"                 /* bit position after the block, tagged with the block's number */
            "ds_write_b32 v47, v46 offset:%[bitrow]\n"
            "s_mov_b64 exec, s[40:41]\n"
            "v_cmp_gt_u32 vcc, s48, v39\n"             /* lanes that can run another block */
            "v_add_u32 v42, s46, %[lanelog]\n"
            "v_add_u32 v47, s46, %[lanebit]\n"
            "s_and_b64 s[42:43], s[52:53], vcc\n"
            "s_cbranch_scc1 1b\n"
            "v_mov_b32 v41, s44\n"
            "ds_write_b32 v43, v41\n"                  /* nobody can: publish the last block */
            "v_cmp_gt_u32 vcc, %[nsym], v39\n"
            "s_cbranch_vccz 2f\n"                      /* every stream has ended */
            "s_mov_b32 s54, 24\n"                      /* some wait for the storing or expanding wavefronts: a few looks from here, */
            "4:\n"                                     /* with fresh hand-over words (leaving and coming back costs a block's time) */
            "ds_read_b128 v[48:51], v43\n"
            "ds_read_b128 v[54:57], v43 offset:16\n"
            "s_waitcnt lgkmcnt(0)\n"
            "v_min_u32 v49, v49, v50\n"
            "v_min3_u32 v50, v54, v55, v56\n"
            "v_readfirstlane_b32 s47, v49\n"
            "v_min_u32 v50, v50, v57\n"
            "s_nop 0\n"
            "v_readfirstlane_b32 s48, v50\n"
            "s_add_u32 s48, s48, %[room]\n"
            "s_min_u32 s48, s48, %[nsym]\n"
            "s_sub_u32 s45, s44, s47\n"
            "s_cmp_lt_u32 s45, %[slots]\n"
            "s_cselect_b64 s[52:53], s[40:41], 0\n"
            "v_cmp_gt_u32 vcc, s48, v39\n"
            "s_and_b64 s[42:43], s[52:53], vcc\n"
            "s_cbranch_scc1 1b\n"
            "s_sleep 1\n"
            "s_sub_u32 s54, s54, 1\n"
            "s_cmp_lg_u32 s54, 0\n"
            "s_cbranch_scc1 4b\n"
            "2:\n"
            "s_waitcnt lgkmcnt(0)\n"
            "v_mov_b32 %[elo], v24\n v_mov_b32 %[ehi], v25\n v_mov_b32 %[ab], v52\n v_mov_b32 %[ne], v39\n"
            "v_mov_b32 %[logged], s44\n"
            : [elo] "+v"(e.x), [ehi] "+v"(e.y), [ab] "+v"(abit), [ne] "+v"(ne), [logged] "+v"(logged_v)
            : [lim] "v"(limit), [room] "s"(uniform(room)), [nstr] "s"(uniform(N)), [nsym] "s"(uniform(n)),
              [lastw] "s"(uniform(last_word)), [ctla] "s"(uniform(pipe_off + kCtlOff)),
              [lanelog] "v"(pipe_off + kLogOff + lane * 2u), [lanebit] "v"(pipe_off + kLogOff + lane * 4u),
              [slots] "n"(kLogSlots), [slotmask] "n"(kLogSlots - 1u), [bitrow] "n"((kBlockLookups + 1u) * 2u * kWave),
              [posrow] "n"((kBlockLookups + 1u) * 2u * kWave + 4u * kWave)
            : "memory", "vcc", "scc", "s40", "s41", "s42", "s43", "s44", "s45", "s46", "s47", "s48", "s49", "s51", "s52", "s53", "s54",
              "v24", "v25", "v26", "v27", "v28", "v29", "v30",
              "v31", "v33", "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v45", "v46", "v47",
              "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57");
        logged = uniform(logged_v);
    }
#undef ANSZP_AB
#undef ANSZP_BA
#undef ANSZP_LOOKUP
#undef ANSZP_SHIFT_W2
#undef ANSZP_SHIFT_W1
#undef ANSZP_SHIFT_W0
    if (gave_up) {
        if (lane == 0) { ctl[kGaveUp] = 1u; report(p.status, ANSZP_ST_INTERNAL); }
        return;
    }
    // no more blocks: the expanding and storing wavefronts finish what is logged
    if (lane == 0) ctl[kOver] = 1u;
}

template <int OUT, bool PER_CHANNEL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(3, 3)))   // one workgroup per CU
void decode_merged(DecodeParams p) { decode_lookahead<OUT, PER_CHANNEL, LargeLds>(p); }

template <int OUT, bool PER_CHANNEL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(6, 6)))   // two workgroups per CU
void decode_merged_small(DecodeParams p) { decode_lookahead<OUT, PER_CHANNEL, SmallLds>(p); }


// ---------------------------------------------------------------------------------------------
// Decode tables built on the device (Sec. II-A table, Sec. III-A one table per layer): one workgroup
// per table, same words as anszp_build_tables_host.
//
// The host merges the per-symbol position sequences (this library's choice of spread, which Sec. II-A
// leaves open: occurrence i of a symbol of frequency f sits at (2i+1)/(2f); ties go to the smaller
// symbol) with a heap.  Here every occurrence computes its
// own rank instead: the number of occurrences of every other symbol that come before it, in exact
// integer arithmetic, is a quotient.  The rank is the state X; the occurrence index gives the
// sub-state f + i, hence nb_bits and newX; the look-ahead entries then follow the step table in LDS.
constexpr uint32_t kBuildThreads = 1024u;

__global__ __launch_bounds__(kBuildThreads) void build_tables_kernel(const uint32_t* freqs, int table_log, uint32_t* tables,
                                                                     uint32_t* status) {
    constexpr uint32_t kStates = 1u << ANSZP_MAX_TABLE_LOG;
    __shared__ uint32_t freq[ANSZP_ALPHABET];           // of every symbol
    __shared__ uint32_t used_sym[ANSZP_ALPHABET];       // symbols with f > 0, in increasing order
    __shared__ uint32_t used_first[ANSZP_ALPHABET + 1]; // occurrences of the symbols before each of them
    __shared__ uint32_t n_used, total, dominant_sym;
    __shared__ uint8_t st_sym[kStates], st_nb[kStates];
    __shared__ uint16_t st_newX[kStates];
    const uint32_t tid = threadIdx.x;
    const uint32_t L = 1u << table_log;
    const uint32_t* f = freqs + size_t(blockIdx.x) * ANSZP_ALPHABET;
    uint32_t* out = tables + size_t(blockIdx.x) * table_stride_words(table_log);
    if (tid < ANSZP_ALPHABET) freq[tid] = f[tid];
    __syncthreads();
    if (tid == 0) {
        uint32_t n = 0, acc = 0, dom = 0xFFFFFFFFu;
        for (uint32_t sy = 0; sy < ANSZP_ALPHABET; ++sy) {
            const uint32_t fs = freq[sy];
            if (fs > L / 2) dom = sy;
            if (fs) {
                used_sym[n] = sy;
                used_first[n] = acc;
                ++n;
            }
            acc = min(acc + min(fs, L + 1u), L + 1u);   // saturating: a row that overshoots is rejected below
        }
        used_first[n] = acc;
        n_used = n;
        total = acc;
        dominant_sym = dom;
    }
    __syncthreads();
    if (total != L) {                                   // not a normalised row: an all-zero table and a status bit
        for (uint32_t i = tid; i < 8u * L; i += kBuildThreads) out[i] = 0u;
        if (tid == 0 && status) report(status, ANSZP_ST_BAD_FREQ);
        return;
    }
    const uint32_t used = n_used;
    for (uint32_t g = tid; g < L; g += kBuildThreads) {
        // occurrence g in symbol order: symbol used_sym[k], its i-th occurrence
        uint32_t lo = 0, hi = used;                     // used_first[lo] <= g < used_first[hi]
        while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (used_first[mid] <= g) lo = mid; else hi = mid;
        }
        const uint32_t sy = used_sym[lo], fs = freq[sy], i = g - used_first[lo];
        uint32_t rank = i;
        for (uint32_t k = 0; k < used; ++k) {
            if (k == lo) continue;
            const uint32_t fo = freq[used_sym[k]];
            // occurrences i' of the other symbol with (2i'+1) fs < (2i+1) fo, or <= when it is the smaller symbol
            // (all quantities are below 2^26: i < fs <= L, fo <= L <= 4096)
            const int32_t q = static_cast<int32_t>((2u * i + 1u) * fo) - static_cast<int32_t>(fs);
            uint32_t before;
            if (k < lo) before = q < 0 ? 0u : static_cast<uint32_t>(q) / (2u * fs) + 1u;
            else before = q <= 0 ? 0u : (static_cast<uint32_t>(q) + 2u * fs - 1u) / (2u * fs);
            rank += min(before, fo);
        }
        // Sec. II-A: sub-state f + i, shifted left until it lies in [L, 2L)
        const uint32_t v = fs + i;
        const uint32_t shift = static_cast<uint32_t>(table_log) - (31u - static_cast<uint32_t>(__clz(v)));
        st_sym[rank] = static_cast<uint8_t>(sy);
        st_nb[rank] = static_cast<uint8_t>(shift);
        st_newX[rank] = static_cast<uint16_t>((v << shift) - L);
    }
    __syncthreads();
    // every word the planes below do not fill is zero
    for (uint32_t i = tid; i < 2u * L; i += kBuildThreads) { out[i] = 0u; if (i < L) out[3u * L + i] = 0u; }
    __syncthreads();
    for (uint32_t X = tid; X < L; X += kBuildThreads) {
        out[table_triples_offset(table_log) + X] = uint32_t(st_newX[X]) | (uint32_t(st_nb[X]) << 16) | (uint32_t(st_sym[X]) << 24);
        if (L <= 256u) {                                // Sec. II-A: three bytes per state
            uint8_t* bytes = reinterpret_cast<uint8_t*>(out + table_bytes_offset(table_log));
            bytes[3u * X] = st_sym[X];
            bytes[3u * X + 1u] = st_nb[X];
            bytes[3u * X + 2u] = static_cast<uint8_t>(st_newX[X]);
        }
    }
    // look-ahead entries: up to kLookaheadMaxSymbols steps merged into one look-up, indexed by the state and
    // the next bit; a run never passes through state 0 (a stream then always ends where an entry ends)
    const uint32_t dominant = dominant_sym;
    uint32_t* ahead = out + table_lookahead_offset(table_log);
    for (uint32_t e = tid; e < 2u * L; e += kBuildThreads) {
        const uint32_t X = e >> 1, b = e & 1u;
        uint32_t Y = X, count = 0, bits = 0, last_sym = 0, saved_Y = 0, saved_count = 0;
        bool took_b = false, may_take_b = true;
        int32_t base = 0;
        for (;;) {
            const uint32_t n = st_nb[Y];
            const bool room = count + 1u < kLookaheadMaxSymbols;       // another symbol may follow this one
            const bool is_dominant = uint32_t(st_sym[Y]) == dominant;
            if (is_dominant && room && n == 0u && st_newX[Y] != 0u) { ++count; Y = st_newX[Y]; continue; }
            if (is_dominant && room && n == 1u && !took_b && may_take_b && (uint32_t(st_newX[Y]) | b) != 0u) {
                saved_Y = Y; saved_count = count;
                took_b = true; ++count; Y = uint32_t(st_newX[Y]) | b;
                continue;
            }
            if (took_b && 1u + n > uint32_t(ANSZP_MAX_TABLE_LOG)) {    // too many bits for one look-up: the 1-bit step is the last
                Y = saved_Y; count = saved_count; took_b = false; may_take_b = false;
                continue;
            }
            bits = (took_b ? 1u : 0u) + n;
            base = int32_t(2u * st_newX[Y]) - (took_b ? int32_t(b << (n + 1u)) : 0);
            last_sym = st_sym[Y];
            ++count;
            break;
        }
        ahead[2u * e] = lookahead_first_word(bits, count, last_sym, X == 0u);
        ahead[2u * e + 1u] = lookahead_second_word(base);
    }
}

// Sec. II-B alone.
template <int OUT>
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* sym, uint64_t n, anszp_layer_t lay,
                                                      const float* scales, uint64_t n_scales, void* out) {
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) {
        float scale = lay.scale;
        if (lay.channel_len) {
            const uint64_t ch = lay.scales_offset + i / lay.channel_len;
            scale = ch < n_scales ? scales[ch] : 0.0f;
        }
        store_weight<OUT>(out, i, sym[i], lay.zero_point, scale);
    }
}

// Compute units of the current device (queried once per device; the cache is a table of atomics, so
// concurrent callers at worst both query).
uint32_t device_cus() {
    static std::atomic<uint32_t> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256u;
    uint32_t n = cached[dev].load(std::memory_order_relaxed);
    if (!n) {
        int count = 0;
        if (hipDeviceGetAttribute(&count, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || count <= 0) count = 256;
        n = static_cast<uint32_t>(count);
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

template <int OUT>
void launch_decode(const DecodeParams& p, uint32_t n_chunks, bool per_channel, bool stepwise, bool shared, bool streaming,
                   bool small, bool byte_table, hipStream_t s) {
    if (byte_table) {
        hipLaunchKernelGGL(decode_byte_table<OUT>, dim3((n_chunks + kByteWaves - 1) / kByteWaves), dim3(kByteWaves * kWave), 0, s, p);
    } else if (stepwise && streaming) {
        // chunks dealt evenly to as many workgroups as fill whole rounds of the device's CUs
        const uint32_t per_round = device_cus() * uint32_t(kStreamDecoders);
        const uint32_t rounds = (n_chunks + per_round - 1u) / per_round;
        const uint32_t groups = std::min(n_chunks, device_cus() * rounds);
        hipLaunchKernelGGL(decode_streaming<OUT>, dim3(groups), dim3(kStreamWaves * kWave), 0, s, p, n_chunks, groups);
    } else if (stepwise && shared)
        hipLaunchKernelGGL(decode_stepwise_shared<OUT>, dim3((n_chunks + kSharedWaves - 1) / kSharedWaves),
                           dim3(kSharedWaves * kWave), 0, s, p, n_chunks);
    else if (stepwise) hipLaunchKernelGGL(decode_stepwise<OUT>, dim3(n_chunks), dim3(kWave), 0, s, p);
    else {
        const dim3 grid(mapped_workgroups(n_chunks));
        if (small && per_channel) hipLaunchKernelGGL((decode_merged_small<OUT, true>), grid, dim3(kBlock), 0, s, p);
        else if (small) hipLaunchKernelGGL((decode_merged_small<OUT, false>), grid, dim3(kBlock), 0, s, p);
        else if (per_channel) hipLaunchKernelGGL((decode_merged<OUT, true>), grid, dim3(kBlock), 0, s, p);
        else hipLaunchKernelGGL((decode_merged<OUT, false>), grid, dim3(kBlock), 0, s, p);
    }
}

// The bound of every wait between wavefronts, in polls.  Tests lower it (anszp_test_set_spin_limit) to see that a
// hand-over that does not complete ends in ANSZP_ST_INTERNAL and a drained launch, not in a hang.
std::atomic<uint32_t> spin_limit_for_tests{kSpinLimit};

// What a launch would be: checks of the arguments, the kernel's parameters, which kernel.
struct LaunchChoice { bool stepwise, byte_table, shared, streaming, small, per_channel; };

int choose_launch(const anszp_decode_args_t* a, int mode, DecodeParams& p, LaunchChoice& k);

// plan: null, or device memory written by plan_units for these arrays (used by the look-ahead kernel only);
// plan_only: write the plan instead of decoding
int decode_impl(const anszp_decode_args_t* a, int mode, void* hip_stream, uint32_t* plan = nullptr, uint64_t plan_bytes = 0,
                bool plan_only = false) {
    if (!a) return ANSZP_E_NULL;
    if (a->n_chunks == 0) return ANSZP_OK;
    DecodeParams p;
    LaunchChoice k;
    const int rc = choose_launch(a, mode, p, k);
    if (rc != ANSZP_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint32_t nc = static_cast<uint32_t>(a->n_chunks);
    const bool lookahead = !k.stepwise && !k.byte_table;
    if (plan || plan_only) {
        if (!plan) return ANSZP_E_NULL;
        if ((reinterpret_cast<uintptr_t>(plan) & 15) || plan_bytes < 2u * uint64_t(mapped_workgroups(nc)) * sizeof(PlanRecord)) return ANSZP_E_RANGE;
    }
    if (plan_only) {
        // (a launch that does not go to the look-ahead kernel needs no plan: the memory stays as it is, and
        // anszp_decode_planned does not read it)
        if (lookahead) {
            const dim3 grid(mapped_workgroups(nc));
            if (k.small) hipLaunchKernelGGL(plan_units<SmallLds>, grid, dim3(kBlock), 0, s, p, reinterpret_cast<PlanRecord*>(plan));
            else hipLaunchKernelGGL(plan_units<LargeLds>, grid, dim3(kBlock), 0, s, p, reinterpret_cast<PlanRecord*>(plan));
            hipLaunchKernelGGL(plan_order, dim3(1), dim3(1024), 0, s, reinterpret_cast<PlanRecord*>(plan), grid.x);
        }
        return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
    }
    p.plan = lookahead ? plan : nullptr;
    switch (a->out_dtype) {
        case ANSZP_OUT_U8: launch_decode<ANSZP_OUT_U8>(p, nc, k.per_channel, k.stepwise, k.shared, k.streaming, k.small, k.byte_table, s); break;
        case ANSZP_OUT_F32: launch_decode<ANSZP_OUT_F32>(p, nc, k.per_channel, k.stepwise, k.shared, k.streaming, k.small, k.byte_table, s); break;
        default: launch_decode<ANSZP_OUT_BF16>(p, nc, k.per_channel, k.stepwise, k.shared, k.streaming, k.small, k.byte_table, s); break;
    }
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}

int choose_launch(const anszp_decode_args_t* a, int mode, DecodeParams& p, LaunchChoice& k) {
    if (!a->tables || !a->chunks || !a->stream_hdr || !a->layers || !a->out || !a->status) return ANSZP_E_NULL;
    if (!a->payload && a->payload_words) return ANSZP_E_NULL;
    if (a->table_log < 1 || a->table_log > ANSZP_MAX_TABLE_LOG || a->n_streams < 1 ||
        a->n_streams > ANSZP_MAX_STREAMS || a->out_dtype > ANSZP_OUT_BF16 || a->n_tables == 0 ||
        a->n_chunks >= (1ull << 31) || (reinterpret_cast<uintptr_t>(a->payload) & 15) ||
        (reinterpret_cast<uintptr_t>(a->tables) & 15) ||
        (reinterpret_cast<uintptr_t>(a->out) & 15) || mode < 0 || mode > 5 || (mode == 5 && a->table_log > 8))
        return ANSZP_E_RANGE;
    p.tables = a->tables; p.chunks = a->chunks; p.stream_hdr = a->stream_hdr; p.payload = a->payload;
    p.layers = a->layers; p.scales = a->scales; p.out = a->out; p.status = a->status;
    p.n_stream_hdr = a->n_stream_hdr; p.payload_words = a->payload_words;
    p.n_scales = a->scales ? a->n_scales : 0; p.out_elems = a->out_elems;
    p.n_tables = a->n_tables; p.table_log = a->table_log; p.n_streams = a->n_streams;
    p.n_cus = device_cus();
    p.n_chunks = static_cast<uint32_t>(a->n_chunks);
    p.plan = nullptr;
    p.spin_limit = spin_limit_for_tests.load(std::memory_order_relaxed);
    // chunks whose compressed words cannot fit the look-ahead kernel's LDS window would all take its
    // fallback: they go to the streaming kernel, whatever their number (measured on 772 to 24,704
    // chunks of 82 KB of words: 5 to 7 times faster than one step-wise wavefront per chunk)
    const uint64_t mean_words = a->payload_words / a->n_chunks;
    k.stepwise = mode == 1 || mode == 3 || mode == 4 || (mode == 0 && mean_words > LargeLds::kPayloadWords);
    k.byte_table = mode == 5;
    k.shared = mode == 3;
    k.streaming = mode == 4 || (mode == 0 && k.stepwise);
    // small tables and short chunks: the variant that fits two workgroups on a CU
    k.small = a->table_log <= SmallLds::kTableLog && 2u * mean_words <= SmallLds::kPayloadWords &&
              kBlockLookups * kLookaheadMaxSymbols * a->n_streams < SmallLds::kRingElems;     // a block must fit its ring
    k.per_channel = a->scales != nullptr && a->n_scales != 0;
    return ANSZP_OK;
}

// The plan that anszp_decode_static_plan keeps: device memory of the library's own, one array per device.
constexpr uint32_t kStaticPlanChunks = 4096u;
static __device__ __align__(256) unsigned char scratch[2u * size_t(kStaticPlanChunks) * sizeof(PlanRecord)];
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_of_device[kMaxDevices];

// The address of this device's copy of `scratch` (looked up once per device).
void* device_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* ptr = scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        scratch_of_device[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

}  // namespace

extern "C" {

int anszp_build_tables(const uint32_t* freqs_host, int n_tables, int table_log,
                       uint32_t* tables_dev, void* hip_stream) {
    if (!freqs_host || !tables_dev) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_tables < 1) return ANSZP_E_RANGE;
    if (reinterpret_cast<uintptr_t>(tables_dev) & 15) return ANSZP_E_RANGE;
    const size_t entries = size_t(n_tables) * table_stride_words(table_log);
    uint32_t* staging = nullptr;
    if (hipHostMalloc(reinterpret_cast<void**>(&staging), entries * sizeof(uint32_t), hipHostMallocDefault) != hipSuccess)
        return ANSZP_E_NOMEM;
    int rc = anszp_build_tables_host(freqs_host, n_tables, table_log, staging);
    if (rc == ANSZP_OK) {
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        if (hipMemcpyAsync(tables_dev, staging, entries * sizeof(uint32_t), hipMemcpyHostToDevice, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            rc = ANSZP_E_HIP;
    }
    (void)hipHostFree(staging);
    return rc;
}

int anszp_build_tables_device(const uint32_t* freqs_dev, int n_tables, int table_log,
                              uint32_t* tables_dev, uint32_t* status_dev, void* hip_stream) {
    if (!freqs_dev || !tables_dev) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_tables < 1) return ANSZP_E_RANGE;
    if (reinterpret_cast<uintptr_t>(tables_dev) & 15) return ANSZP_E_RANGE;
    hipLaunchKernelGGL(build_tables_kernel, dim3(static_cast<uint32_t>(n_tables)), dim3(kBuildThreads), 0,
                       static_cast<hipStream_t>(hip_stream), freqs_dev, table_log, tables_dev, status_dev);
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}

int anszp_decode(const anszp_decode_args_t* args, void* hip_stream) { return decode_impl(args, 0, hip_stream); }

void anszp_test_set_spin_limit(uint32_t polls) { spin_limit_for_tests.store(polls ? polls - 1u : kSpinLimit, std::memory_order_relaxed); }

uint64_t anszp_plan_bytes(uint64_t n_chunks) {
    if (n_chunks >= (1ull << 31)) return 0;
    return 2u * uint64_t(mapped_workgroups(static_cast<uint32_t>(n_chunks))) * sizeof(PlanRecord);
}

int anszp_plan_decode(const anszp_decode_args_t* args, void* plan_dev, uint64_t plan_bytes, void* hip_stream) {
    return decode_impl(args, 0, hip_stream, static_cast<uint32_t*>(plan_dev), plan_bytes, true);
}

int anszp_decode_planned(const anszp_decode_args_t* args, const void* plan_dev, uint64_t plan_bytes, void* hip_stream) {
    if (!plan_dev) return ANSZP_E_NULL;
    return decode_impl(args, 0, hip_stream, static_cast<uint32_t*>(const_cast<void*>(plan_dev)), plan_bytes, false);
}

int anszp_decode_static_plan(const anszp_decode_args_t* args, int replan, void* hip_stream) {
    if (!args) return ANSZP_E_NULL;
    if (args->n_chunks > kStaticPlanChunks) return ANSZP_E_RANGE;
    uint32_t* plan = static_cast<uint32_t*>(device_scratch());
    if (!plan) return ANSZP_E_HIP;
    if (replan) {
        const int rc = decode_impl(args, 0, hip_stream, plan, sizeof(scratch), true);
        if (rc != ANSZP_OK) return rc;
    }
    return decode_impl(args, 0, hip_stream, plan, sizeof(scratch), false);
}

int anszp_decode_variant(const anszp_decode_args_t* args, int variant, void* hip_stream) {
    return decode_impl(args, variant, hip_stream);
}

int anszp_dequant_zp(const uint8_t* symbols_dev, uint64_t n, const anszp_layer_t* layer,
                     const float* scales_dev, uint64_t n_scales, void* out_dev, int out_dtype,
                     void* hip_stream) {
    if (!layer) return ANSZP_E_NULL;
    if (out_dtype != ANSZP_OUT_F32 && out_dtype != ANSZP_OUT_BF16) return ANSZP_E_RANGE;
    if (n == 0) return ANSZP_OK;
    if (!symbols_dev || !out_dev || (layer->channel_len && !scales_dev)) return ANSZP_E_NULL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint64_t want = (n + 255) / 256;
    const dim3 grid(static_cast<uint32_t>(want < 65536 ? want : 65536)), block(256);
    if (out_dtype == ANSZP_OUT_F32)
        hipLaunchKernelGGL(dequant_kernel<ANSZP_OUT_F32>, grid, block, 0, s, symbols_dev, n, *layer, scales_dev, n_scales, out_dev);
    else
        hipLaunchKernelGGL(dequant_kernel<ANSZP_OUT_BF16>, grid, block, 0, s, symbols_dev, n, *layer, scales_dev, n_scales, out_dev);
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}

}  // extern "C"
