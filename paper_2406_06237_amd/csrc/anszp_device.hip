// Device side of libanszp for gfx950 (MI355X): tANS decode kernels with fused zero-point
// dequantisation, and the stand-alone dequantiser.
//
// Paper sections followed: Sec. II-A (one decode step = table look-up, read nb_bits, state =
// newX + bits; empty-label transitions read no bits), Sec. III-B (a vector of states, one per
// stream, all sharing one table: here a 64-lane wavefront is the vector and a lane is a stream),
// Sec. III-A (one table per layer), Sec. II-B (w = scale * (q - z)).
//
// Two code paths produce identical results:
//   decode_chunk_stepwise  one look-up per symbol, words read from global memory; handles every
//                          geometry the ABI allows.
//   decode_chunk_merged    look-ups use the merged half of the table entries (a run of empty-label
//                          transitions of the dominant symbol plus the step that ends it is ONE
//                          look-up), the chunk's compressed words are staged in LDS, symbols are
//                          gathered in an LDS ring and leave as 16-byte-per-lane coalesced stores.
// The merged path needs the chunk's words to fit its LDS window and the chunk's first output
// element to be 16-byte aligned; other chunks take the step-wise path inside the same launch.
#include "anszp.h"

#include <hip/hip_runtime.h>

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 1024;                   // 16 wavefronts stage; wavefront 0 decodes
constexpr uint32_t kTableBytes = 8u << ANSZP_MAX_TABLE_LOG;   // 32 KiB of LDS entries
constexpr uint32_t kRingBytes = 32u * 1024u;   // LDS ring of decoded codes (2 bytes each)
constexpr uint32_t kRingElems = kRingBytes / 2u;
constexpr uint32_t kSlab = 512u;               // elements flushed per wave store (8 per lane)
constexpr uint32_t kPayloadWords = 3584u;      // LDS window for one chunk's compressed words
constexpr uint32_t kMaxMerged = 8u;

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
};

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

// Exclusive prefix sum over the 64 lanes of a wavefront; *total receives the sum.
__device__ __forceinline__ uint32_t wave_exclusive_sum(uint32_t v, uint32_t* total) {
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t up = __shfl_up(inc, d, kWave);
        if (static_cast<int>(threadIdx.x & (kWave - 1)) >= d) inc += up;
    }
    *total = __shfl(inc, kWave - 1, kWave);
    return inc - v;
}

__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) v |= __shfl_xor(v, d, kWave);
    return v;
}

// True (for the whole workgroup) when the chunk descriptor stays inside the caller's buffers.
__device__ __forceinline__ bool chunk_in_bounds(const DecodeParams& p, const anszp_chunk_t& c) {
    return c.layer_id < p.n_tables && c.n_symbols <= (1u << 31) &&
           c.out_offset <= p.out_elems && c.n_symbols <= p.out_elems - c.out_offset &&
           c.payload_offset <= p.payload_words && c.payload_words <= p.payload_words - c.payload_offset &&
           uint64_t(c.stream_offset) + p.n_streams <= p.n_stream_hdr;
}

__device__ __forceinline__ float channel_scale(const DecodeParams& p, const anszp_layer_t& lay, uint64_t layer_elem) {
    const uint64_t ch = lay.scales_offset + layer_elem / lay.channel_len;
    return ch < p.n_scales ? p.scales[ch] : 0.0f;
}

// ---------------------------------------------------------------------------------------------
// One look-up per symbol (Sec. III-B: n look-ups and n small additions for a stream of n
// weights).  Executed by one wavefront; `table` is 2^table_log dwords of LDS holding the
// (newX, nb_bits, symbol) half of the entries.  Returns the chunk's error bits (wave-uniform).
template <int OUT>
__device__ uint32_t decode_chunk_stepwise(const DecodeParams& p, const anszp_chunk_t& c, const anszp_layer_t& lay,
                                          const uint32_t* table, uint32_t lane) {
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
            const uint32_t e = table[X];
            const uint32_t nb = (e >> 16) & 0xFFu;
            if (have < nb) {
                buf |= uint64_t(ahead) << have;
                have += 32;
                ++next_word;
                ahead = word_at(next_word);
            }
            const uint32_t bits = static_cast<uint32_t>(buf) & ((1u << nb) - 1u);
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
    const uint32_t* src = p.tables + (uint64_t(c.layer_id) << (p.table_log + 1));    // first half: the paper's triple
    for (uint32_t i = lane; i < (1u << p.table_log); i += kWave) table[i] = src[i];
    const anszp_layer_t lay = p.layers[c.layer_id];
    __syncthreads();
    const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, table, lane);
    if (err && lane == 0) report(p.status, err);
}

// ---------------------------------------------------------------------------------------------
// Merged-run path.
//
// LDS entry (8 bytes) derived from the merged half of a table entry while staging:
//   lo: newX' * 8, the byte offset of the next entry before the stream bits are OR-ed in
//   hi: bits 0..4 nb_bits' | bits 8..10 c-1 | bit 15 end-flag | bits 16..31 code of symbol'
// One look-up emits c symbols: c-1 copies of the dominant symbol, which the ring already holds
// as background, then symbol'.  code = bf16 weight when the output is bf16 with a per-layer
// scale (dequantisation folded into the table), else the symbol itself and dequantisation
// happens when a slab leaves the ring.
template <int OUT, bool PER_CHANNEL>
struct Flusher {
    // Convert the 8 codes of one lane (elements g .. g+7 of the output) and store them.
    static __device__ __forceinline__ void store8(const DecodeParams& p, const anszp_layer_t& lay, uint64_t g,
                                                  uint64_t layer_elem, uint4 codes) {
        if constexpr (OUT == ANSZP_OUT_BF16 && !PER_CHANNEL) {
            *reinterpret_cast<uint4*>(static_cast<uint16_t*>(p.out) + g) = codes;
        } else {
            const uint32_t w[4] = {codes.x, codes.y, codes.z, codes.w};
            uint32_t sym[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { sym[2 * i] = w[i] & 0xFFFFu; sym[2 * i + 1] = w[i] >> 16; }
            if constexpr (OUT == ANSZP_OUT_U8) {
                uint2 o;
                o.x = sym[0] | (sym[1] << 8) | (sym[2] << 16) | (sym[3] << 24);
                o.y = sym[4] | (sym[5] << 8) | (sym[6] << 16) | (sym[7] << 24);
                *reinterpret_cast<uint2*>(static_cast<uint8_t*>(p.out) + g) = o;
            } else {
                float v[8];
                if constexpr (PER_CHANNEL) {
                    const uint32_t e0 = static_cast<uint32_t>(layer_elem);
                    const uint32_t left = lay.channel_len - e0 % lay.channel_len;   // elements left in this channel
                    if (left >= 8u) {
                        const float s = channel_scale(p, lay, layer_elem);
#pragma unroll
                        for (int i = 0; i < 8; ++i) v[i] = dequant(sym[i], lay.zero_point, s);
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
                    float4* dst = reinterpret_cast<float4*>(static_cast<float*>(p.out) + g);
                    dst[0] = make_float4(v[0], v[1], v[2], v[3]);
                    dst[1] = make_float4(v[4], v[5], v[6], v[7]);
                } else {
                    uint4 o;
                    o.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
                    o.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
                    o.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
                    o.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
                    *reinterpret_cast<uint4*>(static_cast<uint16_t*>(p.out) + g) = o;
                }
            }
        }
    }
    // One element (tail of a chunk).
    static __device__ __forceinline__ void store1(const DecodeParams& p, const anszp_layer_t& lay, uint64_t g,
                                                  uint64_t layer_elem, uint32_t code) {
        if constexpr (OUT == ANSZP_OUT_BF16 && !PER_CHANNEL) {
            static_cast<uint16_t*>(p.out)[g] = static_cast<uint16_t>(code);
        } else {
            const float s = PER_CHANNEL ? channel_scale(p, lay, layer_elem) : lay.scale;
            store_weight<OUT>(p.out, g, code, lay.zero_point, s);
        }
    }
};

template <int OUT, bool PER_CHANNEL>
__global__ __launch_bounds__(kBlock) void decode_merged(DecodeParams p) {
    // one LDS block, carved by hand so that the compressed words sit at offset 0 (their two-dword
    // reads have no room for a large immediate offset), then the table, then the ring
    constexpr uint32_t kWordsBytes = (kPayloadWords + 8u) * 4u;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kWordsBytes + kTableBytes + kRingBytes];
    uint32_t* const lds_words = reinterpret_cast<uint32_t*>(lds);
    uint8_t* const lds_table = lds + kWordsBytes;
    uint16_t* const lds_ring = reinterpret_cast<uint16_t*>(lds + kWordsBytes + kTableBytes);
    constexpr bool kFolded = (OUT == ANSZP_OUT_BF16 && !PER_CHANNEL);
    constexpr uint32_t kElemBytes = OUT == ANSZP_OUT_U8 ? 1u : (OUT == ANSZP_OUT_F32 ? 4u : 2u);
    constexpr uint32_t kTableLoads = ((1u << ANSZP_MAX_TABLE_LOG) / 4u + kBlock - 1u) / kBlock;   // 16-byte loads per thread
    constexpr uint32_t kWordLoads = (kPayloadWords / 4u + kBlock - 1u) / kBlock;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & (kWave - 1);
    const uint32_t N = p.n_streams;
    const uint32_t L = 1u << p.table_log;
    const anszp_chunk_t c = p.chunks[blockIdx.x];
    if (!chunk_in_bounds(p, c)) {
        if (tid == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    // Issue every global read that depends only on the descriptor before waiting for any of them:
    // stream headers, the merged half of the layer's table, the chunk's compressed words (from
    // clamped, always valid indices) and the layer's quantizer.
    const uint32_t hdr = (tid < N) ? p.stream_hdr[c.stream_offset + tid] : 0u;
    const uint32_t* src = p.tables + (uint64_t(c.layer_id) << (p.table_log + 1));
    const uint4* tsrc = reinterpret_cast<const uint4*>(src + L);              // merged half, 4 entries per load
    const uint4* wsrc = reinterpret_cast<const uint4*>(p.payload + c.payload_offset);
    const uint32_t quads = min(c.payload_words, kPayloadWords) >> 2;
    const bool wide = L >= 4;                                                 // a 2-state table has no 16-byte rows
    uint4 tv[kTableLoads], wv[kWordLoads];
    {
        const uint32_t t_last = wide ? (L >> 2) - 1u : 0u;
        const uint32_t w_last = quads ? quads - 1u : 0u;
        const uint4* tsafe = wide ? tsrc : reinterpret_cast<const uint4*>(p.tables);
        const uint4* wsafe = quads ? wsrc : tsafe;
#pragma unroll
        for (uint32_t k = 0; k < kTableLoads; ++k) tv[k] = tsafe[min(tid + k * kBlock, t_last)];
#pragma unroll
        for (uint32_t k = 0; k < kWordLoads; ++k) wv[k] = wsafe[min(tid + k * kBlock, w_last)];
    }
    uint32_t tail = 0;
    if (tid < 8 && (quads << 2) + tid < c.payload_words && c.payload_words <= kPayloadWords)
        tail = p.payload[c.payload_offset + (quads << 2) + tid];
    const uint32_t top = src[L - 1];                     // state L-1 carries the dominant symbol if there is one
    const anszp_layer_t lay = p.layers[c.layer_id];
    const uint64_t layer_elem0 = c.out_offset - lay.out_base;
    const uint32_t n = c.n_symbols;
    const bool merged_ok = wide && c.payload_words <= kPayloadWords && ((c.out_offset * kElemBytes) & 15u) == 0 &&
                           n <= (1u << 24) && PER_CHANNEL == (lay.channel_len != 0) &&
                           (!PER_CHANNEL || layer_elem0 + n < (1ull << 32));

    if (!merged_ok) {                                     // whole workgroup agrees
        uint32_t* table = reinterpret_cast<uint32_t*>(lds_table);
        for (uint32_t i = tid; i < L; i += kBlock) table[i] = src[i];
        __syncthreads();
        if (tid >= kWave) return;
        const uint32_t err = decode_chunk_stepwise<OUT>(p, c, lay, table, lane);
        if (err && lane == 0) report(p.status, err);
        return;
    }

    // ---- stage: table (dequantisation folded in), compressed words, ring background
    {
        auto entry = [&](uint32_t m) {
            const uint32_t sym = (m >> 16) & 0xFFu;
            const uint32_t nb = min(m >> 24, uint32_t(ANSZP_MAX_TABLE_LOG));
            const uint32_t code = kFolded ? bf16_rne(dequant(sym, lay.zero_point, lay.scale)) : sym;
            return make_uint2(m & 0x7FF8u, nb | ((m & 7u) << 8) | (m & 0x8000u) | (code << 16));
        };
        uint4* tdst = reinterpret_cast<uint4*>(lds_table);
#pragma unroll
        for (uint32_t k = 0; k < kTableLoads; ++k) {
            const uint32_t i = tid + k * kBlock;
            if (4u * i < L) {
                const uint2 a = entry(tv[k].x), b = entry(tv[k].y), cc = entry(tv[k].z), d = entry(tv[k].w);
                tdst[2u * i] = make_uint4(a.x, a.y, b.x, b.y);
                tdst[2u * i + 1u] = make_uint4(cc.x, cc.y, d.x, d.y);
            }
        }
        uint4* wdst = reinterpret_cast<uint4*>(lds_words);
#pragma unroll
        for (uint32_t k = 0; k < kWordLoads; ++k) {
            const uint32_t i = tid + k * kBlock;
            if (i < quads) wdst[i] = wv[k];
        }
        if (tid < 8) lds_words[(quads << 2) + tid] = tail;      // tail words, then zeros for clamped reads
    }
    const uint32_t bg_sym = top >> 24;
    const uint32_t bg_code = kFolded ? bf16_rne(dequant(bg_sym, lay.zero_point, lay.scale)) : bg_sym;
    const uint32_t bg2 = bg_code | (bg_code << 16);
    {
        uint4* rdst = reinterpret_cast<uint4*>(lds_ring);
#pragma unroll
        for (uint32_t k = 0; k < (kRingBytes / 16u + kBlock - 1u) / kBlock; ++k)
            if (tid + k * kBlock < kRingBytes / 16u) rdst[tid + k * kBlock] = make_uint4(bg2, bg2, bg2, bg2);
    }
    __syncthreads();
    if (tid >= kWave) return;                            // helper wavefronts are done

    // ---- per-lane stream state (lane == tid in wavefront 0)
    const uint32_t n_words = hdr >> 16;
    uint32_t total_words;
    const uint32_t first_word = wave_exclusive_sum(n_words, &total_words);
    uint32_t err = (total_words != c.payload_words) ? ANSZP_ST_BAD_DESC : 0u;
    const uint32_t last_word4 = c.payload_words << 2;    // byte offset of the zero words behind the payload

    const uint32_t n2 = 2u * n, N2 = 2u * N;             // element indices are kept doubled (ring byte offsets)
    constexpr uint32_t kRing2 = 2u * kRingElems, kSlab2 = 2u * kSlab;
    uint32_t X8 = (hdr & (L - 1u)) << 3;                 // byte offset of the current entry
    uint32_t abit = first_word << 5;                     // bit position in the chunk's payload
    uint32_t ne2 = (lane < N) ? 2u * lane : n2;          // 2 * chunk index of this lane's next symbol
    if (ne2 >= n2 && X8 != 0) err |= ANSZP_ST_BAD_STATE; // empty stream must carry state 0

    uint32_t flushed2 = 0;                               // 2 * elements already stored (wave-uniform)
    constexpr uint32_t kBatch = 16;                      // slabs stored per flush
    constexpr uint32_t kBatch2 = kBatch * kSlab2;

    // two consecutive payload words starting at a 4-byte aligned LDS byte offset
    auto word_pair = [&](uint32_t byte_off) {
        const uint32_t* q = reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(lds_words) + byte_off);
        return make_uint2(q[0], q[1]);
    };
    uint8_t* ring8 = reinterpret_cast<uint8_t*>(lds_ring);
    uint2 e = *reinterpret_cast<const uint2*>(lds_table + X8);
    uint2 w = word_pair(min(first_word << 2, last_word4));

    // One look-up for every lane that is neither finished nor too far ahead of the slowest lane
    // for the ring.  Sec. II-A step on a merged entry: state' = newX' | (next stream bits & mask).
    auto step = [&](uint32_t bound) {
        if (ne2 < bound) {
            const uint32_t window = __builtin_amdgcn_alignbit(w.y, w.x, abit);
            const uint32_t eh = e.y, nb = eh & 31u;
            X8 = e.x | (__builtin_amdgcn_ubfe(window, 0u, nb) << 3);
            e = *reinterpret_cast<const uint2*>(lds_table + X8);
            const uint32_t last2 = __umul24((eh >> 8) & 7u, N2) + ne2;   // doubled index of the entry's last symbol
            abit += nb;
            w = word_pair(min((abit >> 3) & ~3u, last_word4));
            // beyond the chunk's end (stream finished inside a run) this hits a ring slot nobody reads
            *reinterpret_cast<uint16_t*>(ring8 + (last2 & (kRing2 - 1u))) = static_cast<uint16_t>(eh >> 16);
            ne2 = last2 + N2;
            if (ne2 >= n2) {                             // stream finished: it must have arrived in state 0
                bool ok = X8 == 0;
                if (last2 >= n2) {                       // ended inside the run of empty steps: no bits were read
                    ok = (last2 - N2 < n2) && (eh & 0x8000u);
                    abit -= nb;
                }
                if (!ok) err |= ANSZP_ST_BAD_STATE;
            }
        }
    };

    // Slabs of the ring are final once every unfinished lane's next symbol lies beyond them.
    auto flush_ready = [&]() {
        if (flushed2 + kBatch2 <= n2 && __ballot(ne2 < flushed2 + kBatch2) == 0) {
            uint4 codes[kBatch];
            uint4* slot = reinterpret_cast<uint4*>(ring8 + ((flushed2 & (kRing2 - 1u)) + lane * 16u));
#pragma unroll
            for (uint32_t k = 0; k < kBatch; ++k) codes[k] = slot[k * (kSlab2 / 16u)];
#pragma unroll
            for (uint32_t k = 0; k < kBatch; ++k) slot[k * (kSlab2 / 16u)] = make_uint4(bg2, bg2, bg2, bg2);
            const uint32_t first = (flushed2 >> 1) + lane * 8u;
#pragma unroll
            for (uint32_t k = 0; k < kBatch; ++k)
                Flusher<OUT, PER_CHANNEL>::store8(p, lay, c.out_offset + first + k * kSlab,
                                                  layer_elem0 + first + k * kSlab, codes[k]);
            flushed2 += kBatch2;
        }
    };

    // Bulk phase: blocks of 8 look-ups with no per-step checks.  A lane joins a block only if even
    // 8 full-length entries keep it inside its stream and inside the ring, so nothing can finish
    // or overrun in the middle of a block.  The block is hand-scheduled because a lone wavefront
    // issues one instruction every 5-8 cycles: what a look-up costs is its instruction count plus
    // the part of the LDS round trip it cannot cover.  At the start of a block a lane loads four
    // payload words (128 bits, at least 97 of them ahead of its bit position: 8 look-ups read at
    // most 96) and shifts them down so that the stream continues at bit 0 of w0.  Per look-up:
    //   X8   = e.lo | (bfe(w0, 0, nb) << 3);  e' = table[X8]        Sec. II-A: newX' + bits, issued first
    //   w0..w3 >>= nb (funnel shift);  sum += e.hi                   low byte of sum = bits read so far
    //   last = ((e.hi >> 8) & 7) * 2N + ne2;  ring[last & mask] = e.hi >> 16;  ne2 = last + 2N
    // Blocks of 8 look-ups run first; when no lane can take one any more (streams within 64
    // symbols of their end), blocks of 4 and then of 2 take over, and only the last few symbols
    // of each stream go through the checked step below.
    {
        uint32_t e_lo = e.x, e_hi = e.y;
#define ANSZP_STEP(EA0, EA1, EB)                                                       \
        "s_waitcnt lgkmcnt(1)\n"                                                       \
        "v_bfe_u32 v52, v44, 0, " EA1 "\n"                                             \
        "v_lshl_or_b32 v52, v52, 3, " EA0 "\n"                                         \
        "ds_read_b64 " EB ", v52 offset:%[table]\n"                                    \
        "v_alignbit_b32 v44, v45, v44, " EA1 "\n"                                      \
        "v_alignbit_b32 v45, v46, v45, " EA1 "\n"                                      \
        "v_alignbit_b32 v46, v47, v46, " EA1 "\n"                                      \
        "v_lshrrev_b32 v47, " EA1 ", v47\n"                                            \
        "v_bfe_u32 v55, " EA1 ", 8, 3\n"                                               \
        "v_add_u32 v57, v57, " EA1 "\n"                                                \
        "v_mad_u32_u24 v55, v55, %[n2s], v50\n"                                        \
        "v_and_b32 v56, %[rmask], v55\n"                                               \
        "v_add_u32 v50, %[n2s], v55\n"                                                 \
        "ds_write_b16_d16_hi v56, " EA1 " offset:%[ring]\n"
#define ANSZP_STEP_AB ANSZP_STEP("v40", "v41", "v[42:43]")
#define ANSZP_STEP_BA ANSZP_STEP("v42", "v43", "v[40:41]")
// BODY = all look-ups of a block but the last, which is written out below: it skips the window
// shift and requests the next block's four words instead.  Blocks have an even number of
// look-ups, so the entry ends up in v[40:41] again.
#define ANSZP_RUN_BLOCKS(STEPS, BODY)                                                                                 \
        while (n2 > (STEPS) * kMaxMerged * N2) {                                                                      \
            const uint32_t limit = min(n2, flushed2 + kRing2) - (STEPS) * kMaxMerged * N2;                            \
            if (__ballot(ne2 < limit) == 0) break;                                                                    \
            const uint32_t flush_at = (flushed2 + kBatch2 <= n2) ? flushed2 + kBatch2 : 0xFFFFFFFFu;                  \
            asm volatile(                                                                                             \
                "v_mov_b32 v40, %[elo]\n v_mov_b32 v41, %[ehi]\n v_mov_b32 v48, %[ab]\n v_mov_b32 v50, %[ne]\n"       \
                "v_cmp_gt_u32 vcc, %[lim], v50\n"                                                                     \
                "s_and_saveexec_b64 s[40:41], vcc\n" /* lanes that can run a whole block */                           \
                "v_lshrrev_b32 v54, 3, v48\n"                                                                         \
                "v_and_b32 v54, 0x1ffffffc, v54\n"                                                                    \
                "v_min_u32 v54, %[lastw], v54\n"                                                                      \
                "ds_read2_b32 v[44:45], v54 offset1:1\n"                                                              \
                "ds_read2_b32 v[46:47], v54 offset0:2 offset1:3\n"                                                    \
                "1:\n"                                                                                                \
                "v_mov_b32 v57, 0\n"                                                                                  \
                "s_waitcnt lgkmcnt(0)\n"                                                                              \
                "v_alignbit_b32 v44, v45, v44, v48\n"                                                                 \
                "v_alignbit_b32 v45, v46, v45, v48\n"                                                                 \
                "v_alignbit_b32 v46, v47, v46, v48\n"                                                                 \
                "v_lshrrev_b32 v47, v48, v47\n"                                                                       \
                BODY                                                                                                  \
                "s_waitcnt lgkmcnt(1)\n"                                                                              \
                "v_bfe_u32 v52, v44, 0, v43\n"                                                                        \
                "v_lshl_or_b32 v52, v52, 3, v42\n"                                                                    \
                "ds_read_b64 v[40:41], v52 offset:%[table]\n"                                                         \
                "v_add_u32 v57, v57, v43\n"                                                                           \
                "v_bfe_u32 v55, v43, 8, 3\n"                                                                          \
                "v_and_b32 v57, 0xff, v57\n"                                                                          \
                "v_mad_u32_u24 v55, v55, %[n2s], v50\n"                                                               \
                "v_add_u32 v48, v48, v57\n" /* bit position after the block */                                        \
                "v_and_b32 v56, %[rmask], v55\n"                                                                      \
                "v_lshrrev_b32 v54, 3, v48\n"                                                                         \
                "v_add_u32 v50, %[n2s], v55\n"                                                                        \
                "v_and_b32 v54, 0x1ffffffc, v54\n"                                                                    \
                "ds_write_b16_d16_hi v56, v43 offset:%[ring]\n"                                                       \
                "v_min_u32 v54, %[lastw], v54\n"                                                                      \
                "v_cmp_gt_u32 s[42:43], %[fat], v50\n" /* lanes of this block still inside the next slabs */          \
                "v_cmp_gt_u32 vcc, %[lim], v50\n"      /* lanes that can run another block */                         \
                "ds_read2_b32 v[44:45], v54 offset1:1\n"                                                              \
                "ds_read2_b32 v[46:47], v54 offset0:2 offset1:3\n"                                                    \
                "s_cmp_eq_u64 s[42:43], 0\n"                                                                          \
                "s_cbranch_scc1 2f\n"                  /* none: slabs may be ready to leave the ring */               \
                "s_and_b64 exec, exec, vcc\n"                                                                         \
                "s_cbranch_scc1 1b\n"                                                                                 \
                "2:\n"                                                                                                \
                "s_mov_b64 exec, s[40:41]\n"                                                                          \
                "s_waitcnt lgkmcnt(0)\n"                                                                              \
                "v_mov_b32 %[elo], v40\n v_mov_b32 %[ehi], v41\n v_mov_b32 %[ab], v48\n v_mov_b32 %[ne], v50\n"       \
                : [elo] "+v"(e_lo), [ehi] "+v"(e_hi), [ab] "+v"(abit), [ne] "+v"(ne2)                                 \
                : [lim] "s"(limit), [fat] "s"(flush_at), [n2s] "s"(N2), [lastw] "s"(last_word4),                      \
                  [table] "n"(kWordsBytes), [ring] "n"(kWordsBytes + kTableBytes), [rmask] "n"(kRing2 - 1u)           \
                : "memory", "vcc", "scc", "s40", "s41", "s42", "s43", "v40", "v41", "v42", "v43", "v44", "v45",       \
                  "v46", "v47", "v48", "v50", "v52", "v54", "v55", "v56", "v57");                                     \
            flush_ready();                                                                                            \
        }
        ANSZP_RUN_BLOCKS(8u, ANSZP_STEP_AB ANSZP_STEP_BA ANSZP_STEP_AB ANSZP_STEP_BA ANSZP_STEP_AB ANSZP_STEP_BA ANSZP_STEP_AB)
        ANSZP_RUN_BLOCKS(4u, ANSZP_STEP_AB ANSZP_STEP_BA ANSZP_STEP_AB)
        ANSZP_RUN_BLOCKS(2u, ANSZP_STEP_AB)
#undef ANSZP_RUN_BLOCKS
#undef ANSZP_STEP_AB
#undef ANSZP_STEP_BA
#undef ANSZP_STEP
        e = make_uint2(e_lo, e_hi);
        w = word_pair(min((abit >> 3) & ~3u, last_word4));
    }

    // Careful phase: every look-up checks the end of the stream and the room in the ring.
    for (;;) {
        if (__ballot(ne2 < n2) == 0) break;
        const uint32_t bound = min(n2, flushed2 + kRing2 - kMaxMerged * N2 + 1u);
        step(bound);
        step(bound);
        step(bound);
        step(bound);
        flush_ready();
    }
    // every stream is finished: the rest of the ring is final
    uint32_t flushed = flushed2 >> 1;
    while (flushed + kSlab <= n) {
        const uint4 codes = *reinterpret_cast<const uint4*>(lds_ring + ((flushed & (kRingElems - 1u)) + lane * 8u));
        Flusher<OUT, PER_CHANNEL>::store8(p, lay, c.out_offset + flushed + lane * 8u, layer_elem0 + flushed + lane * 8u, codes);
        flushed += kSlab;
    }
    for (uint32_t j = flushed + lane; j < n; j += kWave)
        Flusher<OUT, PER_CHANNEL>::store1(p, lay, c.out_offset + j, layer_elem0 + j, lds_ring[j & (kRingElems - 1u)]);

    if (lane < N) {
        const uint32_t bits_read = abit - (first_word << 5);
        if (((bits_read + 31u) >> 5) != n_words) err |= ANSZP_ST_BAD_LENGTH;
    }
    err = wave_or(err);
    if (err && lane == 0) report(p.status, err);
}

// ---------------------------------------------------------------------------------------------
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

template <int OUT>
void launch_decode(const DecodeParams& p, uint32_t n_chunks, bool per_channel, bool stepwise, hipStream_t s) {
    if (stepwise) hipLaunchKernelGGL(decode_stepwise<OUT>, dim3(n_chunks), dim3(kWave), 0, s, p);
    else if (per_channel) hipLaunchKernelGGL((decode_merged<OUT, true>), dim3(n_chunks), dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL((decode_merged<OUT, false>), dim3(n_chunks), dim3(kBlock), 0, s, p);
}

int decode_impl(const anszp_decode_args_t* a, int mode, void* hip_stream) {
    if (!a) return ANSZP_E_NULL;
    if (a->n_chunks == 0) return ANSZP_OK;
    if (!a->tables || !a->chunks || !a->stream_hdr || !a->layers || !a->out || !a->status) return ANSZP_E_NULL;
    if (!a->payload && a->payload_words) return ANSZP_E_NULL;
    if (a->table_log < 1 || a->table_log > ANSZP_MAX_TABLE_LOG || a->n_streams < 1 ||
        a->n_streams > ANSZP_MAX_STREAMS || a->out_dtype > ANSZP_OUT_BF16 || a->n_tables == 0 ||
        a->n_chunks >= (1ull << 31) || (reinterpret_cast<uintptr_t>(a->payload) & 15) ||
        (reinterpret_cast<uintptr_t>(a->tables) & 15) ||
        (reinterpret_cast<uintptr_t>(a->out) & 15) || mode < 0 || mode > 2)
        return ANSZP_E_RANGE;
    DecodeParams p;
    p.tables = a->tables; p.chunks = a->chunks; p.stream_hdr = a->stream_hdr; p.payload = a->payload;
    p.layers = a->layers; p.scales = a->scales; p.out = a->out; p.status = a->status;
    p.n_stream_hdr = a->n_stream_hdr; p.payload_words = a->payload_words;
    p.n_scales = a->scales ? a->n_scales : 0; p.out_elems = a->out_elems;
    p.n_tables = a->n_tables; p.table_log = a->table_log; p.n_streams = a->n_streams;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint32_t nc = static_cast<uint32_t>(a->n_chunks);
    // chunks whose compressed words cannot fit the merged kernel's LDS window would all take its
    // fallback; launch the light step-wise kernel (many more wavefronts per CU) for them instead
    const bool stepwise = mode == 1 || (mode == 0 && a->payload_words / a->n_chunks > kPayloadWords);
    const bool per_channel = a->scales != nullptr && a->n_scales != 0;
    switch (a->out_dtype) {
        case ANSZP_OUT_U8: launch_decode<ANSZP_OUT_U8>(p, nc, per_channel, stepwise, s); break;
        case ANSZP_OUT_F32: launch_decode<ANSZP_OUT_F32>(p, nc, per_channel, stepwise, s); break;
        default: launch_decode<ANSZP_OUT_BF16>(p, nc, per_channel, stepwise, s); break;
    }
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}

}  // namespace

extern "C" {

int anszp_build_tables(const uint32_t* freqs_host, int n_tables, int table_log,
                       uint32_t* tables_dev, void* hip_stream) {
    if (!freqs_host || !tables_dev) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_tables < 1) return ANSZP_E_RANGE;
    if (reinterpret_cast<uintptr_t>(tables_dev) & 15) return ANSZP_E_RANGE;
    const size_t entries = size_t(n_tables) << (table_log + 1);
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

int anszp_decode(const anszp_decode_args_t* args, void* hip_stream) { return decode_impl(args, 0, hip_stream); }

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
