// Host side of libanszp: frequency normalisation, decode-table construction and the
// offline compressor.  No HIP calls here, so these entry points work on a machine
// without a GPU.
//
// Paper sections followed: Sec. II-A (automaton, look-up table entry = symbol, nb_bits,
// newX; rate depends on how symbols are spread over states), Sec. III-A (one table per
// layer), Sec. III-B (parallel streams sharing one table).
#include "anszp.h"
#include "anszp_layout.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <queue>
#include <vector>

namespace {

bool freqs_ok(const uint32_t* f, int table_log) {
    uint64_t total = 0;
    for (int s = 0; s < ANSZP_ALPHABET; ++s) total += f[s];
    return total == (1ull << table_log);
}

// The spread of symbols over states is this library's choice (Sec. II-A says that the rate depends on
// how the states are initialised, not how to do it): occurrence i of a symbol with frequency f is given
// the position (2i+1)/(2f); states follow that fraction, ties by symbol.  Kept as
// numerator/denominator and compared by cross product.
struct Slot {
    uint64_t num;   // 2i+1
    uint64_t den;   // f (the common factor 2 cancels)
    uint32_t sym;
};
struct SlotLater {
    bool operator()(const Slot& a, const Slot& b) const {
        const uint64_t l = a.num * b.den, r = b.num * a.den;
        if (l != r) return l > r;
        return a.sym > b.sym;
    }
};

// The "initialization of the states" Sec. II-A leaves open: merge the per-symbol position sequences.
void spread_states(const uint32_t* f, int table_log, std::vector<uint8_t>& state_sym) {
    const uint32_t L = 1u << table_log;
    state_sym.resize(L);
    std::priority_queue<Slot, std::vector<Slot>, SlotLater> heap;
    for (uint32_t s = 0; s < ANSZP_ALPHABET; ++s)
        if (f[s]) heap.push(Slot{1, f[s], s});
    for (uint32_t X = 0; X < L; ++X) {
        Slot top = heap.top();
        heap.pop();
        state_sym[X] = static_cast<uint8_t>(top.sym);
        top.num += 2;
        if (top.num < 2ull * top.den) heap.push(top);
    }
}

struct StepTable {
    std::vector<uint8_t> sym, nb;
    std::vector<uint16_t> newX;
};

// Sec. II-A table: the j-th state (in increasing X) of symbol s has sub-state f_s + j; it is
// shifted left until it lies in [L, 2L).
void build_step_table(const uint32_t* f, int table_log, StepTable& t) {
    const uint32_t L = 1u << table_log;
    spread_states(f, table_log, t.sym);
    t.nb.assign(L, 0);
    t.newX.assign(L, 0);
    uint32_t sub[ANSZP_ALPHABET];
    for (int s = 0; s < ANSZP_ALPHABET; ++s) sub[s] = f[s];
    for (uint32_t X = 0; X < L; ++X) {
        uint32_t v = sub[t.sym[X]]++;
        uint32_t shift = 0;
        while (v < L) { v <<= 1; ++shift; }
        t.nb[X] = static_cast<uint8_t>(shift);
        t.newX[X] = static_cast<uint16_t>(v - L);
    }
}

// One table (layout: anszp_layout.h): the byte table of Sec. II-A for L <= 256, the paper's triple
// per state, and the look-ahead entries indexed by 2X + b (b = the next stream bit, peeked, not yet
// consumed).
//
// A look-ahead entry is the same automaton with up to kLookaheadMaxSymbols steps merged into one
// look-up: starting in state X with next bit b it emits c-1 copies of the dominant symbol (the
// symbol with f > L/2: empty-label transitions, and at most one of its 1-bit transitions, which
// consumes b) and then one more symbol, having consumed T <= 12 stream bits in all.  With v = the
// next T+1 stream bits read most significant first (so v ends in the new peeked bit), the next
// index is base + v.  A run never passes through state 0: the step that arrives there is the
// entry's last.  Every stream ends in state 0, so a stream always ends where an entry ends.
void build_one_table(const uint32_t* f, int table_log, uint32_t* out) {
    const uint32_t L = 1u << table_log;
    StepTable t;
    build_step_table(f, table_log, t);
    int dominant = -1;
    for (int s = 0; s < ANSZP_ALPHABET; ++s)
        if (f[s] > L / 2) dominant = s;
    std::memset(out, 0, size_t(table_stride_words(table_log)) * sizeof(uint32_t));
    uint32_t* triples = out + table_triples_offset(table_log);
    uint32_t* ahead = out + table_lookahead_offset(table_log);
    if (L <= 256) {                                       // Sec. II-A: three bytes per state
        uint8_t* bytes = reinterpret_cast<uint8_t*>(out + table_bytes_offset(table_log));
        for (uint32_t X = 0; X < L; ++X) {
            bytes[3 * X] = t.sym[X];
            bytes[3 * X + 1] = t.nb[X];
            bytes[3 * X + 2] = static_cast<uint8_t>(t.newX[X]);
        }
    }
    for (uint32_t X = 0; X < L; ++X) {
        triples[X] = uint32_t(t.newX[X]) | (uint32_t(t.nb[X]) << 16) | (uint32_t(t.sym[X]) << 24);
        for (uint32_t b = 0; b < 2; ++b) {
            uint32_t Y = X, count = 0, bits = 0;
            bool took_b = false, may_take_b = true;
            uint32_t saved_Y = 0, saved_count = 0;
            int32_t base = 0;
            uint32_t last_sym = 0;
            for (;;) {
                const uint32_t n = t.nb[Y];
                const bool room = count + 1 < kLookaheadMaxSymbols;   // another symbol may follow this one
                const bool is_dominant = int(t.sym[Y]) == dominant;
                // a step of the dominant symbol whose bits are known (none, or the peeked one) joins the
                // run unless it arrives in state 0
                if (is_dominant && room && n == 0 && t.newX[Y] != 0) { ++count; Y = t.newX[Y]; continue; }
                if (is_dominant && room && n == 1 && !took_b && may_take_b && (t.newX[Y] | b) != 0) {
                    saved_Y = Y; saved_count = count;
                    took_b = true; ++count; Y = t.newX[Y] | b;
                    continue;
                }
                if (took_b && 1 + n > uint32_t(ANSZP_MAX_TABLE_LOG)) {   // too many bits for one look-up: the 1-bit step is the last
                    Y = saved_Y; count = saved_count; took_b = false; may_take_b = false;
                    continue;
                }
                // the entry's last symbol: its n bits are read into the next index
                bits = (took_b ? 1 : 0) + n;
                base = int32_t(2 * t.newX[Y]) - (took_b ? int32_t(b << (n + 1)) : 0);
                last_sym = t.sym[Y];
                ++count;
                break;
            }
            ahead[2 * (2 * X + b)] = lookahead_first_word(bits, count, last_sym, X == 0);
            ahead[2 * (2 * X + b) + 1] = lookahead_second_word(base);
        }
    }
}

// The low `n` bits of v in reverse order (n <= 16).
uint32_t reversed_bits(uint32_t v, uint32_t n) {
    uint32_t r = 0;
    for (uint32_t i = 0; i < n; ++i) r |= ((v >> i) & 1u) << (n - 1 - i);
    return r;
}

// Writes bit groups from the end of a scratch bit array towards its start (encoding runs over
// the symbols backwards, the decoder reads forwards).
class BackwardBits {
public:
    explicit BackwardBits(uint64_t max_bits) : words_((max_bits + 63) / 64 + 1, 0), pos_(words_.size() * 64) {}
    void put(uint32_t value, uint32_t nbits) {
        if (!nbits) return;
        pos_ -= nbits;
        const uint64_t w = pos_ >> 6, sh = pos_ & 63;
        words_[w] |= uint64_t(value) << sh;
        if (sh + nbits > 64) words_[w + 1] |= uint64_t(value) >> (64 - sh);
    }
    uint64_t bit_count() const { return words_.size() * 64 - pos_; }
    // copy the written bits, first written-last, to 32-bit words starting at bit 0
    void extract(uint32_t* dst, uint64_t n_words32) const {
        const uint64_t total = bit_count();
        for (uint64_t i = 0; i < n_words32; ++i) {
            const uint64_t b = pos_ + 32 * i;
            const uint64_t w = b >> 6, sh = b & 63;
            uint64_t v = words_[w] >> sh;
            if (sh > 32 && w + 1 < words_.size()) v |= words_[w + 1] << (64 - sh);
            uint32_t out = static_cast<uint32_t>(v);
            const uint64_t left = total - 32 * i;
            if (left < 32) out &= (1u << left) - 1u;
            dst[i] = out;
        }
    }
private:
    std::vector<uint64_t> words_;
    uint64_t pos_;
};

struct Encoder {
    uint32_t L;
    uint32_t f[ANSZP_ALPHABET];
    uint32_t first[ANSZP_ALPHABET];        // index of symbol s's first state in `states`
    std::vector<uint16_t> states;          // states of each symbol in increasing X
    void init(const uint32_t* freqs, int table_log) {
        L = 1u << table_log;
        std::vector<uint8_t> state_sym;
        spread_states(freqs, table_log, state_sym);
        uint32_t acc = 0;
        for (int s = 0; s < ANSZP_ALPHABET; ++s) { f[s] = freqs[s]; first[s] = acc; acc += freqs[s]; }
        states.resize(L);
        uint32_t fill[ANSZP_ALPHABET];
        std::memcpy(fill, first, sizeof(fill));
        for (uint32_t X = 0; X < L; ++X) states[fill[state_sym[X]]++] = static_cast<uint16_t>(X);
    }
};

}  // namespace

extern "C" {

int anszp_version(void) { return 100; }

const char* anszp_strerror(int code) {
    switch (code) {
        case ANSZP_OK: return "ok";
        case ANSZP_E_NULL: return "required pointer is NULL";
        case ANSZP_E_RANGE: return "argument out of range";
        case ANSZP_E_FREQ: return "frequencies do not sum to 2^table_log (or cannot be normalised)";
        case ANSZP_E_SYMBOL: return "symbol with zero frequency in the data";
        case ANSZP_E_SPACE: return "output buffer too small or stream longer than 65535 words";
        case ANSZP_E_HIP: return "HIP runtime error";
        case ANSZP_E_NOMEM: return "host allocation failed";
        default: return "unknown error code";
    }
}

int anszp_normalize_freqs(const uint64_t* counts, int table_log, uint32_t* freqs) {
    if (!counts || !freqs) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG) return ANSZP_E_RANGE;
    const uint64_t L = 1ull << table_log;
    unsigned __int128 total = 0;
    uint32_t distinct = 0;
    for (int s = 0; s < ANSZP_ALPHABET; ++s) { total += counts[s]; distinct += counts[s] != 0; }
    if (total == 0 || distinct > L) return ANSZP_E_FREQ;
    int64_t assigned = 0;
    for (int s = 0; s < ANSZP_ALPHABET; ++s) {
        uint64_t share = static_cast<uint64_t>((static_cast<unsigned __int128>(counts[s]) * L) / total);
        if (counts[s] && share == 0) share = 1;
        freqs[s] = static_cast<uint32_t>(share);
        assigned += static_cast<int64_t>(share);
    }
    // the remainder goes, unit by unit, to (or comes from) whichever symbol is largest then
    for (int64_t rest = static_cast<int64_t>(L) - assigned; rest != 0;) {
        uint32_t* top = std::max_element(freqs, freqs + ANSZP_ALPHABET);   // first maximum
        if (rest > 0) { ++*top; --rest; }
        else { if (*top <= 1) return ANSZP_E_FREQ; --*top; ++rest; }
    }
    return ANSZP_OK;
}

int anszp_build_tables_host(const uint32_t* freqs, int n_tables, int table_log, uint32_t* tables) {
    if (!freqs || !tables) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_tables < 1) return ANSZP_E_RANGE;
    for (int t = 0; t < n_tables; ++t)
        if (!freqs_ok(freqs + size_t(t) * ANSZP_ALPHABET, table_log)) return ANSZP_E_FREQ;
    try {
        for (int t = 0; t < n_tables; ++t)
            build_one_table(freqs + size_t(t) * ANSZP_ALPHABET, table_log, tables + size_t(t) * table_stride_words(table_log));
    } catch (const std::bad_alloc&) {
        return ANSZP_E_NOMEM;
    }
    return ANSZP_OK;
}

int anszp_pack_bound(uint64_t n_symbols, int table_log, int n_streams, uint32_t chunk_size,
                     uint64_t* n_chunks, uint64_t* payload_words) {
    if (!n_chunks || !payload_words) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_streams < 1 || n_streams > ANSZP_MAX_STREAMS ||
        chunk_size < 1)
        return ANSZP_E_RANGE;
    const uint64_t nc = (n_symbols + chunk_size - 1) / chunk_size;
    *n_chunks = nc;
    // at most table_log bits per symbol, one partial word per stream, three pad words per chunk
    *payload_words = (n_symbols * uint64_t(table_log) + 31) / 32 + nc * (uint64_t(n_streams) + 3);
    return ANSZP_OK;
}

int anszp_pack_layer(const uint8_t* symbols, uint64_t n_symbols, const uint32_t* freqs,
                     int table_log, int n_streams, uint32_t chunk_size,
                     uint32_t layer_id, uint64_t out_offset, uint64_t payload_word_offset,
                     uint32_t stream_offset,
                     anszp_chunk_t* chunks_out, uint32_t* stream_hdr_out,
                     uint32_t* payload_out, uint64_t payload_cap_words, uint64_t* payload_words_used) {
    if (!freqs || !payload_words_used || (n_symbols && (!symbols || !chunks_out || !stream_hdr_out)))
        return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_streams < 1 || n_streams > ANSZP_MAX_STREAMS ||
        chunk_size < 1 || (payload_word_offset & 3))
        return ANSZP_E_RANGE;
    if (!freqs_ok(freqs, table_log)) return ANSZP_E_FREQ;
    if (!payload_out && payload_cap_words) return ANSZP_E_NULL;
    try {
        Encoder enc;
        enc.init(freqs, table_log);
        const uint32_t N = static_cast<uint32_t>(n_streams);
        const uint64_t n_chunks = (n_symbols + chunk_size - 1) / chunk_size;
        uint64_t cursor = 0;                                   // words written so far
        for (uint64_t c = 0; c < n_chunks; ++c) {
            const uint64_t begin = c * uint64_t(chunk_size);
            const uint32_t cn = static_cast<uint32_t>(std::min<uint64_t>(chunk_size, n_symbols - begin));
            anszp_chunk_t& d = chunks_out[c];
            d.layer_id = layer_id;
            d.n_symbols = cn;
            d.out_offset = out_offset + begin;
            d.payload_offset = payload_word_offset + cursor;
            d.stream_offset = stream_offset + static_cast<uint32_t>(c) * N;
            uint32_t chunk_words = 0;
            for (uint32_t k = 0; k < N; ++k) {
                const uint32_t len = cn > k ? (cn - k + N - 1) / N : 0;
                BackwardBits bits(uint64_t(len) * table_log);
                uint32_t x = enc.L;                            // every stream starts in X = 0
                for (uint32_t i = len; i-- > 0;) {
                    const uint32_t s = symbols[begin + k + uint64_t(i) * N];
                    const uint32_t fs = enc.f[s];
                    if (!fs) return ANSZP_E_SYMBOL;
                    uint32_t drop = 0;
                    while ((x >> drop) >= 2 * fs) ++drop;      // bring x into [f_s, 2 f_s)
                    bits.put(reversed_bits(x & ((1u << drop) - 1u), drop), drop);   // first bit read = top bit
                    x = enc.L + enc.states[enc.first[s] + (x >> drop) - fs];
                }
                const uint64_t nw = (bits.bit_count() + 31) / 32;
                if (nw > 0xFFFF || cursor + nw > payload_cap_words) return ANSZP_E_SPACE;
                bits.extract(payload_out + cursor, nw);
                stream_hdr_out[c * N + k] = (x - enc.L) | (static_cast<uint32_t>(nw) << 16);
                cursor += nw;
                chunk_words += static_cast<uint32_t>(nw);
            }
            d.payload_words = chunk_words;
            while (cursor & 3) {
                if (cursor >= payload_cap_words) return ANSZP_E_SPACE;
                payload_out[cursor++] = 0;
            }
        }
        *payload_words_used = cursor;
    } catch (const std::bad_alloc&) {
        return ANSZP_E_NOMEM;
    }
    return ANSZP_OK;
}

}  // extern "C"
