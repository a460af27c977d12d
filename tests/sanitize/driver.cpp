// Host-side checks meant to run under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU oracle
// (oracle/ans_oracle.c) and the library's host code (csrc/anszp_host.cpp) linked into one program and
// driven through round trips, packer-equals-oracle comparisons, corrupted containers and bad arguments.
// Prints "ok <cases>" and returns 0; any sanitizer report ends the run with a non-zero status.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "anszp.h"

extern "C" {
int orc_normalize(const uint64_t* counts, int R, uint32_t* f);
int orc_build_decode_table(const uint32_t* f, int R, uint8_t* tsym, uint8_t* tnb, uint16_t* tnewX);
int64_t orc_encode_layer(const uint8_t* sym, uint64_t n, const uint32_t* f, int R, uint32_t N, uint32_t chunk_size,
                         uint32_t* chunk_nsym, uint64_t* chunk_payload_off, uint32_t* chunk_payload_words, uint32_t* stream_hdr,
                         uint32_t* payload, uint64_t cap_words);
int orc_decode_chunks(uint64_t c_begin, uint64_t c_end, const uint32_t* chunk_layer, const uint32_t* chunk_nsym,
                      const uint64_t* chunk_out_off, const uint64_t* chunk_payload_off, const uint32_t* chunk_stream_off,
                      const uint32_t* stream_hdr, const uint32_t* payload, uint64_t payload_words, int R, uint32_t N,
                      const uint8_t* tsym, const uint8_t* tnb, const uint16_t* tnewX, uint8_t* out_sym);
}

static uint64_t rng_state = 0x2406062370ull;
static uint64_t rnd() {                                   // SplitMix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); std::exit(1); } } while (0)

struct Case { int R; uint32_t N, chunk; uint64_t n; int bits; double p0; };

static int run_case(const Case& k) {
    const uint32_t L = 1u << k.R, A = 1u << k.bits, z = A / 2;
    std::vector<uint8_t> sym(k.n);
    sym.reserve(k.n + 1);                                  // (an empty layer still has an address to pass)
    for (auto& s : sym) {                                  // peaked at z, geometric tails
        if ((rnd() >> 11) * (1.0 / 9007199254740992.0) < k.p0) { s = uint8_t(z); continue; }
        int d = 1;
        while (d < int(A) && (rnd() & 1)) ++d;
        const int v = (rnd() & 1) ? int(z) + d : int(z) - d;
        s = uint8_t(v < 0 ? 0 : v >= int(A) ? int(A) - 1 : v);
    }
    uint64_t counts[256] = {0};
    for (auto s : sym) counts[s]++;
    uint32_t f_orc[256], f_lib[256];
    if (k.n == 0) counts[z] = 1;
    CHECK(orc_normalize(counts, k.R, f_orc) == 0);
    CHECK(anszp_normalize_freqs(counts, k.R, f_lib) == ANSZP_OK);
    CHECK(std::memcmp(f_orc, f_lib, sizeof f_orc) == 0);
    // tables: the library's triples are the oracle's
    std::vector<uint8_t> tsym(L), tnb(L);
    std::vector<uint16_t> tnewX(L);
    CHECK(orc_build_decode_table(f_orc, k.R, tsym.data(), tnb.data(), tnewX.data()) == 0);
    std::vector<uint32_t> table(size_t(ANSZP_TABLE_WORDS_PER_STATE) * L);
    CHECK(anszp_build_tables_host(f_lib, 1, k.R, table.data()) == ANSZP_OK);
    for (uint32_t X = 0; X < L; ++X) {
        const uint32_t w = table[2 * L + X];
        CHECK((w & 0xFFFF) == tnewX[X] && ((w >> 16) & 0xFF) == tnb[X] && (w >> 24) == tsym[X]);
    }
    // the library's packer writes the oracle's container
    uint64_t n_chunks = 0, cap = 0;
    CHECK(anszp_pack_bound(k.n, k.R, int(k.N), k.chunk, &n_chunks, &cap) == ANSZP_OK);
    CHECK(n_chunks == (k.n + k.chunk - 1) / k.chunk);
    std::vector<anszp_chunk_t> chunks(n_chunks + 1);
    std::vector<uint32_t> hdr(n_chunks * k.N + 1), payload(cap + 4);
    uint64_t used = 0;
    CHECK(anszp_pack_layer(sym.data(), k.n, f_lib, k.R, int(k.N), k.chunk, 0, 0, 0, 0, chunks.data(), hdr.data(), payload.data(),
                           payload.size(), &used) == ANSZP_OK);
    std::vector<uint32_t> o_nsym(n_chunks + 1), o_pw(n_chunks + 1), o_hdr(n_chunks * k.N + 1), o_payload(cap + 8);
    std::vector<uint64_t> o_off(n_chunks + 1);
    const int64_t o_used = orc_encode_layer(sym.data(), k.n, f_orc, k.R, k.N, k.chunk, o_nsym.data(), o_off.data(), o_pw.data(),
                                            o_hdr.data(), o_payload.data(), o_payload.size());
    CHECK(o_used >= 0 && uint64_t(o_used) == used);
    CHECK(std::memcmp(o_payload.data(), payload.data(), used * 4) == 0);
    CHECK(std::memcmp(o_hdr.data(), hdr.data(), n_chunks * k.N * 4) == 0);
    std::vector<uint32_t> c_layer(n_chunks + 1, 0), c_stream(n_chunks + 1);
    std::vector<uint64_t> c_out(n_chunks + 1);
    for (uint64_t c = 0; c < n_chunks; ++c) {
        CHECK(chunks[c].n_symbols == o_nsym[c] && chunks[c].payload_offset == o_off[c] && chunks[c].payload_words == o_pw[c]);
        CHECK(chunks[c].out_offset == c * uint64_t(k.chunk) && chunks[c].stream_offset == c * k.N && chunks[c].layer_id == 0);
        c_stream[c] = chunks[c].stream_offset; c_out[c] = chunks[c].out_offset;
    }
    // round trip through the oracle's decoder
    std::vector<uint8_t> out(k.n + 1, 0xEE);
    CHECK(orc_decode_chunks(0, n_chunks, c_layer.data(), o_nsym.data(), c_out.data(), o_off.data(), c_stream.data(), hdr.data(),
                            payload.data(), used, k.R, k.N, tsym.data(), tnb.data(), tnewX.data(), out.data()) == 0);
    CHECK(std::memcmp(out.data(), sym.data(), k.n) == 0 && out[k.n] == 0xEE);
    // corrupted containers: the decoder must answer with an error code or wrong symbols, never touch memory it was not given
    int flagged = 0;
    for (int t = 0; t < 24 && used > 0; ++t) {
        std::vector<uint32_t> bad_payload(payload.begin(), payload.begin() + used), bad_hdr(hdr.begin(), hdr.begin() + n_chunks * k.N);
        switch (t % 4) {
            case 0: bad_payload[rnd() % used] ^= 1u << (rnd() % 32); break;
            case 1: bad_hdr[rnd() % bad_hdr.size()] ^= 1u << (rnd() % 12); break;                       // initial state
            case 2: bad_hdr[rnd() % bad_hdr.size()] += 0x10000u * uint32_t(1 + rnd() % 7); break;        // stream longer than it is
            default: bad_hdr[rnd() % bad_hdr.size()] = uint32_t(rnd()); break;
        }
        std::vector<uint8_t> o2(k.n + 1, 0xEE);
        const int rc = orc_decode_chunks(0, n_chunks, c_layer.data(), o_nsym.data(), c_out.data(), o_off.data(), c_stream.data(),
                                         bad_hdr.data(), bad_payload.data(), bad_payload.size(), k.R, k.N, tsym.data(), tnb.data(), tnewX.data(), o2.data());
        CHECK(o2[k.n] == 0xEE);
        flagged += rc != 0;
    }
    return flagged;
}

int main() {
    const Case cases[] = {
        {10, 1, 65536, 36864, 4, 0.45}, {11, 32, 16384, 50000, 5, 0.6}, {12, 64, 65536, 150000, 8, 0.76}, {12, 64, 65536, 65536, 1, 0.9},
        {6, 64, 2048, 5000, 3, 0.7}, {8, 48, 1000, 70001, 4, 0.8}, {2, 3, 7, 100, 1, 0.5}, {1, 64, 64, 1000, 1, 1.0}, {12, 64, 4096, 0, 4, 0.8},
        {9, 5, 333, 12345, 6, 0.3}, {12, 64, 262144, 300000, 4, 0.25},
    };
    int flagged = 0, n = 0;
    for (const Case& k : cases) { flagged += run_case(k); ++n; }
    CHECK(flagged > 0);
    // bad arguments to the library's host entry points
    uint32_t f[256] = {0}, t[8 * 4];
    uint64_t counts[256] = {0}, a = 0, b = 0;
    CHECK(anszp_normalize_freqs(nullptr, 4, f) != ANSZP_OK && anszp_normalize_freqs(counts, 4, f) != ANSZP_OK);
    CHECK(anszp_normalize_freqs(counts, 0, f) != ANSZP_OK && anszp_normalize_freqs(counts, 13, f) != ANSZP_OK);
    CHECK(anszp_build_tables_host(f, 1, 2, t) != ANSZP_OK);                 // frequencies that do not sum to 4
    f[7] = 3; f[9] = 1;
    CHECK(anszp_build_tables_host(f, 1, 2, t) == ANSZP_OK && anszp_build_tables_host(f, 0, 2, t) != ANSZP_OK);
    CHECK(anszp_pack_bound(10, 2, 0, 4, &a, &b) != ANSZP_OK && anszp_pack_bound(10, 2, 65, 4, &a, &b) != ANSZP_OK);
    const uint8_t sym[4] = {7, 7, 9, 8};                                   // 8 has no frequency
    anszp_chunk_t ch[2];
    uint32_t hd[8], pl[16];
    CHECK(anszp_pack_layer(sym, 4, f, 2, 2, 4, 0, 0, 0, 0, ch, hd, pl, 16, &a) != ANSZP_OK);
    CHECK(anszp_pack_layer(sym, 3, f, 2, 2, 4, 0, 0, 0, 0, ch, hd, pl, 0, &a) != ANSZP_OK);    // no room
    CHECK(std::strlen(anszp_strerror(-3)) > 0 && std::strlen(anszp_strerror(12345)) > 0);
    std::printf("ok %d\n", n);
    return 0;
}
