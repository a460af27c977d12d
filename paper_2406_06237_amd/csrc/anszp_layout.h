// Layout of one decode table in memory, shared by the host builder, the device builder and the
// kernels (internal to the library; the public description is in anszp.h).
//
// A table of L = 2^table_log states occupies 8 L words:
//   words [0, L)     the byte table of Sec. II-A when L <= 256: 3 L bytes (symbol, nb_bits, newX of
//                    state X at bytes 3X, 3X+1, 3X+2), the rest zero; all zero for larger tables
//   words [L, 2L)    zero
//   words [2L, 3L)   the triple of state X as one word: newX | nb_bits << 16 | symbol << 24
//   words [3L, 4L)   zero
//   words [4L, 8L)   2 L look-ahead entries of two words, entry 2X + b for state X and next stream bit b
#ifndef ANSZP_LAYOUT_H
#define ANSZP_LAYOUT_H

#include <stdint.h>

#if defined(__HIPCC__)
#define ANSZP_HD __host__ __device__ inline
#else
#define ANSZP_HD inline
#endif

constexpr uint32_t kLookaheadMaxSymbols = 8;     // symbols one look-ahead entry can stand for

ANSZP_HD uint64_t table_stride_words(uint32_t table_log) { return uint64_t(8) << table_log; }
ANSZP_HD uint32_t table_bytes_offset(uint32_t) { return 0u; }
ANSZP_HD uint32_t table_triples_offset(uint32_t table_log) { return 2u << table_log; }
ANSZP_HD uint32_t table_lookahead_offset(uint32_t table_log) { return 4u << table_log; }

// Look-ahead entry, first word.  The lower half is what the decoding wavefront shifts by and adds up over a
// block of 16 look-ups (no field's sum reaches the next field); the upper half is what it logs:
//   bits 0..4   31 - T, T <= 12 the stream bits the entry consumes     bits 5..8   zero
//   bits 9..11  c - 1, c <= 8 the symbols the entry stands for         bits 12..15 zero
//   bits 16..23 the entry's last symbol (the c - 1 before it are the dominant symbol)
//   bits 24..27 T      bits 28..30 c - 1      bit 31  set for the entries of state 0
// second word: 8 * base as a signed number; the next entry is number base + v, v the next T + 1
// stream bits read most significant first (the last of them is the new peeked bit).
ANSZP_HD uint32_t lookahead_first_word(uint32_t T, uint32_t count, uint32_t symbol, bool state_zero) {
    return (31u - T) | ((count - 1u) << 9) | (symbol << 16) | (T << 24) | ((count - 1u) << 28) | (state_zero ? 1u << 31 : 0u);
}
ANSZP_HD uint32_t lookahead_second_word(int32_t base) { return static_cast<uint32_t>(base * 8); }

#endif
