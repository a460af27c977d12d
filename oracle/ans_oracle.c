/*
 * ans_oracle.c -- plain, slow, obviously-correct CPU codec for zero-point-quantized
 * network weights entropy-coded with tabled ANS (tANS).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is checked
 * against.  It shares no code, header, table generator or constant with the HIP
 * library; only tests, the smoke check and the benchmark's CPU-baseline leg may
 * call it.  Nothing here is tuned for speed.
 *
 * What it follows (paper sections, in the paper's notation):
 *   - Sec. II-A: tANS is a finite automaton with l states; the decoder is a
 *     look-up table whose entry for a state holds (symbol, nb_bits, newX); one
 *     decode step emits the symbol, reads nb_bits bits from the stream and moves
 *     to state newX + bits.  Some transitions read zero bits, which is what lets
 *     the code go below one bit per symbol.
 *   - Sec. II-A, Eq. 1: the rate depends on how symbols are spread over the
 *     states and approaches the entropy as l grows.
 *   - Sec. III-B: parallel decoding keeps a vector of states, one per stream, all
 *     streams sharing one table; a stream of n weights costs n look-ups and n
 *     small additions.
 *   - Sec. II-B: weights come from a uniform quantizer with a zero-point, so
 *     dequantisation is w = scale * (q - z).
 *   - Sec. III-A: one coder (one table) per layer.
 *
 * The paper fixes none of: frequency normalisation, the spread, bit order,
 * stream split, container layout.  The readings taken are written next to the
 * function that implements each of them.
 *
 * PARITY PINS (tests/test_oracle_*.py): prefix-interval tiling of every table,
 * brute-force enumeration on 2-4 symbol alphabets, dyadic sources coding to
 * exactly -log2 p bits, size against the Shannon/cross-entropy bound, the
 * table-size trend the paper prints (Sec. III-B, Table 3 discussion), the
 * 3*l-byte table of Sec. II-A, and IEEE-754 dequantisation against fp64.
 * The spread itself cannot be pinned to the paper (its Fig. 1 automaton is not
 * available as numbers): "parity unpinned" against the paper for the choice of
 * spread, pinned only through the invariants above.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <pthread.h>

#define ORC_ALPHABET 256
#define ORC_MAX_R 16

/* error codes (negative) */
#define ORC_E_ARG      (-1)
#define ORC_E_FREQ     (-2)   /* frequencies do not describe a valid table */
#define ORC_E_SYMBOL   (-3)   /* symbol with zero frequency in the data     */
#define ORC_E_SPACE    (-4)   /* output buffer too small                    */
#define ORC_E_CORRUPT  (-5)   /* decode ran out of bits / bad final state   */
#define ORC_E_NOMEM    (-6)

/* ------------------------------------------------------------------------- */
/* Frequency normalisation.  Paper: silent.  Reading: counts c_s over n symbols
 * become integers f_s with sum exactly L = 2^R, f_s >= 1 exactly when c_s > 0.
 * f_s starts as max(1, floor(c_s * L / n)); the difference to L is then moved
 * one unit at a time onto (or off) the symbol that currently has the largest
 * f (smallest symbol wins ties; never below 1).                              */
int orc_normalize(const uint64_t *counts, int R, uint32_t *f)
{
    if (!counts || !f || R < 1 || R > ORC_MAX_R) return ORC_E_ARG;
    const uint64_t L = 1ull << R;
    uint64_t n = 0;
    int present = 0;
    for (int s = 0; s < ORC_ALPHABET; s++) {
        n += counts[s];
        if (counts[s]) present++;
    }
    if (n == 0 || (uint64_t)present > L) return ORC_E_FREQ;
    int64_t sum = 0;
    for (int s = 0; s < ORC_ALPHABET; s++) {
        if (counts[s] == 0) { f[s] = 0; continue; }
        /* floor(c*L/n) without overflow: c < 2^48 and L <= 2^16 in practice,
         * use long double free integer split to stay exact for any 64-bit c. */
        uint64_t q = counts[s] / n;            /* 0 or 1 (c <= n)              */
        uint64_t r = counts[s] % n;
        uint64_t v = q * L + (uint64_t)(((unsigned __int128)r * L) / n);
        if (v == 0) v = 1;
        f[s] = (uint32_t)v;
        sum += (int64_t)v;
    }
    int64_t d = (int64_t)L - sum;
    while (d != 0) {
        int best = -1;
        for (int s = 0; s < ORC_ALPHABET; s++)
            if (f[s] > 0 && (best < 0 || f[s] > f[best])) best = s;
        if (d > 0) { f[best] += 1; d -= 1; }
        else {
            if (f[best] <= 1) return ORC_E_FREQ;   /* cannot happen: present <= L */
            f[best] -= 1; d += 1;
        }
    }
    return 0;
}

static int check_freqs(const uint32_t *f, int R)
{
    if (!f || R < 1 || R > ORC_MAX_R) return ORC_E_ARG;
    uint64_t sum = 0;
    for (int s = 0; s < ORC_ALPHABET; s++) sum += f[s];
    return sum == (1ull << R) ? 0 : ORC_E_FREQ;
}

/* ------------------------------------------------------------------------- */
/* Spread ("initialization of the states", Sec. II-A).  Paper: says the rate
 * depends on it, does not say which.  Reading: occurrence i (0-based) of symbol
 * s has ideal position (2i+1)/(2 f_s) in [0,1); all L (symbol, occurrence)
 * pairs are sorted by that fraction, equal fractions by smaller symbol, and
 * the rank of a pair is the state index X it occupies.                      */
typedef struct { uint32_t s, i, f; } occ_t;

static int occ_cmp(const void *pa, const void *pb)
{
    const occ_t *a = (const occ_t *)pa, *b = (const occ_t *)pb;
    /* (2 ia + 1) / (2 fa)  vs  (2 ib + 1) / (2 fb), exact in 64-bit */
    uint64_t lhs = (uint64_t)(2 * a->i + 1) * b->f;
    uint64_t rhs = (uint64_t)(2 * b->i + 1) * a->f;
    if (lhs != rhs) return lhs < rhs ? -1 : 1;
    if (a->s != b->s) return a->s < b->s ? -1 : 1;
    return 0;
}

int orc_spread(const uint32_t *f, int R, uint8_t *spread)
{
    int rc = check_freqs(f, R);
    if (rc) return rc;
    if (!spread) return ORC_E_ARG;
    const uint32_t L = 1u << R;
    occ_t *occ = (occ_t *)malloc(sizeof(occ_t) * L);
    if (!occ) return ORC_E_NOMEM;
    uint32_t k = 0;
    for (uint32_t s = 0; s < ORC_ALPHABET; s++)
        for (uint32_t i = 0; i < f[s]; i++) { occ[k].s = s; occ[k].i = i; occ[k].f = f[s]; k++; }
    qsort(occ, L, sizeof(occ_t), occ_cmp);
    for (uint32_t X = 0; X < L; X++) spread[X] = (uint8_t)occ[X].s;
    free(occ);
    return 0;
}

static int floor_log2_u32(uint32_t v)
{
    int r = -1;
    while (v) { v >>= 1; r++; }
    return r;
}

/* ------------------------------------------------------------------------- */
/* Decode table (Sec. II-A: one symbol, one number of bits and one integer per
 * state).  States are x = X + L in [L, 2L).  Walking X upward, the j-th state
 * that carries symbol s is given the sub-state x_s = f_s + j, so x_s covers
 * [f_s, 2 f_s).  nb = R - floor(log2 x_s) is the number of bits that bring x_s
 * back into [L, 2L); newX = (x_s << nb) - L.                                 */
int orc_build_decode_table(const uint32_t *f, int R,
                           uint8_t *sym, uint8_t *nb, uint16_t *newX)
{
    if (!sym || !nb || !newX) return ORC_E_ARG;
    int rc = orc_spread(f, R, sym);
    if (rc) return rc;
    const uint32_t L = 1u << R;
    uint32_t next[ORC_ALPHABET];
    for (int s = 0; s < ORC_ALPHABET; s++) next[s] = f[s];
    for (uint32_t X = 0; X < L; X++) {
        uint32_t s = sym[X];
        uint32_t xs = next[s]++;
        int n = R - floor_log2_u32(xs);
        nb[X] = (uint8_t)n;
        newX[X] = (uint16_t)(((uint64_t)xs << n) - L);
    }
    return 0;
}

/* Byte-packed table of Sec. II-A for l <= 256 states: three bytes per state
 * (symbol, nb_bits, newX), so 3*l bytes in all.  Returns the byte count.     */
int orc_build_decode_table_bytes(const uint32_t *f, int R, uint8_t *lut /* 3*L */)
{
    if (R > 8 || !lut) return ORC_E_ARG;
    const uint32_t L = 1u << R;
    uint8_t s[256], n[256];
    uint16_t x[256];
    int rc = orc_build_decode_table(f, R, s, n, x);
    if (rc) return rc;
    for (uint32_t X = 0; X < L; X++) {
        lut[3 * X + 0] = s[X];
        lut[3 * X + 1] = n[X];
        lut[3 * X + 2] = (uint8_t)x[X];     /* newX < l <= 256 fits one byte */
    }
    return (int)(3 * L);
}

/* ------------------------------------------------------------------------- */
/* Encoder map (Sec. II-A, Fig. 1: encoding follows a transition of the same
 * automaton).  enc[base[s] + (x_s - f_s)] = X, the state whose decode entry
 * carries (s, x_s).                                                          */
int orc_build_encode_map(const uint32_t *f, int R, uint16_t *enc, uint32_t *base)
{
    if (!enc || !base) return ORC_E_ARG;
    int rc = check_freqs(f, R);
    if (rc) return rc;
    const uint32_t L = 1u << R;
    uint8_t *spread = (uint8_t *)malloc(L);
    if (!spread) return ORC_E_NOMEM;
    rc = orc_spread(f, R, spread);
    if (rc) { free(spread); return rc; }
    uint32_t acc = 0;
    for (int s = 0; s < ORC_ALPHABET; s++) { base[s] = acc; acc += f[s]; }
    uint32_t seen[ORC_ALPHABET];
    memset(seen, 0, sizeof(seen));
    for (uint32_t X = 0; X < L; X++) {
        uint32_t s = spread[X];
        enc[base[s] + seen[s]] = (uint16_t)X;
        seen[s]++;
    }
    free(spread);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* One stream.  Symbols of the stream are sym[first + i*stride], i < count.
 *
 * Encoding (Sec. II-A) runs from the last symbol to the first, starting in
 * state x = L (X = 0).  For symbol s in state x: take the smallest n with
 * (x >> n) < 2 f_s; the n low bits of x are the group of bits for this symbol;
 * the new state is the one whose entry carries (s, x >> n).  The state left
 * after the first symbol has been encoded is the decoder's initial state.
 *
 * Bit order (paper: silent).  Reading: the stream's bit sequence is the groups
 * in DECODE order (symbol 0 first); within a group the most significant bit
 * of its value comes first; the sequence is packed into 32-bit words starting
 * at bit 0 of each word and zero-padded to a whole word.
 *
 * Returns the number of 32-bit words written, or a negative error.          */
int64_t orc_encode_stream(const uint8_t *sym, uint64_t first, uint64_t stride, uint64_t count,
                          const uint32_t *f, int R, const uint16_t *enc, const uint32_t *base,
                          uint32_t *words, uint64_t cap_words, uint16_t *init_state)
{
    const uint32_t L = 1u << R;
    if (count == 0) { *init_state = 0; return 0; }
    uint16_t *gval = (uint16_t *)malloc(sizeof(uint16_t) * count);
    uint8_t *gnb = (uint8_t *)malloc(count);
    if (!gval || !gnb) { free(gval); free(gnb); return ORC_E_NOMEM; }
    uint32_t x = L;
    for (uint64_t i = count; i-- > 0;) {
        uint32_t s = sym[first + i * stride];
        uint32_t fs = f[s];
        if (fs == 0) { free(gval); free(gnb); return ORC_E_SYMBOL; }
        int n = 0;
        while ((x >> n) >= 2 * fs) n++;
        gval[i] = (uint16_t)(x & ((1u << n) - 1u));
        gnb[i] = (uint8_t)n;
        x = L + enc[base[s] + ((x >> n) - fs)];
    }
    *init_state = (uint16_t)(x - L);
    uint64_t bitpos = 0;
    for (uint64_t i = 0; i < count; i++) bitpos += gnb[i];
    uint64_t nwords = (bitpos + 31) / 32;
    if (nwords > cap_words) { free(gval); free(gnb); return ORC_E_SPACE; }
    for (uint64_t w = 0; w < nwords; w++) words[w] = 0;
    bitpos = 0;
    for (uint64_t i = 0; i < count; i++) {
        for (int b = 0; b < gnb[i]; b++) {
            if ((gval[i] >> (gnb[i] - 1 - b)) & 1u) words[bitpos >> 5] |= 1u << (bitpos & 31);
            bitpos++;
        }
    }
    free(gval); free(gnb);
    return (int64_t)nwords;
}

/* Decode one stream (Sec. II-A decoder; Sec. III-B: n look-ups and n small
 * additions for a stream of n weights).  Writes out[first + i*stride].
 * Also reports the total number of bits read.  Returns 0, or ORC_E_CORRUPT if
 * the stream runs out of bits, does not end in state 0, or leaves whole words
 * unread.                                                                    */
int orc_decode_stream(const uint32_t *words, uint64_t nwords, uint16_t init_state, uint64_t count,
                      int R, const uint8_t *tsym, const uint8_t *tnb, const uint16_t *tnewX,
                      uint8_t *out, uint64_t first, uint64_t stride, uint64_t *bits_read)
{
    const uint32_t L = 1u << R;
    uint32_t X = init_state;
    uint64_t bitpos = 0;
    if (X >= L) return ORC_E_CORRUPT;
    for (uint64_t i = 0; i < count; i++) {
        uint32_t n = tnb[X];
        uint32_t v = 0;
        if (bitpos + n > nwords * 32) return ORC_E_CORRUPT;
        for (uint32_t b = 0; b < n; b++) {
            uint64_t p = bitpos + b;
            v = (v << 1) | ((words[p >> 5] >> (p & 31)) & 1u);
        }
        bitpos += n;
        out[first + i * stride] = tsym[X];
        X = (uint32_t)tnewX[X] + v;
        if (X >= L) return ORC_E_CORRUPT;
    }
    if (bits_read) *bits_read = bitpos;
    if (X != 0) return ORC_E_CORRUPT;
    if ((bitpos + 31) / 32 != nwords) return ORC_E_CORRUPT;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Layer container.
 *
 * Stream split (Sec. II-A end / Sec. III-B: the flow of weights is split into
 * concurrent streams that share one decoder).  Paper groups by input channel;
 * the workloads ask for "N interleaved streams per chunk".  Reading: a layer
 * (flat, row-major) is cut into consecutive chunks of chunk_size symbols (the
 * last may be short; chunks never cross layers because tables are per layer,
 * Sec. III-A); inside a chunk element j belongs to stream j mod N and is that
 * stream's symbol number j div N.
 *
 * Container layout (paper: "FIFO", nothing more).  Reading: each stream is a
 * private run of 32-bit words; a chunk's payload is its streams' words back to
 * back in stream order, and every chunk's payload starts on a multiple of 4
 * words (zero words in between).  Per stream one 32-bit header: initial state
 * in bits 0..15, word count in bits 16..31.
 *
 * Outputs, all caller-allocated:
 *   chunk_nsym[c], chunk_payload_off[c] (in words, relative to payload_base),
 *   chunk_payload_words[c], stream_hdr[c*N + k], payload words.
 * Returns the number of payload words used (including alignment padding after
 * every chunk), or a negative error.                                         */
int64_t orc_encode_layer(const uint8_t *sym, uint64_t n, const uint32_t *f, int R,
                         uint32_t N, uint32_t chunk_size,
                         uint32_t *chunk_nsym, uint64_t *chunk_payload_off,
                         uint32_t *chunk_payload_words, uint32_t *stream_hdr,
                         uint32_t *payload, uint64_t cap_words)
{
    if (!sym || N < 1 || chunk_size < 1) return ORC_E_ARG;
    int rc = check_freqs(f, R);
    if (rc) return rc;
    const uint32_t L = 1u << R;
    uint16_t *enc = (uint16_t *)malloc(sizeof(uint16_t) * L);
    uint32_t base[ORC_ALPHABET];
    if (!enc) return ORC_E_NOMEM;
    rc = orc_build_encode_map(f, R, enc, base);
    if (rc) { free(enc); return rc; }
    uint64_t n_chunks = (n + chunk_size - 1) / chunk_size;
    uint64_t pos = 0;                      /* word cursor in payload */
    for (uint64_t c = 0; c < n_chunks; c++) {
        uint64_t start = c * (uint64_t)chunk_size;
        uint64_t cn = n - start < chunk_size ? n - start : chunk_size;
        chunk_nsym[c] = (uint32_t)cn;
        chunk_payload_off[c] = pos;
        uint64_t cw = 0;
        for (uint32_t k = 0; k < N; k++) {
            uint64_t count = cn > k ? (cn - k + N - 1) / N : 0;
            uint16_t X0 = 0;
            int64_t nw = orc_encode_stream(sym, start + k, N, count, f, R, enc, base,
                                           payload + pos + cw, cap_words - pos - cw, &X0);
            if (nw < 0) { free(enc); return nw; }
            if (nw > 0xFFFF) { free(enc); return ORC_E_SPACE; }
            stream_hdr[c * N + k] = (uint32_t)X0 | ((uint32_t)nw << 16);
            cw += (uint64_t)nw;
        }
        chunk_payload_words[c] = (uint32_t)cw;
        pos += cw;
        while (pos & 3u) {
            if (pos >= cap_words) { free(enc); return ORC_E_SPACE; }
            payload[pos++] = 0;
        }
    }
    free(enc);
    return (int64_t)pos;
}

/* Decode a range of chunks of a multi-layer container into symbols.
 * tables: per layer, L entries each of tsym / tnb / tnewX (layer-major).
 * Returns 0 or the first error met.                                          */
int orc_decode_chunks(uint64_t c_begin, uint64_t c_end,
                      const uint32_t *chunk_layer, const uint32_t *chunk_nsym,
                      const uint64_t *chunk_out_off, const uint64_t *chunk_payload_off,
                      const uint32_t *chunk_stream_off,
                      const uint32_t *stream_hdr, const uint32_t *payload, uint64_t payload_words,
                      int R, uint32_t N,
                      const uint8_t *tsym, const uint8_t *tnb, const uint16_t *tnewX,
                      uint8_t *out_sym)
{
    const uint64_t L = 1ull << R;
    int first_err = 0;
    for (uint64_t c = c_begin; c < c_end; c++) {
        uint64_t lay = chunk_layer[c];
        uint64_t cn = chunk_nsym[c];
        uint64_t woff = chunk_payload_off[c];
        for (uint32_t k = 0; k < N; k++) {
            uint32_t hdr = stream_hdr[chunk_stream_off[c] + k];
            uint64_t nw = hdr >> 16;
            uint64_t count = cn > k ? (cn - k + N - 1) / N : 0;
            int rc;
            if (woff > payload_words || nw > payload_words - woff)
                rc = ORC_E_CORRUPT;        /* a header that points outside the payload: the stream is not read */
            else
                rc = orc_decode_stream(payload + woff, nw, (uint16_t)(hdr & 0xFFFFu), count, R,
                                       tsym + lay * L, tnb + lay * L, tnewX + lay * L,
                                       out_sym, chunk_out_off[c] + k, N, NULL);
            if (rc && !first_err) first_err = rc;
            woff += nw;
        }
    }
    return first_err;
}

/* ------------------------------------------------------------------------- */
/* Dequantisation (Sec. II-B: uniform quantizer with a zero-point, symmetric
 * points).  Reading: w = fl32(scale * fl32(q - z)), one IEEE-754 binary32
 * multiplication of an exactly representable integer.  bf16 output is w
 * rounded to nearest, ties to even, to the upper 16 bits of its binary32
 * pattern.  scale index for element e of a layer: per layer when
 * channel_len == 0, else scales[scales_off + e / channel_len].               */
static float dequant_one(uint8_t q, uint32_t z, float scale)
{
    float d = (float)((int)q - (int)z);   /* exact: |q - z| <= 255 */
    return scale * d;                      /* one rounding (build with -ffp-contract=off) */
}

static uint16_t f32_to_bf16_rne(float w)
{
    uint32_t u;
    memcpy(&u, &w, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu))     /* NaN: keep quiet NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

void orc_dequant_f32(const uint8_t *q, uint64_t e_begin, uint64_t e_end, uint64_t layer_first,
                     uint32_t z, float scale, uint32_t channel_len,
                     const float *scales, uint64_t scales_off, float *out)
{
    for (uint64_t e = e_begin; e < e_end; e++) {
        float s = channel_len ? scales[scales_off + (e - layer_first) / channel_len] : scale;
        out[e] = dequant_one(q[e], z, s);
    }
}

void orc_dequant_bf16(const uint8_t *q, uint64_t e_begin, uint64_t e_end, uint64_t layer_first,
                      uint32_t z, float scale, uint32_t channel_len,
                      const float *scales, uint64_t scales_off, uint16_t *out)
{
    for (uint64_t e = e_begin; e < e_end; e++) {
        float s = channel_len ? scales[scales_off + (e - layer_first) / channel_len] : scale;
        out[e] = f32_to_bf16_rne(dequant_one(q[e], z, s));
    }
}

/* ------------------------------------------------------------------------- */
/* Whole path, the thing the GPU is compared with and timed beside: decode
 * every chunk, then dequantise every element, with a plain split of the chunk
 * list over n_threads POSIX threads (contiguous ranges).  out_dtype: 1 = fp32,
 * 2 = bf16.                                                                  */
typedef struct {
    uint64_t c_begin, c_end;
    const uint32_t *chunk_layer, *chunk_nsym;
    const uint64_t *chunk_out_off, *chunk_payload_off;
    const uint32_t *chunk_stream_off, *stream_hdr, *payload;
    uint64_t payload_words;
    int R; uint32_t N;
    const uint8_t *tsym, *tnb; const uint16_t *tnewX;
    const uint32_t *lay_z; const float *lay_scale; const uint32_t *lay_channel_len;
    const uint64_t *lay_scales_off, *lay_out_base; const float *scales;
    uint8_t *out_sym; void *out; int out_dtype;
    int rc;
} job_t;

static void *job_run(void *p)
{
    job_t *j = (job_t *)p;
    j->rc = orc_decode_chunks(j->c_begin, j->c_end, j->chunk_layer, j->chunk_nsym, j->chunk_out_off,
                              j->chunk_payload_off, j->chunk_stream_off, j->stream_hdr, j->payload, j->payload_words,
                              j->R, j->N, j->tsym, j->tnb, j->tnewX, j->out_sym);
    for (uint64_t c = j->c_begin; c < j->c_end; c++) {
        uint32_t lay = j->chunk_layer[c];
        uint64_t b = j->chunk_out_off[c], e = b + j->chunk_nsym[c];
        if (j->out_dtype == 1)
            orc_dequant_f32(j->out_sym, b, e, j->lay_out_base[lay], j->lay_z[lay], j->lay_scale[lay],
                            j->lay_channel_len[lay], j->scales, j->lay_scales_off[lay], (float *)j->out);
        else if (j->out_dtype == 2)
            orc_dequant_bf16(j->out_sym, b, e, j->lay_out_base[lay], j->lay_z[lay], j->lay_scale[lay],
                             j->lay_channel_len[lay], j->scales, j->lay_scales_off[lay], (uint16_t *)j->out);
    }
    return NULL;
}

int orc_decode_dequant(uint64_t n_chunks,
                       const uint32_t *chunk_layer, const uint32_t *chunk_nsym,
                       const uint64_t *chunk_out_off, const uint64_t *chunk_payload_off,
                       const uint32_t *chunk_stream_off,
                       const uint32_t *stream_hdr, const uint32_t *payload, uint64_t payload_words,
                       int R, uint32_t N,
                       const uint8_t *tsym, const uint8_t *tnb, const uint16_t *tnewX,
                       const uint32_t *lay_z, const float *lay_scale, const uint32_t *lay_channel_len,
                       const uint64_t *lay_scales_off, const uint64_t *lay_out_base, const float *scales,
                       uint8_t *out_sym, void *out, int out_dtype, int n_threads)
{
    if (n_threads < 1) n_threads = 1;
    if ((uint64_t)n_threads > n_chunks) n_threads = n_chunks ? (int)n_chunks : 1;
    job_t *jobs = (job_t *)calloc((size_t)n_threads, sizeof(job_t));
    pthread_t *th = (pthread_t *)calloc((size_t)n_threads, sizeof(pthread_t));
    if (!jobs || !th) { free(jobs); free(th); return ORC_E_NOMEM; }
    for (int t = 0; t < n_threads; t++) {
        job_t *j = &jobs[t];
        j->c_begin = n_chunks * (uint64_t)t / (uint64_t)n_threads;
        j->c_end = n_chunks * (uint64_t)(t + 1) / (uint64_t)n_threads;
        j->chunk_layer = chunk_layer; j->chunk_nsym = chunk_nsym; j->chunk_out_off = chunk_out_off;
        j->chunk_payload_off = chunk_payload_off; j->chunk_stream_off = chunk_stream_off;
        j->stream_hdr = stream_hdr; j->payload = payload; j->payload_words = payload_words; j->R = R; j->N = N;
        j->tsym = tsym; j->tnb = tnb; j->tnewX = tnewX;
        j->lay_z = lay_z; j->lay_scale = lay_scale; j->lay_channel_len = lay_channel_len;
        j->lay_scales_off = lay_scales_off; j->lay_out_base = lay_out_base; j->scales = scales;
        j->out_sym = out_sym; j->out = out; j->out_dtype = out_dtype;
    }
    if (n_threads == 1) job_run(&jobs[0]);
    else {
        for (int t = 0; t < n_threads; t++) pthread_create(&th[t], NULL, job_run, &jobs[t]);
        for (int t = 0; t < n_threads; t++) pthread_join(th[t], NULL);
    }
    int rc = 0;
    for (int t = 0; t < n_threads; t++) if (jobs[t].rc && !rc) rc = jobs[t].rc;
    free(jobs); free(th);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Shannon quantities (Sec. II-A, source coding theorem): empirical entropy of
 * the counts, and the cross-entropy of the counts under the table's model
 * p_s = f_s / L, both in bits per symbol.                                    */
double orc_entropy_bits(const uint64_t *counts)
{
    double n = 0.0, h = 0.0;
    for (int s = 0; s < ORC_ALPHABET; s++) n += (double)counts[s];
    if (n == 0.0) return 0.0;
    for (int s = 0; s < ORC_ALPHABET; s++)
        if (counts[s]) { double p = (double)counts[s] / n; h -= p * log2(p); }
    return h;
}

double orc_cross_entropy_bits(const uint64_t *counts, const uint32_t *f, int R)
{
    double n = 0.0, h = 0.0, L = (double)(1u << R);
    for (int s = 0; s < ORC_ALPHABET; s++) n += (double)counts[s];
    if (n == 0.0) return 0.0;
    for (int s = 0; s < ORC_ALPHABET; s++)
        if (counts[s]) {
            if (!f[s]) return INFINITY;
            h -= ((double)counts[s] / n) * log2((double)f[s] / L);
        }
    return h;
}
