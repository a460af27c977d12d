// tANS encoder on the GPU: compresses one layer whose symbols are in device memory into the
// container anszp_decode reads, word for word what the host packer (anszp_pack_layer) writes.
//
// Encoding (Sec. II-A) walks a stream's symbols backwards: to encode symbol s in state x (in
// [L, 2L)) the low bits of x are dropped, and written out, until x lies in [f_s, 2 f_s); the new
// state is the (x - f_s)-th state of s, counted in increasing order, plus L.  The decoder reads the
// bits of the first symbol first, so a stream's bits are laid down from its end: the walk is done
// once to learn the stream's length and once to write.
//
// Three launches, nothing allocated and no scratch memory: sizes (every stream's final state and
// word count into the stream headers, every chunk's descriptor but for its payload offset), a scan
// over the chunks (payload offsets, total), the writing pass.  One lane per stream, one wavefront
// per chunk at a time; every workgroup builds the encoding tables in LDS for itself from the
// frequencies: the states of a symbol in increasing order are the ranks of its occurrences in the
// merged position sequences (the spread this library chose; Sec. II-A says only that the rate depends
// on how the states are initialised), and a rank is a sum of integer quotients.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "anszp.h"

namespace {

constexpr uint32_t kWave = 64;
constexpr uint32_t kThreads = 256;
constexpr uint32_t kWaves = kThreads / kWave;
constexpr uint32_t kStates = 1u << ANSZP_MAX_TABLE_LOG;
constexpr uint32_t kBatch = 8;              // symbols a lane asks for at a time

struct EncParams {
    const uint8_t* symbols;
    const uint32_t* freqs;
    anszp_chunk_t* chunks;
    uint32_t* stream_hdr;
    uint32_t* payload;
    unsigned long long* used;
    uint32_t* status;
    uint64_t n_symbols, n_chunks, out_offset, payload_word_offset, payload_cap_words;
    uint32_t table_log, n_streams, chunk_size, layer_id, stream_offset;
};

struct EncTables {
    uint32_t f[ANSZP_ALPHABET];
    uint32_t first[ANSZP_ALPHABET];        // index of the symbol's first state in `states`
    uint16_t states[kStates];              // the states of each symbol in increasing order
    uint32_t used_sym[ANSZP_ALPHABET];     // symbols with f > 0, in increasing order
    uint32_t n_used, total;
};

__device__ __forceinline__ void report(uint32_t* status, uint32_t bits) {
    atomicOr(&status[0], bits);
    atomicAdd(&status[1], 1u);
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int d = 1; d < int(kWave); d <<= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

__device__ __forceinline__ uint32_t wave_exclusive_sum(uint32_t v, uint32_t lane) {
    uint32_t s = v;
#pragma unroll
    for (int d = 1; d < int(kWave); d <<= 1) {
        const uint32_t t = __shfl_up(s, d, kWave);
        if (lane >= uint32_t(d)) s += t;
    }
    return s - v;
}

// The workgroup's encoding tables.  False (for every thread) when the frequencies do not sum to L.
__device__ bool build_tables(const uint32_t* freqs, uint32_t table_log, EncTables& t) {
    const uint32_t tid = threadIdx.x;
    const uint32_t L = 1u << table_log;
    if (tid < ANSZP_ALPHABET) t.f[tid] = freqs[tid];
    __syncthreads();
    if (tid == 0) {
        uint32_t n = 0, acc = 0;
        for (uint32_t s = 0; s < ANSZP_ALPHABET; ++s) {
            const uint32_t fs = t.f[s];
            t.first[s] = min(acc, L);
            if (fs) t.used_sym[n++] = s;
            acc = min(acc + min(fs, L + 1u), L + 1u);           // saturating
        }
        t.n_used = n;
        t.total = acc;
    }
    __syncthreads();
    if (t.total != L) return false;
    const uint32_t used = t.n_used;
    // occurrence i of symbol s sits at (2i + 1) / (2 f_s) (Sec. II-A), ties going to the smaller symbol: its
    // rank among all occurrences is i plus, for every other symbol, the number of its occurrences before it
    for (uint32_t g = tid; g < L; g += kThreads) {
        uint32_t lo = 0, hi = used;                              // first[used_sym[lo]] <= g
        while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (t.first[t.used_sym[mid]] <= g) lo = mid; else hi = mid;
        }
        const uint32_t s = t.used_sym[lo], fs = t.f[s], i = g - t.first[s];
        uint32_t rank = i;
        for (uint32_t k = 0; k < used; ++k) {
            if (k == lo) continue;
            const uint32_t fo = t.f[t.used_sym[k]];
            const int32_t q = static_cast<int32_t>((2u * i + 1u) * fo) - static_cast<int32_t>(fs);   // below 2^26
            uint32_t before;
            if (k < lo) before = q < 0 ? 0u : static_cast<uint32_t>(q) / (2u * fs) + 1u;
            else before = q <= 0 ? 0u : (static_cast<uint32_t>(q) + 2u * fs - 1u) / (2u * fs);
            rank += min(before, fo);
        }
        t.states[g] = static_cast<uint16_t>(rank);
    }
    __syncthreads();
    return true;
}

// One stream, backwards (Sec. II-A).  WRITE: lay the bits down in `words` (the stream's n_words words);
// otherwise only count them.  Returns the number of bits; x_out: the final state plus L.
// The bits a symbol adds precede, in the stream, everything written so far; the stream is therefore built
// in reverse, padded at its start so that whole reversed words are whole words of the stream, and each
// finished word is bit-reversed into its place, from the stream's last word down to its first.
template <bool WRITE>
__device__ uint32_t walk_stream(const EncParams& p, const EncTables& t, uint64_t begin, uint32_t cn, uint32_t k,
                                uint32_t* words, uint32_t n_words, uint32_t n_bits, uint32_t& x_out, bool& bad_symbol) {
    const uint32_t N = p.n_streams, L = 1u << p.table_log;
    const uint32_t len = (k < N && cn > k) ? (cn - k + N - 1u) / N : 0u;
    uint32_t x = L, bits = 0;
    uint64_t acc = 0;
    uint32_t cnt = WRITE ? 32u * n_words - n_bits : 0u;       // zero bits behind the stream's last bit
    uint32_t at = n_words;                                    // words still to be written
    for (uint32_t hi = len; hi > 0;) {
        const uint32_t batch = min(hi, kBatch);
        uint32_t sym[kBatch];
#pragma unroll
        for (uint32_t j = 0; j < kBatch; ++j)                  // from a clamped, valid index: no load under a condition
            sym[j] = p.symbols[begin + k + uint64_t(hi - 1u - min(j, batch - 1u)) * N];
#pragma unroll
        for (uint32_t j = 0; j < kBatch; ++j) {
            if (j < batch) {
                const uint32_t s = sym[j], fs = t.f[s];
                if (fs == 0) { bad_symbol = true; continue; }
                uint32_t drop = 0;
                while ((x >> drop) >= 2u * fs) ++drop;          // bring x into [f_s, 2 f_s)
                if (WRITE) {
                    acc |= uint64_t(x & ((1u << drop) - 1u)) << cnt;
                    cnt += drop;
                    if (cnt >= 32u) {
                        if (at) words[--at] = __brev(static_cast<uint32_t>(acc));
                        acc >>= 32;
                        cnt -= 32u;
                    }
                }
                bits += drop;
                x = L + t.states[t.first[s] + (x >> drop) - fs];
            }
        }
        hi -= batch;
    }
    x_out = x;
    return bits;
}

__global__ __launch_bounds__(kThreads) void encode_sizes(EncParams p) {
    __shared__ EncTables t;
    if (!build_tables(p.freqs, p.table_log, t)) {
        if (threadIdx.x == 0 && blockIdx.x == 0) report(p.status, ANSZP_ST_BAD_FREQ);
        return;
    }
    const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint32_t N = p.n_streams, L = 1u << p.table_log;
    for (uint64_t c = uint64_t(blockIdx.x) * kWaves + wave; c < p.n_chunks; c += uint64_t(gridDim.x) * kWaves) {
        const uint64_t begin = c * p.chunk_size;
        const uint64_t rest = p.n_symbols - begin;
        const uint32_t cn = rest < p.chunk_size ? static_cast<uint32_t>(rest) : p.chunk_size;
        uint32_t x = L;
        bool bad = false;
        const uint32_t bits = walk_stream<false>(p, t, begin, cn, lane, nullptr, 0u, 0u, x, bad);
        const uint32_t nw = (bits + 31u) >> 5;
        const bool too_long = nw > 0xFFFFu;
        if (lane < N) p.stream_hdr[c * N + lane] = (x - L) | (min(nw, 0xFFFFu) << 16);
        const uint32_t chunk_words = wave_sum(lane < N ? min(nw, 0xFFFFu) : 0u);
        if (__ballot(bad) && lane == 0) report(p.status, ANSZP_ST_BAD_SYMBOL);
        if (__ballot(too_long) && lane == 0) report(p.status, ANSZP_ST_NO_SPACE);
        if (lane == 0) {
            anszp_chunk_t d;
            d.layer_id = p.layer_id;
            d.n_symbols = cn;
            d.out_offset = p.out_offset + begin;
            d.payload_offset = 0;                               // by the scan
            d.payload_words = chunk_words;
            d.stream_offset = p.stream_offset + static_cast<uint32_t>(c) * N;
            p.chunks[c] = d;
        }
    }
}

// Payload offsets: every chunk starts on a multiple of four words.  One workgroup, chunks in order.
__global__ __launch_bounds__(kThreads) void encode_scan(EncParams p) {
    __shared__ unsigned long long part[kThreads];
    __shared__ unsigned long long carry;
    const uint32_t tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (uint64_t base = 0; base < p.n_chunks; base += kThreads) {
        const uint64_t c = base + tid;
        const unsigned long long mine = c < p.n_chunks ? ((unsigned long long)(p.chunks[c].payload_words) + 3ull) & ~3ull : 0ull;
        part[tid] = mine;
        __syncthreads();
        for (uint32_t d = 1; d < kThreads; d <<= 1) {           // inclusive scan
            const unsigned long long v = tid >= d ? part[tid - d] : 0ull;
            __syncthreads();
            part[tid] += v;
            __syncthreads();
        }
        if (c < p.n_chunks) p.chunks[c].payload_offset = p.payload_word_offset + carry + part[tid] - mine;
        __syncthreads();
        if (tid == kThreads - 1) carry += part[tid];
        __syncthreads();
    }
    if (tid == 0) {
        *p.used = carry;
        if (carry > p.payload_cap_words) report(p.status, ANSZP_ST_NO_SPACE);
    }
}

__global__ __launch_bounds__(kThreads) void encode_write(EncParams p) {
    __shared__ EncTables t;
    if (!build_tables(p.freqs, p.table_log, t)) return;          // reported by the first pass
    const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint32_t N = p.n_streams, L = 1u << p.table_log;
    for (uint64_t c = uint64_t(blockIdx.x) * kWaves + wave; c < p.n_chunks; c += uint64_t(gridDim.x) * kWaves) {
        const anszp_chunk_t d = p.chunks[c];
        const uint64_t at = d.payload_offset - p.payload_word_offset;          // in the caller's payload region
        const uint64_t padded = (uint64_t(d.payload_words) + 3ull) & ~3ull;
        if (at > p.payload_cap_words || padded > p.payload_cap_words - at) continue;   // no room: reported by the scan
        const uint64_t begin = c * p.chunk_size;
        const uint32_t nw = lane < N ? p.stream_hdr[c * N + lane] >> 16 : 0u;
        uint32_t* words = p.payload + at + wave_exclusive_sum(nw, lane);
        uint32_t x = L;
        bool bad = false;
        const uint32_t bits = walk_stream<false>(p, t, begin, d.n_symbols, lane, nullptr, 0u, 0u, x, bad);
        if (((bits + 31u) >> 5) == nw)                             // (a stream too long for its header is not written)
            walk_stream<true>(p, t, begin, d.n_symbols, lane, words, nw, bits, x, bad);
        if (lane < padded - d.payload_words) p.payload[at + d.payload_words + lane] = 0u;   // up to three pad words
    }
}

// ---- a whole set of layers in three launches.  One workgroup per chunk: all of it builds the chunk's layer's
// tables, its first wavefront walks the chunk's streams.
struct BatchParams {
    EncParams p;                       // what all layers share (symbols: the set's first symbol; freqs: the first row)
    const anszp_pack_job_t* jobs;
    uint32_t n_layers;
};

// The layer of chunk c (jobs are in chunk order: the last one whose first_chunk is not beyond c), as EncParams
// of that layer alone; local: the chunk's number within its layer.  False when c belongs to no layer.
__device__ bool layer_of_chunk(const BatchParams& b, uint64_t c, EncParams& q, uint64_t& local) {
    uint32_t lo = 0, hi = b.n_layers;
    if (hi == 0 || b.jobs[0].first_chunk > c) return false;
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (b.jobs[mid].first_chunk <= c) lo = mid; else hi = mid;
    }
    const anszp_pack_job_t j = b.jobs[lo];
    local = c - j.first_chunk;
    if (j.chunk_size == 0 || local >= (j.n_symbols + j.chunk_size - 1) / j.chunk_size) return false;
    q = b.p;
    q.symbols = b.p.symbols + j.first_symbol;
    q.freqs = b.p.freqs + size_t(lo) * ANSZP_ALPHABET;
    q.n_symbols = j.n_symbols;
    q.chunk_size = j.chunk_size;
    q.layer_id = lo;
    q.out_offset = j.first_symbol;
    return true;
}

__global__ __launch_bounds__(kThreads) void encode_sizes_batch(BatchParams b) {
    __shared__ EncTables t;
    const uint64_t c = blockIdx.x;
    EncParams q;
    uint64_t local;
    const bool mine = layer_of_chunk(b, c, q, local);           // (alike for every thread)
    if (!mine) {
        if (threadIdx.x == 0) {
            report(b.p.status, ANSZP_ST_BAD_DESC);               // the jobs do not cover the chunks the caller counted
            anszp_chunk_t d = {};
            b.p.chunks[c] = d;
        }
        if (threadIdx.x < b.p.n_streams) b.p.stream_hdr[c * b.p.n_streams + threadIdx.x] = 0u;
        return;
    }
    const bool tables_ok = build_tables(q.freqs, q.table_log, t);
    const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (wave != 0) return;
    const uint32_t N = q.n_streams, L = 1u << q.table_log;
    const uint64_t begin = local * q.chunk_size;
    const uint64_t rest = q.n_symbols - begin;
    const uint32_t cn = rest < q.chunk_size ? static_cast<uint32_t>(rest) : q.chunk_size;
    uint32_t x = L, nw = 0;
    bool bad = false, too_long = false;
    if (tables_ok) {
        const uint32_t bits = walk_stream<false>(q, t, begin, cn, lane, nullptr, 0u, 0u, x, bad);
        nw = (bits + 31u) >> 5;
        too_long = nw > 0xFFFFu;
    } else if (lane == 0 && local == 0) {
        report(q.status, ANSZP_ST_BAD_FREQ);
    }
    if (lane < N) q.stream_hdr[c * N + lane] = (x - L) | (min(nw, 0xFFFFu) << 16);
    const uint32_t chunk_words = wave_sum(lane < N ? min(nw, 0xFFFFu) : 0u);
    if (__ballot(bad) && lane == 0) report(q.status, ANSZP_ST_BAD_SYMBOL);
    if (__ballot(too_long) && lane == 0) report(q.status, ANSZP_ST_NO_SPACE);
    if (lane == 0) {
        anszp_chunk_t d;
        d.layer_id = q.layer_id;
        d.n_symbols = tables_ok ? cn : 0u;
        d.out_offset = q.out_offset + begin;
        d.payload_offset = 0;                                   // by the scan
        d.payload_words = chunk_words;
        d.stream_offset = static_cast<uint32_t>(c) * N;
        q.chunks[c] = d;
    }
}

__global__ __launch_bounds__(kThreads) void encode_write_batch(BatchParams b) {
    __shared__ EncTables t;
    const uint64_t c = blockIdx.x;
    EncParams q;
    uint64_t local;
    if (!layer_of_chunk(b, c, q, local)) return;                 // reported by the first pass
    if (!build_tables(q.freqs, q.table_log, t)) return;
    const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (wave != 0) return;
    const uint32_t N = q.n_streams, L = 1u << q.table_log;
    const anszp_chunk_t d = q.chunks[c];
    const uint64_t at = d.payload_offset;
    const uint64_t padded = (uint64_t(d.payload_words) + 3ull) & ~3ull;
    if (at > q.payload_cap_words || padded > q.payload_cap_words - at) return;     // no room: reported by the scan
    const uint64_t begin = local * q.chunk_size;
    const uint32_t nw = lane < N ? q.stream_hdr[c * N + lane] >> 16 : 0u;
    uint32_t* words = q.payload + at + wave_exclusive_sum(nw, lane);
    uint32_t x = L;
    bool bad = false;
    const uint32_t bits = walk_stream<false>(q, t, begin, d.n_symbols, lane, nullptr, 0u, 0u, x, bad);
    if (((bits + 31u) >> 5) == nw)                               // (a stream too long for its header is not written)
        walk_stream<true>(q, t, begin, d.n_symbols, lane, words, nw, bits, x, bad);
    if (lane < padded - d.payload_words) q.payload[at + d.payload_words + lane] = 0u;   // up to three pad words
}

}  // namespace

extern "C" int anszp_pack_layers_device(const uint8_t* symbols_dev, const anszp_pack_job_t* jobs_dev, uint32_t n_layers,
                                        uint64_t n_chunks, const uint32_t* freqs_dev, int table_log, int n_streams,
                                        anszp_chunk_t* chunks_dev, uint32_t* stream_hdr_dev, uint32_t* payload_dev,
                                        uint64_t payload_cap_words, uint64_t* payload_words_used_dev,
                                        uint32_t* status_dev, void* stream) {
    if (!payload_words_used_dev || !status_dev) return ANSZP_E_NULL;
    if (n_chunks && (!symbols_dev || !jobs_dev || !freqs_dev || !chunks_dev || !stream_hdr_dev)) return ANSZP_E_NULL;
    if (!payload_dev && payload_cap_words) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_streams < 1 || n_streams > ANSZP_MAX_STREAMS ||
        n_chunks >= (1ull << 31) || uint64_t(n_chunks) * uint64_t(n_streams) >= (1ull << 32) || (n_chunks && n_layers == 0))
        return ANSZP_E_RANGE;
    BatchParams b{};
    b.p.symbols = symbols_dev; b.p.freqs = freqs_dev; b.p.chunks = chunks_dev; b.p.stream_hdr = stream_hdr_dev;
    b.p.payload = payload_dev; b.p.used = reinterpret_cast<unsigned long long*>(payload_words_used_dev); b.p.status = status_dev;
    b.p.n_chunks = n_chunks; b.p.payload_word_offset = 0; b.p.payload_cap_words = payload_cap_words;
    b.p.table_log = uint32_t(table_log); b.p.n_streams = uint32_t(n_streams);
    b.jobs = jobs_dev; b.n_layers = n_layers;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_chunks) hipLaunchKernelGGL(encode_sizes_batch, dim3(uint32_t(n_chunks)), dim3(kThreads), 0, s, b);
    hipLaunchKernelGGL(encode_scan, dim3(1), dim3(kThreads), 0, s, b.p);
    if (n_chunks) hipLaunchKernelGGL(encode_write_batch, dim3(uint32_t(n_chunks)), dim3(kThreads), 0, s, b);
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}

extern "C" int anszp_pack_layer_device(const uint8_t* symbols_dev, uint64_t n_symbols, const uint32_t* freqs_dev,
                                       int table_log, int n_streams, uint32_t chunk_size, uint32_t layer_id,
                                       uint64_t out_offset, uint64_t payload_word_offset, uint32_t stream_offset,
                                       anszp_chunk_t* chunks_dev, uint32_t* stream_hdr_dev, uint32_t* payload_dev,
                                       uint64_t payload_cap_words, uint64_t* payload_words_used_dev,
                                       uint32_t* status_dev, void* stream) {
    if (!freqs_dev || !payload_words_used_dev || !status_dev) return ANSZP_E_NULL;
    if (n_symbols && (!symbols_dev || !chunks_dev || !stream_hdr_dev)) return ANSZP_E_NULL;
    if (!payload_dev && payload_cap_words) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_streams < 1 || n_streams > ANSZP_MAX_STREAMS ||
        chunk_size < 1 || (payload_word_offset & 3))
        return ANSZP_E_RANGE;
    EncParams p{};
    p.symbols = symbols_dev; p.freqs = freqs_dev; p.chunks = chunks_dev; p.stream_hdr = stream_hdr_dev;
    p.payload = payload_dev; p.used = reinterpret_cast<unsigned long long*>(payload_words_used_dev); p.status = status_dev;
    p.n_symbols = n_symbols; p.n_chunks = (n_symbols + chunk_size - 1) / chunk_size;
    p.out_offset = out_offset; p.payload_word_offset = payload_word_offset; p.payload_cap_words = payload_cap_words;
    p.table_log = uint32_t(table_log); p.n_streams = uint32_t(n_streams); p.chunk_size = chunk_size;
    p.layer_id = layer_id; p.stream_offset = stream_offset;
    if (p.n_chunks >= (1ull << 32)) return ANSZP_E_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t wanted = (p.n_chunks + kWaves - 1) / kWaves;
    const uint32_t grid = uint32_t(wanted < 1 ? 1 : wanted > 2048 ? 2048 : wanted);
    hipLaunchKernelGGL(encode_sizes, dim3(grid), dim3(kThreads), 0, s, p);
    hipLaunchKernelGGL(encode_scan, dim3(1), dim3(kThreads), 0, s, p);
    hipLaunchKernelGGL(encode_write, dim3(grid), dim3(kThreads), 0, s, p);
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
}
