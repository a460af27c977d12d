// Device side of libanszp for gfx950 (MI355X): tANS decode kernels with fused zero-point
// dequantisation, and the stand-alone dequantiser.
//
// Paper sections followed: Sec. II-A (one decode step = table look-up, read nb_bits, state =
// newX + bits), Sec. III-B (a vector of states, one per stream, all sharing one table: here a
// 64-lane wavefront is the vector and a lane is a stream), Sec. II-B (w = scale * (q - z)).
#include "anszp.h"

#include <hip/hip_runtime.h>

namespace {

constexpr int kWave = 64;

struct DecodeParams {
    const uint64_t* tables;
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

__device__ __forceinline__ uint16_t bf16_rne(float w) {
    uint32_t u = __float_as_uint(w);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

template <int OUT>
__device__ __forceinline__ void store_weight(void* out, uint64_t idx, uint32_t sym, uint32_t z, float scale) {
    if constexpr (OUT == ANSZP_OUT_U8) {
        static_cast<uint8_t*>(out)[idx] = static_cast<uint8_t>(sym);
    } else {
        const float w = scale * static_cast<float>(static_cast<int>(sym) - static_cast<int>(z));
        if constexpr (OUT == ANSZP_OUT_F32) static_cast<float*>(out)[idx] = w;
        else static_cast<uint16_t*>(out)[idx] = bf16_rne(w);
    }
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

// Returns true (for the whole wavefront) when the chunk descriptor stays inside the caller's buffers.
__device__ __forceinline__ bool chunk_in_bounds(const DecodeParams& p, const anszp_chunk_t& c) {
    return c.layer_id < p.n_tables &&
           c.out_offset <= p.out_elems && c.n_symbols <= p.out_elems - c.out_offset &&
           c.payload_offset <= p.payload_words && c.payload_words <= p.payload_words - c.payload_offset &&
           uint64_t(c.stream_offset) + p.n_streams <= p.n_stream_hdr;
}

// ---------------------------------------------------------------------------------------------
// Reference-shaped kernel: one wavefront per chunk, one lane per stream, one table look-up per
// symbol (Sec. III-B: n look-ups and n small additions for a stream of n weights).  Handles
// every geometry the ABI allows; compressed words are read straight from global memory.
template <int OUT>
__global__ __launch_bounds__(kWave) void decode_stepwise(DecodeParams p) {
    __shared__ uint32_t table[1u << ANSZP_MAX_TABLE_LOG];
    const uint32_t lane = threadIdx.x;
    const uint32_t N = p.n_streams;
    const uint32_t L = 1u << p.table_log;
    const anszp_chunk_t c = p.chunks[blockIdx.x];
    if (!chunk_in_bounds(p, c)) {
        if (lane == 0) report(p.status, ANSZP_ST_BAD_DESC);
        return;
    }
    const uint64_t* src = p.tables + (uint64_t(c.layer_id) << p.table_log);
    for (uint32_t i = lane; i < L; i += kWave) table[i] = static_cast<uint32_t>(src[i]);
    const anszp_layer_t lay = p.layers[c.layer_id];
    __syncthreads();

    const uint32_t hdr = lane < N ? p.stream_hdr[c.stream_offset + lane] : 0u;
    uint32_t X = hdr & (L - 1u);
    const uint32_t n_words = hdr >> 16;
    uint32_t total_words;
    const uint32_t first_word = wave_exclusive_sum(n_words, &total_words);
    const uint32_t len = (lane < N && c.n_symbols > lane) ? (c.n_symbols - lane + N - 1u) / N : 0u;
    uint32_t err = (total_words != c.payload_words) ? ANSZP_ST_BAD_DESC : 0u;

    const uint32_t* words = p.payload + c.payload_offset;
    const uint32_t word_limit = c.payload_words;      // reads beyond the chunk see zeros
    uint32_t next_word = first_word;
    uint64_t buf = 0;
    uint32_t have = 0;
    const uint32_t steps = (c.n_symbols + N - 1u) / N;
    const bool per_channel = lay.channel_len != 0;
    const uint64_t layer_elem0 = c.out_offset - lay.out_base;
    for (uint32_t t = 0; t < steps; ++t) {
        if (t < len) {
            const uint32_t e = table[X];
            const uint32_t nb = (e >> 16) & 0xFFu;
            if (have < nb) {
                const uint32_t w = next_word < word_limit ? words[next_word] : 0u;
                ++next_word;
                buf |= uint64_t(w) << have;
                have += 32;
            }
            const uint32_t bits = static_cast<uint32_t>(buf) & ((1u << nb) - 1u);
            buf >>= nb;
            have -= nb;
            X = ((e & 0xFFFFu) + bits) & (L - 1u);
            const uint64_t j = uint64_t(t) * N + lane;
            float scale = lay.scale;
            if (per_channel) {
                const uint64_t ch = lay.scales_offset + (layer_elem0 + j) / lay.channel_len;
                scale = ch < p.n_scales ? p.scales[ch] : 0.0f;
            }
            store_weight<OUT>(p.out, c.out_offset + j, e >> 24, lay.zero_point, scale);
        }
    }
    if (lane < N) {
        if (X != 0) err |= ANSZP_ST_BAD_STATE;
        if (next_word - first_word != n_words) err |= ANSZP_ST_BAD_LENGTH;
    }
    // one report per chunk
    uint32_t any = err;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) any |= __shfl_xor(any, d, kWave);
    if (any && lane == 0) report(p.status, any);
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

}  // namespace

extern "C" {

int anszp_build_tables(const uint32_t* freqs_host, int n_tables, int table_log,
                       uint64_t* tables_dev, void* hip_stream) {
    if (!freqs_host || !tables_dev) return ANSZP_E_NULL;
    if (table_log < 1 || table_log > ANSZP_MAX_TABLE_LOG || n_tables < 1) return ANSZP_E_RANGE;
    const size_t entries = size_t(n_tables) << table_log;
    uint64_t* staging = nullptr;
    if (hipHostMalloc(reinterpret_cast<void**>(&staging), entries * sizeof(uint64_t), hipHostMallocDefault) != hipSuccess)
        return ANSZP_E_NOMEM;
    int rc = anszp_build_tables_host(freqs_host, n_tables, table_log, staging);
    if (rc == ANSZP_OK) {
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        if (hipMemcpyAsync(tables_dev, staging, entries * sizeof(uint64_t), hipMemcpyHostToDevice, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            rc = ANSZP_E_HIP;
    }
    (void)hipHostFree(staging);
    return rc;
}

int anszp_decode(const anszp_decode_args_t* a, void* hip_stream) {
    if (!a) return ANSZP_E_NULL;
    if (a->n_chunks == 0) return ANSZP_OK;
    if (!a->tables || !a->chunks || !a->stream_hdr || !a->layers || !a->out || !a->status) return ANSZP_E_NULL;
    if (!a->payload && a->payload_words) return ANSZP_E_NULL;
    if (a->table_log < 1 || a->table_log > ANSZP_MAX_TABLE_LOG || a->n_streams < 1 ||
        a->n_streams > ANSZP_MAX_STREAMS || a->out_dtype > ANSZP_OUT_BF16 || a->n_tables == 0 ||
        a->n_chunks >= (1ull << 31) || (reinterpret_cast<uintptr_t>(a->payload) & 15) ||
        (reinterpret_cast<uintptr_t>(a->out) & 15))
        return ANSZP_E_RANGE;
    DecodeParams p;
    p.tables = a->tables; p.chunks = a->chunks; p.stream_hdr = a->stream_hdr; p.payload = a->payload;
    p.layers = a->layers; p.scales = a->scales; p.out = a->out; p.status = a->status;
    p.n_stream_hdr = a->n_stream_hdr; p.payload_words = a->payload_words;
    p.n_scales = a->scales ? a->n_scales : 0; p.out_elems = a->out_elems;
    p.n_tables = a->n_tables; p.table_log = a->table_log; p.n_streams = a->n_streams;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const dim3 grid(static_cast<uint32_t>(a->n_chunks)), block(kWave);
    switch (a->out_dtype) {
        case ANSZP_OUT_U8: hipLaunchKernelGGL(decode_stepwise<ANSZP_OUT_U8>, grid, block, 0, s, p); break;
        case ANSZP_OUT_F32: hipLaunchKernelGGL(decode_stepwise<ANSZP_OUT_F32>, grid, block, 0, s, p); break;
        default: hipLaunchKernelGGL(decode_stepwise<ANSZP_OUT_BF16>, grid, block, 0, s, p); break;
    }
    return hipGetLastError() == hipSuccess ? ANSZP_OK : ANSZP_E_HIP;
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
