// Chunk fingerprint: FNV-1a-64 over the little-endian bytes of the token ids
// (paper Sec. 4; Alg. 1 steps 2 and 7).
#include "irm_internal.hpp"

#define FNV_BASIS 0xCBF29CE484222325ull
#define FNV_PRIME 0x00000100000001B3ull

// One lane per chunk, byte-serial.
__global__ __launch_bounds__(64) void chunk_hash_serial(const int32_t *__restrict__ tokens, uint64_t n_tokens,
                                                        const uint32_t *__restrict__ chunk_start,
                                                        const uint32_t *__restrict__ chunk_len,
                                                        const uint32_t *__restrict__ n_chunks_p,
                                                        uint32_t chunk_capacity,
                                                        uint64_t *__restrict__ chunk_hash, uint32_t *err)
{
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t n_chunks = *n_chunks_p;
    if (n_chunks > chunk_capacity) n_chunks = chunk_capacity;
    if (c >= n_chunks) return;
    const uint64_t s = chunk_start[c], len = chunk_len[c];
    if (s + len > n_tokens) {
        atomicOr(err, IRM_FLAG_BAD_CHUNK);
        chunk_hash[c] = 0;
        return;
    }
    uint64_t h = FNV_BASIS;
    for (uint64_t j = 0; j < len; ++j) {
        const uint32_t t = (uint32_t)tokens[s + j];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            h ^= (uint64_t)((t >> (8 * b)) & 0xFFu);
            h *= FNV_PRIME;
        }
    }
    chunk_hash[c] = h;
}

extern "C" irm_status irm_chunk_hash(irm_ctx *ctx, const int32_t *d_tokens, uint64_t n_tokens,
                                     const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                                     const uint32_t *d_n_chunks, uint32_t chunk_capacity,
                                     uint64_t *d_chunk_hash, void *stream)
{
    if (!ctx || !d_chunk_start || !d_chunk_len || !d_n_chunks || !d_chunk_hash) return IRM_ERR_INVALID_ARG;
    if (!d_tokens && n_tokens) return IRM_ERR_INVALID_ARG;
    if (chunk_capacity < 1) return IRM_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t blocks = (chunk_capacity + 63) / 64;
    hipLaunchKernelGGL(chunk_hash_serial, dim3(blocks), dim3(64), 0, s, d_tokens, n_tokens, d_chunk_start,
                       d_chunk_len, d_n_chunks, chunk_capacity, d_chunk_hash, ctx->d_err);
    return irm_launch_status();
}
