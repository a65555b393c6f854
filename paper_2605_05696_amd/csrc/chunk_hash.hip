// Chunk fingerprint: FNV-1a-64 over the little-endian bytes of the token ids
// (paper Sec. 4; Alg. 1 steps 2 and 7).
//
// FNV-1a is a byte-serial chain x <- (x ^ b) * P (mod 2^64), and a chunk is up to
// max_chunk * 4 bytes long, so one lane per chunk would leave the whole pipeline
// waiting for the longest chunk's ~4000 dependent 64-bit multiplies.  The chain
// is split instead:
//
//   * x ^ b only changes the low byte of x, so x ^ b = x + d with
//     d = ((x & 255) ^ b) - (x & 255), and the step becomes the LINEAR recurrence
//     x <- (x + d) * P.  Hence after n bytes
//         x_n = x_0 * P^n + sum_k d_k * P^(n-k),
//     a sum whose terms are independent once the d_k are known.
//   * d_k needs only the low byte l_k of x_k, and because P = 0xB3 (mod 256) the
//     low byte runs its own closed chain  l <- ((l ^ b) * 0xB3) & 255, which costs
//     two cheap 32-bit operations per byte instead of a 64-bit multiply.
//
// One wave per chunk, 1024 tokens at a time: (A) the wave runs the low-byte chain
// over the staged tokens and notes the state at every 16-token segment start;
// (B) lane j re-walks segment j from its noted state, forming the segment's sum
// by Horner's rule in 64-bit arithmetic; (C) each lane weights its sum by the
// power of P that the bytes behind its segment contribute, and a wave reduction
// adds them up.  All of it is exact integer arithmetic: the result is bit-equal
// to the byte-serial definition.
#include "irm_internal.hpp"

#define FNV_BASIS 0xCBF29CE484222325ull
#define FNV_PRIME 0x00000100000001B3ull
#define HASH_BLOCK_TOKENS 1024u
#define HASH_SEG_TOKENS 16u
#define HASH_WAVES 4u

// P^(2^i), i < 16: exponents up to 65535 bytes
__constant__ uint64_t fnv_pow2[16];

static void fill_pow2(uint64_t *t)
{
    uint64_t p = FNV_PRIME;
    for (int i = 0; i < 16; ++i) {
        t[i] = p;
        p *= p;
    }
}

__device__ __forceinline__ uint64_t fnv_pow(uint32_t e)
{
    uint64_t r = 1;
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (e & (1u << i)) r *= fnv_pow2[i];
    return r;
}

// the closed chain of the low byte: four steps for one token (high bits of l are junk)
__device__ __forceinline__ uint32_t low_chain_token(uint32_t l, uint32_t t)
{
    l = __umul24(l ^ t, 0xB3u);
    l = __umul24(l ^ (t >> 8), 0xB3u);
    l = __umul24(l ^ (t >> 16), 0xB3u);
    l = __umul24(l ^ (t >> 24), 0xB3u);
    return l;
}

__global__ __launch_bounds__(HASH_WAVES * 64) void chunk_hash_wave(
    const int32_t *__restrict__ tokens, uint64_t n_tokens, const uint32_t *__restrict__ chunk_start,
    const uint32_t *__restrict__ chunk_len, const uint32_t *__restrict__ n_chunks_p, uint32_t chunk_capacity,
    uint64_t *__restrict__ chunk_hash, uint32_t *err)
{
    __shared__ uint32_t tok_s[HASH_WAVES][HASH_BLOCK_TOKENS];
    __shared__ uint32_t entry_s[HASH_WAVES][HASH_BLOCK_TOKENS / HASH_SEG_TOKENS];

    const uint32_t lane = threadIdx.x & 63, wave = irm_wave_id();
    const uint32_t c = blockIdx.x * HASH_WAVES + wave;
    uint32_t n_chunks = *n_chunks_p;
    if (n_chunks > chunk_capacity) n_chunks = chunk_capacity;
    if (c >= n_chunks) return;                          // whole wave leaves together
    const uint64_t start = chunk_start[c], len = chunk_len[c];
    if (start + len > n_tokens) {
        if (lane == 0) {
            atomicOr(err, IRM_FLAG_BAD_CHUNK);
            chunk_hash[c] = 0;
        }
        return;
    }
    uint32_t *tok = tok_s[wave], *entry = entry_s[wave];
    uint64_t x = FNV_BASIS;                             // state in front of the current block
    for (uint64_t done = 0; done < len; done += HASH_BLOCK_TOKENS) {
        const uint32_t nb = (uint32_t)((len - done < HASH_BLOCK_TOKENS) ? len - done : HASH_BLOCK_TOKENS);
        // stage this block's tokens (wave-private LDS; a wave runs in lockstep)
        for (uint32_t k = lane; k < nb; k += 64) tok[k] = (uint32_t)tokens[start + done + k];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // other lanes' LDS writes are visible
        __builtin_amdgcn_wave_barrier();
        // (A) low-byte chain over the block; every lane walks it, addresses are uniform
        uint32_t l = (uint32_t)x;
        const uint32_t n_seg_full = nb / HASH_SEG_TOKENS;
        for (uint32_t sgm = 0; sgm < n_seg_full; ++sgm) {
            if (lane == 0) entry[sgm] = l & 0xFFu;
            const uint4 *p = (const uint4 *)(tok + sgm * HASH_SEG_TOKENS);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint4 t4 = p[q];
                l = low_chain_token(l, t4.x);
                l = low_chain_token(l, t4.y);
                l = low_chain_token(l, t4.z);
                l = low_chain_token(l, t4.w);
            }
        }
        if (lane == 0 && n_seg_full * HASH_SEG_TOKENS < nb) entry[n_seg_full] = l & 0xFFu;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // (B) lane j: Horner sum of segment j from its entry state
        const uint32_t seg0 = lane * HASH_SEG_TOKENS;
        uint64_t sum = 0;
        uint32_t seg_tokens = 0;
        if (seg0 < nb) {
            seg_tokens = nb - seg0 < HASH_SEG_TOKENS ? nb - seg0 : HASH_SEG_TOKENS;
            uint32_t ls = entry[lane];
            for (uint32_t k = 0; k < seg_tokens; ++k) {
                const uint32_t t = tok[seg0 + k];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t lo = ls & 0xFFu;
                    const uint32_t y = lo ^ ((t >> (8 * b)) & 0xFFu);
                    const int64_t d = (int64_t)(int32_t)(y - lo);
                    sum = (sum + (uint64_t)d) * FNV_PRIME;
                    ls = __umul24(y, 0xB3u);
                }
            }
        }
        // (C) weight by the bytes that follow the segment inside this block, reduce
        const uint32_t after = seg0 < nb ? (nb - seg0 - seg_tokens) * 4u : 0u;
        uint64_t part = sum * fnv_pow(after);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)part, d);
            const uint32_t hi = __shfl_xor((uint32_t)(part >> 32), d);
            part += ((uint64_t)hi << 32) | lo;
        }
        x = x * fnv_pow(nb * 4u) + part;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();                // the next block overwrites tok/entry
    }
    if (lane == 0) chunk_hash[c] = x;
}

static bool g_pow_ready[64];

extern "C" irm_status irm_chunk_hash(irm_ctx *ctx, const int32_t *d_tokens, uint64_t n_tokens,
                                     const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                                     const uint32_t *d_n_chunks, uint32_t chunk_capacity,
                                     uint64_t *d_chunk_hash, void *stream)
{
    if (!ctx || !d_chunk_start || !d_chunk_len || !d_n_chunks || !d_chunk_hash) return IRM_ERR_INVALID_ARG;
    if (!d_tokens && n_tokens) return IRM_ERR_INVALID_ARG;
    if (chunk_capacity < 1) return IRM_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int dev = ctx->device;
    if (dev < 0 || dev >= 64) return IRM_ERR_DEVICE;
    if (!g_pow_ready[dev]) return IRM_ERR_DEVICE;       // irm_ctx_create uploads the table
    const uint32_t blocks = (chunk_capacity + HASH_WAVES - 1) / HASH_WAVES;
    hipLaunchKernelGGL(chunk_hash_wave, dim3(blocks), dim3(HASH_WAVES * 64), 0, s, d_tokens, n_tokens,
                       d_chunk_start, d_chunk_len, d_n_chunks, chunk_capacity, d_chunk_hash, ctx->d_err);
    return irm_launch_status();
}

// called by irm_ctx_create with the context's device current
irm_status irm_chunk_hash_init(int device)
{
    if (device < 0 || device >= 64) return IRM_ERR_DEVICE;
    if (g_pow_ready[device]) return IRM_OK;
    uint64_t t[16];
    fill_pow2(t);
    IRM_HIP_TRY(hipMemcpyToSymbol(HIP_SYMBOL(fnv_pow2), t, sizeof t));
    g_pow_ready[device] = true;
    return IRM_OK;
}
