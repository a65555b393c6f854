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
// One wave per chunk, 1024 tokens at a time; lane j owns the 16-token (64-byte)
// segment j of the block.
//   (A) entry state of every segment.  The byte chain is a T-function: bit r of
//       (y * 0xB3) is y_r xor a function K_r of the lower bits of y only
//       (y = l ^ b).  So, bit by bit from r = 0, the chain of bit r is a running
//       XOR:  l_{k+1,r} = l_{k,r} ^ b_{k,r} ^ K_{k,r}.  Each lane keeps its 64
//       positions as bit planes (one 64-bit word per bit r) and evaluates K_r for
//       all of them at once with bit-sliced full adders (the product is
//       y + 2y + 16y + 32y + 128y with a 3-bit running carry); the running XOR is
//       a 6-step shift-xor inside the word and a ballot + popcount across lanes.
//       Eight rounds give every lane the exact low byte at its segment start.
//   (B) lane j re-walks segment j from that state, forming the segment's sum by
//       Horner's rule in 64-bit arithmetic;
//   (C) each lane weights its sum by the power of P that the bytes behind its
//       segment contribute, and a wave reduction adds them up.
// All of it is exact integer arithmetic: the result is bit-equal to the
// byte-serial definition.
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

// carry-out of a + b + c on bit planes
__device__ __forceinline__ uint64_t maj3(uint64_t a, uint64_t b, uint64_t c) { return (a & b) | (c & (a | b)); }

// Low byte of the FNV state at the start of this lane's 64-byte segment, given the
// low byte l0 in front of the whole block and the lane's 16 tokens (absent tokens = 0).
__device__ __forceinline__ uint32_t segment_entry_state(const uint32_t (&t)[HASH_SEG_TOKENS], uint32_t l0)
{
    // bit planes of the segment's bytes: bit 4q+i of B[r] = bit r of byte i of token q
    uint64_t B[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < (int)HASH_SEG_TOKENS; ++q) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            // bits r, r+8, r+16, r+24 of the token, gathered into one nibble
            const uint32_t nib = (((t[q] >> r) & 0x01010101u) * 0x10204080u) >> 28;
            B[r] |= (uint64_t)nib << (4 * q);
        }
    }
    const uint32_t lane = threadIdx.x & 63;
    uint64_t Y[8];
    uint64_t c0 = 0, c1 = 0, c2 = 0;                    // running carry of the product, 3 bit planes
    uint32_t entry = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        // K = y_{r-1} + y_{r-4} + y_{r-5} + y_{r-7} + carry  (0..8, planes K0..K3)
        const uint64_t a = r >= 1 ? Y[r - 1] : 0, b = r >= 4 ? Y[r - 4] : 0, c = r >= 5 ? Y[r - 5] : 0;
        const uint64_t d = r >= 7 ? Y[r - 7] : 0;
        const uint64_t s1 = a ^ b ^ c, w2a = maj3(a, b, c);
        const uint64_t K0 = s1 ^ d ^ c0, w2b = maj3(s1, d, c0);
        const uint64_t K1 = w2a ^ w2b ^ c1, w4 = maj3(w2a, w2b, c1);
        const uint64_t K2 = w4 ^ c2, K3 = w4 & c2;
        // running XOR of T = b_r ^ K0 along the chain: exclusive prefix inside the word ...
        uint64_t x = B[r] ^ K0;
        x ^= x << 1;
        x ^= x << 2;
        x ^= x << 4;
        x ^= x << 8;
        x ^= x << 16;
        x ^= x << 32;
        const uint32_t total = (uint32_t)(x >> 63);     // parity of the whole segment
        // ... and across the lanes in front of this one, plus the state in front of the block
        const uint64_t votes = __ballot(total != 0);
        const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(votes >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)votes, 0u));
        const uint32_t run = ((l0 >> r) ^ before) & 1u;
        const uint64_t Lr = (x << 1) ^ (run ? ~0ull : 0ull);
        entry |= (uint32_t)(Lr & 1u) << r;
        const uint64_t y = Lr ^ B[r];
        Y[r] = y;
        // carry for the next bit: (y + K) >> 1
        const uint64_t k0 = y & K0;
        c0 = K1 ^ k0;
        const uint64_t k1 = K1 & k0;
        c1 = K2 ^ k1;
        c2 = K3 ^ (K2 & k1);
    }
    (void)lane;
    return entry;
}

__global__ __launch_bounds__(HASH_WAVES * 64) void chunk_hash_wave(
    const int32_t *__restrict__ tokens, uint64_t n_tokens, const uint32_t *__restrict__ chunk_start,
    const uint32_t *__restrict__ chunk_len, const uint32_t *__restrict__ n_chunks_p, uint32_t chunk_capacity,
    uint64_t *__restrict__ chunk_hash, uint32_t *err)
{
    __shared__ uint32_t tok_s[HASH_WAVES][HASH_BLOCK_TOKENS];

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
    uint32_t *tok = tok_s[wave];
    uint64_t x = FNV_BASIS;                             // state in front of the current block
    for (uint64_t done = 0; done < len; done += HASH_BLOCK_TOKENS) {
        const uint32_t nb = (uint32_t)((len - done < HASH_BLOCK_TOKENS) ? len - done : HASH_BLOCK_TOKENS);
        // stage this block's tokens (wave-private LDS; a wave runs in lockstep)
        for (uint32_t k = lane; k < nb; k += 64) tok[k] = (uint32_t)tokens[start + done + k];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // other lanes' LDS writes are visible
        __builtin_amdgcn_wave_barrier();
        // (A) exact low byte of the state at the start of every segment
        const uint32_t seg0 = lane * HASH_SEG_TOKENS;
        uint32_t t[HASH_SEG_TOKENS];
#pragma unroll
        for (int q = 0; q < (int)HASH_SEG_TOKENS; ++q) t[q] = (seg0 + q < nb) ? tok[seg0 + q] : 0u;
        uint32_t ls = segment_entry_state(t, (uint32_t)x & 0xFFu);
        // (B) lane j: Horner sum of segment j from its entry state
        uint64_t sum = 0;
        uint32_t seg_tokens = 0;
        if (seg0 < nb) {
            seg_tokens = nb - seg0 < HASH_SEG_TOKENS ? nb - seg0 : HASH_SEG_TOKENS;
#pragma unroll
            for (uint32_t k = 0; k < HASH_SEG_TOKENS; ++k) {
                if (k >= seg_tokens) break;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t lo = ls & 0xFFu;
                    const uint32_t y = lo ^ ((t[k] >> (8 * b)) & 0xFFu);
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
        __builtin_amdgcn_wave_barrier();                // the next block overwrites tok
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
