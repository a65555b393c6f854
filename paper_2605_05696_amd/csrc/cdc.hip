// Gear-hash content-defined chunking on the GPU (paper Sec. 4, Sec. 7.2, App. B).
//
// The rolling state takes one step per token, h <- (h << 1) + G[id & 0xFF].
// Under a k-bit mask only the last k tokens can reach the masked bits
// (a term shifted k or more times has no bit below 2^k), so
//     h_i & mask == ( sum_{j<k} G[x_{i-j}] << j ) & mask .
// With min_chunk >= k every position at which a cut may be taken has all k
// terms inside its own request, hence the candidate bit of every token can be
// computed independently (kernel 1).  What stays sequential is the greedy
// choice of cuts under the min/max clamps: one wave per request walks the
// candidate bitmap with 64-bit find-first-set over up to 64 words at a time
// (kernel 2).  Kernel 3 turns the per-request lists into the CSR output.
#include "irm_internal.hpp"

#define CDC_SEG_WORDS 4096u   // bitmap words staged in LDS per round: 262,144 tokens, 32 KB

// ---- kernel 1: candidate bit per token -------------------------------------
// bit i of the bitmap is set iff the masked window sum at token i is zero.
// Bits of tokens closer than k-1 to the start of the array use the terms that
// exist; bits within k-1 of a request start mix in the previous request's
// tail, which is harmless: such positions are never eligible (min_chunk >= k).
__global__ __launch_bounds__(256) void cdc_candidates(const int32_t *__restrict__ tokens, uint64_t n_tokens,
                                                      const uint32_t *__restrict__ gear, uint32_t mask,
                                                      uint32_t k_bits, uint64_t *__restrict__ bitmap)
{
    __shared__ uint32_t g[256 + 32];
    const uint64_t block0 = (uint64_t)blockIdx.x * 256;
    const uint32_t tid = threadIdx.x;
    // stage masked gear values of tokens [block0 - 32, block0 + 256)
    for (uint32_t k = tid; k < 256 + 32; k += 256) {
        int64_t i = (int64_t)block0 - 32 + k;
        uint32_t v = 0;
        if (i >= 0 && (uint64_t)i < n_tokens) v = gear[(uint32_t)tokens[i] & 0xFFu] & mask;
        g[k] = v;
    }
    __syncthreads();
    const uint64_t i = block0 + tid;
    uint32_t acc = 0;
    for (uint32_t j = 0; j < k_bits; ++j) acc += g[32 + tid - j] << j;
    const bool cand = (i < n_tokens) && ((acc & mask) == 0);
    const uint64_t word = __ballot(cand);
    if ((tid & 63) == 0 && i < n_tokens) bitmap[i >> 6] = word;   // i is a multiple of 64 here
}

// ---- kernel 2: greedy cut selection, one workgroup per request -------------
__global__ __launch_bounds__(256) void cdc_select(const uint64_t *__restrict__ bitmap,
                                                  const uint32_t *__restrict__ req_offsets,
                                                  uint64_t n_tokens, uint32_t min_chunk, uint32_t max_chunk,
                                                  uint32_t *__restrict__ stage_start,
                                                  uint32_t *__restrict__ stage_len,
                                                  uint32_t *__restrict__ req_count, uint32_t stage_cap,
                                                  uint32_t *err)
{
    __shared__ uint64_t seg[CDC_SEG_WORDS];
    __shared__ uint64_t sh_s, sh_from;
    __shared__ uint32_t sh_count;

    const uint32_t r = blockIdx.x;
    const uint64_t begin = req_offsets[r], end = req_offsets[r + 1];
    if (begin > end || end > n_tokens) {               // malformed offsets: emit nothing
        if (threadIdx.x == 0) {
            req_count[r] = 0;
            atomicOr(err, IRM_FLAG_BAD_CHUNK);
        }
        return;
    }
    const uint64_t base = begin / min_chunk + r;       // this request's staging area
    const uint32_t lane = threadIdx.x & 63;
    const bool walker = threadIdx.x < 64;
    if (threadIdx.x == 0) {
        sh_s = begin;
        sh_from = begin;
        sh_count = 0;
    }
    const uint64_t end_words = (end + 63) >> 6;
    uint64_t w0 = begin >> 6;
    __syncthreads();

    while (sh_s < end) {                               // uniform: read after a barrier
        const uint64_t w1 = (w0 + CDC_SEG_WORDS < end_words) ? w0 + CDC_SEG_WORDS : end_words;
        for (uint64_t w = w0 + threadIdx.x; w < w1; w += blockDim.x) seg[w - w0] = bitmap[w];
        __syncthreads();
        if (walker) {
            const uint64_t avail_end = (w1 << 6) < end ? (w1 << 6) : end;   // bits known below this
            uint64_t s = sh_s, from = sh_from;
            uint32_t count = sh_count;
            while (s < end) {
                const uint64_t first = s + min_chunk - 1;
                const uint64_t lo = first > from ? first : from;
                const uint64_t hard = (s + max_chunk - 1 < end - 1) ? s + max_chunk - 1 : end - 1;
                const uint64_t hi = hard < avail_end - 1 ? hard : avail_end - 1;
                int64_t found = -1;
                if (lo <= hi) {
                    const uint64_t w_lo = lo >> 6, w_hi = hi >> 6;
                    for (uint64_t wb = w_lo; wb <= w_hi; wb += 64) {
                        const uint64_t w = wb + lane;
                        uint64_t word = 0;
                        if (w <= w_hi) {
                            word = seg[w - w0];
                            if (w == w_lo) word &= ~0ull << (lo & 63);
                            if (w == w_hi) word &= (2ull << (hi & 63)) - 1ull;
                        }
                        const uint64_t vote = __ballot(word != 0);
                        if (vote) {
                            const uint32_t f = (uint32_t)__builtin_ctzll(vote);
                            const uint32_t wl = __builtin_amdgcn_readlane((uint32_t)word, f);
                            const uint32_t wh = __builtin_amdgcn_readlane((uint32_t)(word >> 32), f);
                            const uint64_t wf = ((uint64_t)wh << 32) | wl;
                            found = (int64_t)(((wb + f) << 6) + (uint64_t)__builtin_ctzll(wf));
                            break;
                        }
                    }
                }
                uint64_t e;
                if (found >= 0) e = (uint64_t)found;
                else if (hard < avail_end) e = hard;    // searched to the clamp or the request end
                else {                                   // candidate bits past this segment are needed
                    from = avail_end;
                    break;
                }
                if (lane == 0) {
                    if (base + count < stage_cap) {
                        stage_start[base + count] = (uint32_t)s;
                        stage_len[base + count] = (uint32_t)(e - s + 1);
                    } else {
                        atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
                    }
                }
                ++count;
                s = e + 1;
                from = s;
            }
            if (lane == 0) {
                sh_s = s;
                sh_from = from;
                sh_count = count;
            }
        }
        __syncthreads();
        w0 = w1;
        if (w0 >= end_words) break;
    }
    if (threadIdx.x == 0) req_count[r] = sh_count;
}

// ---- kernel 3: per-request lists -> CSR -------------------------------------
__global__ __launch_bounds__(1024) void cdc_compact(const uint32_t *__restrict__ req_offsets, uint32_t n_req,
                                                    uint32_t min_chunk,
                                                    const uint32_t *__restrict__ stage_start,
                                                    const uint32_t *__restrict__ stage_len,
                                                    const uint32_t *__restrict__ req_count, uint32_t stage_cap,
                                                    uint32_t *__restrict__ chunk_start,
                                                    uint32_t *__restrict__ chunk_len,
                                                    uint32_t *__restrict__ req_chunk_offsets,
                                                    uint32_t *__restrict__ n_chunks, uint32_t chunk_capacity,
                                                    uint32_t *err)
{
    __shared__ uint32_t lds[17];
    __shared__ uint32_t carry_sh;
    if (threadIdx.x == 0) carry_sh = 0;
    __syncthreads();
    // exclusive scan of the per-request counts
    for (uint32_t r0 = 0; r0 < n_req; r0 += blockDim.x) {
        const uint32_t r = r0 + threadIdx.x;
        const uint32_t v = r < n_req ? req_count[r] : 0;
        uint32_t total;
        const uint32_t incl = irm_block_scan_incl(v, lds, &total);
        const uint32_t carry = carry_sh;
        if (r < n_req) req_chunk_offsets[r] = carry + incl - v;
        __syncthreads();
        if (threadIdx.x == 0) carry_sh = carry + total;
        __syncthreads();
    }
    const uint32_t total = carry_sh;
    if (threadIdx.x == 0) {
        req_chunk_offsets[n_req] = total;
        *n_chunks = total < chunk_capacity ? total : chunk_capacity;
        if (total > chunk_capacity) atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
    }
    __syncthreads();   // req_chunk_offsets written above are read below by other threads
    __threadfence_block();
    // copy: one wave per request at a time
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n_waves = blockDim.x >> 6;
    for (uint32_t r = wave; r < n_req; r += n_waves) {
        const uint32_t cnt = req_count[r];
        const uint32_t out0 = req_chunk_offsets[r];
        const uint64_t base = (uint64_t)req_offsets[r] / min_chunk + r;
        for (uint32_t j = lane; j < cnt; j += 64) {
            if (out0 + j < chunk_capacity && base + j < stage_cap) {
                chunk_start[out0 + j] = stage_start[base + j];
                chunk_len[out0 + j] = stage_len[base + j];
            }
        }
    }
}

extern "C" irm_status irm_cdc_chunk(irm_ctx *ctx, const int32_t *d_tokens, uint64_t n_tokens,
                                    const uint32_t *d_req_offsets, uint32_t n_req,
                                    uint32_t *d_chunk_start, uint32_t *d_chunk_len,
                                    uint32_t *d_req_chunk_offsets, uint32_t *d_n_chunks,
                                    uint32_t chunk_capacity, void *stream)
{
    if (!ctx || !d_req_offsets || !d_chunk_start || !d_chunk_len || !d_req_chunk_offsets || !d_n_chunks)
        return IRM_ERR_INVALID_ARG;
    if (!d_tokens && n_tokens) return IRM_ERR_INVALID_ARG;
    if (n_req < 1) return IRM_ERR_INVALID_ARG;
    if (n_tokens > ctx->cfg.max_tokens || n_req > ctx->cfg.max_requests) return IRM_ERR_CAPACITY;
    if ((uint64_t)chunk_capacity < irm_chunk_capacity_bound(n_tokens, n_req, ctx->cfg.min_chunk))
        return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const irm_config &c = ctx->cfg;
    if (n_tokens) {
        const uint32_t blocks = (uint32_t)((n_tokens + 255) / 256);
        hipLaunchKernelGGL(cdc_candidates, dim3(blocks), dim3(256), 0, s, d_tokens, n_tokens, ctx->d_gear,
                           c.mask, ctx->k_bits, ctx->d_bitmap);
    }
    hipLaunchKernelGGL(cdc_select, dim3(n_req), dim3(256), 0, s, ctx->d_bitmap, d_req_offsets, n_tokens,
                       c.min_chunk, c.max_chunk, ctx->d_stage_start, ctx->d_stage_len, ctx->d_req_count,
                       ctx->chunk_cap, ctx->d_err);
    hipLaunchKernelGGL(cdc_compact, dim3(1), dim3(1024), 0, s, d_req_offsets, n_req, c.min_chunk,
                       ctx->d_stage_start, ctx->d_stage_len, ctx->d_req_count, ctx->chunk_cap,
                       d_chunk_start, d_chunk_len, d_req_chunk_offsets, d_n_chunks, chunk_capacity,
                       ctx->d_err);
    return irm_launch_status();
}
