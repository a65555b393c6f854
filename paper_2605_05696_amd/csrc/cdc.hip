// Gear-hash content-defined chunking on the GPU (paper Sec. 4, Sec. 7.2, App. B).
//
// The rolling state takes one step per token, h <- (h << 1) + G[id & 0xFF].
// Under a k-bit mask only the last k tokens can reach the masked bits
// (a term shifted k or more times has no bit below 2^k), so
//     h_i & mask == ( sum_{j<k} G[x_{i-j}] << j ) & mask .
// With min_chunk >= k every position at which a cut may be taken has all k
// terms inside its own request, hence the candidate bit of every token can be
// computed independently (kernel 1).  What stays sequential by definition is the
// greedy choice of cuts under the min/max clamps (kernel 2): it is resolved by
// pointer doubling over the candidate positions, with a serial walk of the bitmap
// as the fallback for requests with very many candidates.  The workgroup that
// finishes last turns the per-request lists into the CSR output.
#include "irm_internal.hpp"

#define CDC_SEG_WORDS 4096u   // bitmap words staged in LDS per round: 262,144 tokens, 32 KB

// a value every lane holds identically, moved to scalar registers
__device__ __forceinline__ uint64_t rfl64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// ---- kernel 1: candidate bit per token -------------------------------------
// bit i of the bitmap is set iff the masked window sum at token i is zero.
// Bits of tokens closer than k-1 to the start of the array use the terms that
// exist; bits within k-1 of a request start mix in the previous request's
// tail, which is harmless: such positions are never eligible (min_chunk >= k).
__device__ __forceinline__ void candidates_block(const int32_t *__restrict__ tokens, uint64_t n_tokens,
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

__global__ __launch_bounds__(256) void cdc_candidates(const int32_t *__restrict__ tokens, uint64_t n_tokens,
                                                      const uint32_t *__restrict__ gear, uint32_t mask,
                                                      uint32_t k_bits, uint64_t *__restrict__ bitmap)
{
    candidates_block(tokens, n_tokens, gear, mask, k_bits, bitmap);
}

// ---- kernel 2, serial path: one wave walks the bitmap, one step per chunk ----
// Token positions fit 32 bits (the context caps max_tokens below 2^32 - 65536 - 16, so
// s + max_chunk never wraps).  The walker's state is wave-uniform and kept in 32-bit
// scalars on purpose: 64-bit unsigned compares have no scalar form on this ISA and
// every vector compare feeding a scalar branch costs tens of nanoseconds.
__device__ __forceinline__ void select_serial(const uint64_t *__restrict__ bitmap, uint64_t *seg,
                                              uint32_t r, uint32_t begin, uint32_t end, uint32_t base,
                                              uint32_t min_chunk, uint32_t max_chunk,
                                              uint32_t *__restrict__ stage_start,
                                              uint32_t *__restrict__ stage_len,
                                              uint32_t *__restrict__ req_count, uint32_t stage_cap,
                                              uint32_t *err)
{
    __shared__ uint32_t sh_s, sh_from, sh_count;
    const uint32_t lane = threadIdx.x & 63;
    const bool walker = threadIdx.x < 64;
    if (threadIdx.x == 0) {
        sh_s = begin;
        sh_from = begin;
        sh_count = 0;
    }
    const uint32_t end_words = (uint32_t)(((uint64_t)end + 63) >> 6);
    uint32_t w0 = begin >> 6;
    __syncthreads();

    while ((uint32_t)__builtin_amdgcn_readfirstlane(sh_s) < end) {   // uniform: read after a barrier
        const uint32_t w1 = (end_words - w0 > CDC_SEG_WORDS) ? w0 + CDC_SEG_WORDS : end_words;
        for (uint32_t w = w0 + threadIdx.x; w < w1; w += blockDim.x) seg[w - w0] = bitmap[w];
        __syncthreads();
        if (walker) {
            // candidate bits are known for positions below avail_end
            const uint32_t avail_end = ((uint64_t)w1 << 6) < (uint64_t)end ? (w1 << 6) : end;
            uint32_t s = __builtin_amdgcn_readfirstlane(sh_s);
            uint32_t from = __builtin_amdgcn_readfirstlane(sh_from);
            uint32_t count = __builtin_amdgcn_readfirstlane(sh_count);
            while (s < end) {
                const uint32_t first = s + min_chunk - 1;
                const uint32_t lo = first > from ? first : from;
                const uint32_t hard = (end - s > max_chunk) ? s + max_chunk - 1 : end - 1;
                const uint32_t hi = hard < avail_end ? hard : avail_end - 1;
                uint32_t e = 0;
                bool found = false;
                if (lo <= hi) {
                    const uint32_t w_lo = lo >> 6, w_hi = hi >> 6;
                    for (uint32_t wb = w_lo; wb <= w_hi; wb += 64) {
                        const uint32_t w = wb + lane;
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
                            const uint32_t bit = wl ? (uint32_t)__builtin_ctz(wl) : 32u + (uint32_t)__builtin_ctz(wh);
                            e = ((wb + f) << 6) + bit;
                            found = true;
                            break;
                        }
                    }
                }
                if (!found) {
                    if (hard < avail_end) e = hard;     // searched to the clamp or the request end
                    else {                              // candidate bits past this segment are needed
                        from = avail_end;
                        break;
                    }
                }
                if (lane == 0) {
                    if (base + count < stage_cap) {
                        stage_start[base + count] = s;
                        stage_len[base + count] = e - s + 1;
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

// ---- kernel 2, parallel path -------------------------------------------------
// The chain of cuts only ever stops at candidate positions, at forced cuts
// (max_chunk reached) and at the request's end.  Take the candidates of the request
// as nodes (in position order, node 0 = "just before the request").  For every node
// the next candidate cut the chain would take from there, and the number of
// non-candidate cuts on the way, depend on that node alone, so all of them are
// computed at once; the chain itself is then the orbit of node 0, marked by pointer
// doubling in ceil(log2(nodes)) rounds instead of one step per chunk.
#define CDC_NODE_CAP 4096u

struct cdc_jump_mem {
    uint32_t pos[CDC_NODE_CAP];        // candidate positions, ascending
    uint32_t extra[CDC_NODE_CAP + 2];  // non-candidate cuts between a node and its successor
    uint32_t offset[CDC_NODE_CAP + 2]; // first chunk a marked node emits
    uint16_t jump[CDC_NODE_CAP + 2];
    uint8_t mark[CDC_NODE_CAP + 2];
};

// first index j in pos[0..m) with pos[j] >= target
__device__ __forceinline__ uint32_t cdc_lower_bound(const uint32_t *pos, uint32_t m, uint32_t target)
{
    uint32_t lo = 0, hi = m;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (pos[mid] < target) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Follow the chain from a chunk start s to the next candidate cut.  Returns the node
// of that cut (1-based), or m + 1 when the request ends first; *extra counts the
// forced / tail cuts passed.  With `emit`, every chunk on the way is written out.
template <bool EMIT>
__device__ __forceinline__ uint32_t cdc_advance(const uint32_t *pos, uint32_t m, uint32_t s, uint32_t end,
                                                uint32_t min_chunk, uint32_t max_chunk, uint32_t *extra,
                                                uint32_t *stage_start, uint32_t *stage_len, uint32_t out,
                                                uint32_t stage_cap)
{
    uint32_t n_extra = 0;
    while (s < end) {
        const uint32_t hard = (end - s > max_chunk) ? s + max_chunk - 1 : end - 1;
        const uint32_t j = cdc_lower_bound(pos, m, s + min_chunk - 1);
        const bool hit = j < m && pos[j] <= hard;
        const uint32_t e = hit ? pos[j] : hard;
        if (EMIT && out < stage_cap) {
            stage_start[out] = s;
            stage_len[out] = e - s + 1;
        }
        ++out;
        if (hit) {
            *extra = n_extra;
            return j + 1;
        }
        ++n_extra;
        s = e + 1;
    }
    *extra = n_extra;
    return m + 1;
}

// returns false (having written nothing) when the request has too many candidates
__device__ __forceinline__ bool select_jump(const uint64_t *__restrict__ bitmap, cdc_jump_mem *g,
                                            uint32_t *scan_lds, uint32_t r, uint32_t begin, uint32_t end,
                                            uint32_t base, uint32_t min_chunk, uint32_t max_chunk,
                                            uint32_t *__restrict__ stage_start,
                                            uint32_t *__restrict__ stage_len,
                                            uint32_t *__restrict__ req_count, uint32_t stage_cap,
                                            uint32_t *err)
{
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    // 1. candidates at eligible positions [begin + min - 1, end), ordered compaction
    const uint32_t first_pos = begin + min_chunk - 1;
    uint32_t m = 0;
    if (first_pos < end) {
        const uint32_t w_lo = first_pos >> 6, w_hi = (end - 1) >> 6;
        const uint32_t n_words = w_hi - w_lo + 1;
        const uint32_t per = (n_words + nthr - 1) / nthr;
        const uint32_t my0 = w_lo + tid * per;
        uint32_t cnt = 0;
        for (uint32_t k = 0; k < per; ++k) {
            const uint32_t w = my0 + k;
            if (w > w_hi) break;
            uint64_t word = bitmap[w];
            if (w == w_lo) word &= ~0ull << (first_pos & 63);
            if (w == w_hi) word &= (2ull << ((end - 1) & 63)) - 1ull;
            cnt += (uint32_t)__builtin_popcountll(word);
        }
        uint32_t total;
        const uint32_t incl = irm_block_scan_incl(cnt, scan_lds, &total);
        m = total;
        if (m > CDC_NODE_CAP) return false;             // uniform: every thread sees the same total
        uint32_t o = incl - cnt;
        for (uint32_t k = 0; k < per; ++k) {
            const uint32_t w = my0 + k;
            if (w > w_hi) break;
            uint64_t word = bitmap[w];
            if (w == w_lo) word &= ~0ull << (first_pos & 63);
            if (w == w_hi) word &= (2ull << ((end - 1) & 63)) - 1ull;
            while (word) {
                g->pos[o++] = (w << 6) + (uint32_t)__builtin_ctzll(word);
                word &= word - 1;
            }
        }
    }
    __syncthreads();
    // 2. successor of every node: node 0 starts at `begin`, node i > 0 right after pos[i-1]
    const uint32_t n_nodes = m + 1, term = m + 1;
    for (uint32_t i = tid; i < n_nodes; i += nthr) {
        const uint32_t s = i ? g->pos[i - 1] + 1 : begin;
        uint32_t ex;
        const uint32_t nx = cdc_advance<false>(g->pos, m, s, end, min_chunk, max_chunk, &ex, nullptr, nullptr,
                                               0, 0);
        g->jump[i] = (uint16_t)nx;
        g->extra[i] = ex + (nx != term ? 1u : 0u);      // chunks this node emits when it is on the chain
        g->mark[i] = i == 0 && begin < end;
    }
    if (tid == 0) {
        g->jump[term] = (uint16_t)term;
        g->mark[term] = 0;
        g->extra[term] = 0;
    }
    __syncthreads();
    // 3. orbit of node 0 by pointer doubling
    constexpr int NODE_ITERS = (CDC_NODE_CAP + 2 + 255) / 256;   // nodes per thread at 256 threads
    const uint32_t node_iters = (n_nodes + 255u) >> 8;           // ... of which this request needs so many (uniform)
    for (uint32_t span = 1; span < n_nodes; span <<= 1) {
        uint32_t j1[NODE_ITERS], j2[NODE_ITERS];
#pragma unroll
        for (int k = 0; k < NODE_ITERS; ++k) {
            if ((uint32_t)k >= node_iters) break;                // a typical request has a few hundred nodes: one pass
            const uint32_t i = tid + (uint32_t)k * 256u;
            if (i < n_nodes) {
                j1[k] = g->jump[i];
                j2[k] = g->jump[j1[k]];
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < NODE_ITERS; ++k) {
            if ((uint32_t)k >= node_iters) break;
            const uint32_t i = tid + (uint32_t)k * 256u;
            if (i < n_nodes) {
                if (g->mark[i]) g->mark[j1[k]] = 1;
                g->jump[i] = (uint16_t)j2[k];
            }
        }
        __syncthreads();
    }
    // 4. chunk offsets of the marked nodes (block-ranged scan keeps position order), emit
    const uint32_t per_n = (n_nodes + nthr - 1) / nthr;
    const uint32_t n0 = tid * per_n;
    uint32_t cnt = 0;
    for (uint32_t k = 0; k < per_n; ++k) {
        const uint32_t i = n0 + k;
        if (i < n_nodes && g->mark[i]) cnt += g->extra[i];
    }
    uint32_t total;
    const uint32_t incl = irm_block_scan_incl(cnt, scan_lds, &total);
    uint32_t o = incl - cnt;
    for (uint32_t k = 0; k < per_n; ++k) {
        const uint32_t i = n0 + k;
        if (i < n_nodes && g->mark[i]) {
            const uint32_t s = i ? g->pos[i - 1] + 1 : begin;
            uint32_t ex;
            (void)cdc_advance<true>(g->pos, m, s, end, min_chunk, max_chunk, &ex, stage_start, stage_len,
                                    base + o, stage_cap);
            o += g->extra[i];
        }
    }
    if (tid == 0) {
        req_count[r] = total;
        if (base + total > stage_cap) atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
    }
    return true;
}

// ---- per-request lists -> CSR (run by the workgroup that finishes last) ------
__device__ __forceinline__ void cdc_compact(const uint32_t *__restrict__ req_offsets, uint32_t n_req,
                                            uint32_t min_chunk, const uint32_t *stage_start,
                                            const uint32_t *stage_len, const uint32_t *req_count,
                                            uint32_t stage_cap, uint32_t *__restrict__ chunk_start,
                                            uint32_t *__restrict__ chunk_len,
                                            uint32_t *__restrict__ req_chunk_offsets,
                                            uint32_t *__restrict__ n_chunks, uint32_t chunk_capacity,
                                            uint32_t *lds, uint32_t *err)
{
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

// ---- kernel 2: greedy cut selection, one workgroup per request -------------
// The workgroup that finishes last (ticket counter in the context, left at zero again)
// gathers the per-request lists into the caller's CSR arrays.
struct cdc_select_mem {
    union {
        uint64_t seg[CDC_SEG_WORDS];
        cdc_jump_mem g;
    } sm;
    uint32_t scan_lds[17];
};

// cuts of request r.  `direct` (a batch of one request): its list is the result, written in
// place, no staging and nothing to gather afterwards.
__device__ __forceinline__ void select_request(cdc_select_mem *m, const uint64_t *__restrict__ bitmap,
                                               const uint32_t *__restrict__ req_offsets, uint32_t r, bool direct,
                                               uint64_t n_tokens, uint32_t min_chunk, uint32_t max_chunk,
                                               uint32_t *stage_start, uint32_t *stage_len, uint32_t *req_count,
                                               uint32_t stage_cap, uint32_t force_serial,
                                               uint32_t *__restrict__ chunk_start, uint32_t *__restrict__ chunk_len,
                                               uint32_t *__restrict__ req_chunk_offsets,
                                               uint32_t *__restrict__ n_chunks, uint32_t chunk_capacity, uint32_t *err)
{
    const uint32_t begin = req_offsets[r], end = req_offsets[r + 1];
    if (begin > end || (uint64_t)end > n_tokens) {     // malformed offsets: emit nothing
        if (threadIdx.x == 0) {
            req_count[r] = 0;
            atomicOr(err, IRM_FLAG_BAD_CHUNK);
        }
    } else {
        const uint32_t base = direct ? 0u : begin / min_chunk + r;   // this request's staging area
        uint32_t *out_start = direct ? chunk_start : stage_start, *out_len = direct ? chunk_len : stage_len;
        const uint32_t out_cap = direct ? chunk_capacity : stage_cap;
        if (force_serial || !select_jump(bitmap, &m->sm.g, m->scan_lds, r, begin, end, base, min_chunk, max_chunk,
                                         out_start, out_len, req_count, out_cap, err)) {
            __syncthreads();
            select_serial(bitmap, m->sm.seg, r, begin, end, base, min_chunk, max_chunk, out_start, out_len,
                          req_count, out_cap, err);
        }
    }
    if (direct && threadIdx.x == 0) {                  // thread 0 wrote req_count[0] itself
        const uint32_t total = req_count[0];
        req_chunk_offsets[0] = 0;
        req_chunk_offsets[1] = total;
        *n_chunks = total < chunk_capacity ? total : chunk_capacity;
    }
}

// ---- kernel 2: greedy cut selection, one workgroup per request -------------
// The workgroup that finishes last (ticket counter in the context, left at zero again)
// gathers the per-request lists into the caller's CSR arrays.
__global__ __launch_bounds__(256) void cdc_select(const uint64_t *__restrict__ bitmap,
                                                  const uint32_t *__restrict__ req_offsets, uint32_t n_req,
                                                  uint64_t n_tokens, uint32_t min_chunk, uint32_t max_chunk,
                                                  uint32_t *stage_start, uint32_t *stage_len,
                                                  uint32_t *req_count, uint32_t stage_cap,
                                                  uint32_t force_serial, uint32_t *__restrict__ chunk_start,
                                                  uint32_t *__restrict__ chunk_len,
                                                  uint32_t *__restrict__ req_chunk_offsets,
                                                  uint32_t *__restrict__ n_chunks, uint32_t chunk_capacity,
                                                  uint32_t *tickets, uint32_t *err)
{
    __shared__ cdc_select_mem m;
    __shared__ uint32_t last_sh;
    const bool direct = n_req == 1;
    select_request(&m, bitmap, req_offsets, blockIdx.x, direct, n_tokens, min_chunk, max_chunk, stage_start,
                   stage_len, req_count, stage_cap, force_serial, chunk_start, chunk_len, req_chunk_offsets,
                   n_chunks, chunk_capacity, err);
    if (direct) return;
    // publish this request's list, then take a ticket
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) last_sh = atomicAdd(tickets, 1u) == n_req - 1 ? 1u : 0u;
    __syncthreads();
    if (!last_sh) return;
    __threadfence();                                   // see every other workgroup's list
    cdc_compact(req_offsets, n_req, min_chunk, stage_start, stage_len, req_count, stage_cap, chunk_start,
                chunk_len, req_chunk_offsets, n_chunks, chunk_capacity, m.scan_lds, err);
    if (threadIdx.x == 0) *tickets = 0;
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
    hipLaunchKernelGGL(cdc_select, dim3(n_req), dim3(256), 0, s, ctx->d_bitmap, d_req_offsets, n_req, n_tokens,
                       c.min_chunk, c.max_chunk, ctx->d_stage_start, ctx->d_stage_len, ctx->d_req_count,
                       ctx->chunk_cap, ctx->cdc_serial, d_chunk_start, d_chunk_len, d_req_chunk_offsets,
                       d_n_chunks, chunk_capacity, ctx->d_plan + 1, ctx->d_err);
    return irm_launch_status();
}
