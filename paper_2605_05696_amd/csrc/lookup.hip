// Registry probe with first-chunk carve-out and ordered hit compaction
// (paper Alg. 1 steps 4-8; Sec. 7.1).
#include "irm_internal.hpp"

// keep the hits, in chunk order (run by the workgroup that finishes last)
__device__ __forceinline__ void lookup_compact(const irm_hit *hit_tmp, uint32_t n_chunks,
                                               irm_hit *__restrict__ hits, uint32_t *__restrict__ n_hits,
                                               uint64_t *__restrict__ hit_tokens)
{
    __shared__ uint32_t lds[17];
    __shared__ uint32_t lds2[17];
    uint32_t carry = 0;
    uint64_t tokens = 0;
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += blockDim.x) {
        const uint32_t c = c0 + threadIdx.x;
        irm_hit h = {0u, 0u, 0u, 0};
        if (c < n_chunks) h = hit_tmp[c];
        const uint32_t flag = h.len != 0 ? 1u : 0u;
        uint32_t total, total_len;
        const uint32_t incl = irm_block_scan_incl(flag, lds, &total);
        (void)irm_block_scan_incl(h.len, lds2, &total_len);
        if (flag) hits[carry + incl - 1] = h;
        carry += total;
        tokens += total_len;
    }
    if (threadIdx.x == 0) {
        *n_hits = carry;
        *hit_tokens = tokens;
    }
}

__device__ __forceinline__ void probe_one(const uint64_t *__restrict__ keys, const irm_entry *__restrict__ vals,
                                          uint64_t n_slots, const uint64_t *__restrict__ chunk_hash,
                                          const uint32_t *__restrict__ chunk_start,
                                          const uint32_t *__restrict__ chunk_len,
                                          const uint32_t *__restrict__ req_chunk_offsets,
                                          const uint32_t *__restrict__ req_offsets,
                                          const int32_t *__restrict__ pos_base, uint32_t n_req,
                                          uint32_t carve_out, uint32_t c, int32_t *__restrict__ chunk_entry,
                                          irm_hit *hit_tmp);

// one lane per chunk: position, carve-out, linear probe, length guard
__global__ __launch_bounds__(256) void lookup_probe(const uint64_t *__restrict__ keys,
                                                    const irm_entry *__restrict__ vals, uint64_t n_slots,
                                                    const uint64_t *__restrict__ chunk_hash,
                                                    const uint32_t *__restrict__ chunk_start,
                                                    const uint32_t *__restrict__ chunk_len,
                                                    const uint32_t *__restrict__ req_chunk_offsets,
                                                    const uint32_t *__restrict__ req_offsets,
                                                    const int32_t *__restrict__ pos_base, uint32_t n_req,
                                                    const uint32_t *__restrict__ n_chunks_p,
                                                    uint32_t chunk_capacity, uint32_t carve_out,
                                                    int32_t *__restrict__ chunk_entry, irm_hit *hit_tmp,
                                                    irm_hit *__restrict__ hits,
                                                    uint32_t *__restrict__ n_hits,
                                                    uint64_t *__restrict__ hit_tokens, uint32_t *tickets)
{
    __shared__ uint32_t last_sh;
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t n_chunks = *n_chunks_p;
    if (n_chunks > chunk_capacity) n_chunks = chunk_capacity;
    if (c < n_chunks) probe_one(keys, vals, n_slots, chunk_hash, chunk_start, chunk_len, req_chunk_offsets,
                                req_offsets, pos_base, n_req, carve_out, c, chunk_entry, hit_tmp);
    if (gridDim.x == 1) {
        // the only workgroup reads back what it wrote itself: no device-wide fence, no ticket
        __threadfence_block();
        __syncthreads();
        lookup_compact(hit_tmp, n_chunks, hits, n_hits, hit_tokens);
        return;
    }
    // publish, take a ticket; the last workgroup compacts and leaves the counter at zero
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) last_sh = atomicAdd(tickets, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (!last_sh) return;
    __threadfence();
    lookup_compact(hit_tmp, n_chunks, hits, n_hits, hit_tokens);
    if (threadIdx.x == 0) *tickets = 0;
}

__device__ __forceinline__ void probe_one(const uint64_t *__restrict__ keys, const irm_entry *__restrict__ vals,
                                          uint64_t n_slots, const uint64_t *__restrict__ chunk_hash,
                                          const uint32_t *__restrict__ chunk_start,
                                          const uint32_t *__restrict__ chunk_len,
                                          const uint32_t *__restrict__ req_chunk_offsets,
                                          const uint32_t *__restrict__ req_offsets,
                                          const int32_t *__restrict__ pos_base, uint32_t n_req,
                                          uint32_t carve_out, uint32_t c, int32_t *__restrict__ chunk_entry,
                                          irm_hit *hit_tmp)
{
    const uint32_t start = chunk_start[c], len = chunk_len[c];
    const int64_t pos = irm_chunk_pos(req_chunk_offsets, req_offsets, pos_base, n_req, c, start);
    irm_hit out = {0u, start, 0u, 0};
    int32_t entry = -1;
    if (pos >= (int64_t)carve_out && len != 0) {
        const uint64_t key = chunk_hash[c];
        uint64_t s = n_slots;                        // key 0 lives in the reserved slot
        bool present = false;
        if (key == 0) {
            present = vals[s].len != 0;
        } else {
            s = irm_slot_of(key, n_slots);
            for (uint64_t tries = 0; tries < n_slots; ++tries) {
                const uint64_t k = keys[s];
                if (k == key) { present = true; break; }
                if (k == 0) break;
                s = (s + 1 == n_slots) ? 0 : s + 1;
            }
        }
        if (present) {
            const irm_entry e = vals[s];
            if (e.len == len) {
                entry = (int32_t)e.entry_id;
                out.src_row = e.src_row;
                out.len = len;
                out.delta = (int32_t)(pos - (int64_t)e.p_src);
            }
        }
    }
    chunk_entry[c] = entry;
    hit_tmp[c] = out;
}

extern "C" irm_status irm_lookup(irm_ctx *ctx, const irm_table *table, const uint64_t *d_chunk_hash,
                                 const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                                 const uint32_t *d_req_chunk_offsets, const uint32_t *d_req_offsets,
                                 const int32_t *d_pos_base, uint32_t n_req, const uint32_t *d_n_chunks,
                                 uint32_t chunk_capacity, int32_t *d_chunk_entry, irm_hit *d_hits,
                                 uint32_t *d_n_hits, uint64_t *d_hit_tokens, void *stream)
{
    if (!ctx || !table || !d_chunk_hash || !d_chunk_start || !d_chunk_len || !d_req_chunk_offsets ||
        !d_req_offsets || !d_pos_base || !d_n_chunks || !d_chunk_entry || !d_hits || !d_n_hits ||
        !d_hit_tokens)
        return IRM_ERR_INVALID_ARG;
    if (n_req < 1 || chunk_capacity < 1) return IRM_ERR_INVALID_ARG;
    if (table->ctx != ctx) return IRM_ERR_INVALID_ARG;
    if (n_req > ctx->cfg.max_requests || chunk_capacity > ctx->chunk_cap) return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t blocks = (chunk_capacity + 255) / 256;
    hipLaunchKernelGGL(lookup_probe, dim3(blocks), dim3(256), 0, s, table->d_keys, table->d_vals,
                       table->n_slots, d_chunk_hash, d_chunk_start, d_chunk_len, d_req_chunk_offsets,
                       d_req_offsets, d_pos_base, n_req, d_n_chunks, chunk_capacity, ctx->cfg.carve_out,
                       d_chunk_entry, ctx->d_hit_tmp, d_hits, d_n_hits, d_hit_tokens, ctx->d_plan + 2);
    return irm_launch_status();
}
