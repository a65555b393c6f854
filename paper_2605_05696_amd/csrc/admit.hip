// Miss path (paper Alg. 1 steps 11-13): chunks the lookup missed have been prefilled by
// the engine into the request's slots; copy their rows into fresh rows of the shared
// pool and register hash -> (rows, p, len), insert-if-absent.
//
//   admit_claim   one lane per chunk: an eligible chunk (missed, past the carve-out)
//                 claims the table slot of its hash (64-bit CAS) and bids for it with
//                 its rank (atomicMin), so among equal hashes the lowest chunk wins and
//                 a hash registered earlier always wins.  The workgroup that finishes
//                 last then walks the chunks in order: winners get consecutive pool rows
//                 from the cursor (ordered scan), the first one that does not fit closes
//                 the pool for the batch; it writes the registry values, the per-chunk
//                 result, the new cursor and the copy tiles.
//   admit_rows    grid (tile slots, layers): 16 rows of 72 16-byte vectors per tile,
//                 gathered through the slot map, written to consecutive pool rows.
#include "irm_internal.hpp"

#define ADMIT_TILE_ROWS 16u
#define ADMIT_NONE 0xFFFFFFFFu

__global__ __launch_bounds__(256) void admit_claim(
    uint64_t *keys, uint32_t *owner, irm_entry *vals, uint64_t n_slots, uint32_t *state,
    const uint64_t *__restrict__ chunk_hash, const uint32_t *__restrict__ chunk_start,
    const uint32_t *__restrict__ chunk_len, const uint32_t *__restrict__ req_chunk_offsets,
    const uint32_t *__restrict__ req_offsets, const int32_t *__restrict__ pos_base, uint32_t n_req,
    const uint32_t *__restrict__ n_chunks_p, uint32_t chunk_capacity, uint32_t carve_out,
    const int32_t *__restrict__ chunk_entry, uint64_t n_slot_tokens, uint64_t pool_rows, uint32_t *cursor,
    int32_t *__restrict__ admitted_row, uint32_t *slot_of, irm_tile *__restrict__ tiles, uint32_t tile_cap,
    uint32_t *plan, uint32_t *tickets, uint32_t *err)
{
    __shared__ uint32_t last_sh, admitted_rows_sh, tile_carry_sh;
    __shared__ uint64_t run_rows_sh;
    __shared__ uint32_t lds[17], lds2[17];
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t n_chunks = *n_chunks_p;
    if (n_chunks > chunk_capacity) n_chunks = chunk_capacity;
    // rank base of this batch's bids (see table_claim); the last workgroup advances it
    const uint32_t rank0 = state[0];
    const bool room = rank0 <= 0xFFFFFFFEu - chunk_capacity;
    if (!room && c == 0) atomicOr(err, IRM_FLAG_TABLE_FULL);
    if (c < n_chunks) {
        uint32_t mine = ADMIT_NONE;
        const uint32_t start = chunk_start[c], len = chunk_len[c];
        const int64_t pos = irm_chunk_pos(req_chunk_offsets, req_offsets, pos_base, n_req, c, start);
        if (room && chunk_entry[c] < 0 && pos >= (int64_t)carve_out && len != 0) {
            if ((uint64_t)start + len > n_slot_tokens) {
                atomicOr(err, IRM_FLAG_BAD_CHUNK);
            } else {
                const uint64_t s = irm_claim_slot(keys, n_slots, chunk_hash[c]);
                if (s > n_slots) {
                    atomicOr(err, IRM_FLAG_TABLE_FULL);
                } else {
                    atomicMin(&owner[s], rank0 + c);
                    mine = (uint32_t)s;
                }
            }
        }
        slot_of[c] = mine;
    }
    // publish the bids, take a ticket; the last workgroup allocates
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) last_sh = atomicAdd(tickets, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (!last_sh) return;
    __threadfence();
    // Winners in chunk order get consecutive rows from the cursor.  The running sum counts
    // every winner, so once one of them does not fit, no later one does either: the first
    // misfit closes the pool for the batch, exactly like a sequential walk would.
    if (threadIdx.x == 0) {
        run_rows_sh = *cursor;
        admitted_rows_sh = 0;
        tile_carry_sh = 0;
    }
    __syncthreads();
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += blockDim.x) {
        const uint32_t k = c0 + threadIdx.x;
        uint32_t len = 0, s = ADMIT_NONE;
        bool winner = false;
        if (k < n_chunks) {
            s = slot_of[k];
            len = chunk_len[k];
            winner = s != ADMIT_NONE && owner[s] == rank0 + k;   // lowest bid, and nobody held the hash before
        }
        uint32_t total_rows, total_tiles, total_admitted;
        const uint32_t rows_incl = irm_block_scan_incl(winner ? len : 0u, lds, &total_rows);
        const uint64_t row0 = run_rows_sh + (uint64_t)(rows_incl - (winner ? len : 0u));
        const bool admitted = winner && row0 + len <= pool_rows;
        const uint32_t nt = admitted ? (len + ADMIT_TILE_ROWS - 1) / ADMIT_TILE_ROWS : 0u;
        const uint32_t tiles_incl = irm_block_scan_incl(nt, lds2, &total_tiles);
        (void)irm_block_scan_incl(admitted ? len : 0u, lds, &total_admitted);
        if (k < n_chunks) admitted_row[k] = admitted ? (int32_t)row0 : -1;
        if (winner && !admitted) owner[s] = ADMIT_NONE;      // give the hash back: a later batch may admit it
        if (admitted) {
            const uint32_t start = chunk_start[k];
            irm_entry e;
            e.src_row = (uint32_t)row0;
            e.p_src = (int32_t)irm_chunk_pos(req_chunk_offsets, req_offsets, pos_base, n_req, k, start);
            e.len = len;
            e.entry_id = (uint32_t)row0;
            vals[s] = e;
            uint32_t t = tile_carry_sh + tiles_incl - nt;
            for (uint32_t q = 0; q < nt; ++q, ++t) {
                if (t >= tile_cap) {
                    atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
                    break;
                }
                const uint32_t done = q * ADMIT_TILE_ROWS;
                irm_tile tile;
                tile.src_row0 = (uint32_t)row0 + done;       // destination: pool row
                tile.dst_tok0 = start + done;                // source: token index -> slot
                tile.n_rows = len - done < ADMIT_TILE_ROWS ? len - done : ADMIT_TILE_ROWS;
                tile.hit = k;
                tiles[t] = tile;
            }
        }
        __syncthreads();                                     // all reads of the carries are done
        if (threadIdx.x == 0) {
            run_rows_sh += total_rows;
            admitted_rows_sh += total_admitted;
            tile_carry_sh += total_tiles;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *cursor = *cursor + admitted_rows_sh;
        if (room) state[0] = rank0 + chunk_capacity;
        plan[0] = tile_carry_sh < tile_cap ? tile_carry_sh : tile_cap;
        *tickets = 0;
    }
}

// VPR: 16-byte vectors per row (72 for bf16 rows, 41 for fp8 rows)
template <uint32_t VPR>
__global__ __launch_bounds__(256) void admit_rows(const void *const *__restrict__ req_ptrs, uint64_t req_stride,
                                                  uint64_t req_rows, void *const *__restrict__ pool_ptrs,
                                                  uint64_t pool_stride, const int32_t *__restrict__ slots,
                                                  const irm_tile *__restrict__ tiles,
                                                  const uint32_t *__restrict__ plan, uint32_t xcd_ranges,
                                                  uint32_t n_layers, uint32_t *err)
{
    __shared__ int32_t slot_s[ADMIT_TILE_ROWS];
    const uint32_t n_tiles = plan[0];
    // The grid is a multiple of 8 wide and workgroups go round-robin to the 8 XCDs.  xcd_ranges 1: grid
    // (tile slots, layers), workgroup x serves tile (x % 8) * ceil(n_tiles / 8) + x / 8 of layer
    // blockIdx.y, so each XCD streams one contiguous eighth of the layer's tile list; 2: a 1-D grid
    // over the layer-major list of all (layer, tile) items, an eighth of it per XCD; 0: tile x.
    const bool flat = xcd_ranges == 2;
    const uint32_t n_items = flat ? n_tiles * n_layers : n_tiles;      // flat: below 2^31 (the host checks)
    const uint32_t per_xcd = (n_items + 7) >> 3;
#pragma nounroll
    for (uint32_t x = blockIdx.x; x < per_xcd * 8; x += gridDim.x) {
        const uint32_t item = xcd_ranges ? (x & 7u) * per_xcd + (x >> 3) : x;
        if (item >= n_items) continue;                  // uniform
        const uint32_t layer = flat ? item / n_tiles : blockIdx.y;
        const uint32_t ti = flat ? item - layer * n_tiles : item;
        const irm_tile *tp = tiles + ti;
        const uint32_t row0 = __builtin_amdgcn_readfirstlane(tp->src_row0);
        const uint32_t tok0 = __builtin_amdgcn_readfirstlane(tp->dst_tok0);
        const uint32_t n_rows = __builtin_amdgcn_readfirstlane(tp->n_rows);
        __syncthreads();
        if (threadIdx.x < n_rows) {
            int32_t sl = slots[(uint64_t)tok0 + threadIdx.x];
            if (sl < 0 || (uint64_t)(uint32_t)sl >= req_rows) {
                atomicOr(err, IRM_FLAG_ROW_RANGE);
                sl = -1;
            }
            slot_s[threadIdx.x] = sl;
        }
        __syncthreads();
        const char *sbase = (const char *)req_ptrs[layer];
        char *dbase = (char *)pool_ptrs[layer] + (uint64_t)row0 * pool_stride;
        // a row's vectors are consecutive work items
        for (uint32_t i = threadIdx.x; i < n_rows * VPR; i += blockDim.x) {
            const uint32_t r = i / VPR, col = i - r * VPR;
            const int32_t sl = slot_s[r];
            if (sl < 0) continue;
            const u32x4 v = __builtin_nontemporal_load((const u32x4 *)(sbase + (uint64_t)(uint32_t)sl * req_stride) + col);
            __builtin_nontemporal_store(v, (u32x4 *)(dbase + (uint64_t)r * pool_stride) + col);
        }
    }
}

extern "C" irm_status irm_admit(irm_ctx *ctx, irm_table *table, const uint64_t *d_chunk_hash,
                                const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                                const uint32_t *d_req_chunk_offsets, const uint32_t *d_req_offsets,
                                const int32_t *d_pos_base, uint32_t n_req, const uint32_t *d_n_chunks,
                                uint32_t chunk_capacity, const int32_t *d_chunk_entry,
                                const void *const *d_req_layer_ptrs, uint64_t req_row_stride_bytes,
                                uint64_t req_rows, const int32_t *d_slots, uint64_t n_slot_tokens,
                                void *const *d_pool_layer_ptrs, uint64_t pool_row_stride_bytes,
                                uint64_t pool_rows, uint32_t *d_cursor, int32_t *d_admitted_row, void *stream)
{
    if (!ctx || !table || !d_chunk_hash || !d_chunk_start || !d_chunk_len || !d_req_chunk_offsets ||
        !d_req_offsets || !d_pos_base || !d_n_chunks || !d_chunk_entry || !d_req_layer_ptrs || !d_slots ||
        !d_pool_layer_ptrs || !d_cursor || !d_admitted_row)
        return IRM_ERR_INVALID_ARG;
    if (table->ctx != ctx || n_req < 1 || chunk_capacity < 1 || n_slot_tokens < 1) return IRM_ERR_INVALID_ARG;
    const uint32_t row_bytes = irm_row_bytes(ctx->cfg.row_format);
    if (req_row_stride_bytes < row_bytes || pool_row_stride_bytes < row_bytes ||
        (req_row_stride_bytes & 15) || (pool_row_stride_bytes & 15))
        return IRM_ERR_INVALID_ARG;
    if (req_rows < 1 || pool_rows < 1 || req_rows > 0x7FFFFFFFull || pool_rows > 0x7FFFFFFFull)
        return IRM_ERR_INVALID_ARG;
    if (n_req > ctx->cfg.max_requests || chunk_capacity > ctx->chunk_cap || n_slot_tokens > ctx->cfg.max_tokens ||
        table->n_slots > 0xFFFFFFF0ull)
        return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(admit_claim, dim3((chunk_capacity + 255) / 256), dim3(256), 0, s, table->d_keys,
                       table->d_owner, table->d_vals, table->n_slots, table->d_state, d_chunk_hash, d_chunk_start,
                       d_chunk_len, d_req_chunk_offsets, d_req_offsets, d_pos_base, n_req, d_n_chunks,
                       chunk_capacity, ctx->cfg.carve_out, d_chunk_entry, n_slot_tokens, pool_rows, d_cursor,
                       d_admitted_row, ctx->d_slot_of, ctx->d_tiles, ctx->tile_cap, ctx->d_plan, ctx->d_plan + 3,
                       ctx->d_err);
    // measured: contiguous tile ranges per XCD gain 10 % on a batch of a million tokens, cost 5 % on one of 32 K
    // from 32 layers on an eighth of the whole launch's list per XCD, as in the re-attach row kernel
    const uint32_t L = ctx->cfg.n_layers;
    uint64_t tile_slots = n_slot_tokens / ADMIT_TILE_ROWS + chunk_capacity;
    if (tile_slots > (1u << 24)) tile_slots = 1u << 24;
    const uint32_t grid_x = (uint32_t)((tile_slots + 7) / 8 * 8);
    const bool big = ctx->xcd_ranges && n_slot_tokens >= (1u << 18);
    const bool flat = big && (ctx->xcd_ranges == 2 || (ctx->xcd_ranges == 3 && L >= 32 && ctx->cfg.row_format == IRM_ROW_BF16)) &&
                      ((uint64_t)ctx->tile_cap + 8) * L < (1ull << 31) && (uint64_t)grid_x * L < (1ull << 31);
    hipLaunchKernelGGL(ctx->cfg.row_format == IRM_ROW_FP8 ? admit_rows<IRM_F8_ROW_BYTES / 16> : admit_rows<IRM_ROW_BYTES / 16>,
                       flat ? dim3(grid_x * L) : dim3(grid_x, L), dim3(256), 0, s,
                       d_req_layer_ptrs, req_row_stride_bytes, req_rows, d_pool_layer_ptrs,
                       pool_row_stride_bytes, d_slots, ctx->d_tiles, ctx->d_plan, flat ? 2u : (big ? 1u : 0u), L,
                       ctx->d_err);
    return irm_launch_status();
}
