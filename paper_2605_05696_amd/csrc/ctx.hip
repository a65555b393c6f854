// Context and registry-table lifetime, argument validation, insert-if-absent.
#include <new>
#include <string.h>

#include "irm_internal.hpp"

static void profile_drop(irm_ctx *ctx);

static inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

extern "C" irm_status irm_ctx_create(const irm_config *cfg, irm_ctx **out)
{
    if (!cfg || !out) return IRM_ERR_INVALID_ARG;
    if (cfg->ckv_dim != 512 || cfg->kr_dim != 64 || cfg->pair_mode > IRM_PAIR_INTERLEAVED ||
        cfg->row_format > IRM_ROW_FP8)
        return IRM_ERR_UNSUPPORTED;
    const uint64_t m = cfg->mask;
    if ((m & (m + 1)) != 0) return IRM_ERR_UNSUPPORTED;        // mask must be 2^k - 1
    const uint32_t k_bits = (uint32_t)__builtin_popcountll(m);
    if (cfg->min_chunk < 1 || cfg->min_chunk < k_bits) return IRM_ERR_INVALID_ARG;
    if (cfg->max_chunk < cfg->min_chunk || cfg->max_chunk > 65536) return IRM_ERR_INVALID_ARG;
    if (cfg->n_layers < 1 || cfg->n_layers > 4096) return IRM_ERR_INVALID_ARG;
    if (cfg->max_tokens < 1 || cfg->max_tokens > 0xFFFFFFF0ull - 65536) return IRM_ERR_INVALID_ARG;
    if (cfg->max_requests < 1 || cfg->max_requests > (1u << 20)) return IRM_ERR_INVALID_ARG;
    for (int i = 0; i < IRM_KR_PAIRS; ++i)
        if (!(cfg->inv_freq[i] == cfg->inv_freq[i]) || cfg->inv_freq[i] - cfg->inv_freq[i] != 0.0f)
            return IRM_ERR_INVALID_ARG;                         // NaN or infinite frequency
    const uint64_t chunk_cap64 = cfg->max_tokens / cfg->min_chunk + cfg->max_requests;
    if (chunk_cap64 > 0x7FFFFFFFull) return IRM_ERR_CAPACITY;

    irm_ctx *c = new (std::nothrow) irm_ctx;
    if (!c) return IRM_ERR_DEVICE;
    memset(c, 0, sizeof *c);
    c->cfg = *cfg;
    c->k_bits = k_bits;
    c->chunk_cap = (uint32_t)chunk_cap64;
    c->tile_cap = (uint32_t)(cfg->max_tokens / IRM_TILE_ROWS_MIN + chunk_cap64);
    // tile = 8 waves x 2 rows (bf16 rows, 18 KB) or x 4 rows (fp8 rows, 21 KB: with two rows per wave a
    // workgroup moves too little, 0.62 against 0.69 of peak on the 64 x 16 K batch)
    c->rows_per_wave = cfg->row_format == IRM_ROW_FP8 ? 4 : 2;
    c->block_waves = 8;
    // 656-byte rows begin and end inside 128-byte lines: streaming stores would send the shared lines to
    // memory half written, from each neighbour in turn (measured 3.8 against 5.2 TB/s with cached accesses)
    c->mem_mode = cfg->row_format == IRM_ROW_FP8 ? 0 : 3;
    c->xcd_ranges = 3;
    c->kr_rows_per_lane = 2;
    c->att_spin_limit = 1u << 18;

    hipDeviceProp_t prop;
    if (hipGetDevice(&c->device) != hipSuccess || hipGetDeviceProperties(&prop, c->device) != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return IRM_ERR_DEVICE;
    }
    c->n_cu = (uint32_t)prop.multiProcessorCount;

    // carve one slab
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { uint64_t o = off; off = align_up(off + bytes, 256); return o; };
    const uint64_t o_gear = take(256 * 4), o_inv = take(IRM_KR_PAIRS * 4), o_err = take(4);
    const uint64_t o_bitmap = take((cfg->max_tokens / 64 + 8) * 8);
    const uint64_t o_ss = take((uint64_t)c->chunk_cap * 4), o_sl = take((uint64_t)c->chunk_cap * 4);
    const uint64_t o_rc = take((uint64_t)cfg->max_requests * 4);
    const uint64_t o_ht = take((uint64_t)c->chunk_cap * sizeof(irm_hit));
    const uint64_t o_tiles = take((uint64_t)c->tile_cap * sizeof(irm_tile));
    const uint64_t o_trig = take((uint64_t)c->chunk_cap * IRM_KR_PAIRS * sizeof(float2));
    const uint64_t o_so = take((uint64_t)c->chunk_cap * 4);
    const uint64_t o_plan = take(IRM_PLAN_WORDS * 4);
    if (hipMalloc(&c->slab, off) != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return IRM_ERR_DEVICE;
    }
    char *base = (char *)c->slab;
    c->d_gear = (uint32_t *)(base + o_gear);
    c->d_inv_freq = (float *)(base + o_inv);
    c->d_err = (uint32_t *)(base + o_err);
    c->d_bitmap = (uint64_t *)(base + o_bitmap);
    c->d_stage_start = (uint32_t *)(base + o_ss);
    c->d_stage_len = (uint32_t *)(base + o_sl);
    c->d_req_count = (uint32_t *)(base + o_rc);
    c->d_hit_tmp = (irm_hit *)(base + o_ht);
    c->d_tiles = (irm_tile *)(base + o_tiles);
    c->d_trig = (float2 *)(base + o_trig);
    c->d_slot_of = (uint32_t *)(base + o_so);
    c->d_plan = (uint32_t *)(base + o_plan);
    if (hipMemset(c->slab, 0, off) != hipSuccess ||
        hipMemcpy(c->d_gear, cfg->gear, 256 * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(c->d_inv_freq, cfg->inv_freq, IRM_KR_PAIRS * 4, hipMemcpyHostToDevice) != hipSuccess ||
        irm_chunk_hash_init(c->device) != IRM_OK || irm_attend_init(c->device) != IRM_OK ||
        hipDeviceSynchronize() != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(c->slab);
        delete c;
        return IRM_ERR_DEVICE;
    }
    *out = c;
    return IRM_OK;
}

extern "C" irm_status irm_ctx_destroy(irm_ctx *ctx)
{
    if (!ctx) return IRM_ERR_INVALID_ARG;
    irm_status st = IRM_OK;
    profile_drop(ctx);
    if (ctx->slab && hipFree(ctx->slab) != hipSuccess) {
        (void)hipGetLastError();
        st = IRM_ERR_DEVICE;
    }
    delete ctx;
    return st;
}

extern "C" irm_status irm_ctx_error_flags(irm_ctx *ctx, void *stream, uint32_t *flags)
{
    if (!ctx || !flags) return IRM_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    uint32_t zero = 0;
    IRM_HIP_TRY(hipStreamSynchronize(s));
    IRM_HIP_TRY(hipMemcpy(flags, ctx->d_err, 4, hipMemcpyDeviceToHost));
    IRM_HIP_TRY(hipMemcpy(ctx->d_err, &zero, 4, hipMemcpyHostToDevice));
    return IRM_OK;
}

extern "C" irm_status irm_ctx_tune(irm_ctx *ctx, uint32_t knob, uint32_t value)
{
    if (!ctx) return IRM_ERR_INVALID_ARG;
    if (knob == 0) {
        if (value > (1u << 24)) return IRM_ERR_INVALID_ARG;
        ctx->reattach_grid = value;
        return IRM_OK;
    }
    if (knob == 1) {
        if (value != 1 && value != 2 && value != 4 && value != 8 && value != 16) return IRM_ERR_INVALID_ARG;
        if (value * ctx->block_waves < IRM_TILE_ROWS_MIN) return IRM_ERR_INVALID_ARG;
        if (ctx->cfg.row_format == IRM_ROW_FP8 && value == 1) return IRM_ERR_INVALID_ARG;   // two rows per load
        ctx->rows_per_wave = value;
        return IRM_OK;
    }
    if (knob == 2) {
        if (value > 3) return IRM_ERR_INVALID_ARG;
        ctx->mem_mode = value;
        return IRM_OK;
    }
    if (knob == 4) {
        if (value != 1 && value != 2 && value != 4 && value != 8 && value != 16) return IRM_ERR_INVALID_ARG;
        if (value * ctx->rows_per_wave < IRM_TILE_ROWS_MIN) return IRM_ERR_INVALID_ARG;
        if (ctx->cfg.row_format == IRM_ROW_FP8 && value < 4) return IRM_ERR_INVALID_ARG;
        ctx->block_waves = value;
        return IRM_OK;
    }
    if (knob == 5) {
        if (value > 1) return IRM_ERR_INVALID_ARG;
        ctx->cdc_serial = value;
        return IRM_OK;
    }
    if (knob == 8) {
        ctx->att_spin_limit = value;
        return IRM_OK;
    }
    if (knob == 7) {
        if (value > 4096) return IRM_ERR_INVALID_ARG;
        ctx->kr_layers_per_wg = value;
        return IRM_OK;
    }
    if (knob == 6) {
        if (value != 2 && value != 4 && value != 8) return IRM_ERR_INVALID_ARG;
        ctx->kr_rows_per_lane = value;
        return IRM_OK;
    }
    if (knob == 3) {
        if (value > 3) return IRM_ERR_INVALID_ARG;
        ctx->xcd_ranges = value;
        return IRM_OK;
    }
    return IRM_ERR_INVALID_ARG;
}

static void profile_drop(irm_ctx *ctx)
{
    if (ctx->prof_events) {
        for (uint32_t k = 0; k < 2 * ctx->prof_cap; ++k)
            if (ctx->prof_events[k]) (void)hipEventDestroy(ctx->prof_events[k]);
        delete[] ctx->prof_events;
    }
    ctx->prof_events = nullptr;
    ctx->prof_cap = ctx->prof_n = 0;
}

extern "C" irm_status irm_ctx_profile_begin(irm_ctx *ctx, uint32_t max_samples, uint32_t every)
{
    if (!ctx || max_samples < 1 || max_samples > 65536 || every < 1) return IRM_ERR_INVALID_ARG;
    profile_drop(ctx);
    ctx->prof_events = new (std::nothrow) hipEvent_t[2 * (size_t)max_samples]();
    if (!ctx->prof_events) return IRM_ERR_DEVICE;
    ctx->prof_cap = max_samples;
    ctx->prof_every = every;
    ctx->prof_calls = 0;
    for (uint32_t k = 0; k < 2 * max_samples; ++k) {
        if (hipEventCreate(&ctx->prof_events[k]) != hipSuccess) {
            (void)hipGetLastError();
            profile_drop(ctx);
            return IRM_ERR_DEVICE;
        }
    }
    return IRM_OK;
}

extern "C" irm_status irm_ctx_profile_end(irm_ctx *ctx, void *stream, float *total_ms, uint32_t *n_samples)
{
    if (!ctx || !total_ms || !n_samples) return IRM_ERR_INVALID_ARG;
    *total_ms = 0.0f;
    *n_samples = 0;
    if (!ctx->prof_events) return IRM_OK;
    irm_status st = IRM_OK;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) st = IRM_ERR_DEVICE;
    double sum = 0.0;
    for (uint32_t k = 0; k < ctx->prof_n && st == IRM_OK; ++k) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ctx->prof_events[2 * k], ctx->prof_events[2 * k + 1]) != hipSuccess)
            st = IRM_ERR_DEVICE;
        sum += ms;
    }
    if (st == IRM_OK) {
        *total_ms = (float)sum;
        *n_samples = ctx->prof_n;
    } else {
        (void)hipGetLastError();
    }
    profile_drop(ctx);
    return st;
}

// ---------------------------------------------------------------- registry --

extern "C" irm_status irm_table_create(irm_ctx *ctx, uint64_t n_slots, irm_table **out)
{
    if (!ctx || !out || n_slots < 1) return IRM_ERR_INVALID_ARG;
    if (n_slots > (1ull << 32)) return IRM_ERR_CAPACITY;
    irm_table *t = new (std::nothrow) irm_table;
    if (!t) return IRM_ERR_DEVICE;
    memset(t, 0, sizeof *t);
    t->ctx = ctx;
    t->n_slots = n_slots;
    const uint64_t n = n_slots + 1;
    if (hipMalloc((void **)&t->d_keys, n * 8) != hipSuccess ||
        hipMalloc((void **)&t->d_owner, n * 4) != hipSuccess ||
        hipMalloc((void **)&t->d_vals, n * sizeof(irm_entry)) != hipSuccess ||
        hipMalloc((void **)&t->d_state, 2 * sizeof(uint32_t)) != hipSuccess ||
        hipMemset(t->d_state, 0, 2 * sizeof(uint32_t)) != hipSuccess ||
        hipMemset(t->d_keys, 0, n * 8) != hipSuccess ||
        hipMemset(t->d_owner, 0xFF, n * 4) != hipSuccess ||
        hipMemset(t->d_vals, 0, n * sizeof(irm_entry)) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
        (void)hipGetLastError();
        if (t->d_keys) (void)hipFree(t->d_keys);
        if (t->d_owner) (void)hipFree(t->d_owner);
        if (t->d_vals) (void)hipFree(t->d_vals);
        if (t->d_state) (void)hipFree(t->d_state);
        delete t;
        return IRM_ERR_DEVICE;
    }
    *out = t;
    return IRM_OK;
}

extern "C" irm_status irm_table_destroy(irm_table *table)
{
    if (!table) return IRM_ERR_INVALID_ARG;
    irm_status st = IRM_OK;
    if (hipFree(table->d_keys) != hipSuccess) st = IRM_ERR_DEVICE;
    if (hipFree(table->d_owner) != hipSuccess) st = IRM_ERR_DEVICE;
    if (hipFree(table->d_vals) != hipSuccess) st = IRM_ERR_DEVICE;
    if (hipFree(table->d_state) != hipSuccess) st = IRM_ERR_DEVICE;
    if (st != IRM_OK) (void)hipGetLastError();
    delete table;
    return st;
}

// Offer ranks: offer i of a batch bids with rank state[0] + i, and state[0] grows by the
// batch size afterwards, so an earlier batch always outbids a later one.  A batch that
// would run past 2^32 - 2 offers is refused (IRM_FLAG_TABLE_FULL).
__device__ __forceinline__ bool irm_rank_room(uint32_t rank0, uint32_t n) { return rank0 <= 0xFFFFFFFEu - n; }

// pass 1: claim a slot per key and record the lowest offer rank that wants it
__global__ __launch_bounds__(256) void table_claim(uint64_t *keys, uint32_t *owner, uint64_t n_slots,
                                                   const uint64_t *hash, uint32_t n, const uint32_t *n_p,
                                                   const uint32_t *state, uint32_t *err)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t rank0 = state[0];
    if (!irm_rank_room(rank0, n)) {
        if (i == 0) atomicOr(err, IRM_FLAG_TABLE_FULL);
        return;
    }
    if (n_p && *n_p < n) n = *n_p;                      // count kept on the device
    if (i >= n) return;
    uint64_t s = irm_claim_slot(keys, n_slots, hash[i]);
    if (s > n_slots) {
        atomicOr(err, IRM_FLAG_TABLE_FULL);
        return;
    }
    atomicMin(&owner[s], rank0 + i);
}

// pass 2: the winning offer of a slot that was empty before this batch writes the value;
// the workgroup that finishes last advances the rank base (all have read it by then)
__global__ __launch_bounds__(256) void table_fill(const uint64_t *keys, const uint32_t *owner,
                                                  irm_entry *vals, uint64_t n_slots,
                                                  const uint64_t *hash, const irm_entry *val,
                                                  uint32_t n_launch, const uint32_t *n_p, uint32_t *state)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t rank0 = state[0];
    const bool room = irm_rank_room(rank0, n_launch);
    uint32_t n = n_launch;
    if (n_p && *n_p < n) n = *n_p;
    if (room && i < n) {
        const uint64_t key = hash[i];
        uint64_t s = n_slots;
        bool found = true;
        if (key != 0) {
            s = irm_slot_of(key, n_slots);
            uint64_t tries = 0;
            while (keys[s] != key) {                    // present unless the table was full
                if (keys[s] == 0 || ++tries >= n_slots) {
                    found = false;
                    break;
                }
                s = (s + 1 == n_slots) ? 0 : s + 1;
            }
        }
        if (found && owner[s] == rank0 + i) vals[s] = val[i];
    }
    __syncthreads();                                    // every lane of this workgroup has read state[0]
    if (threadIdx.x == 0) {
        __threadfence();
        if (atomicAdd(&state[1], 1u) == gridDim.x - 1) {
            if (room) state[0] = rank0 + n_launch;
            state[1] = 0;
        }
    }
}

static irm_status table_insert(irm_table *table, const uint64_t *d_hash, const irm_entry *d_val, uint32_t n,
                               const uint32_t *d_n, void *stream)
{
    if (!table || (!d_hash && n) || (!d_val && n)) return IRM_ERR_INVALID_ARG;
    if (n == 0) return IRM_OK;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(table_claim, dim3(blocks), dim3(256), 0, s, table->d_keys, table->d_owner,
                       table->n_slots, d_hash, n, d_n, table->d_state, table->ctx->d_err);
    hipLaunchKernelGGL(table_fill, dim3(blocks), dim3(256), 0, s, table->d_keys, table->d_owner,
                       table->d_vals, table->n_slots, d_hash, d_val, n, d_n, table->d_state);
    return irm_launch_status();
}

extern "C" irm_status irm_table_insert(irm_table *table, const uint64_t *d_hash,
                                       const irm_entry *d_val, uint32_t n, void *stream)
{
    return table_insert(table, d_hash, d_val, n, nullptr, stream);
}

extern "C" irm_status irm_table_insert_counted(irm_table *table, const uint64_t *d_hash,
                                               const irm_entry *d_val, const uint32_t *d_n,
                                               uint32_t capacity, void *stream)
{
    if (!d_n) return IRM_ERR_INVALID_ARG;
    return table_insert(table, d_hash, d_val, capacity, d_n, stream);
}
