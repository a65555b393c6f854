// Internal declarations shared by the HIP sources of libirm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "irm.h"
#include "irm_measure.h"

#define IRM_ROW_BYTES 1152u     // bf16 rows: 576 bf16
#define IRM_CKV_BYTES 1024u     // bf16 rows: 512 bf16
#define IRM_F8_ROW_BYTES 656u   // fp8 rows: 512 e4m3 | 4 fp32 scales | 64 bf16
#define IRM_F8_CKV_BYTES 528u   // their position-free part; the scales are its last 16 bytes
#define IRM_KR_BYTES 128u       // 64 bf16
#define IRM_TILE_ROWS_MIN 4u    // smallest tile of the re-attach row kernel (sizes the tile list)
#define IRM_WAVE 64
#define IRM_PLAN_WORDS 16u

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// One tile of the re-attach row kernel: up to tile_rows consecutive rows of one hit.
struct irm_tile {
    uint32_t src_row0;
    uint32_t dst_tok0;
    uint32_t n_rows;
    uint32_t hit;
};

struct irm_ctx {
    irm_config cfg;
    int device;
    uint32_t k_bits;        // popcount(mask)
    uint32_t chunk_cap;     // max_tokens / min_chunk + max_requests
    uint32_t tile_cap;      // max_tokens / IRM_TILE_ROWS + chunk_cap
    uint32_t reattach_grid; // tuning knob 0: grid.x of the row kernel (tile slots per layer), 0 = default
    uint32_t rows_per_wave; // knob 1: 1, 2, 4, 8 or 16 c_KV rows per wave and tile
    uint32_t block_waves;   // knob 4: 4, 8 or 16 waves per workgroup (tile = waves * rows_per_wave rows)
    uint32_t mem_mode;      // knob 2: bit 0 non-temporal loads, bit 1 non-temporal stores
    uint32_t cdc_serial;    // knob 5: 1 = always use the serial cut selection
    uint32_t kr_rows_per_lane; // knob 6: rows per lane of the k_r-only kernel (2, 4 or 8; tile = 32x that)
    uint32_t kr_layers_per_wg; // knob 7: layers a workgroup of the k_r-only kernel keeps its tile for (0 = by batch size)
    uint32_t att_spin_limit; // knob 8: polls a wave of the attention kernel spends in one wait before it gives up
    uint32_t xcd_ranges;    // knob 3: 2 = each XCD serves a contiguous eighth of the launch's (layer, tile) list,
                            // 1 = of every layer's tiles, 0 = workgroup x serves tile x, 3 = 2 from 32 layers on, else 1
    uint32_t n_cu;
    // one device slab, carved up below
    void *slab;
    uint32_t *d_gear;       // [256]
    float *d_inv_freq;      // [32]
    uint32_t *d_err;        // [1] device error word
    uint64_t *d_bitmap;     // candidate bit per token
    uint32_t *d_stage_start, *d_stage_len; // [chunk_cap] per-request staged chunks
    uint32_t *d_req_count;  // [max_requests]
    irm_hit *d_hit_tmp;     // [chunk_cap] per-chunk probe result, len == 0 for a miss
    irm_tile *d_tiles;      // [tile_cap]
    float2 *d_trig;         // [chunk_cap][32] (cos, sin) per hit and pair
    uint32_t *d_slot_of;    // [chunk_cap] table slot a chunk claimed while being admitted
    uint32_t *d_plan;       // [IRM_PLAN_WORDS]: n_tiles, then the ticket counters of cdc, lookup and admit
    // optional timing of the row kernel
    hipEvent_t *prof_events; // [2 * prof_cap]
    uint32_t prof_cap, prof_n, prof_every, prof_calls;
};

struct irm_table {
    irm_ctx *ctx;
    uint64_t n_slots;       // slot n_slots is reserved for the key 0
    uint32_t *d_state;      // [0] offers made so far: the rank base that makes "first offer wins" hold
                            // across batches; [1] ticket counter of table_fill.  Kept on the device so
                            // that captured launches stay correct when replayed.
    uint64_t *d_keys;       // [n_slots + 1], 0 = empty
    uint32_t *d_owner;      // [n_slots + 1], rank of the winning offer, 0xFFFFFFFF = none
    irm_entry *d_vals;      // [n_slots + 1]
};

// uploads the fingerprint kernel's constant table to the current device (idempotent)
irm_status irm_chunk_hash_init(int device);
// raises the LDS limit of the attention kernel on the current device
irm_status irm_attend_init(int device);

#define IRM_HIP_TRY(expr)                      \
    do {                                       \
        if ((expr) != hipSuccess) {            \
            (void)hipGetLastError();           \
            return IRM_ERR_DEVICE;             \
        }                                      \
    } while (0)

static inline irm_status irm_launch_status()
{
    return hipGetLastError() == hipSuccess ? IRM_OK : IRM_ERR_DEVICE;
}

// slot of a key: Fibonacci mixing, then multiply-shift range reduction
__device__ __forceinline__ uint64_t irm_slot_of(uint64_t key, uint64_t n_slots)
{
    uint64_t m = key * 0x9E3779B97F4A7C15ull;
    m ^= m >> 29;
    return __umul64hi(m, n_slots);
}

// Walk the probe sequence of `key` until its slot is found or claimed.
// Returns the slot, or n_slots + 1 when the table has no room.
__device__ __forceinline__ uint64_t irm_claim_slot(uint64_t *keys, uint64_t n_slots, uint64_t key)
{
    if (key == 0) return n_slots;                       // reserved slot: 0 marks "empty" elsewhere
    uint64_t s = irm_slot_of(key, n_slots);
    for (uint64_t tries = 0; tries < n_slots; ++tries) {
        unsigned long long seen = atomicCAS((unsigned long long *)&keys[s], 0ull, (unsigned long long)key);
        if (seen == 0ull || seen == key) return s;
        s = (s + 1 == n_slots) ? 0 : s + 1;
    }
    return n_slots + 1;
}

// absolute position of chunk c: pos_base of its request + offset of its first token there
__device__ __forceinline__ int64_t irm_chunk_pos(const uint32_t *__restrict__ req_chunk_offsets,
                                                 const uint32_t *__restrict__ req_offsets,
                                                 const int32_t *__restrict__ pos_base, uint32_t n_req,
                                                 uint32_t c, uint32_t start)
{
    uint32_t lo = 0, hi = n_req;                        // last r with req_chunk_offsets[r] <= c
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (req_chunk_offsets[mid] <= c) lo = mid; else hi = mid;
    }
    return (int64_t)pos_base[lo] + ((int64_t)start - (int64_t)req_offsets[lo]);
}

// (cos, sin) of delta * inv_freq, the angle as an fp64 product with fp64 range reduction
// (|delta| reaches 1e5: an fp32 angle would already cost half a bf16 ulp); delta == 0 is the
// exact identity.
__device__ __forceinline__ float2 irm_hit_trig(int32_t delta, float inv_freq)
{
    if (delta == 0) return make_float2(1.0f, 0.0f);
    const double phi = (double)delta * (double)inv_freq;
    double sn, cn;
    sincos(phi, &sn, &cn);
    return make_float2((float)cn, (float)sn);
}

// Where pair i of a hit sits in its 32-entry table.  Half-split: entry i is pair i.
// Interleaved: the lane that holds the 16-byte vectors j and 4+j of a row owns pairs 4j+w and
// 16+4j+w (w < 4); they are stored side by side at entries 8j+2w and 8j+2w+1, where the
// half-split kernel code finds the (cos, sin) of the two halves of word w.
__device__ __forceinline__ uint32_t irm_trig_slot(uint32_t pair_mode, uint32_t i)
{
    return pair_mode ? 8u * ((i & 15u) >> 2) + 2u * (i & 3u) + (i >> 4) : i;
}

// tile k of a hit that is cut into tiles of tile_rows rows
__device__ __forceinline__ irm_tile irm_tile_of(const irm_hit &hit, uint32_t h, uint32_t k, uint32_t tile_rows)
{
    const uint32_t done = k * tile_rows;
    irm_tile tile;
    tile.src_row0 = hit.src_row + done;
    tile.dst_tok0 = hit.dst_tok + done;
    tile.n_rows = hit.len - done < tile_rows ? hit.len - done : tile_rows;
    tile.hit = h;
    return tile;
}

__device__ __forceinline__ uint32_t irm_wave_id()
{
    return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
}

// inclusive scan of one uint32 per thread over a block of up to 1024 threads;
// *total receives the block sum.  `lds` must hold 17 uint32.  All threads call.
__device__ __forceinline__ uint32_t irm_block_scan_incl(uint32_t v, uint32_t *lds, uint32_t *total)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63) >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(x, d);
        if (lane >= (uint32_t)d) x += y;
    }
    __syncthreads();          // protects lds reuse across consecutive calls
    if (lane == 63) lds[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (uint32_t w = 0; w < n_waves; ++w) {
            uint32_t t = lds[w];
            lds[w] = run;
            run += t;
        }
        lds[16] = run;
    }
    __syncthreads();
    *total = lds[16];
    return x + lds[wave];
}
