// Fused gather + delta-rotation + scatter (paper Alg. 1 steps 8-10; Sec. 7.2
// "k_r rotation"; App. C "k_r rotation materialisation").
//
// Two launches.
//   reattach_plan  per hit: the 32 (cos, sin) of delta * inv_freq[i], angle as an
//                  fp64 product with fp64 range reduction (|delta| reaches 1e5, an
//                  fp32 angle would already cost half a bf16 ulp); the hits are cut
//                  into tiles (16 rows of 1152 bytes, 32 rows of 656 bytes), the tile
//                  list is written by all workgroups at once.
//   reattach_rows  one workgroup per tile and layer, every XCD on a contiguous eighth
//                  of the launch's layer-major list of them: a
//                  tile's source rows are one contiguous span; each of the 8 waves
//                  moves 2 rows of c_KV with one 16-byte load and store per lane and
//                  row (a row's 1024 c_KV bytes are exactly one wave-wide access),
//                  and four lanes of wave 0 rotate one row's k_r each: the two
//                  16-byte vectors that hold elements 8j.. and 32+8j.. sit in the
//                  same lane, so the half-split partners never cross lanes.  The
//                  row's 128 k_r bytes are one cache line.  Loads and stores are
//                  non-temporal: every byte is touched once.
//   reattach_kr_rows  the split-pool variant (App. C): only the k_r slice is
//                  materialised, c_KV is handed on as a row index; eight lanes per
//                  row, whole 128-byte lines per access, partners four lanes apart; a
//                  workgroup keeps its tile for several layers.
//   reattach_ref_rows  the no-materialise variant: row references only.
// irm_reattach_static runs the same kernels for a caller without a context, with the
// plan in a static device array.
#include "irm_internal.hpp"

// ---- plan --------------------------------------------------------------------
// tiles a hit is cut into; 0 when it points outside the pools (the hit is skipped)
__device__ __forceinline__ uint32_t hit_tiles(const irm_hit &hit, uint64_t src_rows, uint64_t n_slot_tokens,
                                              uint32_t tile_rows)
{
    const bool ok = (uint64_t)hit.src_row + hit.len <= src_rows &&
                    (uint64_t)hit.dst_tok + hit.len <= n_slot_tokens;
    return ok ? (hit.len + tile_rows - 1) / tile_rows : 0u;
}

// One lane per (hit, pair): 8 hits per workgroup.  Each workgroup sums the tile counts
// of all hits in front of its own (independent loads, a block reduction), so the tile
// list is written by all workgroups at once, 32 lanes per hit.
__device__ __forceinline__ void plan_body(const irm_hit *__restrict__ hits, const uint32_t *__restrict__ n_hits_p,
                                          uint32_t hit_capacity, const float *inv_freq, uint64_t src_rows,
                                          uint64_t n_slot_tokens, float2 *__restrict__ trig,
                                          irm_tile *__restrict__ tiles, uint32_t tile_cap, uint32_t tile_rows,
                                          uint32_t pair_mode, uint32_t *__restrict__ plan, uint32_t *err)
{
    __shared__ uint32_t lds[17];
    __shared__ uint32_t local_nt[8];
    uint32_t n_hits = *n_hits_p;
    if (n_hits > hit_capacity) {
        n_hits = hit_capacity;
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
    }
    const uint32_t h0 = blockIdx.x * 8u;                // first hit of this workgroup
    if (h0 >= n_hits) {
        if (blockIdx.x == 0 && threadIdx.x == 0) plan[0] = 0;   // no hits at all
        return;
    }
    const uint32_t h = h0 + (threadIdx.x >> 5), i = threadIdx.x & 31;
    irm_hit hit = {0u, 0u, 0u, 0};
    uint32_t nt = 0;
    if (h < n_hits) {
        hit = hits[h];
        nt = hit_tiles(hit, src_rows, n_slot_tokens, tile_rows);
        trig[(uint64_t)h * IRM_KR_PAIRS + irm_trig_slot(pair_mode, i)] = irm_hit_trig(hit.delta, inv_freq[i]);
        if (i == 0 && nt == 0 && hit.len != 0) atomicOr(err, IRM_FLAG_ROW_RANGE);
    }
    if (i == 0) local_nt[threadIdx.x >> 5] = nt;
    // tiles in front of this workgroup's first hit
    uint32_t before = 0;
    for (uint32_t k = threadIdx.x; k < h0; k += blockDim.x)
        before += hit_tiles(hits[k], src_rows, n_slot_tokens, tile_rows);
    uint32_t total;
    (void)irm_block_scan_incl(before, lds, &total);     // also orders local_nt for the reads below
    uint32_t t0 = total;
    for (uint32_t k = 0; k < (threadIdx.x >> 5); ++k) t0 += local_nt[k];
    if (h < n_hits) {
        for (uint32_t k = i; k < nt; k += 32) {
            const uint32_t t = t0 + k;
            if (t >= tile_cap) {
                atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
                break;
            }
            tiles[t] = irm_tile_of(hit, h, k, tile_rows);
        }
        if (h == n_hits - 1 && i == 0) plan[0] = t0 + nt < tile_cap ? t0 + nt : tile_cap;
    }
}

__global__ __launch_bounds__(256) void reattach_plan(const irm_hit *__restrict__ hits,
                                                     const uint32_t *__restrict__ n_hits_p,
                                                     uint32_t hit_capacity, const float *__restrict__ inv_freq,
                                                     uint64_t src_rows, uint64_t n_slot_tokens,
                                                     float2 *__restrict__ trig, irm_tile *__restrict__ tiles,
                                                     uint32_t tile_cap, uint32_t tile_rows, uint32_t pair_mode,
                                                     uint32_t *__restrict__ plan, uint32_t *err)
{
    plan_body(hits, n_hits_p, hit_capacity, inv_freq, src_rows, n_slot_tokens, trig, tiles, tile_cap, tile_rows,
              pair_mode, plan, err);
}

// the same with the 32 frequencies passed by value (a caller without a context has no device copy)
struct irm_freq32 {
    float v[IRM_KR_PAIRS];
};

__global__ __launch_bounds__(256) void reattach_plan_byval(const irm_hit *__restrict__ hits,
                                                           const uint32_t *__restrict__ n_hits_p,
                                                           uint32_t hit_capacity, irm_freq32 freq, uint64_t src_rows,
                                                           uint64_t n_slot_tokens, float2 *__restrict__ trig,
                                                           irm_tile *__restrict__ tiles, uint32_t tile_cap,
                                                           uint32_t tile_rows, uint32_t pair_mode,
                                                           uint32_t *__restrict__ plan, uint32_t *err)
{
    __shared__ float f[IRM_KR_PAIRS];
#pragma unroll
    for (int i = 0; i < IRM_KR_PAIRS; ++i)             // constant indices: the values come straight from the argument block
        if (threadIdx.x == (uint32_t)i) f[i] = freq.v[i];
    __syncthreads();
    plan_body(hits, n_hits_p, hit_capacity, f, src_rows, n_slot_tokens, trig, tiles, tile_cap, tile_rows, pair_mode,
              plan, err);
}

// ---- rows ----------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// rotate the two bf16 pairs packed in (wa, wb): wa holds elements (e, e+1) of the
// first halves, wb their partners; cs0/cs1 are (cos, sin) for e and e+1
__device__ __forceinline__ void rotate_word(uint32_t wa, uint32_t wb, float2 cs0, float2 cs1,
                                            uint32_t &oa, uint32_t &ob)
{
    const float a0 = bf16_lo(wa), a1 = bf16_hi(wa), b0 = bf16_lo(wb), b1 = bf16_hi(wb);
    const float ra0 = a0 * cs0.x - b0 * cs0.y, rb0 = b0 * cs0.x + a0 * cs0.y;
    const float ra1 = a1 * cs1.x - b1 * cs1.y, rb1 = b1 * cs1.x + a1 * cs1.y;
    oa = f32_to_bf16(ra0) | (f32_to_bf16(ra1) << 16);
    ob = f32_to_bf16(rb0) | (f32_to_bf16(rb1) << 16);
}

// (x.lo, x.hi), (y.lo, y.hi) -> (x.lo, y.lo), (x.hi, y.hi); its own inverse
__device__ __forceinline__ void pair_regroup(uint32_t &x, uint32_t &y)
{
    const uint32_t lo = (x & 0xFFFFu) | (y << 16), hi = (x >> 16) | (y & 0xFFFF0000u);
    x = lo;
    y = hi;
}

// Interleaved layout, one 16-byte vector = four whole pairs (a in the low half of a word,
// b in the high half); t[k].xy or t[k].zw (upper) is the (cos, sin) of word k's pair.
__device__ __forceinline__ u32x4 rotate_vector_pairs(u32x4 mine, f32x4 t0, f32x4 t1, f32x4 t2, f32x4 t3, bool upper)
{
    const f32x4 tt[4] = {t0, t1, t2, t3};
    const uint32_t mw[4] = {mine.x, mine.y, mine.z, mine.w};
    uint32_t res[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float a = bf16_lo(mw[k]), b = bf16_hi(mw[k]);
        const float c = upper ? tt[k].z : tt[k].x, s = upper ? tt[k].w : tt[k].y;
        res[k] = f32_to_bf16(a * c - b * s) | (f32_to_bf16(b * c + a * s) << 16);
    }
    return u32x4{res[0], res[1], res[2], res[3]};
}

// One 16-byte vector of a k_r row (8 elements) given its partner vector (the other
// half of the same 8 pairs) and the pairs' (cos, sin): mine * c + sgn * other * s, with
// sgn = -1 for the first halves (a c - b s) and +1 for the partners (b c + a s).
__device__ __forceinline__ u32x4 rotate_vector(u32x4 mine, u32x4 other, f32x4 t0, f32x4 t1, f32x4 t2, f32x4 t3,
                                               float sgn)
{
    const f32x4 tt[4] = {t0, t1, t2, t3};
    const uint32_t mw[4] = {mine.x, mine.y, mine.z, mine.w};
    const uint32_t ow[4] = {other.x, other.y, other.z, other.w};
    uint32_t res[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float m0 = bf16_lo(mw[k]), m1 = bf16_hi(mw[k]), o0 = bf16_lo(ow[k]), o1 = bf16_hi(ow[k]);
        const float r0 = m0 * tt[k].x + sgn * (o0 * tt[k].y);
        const float r1 = m1 * tt[k].z + sgn * (o1 * tt[k].w);
        res[k] = f32_to_bf16(r0) | (f32_to_bf16(r1) << 16);
    }
    return u32x4{res[0], res[1], res[2], res[3]};
}

__device__ __forceinline__ u32x4 partner_vector(u32x4 mine)
{
    u32x4 other;                                        // the partner sits four lanes away
    other.x = __shfl_xor(mine.x, 4);
    other.y = __shfl_xor(mine.y, 4);
    other.z = __shfl_xor(mine.z, 4);
    other.w = __shfl_xor(mine.w, 4);
    return other;
}

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT>
__device__ __forceinline__ void st16(u32x4 v, u32x4 *p)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// One tile: up to WAVES * RPW rows.  Wave w moves the c_KV of rows [w*RPW, (w+1)*RPW)
// and rotates the k_r of rows [16w, 16w+16) (four lanes per row).  slot[q] holds the
// destination row of tile row 64q + lane (-1: absent or unusable).
// F8 rows (512 e4m3 bytes | 16 bytes of scales | k_r): the quantised c_KV is 32 vectors, so
// half a wave takes a row and one load covers two rows; the scales travel with the k_r
// lanes, which sit right behind them.
template <int WAVES, int RPW, bool FULL, bool NT_LD, bool NT_ST, bool F8>
__device__ __forceinline__ void reattach_tile(const char *__restrict__ sbase, uint64_t src_stride,
                                              char *__restrict__ dbase, uint64_t dst_stride,
                                              const int32_t (&slot)[(WAVES * RPW + 63) / 64],
                                              uint32_t n_rows, const float2 *__restrict__ trig_hit,
                                              uint32_t wave, uint32_t lane, bool il)
{
    static_assert(!F8 || RPW % 2 == 0, "fp8 rows are moved two at a time");
    constexpr int TILE = WAVES * RPW, NQ = (TILE + 63) / 64;
    constexpr int NLD = F8 ? RPW / 2 : RPW;             // c_KV loads per lane
    constexpr uint32_t CKV = F8 ? IRM_F8_CKV_BYTES : IRM_CKV_BYTES;
    const uint32_t row0 = wave * RPW;
    const uint32_t sub = F8 ? lane >> 5 : 0u, vec = F8 ? lane & 31u : lane;
    // c_KV: issue every load of this wave's rows before the first store
    u32x4 v[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const uint32_t r = F8 ? row0 + 2 * i + sub : row0 + i;
        if (FULL || r < n_rows) v[i] = ld16<NT_LD>((const u32x4 *)(sbase + (uint64_t)r * src_stride) + vec);
    }
    // k_r: lane (rr, j) owns pairs 8j .. 8j+7 of row rr
    const uint32_t rr = wave * 16 + (lane >> 2), j = lane & 3;
    const bool kr_on = rr < n_rows;                   // n_rows <= TILE
    u32x4 ka = {0, 0, 0, 0}, kb = {0, 0, 0, 0}, scales = {0, 0, 0, 0};
    f32x4 t0 = {1, 0, 1, 0}, t1 = t0, t2 = t0, t3 = t0;
    if (kr_on) {
        const u32x4 *kr = (const u32x4 *)(sbase + (uint64_t)rr * src_stride + CKV);
        ka = ld16<NT_LD>(kr + j);
        kb = ld16<NT_LD>(kr + 4 + j);
        if (F8 && j == 0) scales = ld16<NT_LD>(kr - 1);
        const f32x4 *tp = (const f32x4 *)(trig_hit + 8 * j);
        t0 = tp[0];
        t1 = tp[1];
        t2 = tp[2];
        t3 = tp[3];
    }
    // rows 16w .. 16w+15 all lie in slot word (16w)/64 = w/4
    int32_t kr_slot = -1;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int32_t cand = __shfl(slot[q], (int)(rr & 63));
        if ((wave >> 2) == (uint32_t)q) kr_slot = cand;
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        if (F8) {
            // rows r and r + 1 (r even) lie in the same slot word
            const uint32_t r = row0 + 2 * i;
            int32_t s0 = -1, s1 = -1;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                if ((r >> 6) == (uint32_t)q) {
                    s0 = __builtin_amdgcn_readlane(slot[q], (int)(r & 63));
                    s1 = __builtin_amdgcn_readlane(slot[q], (int)((r & 63) + 1));
                }
            const int32_t sl = sub ? s1 : s0;
            if ((FULL || r + sub < n_rows) && sl >= 0)
                st16<NT_ST>(v[i], (u32x4 *)(dbase + (uint64_t)(uint32_t)sl * dst_stride) + vec);
        } else {
            const uint32_t r = row0 + i;
            if (FULL || r < n_rows) {
                int32_t sl = -1;
#pragma unroll
                for (int q = 0; q < NQ; ++q)
                    if ((r >> 6) == (uint32_t)q) sl = __builtin_amdgcn_readlane(slot[q], (int)(r & 63));
                if (sl >= 0) st16<NT_ST>(v[i], (u32x4 *)(dbase + (uint64_t)(uint32_t)sl * dst_stride) + vec);
            }
        }
    }
    if (kr_on && kr_slot >= 0) {
        // interleaved layout: a word holds one whole pair (a, b); regroup the words of the
        // two vectors into (a, a') and (b, b'), rotate as usual, and put them back
        uint32_t wa[4] = {ka.x, ka.y, ka.z, ka.w}, wb[4] = {kb.x, kb.y, kb.z, kb.w};
        if (il) {
#pragma unroll
            for (int k = 0; k < 4; ++k) pair_regroup(wa[k], wb[k]);
        }
        uint32_t a0, a1, a2, a3, b0, b1, b2, b3;
        rotate_word(wa[0], wb[0], make_float2(t0.x, t0.y), make_float2(t0.z, t0.w), a0, b0);
        rotate_word(wa[1], wb[1], make_float2(t1.x, t1.y), make_float2(t1.z, t1.w), a1, b1);
        rotate_word(wa[2], wb[2], make_float2(t2.x, t2.y), make_float2(t2.z, t2.w), a2, b2);
        rotate_word(wa[3], wb[3], make_float2(t3.x, t3.y), make_float2(t3.z, t3.w), a3, b3);
        if (il) {
            pair_regroup(a0, b0);
            pair_regroup(a1, b1);
            pair_regroup(a2, b2);
            pair_regroup(a3, b3);
        }
        const u32x4 oa = {a0, a1, a2, a3}, ob = {b0, b1, b2, b3};
        u32x4 *out = (u32x4 *)(dbase + (uint64_t)(uint32_t)kr_slot * dst_stride + CKV);
        st16<NT_ST>(oa, out + j);
        st16<NT_ST>(ob, out + 4 + j);
        if (F8 && j == 0) st16<NT_ST>(scales, out - 1);
    }
}

// Which tile and layer a workgroup serves.  The dispatcher deals workgroups round-robin to the 8
// XCDs and every grid here is a multiple of 8 wide, so workgroup x runs on XCD x % 8.
//   xcd_ranges 2  1-D grid over the launch's whole list of (layer, tile) items, layer-major: workgroup
//                 x serves item (x % 8) * ceil(items / 8) + x / 8, so every XCD streams one contiguous
//                 eighth of the launch, each in layers of its own (the host's choice for deep models:
//                 3 to 5 % faster at 61 layers than an eighth of every layer each);
//   xcd_ranges 1  grid (tile slots, layers): tile (x % 8) * ceil(tiles / 8) + x / 8 of layer blockIdx.y;
//   xcd_ranges 0  grid (tile slots, layers): tile x of layer blockIdx.y.
// Workgroups past the last item leave at once.  With fewer workgroups than items (a grid set by
// the caller, or more ragged tiles than the grid has slots) a workgroup walks several items; the
// record of the next one is requested before the current tile's rows, so that its latency hides
// behind them.
template <int WAVES, int RPW, bool NT_LD, bool NT_ST, bool F8>
__global__ __launch_bounds__(WAVES * 64) void reattach_rows(
    const void *const *__restrict__ src_ptrs, uint64_t src_stride, void *const *__restrict__ dst_ptrs,
    uint64_t dst_stride, uint64_t dst_rows, const int32_t *__restrict__ dst_slots,
    const irm_tile *__restrict__ tiles, const uint32_t *__restrict__ plan, const float2 *__restrict__ trig,
    uint32_t xcd_ranges, uint32_t n_layers, uint32_t pair_mode, uint32_t *err)
{
    constexpr uint32_t TILE = WAVES * RPW, NQ = (TILE + 63) / 64;
    const bool il = pair_mode != 0;
    const uint32_t n_tiles = plan[0];
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = irm_wave_id();
    const bool flat = xcd_ranges == 2;
    const uint32_t n_items = flat ? n_tiles * n_layers : n_tiles;     // flat: the host keeps the product below 2^31
    const uint32_t per_xcd = (n_items + 7) >> 3;
    const uint32_t limit = per_xcd * 8;
    auto locate = [&](uint32_t x, uint32_t &layer, uint32_t &ti) {
        const uint32_t item = xcd_ranges ? (x & 7u) * per_xcd + (x >> 3) : x;
        if (item >= n_items) return false;
        layer = flat ? item / n_tiles : blockIdx.y;
        ti = flat ? item - layer * n_tiles : item;
        return true;
    };
    uint32_t x = blockIdx.x, layer = 0, ti = 0, cur_layer = 0;
    irm_tile cur = {0u, 0u, 0u, 0u};
    if (x < limit && locate(x, layer, ti)) {
        cur = tiles[ti];
        cur_layer = layer;
    }
#pragma nounroll
    while (x < limit) {
        const uint32_t xn = x + gridDim.x;
        irm_tile nxt = {0u, 0u, 0u, 0u};
        uint32_t nxt_layer = 0;
        if (xn < limit && locate(xn, layer, ti)) {
            nxt = tiles[ti];
            nxt_layer = layer;
        }
        const uint32_t src_row0 = __builtin_amdgcn_readfirstlane(cur.src_row0);
        const uint32_t dst_tok0 = __builtin_amdgcn_readfirstlane(cur.dst_tok0);
        const uint32_t n_rows = __builtin_amdgcn_readfirstlane(cur.n_rows);
        const uint32_t hit = __builtin_amdgcn_readfirstlane(cur.hit);
        if (n_rows != 0) {                              // 0: no tile behind this slot
            const char *sbase = (const char *)src_ptrs[cur_layer] + (uint64_t)src_row0 * src_stride;
            char *const dbase = (char *)dst_ptrs[cur_layer];
            int32_t slot[NQ];                           // -1: row absent or its slot unusable
#pragma unroll
            for (uint32_t q = 0; q < NQ; ++q) {
                const uint32_t r = 64 * q + lane;
                slot[q] = -1;
                if (r < n_rows) {
                    const int32_t sl = dst_slots[(uint64_t)dst_tok0 + r];
                    if (sl < 0 || (uint64_t)(uint32_t)sl >= dst_rows) atomicOr(err, IRM_FLAG_ROW_RANGE);
                    else slot[q] = sl;
                }
            }
            const float2 *trig_hit = trig + (uint64_t)hit * IRM_KR_PAIRS;
            if (n_rows == TILE)
                reattach_tile<WAVES, RPW, true, NT_LD, NT_ST, F8>(sbase, src_stride, dbase, dst_stride, slot,
                                                                  n_rows, trig_hit, wave, lane, il);
            else
                reattach_tile<WAVES, RPW, false, NT_LD, NT_ST, F8>(sbase, src_stride, dbase, dst_stride, slot,
                                                                   n_rows, trig_hit, wave, lane, il);
        }
        cur = nxt;
        cur_layer = nxt_layer;
        x = xn;
    }
}

typedef void (*rows_kernel_t)(const void *const *, uint64_t, void *const *, uint64_t, uint64_t,
                              const int32_t *, const irm_tile *, const uint32_t *, const float2 *, uint32_t,
                              uint32_t, uint32_t, uint32_t *);

template <int WAVES, int RPW, bool F8>
static rows_kernel_t pick_mode(uint32_t mode)
{
    switch (mode & 3u) {
    case 0: return reattach_rows<WAVES, RPW, false, false, F8>;
    case 1: return reattach_rows<WAVES, RPW, true, false, F8>;
    case 2: return reattach_rows<WAVES, RPW, false, true, F8>;
    default: return reattach_rows<WAVES, RPW, true, true, F8>;
    }
}

template <int WAVES>
static rows_kernel_t pick_rpw(uint32_t rpw, uint32_t mode)
{
    switch (rpw) {
    case 1: return pick_mode<WAVES, 1, false>(mode);
    case 2: return pick_mode<WAVES, 2, false>(mode);
    case 4: return pick_mode<WAVES, 4, false>(mode);
    case 8: return pick_mode<WAVES, 8, false>(mode);
    default: return pick_mode<WAVES, 16, false>(mode);
    }
}

// fp8 rows: an even number of rows per wave, 4 waves or more (irm_ctx_tune admits no others)
template <int WAVES>
static rows_kernel_t pick_rpw_f8(uint32_t rpw, uint32_t mode)
{
    switch (rpw) {
    case 2: return pick_mode<WAVES, 2, true>(mode);
    case 4: return pick_mode<WAVES, 4, true>(mode);
    case 8: return pick_mode<WAVES, 8, true>(mode);
    default: return pick_mode<WAVES, 16, true>(mode);
    }
}

static rows_kernel_t pick_kernel(uint32_t waves, uint32_t rpw, uint32_t mode, uint32_t row_format)
{
    if (row_format == IRM_ROW_FP8) {
        switch (waves) {
        case 4: return pick_rpw_f8<4>(rpw, mode);
        case 8: return pick_rpw_f8<8>(rpw, mode);
        default: return pick_rpw_f8<16>(rpw, mode);
        }
    }
    switch (waves) {
    case 1: return pick_rpw<1>(rpw, mode);
    case 2: return pick_rpw<2>(rpw, mode);
    case 4: return pick_rpw<4>(rpw, mode);
    case 8: return pick_rpw<8>(rpw, mode);
    default: return pick_rpw<16>(rpw, mode);
    }
}

// ---- split-pool variant: only k_r is materialised (App. C "Split TokenToKVPool") ----
// Tile = up to 32 * Q rows of one hit, eight lanes per row, one 16-byte vector each.  The source is addressed by the k_r slice of its row 0 and a
// row stride, so it may be the k_r line of packed 1152-byte rows or a dense k_r_base
// pool of 128-byte rows.  c_KV is never read: the kernel only records which shared
// pool row each destination row refers to (once, by the layer-0 workgroups).
// A lane keeps its (cos, sin) values for Q rows: the table read is as large as two rows'
// worth of data, so a tile is 32 * Q rows.
// Grid (tile slots, layer groups): a row's k_r is only 128 bytes, so one tile and layer is a
// few KB, too little for a workgroup of its own (the dispatcher, not the memory, then sets
// the pace: 0.57 of peak).  A workgroup therefore keeps its tile for `lpw` layers: the tile
// record, the slots and the (cos, sin) values are fetched once, the rows of the next layer
// are requested before the current ones are rotated and stored.  The walk is kept short
// (three layers unless the caller sets it): every layer is another page.
template <int Q>
__global__ __launch_bounds__(256) void reattach_kr_rows(
    const void *const *__restrict__ src_ptrs, uint64_t src_stride, void *const *__restrict__ kr_ptrs,
    uint64_t kr_stride, uint64_t kr_rows, const int32_t *__restrict__ dst_slots,
    const irm_tile *__restrict__ tiles, const uint32_t *__restrict__ plan, const float2 *__restrict__ trig,
    int32_t *__restrict__ ckv_index, uint32_t n_layers, uint32_t lpw, uint32_t pair_mode, uint32_t xcd_ranges,
    uint32_t *err)
{
    // Lane l of a wave holds 16-byte vector v = l % 8 of row l / 8 (and of row 8 + l / 8):
    // a wave-wide access covers eight whole 128-byte rows, contiguous when the rows are.
    // Vectors 0..3 are the first halves of the pairs, 4..7 their partners, four lanes on.
    const uint32_t n_tiles = plan[0];
    const uint32_t lane = threadIdx.x & 63, wave = irm_wave_id();
    const uint32_t v = lane & 7, jq = v & 3;
    const float sgn = v < 4 ? -1.0f : 1.0f;            // first half: a c - b s; partner: b c + a s
    // which (tile, layer group) a workgroup serves: as in reattach_rows (xcd_ranges 2: a 1-D grid over the
    // launch's whole list of them, group-major, one contiguous eighth per XCD)
    const bool flat = xcd_ranges == 2;
    const uint32_t n_groups = (n_layers + lpw - 1) / lpw;
    const uint32_t n_items = flat ? n_tiles * n_groups : n_tiles;
    const uint32_t per_xcd = (n_items + 7) >> 3;
#pragma nounroll
    for (uint32_t x = blockIdx.x; x < per_xcd * 8; x += gridDim.x) {
        const uint32_t item = xcd_ranges ? (x & 7u) * per_xcd + (x >> 3) : x;
        if (item >= n_items) continue;
        const uint32_t group = flat ? item / n_tiles : blockIdx.y;
        const uint32_t ti = flat ? item - group * n_tiles : item;
        const uint32_t l0 = group * lpw, l1 = l0 + lpw < n_layers ? l0 + lpw : n_layers;
        const irm_tile *tp = tiles + ti;
        const uint32_t src_row0 = __builtin_amdgcn_readfirstlane(tp->src_row0);
        const uint32_t dst_tok0 = __builtin_amdgcn_readfirstlane(tp->dst_tok0);
        const uint32_t n_rows = __builtin_amdgcn_readfirstlane(tp->n_rows);
        const uint32_t hit = __builtin_amdgcn_readfirstlane(tp->hit);
        const f32x4 *tq = (const f32x4 *)(trig + (uint64_t)hit * IRM_KR_PAIRS + 8 * jq);
        const f32x4 t0 = tq[0], t1 = tq[1], t2 = tq[2], t3 = tq[3];
        int32_t slot[Q];
        bool on[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const uint32_t r = (wave * Q + q) * 8 + (lane >> 3);
            slot[q] = -1;
            on[q] = r < n_rows;
            if (on[q]) {
                const int32_t sl = dst_slots[(uint64_t)dst_tok0 + r];
                if (sl < 0 || (uint64_t)(uint32_t)sl >= kr_rows) {
                    if (v == 0 && l0 == 0) atomicOr(err, IRM_FLAG_ROW_RANGE);
                } else {
                    slot[q] = sl;
                    if (l0 == 0 && v == 0) ckv_index[sl] = (int32_t)(src_row0 + r);
                }
            }
        }
        // two layers' rows are on their way at any time (four were no faster)
        constexpr int D = 2;
        u32x4 buf[D][Q];
        auto fetch = [&](u32x4 (&into)[Q], uint32_t layer) {
            const char *base = (const char *)src_ptrs[layer];
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const uint32_t r = (wave * Q + q) * 8 + (lane >> 3);
                into[q] = u32x4{0, 0, 0, 0};
                if (on[q])
                    into[q] = __builtin_nontemporal_load((const u32x4 *)(base + (uint64_t)(src_row0 + r) * src_stride) + v);
            }
        };
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (l0 + d < l1) fetch(buf[d], l0 + d);
#pragma nounroll
        for (uint32_t layer = l0; layer < l1; layer += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (layer + d >= l1) break;
                char *out_base = (char *)kr_ptrs[layer + d];
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const u32x4 other = partner_vector(buf[d][q]);    // every lane takes part
                    if (slot[q] >= 0) {
                        const u32x4 out = pair_mode ? rotate_vector_pairs(buf[d][q], t0, t1, t2, t3, v >= 4)
                                                    : rotate_vector(buf[d][q], other, t0, t1, t2, t3, sgn);
                        __builtin_nontemporal_store(out, (u32x4 *)(out_base + (uint64_t)(uint32_t)slot[q] * kr_stride) + v);
                    }
                }
                if (layer + d + D < l1) fetch(buf[d], layer + d + D);
            }
        }
    }
}

extern "C" irm_status irm_reattach_kr(irm_ctx *ctx, const void *const *d_src_kr_layer_ptrs,
                                      uint64_t src_kr_row_stride_bytes, uint64_t src_rows,
                                      void *const *d_kr_layer_ptrs, uint64_t kr_row_stride_bytes,
                                      uint64_t kr_rows, int32_t *d_ckv_index, const int32_t *d_dst_slots,
                                      uint64_t n_slot_tokens, const irm_hit *d_hits,
                                      const uint32_t *d_n_hits, uint32_t hit_capacity, void *stream)
{
    if (!ctx || !d_src_kr_layer_ptrs || !d_kr_layer_ptrs || !d_ckv_index || !d_dst_slots || !d_hits ||
        !d_n_hits)
        return IRM_ERR_INVALID_ARG;
    if (src_kr_row_stride_bytes < IRM_KR_BYTES || kr_row_stride_bytes < IRM_KR_BYTES ||
        (src_kr_row_stride_bytes & 15) || (kr_row_stride_bytes & 15))
        return IRM_ERR_INVALID_ARG;
    if (src_rows < 1 || kr_rows < 1 || src_rows > 0x7FFFFFFFull || kr_rows > 0x7FFFFFFFull || n_slot_tokens < 1)
        return IRM_ERR_INVALID_ARG;
    if (hit_capacity < 1) return IRM_ERR_INVALID_ARG;
    if (hit_capacity > ctx->chunk_cap || n_slot_tokens > ctx->cfg.max_tokens) return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t kr_tile_rows = 32u * ctx->kr_rows_per_lane;
    hipLaunchKernelGGL(reattach_plan, dim3((hit_capacity + 7) / 8), dim3(256), 0, s, d_hits, d_n_hits,
                       hit_capacity, ctx->d_inv_freq, src_rows, n_slot_tokens, ctx->d_trig, ctx->d_tiles,
                       ctx->tile_cap, kr_tile_rows, ctx->cfg.pair_mode, ctx->d_plan, ctx->d_err);
    // as for the row kernel: slots for the tiles n_slot_tokens rows can fill, the overflow in a second pass
    uint64_t tile_slots = (n_slot_tokens + kr_tile_rows - 1) / kr_tile_rows;
    if (tile_slots > (1u << 24)) tile_slots = 1u << 24;
    // layers per workgroup: three, fewer while that leaves too few workgroups to fill the chip (about 16
    // per compute unit).  Every layer is a new page for the wave's source and destination, and a wave
    // that walks all layers misses the first-level translation cache once per layer and stream (the
    // second level is then busy 87 % of the time against 5 % for short walks) and runs at anything from
    // 0.62 to 0.76 of peak from one process to the next; walks of three layers give a steady 0.71-0.75,
    // one layer per workgroup 0.56-0.58 (too little work per workgroup).
    const uint32_t L = ctx->cfg.n_layers;
    uint32_t lpw = ctx->kr_layers_per_wg;
    if (!lpw) {
        const uint64_t want = 16ull * ctx->n_cu;
        lpw = tile_slots * L >= 3 * want ? 3u : (uint32_t)((tile_slots * L + want - 1) / want);
    }
    if (lpw < 1) lpw = 1;
    if (lpw > L) lpw = L;
    const bool sample = ctx->prof_events && ctx->prof_n < ctx->prof_cap &&
                        (ctx->prof_calls++ % ctx->prof_every) == 0;
    if (sample) IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n], s));
    void (*kr_kernel)(const void *const *, uint64_t, void *const *, uint64_t, uint64_t, const int32_t *,
                      const irm_tile *, const uint32_t *, const float2 *, int32_t *, uint32_t, uint32_t, uint32_t,
                      uint32_t, uint32_t *) =
        ctx->kr_rows_per_lane == 2 ? reattach_kr_rows<2>
        : ctx->kr_rows_per_lane == 4 ? reattach_kr_rows<4> : reattach_kr_rows<8>;
    // as for the row kernel: from 32 layers on one list over all layer groups, an eighth of it per XCD
    const uint32_t grid_x = (uint32_t)((tile_slots + 7) / 8 * 8), n_groups = (L + lpw - 1) / lpw;
    const bool want_flat = ctx->xcd_ranges == 2 || (ctx->xcd_ranges == 3 && L >= 32 && ctx->cfg.row_format == IRM_ROW_BF16);
    const bool flat = want_flat && ((uint64_t)ctx->tile_cap + 8) * n_groups < (1ull << 31) &&
                      (uint64_t)grid_x * n_groups < (1ull << 31);
    hipLaunchKernelGGL(kr_kernel, flat ? dim3(grid_x * n_groups) : dim3(grid_x, n_groups), dim3(256), 0, s,
                       d_src_kr_layer_ptrs, src_kr_row_stride_bytes, d_kr_layer_ptrs, kr_row_stride_bytes,
                       kr_rows, d_dst_slots, ctx->d_tiles, ctx->d_plan, ctx->d_trig, d_ckv_index, L, lpw,
                       ctx->cfg.pair_mode, flat ? 2u : (ctx->xcd_ranges ? 1u : 0u), ctx->d_err);
    if (sample) {
        IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n + 1], s));
        ++ctx->prof_n;
    }
    return irm_launch_status();
}

// ---- no-materialise variant (Sec. 7.2, App. C: rotation fused into the attention load path) ----
// Nothing of the KV is moved: every destination slot learns which pool row holds its
// (c_KV, k_r_base) and which hit's rotation applies; the per-hit (cos, sin) table goes to
// the caller's memory in pair order.  Tiles of up to 256 rows, one lane per row.
#define IRM_REF_TILE_ROWS 256u

__global__ __launch_bounds__(256) void reattach_ref_rows(uint64_t dst_rows, const int32_t *__restrict__ dst_slots,
                                                         const irm_tile *__restrict__ tiles,
                                                         const uint32_t *__restrict__ plan,
                                                         int32_t *__restrict__ row_index,
                                                         int32_t *__restrict__ hit_index, uint32_t *err)
{
    const uint32_t n_tiles = plan[0];
#pragma nounroll
    for (uint32_t ti = blockIdx.x; ti < n_tiles; ti += gridDim.x) {
        const irm_tile t = tiles[ti];
        if (threadIdx.x >= t.n_rows) continue;
        const int32_t sl = dst_slots[(uint64_t)t.dst_tok0 + threadIdx.x];
        if (sl < 0 || (uint64_t)(uint32_t)sl >= dst_rows) {
            atomicOr(err, IRM_FLAG_ROW_RANGE);
            continue;
        }
        row_index[sl] = (int32_t)(t.src_row0 + threadIdx.x);
        hit_index[sl] = (int32_t)t.hit;
    }
}

extern "C" irm_status irm_reattach_ref(irm_ctx *ctx, uint64_t src_rows, int32_t *d_row_index, int32_t *d_hit_index,
                                       uint64_t dst_rows, float *d_trig, const int32_t *d_dst_slots,
                                       uint64_t n_slot_tokens, const irm_hit *d_hits, const uint32_t *d_n_hits,
                                       uint32_t hit_capacity, void *stream)
{
    if (!ctx || !d_row_index || !d_hit_index || !d_trig || !d_dst_slots || !d_hits || !d_n_hits)
        return IRM_ERR_INVALID_ARG;
    if (src_rows < 1 || dst_rows < 1 || src_rows > 0x7FFFFFFFull || dst_rows > 0x7FFFFFFFull || n_slot_tokens < 1 ||
        hit_capacity < 1 || ((uintptr_t)d_trig & 7))
        return IRM_ERR_INVALID_ARG;
    if (hit_capacity > ctx->chunk_cap || n_slot_tokens > ctx->cfg.max_tokens) return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(reattach_plan, dim3((hit_capacity + 7) / 8), dim3(256), 0, s, d_hits, d_n_hits,
                       hit_capacity, ctx->d_inv_freq, src_rows, n_slot_tokens, (float2 *)d_trig, ctx->d_tiles,
                       ctx->tile_cap, IRM_REF_TILE_ROWS, IRM_PAIR_HALF_SPLIT, ctx->d_plan, ctx->d_err);
    uint64_t tile_slots = n_slot_tokens / IRM_REF_TILE_ROWS + hit_capacity;
    if (tile_slots > (1u << 20)) tile_slots = 1u << 20;
    const bool sample = ctx->prof_events && ctx->prof_n < ctx->prof_cap &&
                        (ctx->prof_calls++ % ctx->prof_every) == 0;
    if (sample) IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n], s));
    hipLaunchKernelGGL(reattach_ref_rows, dim3((uint32_t)tile_slots), dim3(256), 0, s, dst_rows, d_dst_slots,
                       ctx->d_tiles, ctx->d_plan, d_row_index, d_hit_index, ctx->d_err);
    if (sample) {
        IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n + 1], s));
        ++ctx->prof_n;
    }
    return irm_launch_status();
}

// launch shape of the row kernel and where its plan lives
struct rows_launch {
    uint32_t waves, rows_per_wave, mem_mode, xcd_ranges, grid, pair_mode, row_format, n_layers;
    float2 *d_trig;
    irm_tile *d_tiles;
    uint32_t tile_cap;
    uint32_t *d_plan, *d_err;
};

// host-side checks both entry points share
static irm_status reattach_check(uint32_t row_format, const void *const *d_src_layer_ptrs,
                                 uint64_t src_row_stride_bytes, uint64_t src_rows, void *const *d_dst_layer_ptrs,
                                 uint64_t dst_row_stride_bytes, uint64_t dst_rows, const int32_t *d_dst_slots,
                                 uint64_t n_slot_tokens, const irm_hit *d_hits, const uint32_t *d_n_hits,
                                 uint32_t hit_capacity)
{
    if (!d_src_layer_ptrs || !d_dst_layer_ptrs || !d_dst_slots || !d_hits || !d_n_hits) return IRM_ERR_INVALID_ARG;
    const uint32_t row_bytes = irm_row_bytes(row_format);
    if (src_row_stride_bytes < row_bytes || dst_row_stride_bytes < row_bytes ||
        (src_row_stride_bytes & 15) || (dst_row_stride_bytes & 15))
        return IRM_ERR_INVALID_ARG;
    if (src_rows < 1 || dst_rows < 1 || src_rows > 0xFFFFFFFFull || dst_rows > 0x7FFFFFFFull ||
        n_slot_tokens < 1)
        return IRM_ERR_INVALID_ARG;
    if (hit_capacity < 1) return IRM_ERR_INVALID_ARG;
    return IRM_OK;
}

// One workgroup per tile slot and layer: the hardware dispatcher balances the load (measured
// faster than a grid of resident size, whether it strides over the tiles or draws them from a
// device counter, and faster than workgroups that keep their tile for two or more layers).
// The tile count is only known on the device, so the grid covers the tiles that
// n_slot_tokens rows can fill; workgroups without a tile leave on their first compare (their
// number does not show in the launch time: 1,536 to 3,072 slots for 1,660 tiles per layer all
// take 276-278 us on the 32 K-token configuration); the ragged last tiles of the hits, if they
// overflow the grid, are taken by the first workgroups in a second pass.
static void rows_enqueue(const rows_launch &k, const void *const *d_src_layer_ptrs, uint64_t src_row_stride_bytes,
                         void *const *d_dst_layer_ptrs, uint64_t dst_row_stride_bytes, uint64_t dst_rows,
                         const int32_t *d_dst_slots, uint64_t n_slot_tokens, hipStream_t s)
{
    const uint32_t tile_rows = k.waves * k.rows_per_wave;
    uint64_t tile_slots = (n_slot_tokens + tile_rows - 1) / tile_rows;
    if (k.grid) tile_slots = k.grid;
    if (tile_slots > (1u << 24)) tile_slots = 1u << 24;
    const uint32_t grid_x = (uint32_t)((tile_slots + 7) / 8 * 8);
    // One list over all layers pays with many layers (61 layers: 3 to 5 % faster in every run, 54: 2 %;
    // 27 and fewer: from 4 % slower to 4 % faster between processes, 1 % slower on short requests), so
    // the library takes it from 32 layers on, if every index into the list fits 31 bits; else an
    // eighth of every layer per XCD.
    // (bf16 rows; over fp8 rows the per-layer eighths stay ahead at 61 layers too, 0.74-0.75 against 0.68-0.74)
    const bool want_flat = k.xcd_ranges == 2 || (k.xcd_ranges == 3 && k.n_layers >= 32 && k.row_format == IRM_ROW_BF16);
    const bool flat = want_flat && ((uint64_t)k.tile_cap + 8) * k.n_layers < (1ull << 31) &&
                      (uint64_t)grid_x * k.n_layers < (1ull << 31);
    const uint32_t ranges = flat ? 2u : (k.xcd_ranges ? 1u : 0u);
    hipLaunchKernelGGL(pick_kernel(k.waves, k.rows_per_wave, k.mem_mode, k.row_format),
                       flat ? dim3(grid_x * k.n_layers) : dim3(grid_x, k.n_layers), dim3(k.waves * 64), 0, s,
                       d_src_layer_ptrs, src_row_stride_bytes, d_dst_layer_ptrs, dst_row_stride_bytes, dst_rows,
                       d_dst_slots, k.d_tiles, k.d_plan, k.d_trig, ranges, k.n_layers, k.pair_mode, k.d_err);
}

extern "C" irm_status irm_reattach(irm_ctx *ctx, const void *const *d_src_layer_ptrs,
                                   uint64_t src_row_stride_bytes, uint64_t src_rows,
                                   void *const *d_dst_layer_ptrs, uint64_t dst_row_stride_bytes,
                                   uint64_t dst_rows, const int32_t *d_dst_slots, uint64_t n_slot_tokens,
                                   const irm_hit *d_hits, const uint32_t *d_n_hits, uint32_t hit_capacity,
                                   void *stream)
{
    if (!ctx) return IRM_ERR_INVALID_ARG;
    const irm_status st = reattach_check(ctx->cfg.row_format, d_src_layer_ptrs, src_row_stride_bytes, src_rows,
                                         d_dst_layer_ptrs, dst_row_stride_bytes, dst_rows, d_dst_slots,
                                         n_slot_tokens, d_hits, d_n_hits, hit_capacity);
    if (st != IRM_OK) return st;
    if (hit_capacity > ctx->chunk_cap || n_slot_tokens > ctx->cfg.max_tokens) return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const rows_launch k = {ctx->block_waves, ctx->rows_per_wave, ctx->mem_mode, ctx->xcd_ranges, ctx->reattach_grid,
                           ctx->cfg.pair_mode, ctx->cfg.row_format, ctx->cfg.n_layers,
                           ctx->d_trig, ctx->d_tiles, ctx->tile_cap, ctx->d_plan, ctx->d_err};
    hipLaunchKernelGGL(reattach_plan, dim3((hit_capacity + 7) / 8), dim3(256), 0, s, d_hits, d_n_hits, hit_capacity,
                       ctx->d_inv_freq, src_rows, n_slot_tokens, k.d_trig, k.d_tiles, k.tile_cap,
                       k.waves * k.rows_per_wave, k.pair_mode, k.d_plan, k.d_err);
    const bool sample = ctx->prof_events && ctx->prof_n < ctx->prof_cap &&
                        (ctx->prof_calls++ % ctx->prof_every) == 0;
    if (sample) IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n], s));
    rows_enqueue(k, d_src_layer_ptrs, src_row_stride_bytes, d_dst_layer_ptrs, dst_row_stride_bytes, dst_rows,
                 d_dst_slots, n_slot_tokens, s);
    if (sample) {
        IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n + 1], s));
        ++ctx->prof_n;
    }
    return irm_launch_status();
}

// ---- irm_reattach for callers that cannot allocate ----------------------------------------
// Same kernels; the plan (tile list, per-hit rotation table, tile count) lives in a static
// device array instead of a context's slab.  Every GPU holds its own copy of the array at
// its own address: the address is looked up once per device, with that device current, and
// host code only ever uses that pointer (the array's name is not a device address on the
// host side).  Nothing in the array has to start at zero: the plan kernel writes the tile
// count, the tiles and the table before the row kernel reads them.
#define IRM_STATIC_TILE_ROWS 16u     // 8 waves x 2 rows, the row kernel's default shape
#define IRM_STATIC_TILE_CAP (IRM_REATTACH_STATIC_MAX_TOKENS / IRM_STATIC_TILE_ROWS + IRM_REATTACH_STATIC_MAX_HITS)
#define IRM_STATIC_HEAD_BYTES 256u   // word 0: tile count; word 16: error word of callers that pass none
#define IRM_STATIC_TILES_BYTES (IRM_STATIC_TILE_CAP * 16u)
#define IRM_STATIC_TRIG_BYTES (IRM_REATTACH_STATIC_MAX_HITS * IRM_KR_PAIRS * 8u)
#define IRM_STATIC_BYTES (IRM_STATIC_HEAD_BYTES + IRM_STATIC_TILES_BYTES + IRM_STATIC_TRIG_BYTES)
#define IRM_STATIC_MAX_DEVICES 64

static __device__ __align__(256) unsigned char scratch[IRM_STATIC_BYTES];

#include <mutex>
static std::mutex g_static_lock;
static unsigned char *g_static_ptr[IRM_STATIC_MAX_DEVICES];   // per device: where `scratch` lives there

// device address of this device's copy of `scratch` (first call on a device looks it up)
static irm_status static_scratch(unsigned char **out)
{
    int device = -1;
    IRM_HIP_TRY(hipGetDevice(&device));
    if (device < 0 || device >= IRM_STATIC_MAX_DEVICES) return IRM_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_static_lock);
    if (!g_static_ptr[device]) {
        unsigned char *ptr = nullptr;
        IRM_HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return IRM_ERR_DEVICE;
        g_static_ptr[device] = ptr;
    }
    *out = g_static_ptr[device];
    return IRM_OK;
}

extern "C" irm_status irm_reattach_static(const float *inv_freq, uint32_t n_layers, uint32_t pair_mode,
                                          uint32_t row_format, const void *const *d_src_layer_ptrs,
                                          uint64_t src_row_stride_bytes, uint64_t src_rows,
                                          void *const *d_dst_layer_ptrs, uint64_t dst_row_stride_bytes,
                                          uint64_t dst_rows, const int32_t *d_dst_slots, uint64_t n_slot_tokens,
                                          const irm_hit *d_hits, const uint32_t *d_n_hits, uint32_t hit_capacity,
                                          uint32_t *d_error_flags, void *stream)
{
    if (!inv_freq) return IRM_ERR_INVALID_ARG;
    if (pair_mode > IRM_PAIR_INTERLEAVED || row_format > IRM_ROW_FP8) return IRM_ERR_UNSUPPORTED;
    if (n_layers < 1 || n_layers > 4096) return IRM_ERR_INVALID_ARG;
    irm_freq32 freq;
    for (int i = 0; i < IRM_KR_PAIRS; ++i) {
        if (!(inv_freq[i] == inv_freq[i]) || inv_freq[i] - inv_freq[i] != 0.0f) return IRM_ERR_INVALID_ARG;
        freq.v[i] = inv_freq[i];
    }
    const irm_status st = reattach_check(row_format, d_src_layer_ptrs, src_row_stride_bytes, src_rows,
                                         d_dst_layer_ptrs, dst_row_stride_bytes, dst_rows, d_dst_slots,
                                         n_slot_tokens, d_hits, d_n_hits, hit_capacity);
    if (st != IRM_OK) return st;
    if (n_slot_tokens > IRM_REATTACH_STATIC_MAX_TOKENS || hit_capacity > IRM_REATTACH_STATIC_MAX_HITS)
        return IRM_ERR_CAPACITY;                        // beyond what the static array was sized for
    unsigned char *base = nullptr;
    const irm_status got = static_scratch(&base);
    if (got != IRM_OK) return got;
    hipStream_t s = (hipStream_t)stream;
    uint32_t *plan = (uint32_t *)base;
    uint32_t *err = d_error_flags ? d_error_flags : (uint32_t *)base + 16;
    // fp8 rows share 128-byte lines with their neighbours: cached accesses (as in a context)
    const rows_launch k = {8u, 2u, row_format == IRM_ROW_FP8 ? 0u : 3u, 3u, 0u, pair_mode, row_format, n_layers,
                           (float2 *)(base + IRM_STATIC_HEAD_BYTES + IRM_STATIC_TILES_BYTES),
                           (irm_tile *)(base + IRM_STATIC_HEAD_BYTES), IRM_STATIC_TILE_CAP, plan, err};
    hipLaunchKernelGGL(reattach_plan_byval, dim3((hit_capacity + 7) / 8), dim3(256), 0, s, d_hits, d_n_hits,
                       hit_capacity, freq, src_rows, n_slot_tokens, k.d_trig, k.d_tiles, k.tile_cap,
                       IRM_STATIC_TILE_ROWS, pair_mode, k.d_plan, k.d_err);
    rows_enqueue(k, d_src_layer_ptrs, src_row_stride_bytes, d_dst_layer_ptrs, dst_row_stride_bytes, dst_rows,
                 d_dst_slots, n_slot_tokens, s);
    return irm_launch_status();
}
