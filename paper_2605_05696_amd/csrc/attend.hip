// Consumer of the no-materialise variant (paper Sec. 2 "MLA"; Sec. 7.2 and App. C: the
// delta-rotation fused into the attention kernel's load path): MLA decode attention in the
// latent form, one layer, reading (c_KV, k_r_base) rows of the shared pool through the
// per-slot references irm_reattach_ref wrote and rotating k_r by the hit's R(delta) while
// the rows are staged, so no rotated copy ever exists in HBM.
//
//   score[b][h][t] = scale * q[b][h] . [ c_KV(row_t) | R_t k_r_base(row_t) ]
//   out[b][h]      = sum_t softmax_t(score) c_KV(row_t)
//
//   attend_ref_split   grid (head groups of 16, splits, requests), 8 waves.  A workgroup walks
//       its share of the request's tokens in tiles of 64.  Four waves fetch: the tile's 64
//       rows (1152 B each) come from HBM into registers with 16-byte loads, k_r is rotated
//       there (fp32, one rounding to bf16: the same values the materialising kernel writes)
//       and the tile lands in one of two LDS buffers.  Four waves compute on the other buffer
//       without a word to each other; two of them share 32 of the tile's 64 tokens and split the
//       512 latent dims of the output:
//         S^T = K Q^T   32 tokens x 16 heads, 36 MFMA 16x16x32 (bf16 in, fp32 acc): a staged row
//                       is an A operand as it lies, Q lives in registers as B operands (both
//                       waves of a pair compute the same scores: cheaper than sharing them)
//         online softmax over its tokens (the running maximum per head lives in the lanes)
//         O^T += V^T P^T   256 latent dims x 16 heads over the 32 tokens, 16 MFMA: the softmax'd
//                       S^T registers are the B operand as they are, V^T comes through transposing
//                       LDS reads (column pieces of the row-major tile)
//       At the end the two token groups' (max, sum, O) meet once in LDS.  Every KV byte is read
//       from HBM once per head group.
//       With a multiple of 64 heads a workgroup serves four head groups instead, one per
//       compute wave, each wave on all 64 tokens and all 512 dims of a tile: a row is then read
//       from HBM once per 64 heads (a multiple of 32: two groups, two waves each).
//       Pools of fp8 rows (F8: 512 E4M3 codes | four fp32 block scales | k_r) differ in the fetch
//       waves only, up to the block scales, which the compute waves apply (several groups: the fetch waves).
//   attend_ref_merge   combines the splits' (max, sum, O) into out and lse.
#include "irm_internal.hpp"

#define ATT_TILE 64u                   // tokens per tile
#define ATT_KROW 584u                  // bf16 per staged row: 576 + 8 of padding (1168 B)
#define ATT_OROW 516u                  // floats per head of a partial output in LDS: 512 + 4 of padding
#define ATT_HEADS 16u                  // heads per workgroup
#define ATT_KSTEPS 18                  // 576 / 32
#define ATT_RING 8u                    // tiles whose references are kept in LDS (published five tiles ahead)
#define ATT_LOG2E 1.4426950408889634f

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// LDS read with transpose (ds_read_b64_tr_b16).  Within a block of 16 lanes, lane s points at four
// consecutive 16-bit elements; lane i receives, as element j, element (i & 3) of the four that lane
// 4 j + (i >> 2) pointed at.  With lane s pointing at M[r0 + (s >> 2)][c0 + 4 (s & 3) ..] of a
// row-major matrix, lane i ends up with the column piece M[r0 .. r0 + 3][c0 + i].
__device__ __forceinline__ s16x4 att_lds_read_tr(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
}

__device__ __forceinline__ float att_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float att_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t att_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

struct att_smem {
    uint16_t k[2][ATT_TILE * ATT_KROW]; // staged rows, k_r rotated: the tile in work and the next one;
                                        // at the end the compute waves' partial outputs (fp32)
    float wmax[4 * ATT_HEADS];          // per token group (or compute wave) and head: running maximum at the end
    float wsum[4 * ATT_HEADS];          // ... and sum
    int32_t row[ATT_RING][ATT_TILE];    // pool row of each tile token, -1 = no token; slot = tile mod ATT_RING
    int32_t hit[ATT_RING][ATT_TILE];    // rotation of each tile token, -1 = none
    uint32_t landed[4];                 // per fetch wave: tiles it has landed so far
    uint32_t consumed[4];               // per compute wave: tiles it is done with
};

// Barrier that orders LDS traffic only: global loads issued before it stay in flight.
#define ATT_SYNC()                                                          \
    do {                                                                    \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");     \
        __builtin_amdgcn_s_barrier();                                       \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");     \
    } while (0)

// Hand-over between the halves, through LDS counters that only grow: a fetch wave adds one to
// its own `landed` entry per tile it has stored, a compute wave one to its own `consumed` entry
// per tile it is done with.  Nobody waits at a common point: the fetch waves drift apart and HBM
// sees a steady stream instead of four waves' loads in lockstep, and the compute waves never wait
// for each other at all.  Waves of one half may therefore be a tile or more apart, so a sum over
// them would not say that a tile is whole (or wholly worked off): whoever waits, waits for the
// slowest of the four counters.  A wait is bounded: a wave that gives up raises
// IRM_FLAG_WAIT_TIMEOUT and carries on, so every wave reaches the end of the kernel.  Whatever
// a wave then finds in LDS is harmless to follow: every reference slot of the ring holds checked
// values from the prologue on (a row inside the pool or "no token"), tile data is only ever
// multiplied, and every global address comes from a checked reference.
__device__ __forceinline__ void att_signal(uint32_t *counter, uint32_t lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    if (lane == 0) __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void att_wait_all(uint32_t *counters, uint32_t target, uint32_t lane, uint32_t *err,
                                             uint32_t spin_limit)
{
    uint32_t spins = 0;
    for (;;) {
        uint32_t least = __hip_atomic_load(counters, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const uint32_t v = __hip_atomic_load(counters + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            least = (int32_t)(v - least) < 0 ? v : least;
        }
        if ((int32_t)(least - target) >= 0) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > spin_limit) {
            if (lane == 0) atomicOr(err, IRM_FLAG_WAIT_TIMEOUT);
            break;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- fetch half: waves 4..7 -------------------------------------------------------------------
// A fetch lane holds, of a tile's 64 rows: c_KV vector `lane` of rows cw + 4j (a wave reads whole
// 1024-byte c_KV spans), and the two k_r vectors that hold pair partners of row ct / 4.  One
// tile per wave is on its way at any time, requested a whole tile's time before it is needed
// (measured: 18 loads in flight per lane of four waves per compute unit stream 7.2 TB/s, twice
// as many per lane only 4.2).  There is no branch around a load.
struct att_args {
    const char *pool;
    uint64_t pool_stride;
    const float2 *trig;
    uint32_t pair_mode;
};

// fp8 rows (512 E4M3 codes | four fp32 scales | k_r): the codes of a row are 32 vectors, so half a
// wave takes a row and one load covers two; a lane also fetches the scale of the block of 128 its
// 16 codes lie in.  10 + 8 loads per lane and tile instead of 18, for 656 bytes a row.
#define ATT_NV(F8) ((F8) ? 10 : ATT_KSTEPS)

// Where a lane's loads of one tile go: worked out from the tile's references a tile ahead of the
// loads themselves, so that a wave whose registers have just been emptied has its next requests on
// the way within a few instructions (measured: reading the references and forming the addresses
// took a quarter of a tile's time, during which the wave had nothing in flight).
template <bool F8>
struct att_addr {
    const char *row[F8 ? 8 : 16];       // this lane's 16 bytes of each of its rows (an absent token: row 0)
    const u32x4 *kr;                    // the k_r line of the row this lane rotates a part of
    const f32x4 *trig;                  // that row's (cos, sin) for this lane's pairs
    int32_t hit;
};

template <bool F8>
__device__ __forceinline__ void att_addr_rows(att_addr<F8> &ad, const att_smem *sm, uint32_t slot,
                                              const att_args &a, uint32_t cw, uint32_t lane, uint32_t ct)
{
    if (F8) {
        const uint32_t sub = lane >> 5, vec = lane & 31u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int32_t row = sm->row[slot][cw + 4u * (2u * (uint32_t)i + sub)];
            const uint32_t safe = row >= 0 ? (uint32_t)row : 0u;
            ad.row[i] = a.pool + (uint64_t)safe * a.pool_stride + 16u * vec;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int32_t row = sm->row[slot][cw + 4u * (uint32_t)j];
            const uint32_t safe = row >= 0 ? (uint32_t)row : 0u;
            ad.row[j] = a.pool + (uint64_t)safe * a.pool_stride + 16u * lane;
        }
    }
    const int32_t row = sm->row[slot][ct >> 2];
    const uint32_t safe = row >= 0 ? (uint32_t)row : 0u;
    ad.kr = (const u32x4 *)(a.pool + (uint64_t)safe * a.pool_stride + (F8 ? IRM_F8_CKV_BYTES : IRM_CKV_BYTES));
    ad.hit = sm->hit[slot][ct >> 2];
    const uint32_t hsafe = ad.hit >= 0 ? (uint32_t)ad.hit : 0u;     // entry 0 always exists
    ad.trig = (const f32x4 *)(a.trig + (uint64_t)hsafe * IRM_KR_PAIRS + 8u * (ct & 3u));
}

// request a tile: the (cos, sin) first (the landing needs them no later than the rows), then the rows
// NT: streaming loads, for rows that nobody else reads soon (one group of 16 heads); with several head
// groups the same rows are read once per group by workgroups dispatched together, and cached loads let
// the later ones find them on chip (128 heads: 1657 -> 1356 us per layer; 16 heads: 3 % slower).
template <bool NT>
__device__ __forceinline__ u32x4 att_ld(const u32x4 *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <bool F8, bool NT>
__device__ __forceinline__ int32_t att_fire_rows(u32x4 (&vc)[ATT_NV(F8)], float (&sc)[8], f32x4 (&t4)[4],
                                                 const att_addr<F8> &ad, const att_args &a, uint32_t lane,
                                                 uint32_t ct)
{
#pragma unroll
    for (int w = 0; w < 4; ++w) t4[w] = ad.trig[w];         // (c, s, c, s) of two pairs each
    if (F8) {
        const uint32_t vec = lane & 31u;
        const int32_t to_scale = 512 + 4 * (int32_t)(vec >> 3) - 16 * (int32_t)vec;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            vc[i] = att_ld<NT>((const u32x4 *)ad.row[i]);
            sc[i] = *(const float *)(ad.row[i] + to_scale);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) vc[j] = att_ld<NT>((const u32x4 *)ad.row[j]);
    }
    constexpr int KA = F8 ? 8 : 16;
    const uint32_t kj = ct & 3u;
    // half-split: elements 8 kj .. and their partners; interleaved: pairs 8 kj .. 8 kj + 7, whole
    const uint32_t ia = a.pair_mode == IRM_PAIR_HALF_SPLIT ? kj : 2u * kj;
    const uint32_t ib = a.pair_mode == IRM_PAIR_HALF_SPLIT ? 4u + kj : 2u * kj + 1u;
    vc[KA] = att_ld<NT>(ad.kr + ia);
    vc[KA + 1] = att_ld<NT>(ad.kr + ib);
    return ad.hit;
}

// 16 E4M3 codes as bf16, exactly (three fraction bits fit): two 16-byte vectors.  The block scales
// are not applied here but by the compute waves, to the score sums of a block in fp32 and to the
// softmax numerators: one conversion per two codes is all the fetch waves spend (with the multiply
// and the rounding here, they were what bounded the kernel).  The scaled conversion takes only the
// exponent of its scale operand (measured), so it is used with 1.
typedef __bf16 att_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void att_codes16(u32x4 codes, u32x4 &lo, u32x4 &hi)
{
    const uint32_t w[4] = {codes.x, codes.y, codes.z, codes.w};
    uint32_t o[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        o[2 * k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)w[k], 1.0f, false));
        o[2 * k + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)w[k], 1.0f, true));
    }
    lo = u32x4{o[0], o[1], o[2], o[3]};
    hi = u32x4{o[4], o[5], o[6], o[7]};
}

// 16 E4M3 codes times their block's scale, rounded once to bf16 (for the variant whose compute waves
// are the busier half and take the tile as if it came from bf16 rows)
typedef float att_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void att_dequant16(u32x4 codes, float scale, u32x4 &lo, u32x4 &hi)
{
    const uint32_t w[4] = {codes.x, codes.y, codes.z, codes.w};
    uint32_t o[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        att_f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[k], false);    // codes 0, 1 of the word
        att_f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[k], true);     // codes 2, 3
        a *= scale;
        b *= scale;
        o[2 * k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, att_bf16x2));
        o[2 * k + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, att_bf16x2));
    }
    lo = u32x4{o[0], o[1], o[2], o[3]};
    hi = u32x4{o[4], o[5], o[6], o[7]};
}

// rotate k_r in registers (fp32, one rounding to bf16), store the tile into LDS buffer `buf`;
// FOLD (fp8 rows): leave the block scales to the compute waves
template <bool F8, bool FOLD>
__device__ __forceinline__ void att_land_rows(u32x4 (&vc)[ATT_NV(F8)], const float (&sc)[8], const f32x4 (&t4)[4],
                                              int32_t hit, att_smem *sm, uint32_t slot, uint32_t buf,
                                              const att_args &a, uint32_t cw, uint32_t lane, uint32_t ct)
{
    constexpr int KA = F8 ? 8 : 16;
    u32x4 va = vc[KA], vb = vc[KA + 1];
    const uint32_t kr_row = ct >> 2, kj = ct & 3u;
    if (hit >= 0) {
        if (a.pair_mode == IRM_PAIR_HALF_SPLIT) {
            uint32_t aw[4] = {va.x, va.y, va.z, va.w}, bw[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float a0 = att_bf16_lo(aw[w]), a1 = att_bf16_hi(aw[w]);
                const float b0 = att_bf16_lo(bw[w]), b1 = att_bf16_hi(bw[w]);
                const float c0 = t4[w].x, s0 = t4[w].y, c1 = t4[w].z, s1 = t4[w].w;
                aw[w] = att_to_bf16(a0 * c0 - b0 * s0) | (att_to_bf16(a1 * c1 - b1 * s1) << 16);
                bw[w] = att_to_bf16(b0 * c0 + a0 * s0) | (att_to_bf16(b1 * c1 + a1 * s1) << 16);
            }
            va = u32x4{aw[0], aw[1], aw[2], aw[3]};
            vb = u32x4{bw[0], bw[1], bw[2], bw[3]};
        } else {                                            // one word = one pair (a, b)
            uint32_t w8[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                const float a0 = att_bf16_lo(w8[w]), b0 = att_bf16_hi(w8[w]);
                const float c0 = (w & 1) ? t4[w >> 1].z : t4[w >> 1].x;
                const float s0 = (w & 1) ? t4[w >> 1].w : t4[w >> 1].y;
                w8[w] = att_to_bf16(a0 * c0 - b0 * s0) | (att_to_bf16(b0 * c0 + a0 * s0) << 16);
            }
            va = u32x4{w8[0], w8[1], w8[2], w8[3]};
            vb = u32x4{w8[4], w8[5], w8[6], w8[7]};
        }
    }
    uint16_t *kt = sm->k[buf];
    const u32x4 zero = {0, 0, 0, 0};
    // two base addresses, the rest are immediate offsets of the LDS stores
    if (F8) {
        // the codes staged as bf16 in the bf16 rows' layout; the four block scales of a row go into the
        // 16 bytes of padding behind its 576 elements
        const uint32_t sub = lane >> 5, vec = lane & 31u;
        uint16_t *at = kt + (cw + 4u * sub) * ATT_KROW + vec * 16u;
        float *scale_at = (float *)(kt + (cw + 4u * sub) * ATT_KROW + 576u) + (vec >> 3);
        const int32_t *rows = sm->row[slot] + cw + 4u * sub;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            u32x4 w0, w1;
            if (FOLD) att_codes16(vc[i], w0, w1);
            else att_dequant16(vc[i], sc[i], w0, w1);
            const bool live = rows[8 * i] >= 0;
            *(u32x4 *)(at + 8 * i * ATT_KROW) = live ? w0 : zero;
            *(u32x4 *)(at + 8 * i * ATT_KROW + 8) = live ? w1 : zero;
            if (FOLD && (vec & 7u) == 0) scale_at[8 * i * (ATT_KROW / 2)] = live ? sc[i] : 0.0f;
        }
    } else {
        uint16_t *lo = kt + cw * ATT_KROW + lane * 8u, *hi = lo + 32u * ATT_KROW;
        const int32_t *rows = sm->row[slot] + cw;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            *(u32x4 *)(lo + 4 * j * ATT_KROW) = rows[4 * j] >= 0 ? vc[j] : zero;
            *(u32x4 *)(hi + 4 * j * ATT_KROW) = rows[32 + 4 * j] >= 0 ? vc[8 + j] : zero;
        }
    }
    if (sm->row[slot][kr_row] < 0) {
        va = zero;
        vb = zero;
    }
    uint16_t *kr = kt + kr_row * ATT_KROW + IRM_CKV_BYTES / 2;
    if (a.pair_mode == IRM_PAIR_HALF_SPLIT) {
        *(u32x4 *)(kr + 8 * kj) = va;
        *(u32x4 *)(kr + 32 + 8 * kj) = vb;
    } else {
        *(u32x4 *)(kr + 16 * kj) = va;
        *(u32x4 *)(kr + 16 * kj + 8) = vb;
    }
}

// 8 waves: waves 0..3 compute, waves 4..7 fetch; each half runs its own loop (so that each gets
// the whole register file for what it alone needs) and both meet at the same barriers: two in
// the prologue and one at the end; in between the halves hand tiles over through LDS counters.
// While the compute waves work on tile i in one LDS buffer, the fetch waves land tile i + 1,
// requested a tile ago, in the other buffer as its rows arrive, and request tile i + 2 right after.
// GPW, head groups per workgroup.  1: the four compute waves share one group's tile as described above.
// 4: one group per compute wave, each wave on all 64 tokens of a tile: the tile is fetched and staged
// once for 64 heads (models with 64 or 128 heads), no wave needs anything from another, and the kernel is
// bound by the LDS reads of the operands instead of HBM.  2: two waves per group, 32 tokens of the tile
// each, their results joined at the end (32 heads per pass).
template <bool F8, bool NT, int GPW>
__global__ __launch_bounds__(512) void attend_ref_split(
    const uint16_t *__restrict__ q, uint32_t n_heads, const char *__restrict__ pool, uint64_t pool_stride,
    uint64_t pool_rows, const int32_t *__restrict__ kv_slots, const uint32_t *__restrict__ kv_offsets,
    const int32_t *__restrict__ row_index, const int32_t *__restrict__ hit_index, uint64_t dst_rows,
    const float2 *__restrict__ trig, uint32_t trig_hits, float scale_log2, uint32_t pair_mode,
    float *__restrict__ part_o, float2 *__restrict__ part_ml, uint32_t spin_limit, uint32_t *err)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    att_smem *sm = (att_smem *)smem_raw;
    // head groups vary fastest: the workgroups that read the same rows are dispatched together
    const uint32_t split = blockIdx.y, n_splits = gridDim.y;
    constexpr bool MULTI = GPW > 1;
    const uint32_t n_groups = (uint32_t)GPW * gridDim.x;
    // head group of this workgroup; with several, of this compute wave (read by compute waves only)
    const uint32_t group = GPW == 4 ? 4u * blockIdx.x + (irm_wave_id() & 3u)
                           : GPW == 2 ? 2u * blockIdx.x + ((irm_wave_id() & 3u) >> 1) : blockIdx.x;
    const uint32_t b = blockIdx.z;
    const uint32_t lane = threadIdx.x & 63, wave = irm_wave_id();
    const bool fetcher = wave >= 4;                         // uniform per wave
    const uint32_t cw = wave & 3u;                          // index among the waves of its half
    const uint32_t ct = threadIdx.x & 255u;                 // lane index within its half
    const uint32_t begin = kv_offsets[b], end = kv_offsets[b + 1];
    if (end < begin && threadIdx.x == 0) atomicOr(err, IRM_FLAG_BAD_CHUNK);   // offsets that run backwards: no context
    const uint32_t n_tok = end >= begin ? end - begin : 0u;
    const uint32_t n_tiles = (n_tok + ATT_TILE - 1) / ATT_TILE;
    const uint32_t per_split = (n_tiles + n_splits - 1) / n_splits;
    const uint32_t tile0 = split * per_split;
    const uint32_t tile1 = tile0 + per_split < n_tiles ? tile0 + per_split : n_tiles;
    const uint64_t part = ((uint64_t)b * n_groups + group) * n_splits + split;
    if (tile0 >= tile1) {                                   // nothing for this split (uniform exit)
        for (uint32_t g = 0; g < (uint32_t)GPW; ++g) {
            const uint64_t pg = ((uint64_t)b * n_groups + (uint32_t)GPW * blockIdx.x + g) * n_splits + split;
            float *po = part_o + pg * (ATT_HEADS * 512u);
            for (uint32_t i = threadIdx.x; i < ATT_HEADS * 512u; i += blockDim.x) po[i] = 0.0f;
            if (threadIdx.x < ATT_HEADS) part_ml[pg * ATT_HEADS + threadIdx.x] = make_float2(-INFINITY, 0.0f);
        }
        return;
    }
    // tiles are taken two at a time; an odd count is padded by a tile without tokens (its
    // references are -1: it reads row 0, lands zeros and counts for nothing)
    const uint32_t n_pairs = (tile1 - tile0 + 1u) >> 1;
    if (threadIdx.x == 0) {
        for (int w = 0; w < 4; ++w) {
            sm->landed[w] = 0;
            sm->consumed[w] = 0;
        }
    }

    if (fetcher) {
        const att_args a = {pool, pool_stride, trig, pair_mode};
        constexpr uint32_t RM = ATT_RING - 1u;
        u32x4 r[ATT_NV(F8)];
        float sc[8];
        f32x4 t4[4];
        att_addr<F8> ad;
        ATT_SYNC();                                         // prologue 1: references of tiles 0..4 published
        att_addr_rows<F8>(ad, sm, 0, a, cw, lane, ct);
        int32_t hit = att_fire_rows<F8, NT>(r, sc, t4, ad, a, lane, ct);
        att_addr_rows<F8>(ad, sm, 1, a, cw, lane, ct);
        if (F8) {
            // Rows of 656 bytes: one tile per wave is only 42 KB on its way per compute unit, too little
            // for the memory latency, so a wave keeps two tiles in flight in two register sets.  Tile
            // t + 2 is requested right after tile t has landed.
            u32x4 r2[ATT_NV(F8)];
            float sc2[8];
            f32x4 t42[4];
            int32_t hit2 = att_fire_rows<F8, NT>(r2, sc2, t42, ad, a, lane, ct);
            att_addr_rows<F8>(ad, sm, 2, a, cw, lane, ct);
            att_land_rows<F8, F8 && !MULTI>(r, sc, t4, hit, sm, 0, 0, a, cw, lane, ct);
            hit = att_fire_rows<F8, NT>(r, sc, t4, ad, a, lane, ct);
            att_addr_rows<F8>(ad, sm, 3, a, cw, lane, ct);
            ATT_SYNC();                                     // prologue 2: counters are zero, tile 0 is in place
            att_signal(&sm->landed[cw], lane);
            uint32_t t = 1;                                 // t = tile - tile0; odd tiles use the second set
            for (; t + 1u < 2u * n_pairs; t += 2u) {
                att_wait_all(sm->consumed, t - 1u, lane, err, spin_limit);
                att_land_rows<F8, F8 && !MULTI>(r2, sc2, t42, hit2, sm, t & RM, 1u, a, cw, lane, ct);
                att_signal(&sm->landed[cw], lane);
                hit2 = att_fire_rows<F8, NT>(r2, sc2, t42, ad, a, lane, ct);           // tile t + 2
                att_addr_rows<F8>(ad, sm, (t + 3u) & RM, a, cw, lane, ct);
                att_wait_all(sm->consumed, t, lane, err, spin_limit);
                att_land_rows<F8, F8 && !MULTI>(r, sc, t4, hit, sm, (t + 1u) & RM, 0u, a, cw, lane, ct);
                att_signal(&sm->landed[cw], lane);
                hit = att_fire_rows<F8, NT>(r, sc, t4, ad, a, lane, ct);               // tile t + 3
                att_addr_rows<F8>(ad, sm, (t + 4u) & RM, a, cw, lane, ct);
            }
            att_wait_all(sm->consumed, t - 1u, lane, err, spin_limit);  // the last tile, 2 n_pairs - 1: odd
            att_land_rows<F8, F8 && !MULTI>(r2, sc2, t42, hit2, sm, t & RM, 1u, a, cw, lane, ct);
            att_signal(&sm->landed[cw], lane);
        } else {
            att_land_rows<F8, F8 && !MULTI>(r, sc, t4, hit, sm, 0, 0, a, cw, lane, ct);
            hit = att_fire_rows<F8, NT>(r, sc, t4, ad, a, lane, ct);                   // tile 1
            att_addr_rows<F8>(ad, sm, 2, a, cw, lane, ct);
            ATT_SYNC();                                     // prologue 2: counters are zero, tile 0 is in place
            att_signal(&sm->landed[cw], lane);
            for (uint32_t t = 1; t < 2u * n_pairs; ++t) {   // t = tile - tile0
                // Tile t goes into the buffer tile t - 2 was worked off from.  Request t + 1 at once
                // after landing t, so that it has a whole tile's time to arrive (more than 18 loads
                // in flight per lane slow the stream down: measured).
                att_wait_all(sm->consumed, t - 1u, lane, err, spin_limit);
                att_land_rows<F8, F8 && !MULTI>(r, sc, t4, hit, sm, t & RM, t & 1u, a, cw, lane, ct);
                att_signal(&sm->landed[cw], lane);
                hit = att_fire_rows<F8, NT>(r, sc, t4, ad, a, lane, ct);               // tile t + 1
                att_addr_rows<F8>(ad, sm, (t + 2u) & RM, a, cw, lane, ct);
            }
        }
        __syncthreads();                                    // every tile worked off
        __syncthreads();                                    // the compute waves' merge, two steps
        __syncthreads();
        return;
    }

    // ---- compute half: waves 0..3 -------------------------------------------------------------
    const uint32_t lm = lane & 15, lq = lane >> 4;          // MFMA coordinates of this lane
    // References (slot -> pool row, rotation): lanes 0..15 of wave cw for tokens 16 cw .. + 15 of a
    // tile.  The two dependent loads are spread over three tiles' time so that nobody waits for
    // them: during tile i the slot ids of tile i + 7 are requested, the rows and rotations of
    // tile i + 6 (whose slot ids came in during tile i - 1) are requested into one register
    // pair, and those of tile i + 5, requested a tile ago into the other pair, are checked and
    // published: a fetch wave that has landed tile t (every compute wave is done with t - 2
    // then) finds the references up to tile t + 3.  Slot = tile mod ATT_RING.
    const uint32_t ref_tok = 16u * cw + lane;               // meaningful for lane < 16
    auto refs_slot = [&](uint32_t tile) -> int32_t {
        if (lane >= 16u || tile >= tile1) return -1;
        const uint32_t t0 = begin + tile * ATT_TILE;
        if (ref_tok >= end - t0) return -1;
        return kv_slots[(uint64_t)t0 + ref_tok];
    };
    auto refs_rows = [&](uint32_t tile, int32_t sl, int32_t &row, int32_t &hit) {   // request only
        row = -2;                                           // the token does not exist
        hit = -1;
        if (lane >= 16u || tile >= tile1 || ref_tok >= end - (begin + tile * ATT_TILE)) return;
        row = -3;                                           // a token whose slot is out of range
        if (sl >= 0 && (uint64_t)(uint32_t)sl < dst_rows) {
            row = row_index[sl];
            hit = hit_index[sl];
        }
    };
    auto refs_publish = [&](uint32_t slot, int32_t row, int32_t hit) {
        if (row == -2) {
            row = -1;
        } else if (row < 0 || (uint64_t)(uint32_t)row >= pool_rows || hit >= (int32_t)trig_hits) {
            atomicOr(err, IRM_FLAG_ROW_RANGE);              // the token is left out of the attention
            row = -1;
        }
        if (lane < 16u) {
            sm->row[slot][ref_tok] = row;
            sm->hit[slot][ref_tok] = hit < 0 ? -1 : hit;
        }
    };
    // Q as B operands of S^T = K Q^T: lane holds Q[head lm][32 kk + 8 lq .. + 8] for every k-step
    u16x8 qb[ATT_KSTEPS];
    {
        const uint16_t *qrow = q + ((uint64_t)b * n_heads + group * ATT_HEADS + lm) * 576u;
#pragma unroll
        for (int kk = 0; kk < ATT_KSTEPS; ++kk) qb[kk] = *(const u16x8 *)(qrow + 32 * kk + 8 * lq);
    }
    if constexpr (MULTI) {
        // this wave: head group `group`, all 64 tokens of every tile, all 512 output dims.
        // O^T: lane holds O[head lm][dim 16 blk + 4 lq + i]
        f32x4 o[32];
#pragma unroll
        for (int blk = 0; blk < 32; ++blk) o[blk] = f32x4{0, 0, 0, 0};
        float m_run = -INFINITY, l_part = 0.0f;
        int32_t next_sl, ref_a_row, ref_a_hit, ref_b_row = -2, ref_b_hit = -1;
        {
            int32_t sl[6], rw[5], ht[5];
#pragma unroll
            for (uint32_t k = 0; k < 6; ++k) sl[k] = refs_slot(tile0 + k);
            next_sl = refs_slot(tile0 + 6);
#pragma unroll
            for (uint32_t k = 0; k < 5; ++k) refs_rows(tile0 + k, sl[k], rw[k], ht[k]);
            refs_rows(tile0 + 5, sl[5], ref_a_row, ref_a_hit);
#pragma unroll
            for (uint32_t k = 0; k < 5; ++k) refs_publish(k, rw[k], ht[k]);
#pragma unroll
            for (uint32_t k = 5; k < ATT_RING; ++k) refs_publish(k, -2, -1);   // not looked up yet: no token
        }
        ATT_SYNC();                                         // prologue 1
        ATT_SYNC();                                         // prologue 2
        auto tile_step = [&](uint32_t tile, int32_t &req_row, int32_t &req_hit, int32_t pub_row, int32_t pub_hit) {
            const uint32_t k = tile - tile0, cur = k & 1u;
            refs_rows(tile + 6, next_sl, req_row, req_hit);
            next_sl = refs_slot(tile + 7);
            att_wait_all(sm->landed, k + 1u, lane, err, spin_limit);
            // the tile in two halves of 32 tokens, each like a pair's share in the other variant: scores
            // of two blocks of 16 tokens, one softmax step, then 32 blocks of 16 dims with 16x16x32 products
#pragma nounroll
            for (uint32_t th = (GPW == 2 ? cw & 1u : 0u); th < (GPW == 2 ? (cw & 1u) + 1u : 2u); ++th) {
                const uint16_t *krow = sm->k[cur] + (32u * th + lm) * ATT_KROW + 8u * lq;
                f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};     // registers are short here: one accumulator each
#pragma unroll
                for (int kk = 0; kk < ATT_KSTEPS; ++kk) {
                    const u16x8 a0 = *(const u16x8 *)(krow + 32 * kk);
                    const u16x8 b0 = *(const u16x8 *)(krow + 16 * ATT_KROW + 32 * kk);
                    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0),
                                                                 __builtin_bit_cast(bf16x8, qb[kk]), sa, 0, 0, 0);
                    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b0),
                                                                 __builtin_bit_cast(bf16x8, qb[kk]), sb, 0, 0, 0);
                }
                const int32_t *live = sm->row[k & (ATT_RING - 1u)] + 32u * th + 4u * lq;
                float pv[8];
                float tmax = -INFINITY;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pv[i] = live[i] >= 0 ? sa[i] * scale_log2 : -INFINITY;
                    pv[4 + i] = live[16 + i] >= 0 ? sb[i] * scale_log2 : -INFINITY;
                    tmax = fmaxf(tmax, fmaxf(pv[i], pv[4 + i]));
                }
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                const float m_new = fmaxf(m_run, tmax);
                const float alpha = m_new == -INFINITY ? 1.0f : exp2f(m_run - m_new);
                float psum = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    pv[i] = m_new == -INFINITY ? 0.0f : exp2f(pv[i] - m_new);
                    psum += pv[i];
                }
                m_run = m_new;
                l_part = l_part * alpha + psum;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int blk = 0; blk < 32; ++blk) o[blk] *= alpha;
                }
                if (GPW == 2 || th == 0) refs_publish((k + 5u) & (ATT_RING - 1u), pub_row, pub_hit);
                const u16x8 pt = {(uint16_t)att_to_bf16(pv[0]), (uint16_t)att_to_bf16(pv[1]), (uint16_t)att_to_bf16(pv[2]),
                                  (uint16_t)att_to_bf16(pv[3]), (uint16_t)att_to_bf16(pv[4]), (uint16_t)att_to_bf16(pv[5]),
                                  (uint16_t)att_to_bf16(pv[6]), (uint16_t)att_to_bf16(pv[7])};
                const uint16_t *vsrc = sm->k[cur] + (32u * th + 4u * lq + (lm >> 2)) * ATT_KROW + 4u * (lm & 3u);
#pragma unroll
                for (int blk = 0; blk < 32; ++blk) {
                    const s16x4 v0 = att_lds_read_tr(vsrc + 16 * blk);
                    const s16x4 v1 = att_lds_read_tr(vsrc + 16 * ATT_KROW + 16 * blk);
                    const u16x8 vt = {(uint16_t)v0[0], (uint16_t)v0[1], (uint16_t)v0[2], (uint16_t)v0[3],
                                      (uint16_t)v1[0], (uint16_t)v1[1], (uint16_t)v1[2], (uint16_t)v1[3]};
                    o[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt),
                                                                     __builtin_bit_cast(bf16x8, pt), o[blk], 0, 0, 0);
                }
            }
            att_signal(&sm->consumed[cw], lane);
        };
        for (uint32_t pr = 0; pr < n_pairs; ++pr) {
            const uint32_t tile = tile0 + 2u * pr;
            tile_step(tile, ref_b_row, ref_b_hit, ref_a_row, ref_a_hit);
            tile_step(tile + 1, ref_a_row, ref_a_hit, ref_b_row, ref_b_hit);
        }
        l_part += __shfl_xor(l_part, 16);
        l_part += __shfl_xor(l_part, 32);
        if constexpr (GPW == 4) {
            // every wave has its own heads: its partial result goes out as it is
            float *po = part_o + part * (ATT_HEADS * 512u) + (uint64_t)lm * 512u + 4u * lq;
#pragma unroll
            for (int blk = 0; blk < 32; ++blk) *(f32x4 *)(po + 16 * blk) = o[blk];
            if (lq == 0) part_ml[part * ATT_HEADS + lm] = make_float2(m_run, l_part);
            __syncthreads();                                // the fetch waves' three
            __syncthreads();
            __syncthreads();
        } else {
            // two waves per head group, one per half of every tile: join them through LDS
            const uint32_t gl = cw >> 1, th = cw & 1u;      // group within the workgroup, token half
            if (lq == 0) {
                sm->wmax[cw * ATT_HEADS + lm] = m_run;
                sm->wsum[cw * ATT_HEADS + lm] = l_part;
            }
            __syncthreads();                                // every tile worked off: the tile buffers are free
            const float m0 = sm->wmax[(2u * gl) * ATT_HEADS + lm], m1 = sm->wmax[(2u * gl + 1u) * ATT_HEADS + lm];
            const float m_all = fmaxf(m0, m1);
            const float l_all = (m0 == -INFINITY ? 0.0f : sm->wsum[(2u * gl) * ATT_HEADS + lm] * exp2f(m0 - m_all)) +
                                (m1 == -INFINITY ? 0.0f : sm->wsum[(2u * gl + 1u) * ATT_HEADS + lm] * exp2f(m1 - m_all));
            const float mine = m_run == -INFINITY ? 0.0f : exp2f(m_run - m_all);
            float *obuf = (float *)sm->k;                   // [4 waves][16 heads][ATT_OROW]
            {
                float *at = obuf + ((uint64_t)cw * ATT_HEADS + lm) * ATT_OROW + 4u * lq;
#pragma unroll
                for (int blk = 0; blk < 32; ++blk) *(f32x4 *)(at + 16 * blk) = o[blk] * mine;
            }
            __syncthreads();
            // the two waves of a group sum its two halves: 16 heads x 128 groups of four dims, 128 lanes
            float *po = part_o + part * (ATT_HEADS * 512u);
            const uint32_t t128 = 64u * th + lane;
#pragma unroll
            for (uint32_t e = 0; e < ATT_HEADS; ++e) {
                const float *src = obuf + ((uint64_t)(2u * gl) * ATT_HEADS + e) * ATT_OROW + 4u * t128;
                *(f32x4 *)(po + (uint64_t)e * 512u + 4u * t128) = *(const f32x4 *)src + *(const f32x4 *)(src + ATT_HEADS * ATT_OROW);
            }
            if (th == 0 && lq == 0) part_ml[part * ATT_HEADS + lm] = make_float2(m_all, l_all);
            __syncthreads();                                // matches the fetch waves' third
        }
        return;
    }
    // Two waves share 32 of the tile's 64 tokens (tg) and split the latent dims (dh): both compute
    // the scores of their 32 tokens (the same instructions on the same data: the same bits), each
    // accumulates 256 of the 512 output dims.  O^T: lane holds O[head lm][dim 256 dh + 16 blk + 4 lq + i];
    // everything a lane owns belongs to head lm.
    const uint32_t tg = cw >> 1, dh = cw & 1u;
    f32x4 o[16];
#pragma unroll
    for (int blk = 0; blk < 16; ++blk) o[blk] = f32x4{0, 0, 0, 0};
    float m_run = -INFINITY, l_part = 0.0f;                 // of head lm; l over this lane's tokens only
    int32_t next_sl, ref_a_row, ref_a_hit, ref_b_row = -2, ref_b_hit = -1;
    {
        // the first six tiles' references: all slot ids first, then all rows, two round trips in all
        int32_t sl[6], rw[5], ht[5];
#pragma unroll
        for (uint32_t k = 0; k < 6; ++k) sl[k] = refs_slot(tile0 + k);
        next_sl = refs_slot(tile0 + 6);
#pragma unroll
        for (uint32_t k = 0; k < 5; ++k) refs_rows(tile0 + k, sl[k], rw[k], ht[k]);
        refs_rows(tile0 + 5, sl[5], ref_a_row, ref_a_hit);
#pragma unroll
        for (uint32_t k = 0; k < 5; ++k) refs_publish(k, rw[k], ht[k]);
#pragma unroll
        for (uint32_t k = 5; k < ATT_RING; ++k) refs_publish(k, -2, -1);       // not looked up yet: no token
    }
    ATT_SYNC();                                             // prologue 1
    ATT_SYNC();                                             // prologue 2

    // one tile; req_*: register pair that takes the references of tile + 6, pub_*: the pair
    // requested a tile ago (tile + 5), published in the middle
    auto tile_step = [&](uint32_t tile, int32_t &req_row, int32_t &req_hit, int32_t pub_row, int32_t pub_hit) {
        const uint32_t k = tile - tile0, cur = k & 1u;
        refs_rows(tile + 6, next_sl, req_row, req_hit);     // slot ids arrived during the last tile
        next_sl = refs_slot(tile + 7);
        att_wait_all(sm->landed, k + 1u, lane, err, spin_limit);        // tiles 0 .. k are in place, whole
        // S^T for this pair's 32 tokens, two blocks of 16: lane holds S[head lm][token 32 tg + 4 lq + i]
        // and S[head lm][token 32 tg + 16 + 4 lq + i].  Four accumulators, so that neither LDS nor MFMA
        // latency adds up.
        const uint16_t *krow = sm->k[cur] + (32u * tg + lm) * ATT_KROW + 8u * lq;
        f32x4 sa = {0, 0, 0, 0}, sa2 = {0, 0, 0, 0}, sb = {0, 0, 0, 0}, sb2 = {0, 0, 0, 0};
        f32x4 sca[4], scb[4];                               // fp8 rows: the block scales of this lane's 8 tokens
        if constexpr (F8) {
            // codes are staged unscaled: the c_KV part of a score is summed per block of 128 dims (four
            // k-steps) and each block sum takes its token's scale, in fp32; the k_r part has none
            f32x4 ba[4], bb[4];
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                ba[blk] = f32x4{0, 0, 0, 0};
                bb[blk] = f32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int kk = 0; kk < ATT_KSTEPS; ++kk) {
                const u16x8 a0 = *(const u16x8 *)(krow + 32 * kk);
                const u16x8 b0 = *(const u16x8 *)(krow + 16 * ATT_KROW + 32 * kk);
                if (kk < 16) {
                    ba[kk >> 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, a0), __builtin_bit_cast(bf16x8, qb[kk]), ba[kk >> 2], 0, 0, 0);
                    bb[kk >> 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, b0), __builtin_bit_cast(bf16x8, qb[kk]), bb[kk >> 2], 0, 0, 0);
                } else {
                    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0),
                                                                 __builtin_bit_cast(bf16x8, qb[kk]), sa, 0, 0, 0);
                    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b0),
                                                                 __builtin_bit_cast(bf16x8, qb[kk]), sb, 0, 0, 0);
                }
            }
            const uint16_t *srow = sm->k[cur] + (32u * tg + 4u * lq) * ATT_KROW + 576u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sca[i] = *(const f32x4 *)(srow + i * ATT_KROW);
                scb[i] = *(const f32x4 *)(srow + (16 + i) * ATT_KROW);
#pragma unroll
                for (int blk = 0; blk < 4; ++blk) {
                    sa[i] += ba[blk][i] * sca[i][blk];
                    sb[i] += bb[blk][i] * scb[i][blk];
                }
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < ATT_KSTEPS; kk += 2) {
                const u16x8 a0 = *(const u16x8 *)(krow + 32 * kk), a1 = *(const u16x8 *)(krow + 32 * kk + 32);
                const u16x8 b0 = *(const u16x8 *)(krow + 16 * ATT_KROW + 32 * kk);
                const u16x8 b1 = *(const u16x8 *)(krow + 16 * ATT_KROW + 32 * kk + 32);
                sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0),
                                                             __builtin_bit_cast(bf16x8, qb[kk]), sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b0),
                                                             __builtin_bit_cast(bf16x8, qb[kk]), sb, 0, 0, 0);
                sa2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1),
                                                              __builtin_bit_cast(bf16x8, qb[kk + 1]), sa2, 0, 0, 0);
                sb2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b1),
                                                              __builtin_bit_cast(bf16x8, qb[kk + 1]), sb2, 0, 0, 0);
            }
            sa += sa2;
            sb += sb2;
        }
        // scores in the log2 domain; tokens that do not exist score -inf
        const int32_t *live = sm->row[k & (ATT_RING - 1u)] + 32u * tg + 4u * lq;
        float pv[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pv[i] = live[i] >= 0 ? sa[i] * scale_log2 : -INFINITY;
            pv[4 + i] = live[16 + i] >= 0 ? sb[i] * scale_log2 : -INFINITY;
            tmax = fmaxf(tmax, fmaxf(pv[i], pv[4 + i]));
        }
        // maximum over the pair's 32 tokens: the four lanes that share lm
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        // all -inf so far (no live token yet): keep everything at zero
        const float alpha = m_new == -INFINITY ? 1.0f : exp2f(m_run - m_new);
        float psum = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            pv[i] = m_new == -INFINITY ? 0.0f : exp2f(pv[i] - m_new);
            psum += pv[i];
        }
        m_run = m_new;
        l_part = l_part * alpha + psum;
        // the maximum moves on a few tiles only: scale the accumulators when some lane needs it
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int blk = 0; blk < 16; ++blk) o[blk] *= alpha;
        }
        refs_publish((k + 5u) & (ATT_RING - 1u), pub_row, pub_hit);   // that slot held tile - 3: long done with
        // O^T += V^T P^T over the 32 tokens at once.  P^T (bf16) is the B operand as the lanes hold it,
        // contraction slot 8 lq + i standing for token 4 lq + i (i < 4) or 16 + 4 lq + i - 4: the A
        // operand follows the same order, four consecutive tokens of one latent dim from each block of
        // 16, two transposing LDS reads (column pieces of the row-major tile).
        const uint16_t *vsrc = sm->k[cur] + (32u * tg + 4u * lq + (lm >> 2)) * ATT_KROW + 256u * dh + 4u * (lm & 3u);
        // fp8 rows: V = code x scale of the token's block, and a wave's 256 dims are two blocks: the scale
        // goes into the numerators, one B operand per block
        u16x8 pt[F8 ? 2 : 1];
#pragma unroll
        for (int h = 0; h < (F8 ? 2 : 1); ++h) {
            float pw[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (F8) {
                    pw[i] = pv[i] * (dh ? sca[i][2 + h] : sca[i][h]);
                    pw[4 + i] = pv[4 + i] * (dh ? scb[i][2 + h] : scb[i][h]);
                } else {
                    pw[i] = pv[i];
                    pw[4 + i] = pv[4 + i];
                }
            }
            pt[h] = u16x8{(uint16_t)att_to_bf16(pw[0]), (uint16_t)att_to_bf16(pw[1]), (uint16_t)att_to_bf16(pw[2]),
                          (uint16_t)att_to_bf16(pw[3]), (uint16_t)att_to_bf16(pw[4]), (uint16_t)att_to_bf16(pw[5]),
                          (uint16_t)att_to_bf16(pw[6]), (uint16_t)att_to_bf16(pw[7])};
        }
#pragma unroll
        for (int blk = 0; blk < 16; ++blk) {
            const s16x4 v0 = att_lds_read_tr(vsrc + 16 * blk);
            const s16x4 v1 = att_lds_read_tr(vsrc + 16 * ATT_KROW + 16 * blk);
            const u16x8 vt = {(uint16_t)v0[0], (uint16_t)v0[1], (uint16_t)v0[2], (uint16_t)v0[3],
                              (uint16_t)v1[0], (uint16_t)v1[1], (uint16_t)v1[2], (uint16_t)v1[3]};
            o[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt),
                                                             __builtin_bit_cast(bf16x8, pt[F8 ? blk >> 3 : 0]),
                                                             o[blk], 0, 0, 0);
        }
        att_signal(&sm->consumed[cw], lane);                // this wave is done with tile k
    };
    for (uint32_t pr = 0; pr < n_pairs; ++pr) {
        const uint32_t tile = tile0 + 2u * pr;
        tile_step(tile, ref_b_row, ref_b_hit, ref_a_row, ref_a_hit);
        tile_step(tile + 1, ref_a_row, ref_a_hit, ref_b_row, ref_b_hit);
    }
    // this pair's sum per head: over the four lanes that share lm
    l_part += __shfl_xor(l_part, 16);
    l_part += __shfl_xor(l_part, 32);
    if (dh == 0 && lq == 0) {
        sm->wmax[tg * ATT_HEADS + lm] = m_run;
        sm->wsum[tg * ATT_HEADS + lm] = l_part;
    }
    __syncthreads();                                        // every tile worked off: the tile buffers are free
    // the two token groups meet: common maximum, weights, then the outputs summed through LDS
    float m_all = -INFINITY, l_all = 0.0f;
#pragma unroll
    for (uint32_t g = 0; g < 2; ++g) m_all = fmaxf(m_all, sm->wmax[g * ATT_HEADS + lm]);
#pragma unroll
    for (uint32_t g = 0; g < 2; ++g) {
        const float mg = sm->wmax[g * ATT_HEADS + lm];
        l_all += mg == -INFINITY ? 0.0f : sm->wsum[g * ATT_HEADS + lm] * exp2f(mg - m_all);
    }
    const float mine = m_run == -INFINITY ? 0.0f : exp2f(m_run - m_all);
    float *obuf = (float *)sm->k;                           // [2 token groups][16 heads][ATT_OROW]
    {
        float *at = obuf + ((uint64_t)tg * ATT_HEADS + lm) * ATT_OROW + 256u * dh + 4u * lq;
#pragma unroll
        for (int blk = 0; blk < 16; ++blk) *(f32x4 *)(at + 16 * blk) = o[blk] * mine;
    }
    __syncthreads();
    float *po = part_o + part * (ATT_HEADS * 512u);
#pragma unroll
    for (uint32_t e = 0; e < ATT_HEADS * 128u / 256u; ++e) {
        const uint32_t idx = ct + 256u * e, h = idx >> 7, d4 = idx & 127u;   // head, group of four dims
        const float *src = obuf + (uint64_t)h * ATT_OROW + 4u * d4;
        *(f32x4 *)(po + (uint64_t)h * 512u + 4u * d4) = *(const f32x4 *)src + *(const f32x4 *)(src + ATT_HEADS * ATT_OROW);
    }
    if (cw == 0 && lq == 0) part_ml[part * ATT_HEADS + lm] = make_float2(m_all, l_all);
    __syncthreads();                                        // matches the fetch waves' third
}

// grid (16 heads, head groups, requests), 512 lanes: lane d owns latent dim d of one head.
// The splits' (max, sum) pairs are combined once in LDS, then the partial outputs are summed
// with independent loads.
__global__ __launch_bounds__(512) void attend_ref_merge(const float *__restrict__ part_o,
                                                        const float2 *__restrict__ part_ml, uint32_t n_splits,
                                                        uint32_t n_heads, float *__restrict__ out,
                                                        float *__restrict__ lse)
{
    __shared__ float w_s[1024];                             // weight of each split, n_splits <= 1024
    __shared__ float red_s[16];
    const uint32_t h = blockIdx.x, group = blockIdx.y, n_groups = gridDim.y, b = blockIdx.z, d = threadIdx.x;
    const uint64_t part0 = ((uint64_t)b * n_groups + group) * n_splits;
    // overall maximum
    float m = -INFINITY;
    for (uint32_t s = d; s < n_splits; s += blockDim.x) m = fmaxf(m, part_ml[(part0 + s) * ATT_HEADS + h].x);
#pragma unroll
    for (int k = 1; k < 64; k <<= 1) m = fmaxf(m, __shfl_xor(m, k));
    if ((d & 63u) == 0) red_s[d >> 6] = m;
    __syncthreads();
    m = red_s[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) m = fmaxf(m, red_s[k]);
    // weights and the overall sum
    float l = 0.0f;
    for (uint32_t s = d; s < n_splits; s += blockDim.x) {
        const float2 ml = part_ml[(part0 + s) * ATT_HEADS + h];
        const float w = (ml.x == -INFINITY || m == -INFINITY) ? 0.0f : exp2f(ml.x - m);
        w_s[s] = w;
        l += ml.y * w;
    }
#pragma unroll
    for (int k = 1; k < 64; k <<= 1) l += __shfl_xor(l, k);
    __syncthreads();                                        // everybody has read the maxima
    if ((d & 63u) == 0) red_s[8 + (d >> 6)] = l;
    __syncthreads();
    l = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) l += red_s[8 + k];
    // partial outputs: lane (dq, sj) adds dims 4 dq .. 4 dq + 3 of the splits sj, sj + 4, ...,
    // eight independent 16-byte loads at a time; the four partial sums meet in LDS
    __shared__ f32x4 acc_s[4][128];
    {
        const uint32_t dq = d & 127u, sj = d >> 7;
        f32x4 a4 = {0, 0, 0, 0};
        const f32x4 *po = (const f32x4 *)(part_o + (part0 * ATT_HEADS + h) * 512u) + dq;
#pragma unroll 8
        for (uint32_t s = sj; s < n_splits; s += 4u) a4 += po[(uint64_t)s * (ATT_HEADS * 512u / 4u)] * w_s[s];
        acc_s[sj][dq] = a4;
    }
    __syncthreads();
    const float *flat = (const float *)acc_s;
    const float acc = flat[d] + flat[512 + d] + flat[1024 + d] + flat[1536 + d];
    const uint64_t oh = (uint64_t)b * n_heads + group * ATT_HEADS + h;
    out[oh * 512u + d] = l > 0.0f ? acc / l : 0.0f;
    if (d == 0) lse[oh] = l > 0.0f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

// called by irm_ctx_create with the context's device current: the split kernel needs more LDS
// than a launch gets by default
irm_status irm_attend_init(int device)
{
    (void)device;
    const void *kernels[12] = {
        (const void *)attend_ref_split<false, false, 1>, (const void *)attend_ref_split<false, true, 1>,
        (const void *)attend_ref_split<true, false, 1>,  (const void *)attend_ref_split<true, true, 1>,
        (const void *)attend_ref_split<false, false, 2>, (const void *)attend_ref_split<false, true, 2>,
        (const void *)attend_ref_split<true, false, 2>,  (const void *)attend_ref_split<true, true, 2>,
        (const void *)attend_ref_split<false, false, 4>, (const void *)attend_ref_split<false, true, 4>,
        (const void *)attend_ref_split<true, false, 4>,  (const void *)attend_ref_split<true, true, 4>};
    for (const void *k : kernels)
        IRM_HIP_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(att_smem)));
    return IRM_OK;
}

extern "C" uint64_t irm_attend_ref_workspace_bytes(uint32_t n_req, uint32_t n_heads, uint32_t n_splits)
{
    return (uint64_t)n_req * n_heads * n_splits * (512u + 2u) * sizeof(float);
}

extern "C" irm_status irm_attend_ref(irm_ctx *ctx, const void *d_q, uint32_t n_req, uint32_t n_heads,
                                     const void *d_pool_layer, uint64_t pool_row_stride_bytes, uint64_t pool_rows,
                                     const int32_t *d_kv_slots, const uint32_t *d_kv_offsets,
                                     const int32_t *d_row_index, const int32_t *d_hit_index, uint64_t dst_rows,
                                     const float *d_trig, uint32_t trig_hits, float scale, uint32_t n_splits,
                                     void *d_workspace, uint64_t workspace_bytes, float *d_out, float *d_lse,
                                     void *stream)
{
    if (!ctx || !d_q || !d_pool_layer || !d_kv_slots || !d_kv_offsets || !d_row_index || !d_hit_index ||
        !d_trig || !d_workspace || !d_out || !d_lse)
        return IRM_ERR_INVALID_ARG;
    if (n_req < 1 || n_heads < ATT_HEADS || n_heads % ATT_HEADS || n_heads > IRM_ATTEND_MAX_QUERY_ROWS || n_splits < 1 ||
        n_splits > 1024 || n_req > 65535)
        return IRM_ERR_INVALID_ARG;
    const bool f8 = ctx->cfg.row_format == IRM_ROW_FP8;
    if (pool_row_stride_bytes < irm_row_bytes(ctx->cfg.row_format) || (pool_row_stride_bytes & 15) || ((uintptr_t)d_pool_layer & 15) ||
        ((uintptr_t)d_q & 15) || ((uintptr_t)d_trig & 15) || pool_rows < 1 || pool_rows > 0x7FFFFFFFull ||
        dst_rows < 1 || trig_hits < 1 || !(scale > 0.0f))
        return IRM_ERR_INVALID_ARG;
    if (workspace_bytes < irm_attend_ref_workspace_bytes(n_req, n_heads, n_splits) || ((uintptr_t)d_workspace & 15))
        return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t n_groups = n_heads / ATT_HEADS;
    float *part_o = (float *)d_workspace;
    float2 *part_ml = (float2 *)(part_o + (uint64_t)n_req * n_groups * n_splits * ATT_HEADS * 512u);
    const bool sample = ctx->prof_events && ctx->prof_n < ctx->prof_cap &&
                        (ctx->prof_calls++ % ctx->prof_every) == 0;
    if (sample) IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n], s));
    // head groups per workgroup (they share the staged tiles): 4 with a multiple of 64 heads, else 2 with a
    // multiple of 32, else 1
    const uint32_t gpw = n_groups % 4u == 0 ? 4u : n_groups % 2u == 0 ? 2u : 1u;
    const uint32_t grid_x = n_groups / gpw;
    const bool nt = grid_x == 1;                        // see att_ld
    typedef void (*split_kernel_t)(const uint16_t *, uint32_t, const char *, uint64_t, uint64_t, const int32_t *,
                                   const uint32_t *, const int32_t *, const int32_t *, uint64_t, const float2 *,
                                   uint32_t, float, uint32_t, float *, float2 *, uint32_t, uint32_t *);
    static const split_kernel_t table[3][2][2] = {      // [groups per workgroup][fp8][streaming loads]
        {{attend_ref_split<false, false, 1>, attend_ref_split<false, true, 1>},
         {attend_ref_split<true, false, 1>, attend_ref_split<true, true, 1>}},
        {{attend_ref_split<false, false, 2>, attend_ref_split<false, true, 2>},
         {attend_ref_split<true, false, 2>, attend_ref_split<true, true, 2>}},
        {{attend_ref_split<false, false, 4>, attend_ref_split<false, true, 4>},
         {attend_ref_split<true, false, 4>, attend_ref_split<true, true, 4>}}};
    const split_kernel_t split_kernel = table[gpw == 4 ? 2 : gpw == 2 ? 1 : 0][f8 ? 1 : 0][nt ? 1 : 0];
    hipLaunchKernelGGL(split_kernel, dim3(grid_x, n_splits, n_req),
                       dim3(512), sizeof(att_smem), s,
                       (const uint16_t *)d_q, n_heads, (const char *)d_pool_layer, pool_row_stride_bytes, pool_rows,
                       d_kv_slots, d_kv_offsets, d_row_index, d_hit_index, dst_rows, (const float2 *)d_trig,
                       trig_hits, scale * ATT_LOG2E, ctx->cfg.pair_mode, part_o, part_ml, ctx->att_spin_limit, ctx->d_err);
    hipLaunchKernelGGL(attend_ref_merge, dim3(ATT_HEADS, n_groups, n_req), dim3(512), 0, s, part_o, part_ml, n_splits, n_heads,
                       d_out, d_lse);
    if (sample) {
        IRM_HIP_TRY(hipEventRecord(ctx->prof_events[2 * ctx->prof_n + 1], s));
        ++ctx->prof_n;
    }
    return irm_launch_status();
}
