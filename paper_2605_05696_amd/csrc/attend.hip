// Consumer of the no-materialise variant (paper Sec. 2 "MLA"; Sec. 7.2 and App. C: the
// delta-rotation fused into the attention kernel's load path): MLA decode attention in the
// latent form, one layer, reading (c_KV, k_r_base) rows of the shared pool through the
// per-slot references irm_reattach_ref wrote and rotating k_r by the hit's R(delta) while
// the rows are staged, so no rotated copy ever exists in HBM.
//
//   score[b][h][t] = scale * q[b][h] . [ c_KV(row_t) | R_t k_r_base(row_t) ]
//   out[b][h]      = sum_t softmax_t(score) c_KV(row_t)
//
//   attend_ref_split   grid (splits, head groups of 16, requests), 4 waves.  A workgroup walks
//       its share of the request's tokens in tiles of 64: the 64 rows (1152 B each) are
//       gathered into LDS with 16-byte loads, k_r is rotated in place there (fp32, one
//       rounding to bf16: the same values the materialising kernel writes), then
//         S = Q K^T     wave w: 16 heads x its 16 tokens, 18 MFMA 16x16x32 (bf16 in, fp32 acc)
//         online softmax over the tile (running max per head shared through LDS)
//         O += P V      wave w: 16 heads x its 128 of the 512 latent dims, 16 MFMA
//       Q lives in registers as A operands; a row of the tile serves as B operand of S as it
//       lies (k = dims, contiguous), and as B operand of O through 2-byte LDS reads
//       (k = tokens, strided).  Every KV byte is read from HBM once per head group.
//   attend_ref_merge   combines the splits' (max, sum, O) into out and lse.
#include "irm_internal.hpp"

#define ATT_TILE 64u                   // tokens per tile
#define ATT_KROW 584u                  // bf16 per staged row: 576 + 8 of padding (1168 B)
#define ATT_PROW 72u                   // bf16 per row of P: 64 + 8 of padding
#define ATT_HEADS 16u                  // heads per workgroup
#define ATT_KSTEPS 18                  // 576 / 32
#define ATT_LOG2E 1.4426950408889634f

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

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
    uint16_t k[ATT_TILE * ATT_KROW];   // staged rows, k_r rotated
    uint16_t p[ATT_HEADS * ATT_PROW];  // softmax numerators of the tile, bf16
    float red[4 * ATT_HEADS];          // per wave and head: tile maximum
    float mfin[ATT_HEADS];             // running maximum per head at the end
    int32_t row[ATT_TILE];             // pool row of each tile token, -1 = no token
    int32_t hit[ATT_TILE];             // rotation of each tile token, -1 = none
};

__global__ __launch_bounds__(256) void attend_ref_split(
    const uint16_t *__restrict__ q, uint32_t n_heads, const char *__restrict__ pool, uint64_t pool_stride,
    uint64_t pool_rows, const int32_t *__restrict__ kv_slots, const uint32_t *__restrict__ kv_offsets,
    const int32_t *__restrict__ row_index, const int32_t *__restrict__ hit_index, uint64_t dst_rows,
    const float2 *__restrict__ trig, uint32_t trig_hits, float scale_log2, uint32_t pair_mode,
    float *__restrict__ part_o, float2 *__restrict__ part_ml, uint32_t *err)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    att_smem *sm = (att_smem *)smem_raw;
    const uint32_t split = blockIdx.x, n_splits = gridDim.x, group = blockIdx.y, n_groups = gridDim.y;
    const uint32_t b = blockIdx.z;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = irm_wave_id();
    const uint32_t lm = lane & 15, lq = lane >> 4;          // MFMA coordinates of this lane
    const uint32_t begin = kv_offsets[b], end = kv_offsets[b + 1];
    const uint32_t n_tok = end - begin;
    const uint32_t n_tiles = (n_tok + ATT_TILE - 1) / ATT_TILE;
    const uint32_t per_split = (n_tiles + n_splits - 1) / n_splits;
    const uint32_t tile0 = split * per_split;
    const uint32_t tile1 = tile0 + per_split < n_tiles ? tile0 + per_split : n_tiles;

    // Q as A operands: lane holds Q[head lm][32 kk + 8 lq .. + 8] for every k-step
    u16x8 qa[ATT_KSTEPS];
    {
        const uint16_t *qrow = q + ((uint64_t)b * n_heads + group * ATT_HEADS + lm) * 576u;
#pragma unroll
        for (int kk = 0; kk < ATT_KSTEPS; ++kk) qa[kk] = *(const u16x8 *)(qrow + 32 * kk + 8 * lq);
    }
    f32x4 o[8];
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) o[nt] = f32x4{0, 0, 0, 0};
    float m_run[4], l_part[4];                              // heads 4 lq + i
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        m_run[i] = -INFINITY;
        l_part[i] = 0.0f;
    }

    for (uint32_t tile = tile0; tile < tile1; ++tile) {
        const uint32_t t0 = begin + tile * ATT_TILE;
        const uint32_t n_valid = end - t0 < ATT_TILE ? end - t0 : ATT_TILE;
        // (1) references of the tile's tokens
        if (tid < ATT_TILE) {
            int32_t row = -1, hit = -1;
            if (tid < n_valid) {
                const int32_t sl = kv_slots[(uint64_t)t0 + tid];
                if (sl >= 0 && (uint64_t)(uint32_t)sl < dst_rows) {
                    row = row_index[sl];
                    hit = hit_index[sl];
                }
                if (row < 0 || (uint64_t)(uint32_t)row >= pool_rows || hit >= (int32_t)trig_hits) {
                    atomicOr(err, IRM_FLAG_ROW_RANGE);      // the token is left out of the attention
                    row = -1;
                }
                if (hit < 0) hit = -1;
            }
            sm->row[tid] = row;
            sm->hit[tid] = hit;
        }
        __syncthreads();
        // (2) gather 64 rows x 72 16-byte vectors; absent tokens become zero rows
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 v[9];
#pragma unroll
            for (int j = 0; j < 9; ++j) {
                const uint32_t idx = tid + 256u * (uint32_t)(half * 9 + j);   // < 4608
                const uint32_t r = idx / 72u, c = idx - r * 72u;
                const int32_t row = sm->row[r];
                v[j] = u32x4{0, 0, 0, 0};
                if (row >= 0)
                    v[j] = __builtin_nontemporal_load((const u32x4 *)(pool + (uint64_t)(uint32_t)row * pool_stride) + c);
            }
#pragma unroll
            for (int j = 0; j < 9; ++j) {
                const uint32_t idx = tid + 256u * (uint32_t)(half * 9 + j);
                const uint32_t r = idx / 72u, c = idx - r * 72u;
                *(u32x4 *)(sm->k + r * ATT_KROW + c * 8u) = v[j];
            }
        }
        __syncthreads();
        // (3) rotate k_r in place: lane (r, j) turns pairs 8j .. 8j+7 of row r
        {
            const uint32_t r = tid >> 2, j = tid & 3;
            const int32_t hit = sm->hit[r];
            if (hit >= 0) {
                const f32x4 *tp = (const f32x4 *)(trig + (uint64_t)(uint32_t)hit * IRM_KR_PAIRS + 8u * j);
                const f32x4 t4[4] = {tp[0], tp[1], tp[2], tp[3]};              // (c, s, c, s) of two pairs each
                uint16_t *kr = sm->k + r * ATT_KROW + IRM_CKV_BYTES / 2;
                if (pair_mode == IRM_PAIR_HALF_SPLIT) {
                    u32x4 a = *(u32x4 *)(kr + 8 * j), bb = *(u32x4 *)(kr + 32 + 8 * j);
                    uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const float a0 = att_bf16_lo(aw[w]), a1 = att_bf16_hi(aw[w]);
                        const float b0 = att_bf16_lo(bw[w]), b1 = att_bf16_hi(bw[w]);
                        const float c0 = t4[w].x, s0 = t4[w].y, c1 = t4[w].z, s1 = t4[w].w;
                        aw[w] = att_to_bf16(a0 * c0 - b0 * s0) | (att_to_bf16(a1 * c1 - b1 * s1) << 16);
                        bw[w] = att_to_bf16(b0 * c0 + a0 * s0) | (att_to_bf16(b1 * c1 + a1 * s1) << 16);
                    }
                    *(u32x4 *)(kr + 8 * j) = u32x4{aw[0], aw[1], aw[2], aw[3]};
                    *(u32x4 *)(kr + 32 + 8 * j) = u32x4{bw[0], bw[1], bw[2], bw[3]};
                } else {                                    // pair p = elements 2p, 2p+1: one word each
                    u32x4 x = *(u32x4 *)(kr + 16 * j), y = *(u32x4 *)(kr + 16 * j + 8);
                    uint32_t w8[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const float a0 = att_bf16_lo(w8[w]), b0 = att_bf16_hi(w8[w]);
                        const float c0 = (w & 1) ? t4[w >> 1].z : t4[w >> 1].x;
                        const float s0 = (w & 1) ? t4[w >> 1].w : t4[w >> 1].y;
                        w8[w] = att_to_bf16(a0 * c0 - b0 * s0) | (att_to_bf16(b0 * c0 + a0 * s0) << 16);
                    }
                    *(u32x4 *)(kr + 16 * j) = u32x4{w8[0], w8[1], w8[2], w8[3]};
                    *(u32x4 *)(kr + 16 * j + 8) = u32x4{w8[4], w8[5], w8[6], w8[7]};
                }
            }
        }
        __syncthreads();
        // (4) S = Q K^T for this wave's 16 tokens: lane holds S[head 4 lq + i][token 16 wave + lm]
        f32x4 s = {0, 0, 0, 0};
        {
            const uint16_t *krow = sm->k + (16u * wave + lm) * ATT_KROW + 8u * lq;
#pragma unroll
            for (int kk = 0; kk < ATT_KSTEPS; ++kk) {
                const u16x8 kb = *(const u16x8 *)(krow + 32 * kk);
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa[kk]),
                                                            __builtin_bit_cast(bf16x8, kb), s, 0, 0, 0);
            }
        }
        // (5) scores in the log2 domain; tokens that do not exist score -inf
        const bool live = sm->row[16u * wave + lm] >= 0;
        float sc[4], tmax[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sc[i] = live ? s[i] * scale_log2 : -INFINITY;
            tmax[i] = sc[i];
        }
        // (6) tile maximum per head: over the 16 lanes that share lq, then over the waves
#pragma unroll
        for (int d = 1; d < 16; d <<= 1)
#pragma unroll
            for (int i = 0; i < 4; ++i) tmax[i] = fmaxf(tmax[i], __shfl_xor(tmax[i], d));
        if (lm == 0)
#pragma unroll
            for (int i = 0; i < 4; ++i) sm->red[wave * ATT_HEADS + 4 * lq + i] = tmax[i];
        __syncthreads();
        float alpha[4], pv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t h = 4 * lq + i;
            const float tm = fmaxf(fmaxf(sm->red[h], sm->red[ATT_HEADS + h]),
                                   fmaxf(sm->red[2 * ATT_HEADS + h], sm->red[3 * ATT_HEADS + h]));
            const float m_new = fmaxf(m_run[i], tm);
            // all -inf so far (no live token yet): keep everything at zero
            alpha[i] = m_new == -INFINITY ? 1.0f : exp2f(m_run[i] - m_new);
            pv[i] = m_new == -INFINITY ? 0.0f : exp2f(sc[i] - m_new);
            m_run[i] = m_new;
            l_part[i] = l_part[i] * alpha[i] + pv[i];
        }
        // (7) P (bf16) to LDS as the A operand of the second product; rescale O
#pragma unroll
        for (int i = 0; i < 4; ++i)
            sm->p[(4 * lq + i) * ATT_PROW + 16u * wave + lm] = (uint16_t)att_to_bf16(pv[i]);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) o[nt][i] *= alpha[i];
        __syncthreads();
        // (8) O += P V: wave owns latent dims [128 wave, 128 wave + 128)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const u16x8 pa = *(const u16x8 *)(sm->p + lm * ATT_PROW + 32 * ks + 8 * lq);
            const uint16_t *vcol = sm->k + (32u * ks + 8u * lq) * ATT_KROW + 128u * wave + lm;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) {
                u16x8 vb;
#pragma unroll
                for (int i = 0; i < 8; ++i) vb[i] = vcol[i * ATT_KROW + 16 * nt];
                o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa),
                                                                __builtin_bit_cast(bf16x8, vb), o[nt], 0, 0, 0);
            }
        }
        __syncthreads();                                    // the tile buffers are reused
    }
    // sums over the 16 lanes that share lq, then over the waves (each wave saw its own tokens)
#pragma unroll
    for (int d = 1; d < 16; d <<= 1)
#pragma unroll
        for (int i = 0; i < 4; ++i) l_part[i] += __shfl_xor(l_part[i], d);
    if (lm == 0)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sm->red[wave * ATT_HEADS + 4 * lq + i] = l_part[i];
            if (wave == 0) sm->mfin[4 * lq + i] = m_run[i];  // the same in every wave
        }
    __syncthreads();
    const uint64_t part = ((uint64_t)b * n_groups + group) * n_splits + split;
    float *po = part_o + part * (ATT_HEADS * 512u);
#pragma unroll
    for (int nt = 0; nt < 8; ++nt)
#pragma unroll
        for (int i = 0; i < 4; ++i) po[(4 * lq + i) * 512u + 128u * wave + 16u * nt + lm] = o[nt][i];
    if (tid < ATT_HEADS) {
        const float l = sm->red[tid] + sm->red[ATT_HEADS + tid] + sm->red[2 * ATT_HEADS + tid] +
                        sm->red[3 * ATT_HEADS + tid];
        part_ml[part * ATT_HEADS + tid] = make_float2(sm->mfin[tid], l);
    }
}

// grid (head groups, requests), 512 lanes: lane d owns latent dim d of all 16 heads
__global__ __launch_bounds__(512) void attend_ref_merge(const float *__restrict__ part_o,
                                                        const float2 *__restrict__ part_ml, uint32_t n_splits,
                                                        uint32_t n_heads, float *__restrict__ out,
                                                        float *__restrict__ lse)
{
    const uint32_t group = blockIdx.x, n_groups = gridDim.x, b = blockIdx.y, d = threadIdx.x;
    const uint64_t part0 = ((uint64_t)b * n_groups + group) * n_splits;
    for (uint32_t h = 0; h < ATT_HEADS; ++h) {
        float m = -INFINITY;
        for (uint32_t s = 0; s < n_splits; ++s) m = fmaxf(m, part_ml[(part0 + s) * ATT_HEADS + h].x);
        float l = 0.0f, acc = 0.0f;
        if (m != -INFINITY) {
            for (uint32_t s = 0; s < n_splits; ++s) {
                const float2 ml = part_ml[(part0 + s) * ATT_HEADS + h];
                const float w = ml.x == -INFINITY ? 0.0f : exp2f(ml.x - m);
                l += ml.y * w;
                acc += part_o[((part0 + s) * ATT_HEADS + h) * 512u + d] * w;
            }
        }
        const uint64_t oh = (uint64_t)b * n_heads + group * ATT_HEADS + h;
        out[oh * 512u + d] = l > 0.0f ? acc / l : 0.0f;
        if (d == 0) lse[oh] = l > 0.0f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
    }
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
    if (n_req < 1 || n_heads < ATT_HEADS || n_heads % ATT_HEADS || n_heads > 128 || n_splits < 1 ||
        n_splits > 1024 || n_req > 65535)
        return IRM_ERR_INVALID_ARG;
    if (pool_row_stride_bytes < IRM_ROW_BYTES || (pool_row_stride_bytes & 15) || ((uintptr_t)d_pool_layer & 15) ||
        ((uintptr_t)d_q & 15) || ((uintptr_t)d_trig & 15) || pool_rows < 1 || pool_rows > 0x7FFFFFFFull ||
        dst_rows < 1 || !(scale > 0.0f))
        return IRM_ERR_INVALID_ARG;
    if (workspace_bytes < irm_attend_ref_workspace_bytes(n_req, n_heads, n_splits) || ((uintptr_t)d_workspace & 15))
        return IRM_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t n_groups = n_heads / ATT_HEADS;
    float *part_o = (float *)d_workspace;
    float2 *part_ml = (float2 *)(part_o + (uint64_t)n_req * n_groups * n_splits * ATT_HEADS * 512u);
    static bool lds_set = false;
    if (!lds_set) {
        IRM_HIP_TRY(hipFuncSetAttribute((const void *)attend_ref_split, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)sizeof(att_smem)));
        lds_set = true;
    }
    hipLaunchKernelGGL(attend_ref_split, dim3(n_splits, n_groups, n_req), dim3(256), sizeof(att_smem), s,
                       (const uint16_t *)d_q, n_heads, (const char *)d_pool_layer, pool_row_stride_bytes, pool_rows,
                       d_kv_slots, d_kv_offsets, d_row_index, d_hit_index, dst_rows, (const float2 *)d_trig,
                       trig_hits, scale * ATT_LOG2E, ctx->cfg.pair_mode, part_o, part_ml, ctx->d_err);
    hipLaunchKernelGGL(attend_ref_merge, dim3(n_groups, n_req), dim3(512), 0, s, part_o, part_ml, n_splits, n_heads,
                       d_out, d_lse);
    return irm_launch_status();
}
