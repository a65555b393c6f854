/*
 * irm_oracle.c -- plain, slow, sequential CPU statement of the cache-hit
 * re-attachment path of an MLA position-independent KV cache.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something written only from the paper.  It shares no code,
 * header, table or helper with the GPU library and nothing in the product path
 * may call it.  Only the tests, the smoke check and the CPU-baseline leg of the
 * benchmark load it.
 *
 * Four stages, each an exact definition (no approximation, no blocking, no
 * fusion; one token / one byte / one row at a time):
 *
 *   oracle_cdc_chunk     gear-hash content-defined chunking
 *                        (paper Sec. 4 "CDC (gear-hash)", Sec. 7.2 "CDC boundary
 *                        rule", App. B; Alg. 1 step "segments <- CDC(tail)")
 *   oracle_chunk_hash    one 64-bit fingerprint per emitted chunk
 *                        (Sec. 4; Alg. 1 steps 2 and 7).  The fingerprint
 *                        function is FNV-1a-64 over the little-endian bytes of
 *                        the int32 token ids (the workload definition fixes
 *                        FNV-1a-64 in place of the paper's xxHash64).
 *   oracle_lookup        registry R: hash -> (rows, p_src), first-chunk
 *                        carve-out, delta = p - p_src (Alg. 1 steps 4-8,
 *                        12-13; Sec. 7.1 "first-chunk carve-out")
 *   oracle_reattach      c_KV copied verbatim, k_r <- R(delta) k_r_base,
 *                        written into the request's slots (Alg. 1 steps 9-10;
 *                        Sec. 7.2 "k_r rotation"; App. C "k_r rotation
 *                        materialisation": gather-rotate-scatter)
 *   oracle_admit         the miss path: prefilled rows are copied into the pool and
 *                        registered, insert-if-absent (Alg. 1 steps 11-13)
 *   oracle_reattach_kr   the split-pool variant of the same step: c_KV is only
 *                        referenced, k_r alone is materialised (App. C "Split
 *                        TokenToKVPool")
 *   oracle_s1_windows    S1 fallback: fixed windows inside chunks that missed
 *                        (Sec. 4 "CDC+fallback"; App. G "S1")
 *   oracle_reattach_ref  the no-materialise variant: row references and the per-hit
 *                        rotation table (Sec. 7.2; App. C)
 * (its consumer, attention over the references with the rotation applied on load, is
 * stated in numpy in irm_oracle.py: attend_ref)
 *
 * Floating point: fp64 throughout, one round-to-nearest-even to bf16 at the
 * store.  Parity status: every function below is pinned by the CPU tests to
 * closed forms, invariants, textbook vectors or brute force; none is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_ROW_DIM 576 /* 512 c_KV + 64 k_r elements per token row (Sec. 2 "MLA") */
#define ORACLE_CKV_DIM 512
/* Row formats.  A row is a position-free part followed by the 64 bf16 elements of k_r; its
 * size is given in 16-bit words ("ckv_words") wherever a function takes rows:
 *   512  bf16 rows: c_KV as 512 bf16
 *   264  fp8 rows (Sec. 7.2 names FP8 KV quantisation as accepted practice; the layout is the
 *        one published for fp8 MLA caches): c_KV as 512 e4m3 bytes, then four fp32 scales,
 *        one per 128 elements -- 528 bytes that depend on the content only -- and k_r kept
 *        in bf16.
 * The position-free part is copied bit for bit, whatever it encodes; the rotation acts on
 * k_r alone (Alg. 1 steps 9-10). */
#define ORACLE_CKV_WORDS_BF16 512
#define ORACLE_CKV_WORDS_FP8 264
#define ORACLE_KR_DIM 64
#define ORACLE_KR_PAIRS 32

/* ------------------------------------------------------------------------- */
/* Stage 1a: gear-hash CDC (Sec. 4; Sec. 7.2; App. B).                        */
/*                                                                           */
/* Per request the rolling state starts at zero.  Each token advances the    */
/* state by one gear step, h <- (h << 1) + G[low byte of the token id], in   */
/* 32-bit wrap-around arithmetic.  The token that makes the rule true is the  */
/* LAST token of its chunk.  A chunk closes when                              */
/*   - it is at least min_chunk long and the masked state is zero, or        */
/*   - it has reached max_chunk tokens, or                                   */
/*   - the request ends (the tail chunk may be shorter than min_chunk).       */
/* The state is not reset at a cut.                                          */
/*                                                                           */
/* chunk_start / chunk_len are offsets into the concatenated token array;    */
/* req_chunk_offsets[r] .. req_chunk_offsets[r+1] are request r's chunks.     */
/* Returns the number of chunks, or -1 when `capacity` chunks do not suffice  */
/* or an argument is unusable.                                               */
/* ------------------------------------------------------------------------- */
int64_t oracle_cdc_chunk(const int32_t *tokens, const uint32_t *req_offsets, uint32_t n_req,
                         const uint32_t *gear /* [256] */, uint32_t mask, uint32_t min_chunk,
                         uint32_t max_chunk, uint32_t *chunk_start, uint32_t *chunk_len,
                         uint32_t *req_chunk_offsets, uint64_t capacity)
{
    if (min_chunk < 1 || max_chunk < min_chunk) return -1;
    uint64_t n_chunks = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        req_chunk_offsets[r] = (uint32_t)n_chunks;
        uint32_t begin = req_offsets[r], end = req_offsets[r + 1];
        uint32_t h = 0;
        uint32_t s = begin; /* first token of the open chunk */
        for (uint32_t i = begin; i < end; ++i) {
            h = (h << 1) + gear[(uint32_t)tokens[i] & 0xFFu];
            uint32_t len = i - s + 1;
            int content_cut = (len >= min_chunk) && ((h & mask) == 0);
            int size_cut = (len == max_chunk);
            int tail_cut = (i + 1 == end);
            if (content_cut || size_cut || tail_cut) {
                if (n_chunks >= capacity) return -1;
                chunk_start[n_chunks] = s;
                chunk_len[n_chunks] = len;
                ++n_chunks;
                s = i + 1;
            }
        }
    }
    req_chunk_offsets[n_req] = (uint32_t)n_chunks;
    return (int64_t)n_chunks;
}

/* ------------------------------------------------------------------------- */
/* Stage 1b: chunk fingerprint.  FNV-1a, 64 bit: start from the offset basis, */
/* for every byte XOR it in, then multiply by the FNV prime (mod 2^64).       */
/* ------------------------------------------------------------------------- */
uint64_t oracle_fnv1a64_bytes(const uint8_t *bytes, uint64_t n)
{
    uint64_t h = 0xCBF29CE484222325ull;
    for (uint64_t k = 0; k < n; ++k) {
        h ^= (uint64_t)bytes[k];
        h *= 0x00000100000001B3ull;
    }
    return h;
}

/* One fingerprint per chunk over the chunk's token ids, each id taken as its
 * four little-endian bytes, in stream order, nothing else mixed in. */
void oracle_chunk_hash(const int32_t *tokens, const uint32_t *chunk_start,
                       const uint32_t *chunk_len, uint64_t n_chunks, uint64_t *chunk_hash)
{
    for (uint64_t c = 0; c < n_chunks; ++c) {
        uint64_t h = 0xCBF29CE484222325ull;
        for (uint32_t j = 0; j < chunk_len[c]; ++j) {
            uint32_t t = (uint32_t)tokens[chunk_start[c] + j];
            for (int b = 0; b < 4; ++b) {
                h ^= (uint64_t)((t >> (8 * b)) & 0xFFu);
                h *= 0x00000100000001B3ull;
            }
        }
        chunk_hash[c] = h;
    }
}

/* ------------------------------------------------------------------------- */
/* Stage 2: registry lookup (Alg. 1 steps 4-8 and 12-13; Sec. 7.1).           */
/*                                                                           */
/* The registry is an associative map hash -> entry, filled by               */
/* insert-if-absent in the order the entries are listed (Alg. 1 inserts only  */
/* on a miss, so the first entry with a given hash stays).  A request chunk   */
/* at absolute position p = pos_base[r] + (chunk_start - req_offsets[r])      */
/*   - is never served when p < carve_out (first-chunk carve-out),            */
/*   - hits when the map holds its hash AND the stored chunk length equals    */
/*     its own length; then delta = p - p_src,                               */
/*   - misses otherwise.                                                     */
/* chunk_entry[c] is the entry id of the hit or -1.  Hits are listed in       */
/* ascending chunk order.                                                    */
/*                                                                           */
/* The map is realised as the entry list sorted by (hash, list index) and a   */
/* binary search for the first entry of a hash.                              */
/* ------------------------------------------------------------------------- */
typedef struct {
    uint64_t hash;
    uint64_t index;
} oracle_key_t;

static int oracle_key_cmp(const void *a, const void *b)
{
    const oracle_key_t *x = (const oracle_key_t *)a, *y = (const oracle_key_t *)b;
    if (x->hash != y->hash) return x->hash < y->hash ? -1 : 1;
    if (x->index != y->index) return x->index < y->index ? -1 : 1;
    return 0;
}

/* index of the first listed registry entry with this hash, or -1 */
static int64_t oracle_registry_find(const oracle_key_t *sorted, uint64_t n, uint64_t hash)
{
    uint64_t lo = 0, hi = n; /* first position whose hash is >= `hash` */
    while (lo < hi) {
        uint64_t mid = lo + (hi - lo) / 2;
        if (sorted[mid].hash < hash) lo = mid + 1; else hi = mid;
    }
    if (lo < n && sorted[lo].hash == hash) return (int64_t)sorted[lo].index;
    return -1;
}

int oracle_lookup(const uint64_t *reg_hash, const uint32_t *reg_src_row, const int32_t *reg_p_src,
                  const uint32_t *reg_len, const uint32_t *reg_entry_id, uint64_t n_reg,
                  const uint64_t *chunk_hash, const uint32_t *chunk_start,
                  const uint32_t *chunk_len, const uint32_t *req_chunk_offsets,
                  const uint32_t *req_offsets, const int32_t *pos_base, uint32_t n_req,
                  uint32_t carve_out, int32_t *chunk_entry, uint32_t *hit_src_row,
                  uint32_t *hit_dst_tok, uint32_t *hit_len, int32_t *hit_delta,
                  uint32_t *n_hits_out, uint64_t *hit_tokens_out)
{
    oracle_key_t *sorted = (oracle_key_t *)malloc((n_reg ? n_reg : 1) * sizeof(oracle_key_t));
    if (!sorted) return -1;
    for (uint64_t k = 0; k < n_reg; ++k) {
        sorted[k].hash = reg_hash[k];
        sorted[k].index = k;
    }
    qsort(sorted, n_reg, sizeof(oracle_key_t), oracle_key_cmp);

    uint32_t n_hits = 0;
    uint64_t hit_tokens = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        for (uint32_t c = req_chunk_offsets[r]; c < req_chunk_offsets[r + 1]; ++c) {
            int64_t p = (int64_t)pos_base[r] + (int64_t)(chunk_start[c] - req_offsets[r]);
            chunk_entry[c] = -1;
            if (p < (int64_t)carve_out) continue;
            int64_t e = oracle_registry_find(sorted, n_reg, chunk_hash[c]);
            if (e < 0) continue;
            if (reg_len[e] != chunk_len[c]) continue;
            chunk_entry[c] = (int32_t)reg_entry_id[e];
            hit_src_row[n_hits] = reg_src_row[e];
            hit_dst_tok[n_hits] = chunk_start[c];
            hit_len[n_hits] = chunk_len[c];
            hit_delta[n_hits] = (int32_t)(p - (int64_t)reg_p_src[e]);
            ++n_hits;
            hit_tokens += chunk_len[c];
        }
    }
    *n_hits_out = n_hits;
    *hit_tokens_out = hit_tokens;
    free(sorted);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Stage 3: re-attachment (Alg. 1 steps 8-10; Sec. 7.2; App. C).              */
/* ------------------------------------------------------------------------- */

/* bf16 -> fp64, exact: a bf16 is the upper half of an IEEE binary32. */
double oracle_bf16_to_f64(uint16_t v)
{
    uint32_t bits = (uint32_t)v << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* fp64 -> bf16, ONE rounding, to nearest, ties to even.
 * bf16 has 8 significand bits (7 stored) and binary32's exponent range, so a
 * normal value with exponent e is a multiple of 2^(e-7) and a subnormal one a
 * multiple of 2^-133.  Dividing by that spacing is exact (power of two),
 * rint() in the default rounding mode is round-half-even, and the product
 * back is exact; the result is then representable in binary32 exactly. */
uint16_t oracle_f64_to_bf16(double x)
{
    if (isnan(x)) return 0x7FC0;
    double r;
    if (isinf(x) || x == 0.0) {
        r = x;
    } else {
        int e = ilogb(x);
        if (e < -126) e = -126;
        double spacing = ldexp(1.0, e - 7);
        r = rint(x / spacing) * spacing;
        if (fabs(r) >= ldexp(1.0, 128)) r = copysign(INFINITY, x); /* past the largest finite bf16 */
    }
    float f = (float)r; /* exact */
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return (uint16_t)(bits >> 16);
}

/* R(delta) on one 64-element k_r vector, fp64 in and out, no rounding.
 * Pair i is turned counter-clockwise by the angle delta * inv_freq[i] (standard
 * RoPE; R(a)R(b) = R(a+b), Alg. 1 step 9).  Which two elements form pair i is the
 * model's rotary layout (App. D speaks of DSv2-form and DSv3-form rotaries):
 *   pair_mode 0, half-split:  elements i and i + 32;
 *   pair_mode 1, interleaved: elements 2i and 2i + 1.
 * inv_freq are the model's fp32 rotary frequencies (App. D: cos/sin are derived
 * from the inv_freq buffer itself); the angle is the fp64 product of delta and
 * that fp32 value. */
void oracle_rotate_kr_f64(const double *k_in /* [64] */, int64_t delta,
                          const float *inv_freq /* [32] */, uint32_t pair_mode,
                          double *k_out /* [64] */)
{
    for (int i = 0; i < ORACLE_KR_PAIRS; ++i) {
        double phi = (double)delta * (double)inv_freq[i];
        double c = cos(phi), s = sin(phi);
        int ia = pair_mode ? 2 * i : i, ib = pair_mode ? 2 * i + 1 : i + ORACLE_KR_PAIRS;
        double a = k_in[ia], b = k_in[ib];
        k_out[ia] = a * c - b * s;
        k_out[ib] = b * c + a * s;
    }
}

/* One KV row of ckv_words + 64 words: the position-free part copied, k_r rotated and
 * rounded once. */
void oracle_reattach_row(const uint16_t *row_in, int32_t delta, const float *inv_freq,
                         uint32_t pair_mode, uint32_t ckv_words, uint16_t *row_out)
{
    for (uint32_t d = 0; d < ckv_words; ++d) row_out[d] = row_in[d];
    double k[ORACLE_KR_DIM], kr[ORACLE_KR_DIM];
    for (int d = 0; d < ORACLE_KR_DIM; ++d) k[d] = oracle_bf16_to_f64(row_in[ckv_words + d]);
    oracle_rotate_kr_f64(k, (int64_t)delta, inv_freq, pair_mode, kr);
    for (int d = 0; d < ORACLE_KR_DIM; ++d) row_out[ckv_words + d] = oracle_f64_to_bf16(kr[d]);
}

/* For every hit h, layer l and j < len[h]:
 *   dst[l][ dst_slots[dst_tok[h] + j] ] <- reattach_row( src[l][ src_row[h] + j ], delta[h] )
 * src is [n_layers][src_rows][ckv_words + 64], dst is [n_layers][dst_rows][ckv_words + 64],
 * both dense.  Rows of dst that no hit covers are left as they were.
 * Returns 0, or -1 when an index falls outside its pool. */
int oracle_reattach(const uint16_t *src, uint64_t src_rows, uint16_t *dst, uint64_t dst_rows,
                    uint32_t n_layers, const int32_t *dst_slots, const uint32_t *hit_src_row,
                    const uint32_t *hit_dst_tok, const uint32_t *hit_len,
                    const int32_t *hit_delta, uint32_t n_hits, const float *inv_freq,
                    uint32_t pair_mode, uint32_t ckv_words)
{
    const uint64_t row_words = (uint64_t)ckv_words + ORACLE_KR_DIM;
    for (uint32_t h = 0; h < n_hits; ++h) {
        for (uint32_t l = 0; l < n_layers; ++l) {
            for (uint32_t j = 0; j < hit_len[h]; ++j) {
                uint64_t srow = (uint64_t)hit_src_row[h] + j;
                int64_t drow = dst_slots[(uint64_t)hit_dst_tok[h] + j];
                if (srow >= src_rows || drow < 0 || (uint64_t)drow >= dst_rows) return -1;
                const uint16_t *in = src + ((uint64_t)l * src_rows + srow) * row_words;
                uint16_t *out = dst + ((uint64_t)l * dst_rows + (uint64_t)drow) * row_words;
                oracle_reattach_row(in, hit_delta[h], inv_freq, pair_mode, ckv_words, out);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Split-pool variant (App. C "Split TokenToKVPool"): the 512-dim c_KV stays in */
/* the shared, content-addressed pool and is only REFERENCED; the 64-dim k_r   */
/* slice alone is materialised per request, rotated by delta.                  */
/* For every hit h, j < len[h], slot = dst_slots[dst_tok[h] + j]:              */
/*   ckv_index[slot]      <- src_row[h] + j              (same for all layers) */
/*   kr_dst[l][slot][0:64] <- R(delta[h]) k_r of src[l][src_row[h] + j]         */
/* src is [n_layers][src_rows][ckv_words + 64], kr_dst is [n_layers][kr_rows][64]. */
/* ------------------------------------------------------------------------- */
int oracle_reattach_kr(const uint16_t *src, uint64_t src_rows, uint16_t *kr_dst, uint64_t kr_rows,
                       int32_t *ckv_index, uint32_t n_layers, const int32_t *dst_slots,
                       const uint32_t *hit_src_row, const uint32_t *hit_dst_tok,
                       const uint32_t *hit_len, const int32_t *hit_delta, uint32_t n_hits,
                       const float *inv_freq, uint32_t pair_mode, uint32_t ckv_words)
{
    const uint64_t row_words = (uint64_t)ckv_words + ORACLE_KR_DIM;
    for (uint32_t h = 0; h < n_hits; ++h) {
        for (uint32_t j = 0; j < hit_len[h]; ++j) {
            uint64_t srow = (uint64_t)hit_src_row[h] + j;
            int64_t slot = dst_slots[(uint64_t)hit_dst_tok[h] + j];
            if (srow >= src_rows || slot < 0 || (uint64_t)slot >= kr_rows) return -1;
            ckv_index[slot] = (int32_t)srow;
            for (uint32_t l = 0; l < n_layers; ++l) {
                const uint16_t *in = src + ((uint64_t)l * src_rows + srow) * row_words + ckv_words;
                uint16_t *out = kr_dst + ((uint64_t)l * kr_rows + (uint64_t)slot) * ORACLE_KR_DIM;
                double k[ORACLE_KR_DIM], kr[ORACLE_KR_DIM];
                for (int d = 0; d < ORACLE_KR_DIM; ++d) k[d] = oracle_bf16_to_f64(in[d]);
                oracle_rotate_kr_f64(k, (int64_t)hit_delta[h], inv_freq, pair_mode, kr);
                for (int d = 0; d < ORACLE_KR_DIM; ++d) out[d] = oracle_f64_to_bf16(kr[d]);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Miss path (Alg. 1 steps 11-13): after the engine has prefilled a chunk that */
/* missed, its KV rows sit in the request's slots; they are copied into fresh  */
/* rows of the shared pool and the registry learns hash -> (rows, p, len).     */
/*                                                                           */
/* Chunks are taken in ascending order.  A chunk is admitted when              */
/*   - the lookup missed it (chunk_entry < 0),                                 */
/*   - its position p >= carve_out (Alg. 1 prefills p < 32 without inserting), */
/*   - the registry does not hold its hash yet, neither from before nor from   */
/*     an earlier chunk of this batch (insert-if-absent),                      */
/*   - the pool has len free rows left after *cursor; the first chunk that     */
/*     does not fit closes the pool for the rest of the batch.                 */
/* An admitted chunk gets rows [*cursor, *cursor + len), every layer's rows are */
/* copied bit for bit from the request's slots (k_r stays as computed at p, so  */
/* p_src = p), *cursor advances, and admitted_row[c] is the first row; all      */
/* other chunks get admitted_row[c] = -1.  new_* receive the registry entries   */
/* in admission order (entry_id = first pool row).  Returns their number.       */
/* req is [n_layers][req_rows][ckv_words + 64], pool the same with pool_rows.   */
/* ------------------------------------------------------------------------- */
int64_t oracle_admit(const uint64_t *reg_hash, uint64_t n_reg, const uint64_t *chunk_hash,
                     const uint32_t *chunk_start, const uint32_t *chunk_len,
                     const uint32_t *req_chunk_offsets, const uint32_t *req_offsets,
                     const int32_t *pos_base, uint32_t n_req, uint32_t carve_out,
                     const int32_t *chunk_entry, const uint16_t *req, uint64_t req_rows,
                     const int32_t *slots, uint16_t *pool, uint64_t pool_rows, uint32_t n_layers,
                     uint32_t *cursor, int32_t *admitted_row, uint64_t *new_hash,
                     uint32_t *new_src_row, int32_t *new_p_src, uint32_t *new_len, uint32_t ckv_words)
{
    const uint64_t row_words = (uint64_t)ckv_words + ORACLE_KR_DIM;
    int64_t n_new = 0;
    int pool_closed = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        for (uint32_t c = req_chunk_offsets[r]; c < req_chunk_offsets[r + 1]; ++c) {
            admitted_row[c] = -1;
            int64_t p = (int64_t)pos_base[r] + (int64_t)(chunk_start[c] - req_offsets[r]);
            if (chunk_entry[c] >= 0 || p < (int64_t)carve_out || chunk_len[c] == 0) continue;
            int known = 0;
            for (uint64_t k = 0; k < n_reg && !known; ++k) known = reg_hash[k] == chunk_hash[c];
            for (int64_t k = 0; k < n_new && !known; ++k) known = new_hash[k] == chunk_hash[c];
            if (known) continue;
            if (pool_closed || (uint64_t)*cursor + chunk_len[c] > pool_rows) {
                pool_closed = 1;
                continue;
            }
            for (uint32_t l = 0; l < n_layers; ++l) {
                for (uint32_t j = 0; j < chunk_len[c]; ++j) {
                    int64_t slot = slots[(uint64_t)chunk_start[c] + j];
                    if (slot < 0 || (uint64_t)slot >= req_rows) return -1;
                    memcpy(pool + ((uint64_t)l * pool_rows + *cursor + j) * row_words,
                           req + ((uint64_t)l * req_rows + (uint64_t)slot) * row_words,
                           row_words * sizeof(uint16_t));
                }
            }
            admitted_row[c] = (int32_t)*cursor;
            new_hash[n_new] = chunk_hash[c];
            new_src_row[n_new] = *cursor;
            new_p_src[n_new] = (int32_t)p;
            new_len[n_new] = chunk_len[c];
            ++n_new;
            *cursor += chunk_len[c];
        }
    }
    return n_new;
}

/* ------------------------------------------------------------------------- */
/* S1, detect-and-recover (Sec. 4 "CDC+fallback"; App. G "S1"): a chunk whose  */
/* fingerprint missed is sub-divided into fixed windows of `window` tokens     */
/* (the paper's 128) and every window is fingerprinted and looked up on its    */
/* own, so content that is shared but sits in a chunk with drifted boundaries  */
/* is still found.  This function is the sub-division only; the windows it     */
/* lists are then fingerprinted and looked up exactly like chunks              */
/* (oracle_chunk_hash, oracle_lookup with req_win_offsets as the CSR).         */
/*                                                                           */
/* For every request r and every chunk c of r with expand[c] != 0, in order:   */
/* n = len[c] / window whole windows; a remainder shorter than a window is not */
/* probed.  anchor 0: the windows start at the chunk's first token,            */
/* [s + j w, s + (j+1) w); anchor 1: they end at the chunk's last token,       */
/* [e - (n-j) w, e - (n-j-1) w) with e = s + len.  (A chunk's end is fixed by  */
/* content alone; its start also depends on what came before it.  Which side   */
/* the paper anchors is not stated: both are offered.)                         */
/* Windows come out in ascending token order.  win_start, win_parent receive   */
/* one entry per window (first token, index of the chunk it was cut from);     */
/* req_win_offsets[n_req + 1] is the CSR over requests.  Returns the count.    */
/* ------------------------------------------------------------------------- */
int64_t oracle_s1_windows(const uint32_t *chunk_start, const uint32_t *chunk_len,
                          const uint32_t *req_chunk_offsets, uint32_t n_req,
                          const uint8_t *expand, uint32_t window, uint32_t anchor,
                          uint32_t *win_start, uint32_t *win_parent, uint32_t *req_win_offsets)
{
    int64_t n_win = 0;
    if (window == 0) return -1;
    for (uint32_t r = 0; r < n_req; ++r) {
        req_win_offsets[r] = (uint32_t)n_win;
        for (uint32_t c = req_chunk_offsets[r]; c < req_chunk_offsets[r + 1]; ++c) {
            if (!expand[c]) continue;
            uint32_t n = chunk_len[c] / window;
            uint32_t first = anchor ? chunk_start[c] + chunk_len[c] - n * window : chunk_start[c];
            for (uint32_t j = 0; j < n; ++j) {
                win_start[n_win] = first + j * window;
                win_parent[n_win] = c;
                ++n_win;
            }
        }
    }
    req_win_offsets[n_req] = (uint32_t)n_win;
    return n_win;
}

/* ------------------------------------------------------------------------- */
/* No-materialise variant (Sec. 7.2 "fuseable into the attention kernel's load */
/* path"; App. C "keep k_r_base in HBM and fuse the rotation into the load     */
/* path so the rotated tensor never materialises"): re-attachment writes no KV */
/* at all, only what the load path needs to rotate on the fly.                 */
/* For every hit h, j < len[h], slot = dst_slots[dst_tok[h] + j]:              */
/*   row_index[slot] <- src_row[h] + j     pool row holding (c_KV, k_r_base)   */
/*   hit_index[slot] <- h                  which rotation the row needs        */
/* and per hit the rotation itself, trig[h][i] = (cos, sin)(delta[h] *         */
/* inv_freq[i]) for the 32 pairs, angle as the fp64 product, exactly (1, 0)    */
/* when delta = 0.  Slots no hit covers are left as they were.                 */
/* Returns 0, or -1 when an index falls outside its pool.                      */
/* ------------------------------------------------------------------------- */
int oracle_reattach_ref(uint64_t src_rows, int32_t *row_index, int32_t *hit_index, uint64_t dst_rows,
                        double *trig /* [n_hits][32][2] */, const int32_t *dst_slots,
                        const uint32_t *hit_src_row, const uint32_t *hit_dst_tok,
                        const uint32_t *hit_len, const int32_t *hit_delta, uint32_t n_hits,
                        const float *inv_freq)
{
    for (uint32_t h = 0; h < n_hits; ++h) {
        for (int i = 0; i < ORACLE_KR_PAIRS; ++i) {
            double phi = (double)hit_delta[h] * (double)inv_freq[i];
            trig[((uint64_t)h * ORACLE_KR_PAIRS + i) * 2 + 0] = hit_delta[h] ? cos(phi) : 1.0;
            trig[((uint64_t)h * ORACLE_KR_PAIRS + i) * 2 + 1] = hit_delta[h] ? sin(phi) : 0.0;
        }
        for (uint32_t j = 0; j < hit_len[h]; ++j) {
            uint64_t srow = (uint64_t)hit_src_row[h] + j;
            int64_t slot = dst_slots[(uint64_t)hit_dst_tok[h] + j];
            if (srow >= src_rows || slot < 0 || (uint64_t)slot >= dst_rows) return -1;
            row_index[slot] = (int32_t)srow;
            hit_index[slot] = (int32_t)h;
        }
    }
    return 0;
}
