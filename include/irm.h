/*
 * irm.h -- C ABI of the cache-hit re-attachment path of an MLA-native
 * position-independent KV cache, for AMD MI355X (gfx950).
 *
 * The path serves one batch of prompts (paper Alg. 1, "serve path"):
 *
 *   irm_cdc_chunk    cut each prompt's token ids into content-defined chunks
 *   irm_chunk_hash   one 64-bit fingerprint per chunk
 *   irm_lookup       probe the registry of cached chunks; list the hits with
 *                    delta = new position - stored position
 *   irm_reattach     for every hit and every layer, copy the position-free
 *                    c_KV part of each cached row verbatim and write the
 *                    RoPE part k_r rotated by delta into the request's slots
 *
 * Around it (each declared below with the passage it follows):
 *
 *   irm_reattach_kr   split pool: only k_r is materialised, c_KV is referenced
 *   irm_reattach_ref  nothing is materialised: row references and the per-hit
 *                     rotation table for a load path that rotates on the fly
 *   irm_attend_ref    such a load path: MLA decode attention over the references
 *   irm_admit, irm_table_insert[_counted]   miss path: prefilled chunks into the
 *                     shared pool and the registry, insert-if-absent
 *   irm_s1_windows    S1 fallback: fixed windows inside the chunks that missed
 *
 * Conventions
 *   - Plain C, no C++ or framework types.  Every call returns an irm_status.
 *   - Pointers named d_* are DEVICE pointers owned by the caller; all others
 *     are host pointers.  The library never frees or reallocates caller
 *     memory.  The hot-path calls (cdc_chunk, chunk_hash, lookup, reattach)
 *     allocate nothing, do not synchronise, and only enqueue kernels on the
 *     caller's stream (`stream` is a hipStream_t passed as void*; NULL is the
 *     default stream).  They record no memset nodes, so a caller may capture
 *     them into a HIP graph.
 *   - Host-checkable preconditions are verified before anything is launched
 *     and reported as IRM_ERR_INVALID_ARG / IRM_ERR_CAPACITY /
 *     IRM_ERR_UNSUPPORTED.  Conditions only the device can see (an index
 *     outside its pool, a full table, more chunks than `chunk_capacity`) make
 *     the kernel skip the offending item and raise a bit in the context's
 *     device error word, read with irm_ctx_error_flags().
 *   - Counts produced on the device (number of chunks, number of hits) stay
 *     on the device and are consumed there by the next call: nothing between
 *     the four calls needs the host.
 *   - A context serialises its scratch memory: calls on the same context must
 *     be ordered on one stream (or otherwise not overlap).
 *
 * KV row layout: 576 bf16 = [ c_KV: 512 | k_r: 64 ] = 1152 bytes
 * (paper Sec. 2 "MLA", App. C), or, with irm_config.row_format = IRM_ROW_FP8,
 * 656 bytes = [ c_KV: 512 E4M3 codes | 4 fp32 block scales | k_r: 64 bf16 ].
 * Rotary pair i of k_r is elements (i, i + 32) (half-split, the default) or
 * (2i, 2i + 1) (interleaved): irm_config.pair_mode.
 */
#ifndef IRM_H
#define IRM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum irm_status {
    IRM_OK = 0,
    IRM_ERR_INVALID_ARG = 1, /* null pointer, zero size, misaligned row, min > max ...      */
    IRM_ERR_CAPACITY = 2,    /* an argument exceeds what the context / a buffer was sized for */
    IRM_ERR_UNSUPPORTED = 3, /* dims other than 512+64, pair mode other than half-split ...  */
    IRM_ERR_DEVICE = 4,      /* a HIP runtime call failed (no GPU, out of memory, ...)       */
    IRM_ERR_TABLE_FULL = 5   /* irm_table_insert found no free slot                          */
} irm_status;

/* bits of the device error word */
#define IRM_FLAG_CHUNK_OVERFLOW 0x1u /* more chunks than chunk_capacity; extra chunks dropped   */
#define IRM_FLAG_TABLE_FULL 0x2u     /* an insert found no free slot                             */
#define IRM_FLAG_ROW_RANGE 0x4u      /* a hit or slot pointed outside its pool; row skipped      */
#define IRM_FLAG_BAD_CHUNK 0x8u      /* a chunk record pointed outside the token array; skipped  */
#define IRM_FLAG_WAIT_TIMEOUT 0x10u  /* a bounded in-kernel wait gave up (irm_attend_ref); the
                                        kernel ended, its results are not to be used              */

/* which two k_r elements form rotary pair i (App. D: DSv2-form and DSv3-form rotaries) */
#define IRM_PAIR_HALF_SPLIT 0u  /* elements i and i + 32 */
#define IRM_PAIR_INTERLEAVED 1u /* elements 2i and 2i + 1 */
#define IRM_KR_PAIRS 32

/* layout of one token's KV row in every pool the library reads or writes: a position-free
 * part, then k_r as 64 bf16 elements.  The position-free part is moved bit for bit, the
 * rotation acts on k_r alone (Alg. 1 steps 9-10), so a quantised c_KV needs no arithmetic. */
#define IRM_ROW_BF16 0u /* 1152 bytes: c_KV as 512 bf16 | k_r                                   */
#define IRM_ROW_FP8 1u  /* 656 bytes: c_KV as 512 e4m3 bytes | four fp32 scales, one per 128
                           elements | k_r (Sec. 7.2 counts FP8 KV quantisation as accepted
                           practice; this is the layout published for fp8 MLA caches)          */

typedef struct irm_config {
    /* CDC (paper Sec. 4, Sec. 7.2 "CDC boundary rule", App. B) */
    uint32_t gear[256];   /* gear table; one step per token, indexed by the id's low byte */
    uint32_t mask;        /* 2^k - 1, k <= 32; a cut needs (state & mask) == 0             */
    uint32_t min_chunk;   /* >= max(k, 1)                                                   */
    uint32_t max_chunk;   /* >= min_chunk, <= 65536                                         */
    /* lookup (Sec. 7.1): chunks at absolute position < carve_out are never served; 0 = off */
    uint32_t carve_out;
    /* KV geometry: only 512 + 64; pair_mode is IRM_PAIR_HALF_SPLIT or IRM_PAIR_INTERLEAVED;
     * row_format is IRM_ROW_BF16 or IRM_ROW_FP8 */
    uint32_t n_layers;
    uint32_t ckv_dim;
    uint32_t kr_dim;
    uint32_t pair_mode;
    uint32_t row_format;
    /* the model's fp32 rotary inverse frequencies (App. D: cos/sin are derived from
     * this buffer, never from a position table); pure rotation, no magnitude factor */
    float inv_freq[IRM_KR_PAIRS];
    /* sizing of the context's scratch: largest token count / request count per call */
    uint64_t max_tokens;
    uint32_t max_requests;
} irm_config;

/* registry value: where a cached chunk's rows live and where it was computed */
typedef struct irm_entry {
    uint32_t src_row;  /* first row in the source pool; the chunk's rows are contiguous */
    int32_t p_src;     /* absolute position of the chunk's first token when cached      */
    uint32_t len;      /* tokens in the chunk                                           */
    uint32_t entry_id; /* caller's tag, < 2^31; reported in chunk_entry on a hit        */
} irm_entry;

/* one re-attachable chunk of the current batch */
typedef struct irm_hit {
    uint32_t src_row; /* first source-pool row                                           */
    uint32_t dst_tok; /* index of the chunk's first token in the batch (into dst_slots) */
    uint32_t len;     /* rows                                                            */
    int32_t delta;    /* new position - stored position                                  */
} irm_hit;

typedef struct irm_ctx irm_ctx;
typedef struct irm_table irm_table;

/* bytes of one row, and of its position-free part, in a row format */
static inline uint32_t irm_row_bytes(uint32_t row_format) { return row_format == IRM_ROW_FP8 ? 656u : 1152u; }
static inline uint32_t irm_ckv_bytes(uint32_t row_format) { return row_format == IRM_ROW_FP8 ? 528u : 1024u; }

/* Chunks a batch can produce at most, given per-request lengths n_r:
 * sum over r of (n_r / min_chunk + 1).  A safe bound from totals only. */
static inline uint64_t irm_chunk_capacity_bound(uint64_t n_tokens, uint32_t n_req, uint32_t min_chunk)
{
    return n_tokens / (min_chunk ? min_chunk : 1) + n_req;
}

/* ---- lifetime (not on the hot path; these allocate and may synchronise) ---- */

/* Validates cfg, allocates the context's constant tables and scratch on the
 * current HIP device.  *out is set only on IRM_OK. */
irm_status irm_ctx_create(const irm_config *cfg, irm_ctx **out);
irm_status irm_ctx_destroy(irm_ctx *ctx);

/* Blocks until `stream` is idle, then returns the device error word in *flags
 * and clears it. */
irm_status irm_ctx_error_flags(irm_ctx *ctx, void *stream, uint32_t *flags);

/* Registry R: hash -> entry (Alg. 1 "Require", steps 7 and 13), an
 * open-addressing table of n_slots slots in device memory owned by the table. */
irm_status irm_table_create(irm_ctx *ctx, uint64_t n_slots, irm_table **out);
irm_status irm_table_destroy(irm_table *table);

/* Insert-if-absent of n (hash, entry) pairs (Alg. 1 step 13 inserts only on a
 * miss, so the first entry offered for a hash stays: within a batch the lowest
 * index wins, and earlier batches win over later ones).  Deterministic.
 * d_hash, d_val: device arrays of n.  A full table raises IRM_FLAG_TABLE_FULL. */
irm_status irm_table_insert(irm_table *table, const uint64_t *d_hash, const irm_entry *d_val,
                            uint32_t n, void *stream);

/* ---- hot path ------------------------------------------------------------ */

/* Gear-hash CDC (Sec. 4; Sec. 7.2; App. B).  Per request the rolling state
 * starts at 0 and takes one step per token, h = (h << 1) + gear[id & 0xFF]
 * (32-bit); the chunk that starts at s ends at the first token i with
 * i - s + 1 >= min_chunk and (h_i & mask) == 0, or at s + max_chunk - 1, or at
 * the request's last token, whichever comes first.
 *   d_tokens           int32[n_tokens], all requests concatenated
 *   d_req_offsets      uint32[n_req + 1], ascending, [0] = 0, [n_req] = n_tokens
 *   d_chunk_start/len  uint32[chunk_capacity] out, offsets into d_tokens, ascending
 *   d_req_chunk_offsets uint32[n_req + 1] out, request r owns chunks [r], [r+1])
 *   d_n_chunks         uint32[1] out
 * Needs n_tokens <= cfg.max_tokens, n_req <= cfg.max_requests and
 * chunk_capacity >= irm_chunk_capacity_bound(n_tokens, n_req, min_chunk)
 * (else IRM_ERR_CAPACITY).  The offsets are only seen on the device: a request whose
 * offsets run backwards or past n_tokens yields no chunks and raises IRM_FLAG_BAD_CHUNK;
 * the chunks of requests that overlap such a one are then unspecified (every access
 * stays inside the arrays). */
irm_status irm_cdc_chunk(irm_ctx *ctx, const int32_t *d_tokens, uint64_t n_tokens,
                         const uint32_t *d_req_offsets, uint32_t n_req, uint32_t *d_chunk_start,
                         uint32_t *d_chunk_len, uint32_t *d_req_chunk_offsets,
                         uint32_t *d_n_chunks, uint32_t chunk_capacity, void *stream);

/* Chunk fingerprint (Sec. 4; Alg. 1 steps 2, 7): FNV-1a-64 over the chunk's
 * token ids taken as little-endian bytes.
 *   d_chunk_hash uint64[chunk_capacity] out; entries >= *d_n_chunks untouched. */
irm_status irm_chunk_hash(irm_ctx *ctx, const int32_t *d_tokens, uint64_t n_tokens,
                          const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                          const uint32_t *d_n_chunks, uint32_t chunk_capacity,
                          uint64_t *d_chunk_hash, void *stream);

/* Registry probe (Alg. 1 steps 4-8; Sec. 7.1).  Chunk c of request r sits at
 * p = d_pos_base[r] + (chunk_start[c] - req_offsets[r]).  It is a miss if
 * p < carve_out, a hit if the table holds its hash with the same length, a
 * miss otherwise.
 *   d_chunk_entry int32[chunk_capacity] out: entry_id or -1
 *   d_hits        irm_hit[chunk_capacity] out: the hits in ascending chunk order
 *   d_n_hits      uint32[1] out;  d_hit_tokens uint64[1] out (sum of hit lengths) */
irm_status irm_lookup(irm_ctx *ctx, const irm_table *table, const uint64_t *d_chunk_hash,
                      const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                      const uint32_t *d_req_chunk_offsets, const uint32_t *d_req_offsets,
                      const int32_t *d_pos_base, uint32_t n_req, const uint32_t *d_n_chunks,
                      uint32_t chunk_capacity, int32_t *d_chunk_entry, irm_hit *d_hits,
                      uint32_t *d_n_hits, uint64_t *d_hit_tokens, void *stream);

/* Fused gather + delta-rotation + scatter (Alg. 1 steps 8-10; Sec. 7.2 "k_r
 * rotation"; App. C "k_r rotation materialisation").  For every hit h, layer l
 * and j < len:
 *   dst[l][ d_dst_slots[dst_tok + j] ][0:512]  = src[l][src_row + j][0:512]   (bit copy)
 *   dst[l][ ... ][512 + i], [512 + 32 + i]     = the pair (k_i, k_{i+32}) turned by
 *                                                delta * inv_freq[i], i < 32
 * with the angle reduced in fp64, the rotation in fp32 and one
 * round-to-nearest-even to bf16.  (Element indices of IRM_ROW_BF16 rows; in IRM_ROW_FP8
 * rows the first 528 bytes are the bit copy and the 64 bf16 of k_r follow them.)
 *   d_src_layer_ptrs / d_dst_layer_ptrs  device arrays of n_layers device pointers
 *                                        to row 0 of each layer (16-byte aligned)
 *   *_row_stride_bytes                   >= irm_row_bytes(row_format), multiple of 16
 *   src_rows / dst_rows                  rows per layer (bounds: a hit that reaches outside the
 *                                        source pool or past d_dst_slots, and a row whose slot
 *                                        lies outside the destination pool, are skipped and
 *                                        raise IRM_FLAG_ROW_RANGE)
 *   d_dst_slots                          int32[n_slots_tokens]: destination row per batch token
 *   d_hits, d_n_hits                     as written by irm_lookup; *d_n_hits <= hit_capacity
 * Destination rows of different hits must not overlap; src and dst pools must
 * not alias.  Rows no hit covers are not touched. */
irm_status irm_reattach(irm_ctx *ctx, const void *const *d_src_layer_ptrs,
                        uint64_t src_row_stride_bytes, uint64_t src_rows,
                        void *const *d_dst_layer_ptrs, uint64_t dst_row_stride_bytes,
                        uint64_t dst_rows, const int32_t *d_dst_slots, uint64_t n_slot_tokens,
                        const irm_hit *d_hits, const uint32_t *d_n_hits, uint32_t hit_capacity,
                        void *stream);

/* irm_reattach for callers that cannot allocate device memory and hold no context: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arithmetic, kernels, preconditions and results as irm_reattach; what a context would
 * supply comes as arguments (inv_freq: HOST array of the 32 fp32 inverse frequencies;
 * n_layers, pair_mode, row_format as in irm_config), and the call's scratch (tile list,
 * per-hit rotation table) lives in a fixed array inside the library's device image, about
 * 1.25 MB on every GPU the library runs on, held until the process ends.  The call
 * allocates nothing, frees nothing and does not synchronise.  The first call on a device
 * looks the array's address up (once per device); make that call outside a graph capture.
 *   n_slot_tokens  <= IRM_REATTACH_STATIC_MAX_TOKENS, hit_capacity <= IRM_REATTACH_STATIC_MAX_HITS
 *                  (else IRM_ERR_CAPACITY, nothing is launched)
 *   d_error_flags  optional device word the kernels OR the IRM_FLAG_* bits into (the
 *                  caller clears and reads it); NULL: the bits are dropped
 * All calls on one GPU share that GPU's array: calls that overlap in time on the same GPU
 * (two streams, two threads) race on it and must be ordered by the caller. */
#define IRM_REATTACH_STATIC_MAX_TOKENS 131072u
#define IRM_REATTACH_STATIC_MAX_HITS 4096u
irm_status irm_reattach_static(const float *inv_freq, uint32_t n_layers, uint32_t pair_mode, uint32_t row_format,
                               const void *const *d_src_layer_ptrs, uint64_t src_row_stride_bytes,
                               uint64_t src_rows, void *const *d_dst_layer_ptrs, uint64_t dst_row_stride_bytes,
                               uint64_t dst_rows, const int32_t *d_dst_slots, uint64_t n_slot_tokens,
                               const irm_hit *d_hits, const uint32_t *d_n_hits, uint32_t hit_capacity,
                               uint32_t *d_error_flags, void *stream);

/* Split-pool variant of irm_reattach (App. C "Split TokenToKVPool"): the shared,
 * content-addressed pool keeps the position-free c_KV, which is only referenced; the
 * 64-dim k_r slice alone is materialised per request.  For every hit h, j < len,
 * slot = d_dst_slots[dst_tok + j]:
 *   d_ckv_index[slot]          = src_row + j   (the pool row whose c_KV the token uses)
 *   kr[l][slot][0:64]          = the k_r of source row src_row + j of layer l, rotated by delta
 *   d_src_kr_layer_ptrs        device array of n_layers pointers to the k_r slice (64 bf16) of
 *                              source row 0: base + irm_ckv_bytes(row_format) for packed
 *                              rows, or the base of a dense k_r_base pool
 *   src_kr_row_stride_bytes    >= 128, multiple of 16 (1152 for packed rows, 128 for a dense pool)
 *   d_kr_layer_ptrs            device array of n_layers pointers to [kr_rows][64] bf16
 *   kr_row_stride_bytes        >= 128, multiple of 16
 *   d_ckv_index                int32[kr_rows]; entries of rows no hit covers are untouched
 * Same arithmetic, error reporting and preconditions as irm_reattach.  Traffic is
 * 256 bytes per token and layer instead of 2304. */
irm_status irm_reattach_kr(irm_ctx *ctx, const void *const *d_src_kr_layer_ptrs,
                           uint64_t src_kr_row_stride_bytes, uint64_t src_rows,
                           void *const *d_kr_layer_ptrs, uint64_t kr_row_stride_bytes, uint64_t kr_rows,
                           int32_t *d_ckv_index, const int32_t *d_dst_slots, uint64_t n_slot_tokens,
                           const irm_hit *d_hits, const uint32_t *d_n_hits, uint32_t hit_capacity,
                           void *stream);

/* No-materialise variant of the re-attachment (Sec. 7.2 and App. C propose to apply the
 * rotation inside the attention kernel while it loads the keys, leaving k_r_base in HBM as
 * it was stored and writing no rotated copy).  No KV is moved.  For every hit h, j < len and
 * slot = d_dst_slots[dst_tok + j]:
 *   d_row_index[slot] = src_row + j   pool row that holds the slot's (c_KV, k_r_base)
 *   d_hit_index[slot] = h             which rotation the load path applies to that row
 * and d_trig[h][i] = (cos, sin)(delta_h * inv_freq[i]), i < 32, fp32 pairs in pair order
 * (exactly (1, 0) when delta = 0; angle reduced in fp64).  A consumer, an attention
 * kernel that rotates k_r on load, is irm_attend_ref below.
 *   d_row_index, d_hit_index  int32[dst_rows], slots no hit covers are left as they were
 *   d_trig                    float[hit_capacity][32][2], 8-byte aligned
 * Bad indices are skipped and flagged like in irm_reattach. */
irm_status irm_reattach_ref(irm_ctx *ctx, uint64_t src_rows, int32_t *d_row_index, int32_t *d_hit_index,
                            uint64_t dst_rows, float *d_trig, const int32_t *d_dst_slots,
                            uint64_t n_slot_tokens, const irm_hit *d_hits, const uint32_t *d_n_hits,
                            uint32_t hit_capacity, void *stream);

/* The consumer of irm_reattach_ref: MLA decode attention in the latent form, one layer
 * (Sec. 2 "MLA": per token a 512-dim c_KV and a 64-dim RoPE key, V derived from c_KV;
 * Sec. 7.2, App. C: the delta-rotation fused into the attention load path).  For request
 * b, head h and the request's context slots s_t = d_kv_slots[d_kv_offsets[b] + t]:
 *   row_t = d_row_index[s_t],  R_t = rotation d_trig[d_hit_index[s_t]] (identity if < 0)
 *   score_t = scale * q[b][h] . [ c_KV(row_t) | R_t k_r_base(row_t) ],  p = softmax_t
 *   d_out[b][h][0:512] = sum_t p_t c_KV(row_t),   d_lse[b][h] = log sum_t exp(score_t)
 * k_r is rotated in fp32 and rounded once to bf16 while the rows are staged on chip (the
 * values irm_reattach would have written); products in bf16 MFMA with fp32 accumulation.
 *   d_q            bf16 [n_req][n_heads][576] (latent-space query | rotary query), 16-byte aligned;
 *                  n_heads a multiple of 16, at most IRM_ATTEND_MAX_QUERY_ROWS (the pool rows are
 *                  streamed once per 16 heads, or once per 32 / 64 when n_heads is a multiple of
 *                  32 / 64).  In the latent form every (query token, head) pair is one more query
 *                  row over the same keys, so a step with several query tokens per request whose
 *                  context lies wholly before them (new tokens over a re-attached prefix) passes
 *                  n_heads = tokens * heads, rows ordered [token][head]; attention among the new
 *                  tokens themselves is the caller's, joined through d_lse
 *   d_pool_layer   one layer of the pool, rows of 576 bf16 (or fp8 rows, see below) at
 *                  pool_row_stride_bytes
 *   d_kv_slots     int32, d_kv_offsets uint32[n_req + 1]: CSR of every request's context slots
 *   d_row_index, d_hit_index  int32[dst_rows] as written by irm_reattach_ref (plain rows of
 *                  prefilled tokens: any pool row with hit index -1)
 *   d_trig         float[trig_hits][32][2] as written by irm_reattach_ref, trig_hits >= 1
 *   n_splits       workgroups per request and 16 heads (split of the context, merged afterwards)
 *   d_workspace    irm_attend_ref_workspace_bytes(n_req, n_heads, n_splits) bytes, 16-byte aligned
 *   d_out          float[n_req][n_heads][512];  d_lse float[n_req][n_heads]
 * A request without context gives out = 0, lse = -inf (so does one whose offsets run
 * backwards, which also raises IRM_FLAG_BAD_CHUNK; d_kv_slots must hold d_kv_offsets[n_req]
 * entries).  A slot, row or hit index out of range leaves that token out and raises
 * IRM_FLAG_ROW_RANGE.  Allocates nothing, does not
 * synchronise.  In an IRM_ROW_FP8 context d_pool_layer holds 656-byte rows: c_KV element d is
 * then the E4M3 value (finite-only form, largest 448) of byte d times the fp32 scale of its
 * block of 128.  The codes enter the products exactly (as bf16); a score's four block sums
 * take their scales in fp32, and on the output side the scale goes into the softmax
 * numerator before that is rounded to bf16.  (With a multiple of 32 heads the elements are
 * scaled and rounded once to bf16 as the rows are staged instead.)  Everything else is the
 * same. */
#define IRM_ATTEND_MAX_QUERY_ROWS 8192u
uint64_t irm_attend_ref_workspace_bytes(uint32_t n_req, uint32_t n_heads, uint32_t n_splits);
irm_status irm_attend_ref(irm_ctx *ctx, const void *d_q, uint32_t n_req, uint32_t n_heads,
                          const void *d_pool_layer, uint64_t pool_row_stride_bytes, uint64_t pool_rows,
                          const int32_t *d_kv_slots, const uint32_t *d_kv_offsets, const int32_t *d_row_index,
                          const int32_t *d_hit_index, uint64_t dst_rows, const float *d_trig, uint32_t trig_hits,
                          float scale, uint32_t n_splits, void *d_workspace, uint64_t workspace_bytes,
                          float *d_out, float *d_lse, void *stream);

/* irm_table_insert with the count kept on the device: the first min(*d_n, capacity)
 * pairs are offered (for lists another call of this library produced). */
irm_status irm_table_insert_counted(irm_table *table, const uint64_t *d_hash, const irm_entry *d_val,
                                    const uint32_t *d_n, uint32_t capacity, void *stream);

/* S1, detect-and-recover (Sec. 4 "CDC+fallback"; App. G "S1"): chunks whose fingerprint
 * missed are sub-divided into fixed windows of `window` tokens (the paper's 128), which are
 * then fingerprinted and looked up like chunks: hand the window list to irm_chunk_hash and
 * irm_lookup (d_req_win_offsets in the place of d_req_chunk_offsets, d_n_windows in the
 * place of d_n_chunks) and the hits to irm_reattach.  This call is the sub-division.
 * A selected chunk of length len yields floor(len / window) whole windows; a remainder is
 * not probed.  anchor IRM_S1_ANCHOR_START counts them from the chunk's first token,
 * IRM_S1_ANCHOR_END back from its last token (the paper does not say; a chunk's end is
 * fixed by content alone, its start also by what precedes it).
 *   d_select / select_mode   which chunks: IRM_S1_SELECT_NEGATIVE (d_select[c] < 0: the
 *                            misses of irm_lookup's d_chunk_entry), IRM_S1_SELECT_NONNEGATIVE
 *                            (d_select[c] >= 0: the chunks irm_admit placed, d_admitted_row),
 *                            IRM_S1_SELECT_ALL (d_select may be null)
 *   d_win_start, d_win_len, d_win_parent   uint32[window_capacity] out: first token, length
 *                            (= window), index of the chunk the window was cut from;
 *                            ascending token order
 *   d_req_win_offsets        uint32[n_req + 1] out, CSR over requests;  d_n_windows uint32[1] out
 *   d_win_entry              optional irm_entry[window_capacity] out, only with
 *                            IRM_S1_SELECT_NONNEGATIVE and d_select = irm_admit's d_admitted_row:
 *                            the registry value of each window (rows inside its chunk's pool
 *                            rows, its own position), ready for irm_table_insert_counted;
 *                            needs d_req_offsets and d_pos_base (else they may be null)
 * More windows than window_capacity: the surplus is dropped, IRM_FLAG_CHUNK_OVERFLOW. */
#define IRM_S1_SELECT_NEGATIVE 0u
#define IRM_S1_SELECT_NONNEGATIVE 1u
#define IRM_S1_SELECT_ALL 2u
#define IRM_S1_ANCHOR_START 0u
#define IRM_S1_ANCHOR_END 1u
irm_status irm_s1_windows(irm_ctx *ctx, const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                          const uint32_t *d_req_chunk_offsets, uint32_t n_req, const uint32_t *d_n_chunks,
                          uint32_t chunk_capacity, const int32_t *d_select, uint32_t select_mode,
                          uint32_t window, uint32_t anchor, const uint32_t *d_req_offsets,
                          const int32_t *d_pos_base, uint32_t *d_win_start, uint32_t *d_win_len,
                          uint32_t *d_win_parent, uint32_t *d_req_win_offsets, uint32_t *d_n_windows,
                          uint32_t window_capacity, irm_entry *d_win_entry, void *stream);

/* Miss path (Alg. 1 steps 11-13).  Chunks the lookup missed have been prefilled by the
 * engine into the request's slots; irm_admit copies their rows into fresh rows of the
 * shared pool and registers them, insert-if-absent.  Chunks are taken in ascending order;
 * chunk c is admitted when d_chunk_entry[c] < 0, its position p >= carve_out, its hash is
 * not registered yet (earlier batches win, then the lowest chunk of this batch), and the
 * pool still has len rows behind *d_cursor; the first chunk that does not fit closes the
 * pool for the rest of the batch (refused chunks leave the registry as it was).  An admitted chunk gets rows [cursor, cursor + len): every layer's rows are
 * copied bit for bit from req[l][d_slots[chunk_start + j]], the registry learns
 * hash -> {src_row = first row, p_src = p, len, entry_id = first row}, the cursor advances.
 *   d_chunk_* / d_req_* / d_pos_base / d_n_chunks   as written by irm_cdc_chunk / irm_chunk_hash
 *   d_chunk_entry        int32[chunk_capacity] as written by irm_lookup for the same batch
 *   d_req_layer_ptrs     request KV pool, rows of 576 bf16 (read);  d_pool_layer_ptrs: shared pool (written)
 *   d_cursor             uint32[1] in/out: first free pool row
 *   d_admitted_row       int32[chunk_capacity] out: first pool row of chunk c, or -1
 * Deterministic.  Needs table n_slots < 2^32 - 16.  Not to be overlapped with lookups of
 * the same table.  The rank that makes "first offer wins" hold across batches lives in
 * device memory, so this call (like irm_table_insert) may be captured and replayed. */
irm_status irm_admit(irm_ctx *ctx, irm_table *table, const uint64_t *d_chunk_hash,
                     const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                     const uint32_t *d_req_chunk_offsets, const uint32_t *d_req_offsets,
                     const int32_t *d_pos_base, uint32_t n_req, const uint32_t *d_n_chunks,
                     uint32_t chunk_capacity, const int32_t *d_chunk_entry,
                     const void *const *d_req_layer_ptrs, uint64_t req_row_stride_bytes, uint64_t req_rows,
                     const int32_t *d_slots, uint64_t n_slot_tokens, void *const *d_pool_layer_ptrs,
                     uint64_t pool_row_stride_bytes, uint64_t pool_rows, uint32_t *d_cursor,
                     int32_t *d_admitted_row, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* IRM_H */
