/* A plain C99 caller of libirm.so: no Python, no C++, only the header and the HIP runtime's C
 * API for device memory.  It caches a token stream (chunk, fingerprint, register), serves a
 * request that carries two slices of that stream behind a fresh head (Alg. 1 steps 2-10), and
 * checks what the path guarantees without an oracle: every hit is found at the shift it was moved
 * by, its c_KV arrives bit for bit, the rotation keeps every rotary pair's length to within bf16
 * rounding, and rows no hit covers are left alone.  Prints one line and returns 0 when all of
 * it holds.
 *
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude abi_client.c -lirm -lamdhip64 -lm
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "irm.h"

#define LAYERS 2u
#define ROW_ELEMS 576u
#define POOL_TOKENS 6000u
#define MAX_TOKENS 8192u

#define HIP_OK(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                   \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define IRM_OK_(call)                                                                    \
    do {                                                                                 \
        irm_status s_ = (call);                                                          \
        if (s_ != IRM_OK) {                                                              \
            fprintf(stderr, "%s: status %d\n", #call, (int)s_);                          \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}

static uint16_t to_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
static float from_bf16(uint16_t b)
{
    const uint32_t u = (uint32_t)b << 16;
    float x;
    memcpy(&x, &u, 4);
    return x;
}

typedef struct front {
    uint32_t *start, *len, *rco, *n_chunks;   /* device */
    uint64_t *hash;                           /* device */
    uint32_t cap;
} front;

static int front_alloc(front *f, uint32_t cap, uint32_t n_req)
{
    f->cap = cap;
    HIP_OK(hipMalloc((void **)&f->start, cap * 4u));
    HIP_OK(hipMalloc((void **)&f->len, cap * 4u));
    HIP_OK(hipMalloc((void **)&f->rco, (n_req + 1u) * 4u));
    HIP_OK(hipMalloc((void **)&f->n_chunks, 4u));
    HIP_OK(hipMalloc((void **)&f->hash, cap * 8u));
    return 0;
}

int main(void)
{
    /* context: the measured configurations' CDC rule, plain RoPE frequencies */
    static irm_config cfg;
    for (int i = 0; i < 256; ++i) cfg.gear[i] = rnd();
    cfg.mask = 0xFFu;
    cfg.min_chunk = 64;
    cfg.max_chunk = 1024;
    cfg.carve_out = 32;
    cfg.n_layers = LAYERS;
    cfg.ckv_dim = 512;
    cfg.kr_dim = 64;
    cfg.pair_mode = IRM_PAIR_HALF_SPLIT;
    cfg.row_format = IRM_ROW_BF16;
    for (int i = 0; i < IRM_KR_PAIRS; ++i) cfg.inv_freq[i] = (float)pow(10000.0, -2.0 * i / 64.0);
    cfg.max_tokens = MAX_TOKENS;
    cfg.max_requests = 1;
    irm_ctx *ctx = NULL;
    IRM_OK_(irm_ctx_create(&cfg, &ctx));

    /* the cached stream: chunk and fingerprint it, register every chunk where it lies */
    static int32_t pool_tok[POOL_TOKENS];
    for (uint32_t i = 0; i < POOL_TOKENS; ++i) pool_tok[i] = (int32_t)(rnd() % 102400u);
    int32_t *d_tok = NULL;
    uint32_t *d_off = NULL;
    HIP_OK(hipMalloc((void **)&d_tok, MAX_TOKENS * 4u));
    HIP_OK(hipMalloc((void **)&d_off, 8u));
    const uint32_t cap = (uint32_t)irm_chunk_capacity_bound(MAX_TOKENS, 1, cfg.min_chunk);
    front f;
    if (front_alloc(&f, cap, 1)) return 2;
    uint32_t off[2] = {0u, POOL_TOKENS};
    HIP_OK(hipMemcpy(d_tok, pool_tok, sizeof pool_tok, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_off, off, sizeof off, hipMemcpyHostToDevice));
    IRM_OK_(irm_cdc_chunk(ctx, d_tok, POOL_TOKENS, d_off, 1, f.start, f.len, f.rco, f.n_chunks, cap, NULL));
    IRM_OK_(irm_chunk_hash(ctx, d_tok, POOL_TOKENS, f.start, f.len, f.n_chunks, cap, f.hash, NULL));
    uint32_t n_pool_chunks = 0;
    HIP_OK(hipMemcpy(&n_pool_chunks, f.n_chunks, 4, hipMemcpyDeviceToHost));
    if (n_pool_chunks < 12 || n_pool_chunks > cap) {
        fprintf(stderr, "unexpected chunk count %u\n", n_pool_chunks);
        return 4;
    }
    uint32_t *p_start = malloc(n_pool_chunks * 4u), *p_len = malloc(n_pool_chunks * 4u);
    irm_entry *entries = malloc(n_pool_chunks * sizeof(irm_entry));
    HIP_OK(hipMemcpy(p_start, f.start, n_pool_chunks * 4u, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(p_len, f.len, n_pool_chunks * 4u, hipMemcpyDeviceToHost));
    for (uint32_t c = 0; c < n_pool_chunks; ++c) {
        entries[c].src_row = p_start[c];
        entries[c].p_src = (int32_t)p_start[c];
        entries[c].len = p_len[c];
        entries[c].entry_id = c;
    }
    irm_table *table = NULL;
    IRM_OK_(irm_table_create(ctx, 4u * n_pool_chunks, &table));
    irm_entry *d_entries = NULL;
    HIP_OK(hipMalloc((void **)&d_entries, n_pool_chunks * sizeof(irm_entry)));
    HIP_OK(hipMemcpy(d_entries, entries, n_pool_chunks * sizeof(irm_entry), hipMemcpyHostToDevice));
    IRM_OK_(irm_table_insert(table, f.hash, d_entries, n_pool_chunks, NULL));

    /* the request: a fresh head, then chunks 6..9 and 2..4 of the cached stream */
    static int32_t req_tok[MAX_TOKENS];
    uint32_t n = 0;
    for (uint32_t i = 0; i < 333; ++i) req_tok[n++] = (int32_t)(rnd() % 102400u);
    const uint32_t a0 = p_start[6], a1 = p_start[10], b0 = p_start[2], b1 = p_start[5];
    memcpy(req_tok + n, pool_tok + a0, (a1 - a0) * 4u);
    n += a1 - a0;
    memcpy(req_tok + n, pool_tok + b0, (b1 - b0) * 4u);
    n += b1 - b0;
    off[1] = n;
    HIP_OK(hipMemcpy(d_tok, req_tok, n * 4u, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_off, off, sizeof off, hipMemcpyHostToDevice));

    /* pools: the cached rows, and the request's slots (token t -> row t) */
    const size_t row_bytes = ROW_ELEMS * 2u;
    const size_t src_bytes = (size_t)LAYERS * POOL_TOKENS * row_bytes, dst_bytes = (size_t)LAYERS * n * row_bytes;
    uint16_t *src_h = malloc(src_bytes), *dst_h = malloc(dst_bytes);
    for (size_t i = 0; i < src_bytes / 2; ++i) src_h[i] = to_bf16(((float)(rnd() & 0xFFFF) - 32768.0f) / 8192.0f);
    char *d_src = NULL, *d_dst = NULL;
    HIP_OK(hipMalloc((void **)&d_src, src_bytes));
    HIP_OK(hipMalloc((void **)&d_dst, dst_bytes));
    HIP_OK(hipMemcpy(d_src, src_h, src_bytes, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_dst, 0x7F, dst_bytes));
    const void *src_layers[LAYERS];
    void *dst_layers[LAYERS];
    for (uint32_t l = 0; l < LAYERS; ++l) {
        src_layers[l] = d_src + (size_t)l * POOL_TOKENS * row_bytes;
        dst_layers[l] = d_dst + (size_t)l * n * row_bytes;
    }
    const void **d_src_layers = NULL;
    void **d_dst_layers = NULL;
    HIP_OK(hipMalloc((void **)&d_src_layers, sizeof src_layers));
    HIP_OK(hipMalloc((void **)&d_dst_layers, sizeof dst_layers));
    HIP_OK(hipMemcpy(d_src_layers, src_layers, sizeof src_layers, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_dst_layers, dst_layers, sizeof dst_layers, hipMemcpyHostToDevice));
    int32_t *slots_h = malloc(n * 4u), *d_slots = NULL, *d_pos = NULL, *d_entry = NULL;
    for (uint32_t t = 0; t < n; ++t) slots_h[t] = (int32_t)t;
    HIP_OK(hipMalloc((void **)&d_slots, n * 4u));
    HIP_OK(hipMemcpy(d_slots, slots_h, n * 4u, hipMemcpyHostToDevice));
    HIP_OK(hipMalloc((void **)&d_pos, 4u));
    HIP_OK(hipMemset(d_pos, 0, 4u));
    HIP_OK(hipMalloc((void **)&d_entry, cap * 4u));
    irm_hit *d_hits = NULL;
    uint32_t *d_n_hits = NULL;
    uint64_t *d_hit_tokens = NULL;
    HIP_OK(hipMalloc((void **)&d_hits, cap * sizeof(irm_hit)));
    HIP_OK(hipMalloc((void **)&d_n_hits, 4u));
    HIP_OK(hipMalloc((void **)&d_hit_tokens, 8u));

    /* the serve path: four calls on one stream, nothing comes back in between */
    IRM_OK_(irm_cdc_chunk(ctx, d_tok, n, d_off, 1, f.start, f.len, f.rco, f.n_chunks, cap, NULL));
    IRM_OK_(irm_chunk_hash(ctx, d_tok, n, f.start, f.len, f.n_chunks, cap, f.hash, NULL));
    IRM_OK_(irm_lookup(ctx, table, f.hash, f.start, f.len, f.rco, d_off, d_pos, 1, f.n_chunks, cap, d_entry, d_hits,
                       d_n_hits, d_hit_tokens, NULL));
    IRM_OK_(irm_reattach(ctx, d_src_layers, row_bytes, POOL_TOKENS, d_dst_layers, row_bytes, n, d_slots, n, d_hits,
                         d_n_hits, cap, NULL));
    uint32_t flags = 0;
    IRM_OK_(irm_ctx_error_flags(ctx, NULL, &flags));
    if (flags) {
        fprintf(stderr, "device error word %#x\n", flags);
        return 5;
    }

    /* what came back */
    uint32_t n_hits = 0;
    uint64_t hit_tokens = 0;
    HIP_OK(hipMemcpy(&n_hits, d_n_hits, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&hit_tokens, d_hit_tokens, 8, hipMemcpyDeviceToHost));
    if (n_hits < 3 || n_hits > 7) {   /* seven cached chunks were offered; chunks behind a junction may drift */
        fprintf(stderr, "unexpected hit count %u\n", n_hits);
        return 6;
    }
    irm_hit *hits = malloc(n_hits * sizeof(irm_hit));
    HIP_OK(hipMemcpy(hits, d_hits, n_hits * sizeof(irm_hit), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dst_h, d_dst, dst_bytes, hipMemcpyDeviceToHost));
    double worst = 0.0;
    for (uint32_t h = 0; h < n_hits; ++h) {
        if ((int32_t)hits[h].dst_tok - (int32_t)hits[h].src_row != hits[h].delta) {   /* stored at its own offset */
            fprintf(stderr, "hit %u: delta %d does not match its rows\n", h, hits[h].delta);
            return 7;
        }
        for (uint32_t l = 0; l < LAYERS; ++l)
            for (uint32_t j = 0; j < hits[h].len; ++j) {
                const uint16_t *s = src_h + ((size_t)l * POOL_TOKENS + hits[h].src_row + j) * ROW_ELEMS;
                const uint16_t *d = dst_h + ((size_t)l * n + hits[h].dst_tok + j) * ROW_ELEMS;
                if (memcmp(s, d, 1024) != 0) {
                    fprintf(stderr, "hit %u layer %u row %u: c_KV differs\n", h, l, j);
                    return 8;
                }
                for (uint32_t i = 0; i < 32; ++i) {
                    const double a = from_bf16(s[512 + i]), b = from_bf16(s[544 + i]);
                    const double x = from_bf16(d[512 + i]), y = from_bf16(d[544 + i]);
                    const double before = sqrt(a * a + b * b), after = sqrt(x * x + y * y);
                    const double err = fabs(after - before) / (before + 1e-3);
                    if (err > worst) worst = err;
                }
            }
    }
    if (worst > 1.0 / 128.0) {   /* two bf16 roundings of a pair: 2^-8 each at most */
        fprintf(stderr, "a rotary pair changed its length by %.4g\n", worst);
        return 9;
    }
    /* rows no hit covers keep what was there */
    if (dst_h[0] != 0x7F7Fu) {
        fprintf(stderr, "the fresh head was written to\n");
        return 10;
    }
    printf("abi_client ok: %u cached chunks, %u hits covering %llu of %u tokens, pair lengths within %.2e\n",
           n_pool_chunks, n_hits, (unsigned long long)hit_tokens, n, worst);
    IRM_OK_(irm_table_destroy(table));
    IRM_OK_(irm_ctx_destroy(ctx));
    return 0;
}
