// S1, detect-and-recover (paper Sec. 4 "CDC+fallback"; App. G "S1"): chunks whose
// fingerprint missed are sub-divided into fixed windows (the paper's 128 tokens) that are
// then fingerprinted and looked up like chunks, by the same kernels.  This file holds the
// sub-division only: a selected chunk of length len yields floor(len / window) whole
// windows, counted from its first token (anchor 0) or back from its last token (anchor 1;
// a chunk's end is fixed by content alone, its start also by what precedes it).
//
//   s1_expand   one workgroup walks the chunk list 1024 chunks at a time: a block scan of
//               the window counts gives every chunk the index of its first window, each
//               lane writes its own chunk's windows (at most max_chunk / window of them),
//               and the per-request CSR is read off the per-chunk prefix afterwards.
//               With an admitted-row array as the selector it also emits the registry
//               value of every window (rows inside the parent chunk's pool rows).
#include "irm_internal.hpp"

__global__ __launch_bounds__(1024) void s1_expand(
    const uint32_t *__restrict__ chunk_start, const uint32_t *__restrict__ chunk_len,
    const uint32_t *__restrict__ req_chunk_offsets, uint32_t n_req, const uint32_t *__restrict__ n_chunks_p,
    uint32_t chunk_capacity, const int32_t *__restrict__ select, uint32_t select_mode, uint32_t window,
    uint32_t anchor, const uint32_t *__restrict__ req_offsets, const int32_t *__restrict__ pos_base,
    uint32_t *__restrict__ win_start, uint32_t *__restrict__ win_len, uint32_t *__restrict__ win_parent,
    uint32_t *__restrict__ req_win_offsets, uint32_t *__restrict__ n_windows, uint32_t window_capacity,
    irm_entry *__restrict__ win_entry, uint32_t *prefix, uint32_t *err)
{
    __shared__ uint32_t lds[17];
    __shared__ uint32_t carry_sh;
    uint32_t n_chunks = *n_chunks_p;
    if (n_chunks > chunk_capacity) n_chunks = chunk_capacity;
    if (threadIdx.x == 0) carry_sh = 0;
    __syncthreads();
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += blockDim.x) {
        const uint32_t c = c0 + threadIdx.x;
        uint32_t n = 0, start = 0, len = 0;
        int32_t sel = 0;
        if (c < n_chunks) {
            start = chunk_start[c];
            len = chunk_len[c];
            bool on = true;
            if (select_mode != 2u) {
                sel = select[c];
                on = select_mode == 0u ? sel < 0 : sel >= 0;
            }
            if (on) n = len / window;
        }
        uint32_t total;
        const uint32_t incl = irm_block_scan_incl(n, lds, &total);
        const uint32_t first = carry_sh + incl - n;
        if (c < n_chunks) prefix[c] = first < window_capacity ? first : window_capacity;
        const uint32_t tok0 = anchor ? start + len - n * window : start;
        for (uint32_t j = 0; j < n; ++j) {
            const uint32_t w = first + j;
            if (w >= window_capacity) {
                atomicOr(err, IRM_FLAG_CHUNK_OVERFLOW);
                break;
            }
            const uint32_t ws = tok0 + j * window;
            win_start[w] = ws;
            win_len[w] = window;
            win_parent[w] = c;
            if (win_entry) {                                 // select holds the chunk's first pool row
                irm_entry e;
                e.src_row = (uint32_t)sel + (ws - start);
                e.p_src = (int32_t)irm_chunk_pos(req_chunk_offsets, req_offsets, pos_base, n_req, c, ws);
                e.len = window;
                e.entry_id = e.src_row;
                win_entry[w] = e;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) carry_sh += total;
        __syncthreads();
    }
    const uint32_t total = carry_sh < window_capacity ? carry_sh : window_capacity;
    for (uint32_t r = threadIdx.x; r <= n_req; r += blockDim.x) {
        const uint32_t c = r < n_req ? req_chunk_offsets[r] : n_chunks;
        req_win_offsets[r] = c < n_chunks ? prefix[c] : total;
    }
    if (threadIdx.x == 0) *n_windows = total;
}

extern "C" irm_status irm_s1_windows(irm_ctx *ctx, const uint32_t *d_chunk_start, const uint32_t *d_chunk_len,
                                     const uint32_t *d_req_chunk_offsets, uint32_t n_req,
                                     const uint32_t *d_n_chunks, uint32_t chunk_capacity, const int32_t *d_select,
                                     uint32_t select_mode, uint32_t window, uint32_t anchor,
                                     const uint32_t *d_req_offsets, const int32_t *d_pos_base,
                                     uint32_t *d_win_start, uint32_t *d_win_len, uint32_t *d_win_parent,
                                     uint32_t *d_req_win_offsets, uint32_t *d_n_windows,
                                     uint32_t window_capacity, irm_entry *d_win_entry, void *stream)
{
    if (!ctx || !d_chunk_start || !d_chunk_len || !d_req_chunk_offsets || !d_n_chunks || !d_win_start ||
        !d_win_len || !d_win_parent || !d_req_win_offsets || !d_n_windows)
        return IRM_ERR_INVALID_ARG;
    if (select_mode > IRM_S1_SELECT_ALL || anchor > IRM_S1_ANCHOR_END || window < 1 || n_req < 1 ||
        chunk_capacity < 1 || window_capacity < 1)
        return IRM_ERR_INVALID_ARG;
    if (select_mode != IRM_S1_SELECT_ALL && !d_select) return IRM_ERR_INVALID_ARG;
    if (d_win_entry && (select_mode != IRM_S1_SELECT_NONNEGATIVE || !d_req_offsets || !d_pos_base))
        return IRM_ERR_INVALID_ARG;
    if (n_req > ctx->cfg.max_requests || chunk_capacity > ctx->chunk_cap) return IRM_ERR_CAPACITY;
    hipLaunchKernelGGL(s1_expand, dim3(1), dim3(1024), 0, (hipStream_t)stream, d_chunk_start, d_chunk_len,
                       d_req_chunk_offsets, n_req, d_n_chunks, chunk_capacity, d_select, select_mode, window,
                       anchor, d_req_offsets, d_pos_base, d_win_start, d_win_len, d_win_parent, d_req_win_offsets,
                       d_n_windows, window_capacity, d_win_entry, ctx->d_slot_of, ctx->d_err);
    return irm_launch_status();
}
