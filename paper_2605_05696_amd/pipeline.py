"""Buffer ownership around the four C-ABI calls: a context, a registry table and
the device arrays the calls hand to each other.  Allocation and marshalling
only -- every computation is a library call in ``binding``.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _u32(x) -> torch.Tensor:
    """numpy uint32/int32 -> int32 device-ready CPU tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(x).astype(np.uint32, copy=False).view(np.int32).copy())


def _u64(x) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint64).view(np.int64).copy())


class Session:
    """One context (+ optional registry) on the current device."""

    def __init__(self, gear, mask, min_chunk, max_chunk, carve_out, n_layers, inv_freq,
                 max_tokens, max_requests, device="cuda:0", pair_mode=0, row_format=0):
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = B.make_config(gear, mask, min_chunk, max_chunk, carve_out, n_layers, inv_freq,
                                 max_tokens, max_requests, pair_mode=pair_mode, row_format=row_format)
        self.min_chunk = min_chunk
        self.n_layers = n_layers
        self.ctx = B.irm_ctx_create(self.cfg)
        self.table = None

    @classmethod
    def for_workload(cls, w, device="cuda:0", max_tokens=None, max_requests=None, pair_mode=0, row_format=0):
        n_max = max(len(w.tokens), len(w.pool_tokens), 1)
        return cls(w.gear, w.mask, w.min_chunk, w.max_chunk, w.carve_out, w.n_layers, w.inv_freq,
                   max_tokens or n_max, max_requests or max(w.n_req, 1), device, pair_mode, row_format)

    def close(self):
        if self.table is not None:
            B.irm_table_destroy(self.table)
            self.table = None
        if self.ctx is not None:
            B.irm_ctx_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- helpers that move small host arrays to the device --------------------
    def to_dev_u32(self, x):
        return _u32(x).to(self.device)

    def to_dev_u64(self, x):
        return _u64(x).to(self.device)

    def error_flags(self) -> int:
        return B.irm_ctx_error_flags(self.ctx)

    # -- front end: chunk + fingerprint ---------------------------------------
    def alloc_front(self, n_tokens: int, n_req: int):
        cap = int(n_tokens // self.min_chunk + n_req)
        cap = max(cap, 1)
        d = self.device
        i32, i64 = torch.int32, torch.int64
        return dict(cap=cap,
                    chunk_start=torch.zeros(cap, dtype=i32, device=d),
                    chunk_len=torch.zeros(cap, dtype=i32, device=d),
                    req_chunk_offsets=torch.zeros(n_req + 1, dtype=i32, device=d),
                    n_chunks=torch.zeros(1, dtype=i32, device=d),
                    chunk_hash=torch.zeros(cap, dtype=i64, device=d),
                    chunk_entry=torch.full((cap,), -1, dtype=i32, device=d),
                    hits=torch.zeros((cap, 4), dtype=i32, device=d),
                    n_hits=torch.zeros(1, dtype=i32, device=d),
                    hit_tokens=torch.zeros(1, dtype=i64, device=d))

    def chunk_and_hash(self, d_tokens, d_req_offsets, buf):
        B.irm_cdc_chunk(self.ctx, d_tokens, d_req_offsets, buf["chunk_start"], buf["chunk_len"],
                        buf["req_chunk_offsets"], buf["n_chunks"])
        B.irm_chunk_hash(self.ctx, d_tokens, buf["chunk_start"], buf["chunk_len"], buf["n_chunks"],
                         buf["chunk_hash"])

    def chunk_host(self, tokens, req_offsets):
        """Chunk + fingerprint host arrays on the GPU and bring the results back.
        -> (chunk_start u32, chunk_len u32, req_chunk_offsets u32, chunk_hash u64)"""
        tokens = np.ascontiguousarray(tokens, np.int32)
        n_req = len(req_offsets) - 1
        buf = self.alloc_front(len(tokens), n_req)
        d_tok = torch.from_numpy(tokens).to(self.device) if len(tokens) else \
            torch.zeros(1, dtype=torch.int32, device=self.device)[:0]
        self.chunk_and_hash(d_tok, self.to_dev_u32(req_offsets), buf)
        n = int(buf["n_chunks"].item())
        view = lambda t, dt: t.cpu().numpy().view(dt)
        return (view(buf["chunk_start"], np.uint32)[:n].copy(), view(buf["chunk_len"], np.uint32)[:n].copy(),
                view(buf["req_chunk_offsets"], np.uint32).copy(), view(buf["chunk_hash"], np.uint64)[:n].copy())

    # -- registry ---------------------------------------------------------------
    def build_table(self, n_slots: int, reg: dict, batch: int = 1 << 20):
        """Create the table and insert the registry entry list in order."""
        if self.table is not None:
            B.irm_table_destroy(self.table)
        self.table = B.irm_table_create(self.ctx, int(n_slots))
        n = len(reg["hash"])
        vals = np.zeros(n, B.ENTRY_DTYPE)
        for k in ("src_row", "p_src", "len", "entry_id"):
            vals[k] = reg[k]
        vals = vals.view(np.int32).reshape(n, 4)
        for a in range(0, n, batch):
            b = min(n, a + batch)
            B.irm_table_insert(self.table, self.to_dev_u64(reg["hash"][a:b]),
                               torch.from_numpy(vals[a:b].copy()).to(self.device))
        torch.cuda.synchronize(self.device)

    # -- the hot path -------------------------------------------------------------
    def serve(self, d_tokens, d_req_offsets, d_pos_base, d_dst_slots, src_ptrs, src_stride, src_rows,
              dst_ptrs, dst_stride, dst_rows, buf, stream=None):
        """The four calls back to back on one stream; nothing returns to the host."""
        B.irm_cdc_chunk(self.ctx, d_tokens, d_req_offsets, buf["chunk_start"], buf["chunk_len"],
                        buf["req_chunk_offsets"], buf["n_chunks"], stream)
        B.irm_chunk_hash(self.ctx, d_tokens, buf["chunk_start"], buf["chunk_len"], buf["n_chunks"],
                         buf["chunk_hash"], stream)
        B.irm_lookup(self.ctx, self.table, buf["chunk_hash"], buf["chunk_start"], buf["chunk_len"],
                     buf["req_chunk_offsets"], d_req_offsets, d_pos_base, buf["n_chunks"],
                     buf["chunk_entry"], buf["hits"], buf["n_hits"], buf["hit_tokens"], stream)
        B.irm_reattach(self.ctx, src_ptrs, src_stride, src_rows, dst_ptrs, dst_stride, dst_rows,
                       d_dst_slots, buf["hits"], buf["n_hits"], stream)

    def serve_kr(self, d_tokens, d_req_offsets, d_pos_base, d_dst_slots, src_ptrs, src_stride, src_rows,
                 kr_ptrs, kr_stride, kr_rows, d_ckv_index, buf, stream=None):
        """Same front end, split-pool back end: only k_r is materialised, c_KV is referenced.
        ``src_ptrs`` point at the k_r slice of source row 0 of every layer."""
        B.irm_cdc_chunk(self.ctx, d_tokens, d_req_offsets, buf["chunk_start"], buf["chunk_len"],
                        buf["req_chunk_offsets"], buf["n_chunks"], stream)
        B.irm_chunk_hash(self.ctx, d_tokens, buf["chunk_start"], buf["chunk_len"], buf["n_chunks"],
                         buf["chunk_hash"], stream)
        B.irm_lookup(self.ctx, self.table, buf["chunk_hash"], buf["chunk_start"], buf["chunk_len"],
                     buf["req_chunk_offsets"], d_req_offsets, d_pos_base, buf["n_chunks"],
                     buf["chunk_entry"], buf["hits"], buf["n_hits"], buf["hit_tokens"], stream)
        B.irm_reattach_kr(self.ctx, src_ptrs, src_stride, src_rows, kr_ptrs, kr_stride, kr_rows,
                          d_ckv_index, d_dst_slots, buf["hits"], buf["n_hits"], stream)

    def serve_ref(self, d_tokens, d_req_offsets, d_pos_base, d_dst_slots, src_rows, d_row_index, d_hit_index,
                  d_trig, buf, stream=None):
        """Same front end, no-materialise back end: references and the per-hit rotation table only."""
        B.irm_cdc_chunk(self.ctx, d_tokens, d_req_offsets, buf["chunk_start"], buf["chunk_len"],
                        buf["req_chunk_offsets"], buf["n_chunks"], stream)
        B.irm_chunk_hash(self.ctx, d_tokens, buf["chunk_start"], buf["chunk_len"], buf["n_chunks"],
                         buf["chunk_hash"], stream)
        B.irm_lookup(self.ctx, self.table, buf["chunk_hash"], buf["chunk_start"], buf["chunk_len"],
                     buf["req_chunk_offsets"], d_req_offsets, d_pos_base, buf["n_chunks"],
                     buf["chunk_entry"], buf["hits"], buf["n_hits"], buf["hit_tokens"], stream)
        B.irm_reattach_ref(self.ctx, src_rows, d_row_index, d_hit_index, d_trig, d_dst_slots, buf["hits"],
                           buf["n_hits"], stream)

    def admit(self, d_req_offsets, d_pos_base, d_slots, req_ptrs, req_stride, req_rows, pool_ptrs, pool_stride,
              pool_rows, d_cursor, d_admitted_row, buf, stream=None):
        """Miss path after the engine prefilled the missed chunks into the request's slots:
        copy them into free pool rows and register them.  ``buf`` holds the chunk arrays and
        chunk_entry of the lookup of the same batch."""
        B.irm_admit(self.ctx, self.table, buf["chunk_hash"], buf["chunk_start"], buf["chunk_len"],
                    buf["req_chunk_offsets"], d_req_offsets, d_pos_base, buf["n_chunks"], buf["chunk_entry"],
                    req_ptrs, req_stride, req_rows, d_slots, pool_ptrs, pool_stride, pool_rows, d_cursor,
                    d_admitted_row, stream)

    # -- S1 fallback: fixed windows inside the chunks that missed -------------------------
    def alloc_windows(self, n_tokens: int, n_req: int, window: int = 128):
        """Buffers of a window list: laid out like ``alloc_front`` so that the same calls take it."""
        cap = max(int(n_tokens // window), 1)
        d = self.device
        i32, i64 = torch.int32, torch.int64
        return dict(cap=cap, window=window,
                    chunk_start=torch.zeros(cap, dtype=i32, device=d),
                    chunk_len=torch.zeros(cap, dtype=i32, device=d),
                    parent=torch.zeros(cap, dtype=i32, device=d),
                    req_chunk_offsets=torch.zeros(n_req + 1, dtype=i32, device=d),
                    n_chunks=torch.zeros(1, dtype=i32, device=d),
                    chunk_hash=torch.zeros(cap, dtype=i64, device=d),
                    chunk_entry=torch.full((cap,), -1, dtype=i32, device=d),
                    entries=torch.zeros((cap, 4), dtype=i32, device=d),
                    hits=torch.zeros((cap, 4), dtype=i32, device=d),
                    n_hits=torch.zeros(1, dtype=i32, device=d),
                    hit_tokens=torch.zeros(1, dtype=i64, device=d))

    def windows_host(self, tokens, chunk_start, chunk_len, req_chunk_offsets, window=128, anchor=B.S1_ANCHOR_END):
        """All fixed windows of a host chunk list, cut and fingerprinted on the GPU.
        -> (win_start u32, win_len u32, win_parent u32, win_hash u64)"""
        n_tok, n_req = len(tokens), len(req_chunk_offsets) - 1
        wbuf = self.alloc_windows(n_tok, n_req, window)
        d_tok = torch.from_numpy(np.ascontiguousarray(tokens, np.int32)).to(self.device)
        B.irm_s1_windows(self.ctx, self.to_dev_u32(chunk_start), self.to_dev_u32(chunk_len),
                         self.to_dev_u32(req_chunk_offsets),
                         torch.tensor([len(chunk_start)], dtype=torch.int32, device=self.device), None,
                         B.S1_SELECT_ALL, window, anchor, wbuf["chunk_start"], wbuf["chunk_len"], wbuf["parent"],
                         wbuf["req_chunk_offsets"], wbuf["n_chunks"])
        B.irm_chunk_hash(self.ctx, d_tok, wbuf["chunk_start"], wbuf["chunk_len"], wbuf["n_chunks"],
                         wbuf["chunk_hash"])
        n = int(wbuf["n_chunks"].item())
        view = lambda t, dt: t.cpu().numpy().view(dt)[:n].copy()
        return (view(wbuf["chunk_start"], np.uint32), view(wbuf["chunk_len"], np.uint32),
                view(wbuf["parent"], np.uint32), view(wbuf["chunk_hash"], np.uint64))

    def s1_serve(self, d_tokens, d_req_offsets, d_pos_base, d_dst_slots, src_ptrs, src_stride, src_rows,
                 dst_ptrs, dst_stride, dst_rows, buf, wbuf, anchor=B.S1_ANCHOR_END, stream=None):
        """After ``serve`` on the same batch: sub-divide the chunks it missed, fingerprint and look
        up the windows, re-attach the window hits."""
        B.irm_s1_windows(self.ctx, buf["chunk_start"], buf["chunk_len"], buf["req_chunk_offsets"], buf["n_chunks"],
                         buf["chunk_entry"], B.S1_SELECT_NEGATIVE, wbuf["window"], anchor, wbuf["chunk_start"],
                         wbuf["chunk_len"], wbuf["parent"], wbuf["req_chunk_offsets"], wbuf["n_chunks"],
                         stream=stream)
        B.irm_chunk_hash(self.ctx, d_tokens, wbuf["chunk_start"], wbuf["chunk_len"], wbuf["n_chunks"],
                         wbuf["chunk_hash"], stream)
        B.irm_lookup(self.ctx, self.table, wbuf["chunk_hash"], wbuf["chunk_start"], wbuf["chunk_len"],
                     wbuf["req_chunk_offsets"], d_req_offsets, d_pos_base, wbuf["n_chunks"],
                     wbuf["chunk_entry"], wbuf["hits"], wbuf["n_hits"], wbuf["hit_tokens"], stream)
        B.irm_reattach(self.ctx, src_ptrs, src_stride, src_rows, dst_ptrs, dst_stride, dst_rows,
                       d_dst_slots, wbuf["hits"], wbuf["n_hits"], stream)

    def s1_register(self, d_tokens, d_req_offsets, d_pos_base, d_admitted_row, buf, wbuf,
                    anchor=B.S1_ANCHOR_END, stream=None):
        """After ``admit``: register the windows of the chunks it placed (rows inside their pool rows)."""
        B.irm_s1_windows(self.ctx, buf["chunk_start"], buf["chunk_len"], buf["req_chunk_offsets"], buf["n_chunks"],
                         d_admitted_row, B.S1_SELECT_NONNEGATIVE, wbuf["window"], anchor, wbuf["chunk_start"],
                         wbuf["chunk_len"], wbuf["parent"], wbuf["req_chunk_offsets"], wbuf["n_chunks"],
                         d_req_offsets, d_pos_base, wbuf["entries"], stream)
        B.irm_chunk_hash(self.ctx, d_tokens, wbuf["chunk_start"], wbuf["chunk_len"], wbuf["n_chunks"],
                         wbuf["chunk_hash"], stream)
        B.irm_table_insert_counted(self.table, wbuf["chunk_hash"], wbuf["entries"], wbuf["n_chunks"], stream)
