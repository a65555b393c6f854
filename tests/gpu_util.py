"""Shared helpers of the GPU parity tests (not collected by pytest).

Every expected value comes from ``oracle/``; the GPU library is only ever the
thing under test.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl
from paper_2605_05696_amd.pipeline import Session

DEV = "cuda:0"
ROW = 576


def oracle_front(w):
    """Oracle chunking, fingerprints, registry and lookup of a workload."""
    st, ln, rco = orc.cdc_chunk(w.tokens, w.req_offsets, w.gear, w.mask, w.min_chunk, w.max_chunk)
    ch = orc.chunk_hash(w.tokens, st, ln)
    reg = w.registry(orc.chunk_hash(w.pool_tokens, w.pool_chunk_start, w.pool_chunk_len))
    entry, hits, hit_tokens = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"],
                                         reg["entry_id"], ch, st, ln, rco, w.req_offsets, w.pos_base,
                                         w.carve_out)
    return dict(start=st, len=ln, rco=rco, hash=ch, reg=reg, entry=entry, hits=hits,
                hit_tokens=hit_tokens)


def hits_to_dev(hits: orc.Hits, cap: int, device=DEV):
    """Oracle hit list -> device tensor laid out as irm_hit[cap] plus the count."""
    rec = np.zeros(cap, B.HIT_DTYPE)
    n = len(hits)
    rec["src_row"][:n], rec["dst_tok"][:n] = hits.src_row, hits.dst_tok
    rec["len"][:n], rec["delta"][:n] = hits.len, hits.delta
    d_hits = torch.from_numpy(rec.view(np.int32).reshape(cap, 4).copy()).to(device)
    d_n = torch.tensor([n], dtype=torch.int32, device=device)
    return d_hits, d_n


def hits_from_dev(d_hits, n) -> orc.Hits:
    rec = d_hits.cpu().numpy().view(np.uint32).reshape(-1, 4)[:n]
    return orc.Hits(rec[:, 0].copy(), rec[:, 1].copy(), rec[:, 2].copy(), rec[:, 3].view(np.int32).copy())


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor (any device) -> uint16 numpy bit patterns."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def ordered(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> integers whose difference counts representable steps."""
    mag = (b & 0x7FFF).astype(np.int32)
    return np.where(b & 0x8000, -mag, mag)


def compare_rows(got: np.ndarray, want: np.ndarray, what=""):
    """got/want: [..., 576 or 328] uint16.  The position-free part (c_KV, for fp8 rows with its
    scales) bit-exact; k_r within 2 bf16 steps of the oracle's fp64-rounded value, or within 1e-2
    absolute."""
    assert got.shape == want.shape and got.shape[-1] in (576, 328)
    ckv = got.shape[-1] - 64
    ckv_bad = np.nonzero(got[..., :ckv] != want[..., :ckv])
    assert len(ckv_bad[0]) == 0, f"{what}: c_KV differs at {[a[:5] for a in ckv_bad]}"
    g, o = got[..., ckv:], want[..., ckv:]
    step = np.abs(ordered(g) - ordered(o))
    far = step > 2
    if far.any():
        diff = np.abs(orc.bf16_to_f64(g[far]) - orc.bf16_to_f64(o[far]))
        assert np.all(diff <= 1e-2), f"{what}: k_r off by {diff.max()} ({int(far.sum())} values past 2 steps)"
    return dict(max_step=int(step.max()) if step.size else 0,
                exact=float((step == 0).mean()) if step.size else 1.0)


def verify_reattach(w, hits: orc.Hits, src_dev, dst_dev, hit_sel=None, layers=None, what="", pair_mode=0):
    """Recompute the selected hits x layers with the oracle from D2H copies of the
    source rows and compare with the rows the GPU wrote."""
    L = src_dev.shape[0]
    layers = list(range(L)) if layers is None else list(layers)
    sel = np.arange(len(hits)) if hit_sel is None else np.asarray(hit_sel)
    if len(sel) == 0:
        return dict(max_step=0, exact=1.0, rows=0)
    lens = hits.len[sel].astype(np.int64)
    off = np.concatenate([[0], np.cumsum(lens)])
    within = np.arange(off[-1]) - np.repeat(off[:-1], lens)
    src_idx = np.repeat(hits.src_row[sel].astype(np.int64), lens) + within
    tok_idx = np.repeat(hits.dst_tok[sel].astype(np.int64), lens) + within
    dst_idx = w.dst_slots[tok_idx].astype(np.int64)
    d_src_idx = torch.from_numpy(src_idx).to(src_dev.device)
    d_dst_idx = torch.from_numpy(dst_idx).to(src_dev.device)
    src_c = np.stack([bits(src_dev[l].index_select(0, d_src_idx)) for l in layers])
    got = np.stack([bits(dst_dev[l].index_select(0, d_dst_idx)) for l in layers])
    want = np.full_like(got, wl.SENTINEL_BF16)
    compact = orc.Hits(off[:-1].astype(np.uint32), off[:-1].astype(np.uint32), lens.astype(np.uint32),
                       hits.delta[sel].copy())
    orc.reattach(src_c, want, np.arange(off[-1], dtype=np.int32), compact, w.inv_freq, pair_mode)
    out = compare_rows(got, want, what)
    out["rows"] = int(off[-1]) * len(layers)
    return out


def covered_rows(w, hits: orc.Hits) -> np.ndarray:
    """Boolean mask over destination rows that some hit writes."""
    mask = np.zeros(w.dst_rows, bool)
    for t, l in zip(hits.dst_tok.astype(np.int64), hits.len.astype(np.int64)):
        mask[w.dst_slots[t:t + l]] = True
    return mask


class Rig:
    """A workload on the device: session, token arrays, pools, table."""

    def __init__(self, w, o=None, with_pools=True, with_table=True, pair_mode=0, row_format=0):
        self.w = w
        self.o = o if o is not None else oracle_front(w)
        self.s = Session.for_workload(w, DEV, pair_mode=pair_mode, row_format=row_format)
        self.row_bytes = B.ROW_WORDS[row_format] * 2
        self.d_tokens = torch.from_numpy(w.tokens).to(DEV)
        self.d_req_offsets = self.s.to_dev_u32(w.req_offsets)
        self.d_pos_base = torch.from_numpy(w.pos_base).to(DEV)
        self.d_dst_slots = torch.from_numpy(w.dst_slots).to(DEV)
        self.buf = self.s.alloc_front(len(w.tokens), w.n_req)
        if with_table:
            self.s.build_table(w.table_slots, self.o["reg"])
        if with_pools:
            name = w.name.split("-")[0]
            make = wl.kv_pool_fp8_torch if row_format == B.IRM_ROW_FP8 else wl.kv_pool_torch
            self.src = make(w.n_layers, w.src_rows, wl.kv_seed(name), DEV)
            self.dst = wl.sentinel_pool_torch(w.n_layers, w.dst_rows, DEV, B.ROW_WORDS[row_format])
            self.src_ptrs = B.layer_pointers(self.src)
            self.dst_ptrs = B.layer_pointers(self.dst)

    def reattach(self, d_hits, d_n_hits):
        B.irm_reattach(self.s.ctx, self.src_ptrs, self.row_bytes, self.w.src_rows, self.dst_ptrs, self.row_bytes,
                       self.w.dst_rows, self.d_dst_slots, d_hits, d_n_hits)

    def serve(self):
        self.s.serve(self.d_tokens, self.d_req_offsets, self.d_pos_base, self.d_dst_slots, self.src_ptrs,
                     self.row_bytes, self.w.src_rows, self.dst_ptrs, self.row_bytes, self.w.dst_rows, self.buf)

    def close(self):
        self.s.close()
