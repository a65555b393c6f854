"""A serving loop in miniature: ``python -m paper_2605_05696_amd.example`` (needs an MI355X).

A shared pool starts empty.  A first request misses everywhere, is "prefilled" by the caller
(here: random rows stand in for the model's KV) and admitted (Alg. 1 steps 11-13).  A second
request carries the later part of the first one's text behind a fresh head: its chunks are found
at other positions and re-attached, c_KV copied and k_r rotated by the shift (Alg. 1 steps 2-10).
Everything runs through the C ABI of ``libirm.so``; this file only owns buffers.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workloads as wl
from .pipeline import Session

L, MAX_TOKENS, POOL_ROWS = 4, 16384, 32768           # layers, longest batch, rows of the shared pool
ROW = 576                                            # bf16 per row: 512 of c_KV, 64 of k_r


def main() -> dict:
    assert torch.cuda.is_available(), "this example needs a GPU"
    dev = "cuda:0"
    rng = np.random.default_rng(7)
    text = rng.integers(0, 102400, 12000).astype(np.int32)

    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, L, wl.inv_freq_plain(), MAX_TOKENS, 1, dev)
    try:
        s.table = B.irm_table_create(s.ctx, 4096)    # empty registry
        pool = torch.zeros((L, POOL_ROWS, ROW), dtype=torch.bfloat16, device=dev)
        pool_ptrs = B.layer_pointers(pool)
        cursor = torch.zeros(1, dtype=torch.int32, device=dev)      # next free pool row

        def request(tokens, kv_seed):
            """One request through the path: serve what is cached, admit what was not."""
            n = len(tokens)
            d_tok = torch.from_numpy(tokens).to(dev)
            d_off = s.to_dev_u32(np.array([0, n], np.uint32))
            d_pos = torch.zeros(1, dtype=torch.int32, device=dev)
            d_slots = torch.arange(n, dtype=torch.int32, device=dev)                # token t -> KV slot t
            kv = torch.zeros((L, n, ROW), dtype=torch.bfloat16, device=dev)         # the request's KV slots
            buf = s.alloc_front(n, 1)
            s.serve(d_tok, d_off, d_pos, d_slots, pool_ptrs, ROW * 2, POOL_ROWS, B.layer_pointers(kv), ROW * 2, n, buf)
            hit_tokens = int(buf["hit_tokens"].item())
            # the model would now prefill the tokens no hit covered; random rows stand in for it
            covered = torch.zeros(n, dtype=torch.bool, device=dev)
            hits = buf["hits"][:int(buf["n_hits"].item())].cpu().numpy().view(np.uint32)
            for _, dst_tok, length, _ in hits:
                covered[int(dst_tok):int(dst_tok) + int(length)] = True
            fresh = wl.kv_pool_torch(L, n, kv_seed, dev)
            kv[:, ~covered] = fresh[:, ~covered]
            admitted = torch.full((buf["cap"],), -1, dtype=torch.int32, device=dev)
            s.admit(d_off, d_pos, d_slots, B.layer_pointers(kv), ROW * 2, n, pool_ptrs, ROW * 2, POOL_ROWS, cursor,
                    admitted, buf)
            torch.cuda.synchronize()
            assert s.error_flags() == 0
            n_chunks = int(buf["n_chunks"].item())
            return dict(chunks=n_chunks, hits=len(hits), hit_tokens=hit_tokens,
                        admitted=int((admitted[:n_chunks] >= 0).sum().item()), kv=kv, hit_list=hits)

        # first request: nothing is cached yet
        a = request(text, 1)
        print(f"request 1: {len(text)} tokens, {a['chunks']} chunks, {a['hits']} hits, {a['admitted']} chunks admitted, "
              f"pool rows in use {int(cursor.item())}")
        # second request: a fresh head, then the same text from its 21st chunk on (found at shifted positions)
        buf = s.alloc_front(len(text), 1)
        s.chunk_and_hash(torch.from_numpy(text).to(dev), s.to_dev_u32(np.array([0, len(text)], np.uint32)), buf)
        cut = int(buf["chunk_start"][20].item())                  # a chunk boundary of the stored text
        head = rng.integers(0, 102400, 777).astype(np.int32)
        b = request(np.concatenate([head, text[cut:]]), 2)
        print(f"request 2: {777 + len(text) - cut} tokens, {b['chunks']} chunks, {b['hits']} hits covering "
              f"{b['hit_tokens']} tokens, {b['admitted']} new chunks admitted")
        # what a hit did: c_KV equals the first request's rows bit for bit, k_r is rotated by delta
        src_row, dst_tok, length, delta = (int(v) for v in b["hit_list"][len(b["hit_list"]) // 2])
        delta -= (1 << 32) if delta >= (1 << 31) else 0
        same = torch.equal(b["kv"][:, dst_tok:dst_tok + length, :512].view(torch.int16),
                           pool[:, src_row:src_row + length, :512].view(torch.int16))
        print(f"a hit: {length} tokens from pool row {src_row} to slot {dst_tok}, delta {delta}: c_KV identical: {same}")
        return dict(first=(a["chunks"], a["hits"], a["admitted"]), second=(b["chunks"], b["hits"], b["hit_tokens"]),
                    delta=delta, ckv_identical=same)
    finally:
        s.close()


if __name__ == "__main__":
    main()
