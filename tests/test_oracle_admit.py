"""Pins for the oracle's miss path (paper Alg. 1 steps 11-13: prefill, then
R[hash] <- (c_KV, k_r_base, p)).

Closed loop: serve a batch, admit its misses, serve the SAME batch again: every
chunk past the carve-out must now hit with delta = 0, and re-attaching it must
reproduce the prefilled rows bit for bit (delta = 0 is the identity).  Plus the
insert-if-absent rules on a hand-made case.
"""
import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import workloads as wl


def bf16_bits(x):
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def concat_reg(a, b):
    return {k: np.concatenate([a[k], b[k]]) for k in a}


@pytest.mark.parametrize("name", ["c1", "c2", "c4"])
def test_admit_then_everything_hits_at_delta_zero(name):
    w = wl.make_workload(name, orc.cdc_chunk, size="small")
    rng = np.random.default_rng(11)
    L = 2
    st, ln, rco = orc.cdc_chunk(w.tokens, w.req_offsets, w.gear, w.mask, w.min_chunk, w.max_chunk)
    ch = orc.chunk_hash(w.tokens, st, ln)
    reg = w.registry(orc.chunk_hash(w.pool_tokens, w.pool_chunk_start, w.pool_chunk_len))
    look = lambda rg: orc.lookup(rg["hash"], rg["src_row"], rg["p_src"], rg["len"], rg["entry_id"], ch, st, ln,
                                 rco, w.req_offsets, w.pos_base, w.carve_out)
    entry, hits, hit_tokens = look(reg)
    n_miss_tokens = int(ln[entry < 0].sum())
    assert 0 < n_miss_tokens < len(w.tokens)
    # the request pool as the engine left it after prefilling the misses
    req = bf16_bits(rng.standard_normal((L, w.dst_rows, 576)))
    free0 = w.src_rows
    pool = np.full((L, free0 + n_miss_tokens, 576), wl.SENTINEL_BF16, np.uint16)
    admitted, new, cursor = orc.admit(reg["hash"], ch, st, ln, rco, w.req_offsets, w.pos_base, w.carve_out,
                                      entry, req, w.dst_slots, pool, free0)
    # who was admitted: misses past the carve-out (fresh content is unique here)
    pos = np.concatenate([w.pos_base[r] + st[rco[r]:rco[r + 1]].astype(np.int64) - int(w.req_offsets[r])
                          for r in range(w.n_req)])
    eligible = (entry < 0) & (pos >= w.carve_out)
    assert np.array_equal(admitted >= 0, eligible)
    assert cursor == free0 + int(ln[eligible].sum())
    rows = admitted[eligible]
    assert np.array_equal(rows, free0 + np.concatenate([[0], np.cumsum(ln[eligible])[:-1]]))  # packed, in order
    assert np.array_equal(new["p_src"], pos[eligible]) and np.array_equal(new["len"], ln[eligible])
    assert np.all(pool[:, :free0] == wl.SENTINEL_BF16)                       # old rows untouched
    # second pass over the same batch
    entry2, hits2, hit_tokens2 = look(concat_reg(reg, new))
    assert np.array_equal(entry2 >= 0, pos >= w.carve_out)
    was_miss = np.isin(hits2.dst_tok, st[eligible])
    assert np.all(hits2.delta[was_miss] == 0)
    assert hit_tokens2 == hit_tokens + int(ln[eligible].sum())
    # re-attaching the admitted chunks gives back the prefilled rows exactly
    out = np.full((L, w.dst_rows, 576), wl.SENTINEL_BF16, np.uint16)
    sel = orc.Hits(hits2.src_row[was_miss], hits2.dst_tok[was_miss], hits2.len[was_miss], hits2.delta[was_miss])
    orc.reattach(pool, out, w.dst_slots, sel, w.inv_freq)
    for t0, l in zip(sel.dst_tok.astype(np.int64), sel.len.astype(np.int64)):
        rws = w.dst_slots[t0:t0 + l]
        assert np.array_equal(out[:, rws], req[:, rws])


def test_insert_if_absent_carve_out_and_pool_full():
    L = 1
    start = np.array([0, 64, 128, 192, 256, 320, 448], np.uint32)
    length = np.array([64, 64, 64, 64, 64, 128, 8], np.uint32)
    rco = np.array([0, 7], np.uint32)
    off = np.array([0, 456], np.uint32)
    pos_base = np.array([0], np.int32)
    ch = np.array([10, 11, 11, 12, 13, 14, 15], np.uint64)   # chunk 2 repeats chunk 1's content
    reg_hash = np.array([12], np.uint64)                     # hash 12 is known (with another length, say)
    entry = np.array([-1, -1, -1, -1, 5, -1, -1], np.int32)  # chunk 4 was a hit
    req = (np.arange(L * 456 * 576) % 65521).astype(np.uint16).reshape(L, 456, 576)
    slots = np.arange(456, dtype=np.int32)[::-1].copy()
    pool = np.zeros((L, 100 + 64 + 10, 576), np.uint16)      # room for ONE more 64-row chunk after row 100
    admitted, new, cursor = orc.admit(reg_hash, ch, start, length, rco, off, pos_base, 32, entry, req, slots,
                                      pool, 100)
    # chunk 0: carve-out; 1: admitted; 2: same hash as 1 -> absent no more; 3: hash known; 4: hit;
    # 5: does not fit and closes the pool; 6: would fit (8 rows) but the pool is closed for this batch
    assert admitted.tolist() == [-1, 100, -1, -1, -1, -1, -1]
    assert cursor == 164 and new["hash"].tolist() == [11] and new["p_src"].tolist() == [64]
    assert np.array_equal(pool[0, 100:164], req[0, slots[64:128]])
    assert np.all(pool[0, 164:] == 0) and np.all(pool[0, :100] == 0)


def test_fp8_rows_are_admitted_whole():
    """656-byte rows (quantised c_KV, its scales, bf16 k_r) go into the pool bit for bit."""
    rng = np.random.default_rng(5)
    L, n = 2, 200
    start = np.array([0, 70, 140], np.uint32)
    length = np.array([70, 70, 60], np.uint32)
    req = rng.integers(0, 65536, (L, n, 328), dtype=np.uint16)
    slots = rng.permutation(n).astype(np.int32)
    pool = np.zeros((L, 150, 328), np.uint16)
    admitted, new, cursor = orc.admit(np.zeros(0, np.uint64), np.array([7, 8, 9], np.uint64), start, length,
                                      np.array([0, 3], np.uint32), np.array([0, n], np.uint32),
                                      np.array([100], np.int32), 32, np.full(3, -1, np.int32), req, slots, pool, 5)
    assert admitted.tolist() == [5, 75, -1] and cursor == 145       # the third chunk does not fit
    assert np.array_equal(pool[:, 5:75], req[:, slots[0:70]]) and np.array_equal(pool[:, 75:145], req[:, slots[70:140]])
    assert np.all(pool[:, :5] == 0) and np.all(pool[:, 145:] == 0)
    assert new["p_src"].tolist() == [100, 170] and new["src_row"].tolist() == [5, 75]
