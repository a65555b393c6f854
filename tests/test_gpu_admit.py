"""GPU parity of the miss path (paper Alg. 1 steps 11-13) against the oracle:
which chunks are admitted and where, the pool bytes, the cursor, and what the
registry answers afterwards (a second lookup of the same batch)."""
import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl
from paper_2605_05696_amd.pipeline import Session

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_util import DEV, ROW, Rig, bits, hits_from_dev


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


def concat_reg(a, b):
    return {k: np.concatenate([a[k], b[k]]) for k in a}


def look(reg, o, w):
    return orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"], o["hash"],
                      o["start"], o["len"], o["rco"], w.req_offsets, w.pos_base, w.carve_out)


@pytest.mark.parametrize("room", ["all", "half"])
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_serve_admit_serve_matches_oracle(name, room):
    w = wl.make_workload(name, orc.cdc_chunk, size="small")
    rig = Rig(w)
    o, L = rig.o, w.n_layers
    try:
        n_chunks = len(o["start"])
        miss_tokens = int(o["len"][o["entry"] < 0].sum())
        extra = miss_tokens if room == "all" else miss_tokens // 2
        pool_rows = w.src_rows + extra
        pool = torch.cat([rig.src, wl.sentinel_pool_torch(L, extra, DEV)], dim=1).contiguous()
        pool_ptrs = B.layer_pointers(pool)
        # request pool: random rows everywhere, then the hits re-attached over them = "after prefill"
        rig.dst.copy_(wl.kv_pool_torch(L, w.dst_rows, 977, DEV))
        rig.serve()
        torch.cuda.synchronize()
        assert np.array_equal(rig.buf["chunk_entry"].cpu().numpy()[:n_chunks], o["entry"])
        req_h, pool_h = bits(rig.dst), bits(pool)
        d_cursor = torch.tensor([w.src_rows], dtype=torch.int32, device=DEV)
        d_adm = torch.full((rig.buf["cap"],), -7, dtype=torch.int32, device=DEV)
        rig.s.admit(rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.dst_ptrs, ROW * 2, w.dst_rows,
                    pool_ptrs, ROW * 2, pool_rows, d_cursor, d_adm, rig.buf)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        want_adm, new, want_cursor = orc.admit(o["reg"]["hash"], o["hash"], o["start"], o["len"], o["rco"],
                                               w.req_offsets, w.pos_base, w.carve_out, o["entry"], req_h,
                                               w.dst_slots, pool_h, w.src_rows)
        assert np.array_equal(d_adm.cpu().numpy()[:n_chunks], want_adm)
        assert int(d_cursor.item()) == want_cursor
        if room == "half":                                             # the case really runs out of rows
            pos = np.concatenate([w.pos_base[r] + o["start"][o["rco"][r]:o["rco"][r + 1]].astype(np.int64)
                                  - int(w.req_offsets[r]) for r in range(w.n_req)])
            assert ((o["entry"] < 0) & (pos >= w.carve_out) & (want_adm < 0)).any() and want_cursor <= pool_rows
        assert np.array_equal(bits(pool), pool_h)                      # pool_h was updated by the oracle
        assert np.array_equal(bits(rig.dst), req_h)                    # the request pool is only read
        # the same batch again: the registry now answers for the admitted chunks, delta = 0
        dst2 = wl.sentinel_pool_torch(L, w.dst_rows, DEV)
        rig.s.serve(rig.d_tokens, rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, pool_ptrs, ROW * 2,
                    pool_rows, B.layer_pointers(dst2), ROW * 2, w.dst_rows, rig.buf)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        entry2, hits2, hit_tokens2 = look(concat_reg(o["reg"], new), o, w)
        assert np.array_equal(rig.buf["chunk_entry"].cpu().numpy()[:n_chunks], entry2)
        got = hits_from_dev(rig.buf["hits"], int(rig.buf["n_hits"].item()))
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(got, f), getattr(hits2, f)), f
        assert int(rig.buf["hit_tokens"].item()) == hit_tokens2
        fresh = np.isin(hits2.dst_tok, o["start"][want_adm >= 0])
        assert fresh.sum() == (want_adm >= 0).sum() and np.all(hits2.delta[fresh] == 0)
        out2 = bits(dst2)
        for t0, l in zip(hits2.dst_tok[fresh].astype(np.int64), hits2.len[fresh].astype(np.int64)):
            rws = w.dst_slots[t0:t0 + l]
            assert np.array_equal(out2[:, rws], req_h[:, rws])         # delta = 0 gives the prefilled rows back
    finally:
        rig.close()


def hand_case():
    start = np.array([0, 64, 128, 192, 256, 320, 448, 456], np.uint32)
    length = np.array([64, 64, 64, 64, 64, 128, 8, 40], np.uint32)
    rco = np.array([0, 7, 8], np.uint32)
    off = np.array([0, 456, 496], np.uint32)
    pos_base = np.array([0, 1000], np.int32)
    ch = np.array([10, 11, 11, 12, 13, 14, 15, 0], np.uint64)   # chunk 2 repeats chunk 1; a zero fingerprint
    entry = np.array([-1, -1, -1, -1, 5, -1, -1, -1], np.int32)  # chunk 4 was a hit
    return start, length, rco, off, pos_base, ch, entry


def test_insert_if_absent_pool_closing_and_a_later_batch():
    """Duplicates inside the batch, a hash registered before, the carve-out, a chunk that
    closes the pool; then the same batch against a larger pool: the refused chunks are
    admitted now, the ones registered by the first call are not admitted twice."""
    L, n_tok = 2, 496
    start, length, rco, off, pos_base, ch, entry = hand_case()
    rng = np.random.default_rng(5)
    req_h = rng.integers(0, 65536, (L, n_tok, ROW), dtype=np.uint16)
    slots = rng.permutation(n_tok).astype(np.int32)
    pool_h = np.zeros((L, 400, ROW), np.uint16)
    gear = wl.gear_table()
    s = Session(gear, 0x3F, 8, 128, 32, L, wl.inv_freq_plain(), 1024, 4, DEV)
    try:
        reg = dict(hash=np.array([12], np.uint64), src_row=np.array([0], np.uint32), p_src=np.array([0], np.int32),
                   len=np.array([3], np.uint32), entry_id=np.array([0], np.uint32))
        s.build_table(64, reg)
        cap = 16
        pad = lambda a, dt: np.concatenate([a, np.zeros(cap - len(a), dt)])
        buf = dict(chunk_hash=s.to_dev_u64(pad(ch, np.uint64)), chunk_start=s.to_dev_u32(pad(start, np.uint32)),
                   chunk_len=s.to_dev_u32(pad(length, np.uint32)), req_chunk_offsets=s.to_dev_u32(rco),
                   n_chunks=torch.tensor([len(ch)], dtype=torch.int32, device=DEV),
                   chunk_entry=torch.from_numpy(pad(entry, np.int32)).to(DEV))
        req = torch.from_numpy(req_h.view(np.int16)).to(DEV).view(torch.bfloat16)
        pool = torch.from_numpy(pool_h.view(np.int16)).to(DEV).view(torch.bfloat16)
        d_off, d_pos, d_slots = s.to_dev_u32(off), torch.from_numpy(pos_base).to(DEV), torch.from_numpy(slots).to(DEV)
        d_cursor = torch.tensor([100], dtype=torch.int32, device=DEV)
        d_adm = torch.full((cap,), -7, dtype=torch.int32, device=DEV)
        known = reg["hash"]
        cursor = 100
        # 174 rows: one 64-row chunk fits, the 128-row chunk closes the pool; 400 rows: all the rest fits
        for pool_rows, expect in ((174, [-1, 100, -1, -1, -1, -1, -1, -1]), (400, [-1, -1, -1, -1, -1, 164, 292, 300])):
            s.admit(d_off, d_pos, d_slots, B.layer_pointers(req), ROW * 2, n_tok, B.layer_pointers(pool), ROW * 2,
                    pool_rows, d_cursor, d_adm, buf)
            torch.cuda.synchronize()
            assert s.error_flags() == 0
            visible = np.ascontiguousarray(pool_h[:, :pool_rows])
            want, new, cursor = orc.admit(known, ch, start, length, rco, off, pos_base, 32, entry, req_h, slots,
                                          visible, cursor)
            pool_h[:, :pool_rows] = visible
            assert want.tolist() == expect
            assert d_adm.cpu().numpy()[:len(ch)].tolist() == expect
            assert int(d_cursor.item()) == cursor
            assert np.array_equal(bits(pool), pool_h)
            known = np.concatenate([known, new["hash"]])
    finally:
        s.close()


def test_admit_rejects_bad_arguments_and_flags_bad_slots():
    L, n_tok = 1, 64
    s = Session(wl.gear_table(), 0x3F, 8, 128, 0, L, wl.inv_freq_plain(), 256, 2, DEV)
    try:
        s.table = B.irm_table_create(s.ctx, 16)
        cap = 4
        buf = dict(chunk_hash=s.to_dev_u64(np.array([7, 8, 0, 0], np.uint64)),
                   chunk_start=s.to_dev_u32(np.array([0, 32, 0, 0], np.uint32)),
                   chunk_len=s.to_dev_u32(np.array([32, 32, 0, 0], np.uint32)),
                   req_chunk_offsets=s.to_dev_u32(np.array([0, 2], np.uint32)),
                   n_chunks=torch.tensor([2], dtype=torch.int32, device=DEV),
                   chunk_entry=torch.full((cap,), -1, dtype=torch.int32, device=DEV))
        req = wl.kv_pool_torch(L, n_tok, 3, DEV)
        pool = wl.sentinel_pool_torch(L, 64, DEV)
        slots = np.arange(n_tok, dtype=np.int32)
        slots[40] = 64                                             # one row past the request pool
        slots[41] = -1
        d_off, d_pos = s.to_dev_u32(np.array([0, 64], np.uint32)), torch.zeros(1, dtype=torch.int32, device=DEV)
        d_cursor = torch.zeros(1, dtype=torch.int32, device=DEV)
        d_adm = torch.zeros(cap, dtype=torch.int32, device=DEV)
        args = lambda stride: (d_off, d_pos, torch.from_numpy(slots).to(DEV), B.layer_pointers(req), stride, n_tok,
                               B.layer_pointers(pool), ROW * 2, 64, d_cursor, d_adm, buf)
        with pytest.raises(B.IrmError):
            s.admit(*args(ROW * 2 - 2))                            # rows overlap: stride below a row
        with pytest.raises(B.IrmError):
            s.admit(*args(ROW * 2 + 8))                            # stride not a multiple of 16
        s.admit(*args(ROW * 2))
        torch.cuda.synchronize()
        assert s.error_flags() == B.IRM_FLAG_ROW_RANGE             # reading clears the word
        assert d_adm.cpu().numpy()[:2].tolist() == [0, 32] and int(d_cursor.item()) == 64
        got, src = bits(pool)[0], bits(req)[0]
        ok = np.ones(64, bool)
        ok[[40, 41]] = False
        assert np.array_equal(got[ok], src[ok]) and np.all(got[~ok] == wl.SENTINEL_BF16)   # bad slots are skipped
    finally:
        s.close()


def test_serve_and_admit_captured_in_a_graph_replay_over_changing_batches():
    """serve + admit recorded once; the graph is replayed on batch A, batch B, batch A again
    (tokens swapped in place between replays).  The registry must accumulate exactly as the
    oracle's does: the offer ranks that decide "first wins" live on the device."""
    wa = wl.make_workload("c2", orc.cdc_chunk, size="small", variant=0)
    wb = wl.make_workload("c2", orc.cdc_chunk, size="small", variant=1)
    assert np.array_equal(wa.req_offsets, wb.req_offsets) and np.array_equal(wa.pool_tokens, wb.pool_tokens)
    rig = Rig(wa)
    w, L = wa, wa.n_layers
    try:
        extra = len(w.tokens)
        pool_rows = w.src_rows + extra
        pool = torch.cat([rig.src, wl.sentinel_pool_torch(L, extra, DEV)], dim=1).contiguous()
        pool_ptrs = B.layer_pointers(pool)
        d_cursor = torch.tensor([w.src_rows], dtype=torch.int32, device=DEV)
        d_adm = torch.full((rig.buf["cap"],), -7, dtype=torch.int32, device=DEV)
        stream = torch.cuda.Stream(device=DEV)

        def both():
            rig.s.serve(rig.d_tokens, rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, pool_ptrs, ROW * 2,
                        pool_rows, rig.dst_ptrs, ROW * 2, w.dst_rows, rig.buf, stream)
            rig.s.admit(rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.dst_ptrs, ROW * 2, w.dst_rows,
                        pool_ptrs, ROW * 2, pool_rows, d_cursor, d_adm, rig.buf, stream)

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):                                   # recording runs nothing
            with torch.cuda.graph(graph, stream=stream):
                both()
        torch.cuda.synchronize()
        reg = dict(rig.o["reg"])
        pool_h, cursor = bits(pool), w.src_rows
        for rep, wk in enumerate((wa, wb, wa)):
            rig.d_tokens.copy_(torch.from_numpy(wk.tokens).to(DEV))
            rig.dst.copy_(wl.kv_pool_torch(L, w.dst_rows, 600 + rep, DEV))     # rows "prefilled" for the misses
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert rig.s.error_flags() == 0
            st, ln, rco = orc.cdc_chunk(wk.tokens, wk.req_offsets, wk.gear, wk.mask, wk.min_chunk, wk.max_chunk)
            ch = orc.chunk_hash(wk.tokens, st, ln)
            entry, hits, hit_tokens = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"],
                                                 ch, st, ln, rco, wk.req_offsets, wk.pos_base, wk.carve_out)
            n = len(st)
            assert int(rig.buf["n_chunks"].item()) == n
            assert np.array_equal(rig.buf["chunk_entry"].cpu().numpy()[:n], entry), rep
            assert int(rig.buf["hit_tokens"].item()) == hit_tokens
            req_h = bits(rig.dst)
            adm, new, cursor = orc.admit(reg["hash"], ch, st, ln, rco, wk.req_offsets, wk.pos_base, wk.carve_out,
                                         entry, req_h, wk.dst_slots, pool_h, cursor)
            assert np.array_equal(d_adm.cpu().numpy()[:n], adm), rep
            assert int(d_cursor.item()) == cursor
            assert np.array_equal(bits(pool), pool_h)
            reg = concat_reg(reg, new)
            if rep == 2:                                                        # batch A again: nothing left to admit
                assert np.all(adm < 0)
                pos_ok = np.concatenate([wk.pos_base[r] + st[rco[r]:rco[r + 1]].astype(np.int64)
                                         - int(wk.req_offsets[r]) for r in range(wk.n_req)]) >= wk.carve_out
                assert np.array_equal(entry >= 0, pos_ok)
            else:
                assert (adm >= 0).sum() > 0
    finally:
        rig.close()
