"""GPU parity of the S1 fallback (paper Sec. 4 "CDC+fallback"; App. G "S1") against the
oracle: the sub-division into fixed windows, and the windows' trip through the same
fingerprint, lookup and re-attach calls as chunks."""
import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl
from paper_2605_05696_amd.pipeline import Session

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_util import DEV, ROW, Rig, bits, covered_rows, hits_from_dev, verify_reattach


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def gpu_windows(s, starts, lens, rco, select, mode, window, anchor, cap, with_entries=None):
    d = lambda a: s.to_dev_u32(np.asarray(a, np.uint32))
    C = max(len(starts), 1)
    pad = lambda a: np.concatenate([np.asarray(a, np.uint32), np.zeros(C - len(a), np.uint32)])
    out = dict(ws=torch.full((cap,), -1, dtype=torch.int32, device=DEV), wl=torch.zeros(cap, dtype=torch.int32, device=DEV),
               wp=torch.zeros(cap, dtype=torch.int32, device=DEV), rwo=torch.zeros(len(rco), dtype=torch.int32, device=DEV),
               n=torch.zeros(1, dtype=torch.int32, device=DEV))
    d_sel = None if select is None else torch.from_numpy(
        np.concatenate([np.asarray(select, np.int32), np.zeros(C - len(select), np.int32)])).to(DEV)
    kw = {}
    if with_entries is not None:
        out["entries"] = torch.zeros((cap, 4), dtype=torch.int32, device=DEV)
        kw = dict(d_req_offsets=d(with_entries[0]), d_pos_base=torch.from_numpy(with_entries[1]).to(DEV),
                  d_win_entry=out["entries"])
    B.irm_s1_windows(s.ctx, d(pad(starts)), d(pad(lens)), d(rco), torch.tensor([len(starts)], dtype=torch.int32, device=DEV),
                     d_sel, mode, window, anchor, out["ws"], out["wl"], out["wp"], out["rwo"], out["n"], **kw)
    torch.cuda.synchronize()
    n = int(out["n"].item())
    res = dict(n=n, ws=u32(out["ws"])[:n], wl=u32(out["wl"])[:n], wp=u32(out["wp"])[:n], rwo=u32(out["rwo"]))
    if with_entries is not None:
        res["entries"] = out["entries"].cpu().numpy()[:n]
    return res


def test_subdivision_bit_exact_random_chunk_lists():
    rng = np.random.default_rng(0)
    s = Session(wl.gear_table(), 0x7, 4, 4096, 0, 1, wl.inv_freq_plain(), 1 << 16, 8, DEV)
    try:
        for trial in range(40):
            n_req = int(rng.integers(1, 8))
            W = int(rng.choice([1, 5, 32, 128]))
            starts, lens, rco, cur = [], [], [0], 0
            n_per = int(rng.choice([0, 3, 40, 700]))                        # up to several 1024-chunk rounds
            for _ in range(n_req):
                for _ in range(int(rng.integers(0, n_per + 1))):
                    l = int(rng.integers(1, 4 * W + 2))
                    starts.append(cur)
                    lens.append(l)
                    cur += l
                rco.append(len(starts))
            sel = rng.integers(-3, 4, len(starts)).astype(np.int32)
            for mode, expand in ((0, sel < 0), (1, sel >= 0), (2, np.ones(len(sel), bool))):
                for anchor in (0, 1):
                    ws, wln, wp, rwo = orc.s1_windows(np.array(starts, np.uint32), np.array(lens, np.uint32), rco,
                                                      expand, W, anchor)
                    g = gpu_windows(s, starts, lens, rco, sel, mode, W, anchor, cap=len(ws) + 3)
                    assert g["n"] == len(ws), (trial, mode, anchor)
                    assert np.array_equal(g["ws"], ws) and np.array_equal(g["wl"], wln)
                    assert np.array_equal(g["wp"], wp) and np.array_equal(g["rwo"], rwo)
            assert s.error_flags() == 0
        # capacity: the surplus is dropped and flagged, the CSR stays inside the list
        g = gpu_windows(s, [0, 100], [100, 100], [0, 2], None, 2, 10, 0, cap=13)
        assert g["n"] == 13 and g["ws"].tolist() == [10 * k for k in range(10)] + [100, 110, 120]
        assert g["rwo"].tolist() == [0, 13] and s.error_flags() == B.IRM_FLAG_CHUNK_OVERFLOW
    finally:
        s.close()


def full_registry(w, anchor, window=128):
    """pool chunks (+ fillers), then the pool chunks' windows, all by the oracle"""
    ph = orc.chunk_hash(w.pool_tokens, w.pool_chunk_start, w.pool_chunk_len)
    reg = w.registry(ph)
    ws, wln, wp, _ = orc.s1_windows(w.pool_chunk_start, w.pool_chunk_len, [0, len(ph)], np.ones(len(ph), bool),
                                    window, anchor)
    wreg = w.window_registry(ws, wln, wp, orc.chunk_hash(w.pool_tokens, ws, wln), len(reg["hash"]))
    return {k: np.concatenate([reg[k], wreg[k]]) for k in reg}


@pytest.mark.parametrize("anchor", [0, 1])
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_s1_recovers_windows_on_unaligned_batches(name, anchor):
    W = 128
    w = wl.make_workload(name, orc.cdc_chunk, size="small", assembly="unaligned", s1_window=W)
    reg = full_registry(w, anchor, W)
    st, ln, rco = orc.cdc_chunk(w.tokens, w.req_offsets, w.gear, w.mask, w.min_chunk, w.max_chunk)
    ch = orc.chunk_hash(w.tokens, st, ln)
    look = lambda h, s_, l_, r_: orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"],
                                            h, s_, l_, r_, w.req_offsets, w.pos_base, w.carve_out)
    entry, hits, hit_tokens = look(ch, st, ln, rco)
    o = dict(start=st, len=ln, rco=rco, hash=ch, reg=reg, entry=entry, hits=hits, hit_tokens=hit_tokens)
    rig = Rig(w, o=o)
    try:
        wbuf = rig.s.alloc_windows(len(w.tokens), w.n_req, W)
        rig.serve()
        rig.s.s1_serve(rig.d_tokens, rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.src_ptrs, ROW * 2,
                       w.src_rows, rig.dst_ptrs, ROW * 2, w.dst_rows, rig.buf, wbuf, anchor)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        assert np.array_equal(rig.buf["chunk_entry"].cpu().numpy()[:len(st)], entry)
        # windows, their fingerprints, their lookup: bit for bit
        ws, wln, wp, rwo = orc.s1_windows(st, ln, rco, entry < 0, W, anchor)
        n = int(wbuf["n_chunks"].item())
        assert n == len(ws) and n > 0
        assert np.array_equal(u32(wbuf["chunk_start"])[:n], ws) and np.array_equal(u32(wbuf["chunk_len"])[:n], wln)
        assert np.array_equal(u32(wbuf["parent"])[:n], wp) and np.array_equal(u32(wbuf["req_chunk_offsets"]), rwo)
        wh = orc.chunk_hash(w.tokens, ws, wln)
        assert np.array_equal(wbuf["chunk_hash"].cpu().numpy().view(np.uint64)[:n], wh)
        wentry, whits, wtok = look(wh, ws, wln, rwo)
        assert np.array_equal(wbuf["chunk_entry"].cpu().numpy()[:n], wentry)
        got = hits_from_dev(wbuf["hits"], int(wbuf["n_hits"].item()))
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(got, f), getattr(whits, f)), f
        assert int(wbuf["hit_tokens"].item()) == wtok
        if anchor == 1:
            assert wtok >= 2 * W                                            # the fallback really recovers something
        # rows: chunk hits and window hits against the oracle, everything else untouched
        verify_reattach(w, hits, rig.src, rig.dst, what=f"{w.name} chunks")
        stats = verify_reattach(w, whits, rig.src, rig.dst, what=f"{w.name} windows")
        assert stats["rows"] == wtok * w.n_layers
        both = orc.Hits(np.concatenate([hits.src_row, whits.src_row]), np.concatenate([hits.dst_tok, whits.dst_tok]),
                        np.concatenate([hits.len, whits.len]), np.concatenate([hits.delta, whits.delta]))
        untouched = ~covered_rows(w, both)
        rest = bits(rig.dst[:, torch.from_numpy(np.nonzero(untouched)[0]).to(DEV), :])
        assert np.all(rest == wl.SENTINEL_BF16)
    finally:
        rig.close()


def test_s1_register_after_admit_then_a_shifted_request_finds_the_windows():
    """Serve a batch against an empty registry, admit all of it, register the windows of what
    was admitted; the same text behind a different, unaligned preamble then loses its first
    chunk to drift and gets its windows back (end anchor)."""
    W, L, anchor = 128, 2, 1
    rng = np.random.default_rng(9)
    gear, mask, lo, hi, carve = wl.gear_table(), 0xFF, 64, 1024, 32
    body = rng.integers(0, 102400, 6000).astype(np.int32)
    first = np.concatenate([rng.integers(0, 102400, 300).astype(np.int32), body])
    second = np.concatenate([rng.integers(0, 102400, 517).astype(np.int32), body])
    pool_rows = 8192
    s = Session(gear, mask, lo, hi, carve, L, wl.inv_freq_plain(), 8192, 1, DEV)
    try:
        s.table = B.irm_table_create(s.ctx, 1024)
        pool = wl.sentinel_pool_torch(L, pool_rows, DEV)
        pool_ptrs = B.layer_pointers(pool)
        d_cursor = torch.zeros(1, dtype=torch.int32, device=DEV)
        reg = {k: np.zeros(0, t) for k, t in (("hash", np.uint64), ("src_row", np.uint32), ("p_src", np.int32),
                                              ("len", np.uint32), ("entry_id", np.uint32))}
        pool_h = bits(pool)
        cursor = 0
        for step, toks in enumerate((first, second)):
            n = len(toks)
            off = np.array([0, n], np.uint32)
            pos_base = np.array([40], np.int32)
            slots = rng.permutation(n).astype(np.int32)
            d_tok, d_off = torch.from_numpy(toks).to(DEV), s.to_dev_u32(off)
            d_pos, d_slots = torch.from_numpy(pos_base).to(DEV), torch.from_numpy(slots).to(DEV)
            buf, wbuf = s.alloc_front(n, 1), s.alloc_windows(n, 1, W)
            req = wl.kv_pool_torch(L, n, 500 + step, DEV)                    # "prefilled" rows of this request
            req_ptrs = B.layer_pointers(req)
            s.serve(d_tok, d_off, d_pos, d_slots, pool_ptrs, ROW * 2, pool_rows, req_ptrs, ROW * 2, n, buf)
            s.s1_serve(d_tok, d_off, d_pos, d_slots, pool_ptrs, ROW * 2, pool_rows, req_ptrs, ROW * 2, n, buf, wbuf,
                       anchor)
            torch.cuda.synchronize()
            assert s.error_flags() == 0
            # the oracle's view of the same step
            st, ln, rco = orc.cdc_chunk(toks, off, gear, mask, lo, hi)
            ch = orc.chunk_hash(toks, st, ln)
            look = lambda h, s_, l_, r_: orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"],
                                                    reg["entry_id"], h, s_, l_, r_, off, pos_base, carve)
            entry, hits, _ = look(ch, st, ln, rco)
            ws, wln, wp, rwo = orc.s1_windows(st, ln, rco, entry < 0, W, anchor)
            wentry, whits, wtok = look(orc.chunk_hash(toks, ws, wln), ws, wln, rwo)
            assert np.array_equal(buf["chunk_entry"].cpu().numpy()[:len(st)], entry)
            got = hits_from_dev(wbuf["hits"], int(wbuf["n_hits"].item()))
            for f in ("src_row", "dst_tok", "len", "delta"):
                assert np.array_equal(getattr(got, f), getattr(whits, f)), (step, f)
            if step == 0:
                assert len(hits) == 0 and wtok == 0
            else:
                # the drifted first chunk of the shared body is lost, its windows come back, delta = 517 - 300
                assert len(hits) > 0 and wtok >= 2 * W and np.all(whits.delta == 217) and np.all(hits.delta == 217)

                class Wd:
                    dst_slots, inv_freq = slots, wl.inv_freq_plain()
                verify_reattach(Wd, whits, pool, req, what="window hits")
            # admit what missed, then register the windows of what was admitted
            req_h = bits(req)
            d_adm = torch.full((buf["cap"],), -7, dtype=torch.int32, device=DEV)
            s.admit(d_off, d_pos, d_slots, req_ptrs, ROW * 2, n, pool_ptrs, ROW * 2, pool_rows, d_cursor, d_adm, buf)
            s.s1_register(d_tok, d_off, d_pos, d_adm, buf, wbuf, anchor)
            torch.cuda.synchronize()
            assert s.error_flags() == 0
            # window hits are not chunk hits: chunk_entry still says miss for their parents, so
            # the oracle admits the same chunks
            adm, new, cursor = orc.admit(reg["hash"], ch, st, ln, rco, off, pos_base, carve, entry, req_h, slots,
                                         pool_h, cursor)
            assert np.array_equal(d_adm.cpu().numpy()[:len(st)], adm) and int(d_cursor.item()) == cursor
            assert np.array_equal(bits(pool), pool_h)
            aws, awl, awp, _ = orc.s1_windows(st, ln, rco, adm >= 0, W, anchor)
            nw = int(wbuf["n_chunks"].item())
            assert nw == len(aws) and np.array_equal(u32(wbuf["chunk_start"])[:nw], aws)
            ent = wbuf["entries"].cpu().numpy()[:nw]
            want_row = adm[awp].astype(np.int64) + (aws.astype(np.int64) - st[awp].astype(np.int64))
            want_pos = pos_base[0] + aws.astype(np.int64)
            assert np.array_equal(ent[:, 0].view(np.uint32), want_row) and np.array_equal(ent[:, 1], want_pos)
            assert np.all(ent[:, 2] == W) and np.array_equal(ent[:, 3].view(np.uint32), want_row)
            wreg = dict(hash=orc.chunk_hash(toks, aws, awl), src_row=want_row.astype(np.uint32),
                        p_src=want_pos.astype(np.int32), len=awl, entry_id=want_row.astype(np.uint32))
            reg = {k: np.concatenate([reg[k], new[k], wreg[k]]) for k in reg}
    finally:
        s.close()
