"""GPU parity at the full sizes of the five measured configurations, in the launch
configuration bench.py times (library defaults, contiguous slots, the four calls
chained on one stream).

Integer stages are compared bit for bit on every token and chunk.  Re-attached
rows are recomputed by the oracle: all of them for c0, c1 and c3; for c2 and c4
(tens to hundreds of GB) a seeded sample -- every layer of 256 random hits and
every layer of every hit's first and last row -- plus checks that hold at any
size and run on EVERY layer: c_KV of every re-attached row equals its source row
bit for bit, pair norms of k_r survive the rotation to bf16 rounding, and rows no
hit covers keep the sentinel.  The paper's own chunking rule (mask 0x7F, chunks of
32..512 tokens) runs the same checks at the c1 and c2 sizes.
"""
import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_util import DEV, Rig, bits, covered_rows, hits_from_dev, verify_reattach


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"
    yield
    torch.cuda.empty_cache()


def check_front(rig):
    """chunks, fingerprints, lookup: every element against the oracle"""
    o, buf = rig.o, rig.buf
    n = int(buf["n_chunks"].item())
    assert n == len(o["start"])
    u32 = lambda t: t.cpu().numpy().view(np.uint32)
    assert np.array_equal(u32(buf["chunk_start"])[:n], o["start"])
    assert np.array_equal(u32(buf["chunk_len"])[:n], o["len"])
    assert np.array_equal(u32(buf["req_chunk_offsets"]), o["rco"])
    assert np.array_equal(buf["chunk_hash"].cpu().numpy().view(np.uint64)[:n], o["hash"])
    assert np.array_equal(buf["chunk_entry"].cpu().numpy()[:n], o["entry"])
    n_hits = int(buf["n_hits"].item())
    assert n_hits == len(o["hits"]) and int(buf["hit_tokens"].item()) == o["hit_tokens"]
    g = hits_from_dev(buf["hits"], n_hits)
    for f in ("src_row", "dst_tok", "len", "delta"):
        assert np.array_equal(getattr(g, f), getattr(o["hits"], f)), f


def check_properties(rig, layers):
    """size-independent checks on whole layers, computed on the device"""
    w, hits = rig.w, rig.o["hits"]
    lens = hits.len.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(lens)])
    within = np.arange(off[-1]) - np.repeat(off[:-1], lens)
    src_idx = torch.from_numpy(np.repeat(hits.src_row.astype(np.int64), lens) + within).to(DEV)
    dst_idx = torch.from_numpy(w.dst_slots[np.repeat(hits.dst_tok.astype(np.int64), lens) + within]
                               .astype(np.int64)).to(DEV)
    untouched = torch.from_numpy(np.nonzero(~covered_rows(w, hits))[0]).to(DEV)
    step = 1 << 18
    for l in layers:
        for a in range(0, len(src_idx), step):
            s = rig.src[l].index_select(0, src_idx[a:a + step])
            d = rig.dst[l].index_select(0, dst_idx[a:a + step])
            assert torch.equal(s[:, :512].view(torch.int16), d[:, :512].view(torch.int16)), f"c_KV layer {l}"
            ns = torch.hypot(s[:, 512:544].float(), s[:, 544:].float())
            nd = torch.hypot(d[:, 512:544].float(), d[:, 544:].float())
            assert torch.all((nd - ns).abs() <= ns * 2.0 ** -7 + 1e-30), f"pair norms layer {l}"
        rest = rig.dst[l].index_select(0, untouched)
        assert torch.all(rest.view(torch.int16) == wl.SENTINEL_BF16), f"untouched rows layer {l}"


@pytest.mark.parametrize("name", ["c0", "c1", "c3"])
def test_full_size_all_rows(name):
    w = wl.make_workload(name, orc.cdc_chunk, size="full")
    rig = Rig(w)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        check_front(rig)
        hits = rig.o["hits"]
        L = w.n_layers
        total = 0
        for l0 in range(0, L, 9):                              # a few layers at a time bounds host memory
            stats = verify_reattach(w, hits, rig.src, rig.dst, layers=range(l0, min(L, l0 + 9)), what=w.name)
            total += stats["rows"]
        assert total == rig.o["hit_tokens"] * L
        check_properties(rig, range(L))
        if name == "c3":
            assert np.abs(hits.delta).max() > 90000 and np.abs(hits.delta).max() <= 100000
        if name == "c1":
            assert 0.75 < rig.o["hit_tokens"] / len(w.tokens) <= 0.80
    finally:
        rig.close()


@pytest.mark.parametrize("name", ["c2", "c4"])
def test_full_size_sampled(name):
    w = wl.make_workload(name, orc.cdc_chunk, size="full")
    rig = Rig(w)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        check_front(rig)
        hits = rig.o["hits"]
        L = w.n_layers
        rng = np.random.default_rng(4000 + wl.CONFIG_NAMES.index(name))
        sample = np.sort(rng.choice(len(hits), size=256, replace=False))
        stats = verify_reattach(w, hits, rig.src, rig.dst, hit_sel=sample, what=f"{w.name} sample")
        assert stats["rows"] == int(hits.len[sample].sum()) * L
        # first and last row of every hit, every layer (a few layers at a time)
        ends = orc.Hits(np.concatenate([hits.src_row, hits.src_row + hits.len - 1]),
                        np.concatenate([hits.dst_tok, hits.dst_tok + hits.len - 1]),
                        np.ones(2 * len(hits), np.uint32), np.concatenate([hits.delta, hits.delta]))
        for l0 in range(0, L, 16):
            verify_reattach(w, ends, rig.src, rig.dst, layers=range(l0, min(L, l0 + 16)), what=f"{w.name} ends")
        check_properties(rig, range(L))
        if name == "c4":
            assert len(rig.o["reg"]["hash"]) == 4194304 and w.table_slots == int(np.ceil(4194304 / 0.7))
        if name == "c2":
            assert np.abs(hits.delta).max() < 16384 and w.n_req == 64
    finally:
        rig.close()


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_full_size_paper_native_rule(name):
    """The paper's own CDC rule (Sec. 7.2 "CDC boundary rule", App. B: low 7 bits, chunks of 32..512
    tokens, about 2.4 times as many and as short hits) end to end at full size: front end bit for bit,
    all re-attached rows of c1 and a sample of c2 against the oracle, the size-independent checks on
    every layer."""
    w = wl.make_workload(name, orc.cdc_chunk, size="full", cdc="paper")
    assert (w.mask, w.min_chunk, w.max_chunk) == (0x7F, 32, 512)
    rig = Rig(w)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        check_front(rig)
        hits = rig.o["hits"]
        L = w.n_layers
        assert 100 < hits.len.mean() < 190 and hits.len.max() <= 512 and hits.len.min() >= 32
        if name == "c1":
            total = 0
            for l0 in range(0, L, 9):
                total += verify_reattach(w, hits, rig.src, rig.dst, layers=range(l0, min(L, l0 + 9)),
                                         what=f"{w.name} paper rule")["rows"]
            assert total == rig.o["hit_tokens"] * L
        else:
            rng = np.random.default_rng(4100)
            sample = np.sort(rng.choice(len(hits), size=256, replace=False))
            verify_reattach(w, hits, rig.src, rig.dst, hit_sel=sample, what=f"{w.name} paper rule, sample")
            ends = orc.Hits(np.concatenate([hits.src_row, hits.src_row + hits.len - 1]),
                            np.concatenate([hits.dst_tok, hits.dst_tok + hits.len - 1]),
                            np.ones(2 * len(hits), np.uint32), np.concatenate([hits.delta, hits.delta]))
            for l0 in range(0, L, 9):
                verify_reattach(w, ends, rig.src, rig.dst, layers=range(l0, min(L, l0 + 9)),
                                what=f"{w.name} paper rule, ends")
        check_properties(rig, range(L))
    finally:
        rig.close()


def test_full_size_split_pool_variant_c1():
    """irm_reattach_kr at the c1 size: every k_r row and every c_KV reference against the oracle."""
    from tests.gpu_util import ROW, compare_rows, hits_to_dev
    from paper_2605_05696_amd import binding as B
    w = wl.make_workload("c1", orc.cdc_chunk, size="full")
    rig = Rig(w)
    try:
        hits = rig.o["hits"]
        L = w.n_layers
        kr = torch.empty((L, w.dst_rows, 64), dtype=torch.bfloat16, device=DEV)
        kr.view(torch.int16).fill_(wl.SENTINEL_BF16)
        idx = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        B.irm_reattach_kr(rig.s.ctx, B.kr_slice_pointers(rig.src), ROW * 2, w.src_rows, B.kr_layer_pointers(kr), 128,
                          w.dst_rows, idx, rig.d_dst_slots, d_hits, d_n)
        assert rig.s.error_flags() == 0
        # the oracle works on the source rows the hits name, compacted
        lens = hits.len.astype(np.int64)
        off = np.concatenate([[0], np.cumsum(lens)])
        within = np.arange(off[-1]) - np.repeat(off[:-1], lens)
        src_idx = np.repeat(hits.src_row.astype(np.int64), lens) + within
        dst_idx = w.dst_slots[np.repeat(hits.dst_tok.astype(np.int64), lens) + within].astype(np.int64)
        d_src_idx = torch.from_numpy(src_idx).to(DEV)
        src_c = np.stack([bits(rig.src[l].index_select(0, d_src_idx)) for l in range(L)])
        want_kr = np.full((L, w.dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
        want_idx = np.full(w.dst_rows, -1, np.int32)
        compact = orc.Hits(off[:-1].astype(np.uint32), hits.dst_tok, hits.len, hits.delta)
        orc.reattach_kr(src_c, want_kr, want_idx, w.dst_slots, compact, w.inv_freq)
        got_idx = idx.cpu().numpy()
        touched = want_idx >= 0
        assert np.array_equal(got_idx >= 0, touched) and int(touched.sum()) == rig.o["hit_tokens"]
        # compacted index k stands for pool row src_idx[k]
        assert np.array_equal(got_idx[touched], src_idx[want_idx[touched]])
        got_kr = bits(kr)
        pad = lambda k: np.concatenate([np.zeros(k.shape[:2] + (512,), np.uint16), k], axis=2)
        compare_rows(pad(got_kr), pad(want_kr), what="c1 k_r only")
        assert np.array_equal(np.sort(dst_idx), np.nonzero(touched)[0])
    finally:
        rig.close()


@pytest.mark.parametrize("name,ranges", [("c1", 3), ("c2", 3), ("c2", 2)])
def test_full_size_admit(name, ranges):
    """irm_admit on the misses of a full-size batch.  The oracle decides who is admitted and
    where (it sees layer 0 only, and the free tail of the pool as rows 0.. of its own array);
    layer 0 of the free tail is compared with it byte for byte, every other layer on the
    device: admitted pool rows equal the request rows their tokens were prefilled into.
    ``ranges`` 2: the copy (and the serve before it) with an eighth of the whole launch's tile
    list per XCD, the mapping the library itself takes from 32 layers on."""
    from paper_2605_05696_amd import binding as B
    from tests.gpu_util import ROW
    w = wl.make_workload(name, orc.cdc_chunk, size="full")
    rig = Rig(w)
    try:
        B.irm_ctx_tune(rig.s.ctx, 3, ranges)
        o, L = rig.o, w.n_layers
        n_chunks = len(o["start"])
        miss_tokens = int(o["len"][o["entry"] < 0].sum())
        cursor0 = w.src_rows - miss_tokens + 100                   # the last eligible chunks will not fit
        gen = torch.Generator(device=DEV).manual_seed(31)
        for l in range(L):                                         # "prefilled" request pool: random bit patterns
            rig.dst[l].view(torch.int16).random_(-32768, 32767, generator=gen)
        rig.serve()
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        assert np.array_equal(rig.buf["chunk_entry"].cpu().numpy()[:n_chunks], o["entry"])
        d_cursor = torch.tensor([cursor0], dtype=torch.int32, device=DEV)
        d_adm = torch.full((rig.buf["cap"],), -7, dtype=torch.int32, device=DEV)
        rig.s.admit(rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.dst_ptrs, ROW * 2, w.dst_rows,
                    rig.src_ptrs, ROW * 2, w.src_rows, d_cursor, d_adm, rig.buf)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        req0 = bits(rig.dst[0])[None]
        tail = np.full((1, w.src_rows - cursor0, 576), wl.SENTINEL_BF16, np.uint16)
        want, new, cur = orc.admit(o["reg"]["hash"], o["hash"], o["start"], o["len"], o["rco"], w.req_offsets,
                                   w.pos_base, w.carve_out, o["entry"], req0, w.dst_slots, tail, 0)
        got = d_adm.cpu().numpy()[:n_chunks]
        assert np.array_equal(got, np.where(want >= 0, want + cursor0, -1))
        assert int(d_cursor.item()) == cur + cursor0 and cur + cursor0 <= w.src_rows
        assert (want >= 0).sum() > 0.8 * (o["entry"] < 0).sum() and (want < 0)[o["entry"] < 0].any()
        written = cur
        assert np.array_equal(bits(rig.src[0, cursor0:cursor0 + written]), tail[0, :written])
        sel = want >= 0
        lens = o["len"][sel].astype(np.int64)
        off = np.concatenate([[0], np.cumsum(lens)])
        within = np.arange(off[-1]) - np.repeat(off[:-1], lens)
        tok = np.repeat(o["start"][sel].astype(np.int64), lens) + within
        d_req_idx = torch.from_numpy(w.dst_slots[tok].astype(np.int64)).to(DEV)
        for l in range(L):
            a = rig.src[l, cursor0:cursor0 + written].view(torch.int16)
            b = rig.dst[l].index_select(0, d_req_idx).view(torch.int16)
            assert torch.equal(a, b), f"layer {l}"
    finally:
        rig.close()


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_full_size_s1_fallback(name):
    """Unaligned assembly at full size: the window list, its fingerprints and lookup bit for
    bit against the oracle; window rows recomputed by the oracle (all for c1, 256 hits for c2)."""
    from tests.gpu_util import ROW
    from tests.test_gpu_s1 import full_registry, u32
    W, anchor = 128, 1
    w = wl.make_workload(name, orc.cdc_chunk, size="full", assembly="unaligned", s1_window=W)
    reg = full_registry(w, anchor, W)
    st, ln, rco = orc.cdc_chunk(w.tokens, w.req_offsets, w.gear, w.mask, w.min_chunk, w.max_chunk)
    ch = orc.chunk_hash(w.tokens, st, ln)
    look = lambda h, s_, l_, r_: orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"],
                                            h, s_, l_, r_, w.req_offsets, w.pos_base, w.carve_out)
    entry, hits, hit_tokens = look(ch, st, ln, rco)
    rig = Rig(w, o=dict(start=st, len=ln, rco=rco, hash=ch, reg=reg, entry=entry, hits=hits, hit_tokens=hit_tokens))
    try:
        wbuf = rig.s.alloc_windows(len(w.tokens), w.n_req, W)
        rig.serve()
        rig.s.s1_serve(rig.d_tokens, rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.src_ptrs, ROW * 2,
                       w.src_rows, rig.dst_ptrs, ROW * 2, w.dst_rows, rig.buf, wbuf, anchor)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        check_front(rig)
        ws, wln, wp, rwo = orc.s1_windows(st, ln, rco, entry < 0, W, anchor)
        n = int(wbuf["n_chunks"].item())
        assert n == len(ws)
        assert np.array_equal(u32(wbuf["chunk_start"])[:n], ws) and np.array_equal(u32(wbuf["parent"])[:n], wp)
        assert np.array_equal(u32(wbuf["req_chunk_offsets"]), rwo)
        wh = orc.chunk_hash(w.tokens, ws, wln)
        assert np.array_equal(wbuf["chunk_hash"].cpu().numpy().view(np.uint64)[:n], wh)
        wentry, whits, wtok = look(wh, ws, wln, rwo)
        assert np.array_equal(wbuf["chunk_entry"].cpu().numpy()[:n], wentry)
        got = hits_from_dev(wbuf["hits"], int(wbuf["n_hits"].item()))
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(got, f), getattr(whits, f)), f
        assert wtok > 0.02 * len(w.tokens)                               # the fallback recovers a real share
        sel = None if name == "c1" else np.sort(np.random.default_rng(77).choice(len(whits), 256, replace=False))
        stats = verify_reattach(w, whits, rig.src, rig.dst, hit_sel=sel, what=f"{w.name} windows")
        assert stats["rows"] == (wtok if sel is None else 256 * W) * w.n_layers
        both = orc.Hits(np.concatenate([hits.src_row, whits.src_row]), np.concatenate([hits.dst_tok, whits.dst_tok]),
                        np.concatenate([hits.len, whits.len]), np.concatenate([hits.delta, whits.delta]))
        untouched = torch.from_numpy(np.nonzero(~covered_rows(w, both))[0]).to(DEV)
        for l in (0, w.n_layers - 1):
            assert torch.all(rig.dst[l].index_select(0, untouched).view(torch.int16) == wl.SENTINEL_BF16)
    finally:
        rig.close()


def test_full_size_attend_ref_c2():
    """The rotate-on-load consumer at the c2 size, in the launch shape bench.py times (16 heads,
    4 splits): 64 requests x 16,384 context tokens, one layer, every output against the fp64 oracle."""
    from tests.gpu_util import ROW, hits_to_dev
    from paper_2605_05696_amd import binding as B
    w = wl.make_workload("c2", orc.cdc_chunk, size="full")
    rig = Rig(w, with_table=False)
    try:
        hits = rig.o["hits"]
        pool = rig.src[0]
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        row = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        hit = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        trig = torch.zeros((rig.buf["cap"], 32, 2), dtype=torch.float32, device=DEV)
        B.irm_reattach_ref(rig.s.ctx, w.src_rows, row, hit, trig, rig.d_dst_slots, d_hits, d_n)
        row_h = row.cpu().numpy()
        fresh = np.nonzero(row_h < 0)[0]                                  # prefilled tokens: plain rows anywhere
        row_h[fresh] = np.random.default_rng(5).integers(0, w.src_rows, len(fresh))
        row.copy_(torch.from_numpy(row_h))
        hit_h = hit.cpu().numpy()
        n_req, H, splits, scale = w.n_req, 16, 4, 1.0 / np.sqrt(192.0)
        q = torch.randn((n_req, H, 576), device=DEV, generator=torch.Generator(DEV).manual_seed(3)).to(torch.bfloat16)
        out = torch.zeros((n_req, H, 512), dtype=torch.float32, device=DEV)
        lse = torch.zeros((n_req, H), dtype=torch.float32, device=DEV)
        ws = torch.empty(B.irm_attend_ref_workspace_bytes(n_req, H, splits), dtype=torch.uint8, device=DEV)
        B.irm_attend_ref(rig.s.ctx, q, pool, ROW * 2, rig.d_dst_slots, rig.d_req_offsets, row, hit, trig, scale, splits,
                         ws, out, lse)
        first = out.clone()
        for _ in range(3):                                                # same bits every time: no tile is handed
            out.zero_()                                                   # over early or late now and then
            B.irm_attend_ref(rig.s.ctx, q, pool, ROW * 2, rig.d_dst_slots, rig.d_req_offsets, row, hit, trig, scale,
                             splits, ws, out, lse)
            assert torch.equal(out, first)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        want_row = np.full(w.dst_rows, -1, np.int32)
        want_hit = np.full(w.dst_rows, -1, np.int32)
        trig64 = orc.reattach_ref(w.src_rows, want_row, want_hit, w.dst_slots, hits, w.inv_freq)
        assert np.array_equal(want_hit, hit_h)
        want, want_lse = orc.attend_ref(bits(q), bits(pool), w.dst_slots, w.req_offsets, row_h, hit_h, trig64, scale)
        err = np.abs(out.cpu().numpy() - want)
        # 16,384 tokens per softmax: the bf16 roundings average out (measured 6e-4 and 2e-4); one 64-token
        # tile lost or doubled would move the lse by 4e-3 and the outputs by about as much
        assert err.max() < 2e-3 and err.mean() < 2e-4, (err.max(), err.mean())
        assert np.abs(lse.cpu().numpy() - want_lse).max() < 6e-4
        # other splits of the same contexts (64 to 1024 workgroups in flight): the same result up to the
        # order of the partial sums, and the same bits from one call to the next
        lse4 = lse.clone()
        for other in (1, 8, 16):
            ws2 = torch.empty(B.irm_attend_ref_workspace_bytes(n_req, H, other), dtype=torch.uint8, device=DEV)
            outs = []
            for _ in range(2):
                o2 = torch.zeros_like(out)
                l2 = torch.zeros_like(lse)
                B.irm_attend_ref(rig.s.ctx, q, pool, ROW * 2, rig.d_dst_slots, rig.d_req_offsets, row, hit, trig, scale,
                                 other, ws2, o2, l2)
                outs.append((o2, l2))
            assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]), other
            assert (outs[0][0] - first).abs().max().item() < 1e-3 and (outs[0][1] - lse4).abs().max().item() < 3e-4, other
        assert rig.s.error_flags() == 0
    finally:
        rig.close()


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_full_size_fp8_rows(name):
    """656-byte rows at the benchmark's sizes and launch shape: c1 every row, c2 a sample of hits; the
    528 position-free bytes bit for bit on every re-attached row of two layers, untouched rows untouched."""
    from paper_2605_05696_amd import binding as B
    w = wl.make_workload(name, orc.cdc_chunk, size="full")
    rig = Rig(w, row_format=B.IRM_ROW_FP8)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        check_front(rig)
        hits = rig.o["hits"]
        L = w.n_layers
        if name == "c1":
            total = 0
            for l0 in range(0, L, 9):
                total += verify_reattach(w, hits, rig.src, rig.dst, layers=range(l0, min(L, l0 + 9)), what=w.name)["rows"]
            assert total == rig.o["hit_tokens"] * L
        else:
            sel = np.sort(np.random.default_rng(41).choice(len(hits), size=256, replace=False))
            stats = verify_reattach(w, hits, rig.src, rig.dst, hit_sel=sel, what=f"{w.name} sample")
            assert stats["rows"] == int(hits.len[sel].sum()) * L
        lens = hits.len.astype(np.int64)
        off = np.concatenate([[0], np.cumsum(lens)])
        within = np.arange(off[-1]) - np.repeat(off[:-1], lens)
        src_idx = torch.from_numpy(np.repeat(hits.src_row.astype(np.int64), lens) + within).to(DEV)
        dst_idx = torch.from_numpy(w.dst_slots[np.repeat(hits.dst_tok.astype(np.int64), lens) + within].astype(np.int64)).to(DEV)
        untouched = torch.from_numpy(np.nonzero(~covered_rows(w, hits))[0]).to(DEV)
        for l in (0, L - 1):
            for a in range(0, len(src_idx), 1 << 18):
                s = rig.src[l].index_select(0, src_idx[a:a + (1 << 18)])
                d = rig.dst[l].index_select(0, dst_idx[a:a + (1 << 18)])
                assert torch.equal(s[:, :264].view(torch.int16), d[:, :264].view(torch.int16)), f"layer {l}"
            assert torch.all(rig.dst[l].index_select(0, untouched).view(torch.int16) == wl.SENTINEL_BF16)
    finally:
        rig.close()


def test_full_size_attend_ref_fp8_rows_c2():
    """The rotate-on-load consumer over 656-byte rows at the c2 size and the bench's launch shape:
    c_KV dequantised while staged; every output against the fp64 oracle, same bits twice."""
    from tests.gpu_util import hits_to_dev
    from paper_2605_05696_amd import binding as B
    w = wl.make_workload("c2", orc.cdc_chunk, size="full")
    rig = Rig(w, with_table=False, with_pools=False, row_format=B.IRM_ROW_FP8)
    try:
        hits = rig.o["hits"]
        pool = wl.kv_pool_fp8_torch(1, w.src_rows, wl.kv_seed("c2"), DEV, codes="quantised")[0]
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        row = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        hit = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        trig = torch.zeros((rig.buf["cap"], 32, 2), dtype=torch.float32, device=DEV)
        B.irm_reattach_ref(rig.s.ctx, w.src_rows, row, hit, trig, rig.d_dst_slots, d_hits, d_n)
        row_h = row.cpu().numpy()
        fresh = np.nonzero(row_h < 0)[0]
        row_h[fresh] = np.random.default_rng(6).integers(0, w.src_rows, len(fresh))
        row.copy_(torch.from_numpy(row_h))
        hit_h = hit.cpu().numpy()
        n_req, H, splits, scale = w.n_req, 16, 4, 1.0 / np.sqrt(192.0)
        q = torch.randn((n_req, H, 576), device=DEV, generator=torch.Generator(DEV).manual_seed(4)).to(torch.bfloat16)
        outs = []
        for _ in range(2):
            out = torch.zeros((n_req, H, 512), dtype=torch.float32, device=DEV)
            lse = torch.zeros((n_req, H), dtype=torch.float32, device=DEV)
            ws = torch.empty(B.irm_attend_ref_workspace_bytes(n_req, H, splits), dtype=torch.uint8, device=DEV)
            B.irm_attend_ref(rig.s.ctx, q, pool, 656, rig.d_dst_slots, rig.d_req_offsets, row, hit, trig, scale, splits,
                             ws, out, lse)
            outs.append((out, lse))
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
        want_row = np.full(w.dst_rows, -1, np.int32)
        want_hit = np.full(w.dst_rows, -1, np.int32)
        trig64 = orc.reattach_ref(w.src_rows, want_row, want_hit, w.dst_slots, hits, w.inv_freq)
        want, want_lse = orc.attend_ref(bits(q), bits(pool), w.dst_slots, w.req_offsets, row_h, hit_h, trig64, scale)
        err = np.abs(outs[0][0].cpu().numpy() - want)
        lerr = np.abs(outs[0][1].cpu().numpy() - want_lse).max()
        # codes exact, scales in fp32 on the scores: the bf16 rows' bounds hold; a lost 64-token tile would
        # show (4e-3 on the lse), and so would a call that differs
        assert err.max() < 3e-3 and err.mean() < 2e-4, (err.max(), err.mean())
        assert lerr < 6e-4, lerr
    finally:
        rig.close()
