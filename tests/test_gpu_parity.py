"""GPU parity: every stage of the HIP path against the CPU oracle, through the C ABI.

Integer stages (chunk boundaries, fingerprints, lookup results, c_KV bytes) are
compared bit for bit; rotated k_r within 2 bf16 steps of the oracle's
fp64-rounded value or 1e-2 absolute.
"""
import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl
from paper_2605_05696_amd.pipeline import Session

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_util import (DEV, ROW, Rig, bits, compare_rows, covered_rows, hits_from_dev,
                                hits_to_dev, oracle_front, verify_reattach)


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


def small(name, **kw):
    return wl.make_workload(name, orc.cdc_chunk, size="small", **kw)


# ------------------------------------------------------------ chunk + hash --

def gpu_chunks(tokens, req_offsets, gear, mask, lo, hi, serial=False):
    n_req = len(req_offsets) - 1
    s = Session(gear, mask, lo, hi, 32, 1, wl.inv_freq_plain(), max(len(tokens), 1), max(n_req, 1), DEV)
    try:
        B.irm_ctx_tune(s.ctx, 5, 1 if serial else 0)
        out = s.chunk_host(tokens, req_offsets)
        assert s.error_flags() == 0
    finally:
        s.close()
    return out


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_cdc_and_hash_bit_exact_small_configs(name):
    w = small(name)
    for tokens, off in ((w.tokens, w.req_offsets), (w.pool_tokens, np.array([0, len(w.pool_tokens)], np.uint32))):
        st, ln, rco, ch = gpu_chunks(tokens, off, w.gear, w.mask, w.min_chunk, w.max_chunk)
        o_st, o_ln, o_rco = orc.cdc_chunk(tokens, off, w.gear, w.mask, w.min_chunk, w.max_chunk)
        assert np.array_equal(st, o_st) and np.array_equal(ln, o_ln) and np.array_equal(rco, o_rco)
        assert np.array_equal(ch, orc.chunk_hash(tokens, o_st, o_ln))


@pytest.mark.parametrize("serial", [False, True])
def test_cdc_ragged_requests_and_edge_lengths(serial):
    """Both cut-selection paths (pointer doubling over candidates, serial bitmap walk)."""
    rng = np.random.default_rng(17)
    gear = wl.gear_table()
    lens = [1, 0, 63, 64, 65, 127, 128, 1023, 1024, 1025, 2048, 0, 5000, 7, 300000, 1, 1300000, 3]
    tokens = rng.integers(0, 102400, size=sum(lens)).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    st, ln, rco, ch = gpu_chunks(tokens, off, gear, 0xFF, 64, 1024, serial=serial)
    o_st, o_ln, o_rco = orc.cdc_chunk(tokens, off, gear, 0xFF, 64, 1024)
    assert np.array_equal(rco, o_rco) and np.array_equal(st, o_st) and np.array_equal(ln, o_ln)
    assert np.array_equal(ch, orc.chunk_hash(tokens, o_st, o_ln))


@pytest.mark.parametrize("mask,lo,hi", [(0x7F, 32, 512), (0x1, 1, 3), (0xFFFF, 16, 100), (0x0, 4, 9),
                                        (0xF, 4, 4), (0xFFFFF, 64, 65536), (0xFF, 64, 1024),
                                        (0xFFFFFFFF, 32, 40), (0xFF, 128, 128), (0x1, 1, 1)])   # last two: fixed blocks
@pytest.mark.parametrize("serial", [False, True])
def test_cdc_other_masks_and_clamps(mask, lo, hi, serial):
    rng = np.random.default_rng(mask % 1000 + lo)
    gear = wl.gear_table(seed=99)
    n = 200000 if hi > 1024 else 30000
    tokens = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
    off = np.array([0, 11, n // 3, n], np.uint32)
    st, ln, rco, ch = gpu_chunks(tokens, off, gear, mask, lo, hi, serial=serial)
    o_st, o_ln, o_rco = orc.cdc_chunk(tokens, off, gear, mask, lo, hi)
    assert np.array_equal(rco, o_rco) and np.array_equal(st, o_st) and np.array_equal(ln, o_ln)
    assert np.array_equal(ch, orc.chunk_hash(tokens, o_st, o_ln))


def test_cdc_degenerate_streams():
    gear = wl.gear_table()
    same = np.full(5000, 7, np.int32)                    # constant stream: all or no candidates
    for tokens in (same, np.arange(5000, dtype=np.int32) % 3):
        off = np.array([0, len(tokens)], np.uint32)
        st, ln, _, ch = gpu_chunks(tokens, off, gear, 0xFF, 64, 1024)
        o_st, o_ln, _ = orc.cdc_chunk(tokens, off, gear, 0xFF, 64, 1024)
        assert np.array_equal(st, o_st) and np.array_equal(ln, o_ln)
        assert np.array_equal(ch, orc.chunk_hash(tokens, o_st, o_ln))


# ------------------------------------------------------------------ lookup --

@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_lookup_bit_exact_small_configs(name):
    w = small(name)
    rig = Rig(w, with_pools=False)
    try:
        o, buf = rig.o, rig.buf
        rig.s.chunk_and_hash(rig.d_tokens, rig.d_req_offsets, buf)
        B.irm_lookup(rig.s.ctx, rig.s.table, buf["chunk_hash"], buf["chunk_start"], buf["chunk_len"],
                     buf["req_chunk_offsets"], rig.d_req_offsets, rig.d_pos_base, buf["n_chunks"],
                     buf["chunk_entry"], buf["hits"], buf["n_hits"], buf["hit_tokens"])
        assert rig.s.error_flags() == 0
        n = int(buf["n_chunks"].item())
        assert n == len(o["start"])
        assert np.array_equal(buf["chunk_entry"].cpu().numpy()[:n], o["entry"])
        n_hits = int(buf["n_hits"].item())
        assert n_hits == len(o["hits"]) and int(buf["hit_tokens"].item()) == o["hit_tokens"]
        g = hits_from_dev(buf["hits"], n_hits)
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(g, f), getattr(o["hits"], f)), f
    finally:
        rig.close()


def test_table_first_wins_batches_zero_key_and_length_guard():
    rng = np.random.default_rng(3)
    n_reg, n_chunks = 5000, 3000
    keys = rng.integers(0, 1500, size=n_reg, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)  # key 0 included
    reg = dict(hash=keys, src_row=rng.integers(0, 10**6, n_reg).astype(np.uint32),
               p_src=rng.integers(0, 5000, n_reg).astype(np.int32),
               len=rng.integers(64, 67, n_reg).astype(np.uint32),
               entry_id=np.arange(n_reg, dtype=np.uint32))
    length = rng.integers(64, 67, n_chunks).astype(np.uint32)
    start = np.concatenate([[0], np.cumsum(length)[:-1]]).astype(np.uint32)
    rco = np.array([0, 1000, 1000, n_chunks], np.uint32)            # an empty request in the middle
    off = np.array([0, start[1000], start[1000], int(length.sum())], np.uint32)
    ch = rng.integers(0, 1600, size=n_chunks, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    pos_base = np.array([0, 5, 40], np.int32)
    o_entry, o_hits, o_tok = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"],
                                        reg["entry_id"], ch, start, length, rco, off, pos_base, 32)
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, 1, wl.inv_freq_plain(), int(length.sum()), 3, DEV)
    try:
        s.build_table(int(n_reg / 0.7), reg, batch=1234)             # several insert batches
        cap = n_chunks
        i32, i64 = torch.int32, torch.int64
        d = lambda a: s.to_dev_u32(a)
        entry = torch.full((cap,), -7, dtype=i32, device=DEV)
        hits = torch.zeros((cap, 4), dtype=i32, device=DEV)
        n_hits = torch.zeros(1, dtype=i32, device=DEV)
        tok = torch.zeros(1, dtype=i64, device=DEV)
        B.irm_lookup(s.ctx, s.table, s.to_dev_u64(ch), d(start), d(length), d(rco), d(off),
                     torch.from_numpy(pos_base).to(DEV), torch.tensor([n_chunks], dtype=i32, device=DEV),
                     entry, hits, n_hits, tok)
        assert s.error_flags() == 0
        assert np.array_equal(entry.cpu().numpy(), o_entry)
        g = hits_from_dev(hits, int(n_hits.item()))
        assert int(n_hits.item()) == len(o_hits) and int(tok.item()) == o_tok
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(g, f), getattr(o_hits, f)), f
        assert (o_entry >= 0).sum() > 100 and (o_entry < 0).sum() > 100
    finally:
        s.close()


def test_table_full_is_reported_not_fatal():
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, 1, wl.inv_freq_plain(), 1024, 1, DEV)
    try:
        n = 64
        reg = dict(hash=np.arange(1, n + 1, dtype=np.uint64), src_row=np.zeros(n, np.uint32),
                   p_src=np.zeros(n, np.int32), len=np.full(n, 64, np.uint32),
                   entry_id=np.arange(n, dtype=np.uint32))
        s.build_table(16, reg)
        assert s.error_flags() & B.IRM_FLAG_TABLE_FULL
        assert s.error_flags() == 0                                  # reading clears
    finally:
        s.close()


# ---------------------------------------------------------------- reattach --

@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
@pytest.mark.parametrize("slots", ["contiguous", "permuted"])
def test_reattach_small_configs_all_rows(name, slots):
    """Driven by the ORACLE's hit list, so this stage is tested on its own."""
    w = small(name, slots=slots)
    rig = Rig(w, with_table=False)
    try:
        hits = rig.o["hits"]
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        rig.reattach(d_hits, d_n)
        assert rig.s.error_flags() == 0
        stats = verify_reattach(w, hits, rig.src, rig.dst, what=w.name)
        assert stats["rows"] == rig.o["hit_tokens"] * w.n_layers
        assert stats["exact"] > 0.95                                 # nearly all k_r values match exactly
        # rows no hit covers still hold the sentinel
        untouched = ~covered_rows(w, hits)
        rest = bits(rig.dst[:, torch.from_numpy(np.nonzero(untouched)[0]).to(DEV), :])
        assert np.all(rest == wl.SENTINEL_BF16)
        # bit-for-bit repeatable
        first = rig.dst.clone()
        rig.reattach(d_hits, d_n)
        torch.cuda.synchronize()
        assert torch.equal(first.view(torch.int16), rig.dst.view(torch.int16))
    finally:
        rig.close()


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_end_to_end_small_configs(name):
    """The four calls chained on one stream with device-side counts."""
    w = small(name)
    rig = Rig(w)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        o = rig.o
        n_hits = int(rig.buf["n_hits"].item())
        g = hits_from_dev(rig.buf["hits"], n_hits)
        assert n_hits == len(o["hits"]) and np.array_equal(g.delta, o["hits"].delta)
        assert np.array_equal(g.src_row, o["hits"].src_row) and np.array_equal(g.dst_tok, o["hits"].dst_tok)
        verify_reattach(w, o["hits"], rig.src, rig.dst, what=w.name)
    finally:
        rig.close()


def test_reattach_special_deltas_and_tile_tails():
    """delta = 0 must reproduce the row bit for bit; hit lengths around the 64-row
    tile size; extreme |delta|; strided pools."""
    rng = np.random.default_rng(5)
    L, src_rows, dst_rows = 2, 3000, 2600
    lens = np.array([1, 63, 64, 65, 128, 129, 1024, 7], np.uint32)
    src_row = np.array([0, 10, 100, 200, 300, 500, 700, 2900], np.uint32)
    dst_tok = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint32)
    delta = np.array([0, 1, -1, 131071, -131072, 2**31 - 1, -2**31, 0], np.int32)
    hits = orc.Hits(src_row, dst_tok, lens, delta)
    n_tok = int(lens.sum())
    inv = wl.inv_freq_yarn()
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, L, inv, 4096, 1, DEV)
    try:
        stride_elems = ROW + 64                                       # padded rows: stride 1280 B
        src_full = torch.randn((L, src_rows, stride_elems), device=DEV).to(torch.bfloat16)
        dst_full = torch.empty((L, dst_rows, stride_elems), dtype=torch.bfloat16, device=DEV)
        dst_full.view(torch.int16).fill_(wl.SENTINEL_BF16)
        src, dst = src_full[:, :, :ROW], dst_full[:, :, :ROW]
        slots = rng.permutation(dst_rows)[:n_tok].astype(np.int32)
        d_hits, d_n = hits_to_dev(hits, 16)
        B.irm_reattach(s.ctx, B.layer_pointers(src), stride_elems * 2, src_rows, B.layer_pointers(dst),
                       stride_elems * 2, dst_rows, torch.from_numpy(slots).to(DEV), d_hits, d_n)
        assert s.error_flags() == 0

        class W:                                                      # what verify_reattach reads
            dst_slots, inv_freq = slots, inv
        stats = verify_reattach(W, hits, src, dst, what="special")
        assert stats["rows"] == n_tok * L
        # delta == 0 hits are exact copies of whole rows
        for h in (0, 7):
            for j in range(int(lens[h])):
                a = bits(src[:, int(src_row[h]) + j]), bits(dst[:, int(slots[int(dst_tok[h]) + j])])
                assert np.array_equal(a[0], a[1])
        # padding columns and unlisted rows untouched
        assert torch.all(dst_full[:, :, ROW:].view(torch.int16) == wl.SENTINEL_BF16)
        mask = torch.ones(dst_rows, dtype=torch.bool, device=DEV)
        mask[torch.from_numpy(slots.astype(np.int64)).to(DEV)] = False
        assert torch.all(dst[:, mask].contiguous().view(torch.int16) == wl.SENTINEL_BF16)
    finally:
        s.close()


@pytest.mark.parametrize("waves,rpw,grid,ranges", [(8, 2, 0, 2), (8, 2, 8, 2), (8, 2, 64, 2), (8, 4, 0, 2), (4, 4, 16, 2),
                                                   (16, 2, 0, 2), (4, 8, 24, 2), (16, 4, 8, 2), (8, 2, 0, 0), (8, 2, 0, 1),
                                                   (8, 2, 8, 1), (8, 2, 64, 1), (16, 4, 8, 0)])
@pytest.mark.parametrize("name,slots", [("c2", "permuted"), ("c4", "contiguous")])
def test_reattach_launch_shapes(name, slots, waves, rpw, grid, ranges):
    """Every launch shape of the row kernel writes the same rows: tile shapes, grids smaller than
    the tile count, where a workgroup walks several tiles, and every mapping of workgroups to tiles
    (2: an eighth of the whole launch per XCD, the default; 1: an eighth of every layer; 0: tile x).
    All rows against the oracle; rows no hit covers keep the sentinel."""
    w = small(name, slots=slots)
    rig = Rig(w)
    try:
        for knob, value in ((4, 16), (1, rpw), (4, waves), (0, grid), (3, ranges)):
            B.irm_ctx_tune(rig.s.ctx, knob, value)
        hits = rig.o["hits"]
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        for _ in range(2):
            rig.dst.view(torch.int16).fill_(wl.SENTINEL_BF16 - 0x10000 if wl.SENTINEL_BF16 >= 0x8000 else wl.SENTINEL_BF16)
            rig.reattach(d_hits, d_n)
            assert rig.s.error_flags() == 0
            stats = verify_reattach(w, hits, rig.src, rig.dst, what=f"{w.name} {waves}x{rpw} g{grid}")
            assert stats["rows"] == rig.o["hit_tokens"] * w.n_layers
            untouched = ~covered_rows(w, hits)
            assert np.all(bits(rig.dst)[:, untouched] == wl.SENTINEL_BF16)
    finally:
        rig.close()


def test_reattach_no_hits_and_bad_indices_are_skipped_and_flagged():
    L, rows = 1, 256
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, L, wl.inv_freq_plain(), 1024, 1, DEV)
    try:
        src = wl.kv_pool_torch(L, rows, 1, DEV)
        dst = wl.sentinel_pool_torch(L, rows, DEV)
        slots = np.arange(rows, dtype=np.int32)
        slots[5] = rows + 3                                           # outside the pool
        slots[6] = -1
        d_slots = torch.from_numpy(slots).to(DEV)
        sp, dp = B.layer_pointers(src), B.layer_pointers(dst)
        # no hits: nothing written
        d_hits, d_n = hits_to_dev(orc.Hits(*(np.zeros(0, t) for t in (np.uint32, np.uint32, np.uint32, np.int32))), 8)
        B.irm_reattach(s.ctx, sp, ROW * 2, rows, dp, ROW * 2, rows, d_slots, d_hits, d_n)
        assert s.error_flags() == 0
        assert torch.all(dst.view(torch.int16) == wl.SENTINEL_BF16)
        # hit 0 touches the two bad slots, hit 1 reads past the source pool, hit 2 is fine
        hits = orc.Hits(np.array([0, 250, 100], np.uint32), np.array([0, 64, 128], np.uint32),
                        np.array([10, 10, 10], np.uint32), np.array([3, 3, 3], np.int32))
        d_hits, d_n = hits_to_dev(hits, 8)
        B.irm_reattach(s.ctx, sp, ROW * 2, rows, dp, ROW * 2, rows, d_slots, d_hits, d_n)
        assert s.error_flags() & B.IRM_FLAG_ROW_RANGE
        got = bits(dst)
        written = np.any(got != wl.SENTINEL_BF16, axis=2)[0]
        want = np.zeros(rows, bool)
        want[[0, 1, 2, 3, 4, 7, 8, 9]] = True                         # hit 0 minus slots 5, 6
        want[128:138] = True                                          # hit 2
        assert np.array_equal(written, want)
    finally:
        s.close()


def test_more_hits_than_the_list_holds_are_dropped_and_flagged():
    """A hit count above the list's capacity (a caller's mistake, or a count another call left there):
    the hits the list holds are re-attached, the flag says that some were dropped."""
    L, rows = 2, 512
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, L, wl.inv_freq_plain(), 1024, 1, DEV)
    try:
        src = wl.kv_pool_torch(L, rows, 3, DEV)
        dst = wl.sentinel_pool_torch(L, rows, DEV)
        d_slots = torch.arange(rows, dtype=torch.int32, device=DEV)
        hits = orc.Hits(np.array([0, 100, 200], np.uint32), np.array([300, 0, 100], np.uint32),
                        np.array([40, 70, 17], np.uint32), np.array([5, -9, 0], np.int32))
        d_hits, d_n = hits_to_dev(hits, 3)
        d_n.fill_(7)                                                  # the list has room for three
        B.irm_reattach(s.ctx, B.layer_pointers(src), ROW * 2, rows, B.layer_pointers(dst), ROW * 2, rows, d_slots,
                       d_hits, d_n)
        assert s.error_flags() == B.IRM_FLAG_CHUNK_OVERFLOW
        want = np.full((L, rows, ROW), wl.SENTINEL_BF16, np.uint16)
        orc.reattach(bits(src), want, np.arange(rows, dtype=np.int32), hits, wl.inv_freq_plain())
        compare_rows(bits(dst), want, what="three of seven")
    finally:
        s.close()


def test_chunk_records_outside_the_tokens_are_skipped_and_flagged():
    """irm_chunk_hash: a record that runs past the token array gets fingerprint 0 and raises the flag, the
    others are fingerprinted as usual.  irm_cdc_chunk: a request whose offsets run backwards or past the
    token array yields no chunks and raises the flag, the request in front of it is chunked as usual."""
    rng = np.random.default_rng(11)
    tokens = rng.integers(0, 102400, 3000).astype(np.int32)
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, 1, wl.inv_freq_plain(), 4096, 2, DEV)
    try:
        d_tok = torch.from_numpy(tokens).to(DEV)
        start = np.array([0, 500, 2900, 1000], np.uint32)
        length = np.array([500, 300, 101, 64], np.uint32)             # record 2 ends one token past the array
        d_hash = torch.full((4,), -1, dtype=torch.int64, device=DEV)
        B.irm_chunk_hash(s.ctx, d_tok, s.to_dev_u32(start), s.to_dev_u32(length),
                         torch.tensor([4], dtype=torch.int32, device=DEV), d_hash)
        assert s.error_flags() == B.IRM_FLAG_BAD_CHUNK
        got = d_hash.cpu().numpy().view(np.uint64)
        ok = [0, 1, 3]
        assert np.array_equal(got[ok], orc.chunk_hash(tokens, start[ok], length[ok])) and got[2] == 0
        # chunking: the second request claims tokens the array does not have
        for off in ([0, 1700, 3001], [2000, 1000]):
            off = np.array(off, np.uint32)
            buf = s.alloc_front(len(tokens), len(off) - 1)
            B.irm_cdc_chunk(s.ctx, d_tok, s.to_dev_u32(off), buf["chunk_start"], buf["chunk_len"],
                            buf["req_chunk_offsets"], buf["n_chunks"])
            assert s.error_flags() == B.IRM_FLAG_BAD_CHUNK
            n = int(buf["n_chunks"].item())
            rco = buf["req_chunk_offsets"].cpu().numpy().view(np.uint32)
            if len(off) == 3:
                st, ln, _ = orc.cdc_chunk(tokens[:1700], [0, 1700], wl.gear_table(), 0xFF, 64, 1024)
                assert n == len(st) and list(rco) == [0, n, n]
                assert np.array_equal(buf["chunk_start"].cpu().numpy().view(np.uint32)[:n], st)
                assert np.array_equal(buf["chunk_len"].cpu().numpy().view(np.uint32)[:n], ln)
            else:
                assert n == 0 and list(rco) == [0, 0]
    finally:
        s.close()


# ------------------------------------------------- split pool (k_r only) --

def run_kr_variant(w, hits, src, dense=False, pair_mode=0, knobs=()):
    """irm_reattach_kr on a workload; returns (kr bits [L][rows][64], ckv_index).
    ``dense``: the source k_r comes from a separate [L][rows][64] k_r_base pool."""
    L = w.n_layers
    s = Session.for_workload(w, DEV, pair_mode=pair_mode)
    try:
        for knob, value in knobs:
            B.irm_ctx_tune(s.ctx, knob, value)
        kr = torch.empty((L, w.dst_rows, 64), dtype=torch.bfloat16, device=DEV)
        kr.view(torch.int16).fill_(wl.SENTINEL_BF16)
        idx = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        cap = max(len(hits), 1) + 3
        d_hits, d_n = hits_to_dev(hits, cap)
        if dense:
            base = src[:, :, 512:].contiguous()
            sp, stride = B.kr_layer_pointers(base), 128
        else:
            sp, stride = B.kr_slice_pointers(src), ROW * 2
        B.irm_reattach_kr(s.ctx, sp, stride, w.src_rows, B.kr_layer_pointers(kr), 128,
                          w.dst_rows, idx, torch.from_numpy(w.dst_slots).to(DEV), d_hits, d_n)
        assert s.error_flags() == 0
        return bits(kr), idx.cpu().numpy()
    finally:
        s.close()


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
@pytest.mark.parametrize("slots,dense", [("contiguous", False), ("permuted", False), ("contiguous", True)])
def test_reattach_kr_small_configs(name, slots, dense):
    w = small(name, slots=slots)
    o = oracle_front(w)
    hits = o["hits"]
    src = wl.kv_pool_torch(w.n_layers, w.src_rows, wl.kv_seed(name), DEV)
    got_kr, got_idx = run_kr_variant(w, hits, src, dense=dense)
    want_kr = np.full((w.n_layers, w.dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
    want_idx = np.full(w.dst_rows, -1, np.int32)
    orc.reattach_kr(bits(src), want_kr, want_idx, w.dst_slots, hits, w.inv_freq)
    assert np.array_equal(got_idx, want_idx)                          # references: bit-exact
    pad = lambda k: np.concatenate([np.zeros(k.shape[:2] + (512,), np.uint16), k], axis=2)
    compare_rows(pad(got_kr), pad(want_kr), what=f"{w.name} k_r only")
    untouched = want_idx < 0
    assert np.all(got_kr[:, untouched] == wl.SENTINEL_BF16)


@pytest.mark.parametrize("rows_per_lane,layers_per_wg,ranges", [(2, 1, 3), (2, 2, 3), (4, 3, 3), (8, 1, 3), (2, 0, 3),
                                                                (4, 5, 3), (2, 1, 2), (2, 2, 2), (4, 0, 2), (2, 2, 0)])
@pytest.mark.parametrize("name,slots,pair_mode", [("c4", "permuted", 0), ("c1", "contiguous", 1)])
def test_reattach_kr_launch_shapes(name, slots, pair_mode, rows_per_lane, layers_per_wg, ranges):
    """Rows per lane, layers a workgroup keeps its tile for (c1 and c4 have three layers: one, two
    with a remainder, all, more than there are) and which XCD serves which (tile, layer group)
    (3: the library's choice, 2: an eighth of the whole launch, 0: round-robin): same rows."""
    w = small(name, slots=slots)
    hits = oracle_front(w)["hits"]
    src = wl.kv_pool_torch(w.n_layers, w.src_rows, wl.kv_seed(name), DEV)
    got_kr, got_idx = run_kr_variant(w, hits, src, pair_mode=pair_mode,
                                     knobs=((6, rows_per_lane), (7, layers_per_wg), (3, ranges)))
    want_kr = np.full((w.n_layers, w.dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
    want_idx = np.full(w.dst_rows, -1, np.int32)
    orc.reattach_kr(bits(src), want_kr, want_idx, w.dst_slots, hits, w.inv_freq, pair_mode)
    assert np.array_equal(got_idx, want_idx)
    pad = lambda k: np.concatenate([np.zeros(k.shape[:2] + (512,), np.uint16), k], axis=2)
    compare_rows(pad(got_kr), pad(want_kr), what=f"{w.name} k_r only, shape {rows_per_lane}/{layers_per_wg}")
    assert np.all(got_kr[:, want_idx < 0] == wl.SENTINEL_BF16)


# ------------------------------------------------ interleaved rotary pairs --

@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
@pytest.mark.parametrize("slots", ["contiguous", "permuted"])
def test_interleaved_pairs_small_configs(name, slots):
    """pair i = elements (2i, 2i+1) of k_r: the whole path, then the k_r-only variant."""
    w = small(name, slots=slots)
    rig = Rig(w, pair_mode=1)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        hits = rig.o["hits"]
        stats = verify_reattach(w, hits, rig.src, rig.dst, what=f"{w.name} interleaved", pair_mode=1)
        assert stats["rows"] == rig.o["hit_tokens"] * w.n_layers and stats["exact"] > 0.95
        # the half-split answer is a different one: the switch really switched
        half = np.full((1, w.dst_rows, 576), wl.SENTINEL_BF16, np.uint16)
        one = orc.Hits(hits.src_row[:1], hits.dst_tok[:1], hits.len[:1], hits.delta[:1])
        orc.reattach(bits(rig.src[:1]), half, w.dst_slots, one, w.inv_freq, 0)
        rows = w.dst_slots[int(one.dst_tok[0]):int(one.dst_tok[0]) + int(one.len[0])]
        assert one.delta[0] != 0 and not np.array_equal(half[0, rows], bits(rig.dst[0])[rows])
        got_kr, got_idx = run_kr_variant(w, hits, rig.src, pair_mode=1)
        want_kr = np.full((w.n_layers, w.dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
        want_idx = np.full(w.dst_rows, -1, np.int32)
        orc.reattach_kr(bits(rig.src), want_kr, want_idx, w.dst_slots, hits, w.inv_freq, 1)
        assert np.array_equal(got_idx, want_idx)
        pad = lambda k: np.concatenate([np.zeros(k.shape[:2] + (512,), np.uint16), k], axis=2)
        compare_rows(pad(got_kr), pad(want_kr), what=f"{w.name} interleaved k_r only")
    finally:
        rig.close()


def test_interleaved_pairs_special_deltas():
    """delta = 0 stays the exact identity; tile tails; extreme |delta| (YaRN frequencies)."""
    rng = np.random.default_rng(6)
    L, src_rows, dst_rows = 2, 1500, 1400
    lens = np.array([1, 15, 16, 17, 33, 1024, 7], np.uint32)
    src_row = np.array([0, 10, 100, 200, 300, 400, 1490], np.uint32)
    dst_tok = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint32)
    delta = np.array([0, 1, -1, 131071, -2**31, 2**31 - 1, 0], np.int32)
    hits = orc.Hits(src_row, dst_tok, lens, delta)
    n_tok = int(lens.sum())
    inv = wl.inv_freq_yarn()
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, L, inv, 4096, 1, DEV, pair_mode=1)
    try:
        src = wl.kv_pool_torch(L, src_rows, 77, DEV)
        dst = wl.sentinel_pool_torch(L, dst_rows, DEV)
        slots = rng.permutation(dst_rows)[:n_tok].astype(np.int32)
        d_hits, d_n = hits_to_dev(hits, 16)
        B.irm_reattach(s.ctx, B.layer_pointers(src), ROW * 2, src_rows, B.layer_pointers(dst), ROW * 2, dst_rows,
                       torch.from_numpy(slots).to(DEV), d_hits, d_n)
        assert s.error_flags() == 0

        class W:
            dst_slots, inv_freq = slots, inv
        stats = verify_reattach(W, hits, src, dst, what="interleaved special", pair_mode=1)
        assert stats["rows"] == n_tok * L
        for h in (0, 6):
            for j in range(int(lens[h])):
                assert np.array_equal(bits(src[:, int(src_row[h]) + j]), bits(dst[:, int(slots[int(dst_tok[h]) + j])]))
    finally:
        s.close()


# ------------------------------------------------------------ graph capture --

def test_hot_path_captured_in_a_graph_replays_like_eager():
    """The four calls allocate nothing, never synchronise and record no memset nodes: they can be
    captured once and replayed.  Several replays, with eager work and synchronisation between
    them, against the eager result."""
    w = small("c2")
    rig = Rig(w)
    try:
        rig.serve()
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        want_dst = rig.dst.clone()
        keys = ("chunk_start", "chunk_len", "req_chunk_offsets", "n_chunks", "chunk_hash", "chunk_entry", "hits",
                "n_hits", "hit_tokens")
        want = {k: rig.buf[k].clone() for k in keys}
        n_hits = int(want["n_hits"].item())
        stream = torch.cuda.Stream(device=DEV)
        graph = torch.cuda.CUDAGraph()
        serve = lambda: rig.s.serve(rig.d_tokens, rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.src_ptrs,
                                    ROW * 2, w.src_rows, rig.dst_ptrs, ROW * 2, w.dst_rows, rig.buf, stream)
        with torch.cuda.stream(stream):
            serve()
            stream.synchronize()
            with torch.cuda.graph(graph, stream=stream):
                serve()
        torch.cuda.synchronize()
        for rep in range(4):
            rig.dst.view(torch.int16).fill_(wl.SENTINEL_BF16)          # eager work between the replays
            for k in keys:
                rig.buf[k].fill_(-1 if k != "hit_tokens" else 7)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert rig.s.error_flags() == 0
            assert torch.equal(rig.dst.view(torch.int16), want_dst.view(torch.int16)), rep
            n = int(want["n_chunks"].item())
            for k in ("chunk_start", "chunk_len", "chunk_hash", "chunk_entry"):
                assert torch.equal(rig.buf[k][:n], want[k][:n]), (rep, k)
            assert torch.equal(rig.buf["hits"][:n_hits], want["hits"][:n_hits])
            for k in ("req_chunk_offsets", "n_chunks", "n_hits", "hit_tokens"):
                assert torch.equal(rig.buf[k], want[k]), (rep, k)
    finally:
        rig.close()


# ------------------------------------------------- no-materialise variant --

@pytest.mark.parametrize("name", ["c0", "c1", "c2", "c3", "c4"])
@pytest.mark.parametrize("slots", ["contiguous", "permuted"])
def test_reattach_ref_small_configs(name, slots):
    """References bit for bit; the rotation table within one fp32 step of the oracle's fp64 values,
    and good enough that rotating at load time lands within the k_r tolerance."""
    w = small(name, slots=slots)
    o = oracle_front(w)
    hits = o["hits"]
    s = Session.for_workload(w, DEV)
    try:
        cap = max(len(hits), 1) + 5
        d_hits, d_n = hits_to_dev(hits, cap)
        row = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        hit = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        trig = torch.full((cap, 32, 2), 9.0, dtype=torch.float32, device=DEV)
        B.irm_reattach_ref(s.ctx, w.src_rows, row, hit, trig, torch.from_numpy(w.dst_slots).to(DEV), d_hits, d_n)
        torch.cuda.synchronize()
        assert s.error_flags() == 0
        want_row = np.full(w.dst_rows, -1, np.int32)
        want_hit = np.full(w.dst_rows, -1, np.int32)
        want_trig = orc.reattach_ref(w.src_rows, want_row, want_hit, w.dst_slots, hits, w.inv_freq)
        assert np.array_equal(row.cpu().numpy(), want_row) and np.array_equal(hit.cpu().numpy(), want_hit)
        got_trig = trig.cpu().numpy()
        n = len(hits)
        assert np.all(got_trig[n:] == 9.0)                                   # nothing past the hit count
        err = np.abs(got_trig[:n].astype(np.float64) - want_trig)
        assert err.max() <= 2.0 ** -23                                       # fp32 rounding of values in [-1, 1]
        zero = hits.delta == 0
        assert np.all(got_trig[:n][zero] == np.array([1.0, 0.0], np.float32))
        # a load path using this table: rows of layer 0 of a few hits
        src = wl.kv_pool_torch(1, w.src_rows, wl.kv_seed(name), DEV)
        src_h = bits(src)
        for h in range(0, n, max(1, n // 6)):
            rows = src_h[0, hits.src_row[h]:hits.src_row[h] + hits.len[h]]
            k = orc.bf16_to_f64(rows[:, 512:])
            z = (k[:, :32] + 1j * k[:, 32:]) * (got_trig[h, :, 0].astype(np.float64) + 1j * got_trig[h, :, 1])
            lazy = rows.copy()
            lazy[:, 512:] = orc.f64_to_bf16(np.concatenate([z.real, z.imag], axis=1))
            want = np.stack([orc.reattach_row(r, int(hits.delta[h]), w.inv_freq) for r in rows])
            compare_rows(lazy[None], want[None], what=f"{w.name} hit {h} rotated at load")
    finally:
        s.close()


def test_reattach_ref_bad_indices_are_skipped_and_flagged():
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, 1, wl.inv_freq_plain(), 4096, 1, DEV)
    try:
        hits = orc.Hits(np.array([0, 90, 10], np.uint32), np.array([0, 300, 600], np.uint32),
                        np.array([300, 300, 100], np.uint32), np.array([5, -5, 0], np.int32))   # hit 1 leaves the pool
        d_hits, d_n = hits_to_dev(hits, 4)
        slots = np.arange(700, dtype=np.int32)
        slots[7] = 900                                                       # outside the destination
        row = torch.full((800,), -1, dtype=torch.int32, device=DEV)
        hit = torch.full((800,), -1, dtype=torch.int32, device=DEV)
        trig = torch.zeros((4, 32, 2), dtype=torch.float32, device=DEV)
        B.irm_reattach_ref(s.ctx, 350, row, hit, trig, torch.from_numpy(slots).to(DEV), d_hits, d_n)
        torch.cuda.synchronize()
        assert s.error_flags() == B.IRM_FLAG_ROW_RANGE
        r = row.cpu().numpy()
        want = np.full(800, -1, np.int32)
        want[:300] = np.arange(300)
        want[7] = -1
        want[600:700] = 10 + np.arange(100)
        assert np.array_equal(r, want)
        assert np.array_equal(hit.cpu().numpy() >= 0, want >= 0)
    finally:
        s.close()
