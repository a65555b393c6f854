"""GPU parity for pools of fp8 rows (IRM_ROW_FP8: 512 e4m3 bytes | four fp32 scales | k_r as 64
bf16; the paper's Sec. 7.2 counts FP8 KV quantisation as accepted practice), against the oracle.

The 528 position-free bytes must arrive bit for bit; the rotated k_r is held to the bf16 rows'
bound (2 bf16 steps of the oracle's fp64-rounded value or 1e-2 absolute); bytes of rows and of
padding that nothing should write keep their sentinel.
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
    from tests.gpu_util import (DEV, Rig, bits, compare_rows, covered_rows, hits_from_dev, hits_to_dev,
                                oracle_front, verify_reattach)

F8 = B.IRM_ROW_FP8
W8 = 328                                                                # 16-bit words of an fp8 row


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
@pytest.mark.parametrize("slots,pair_mode", [("contiguous", 0), ("permuted", 0), ("permuted", 1)])
def test_reattach_fp8_rows_small_configs_all_rows(name, slots, pair_mode):
    w = wl.make_workload(name, orc.cdc_chunk, size="small", slots=slots)
    rig = Rig(w, with_table=False, pair_mode=pair_mode, row_format=F8)
    try:
        assert rig.src.shape[2] == W8 and rig.row_bytes == 656
        hits = rig.o["hits"]
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        rig.reattach(d_hits, d_n)
        assert rig.s.error_flags() == 0
        stats = verify_reattach(w, hits, rig.src, rig.dst, what=w.name, pair_mode=pair_mode)
        assert stats["rows"] == rig.o["hit_tokens"] * w.n_layers
        assert stats["exact"] > 0.95
        untouched = ~covered_rows(w, hits)
        rest = bits(rig.dst[:, torch.from_numpy(np.nonzero(untouched)[0]).to(DEV), :])
        assert np.all(rest == wl.SENTINEL_BF16)
        first = rig.dst.clone()
        rig.reattach(d_hits, d_n)
        torch.cuda.synchronize()
        assert torch.equal(first.view(torch.int16), rig.dst.view(torch.int16))
    finally:
        rig.close()


@pytest.mark.parametrize("name", ["c0", "c1", "c3"])
def test_end_to_end_fp8_rows(name):
    w = wl.make_workload(name, orc.cdc_chunk, size="small")
    rig = Rig(w, row_format=F8)
    try:
        rig.serve()
        assert rig.s.error_flags() == 0
        o = rig.o
        g = hits_from_dev(rig.buf["hits"], int(rig.buf["n_hits"].item()))
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(g, f), getattr(o["hits"], f)), f
        verify_reattach(w, o["hits"], rig.src, rig.dst, what=w.name)
    finally:
        rig.close()


@pytest.mark.parametrize("waves,rpw", [(8, 4), (8, 2), (4, 4), (4, 16), (8, 8), (16, 2), (16, 16)])
def test_fp8_rows_tile_shapes_tails_strides_and_special_deltas(waves, rpw):
    """Hit lengths around every tile size, delta = 0 as the exact identity, extreme deltas, rows padded
    to a larger stride (the padding must stay untouched), every launch shape the library admits."""
    rng = np.random.default_rng(5)
    L, src_rows, dst_rows = 2, 3000, 2700
    lens = np.array([1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 255, 257, 1024, 7], np.uint32)
    src_row = np.array([0, 3, 10, 50, 100, 150, 230, 300, 400, 550, 700, 1000, 1300, 2900], np.uint32)
    dst_tok = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint32)
    delta = np.array([0, 1, -1, 131071, -131072, 2**31 - 1, -2**31, 5, -9, 77, 1000, -1000, 31, 0], np.int32)
    hits = orc.Hits(src_row, dst_tok, lens, delta)
    n_tok = int(lens.sum())
    inv = wl.inv_freq_yarn()
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, L, inv, 4096, 1, DEV, row_format=F8)
    try:
        B.irm_ctx_tune(s.ctx, 4, 16)                                   # so that any rows-per-wave passes the tile check
        B.irm_ctx_tune(s.ctx, 1, rpw)
        B.irm_ctx_tune(s.ctx, 4, waves)
        stride_words = W8 + 24                                         # 704-byte stride
        src_full = torch.cat([wl.kv_pool_fp8_torch(L, src_rows, 3, DEV),
                              torch.zeros((L, src_rows, 24), dtype=torch.bfloat16, device=DEV)], dim=2).contiguous()
        dst_full = torch.empty((L, dst_rows, stride_words), dtype=torch.bfloat16, device=DEV)
        dst_full.view(torch.int16).fill_(wl.SENTINEL_BF16)
        src, dst = src_full[:, :, :W8], dst_full[:, :, :W8]
        slots = rng.permutation(dst_rows)[:n_tok].astype(np.int32)
        d_hits, d_n = hits_to_dev(hits, 16)
        B.irm_reattach(s.ctx, B.layer_pointers(src), stride_words * 2, src_rows, B.layer_pointers(dst),
                       stride_words * 2, dst_rows, torch.from_numpy(slots).to(DEV), d_hits, d_n)
        assert s.error_flags() == 0

        class W:
            dst_slots, inv_freq = slots, inv
        stats = verify_reattach(W, hits, src, dst, what=f"fp8 {waves}x{rpw}")
        assert stats["rows"] == n_tok * L
        for h in (0, 13):                                              # delta == 0: whole rows, bit for bit
            for j in range(int(lens[h])):
                a = bits(src[:, int(src_row[h]) + j]), bits(dst[:, int(slots[int(dst_tok[h]) + j])])
                assert np.array_equal(a[0], a[1])
        assert torch.all(dst_full[:, :, W8:].view(torch.int16) == wl.SENTINEL_BF16)
        mask = torch.ones(dst_rows, dtype=torch.bool, device=DEV)
        mask[torch.from_numpy(slots.astype(np.int64)).to(DEV)] = False
        assert torch.all(dst[:, mask].contiguous().view(torch.int16) == wl.SENTINEL_BF16)
    finally:
        s.close()


def test_fp8_rows_launch_shapes_and_strides_that_are_refused():
    s = Session(wl.gear_table(), 0xFF, 64, 1024, 32, 1, wl.inv_freq_plain(), 1024, 1, DEV, row_format=F8)
    try:
        for knob, value in ((1, 1), (4, 1), (4, 2)):                   # one row per wave, fewer than 4 waves
            with pytest.raises(B.IrmError):
                B.irm_ctx_tune(s.ctx, knob, value)
        src = wl.kv_pool_fp8_torch(1, 64, 1, DEV)
        dst = wl.sentinel_pool_torch(1, 64, DEV, W8)
        none = orc.Hits(*(np.zeros(0, t) for t in (np.uint32, np.uint32, np.uint32, np.int32)))
        d_hits, d_n = hits_to_dev(none, 4)
        slots = torch.arange(64, dtype=torch.int32, device=DEV)
        for stride in (640, 656 + 8):                                  # below a row; not a multiple of 16
            with pytest.raises(B.IrmError):
                B.irm_reattach(s.ctx, B.layer_pointers(src), stride, 64, B.layer_pointers(dst), 656, 64, slots,
                               d_hits, d_n)
        B.irm_reattach(s.ctx, B.layer_pointers(src), 656, 64, B.layer_pointers(dst), 656, 64, slots, d_hits, d_n)
        assert s.error_flags() == 0 and torch.all(dst.view(torch.int16) == wl.SENTINEL_BF16)
        # the rotate-on-load attention of this context wants whole 656-byte rows
        q = torch.zeros((1, 16, 576), dtype=torch.bfloat16, device=DEV)
        row = torch.zeros(64, dtype=torch.int32, device=DEV)
        trig = torch.zeros((1, 32, 2), dtype=torch.float32, device=DEV)
        out = torch.zeros((1, 16, 512), dtype=torch.float32, device=DEV)
        lse = torch.zeros((1, 16), dtype=torch.float32, device=DEV)
        ws = torch.empty(B.irm_attend_ref_workspace_bytes(1, 16, 1), dtype=torch.uint8, device=DEV)
        with pytest.raises(B.IrmError) as e:
            B.irm_attend_ref(s.ctx, q, src[0], 640, slots, s.to_dev_u32(np.array([0, 64], np.uint32)), row, row,
                             trig, 0.1, 1, ws, out, lse)
        assert e.value.status == B.IRM_ERR_INVALID_ARG
    finally:
        s.close()


@pytest.mark.parametrize("name", ["c1", "c4"])
def test_split_pool_over_fp8_rows(name):
    """k_r-only materialisation reading the k_r line of packed fp8 rows (528 bytes into each row)."""
    w = wl.make_workload(name, orc.cdc_chunk, size="small", slots="permuted")
    hits = oracle_front(w)["hits"]
    L = w.n_layers
    s = Session.for_workload(w, DEV, row_format=F8)
    try:
        src = wl.kv_pool_fp8_torch(L, w.src_rows, wl.kv_seed(name), DEV)
        kr = torch.empty((L, w.dst_rows, 64), dtype=torch.bfloat16, device=DEV)
        kr.view(torch.int16).fill_(wl.SENTINEL_BF16)
        idx = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=DEV)
        d_hits, d_n = hits_to_dev(hits, len(hits) + 3)
        B.irm_reattach_kr(s.ctx, B.kr_slice_pointers(src), 656, w.src_rows, B.kr_layer_pointers(kr), 128,
                          w.dst_rows, idx, torch.from_numpy(w.dst_slots).to(DEV), d_hits, d_n)
        assert s.error_flags() == 0
        want_kr = np.full((L, w.dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
        want_idx = np.full(w.dst_rows, -1, np.int32)
        orc.reattach_kr(bits(src), want_kr, want_idx, w.dst_slots, hits, w.inv_freq)
        assert np.array_equal(idx.cpu().numpy(), want_idx)
        pad = lambda k: np.concatenate([np.zeros(k.shape[:2] + (512,), np.uint16), k], axis=2)
        compare_rows(pad(bits(kr)), pad(want_kr), what=f"{w.name} k_r only, fp8 rows")
    finally:
        s.close()


@pytest.mark.parametrize("name", ["c1", "c3"])
def test_serve_admit_serve_fp8_rows(name):
    """Miss path on fp8 rows: prefilled rows enter the pool whole (656 bytes), a second pass over the
    same batch re-attaches them at delta = 0, i.e. gives the prefilled rows back bit for bit."""
    w = wl.make_workload(name, orc.cdc_chunk, size="small")
    rig = Rig(w, row_format=F8)
    o, L = rig.o, w.n_layers
    try:
        n_chunks = len(o["start"])
        extra = int(o["len"][o["entry"] < 0].sum())
        pool_rows = w.src_rows + extra
        pool = torch.cat([rig.src, wl.sentinel_pool_torch(L, extra, DEV, W8)], dim=1).contiguous()
        pool_ptrs = B.layer_pointers(pool)
        rig.dst.copy_(wl.kv_pool_fp8_torch(L, w.dst_rows, 977, DEV))     # "after prefill"
        rig.serve()
        torch.cuda.synchronize()
        req_h, pool_h = bits(rig.dst), bits(pool)
        d_cursor = torch.tensor([w.src_rows], dtype=torch.int32, device=DEV)
        d_adm = torch.full((rig.buf["cap"],), -7, dtype=torch.int32, device=DEV)
        rig.s.admit(rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, rig.dst_ptrs, 656, w.dst_rows,
                    pool_ptrs, 656, pool_rows, d_cursor, d_adm, rig.buf)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        want_adm, new, want_cursor = orc.admit(o["reg"]["hash"], o["hash"], o["start"], o["len"], o["rco"],
                                               w.req_offsets, w.pos_base, w.carve_out, o["entry"], req_h,
                                               w.dst_slots, pool_h, w.src_rows)
        assert (want_adm >= 0).sum() > 0
        assert np.array_equal(d_adm.cpu().numpy()[:n_chunks], want_adm) and int(d_cursor.item()) == want_cursor
        assert np.array_equal(bits(pool), pool_h) and np.array_equal(bits(rig.dst), req_h)
        dst2 = wl.sentinel_pool_torch(L, w.dst_rows, DEV, W8)
        rig.s.serve(rig.d_tokens, rig.d_req_offsets, rig.d_pos_base, rig.d_dst_slots, pool_ptrs, 656, pool_rows,
                    B.layer_pointers(dst2), 656, w.dst_rows, rig.buf)
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        out2 = bits(dst2)
        for c in np.nonzero(want_adm >= 0)[0]:
            rws = w.dst_slots[int(o["start"][c]):int(o["start"][c]) + int(o["len"][c])]
            assert np.array_equal(out2[:, rws], req_h[:, rws])
    finally:
        rig.close()
