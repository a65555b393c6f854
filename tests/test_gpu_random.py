"""Randomised end-to-end parity: random CDC parameters, gear tables, vocabularies, request
mixes (empty and tiny requests included), registries with repeated content, both pair
layouts; every stage, every re-attachment variant (full rows with and without a context,
k_r alone, references) and the miss path against the oracle on each case."""
import os

import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl
from paper_2605_05696_amd.pipeline import Session

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_util import DEV, ROW, bits, compare_rows, hits_from_dev


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


def random_case(seed):
    rng = np.random.default_rng(seed)
    k = int(rng.integers(0, 11))
    mask = (1 << k) - 1
    lo = int(rng.integers(max(k, 1), 80))
    hi = int(rng.integers(lo, lo + int(rng.choice([0, 5, 300, 3000]))  + 1))
    vocab = int(rng.choice([2, 5, 300, 102400]))
    gear = rng.integers(0, 2**32, 256, dtype=np.uint64).astype(np.uint32)
    library = rng.integers(0, vocab, int(rng.integers(500, 20000))).astype(np.int32)
    n_req = int(rng.integers(1, 12))
    reqs = []
    for _ in range(n_req):
        kind = rng.integers(0, 6)
        if kind == 0:
            reqs.append(np.zeros(0, np.int32))                          # empty request
            continue
        parts = []
        for _ in range(int(rng.integers(1, 6))):
            if rng.random() < 0.6:                                      # a slice of the library, any offset
                a = int(rng.integers(0, len(library)))
                parts.append(library[a:a + int(rng.integers(1, 4000))])
            else:
                parts.append(rng.integers(0, vocab, int(rng.integers(1, 1500))).astype(np.int32))
        reqs.append(np.concatenate(parts))
    tokens = np.concatenate(reqs) if sum(len(r) for r in reqs) else np.zeros(0, np.int32)
    off = np.concatenate([[0], np.cumsum([len(r) for r in reqs])]).astype(np.uint32)
    pos_base = rng.integers(0, 50, n_req).astype(np.int32) * rng.integers(0, 2, n_req).astype(np.int32)
    carve = int(rng.choice([0, 32]))
    inv = wl.inv_freq_plain() if rng.random() < 0.5 else wl.inv_freq_yarn()
    return dict(rng=rng, mask=mask, lo=lo, hi=hi, gear=gear, library=library, tokens=tokens, off=off,
                pos_base=pos_base, carve=carve, inv=inv, pair_mode=int(rng.integers(0, 2)), L=int(rng.integers(1, 3)))


# IRM_TEST_SEEDS=N widens the sweep for a longer soak (default 40 cases)
@pytest.mark.parametrize("seed", range(int(os.environ.get("IRM_TEST_SEEDS", "40"))))
def test_random_case_every_stage(seed):
    c = random_case(seed)
    rng, tokens, off = c["rng"], c["tokens"], c["off"]
    n_tok, n_req, L = len(tokens), len(off) - 1, c["L"]
    if n_tok == 0:
        pytest.skip("all requests empty")
    lib = c["library"]
    # the oracle's view
    pst, pln, _ = orc.cdc_chunk(lib, [0, len(lib)], c["gear"], c["mask"], c["lo"], c["hi"])
    reg = dict(hash=orc.chunk_hash(lib, pst, pln), src_row=pst.astype(np.uint32),
               p_src=rng.integers(0, 5000, len(pst)).astype(np.int32), len=pln.astype(np.uint32),
               entry_id=np.arange(len(pst), dtype=np.uint32))
    st, ln, rco = orc.cdc_chunk(tokens, off, c["gear"], c["mask"], c["lo"], c["hi"])
    ch = orc.chunk_hash(tokens, st, ln)
    entry, hits, hit_tokens = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"], ch,
                                         st, ln, rco, off, c["pos_base"], c["carve"])
    # the library's view
    s = Session(c["gear"], c["mask"], c["lo"], c["hi"], c["carve"], L, c["inv"], max(n_tok, len(lib)), n_req, DEV,
                pair_mode=c["pair_mode"])
    try:
        B.irm_ctx_tune(s.ctx, 3, seed % 4)                                 # every mapping of workgroups to tiles
        g_pst, g_pln, _, g_ph = s.chunk_host(lib, np.array([0, len(lib)], np.uint32))
        assert np.array_equal(g_pst, pst) and np.array_equal(g_pln, pln) and np.array_equal(g_ph, reg["hash"])
        s.build_table(int((len(pst) + len(st)) / 0.6) + 4, reg)            # room for what the miss path adds
        d_tok, d_off = torch.from_numpy(tokens).to(DEV), s.to_dev_u32(off)
        d_pos = torch.from_numpy(c["pos_base"]).to(DEV)
        slots = rng.permutation(n_tok).astype(np.int32)
        d_slots = torch.from_numpy(slots).to(DEV)
        free = int(ln[entry < 0].sum()) // 2 + 1                          # the pool runs out half way
        pool_rows = len(lib) + free
        pool = torch.cat([wl.kv_pool_torch(L, len(lib), 800 + seed, DEV), wl.sentinel_pool_torch(L, free, DEV)],
                         dim=1).contiguous()
        req = wl.kv_pool_torch(L, n_tok, 900 + seed, DEV)
        pool_ptrs, req_ptrs = B.layer_pointers(pool), B.layer_pointers(req)
        buf = s.alloc_front(n_tok, n_req)
        want_rows = bits(req)
        if len(hits):
            orc.reattach(bits(pool), want_rows, slots, hits, c["inv"], c["pair_mode"])
        s.serve(d_tok, d_off, d_pos, d_slots, pool_ptrs, ROW * 2, pool_rows, req_ptrs, ROW * 2, n_tok, buf)
        torch.cuda.synchronize()
        assert s.error_flags() == 0
        n = int(buf["n_chunks"].item())
        u32 = lambda t: t.cpu().numpy().view(np.uint32)
        assert n == len(st) and np.array_equal(u32(buf["chunk_start"])[:n], st)
        assert np.array_equal(u32(buf["chunk_len"])[:n], ln) and np.array_equal(u32(buf["req_chunk_offsets"]), rco)
        assert np.array_equal(buf["chunk_hash"].cpu().numpy().view(np.uint64)[:n], ch)
        assert np.array_equal(buf["chunk_entry"].cpu().numpy()[:n], entry)
        got = hits_from_dev(buf["hits"], int(buf["n_hits"].item()))
        for f in ("src_row", "dst_tok", "len", "delta"):
            assert np.array_equal(getattr(got, f), getattr(hits, f)), f
        assert int(buf["hit_tokens"].item()) == hit_tokens
        compare_rows(bits(req), want_rows, what=f"seed {seed}")
        # the same hit list through the other re-attachment variants
        n_hits_max = buf["hits"].shape[0]
        if len(hits) and n_tok <= B.REATTACH_STATIC_MAX_TOKENS and n_hits_max <= B.REATTACH_STATIC_MAX_HITS:
            again = wl.kv_pool_torch(L, n_tok, 900 + seed, DEV)            # without a context: bit-equal to the above
            flags = torch.zeros(1, dtype=torch.int32, device=DEV)
            B.irm_reattach_static(c["inv"], L, c["pair_mode"], B.IRM_ROW_BF16, pool_ptrs, ROW * 2, pool_rows,
                                  B.layer_pointers(again), ROW * 2, n_tok, d_slots, buf["hits"], buf["n_hits"], flags)
            torch.cuda.synchronize()
            assert int(flags.item()) == 0 and torch.equal(again.view(torch.int16), req.view(torch.int16))
        kr = torch.empty((L, n_tok, 64), dtype=torch.bfloat16, device=DEV)  # split pool: k_r alone
        kr.view(torch.int16).fill_(wl.SENTINEL_BF16 - 0x10000 if wl.SENTINEL_BF16 >= 0x8000 else wl.SENTINEL_BF16)
        idx = torch.full((n_tok,), -1, dtype=torch.int32, device=DEV)
        B.irm_reattach_kr(s.ctx, B.kr_slice_pointers(pool), ROW * 2, pool_rows, B.kr_layer_pointers(kr), 128, n_tok,
                          idx, d_slots, buf["hits"], buf["n_hits"])
        row = torch.full((n_tok,), -1, dtype=torch.int32, device=DEV)       # no-materialise: references
        hit = torch.full((n_tok,), -1, dtype=torch.int32, device=DEV)
        trig = torch.zeros((n_hits_max, 32, 2), dtype=torch.float32, device=DEV)
        B.irm_reattach_ref(s.ctx, pool_rows, row, hit, trig, d_slots, buf["hits"], buf["n_hits"])
        torch.cuda.synchronize()
        assert s.error_flags() == 0
        want_kr = np.full((L, n_tok, 64), wl.SENTINEL_BF16, np.uint16)
        want_idx = np.full(n_tok, -1, np.int32)
        want_row, want_hit = np.full(n_tok, -1, np.int32), np.full(n_tok, -1, np.int32)
        if len(hits):
            orc.reattach_kr(bits(pool), want_kr, want_idx, slots, hits, c["inv"], c["pair_mode"])
            want_trig = orc.reattach_ref(pool_rows, want_row, want_hit, slots, hits, c["inv"])
            assert np.abs(trig.cpu().numpy()[:len(hits)].astype(np.float64) - want_trig).max() <= 2.0 ** -23
        assert np.array_equal(idx.cpu().numpy(), want_idx)
        assert np.array_equal(row.cpu().numpy(), want_row) and np.array_equal(hit.cpu().numpy(), want_hit)
        pad = lambda k: np.concatenate([np.zeros(k.shape[:2] + (512,), np.uint16), k], axis=2)
        compare_rows(pad(bits(kr)), pad(want_kr), what=f"seed {seed} k_r only")
        # miss path
        d_cursor = torch.tensor([len(lib)], dtype=torch.int32, device=DEV)
        d_adm = torch.full((buf["cap"],), -7, dtype=torch.int32, device=DEV)
        s.admit(d_off, d_pos, d_slots, req_ptrs, ROW * 2, n_tok, pool_ptrs, ROW * 2, pool_rows, d_cursor, d_adm, buf)
        torch.cuda.synchronize()
        assert s.error_flags() == 0
        pool_h = bits(pool)                                                # taken after the call: compare the tail only
        want_pool = pool_h.copy()
        want_pool[:, len(lib):] = wl.SENTINEL_BF16
        adm, new, cursor = orc.admit(reg["hash"], ch, st, ln, rco, off, c["pos_base"], c["carve"], entry, bits(req),
                                     slots, want_pool, len(lib))
        assert np.array_equal(d_adm.cpu().numpy()[:n], adm) and int(d_cursor.item()) == cursor
        assert np.array_equal(pool_h, want_pool)
    finally:
        s.close()
