"""irm_reattach_static, the entry point for callers that cannot allocate: its output against
irm_reattach's (same kernels, so bit for bit) and against the CPU oracle, on two calls in a
row that share the library's static scratch, the second with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests.gpu_util import DEV, Rig, bits, covered_rows, hits_to_dev, verify_reattach


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


def one_call(name, pair_mode=0, row_format=0):
    """One workload through both entry points; returns nothing, asserts everything."""
    w = wl.make_workload(name, orc.cdc_chunk, size="small")
    rig = Rig(w, pair_mode=pair_mode, row_format=row_format)
    try:
        hits = rig.o["hits"]
        assert 0 < len(hits) <= B.REATTACH_STATIC_MAX_HITS and len(w.tokens) <= B.REATTACH_STATIC_MAX_TOKENS
        d_hits, d_n = hits_to_dev(hits, rig.buf["cap"])
        rig.reattach(d_hits, d_n)                                   # the existing entry point
        torch.cuda.synchronize()
        assert rig.s.error_flags() == 0
        want = bits(rig.dst)
        dst2 = wl.sentinel_pool_torch(w.n_layers, w.dst_rows, DEV, B.ROW_WORDS[row_format])
        flags = torch.zeros(1, dtype=torch.int32, device=DEV)
        B.irm_reattach_static(w.inv_freq, w.n_layers, pair_mode, row_format, rig.src_ptrs, rig.row_bytes, w.src_rows,
                              B.layer_pointers(dst2), rig.row_bytes, w.dst_rows, rig.d_dst_slots, d_hits, d_n, flags)
        torch.cuda.synchronize()
        assert int(flags.item()) == 0
        got = bits(dst2)
        assert np.array_equal(got, want), f"{name}: the two entry points differ"
        if row_format == 0:
            # and against the oracle itself, to the path's own bar
            stats = verify_reattach(w, hits, rig.src, dst2, what=f"static {name}", pair_mode=pair_mode)
            assert stats["rows"] > 0
        untouched = ~covered_rows(w, hits)
        assert np.all(got[:, untouched] == wl.SENTINEL_BF16)
    finally:
        rig.close()


def test_two_calls_in_a_row_share_the_static_scratch():
    one_call("c2")          # 5 requests, 20 K tokens, two layers
    one_call("c0")          # then a smaller batch: one request, 4 K tokens, one layer
    one_call("c3", pair_mode=1)
    one_call("c1", row_format=1)


def test_bad_indices_are_flagged_and_skipped():
    w = wl.make_workload("c0", orc.cdc_chunk, size="small")
    rig = Rig(w)
    try:
        hits = rig.o["hits"]
        bad = orc.Hits(hits.src_row.copy(), hits.dst_tok.copy(), hits.len.copy(), hits.delta.copy())
        bad.src_row[0] = w.src_rows                                 # past the pool
        d_hits, d_n = hits_to_dev(bad, rig.buf["cap"])
        flags = torch.zeros(1, dtype=torch.int32, device=DEV)
        B.irm_reattach_static(w.inv_freq, w.n_layers, 0, 0, rig.src_ptrs, rig.row_bytes, w.src_rows, rig.dst_ptrs,
                              rig.row_bytes, w.dst_rows, rig.d_dst_slots, d_hits, d_n, flags)
        torch.cuda.synchronize()
        assert int(flags.item()) & B.IRM_FLAG_ROW_RANGE
        rows = w.dst_slots[int(bad.dst_tok[0]):int(bad.dst_tok[0]) + int(bad.len[0])]
        assert np.all(bits(rig.dst)[:, rows] == wl.SENTINEL_BF16)
        good = orc.Hits(hits.src_row[1:], hits.dst_tok[1:], hits.len[1:], hits.delta[1:])
        verify_reattach(w, good, rig.src, rig.dst, what="static, bad hit skipped")
        # the same call without a flag word: the bits are dropped, the good rows still land
        B.irm_reattach_static(w.inv_freq, w.n_layers, 0, 0, rig.src_ptrs, rig.row_bytes, w.src_rows, rig.dst_ptrs,
                              rig.row_bytes, w.dst_rows, rig.d_dst_slots, d_hits, d_n, None)
        torch.cuda.synchronize()
        verify_reattach(w, good, rig.src, rig.dst, what="static, no flag word")
    finally:
        rig.close()


def test_sizes_beyond_the_static_array_are_refused():
    L = B.lib()
    import ctypes
    f = (ctypes.c_float * 32)(*([1.0] * 32))
    one = ctypes.c_void_p(16)                                       # never dereferenced: the check comes first
    st = L.irm_reattach_static(f, 1, 0, 0, one, 1152, 1, one, 1152, 1, one, B.REATTACH_STATIC_MAX_TOKENS + 1, one,
                               one, 1, None, None)
    assert st == B.IRM_ERR_CAPACITY
    st = L.irm_reattach_static(f, 1, 0, 0, one, 1152, 1, one, 1152, 1, one, 1, one, one,
                               B.REATTACH_STATIC_MAX_HITS + 1, None, None)
    assert st == B.IRM_ERR_CAPACITY
