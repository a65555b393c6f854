"""Pins for the oracle's registry lookup (paper Alg. 1 steps 4-8, 12-13; Sec. 7.1 carve-out).

Pinned to a linear search over the entry list, to a python dict filled by
insert-if-absent, and to the construction of the synthetic requests: a request
assembled from whole pool chunks must find exactly those chunks, with
delta = new position - stored position, and must miss the chunk at position 0
even though the registry holds it.
"""
import numpy as np
import pytest

from oracle import irm_oracle as orc
from paper_2605_05696_amd import workloads as wl


def run_lookup(reg, chunk_hash, start, length, rco, req_offsets, pos_base, carve_out):
    return orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"],
                      chunk_hash, start, length, rco, req_offsets, pos_base, carve_out)


def linear_search_lookup(reg, chunk_hash, start, length, rco, req_offsets, pos_base, carve_out):
    entry, hits = [], []
    for r in range(len(req_offsets) - 1):
        for c in range(int(rco[r]), int(rco[r + 1])):
            p = int(pos_base[r]) + int(start[c]) - int(req_offsets[r])
            found = -1
            if p >= carve_out:
                for e in range(len(reg["hash"])):          # first listed entry with this hash
                    if int(reg["hash"][e]) == int(chunk_hash[c]):
                        found = e
                        break
                if found >= 0 and int(reg["len"][found]) != int(length[c]):
                    found = -1
            if found >= 0:
                entry.append(int(reg["entry_id"][found]))
                hits.append((int(reg["src_row"][found]), int(start[c]), int(length[c]),
                             p - int(reg["p_src"][found])))
            else:
                entry.append(-1)
    return entry, hits


def random_case(seed, n_reg=40, n_chunks=60, n_req=4):
    rng = np.random.default_rng(seed)
    keys = rng.integers(0, 12, size=n_reg, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)  # many duplicates
    reg = dict(hash=keys, src_row=rng.integers(0, 10**6, n_reg).astype(np.uint32),
               p_src=rng.integers(0, 5000, n_reg).astype(np.int32),
               len=rng.integers(64, 67, n_reg).astype(np.uint32),
               entry_id=rng.permutation(n_reg).astype(np.uint32) + np.uint32(100))
    length = rng.integers(64, 67, n_chunks).astype(np.uint32)
    cuts = np.sort(rng.choice(np.arange(1, n_chunks), size=n_req - 1, replace=False))
    rco = np.concatenate([[0], cuts, [n_chunks]]).astype(np.uint32)
    start = np.concatenate([[0], np.cumsum(length)[:-1]]).astype(np.uint32)
    req_offsets = np.concatenate([start[rco[:-1]], [int(length.sum())]]).astype(np.uint32)
    chunk_hash = rng.integers(0, 14, size=n_chunks, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    pos_base = rng.integers(0, 40, n_req).astype(np.int32)
    pos_base[0] = 0
    return reg, chunk_hash, start, length, rco, req_offsets, pos_base


@pytest.mark.parametrize("seed", range(6))
def test_against_linear_search(seed):
    args = random_case(seed)
    entry, hits, hit_tokens = run_lookup(*args, 32)
    want_entry, want_hits = linear_search_lookup(*args, 32)
    assert entry.tolist() == want_entry
    assert list(zip(hits.src_row.tolist(), hits.dst_tok.tolist(), hits.len.tolist(),
                    hits.delta.tolist())) == want_hits
    assert hit_tokens == sum(h[2] for h in want_hits)
    assert any(e >= 0 for e in want_entry) and any(e < 0 for e in want_entry)


def test_against_python_dict_insert_if_absent():
    reg, chunk_hash, start, length, rco, req_offsets, pos_base = random_case(99, 500, 300, 7)
    table = {}
    for e, h in enumerate(reg["hash"].tolist()):
        table.setdefault(h, e)                               # insert-if-absent: first wins
    entry, hits, _ = run_lookup(reg, chunk_hash, start, length, rco, req_offsets, pos_base, 0)
    for c in range(len(chunk_hash)):
        e = table.get(int(chunk_hash[c]), -1)
        if e >= 0 and int(reg["len"][e]) != int(length[c]):
            e = -1
        assert entry[c] == (int(reg["entry_id"][e]) if e >= 0 else -1)
    assert np.all(np.diff(hits.dst_tok.astype(np.int64)) > 0)     # ascending chunk order


def test_carve_out_and_pos_base():
    reg = dict(hash=np.array([7, 8], np.uint64), src_row=np.array([10, 20], np.uint32),
               p_src=np.array([1000, 5], np.int32), len=np.array([64, 64], np.uint32),
               entry_id=np.array([0, 1], np.uint32))
    ch = np.array([7, 8, 7], np.uint64)
    start = np.array([0, 64, 128], np.uint32)
    length = np.array([64, 64, 64], np.uint32)
    rco = np.array([0, 2, 3], np.uint32)
    off = np.array([0, 128, 192], np.uint32)
    # request 0 starts at position 0: its first chunk is carved out although registered
    entry, hits, tok = run_lookup(reg, ch, start, length, rco, off, np.array([0, 31], np.int32), 32)
    assert entry.tolist() == [-1, 1, -1]           # chunk 2 sits at position 31 < 32
    assert hits.delta.tolist() == [64 - 5] and tok == 64
    # one position further and it is served; delta may be negative
    entry, hits, _ = run_lookup(reg, ch, start, length, rco, off, np.array([0, 32], np.int32), 32)
    assert entry.tolist() == [-1, 1, 0] and hits.delta.tolist() == [59, 32 - 1000]
    # carve-out disabled
    entry, _, _ = run_lookup(reg, ch, start, length, rco, off, np.array([0, 0], np.int32), 0)
    assert entry.tolist() == [0, 1, 0]


def test_length_guard_and_first_wins():
    reg = dict(hash=np.array([5, 5, 6], np.uint64), src_row=np.array([1, 2, 3], np.uint32),
               p_src=np.array([0, 0, 0], np.int32), len=np.array([70, 64, 64], np.uint32),
               entry_id=np.array([0, 1, 2], np.uint32))
    ch = np.array([5, 5, 6], np.uint64)
    start = np.array([100, 170, 234], np.uint32)
    length = np.array([70, 64, 64], np.uint32)
    entry, hits, _ = run_lookup(reg, ch, start, length, np.array([0, 3], np.uint32),
                                np.array([0, 298], np.uint32), np.array([0], np.int32), 32)
    # the second listed entry with hash 5 never made it into the registry, so a
    # 64-token chunk with that hash fails the length guard
    assert entry.tolist() == [0, -1, 2]
    assert hits.src_row.tolist() == [1, 3]


@pytest.mark.parametrize("cdc", ["config", "paper"])
@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_planted_requests_are_recovered(name, cdc):
    """End-to-end closed form: chunk + fingerprint + lookup of an assembled request
    returns exactly the planted pool chunks (position independence of the whole
    front end), each with delta = new position - stored position.  Under the measured
    configurations' rule and under the paper's own (Sec. 7.2, App. B: 7 bits, 32..512)."""
    w = wl.make_workload(name, orc.cdc_chunk, size="small", cdc=cdc)
    assert (w.mask, w.min_chunk, w.max_chunk) == ((0xFF, 64, 1024) if cdc == "config" else (0x7F, 32, 512))
    st, ln, rco = orc.cdc_chunk(w.tokens, w.req_offsets, w.gear, w.mask, w.min_chunk, w.max_chunk)
    assert st.astype(np.int64).tolist() == w.piece_start.tolist()
    assert ln.astype(np.int64).tolist() == w.piece_len.tolist()
    reg = w.registry(orc.chunk_hash(w.pool_tokens, w.pool_chunk_start, w.pool_chunk_len))
    ch = orc.chunk_hash(w.tokens, st, ln)
    entry, hits, hit_tokens = run_lookup(reg, ch, st, ln, rco, w.req_offsets, w.pos_base, w.carve_out)
    e_start, e_len, e_chunk, e_delta = w.expected_hits()
    assert hits.dst_tok.astype(np.int64).tolist() == e_start.tolist()
    assert hits.len.astype(np.int64).tolist() == e_len.tolist()
    assert hits.delta.astype(np.int64).tolist() == e_delta.tolist()
    assert hits.src_row.astype(np.int64).tolist() == w.pool_chunk_start[e_chunk].astype(np.int64).tolist()
    assert hit_tokens == int(e_len.sum())
    assert entry[entry >= 0].tolist() == e_chunk.tolist()
    # the chunk at position 0 of a request that starts at position 0 is never served
    for r in range(w.n_req):
        if w.pos_base[r] == 0:
            assert entry[rco[r]] == -1
    if name == "c0":
        assert np.all(np.abs(hits.delta) <= 2048) and len(hits) == len(st) - 1
        assert w.piece_pool_chunk[0] >= 0        # it IS registered; only the carve-out stops it
