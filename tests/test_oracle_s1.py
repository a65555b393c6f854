"""Pins for the oracle's S1 fallback (paper Sec. 4 "CDC+fallback"; App. G "S1:
detect-and-recover"): a chunk that missed is cut into fixed 128-token windows,
each window is fingerprinted and looked up on its own.

The sub-division is pinned to its invariants and to a brute-force enumeration;
the composed pipeline (sub-divide, fingerprint, look up) is pinned to a search by
token CONTENT that never computes a hash, and to the recovery it exists for: a
shared region whose first chunk drifted because different text precedes it.
"""
import numpy as np
import pytest

from oracle import irm_oracle as orc
from paper_2605_05696_amd import workloads as wl

GEAR = wl.gear_table()


def test_subdivision_invariants_and_brute_force():
    rng = np.random.default_rng(0)
    for trial in range(200):
        n_req = int(rng.integers(1, 4))
        W = int(rng.choice([1, 3, 8, 128]))
        starts, lens, rco, cur = [], [], [0], 0
        for _ in range(n_req):
            for _ in range(int(rng.integers(0, 6))):
                l = int(rng.integers(1, 5 * W + 2))
                starts.append(cur)
                lens.append(l)
                cur += l
            rco.append(len(starts))
        starts, lens = np.array(starts, np.uint32), np.array(lens, np.uint32)
        expand = rng.random(len(starts)) < 0.6
        for anchor in (0, 1):
            ws, wl_, wp, rwo = orc.s1_windows(starts, lens, rco, expand, W, anchor)
            # brute force: mark every token a window may cover, token by token
            want = []
            for c in range(len(starts)):
                if not expand[c]:
                    continue
                n = int(lens[c]) // W
                for j in range(n):
                    first = int(starts[c]) + j * W if anchor == 0 else int(starts[c]) + int(lens[c]) - (n - j) * W
                    want.append((first, c))
            assert list(zip(ws.tolist(), wp.tolist())) == want
            assert np.all(wl_ == W) and len(ws) == int((lens[expand] // W).sum())
            assert np.all(np.diff(ws.astype(np.int64)) >= W)               # ascending and disjoint
            assert np.all(ws >= starts[wp]) and np.all(ws + W <= starts[wp] + lens[wp])
            for r in range(n_req):                                          # CSR follows the chunks' requests
                inside = wp[rwo[r]:rwo[r + 1]]
                assert np.all((inside >= rco[r]) & (inside < rco[r + 1]))
            assert rwo[0] == 0 and rwo[-1] == len(ws)
            if anchor == 0:
                firsts = ws[np.concatenate([[True], wp[1:] != wp[:-1]])] if len(ws) else ws
                assert np.all(firsts == starts[np.unique(wp)])
            else:
                lasts = ws[np.concatenate([wp[1:] != wp[:-1], [True]])] if len(ws) else ws
                assert np.all(lasts + W == (starts + lens)[np.unique(wp)])


def test_whole_multiples_give_the_same_windows_for_both_anchors():
    starts = np.array([0, 256, 640], np.uint32)
    lens = np.array([256, 384, 128], np.uint32)
    a = orc.s1_windows(starts, lens, [0, 3], [1, 1, 1], 128, 0)
    b = orc.s1_windows(starts, lens, [0, 3], [1, 1, 1], 128, 1)
    assert np.array_equal(a[0], b[0]) and a[0].tolist() == [0, 128, 256, 384, 512, 640]


def drifted_case(seed, W=128, anchor=1, n_shared=6):
    """A pool stream registered as chunks AND as their windows; a request in which runs of
    consecutive pool chunks follow fresh text that does NOT end on a cut."""
    rng = np.random.default_rng(seed)
    mask, lo, hi = 0xFF, 64, 1024
    pool = rng.integers(0, 102400, 40000).astype(np.int32)
    ps, pl, _ = orc.cdc_chunk(pool, [0, len(pool)], GEAR, mask, lo, hi)
    p_pos = rng.integers(0, 30000, len(ps)).astype(np.int32)
    parts, planted = [], []
    cur = 0
    for _ in range(n_shared):
        fresh = rng.integers(0, 102400, int(rng.integers(200, 900))).astype(np.int32)
        c0 = int(rng.integers(0, len(ps) - 4))
        run = pool[ps[c0]:ps[c0 + 3]]                                      # three consecutive pool chunks
        parts += [fresh, run]
        planted.append((cur + len(fresh), int(ps[c0]), len(run)))          # (request token, pool token, length)
        cur += len(fresh) + len(run)
    tokens = np.concatenate(parts)
    off = np.array([0, len(tokens)], np.uint32)
    st, ln, rco = orc.cdc_chunk(tokens, off, GEAR, mask, lo, hi)
    # registry: pool chunks, then the windows of every pool chunk
    ch_pool = orc.chunk_hash(pool, ps, pl)
    pws, pwl, pwp, _ = orc.s1_windows(ps, pl, [0, len(ps)], np.ones(len(ps), bool), W, anchor)
    wh_pool = orc.chunk_hash(pool, pws, pwl)
    reg = dict(hash=np.concatenate([ch_pool, wh_pool]),
               src_row=np.concatenate([ps, pws]).astype(np.uint32),
               p_src=np.concatenate([p_pos, p_pos[pwp] + (pws - ps[pwp]).astype(np.int32)]).astype(np.int32),
               len=np.concatenate([pl, pwl]).astype(np.uint32),
               entry_id=np.arange(len(ps) + len(pws), dtype=np.uint32))
    return dict(pool=pool, tokens=tokens, off=off, st=st, ln=ln, rco=rco, reg=reg, planted=planted, W=W,
                anchor=anchor, pos_base=np.array([0], np.int32))


def s1_pipeline(d, carve_out=32):
    reg = d["reg"]
    ch = orc.chunk_hash(d["tokens"], d["st"], d["ln"])
    entry, hits, hit_tokens = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"], ch,
                                         d["st"], d["ln"], d["rco"], d["off"], d["pos_base"], carve_out)
    ws, wln, wp, rwo = orc.s1_windows(d["st"], d["ln"], d["rco"], entry < 0, d["W"], d["anchor"])
    wh = orc.chunk_hash(d["tokens"], ws, wln)
    wentry, whits, wtok = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"], reg["entry_id"], wh,
                                     ws, wln, rwo, d["off"], d["pos_base"], carve_out)
    return entry, hits, hit_tokens, ws, wentry, whits, wtok


@pytest.mark.parametrize("anchor", [0, 1])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_window_hits_are_exactly_the_windows_whose_content_is_registered(seed, anchor):
    """No hash on the checking side: a window must hit iff its 128 tokens equal the tokens of
    some registered window, the first registered one gives rows and delta."""
    d = drifted_case(seed, anchor=anchor)
    entry, hits, _, ws, wentry, whits, wtok = s1_pipeline(d)
    reg, pool, tokens, W = d["reg"], d["pool"], d["tokens"], d["W"]
    is_win = reg["len"] == W
    by_content = {}
    for k in np.nonzero(is_win)[0]:                                        # registered 128-token contents
        by_content.setdefault(pool[reg["src_row"][k]:reg["src_row"][k] + W].tobytes(), int(k))
    want = []
    for s in ws:
        k = by_content.get(tokens[s:s + W].tobytes())
        if k is not None and s >= 32:
            want.append((int(reg["src_row"][k]), int(s), W, int(s) - int(reg["p_src"][k])))
    got = list(zip(whits.src_row.tolist(), whits.dst_tok.tolist(), whits.len.tolist(), whits.delta.tolist()))
    assert got == want and wtok == W * len(want)
    assert np.array_equal(wentry >= 0, np.isin(ws, [w[1] for w in want]))


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_end_anchored_windows_recover_a_shared_region_behind_unaligned_text(seed):
    d = drifted_case(seed, anchor=1)
    entry, hits, hit_tokens, ws, wentry, whits, wtok = s1_pipeline(d)
    pool, tokens = d["pool"], d["tokens"]
    # every re-attached row, from chunks or windows, carries the KV of an identical token
    for h in (hits, whits):
        for sr, dt, l in zip(h.src_row.astype(np.int64), h.dst_tok.astype(np.int64), h.len.astype(np.int64)):
            assert np.array_equal(pool[sr:sr + l], tokens[dt:dt + l])
    shared = sum(l for _, _, l in d["planted"])
    covered = np.zeros(len(tokens), bool)
    for h in (hits, whits):
        for dt, l in zip(h.dst_tok.astype(np.int64), h.len.astype(np.int64)):
            assert not covered[dt:dt + l].any()                            # chunk hits and window hits never overlap
            covered[dt:dt + l] = True
    in_shared = np.zeros(len(tokens), bool)
    for t, _, l in d["planted"]:
        in_shared[t:t + l] = True
    assert not covered[~in_shared].any()                                   # fresh text is never served
    chunk_only = int(hits.len.sum())
    assert wtok > 0 and chunk_only + wtok <= shared
    # The chunk that straddles fresh text and shared text is lost to whole-chunk lookup.  When it
    # ends where the first shared pool chunk ends (a content-defined cut; it may also end earlier,
    # on a candidate the pool's chunking had to skip for the minimum length), windows counted from
    # its end line up with the pool's, and every whole window inside the shared part is recovered.
    pool_len_at = dict(zip(d["reg"]["src_row"][d["reg"]["len"] != d["W"]].tolist(),
                           d["reg"]["len"][d["reg"]["len"] != d["W"]].tolist()))
    straddlers = aligned_ends = 0
    for t, p, l in d["planted"]:
        c = np.searchsorted(d["st"], t, side="right") - 1                  # request chunk that holds token t
        if d["st"][c] < t:                                                 # it starts in the fresh text
            straddlers += 1
            assert entry[c] < 0
            end = int(d["st"][c] + d["ln"][c])
            if end - t == pool_len_at[p]:
                aligned_ends += 1
                n_inside = (end - t) // d["W"]
                assert covered[end - n_inside * d["W"]:end].all()
                assert not covered[d["st"][c]:end - n_inside * d["W"]].any()
    assert straddlers >= 3 and aligned_ends >= 1
