"""Pins for the oracle's gear-hash CDC (paper Sec. 4, Sec. 7.2 "CDC boundary rule", App. B).

The oracle walks a rolling state token by token.  It is pinned here to things
that are not that loop: a windowed closed form plus a set-minimum search
(brute force), the structural invariants of min/max-clamped CDC, position
independence after a flushed window (App. G), the expected chunk-length law
(App. B: about 2^k tokens, clamped), and independence from the state width.
"""
import itertools

import numpy as np
import pytest

from oracle import irm_oracle as orc
from paper_2605_05696_amd import workloads as wl


def brute_force_chunks(tokens, gear, mask, min_chunk, max_chunk):
    """Boundaries of ONE request from first principles.

    Closed form of the masked state: with a shift-by-one gear hash and a k-bit
    mask only the last k tokens can influence the masked value,
        h_i & mask = ( sum_{j<k} G[x_{i-j}] << j ) & mask,
    (terms before the start of the request are absent).  A chunk that starts at
    s ends at the smallest member of
        {i >= s+min-1 : candidate(i)}  U  {s+max-1}  U  {n-1}."""
    n = len(tokens)
    k = int(mask).bit_length()
    assert mask == (1 << k) - 1
    g = [int(gear[int(t) & 0xFF]) for t in tokens]
    cand = set()
    for i in range(n):
        acc = 0
        for j in range(k):
            if i - j >= 0:
                acc += g[i - j] << j
        if acc & mask == 0:
            cand.add(i)
    out, s = [], 0
    while s < n:
        options = {i for i in cand if i >= s + min_chunk - 1} | {s + max_chunk - 1, n - 1}
        e = min(options)
        out.append((s, e - s + 1))
        s = e + 1
    return out


def oracle_chunks(tokens, gear, mask, lo, hi, req_offsets=None):
    tokens = np.asarray(tokens, np.int32)
    if req_offsets is None:
        req_offsets = [0, len(tokens)]
    st, ln, rco = orc.cdc_chunk(tokens, np.asarray(req_offsets, np.uint32), gear, mask, lo, hi)
    return list(zip(st.tolist(), ln.tolist())), rco


def test_brute_force_all_short_streams_over_three_symbols():
    # every stream of length 1..10 over 3 symbols, tiny parameters (window 2 <= min 2)
    rng = np.random.default_rng(5)
    gear = rng.integers(0, 1 << 32, size=256, dtype=np.uint64).astype(np.uint32)
    n_cut_content = 0
    for n in range(1, 11):
        for stream in itertools.product((0, 1, 2), repeat=n):
            got, _ = oracle_chunks(stream, gear, 0x3, 2, 5)
            want = brute_force_chunks(stream, gear, 0x3, 2, 5)
            assert got == want, (stream, got, want)
            n_cut_content += sum(1 for (_, l) in got[:-1] if l < 5)
    assert n_cut_content > 1000  # the content rule was really exercised


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_real_parameters(seed):
    rng = np.random.default_rng(seed)
    gear = wl.gear_table()
    tokens = rng.integers(0, 102400, size=4096).astype(np.int32)
    got, _ = oracle_chunks(tokens, gear, 0xFF, 64, 1024)
    assert got == brute_force_chunks(tokens, gear, 0xFF, 64, 1024)


def test_brute_force_other_masks_and_clamps():
    rng = np.random.default_rng(11)
    gear = wl.gear_table(seed=77)
    tokens = rng.integers(0, 1 << 20, size=3000).astype(np.int32)
    for mask, lo, hi in [(0x7F, 32, 512), (0x1, 1, 3), (0xFFFF, 16, 100), (0x0, 4, 9), (0xF, 4, 4)]:
        got, _ = oracle_chunks(tokens, gear, mask, lo, hi)
        assert got == brute_force_chunks(tokens, gear, mask, lo, hi), (mask, lo, hi)


def test_invariants_tiling_clamps_and_first_candidate():
    rng = np.random.default_rng(3)
    gear = wl.gear_table()
    lens = [1, 63, 64, 65, 1024, 1025, 5000, 0, 20000]
    tokens = rng.integers(0, 102400, size=sum(lens)).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    chunks, rco = oracle_chunks(tokens, gear, 0xFF, 64, 1024, off)
    assert rco[0] == 0 and rco[-1] == len(chunks)
    for r, n in enumerate(lens):
        mine = chunks[rco[r]:rco[r + 1]]
        # exact tiling of the request, in order, no empty chunk
        pos = int(off[r])
        for (s, l) in mine:
            assert s == pos and l >= 1
            pos += l
        assert pos == int(off[r + 1])
        # rolling state restarted per request: recompute it here
        h, states = 0, {}
        for i in range(int(off[r]), int(off[r + 1])):
            h = ((h << 1) + int(gear[int(tokens[i]) & 0xFF])) & 0xFFFFFFFF
            states[i] = h
        for idx, (s, l) in enumerate(mine):
            last = idx == len(mine) - 1
            assert l <= 1024
            if not last:
                assert l >= 64
            if not last and l < 1024:
                assert states[s + l - 1] & 0xFF == 0           # ends on a candidate
            # no earlier eligible candidate was skipped
            for i in range(s + 63, s + l - 1):
                assert states[i] & 0xFF != 0
    assert len(chunks[rco[7]:rco[8]]) == 0                      # empty request -> no chunk


def test_position_independence_after_a_cut():
    """Identical content that starts right after a boundary is chunked identically
    whatever precedes it (App. G: a flushed window gives identical boundaries)."""
    rng = np.random.default_rng(9)
    gear = wl.gear_table()
    x = rng.integers(0, 102400, size=6000).astype(np.int32)
    cx, _ = oracle_chunks(x, gear, 0xFF, 64, 1024)
    whole = sum(l for _, l in cx[:-1])            # X up to its last interior cut
    x = x[:whole]
    cx, _ = oracle_chunks(x, gear, 0xFF, 64, 1024)
    for seed, n_prefix in [(1, 3000), (2, 5555)]:
        a = np.random.default_rng(seed).integers(0, 102400, size=n_prefix).astype(np.int32)
        ca, _ = oracle_chunks(a, gear, 0xFF, 64, 1024)
        a = a[:sum(l for _, l in ca[:-1])]        # prefix that ends on a cut
        cat, _ = oracle_chunks(np.concatenate([a, x]), gear, 0xFF, 64, 1024)
        inside = [(s - len(a), l) for (s, l) in cat if s >= len(a)]
        assert inside == cx


def test_misaligned_content_does_drift():
    """Negative control (App. E: without alignment the boundaries diverge): the same
    content behind a prefix that does NOT end on a cut may start with a different
    chunk, but re-synchronises at a later candidate."""
    rng = np.random.default_rng(21)
    gear = wl.gear_table()
    x = rng.integers(0, 102400, size=8000).astype(np.int32)
    cx, _ = oracle_chunks(x, gear, 0xFF, 64, 1024)
    a = rng.integers(0, 102400, size=100).astype(np.int32)
    cat, _ = oracle_chunks(np.concatenate([a, x]), gear, 0xFF, 64, 1024)
    own = set(cx)
    behind_prefix = {(s - len(a), l) for s, l in cat}
    assert cx[0] not in behind_prefix            # the first chunk of the content is lost
    assert len(own & behind_prefix) >= 3         # later chunks are found again


def test_chunk_length_statistics_uniform_ids():
    """App. B: expected chunk length is about 2^k tokens, clamped.  With ideal
    1/256 candidates the length is 64 + a geometric(1/256) wait cut off at 1024:
    mean = 64 + 255*(1 - q^960) = 313.1 with q = 255/256, P(len = 1024) = q^960
    = 2.3 %.  A single gear table is biased (its low bits are not exactly
    balanced), so the law is checked on the average over 32 random tables; the
    spread between tables sets the tolerance (about 3 standard errors)."""
    means, p_max = [], []
    for seed in range(32):
        rng = np.random.default_rng(seed)
        gear = rng.integers(0, 1 << 32, size=256, dtype=np.uint64).astype(np.uint32)
        tokens = rng.integers(0, 102400, size=400_000).astype(np.int32)
        chunks, _ = oracle_chunks(tokens, gear, 0xFF, 64, 1024)
        ln = np.array([l for _, l in chunks[:-1]], np.float64)
        means.append(ln.mean())
        p_max.append((ln == 1024).mean())
    q = 255.0 / 256.0
    assert abs(np.mean(means) - (64.0 + 255.0 * (1.0 - q ** 960))) < 10.0
    assert abs(np.mean(p_max) - q ** 960) < 0.004


def test_state_width_and_high_gear_bits_do_not_matter():
    rng = np.random.default_rng(8)
    gear = wl.gear_table()
    tokens = rng.integers(0, 102400, size=5000).astype(np.int32)
    ref, _ = oracle_chunks(tokens, gear, 0xFF, 64, 1024)
    # 64-bit state, python integers
    out, h, s = [], 0, 0
    for i, t in enumerate(tokens):
        h = ((h << 1) + int(gear[int(t) & 0xFF])) & ((1 << 64) - 1)
        l = i - s + 1
        if (l >= 64 and h & 0xFF == 0) or l == 1024 or i == len(tokens) - 1:
            out.append((s, l))
            s = i + 1
    assert out == ref
    # only the low byte of each gear entry can matter for an 8-bit mask
    low, _ = oracle_chunks(tokens, gear & np.uint32(0xFF), 0xFF, 64, 1024)
    assert low == ref


def test_negative_token_ids_use_their_low_byte():
    gear = wl.gear_table()
    t = np.array([-1, -256, 255, 0] * 50, np.int32)
    got, _ = oracle_chunks(t, gear, 0x3, 2, 7)
    assert got == brute_force_chunks(t, gear, 0x3, 2, 7)


def test_gear_table_is_the_splitmix64_stream():
    # first outputs of SplitMix64 from seed 0 are published with the generator:
    # 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F
    g = wl.gear_table(seed=0)
    assert [int(v) for v in g[:3]] == [0x7B1DCDAF, 0xA1B965F4, 0x8009454F]
    assert len(set(wl.gear_table().tolist())) == 256


def test_equal_clamps_give_the_fixed_block_chunking():
    """min = max = B turns the rule into fixed-size blocks counted from each request's start (the
    fixed-block hashing the paper compares against in Sec. 4): no candidate can cut before B tokens,
    the clamp cuts at B, only a request's tail is shorter.  Content plays no part."""
    rng = np.random.default_rng(12)
    off = np.array([0, 1000, 1000, 1128, 1500], np.uint32)
    for B in (128, 64, 1):
        outs = []
        for gear_seed in (0, 5):
            tokens = rng.integers(0, 102400, 1500).astype(np.int32)
            st, ln, rco = orc.cdc_chunk(tokens, off, wl.gear_table(seed=gear_seed), 0xFF, B, B)
            want_st, want_ln, want_rco = [], [], [0]
            for r in range(4):
                for s in range(int(off[r]), int(off[r + 1]), B):
                    want_st.append(s)
                    want_ln.append(min(B, int(off[r + 1]) - s))
                want_rco.append(len(want_st))
            assert st.tolist() == want_st and ln.tolist() == want_ln and rco.tolist() == want_rco
            outs.append((st, ln))
        assert np.array_equal(outs[0][0], outs[1][0])
