"""Seeded synthetic inputs for the re-attachment path.

This module serves both the GPU library's callers and the CPU oracle's tests,
so it holds NONE of the method's arithmetic: chunking and fingerprinting are
handed in as callables (``chunker``), and everything here is drawing random
numbers, slicing and concatenating.  It imports neither the GPU binding nor
the oracle.

The inputs stand in for agentic serving traffic in which a shared region (a
tool schema, a retrieved document, a system prompt behind per-agent metadata)
re-appears in a later prompt at a shifted absolute position (paper Sec. 1,
Sec. 3).  A *pool* stream is chunked once; its chunks are the cached content.
A *request* is a random sequence of whole pool chunks and of whole chunks of a
separate fresh stream.  Because every such piece ends on a boundary that
depends only on its own trailing tokens, the request re-chunks into exactly
the pieces it was assembled from -- the synthetic counterpart of the 64-token
boundary marker that pins shared regions in the paper (App. G, strategy S2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Optional

import numpy as np

# ---------------------------------------------------------------------------
# Method parameters that are *inputs* of the library (tables, frequencies).
# ---------------------------------------------------------------------------

GEAR_SEED = 0x49524D494E53554C  # "IRMINSUL"
_M64 = (1 << 64) - 1


def gear_table(seed: int = GEAR_SEED) -> np.ndarray:
    """256 pseudo-random uint32: the k-th SplitMix64 output, truncated to 32 bits."""
    out = np.zeros(256, np.uint32)
    state = seed & _M64
    for k in range(256):
        state = (state + 0x9E3779B97F4A7C15) & _M64
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
        z = z ^ (z >> 31)
        out[k] = z & 0xFFFFFFFF
    return out


def inv_freq_plain(theta: float = 10000.0, dim: int = 64) -> np.ndarray:
    """theta^(-2i/dim), i < dim/2, computed in fp64 and rounded once to fp32."""
    i = np.arange(dim // 2, dtype=np.float64)
    return (theta ** (-2.0 * i / dim)).astype(np.float32)


def inv_freq_yarn(theta: float = 10000.0, scale: float = 40.0, original_ctx: int = 4096,
                  beta_fast: float = 32.0, beta_slow: float = 1.0, dim: int = 64) -> np.ndarray:
    """YaRN "NTK-by-parts" inverse frequencies (the DeepSeek-V2/V3-form rotary).

    Dimensions that turn more than beta_fast times inside the original context
    keep their frequency, those that turn fewer than beta_slow times are divided
    by ``scale``, and a linear ramp blends between.  No magnitude factor is part
    of the frequencies."""
    def corr_dim(n_rot):
        return dim * np.log(original_ctx / (n_rot * 2.0 * np.pi)) / (2.0 * np.log(theta))
    low = max(int(np.floor(corr_dim(beta_fast))), 0)
    high = min(int(np.ceil(corr_dim(beta_slow))), dim - 1)
    i = np.arange(dim // 2, dtype=np.float64)
    extrapolated = theta ** (-2.0 * i / dim)
    interpolated = extrapolated / scale
    span = max(high - low, 1e-3)
    ramp = np.clip((i - low) / span, 0.0, 1.0)
    return ((1.0 - ramp) * extrapolated + ramp * interpolated).astype(np.float32)


# ---------------------------------------------------------------------------
# Workload container
# ---------------------------------------------------------------------------

# chunker(tokens int32[N], req_offsets uint32[R+1], gear, mask, min_chunk, max_chunk)
#   -> (chunk_start uint32[C], chunk_len uint32[C], req_chunk_offsets uint32[R+1])
Chunker = Callable[..., tuple]


@dataclass
class Workload:
    name: str
    n_layers: int
    # CDC / lookup / rotation parameters
    gear: np.ndarray
    mask: int
    min_chunk: int
    max_chunk: int
    carve_out: int
    inv_freq: np.ndarray
    # cached content: source pool row r holds the KV of pool_tokens[r]
    pool_tokens: np.ndarray
    pool_chunk_start: np.ndarray
    pool_chunk_len: np.ndarray
    pool_p_src: np.ndarray            # position each cached chunk was computed at
    # extra registry entries that only load the table (random keys, never matched)
    n_filler: int
    filler_seed: int
    table_slots: int
    # request batch
    tokens: np.ndarray
    req_offsets: np.ndarray
    pos_base: np.ndarray
    dst_slots: np.ndarray
    # how the requests were assembled: piece start (global token index), length,
    # pool chunk index or -1 for fresh content
    piece_start: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    piece_len: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    piece_pool_chunk: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))

    @property
    def src_rows(self) -> int:
        return int(len(self.pool_tokens))

    @property
    def dst_rows(self) -> int:
        return int(len(self.tokens))

    @property
    def n_req(self) -> int:
        return int(len(self.req_offsets) - 1)

    def chunk_capacity(self) -> int:
        n = np.diff(self.req_offsets.astype(np.int64))
        return int((n // self.min_chunk + 1).sum())

    def filler_keys(self) -> np.ndarray:
        rng = np.random.default_rng(self.filler_seed)
        return rng.integers(1, 1 << 63, size=self.n_filler, dtype=np.uint64) * np.uint64(2) + np.uint64(1)

    def registry(self, pool_hashes: np.ndarray):
        """Registry entry list in insertion order: the pool's chunks, then fillers.

        ``pool_hashes`` are the fingerprints of the pool chunks (computed by the
        caller with whichever implementation it is exercising).
        -> dict of arrays hash u64, src_row u32, p_src i32, len u32, entry_id u32."""
        n_pool = len(self.pool_chunk_start)
        assert len(pool_hashes) == n_pool
        n = n_pool + self.n_filler
        h = np.empty(n, np.uint64)
        h[:n_pool] = pool_hashes
        src_row = np.zeros(n, np.uint32)
        src_row[:n_pool] = self.pool_chunk_start
        p_src = np.zeros(n, np.int32)
        p_src[:n_pool] = self.pool_p_src
        ln = np.full(n, self.min_chunk, np.uint32)
        ln[:n_pool] = self.pool_chunk_len
        if self.n_filler:
            h[n_pool:] = self.filler_keys()
        return dict(hash=h, src_row=src_row, p_src=p_src, len=ln,
                    entry_id=np.arange(n, dtype=np.uint32))

    def window_registry(self, win_start, win_len, win_parent, win_hash, first_id: int):
        """Registry entries of fixed windows cut from the pool's chunks (the caller made the
        window list and its fingerprints with the implementation it is exercising): a window
        keeps the rows of its tokens and the position its parent chunk gives it."""
        win_start = np.asarray(win_start, np.int64)
        parent = np.asarray(win_parent, np.int64)
        off = win_start - self.pool_chunk_start[parent].astype(np.int64)
        n = len(win_start)
        return dict(hash=np.asarray(win_hash, np.uint64), src_row=win_start.astype(np.uint32),
                    p_src=(self.pool_p_src[parent].astype(np.int64) + off).astype(np.int32),
                    len=np.asarray(win_len, np.uint32),
                    entry_id=(first_id + np.arange(n)).astype(np.uint32))

    def expected_hits(self):
        """Pieces that were planted from the pool and lie past the carve-out:
        (dst_tok, len, pool_chunk, delta) -- what a correct pipeline must find,
        provided no two pool chunks hold the same tokens."""
        req_of = np.searchsorted(self.req_offsets.astype(np.int64), self.piece_start, side="right") - 1
        pos = self.pos_base[req_of].astype(np.int64) + self.piece_start - self.req_offsets[req_of].astype(np.int64)
        keep = (self.piece_pool_chunk >= 0) & (pos >= self.carve_out)
        pc = self.piece_pool_chunk[keep]
        return (self.piece_start[keep], self.piece_len[keep], pc,
                pos[keep] - self.pool_p_src[pc].astype(np.int64))


# ---------------------------------------------------------------------------
# Token-id distributions
# ---------------------------------------------------------------------------

def _uniform_ids(rng, n, vocab=102400):
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def _zipf_ids(rng, n, vocab=131072, s=1.1):
    """Zipf(s) truncated to ``vocab`` ranks, id = rank - 1 (inverse-CDF sampling)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    ids = np.searchsorted(cdf, rng.random(n), side="right")
    return np.minimum(ids, vocab - 1).astype(np.int32)


# ---------------------------------------------------------------------------
# Configurations
# ---------------------------------------------------------------------------

# name -> parameters.  "full" sizes follow the five measured configurations;
# "small" keeps the structure (layer count > 1, several requests, ragged tails,
# the same id distribution and rotary) at a size a CPU oracle finishes in seconds.
CONFIGS = {
    "c0": dict(full=dict(n_layers=1, pool=4096), small=dict(n_layers=1, pool=4096)),
    "c1": dict(ids="uniform", rotary="plain", hit=0.8, delta_limit=None,
               full=dict(n_layers=27, pool=262144, n_req=1, req_len=32768),
               small=dict(n_layers=3, pool=16384, n_req=1, req_len=8192)),
    "c2": dict(ids="uniform", rotary="plain", hit=0.9, delta_limit=None,
               full=dict(n_layers=27, pool=2000000, n_req=64, req_len=16384),
               small=dict(n_layers=2, pool=32768, n_req=5, req_len=4099, pos_base=(0, 7, 4096, 0, 12000))),
    "c3": dict(ids="uniform", rotary="yarn", hit=0.9, delta_limit=100000,
               full=dict(n_layers=27, pool=262144, n_req=1, req_len=131072),
               small=dict(n_layers=2, pool=32768, n_req=1, req_len=16384, pos_base=(100000,))),
    "c4": dict(ids="zipf", rotary="plain", hit=0.8, delta_limit=None,
               full=dict(n_layers=61, pool=524288, n_req=32, req_len=65536, entries=4194304),
               small=dict(n_layers=3, pool=16384, n_req=3, req_len=8192, entries=50000)),
}
CONFIG_NAMES = tuple(CONFIGS)
LOAD_FACTOR = 0.7

# CDC rule -> (mask, min_chunk, max_chunk).  "config": the rule the five measured configurations
# state; "paper": the paper's own (Sec. 7.2 "CDC boundary rule", App. B): low 7 bits, 32..512 tokens.
CDC_RULES = {"config": (0xFF, 64, 1024), "paper": (0x7F, 32, 512)}


def _seeds(name, variant):
    k = CONFIG_NAMES.index(name)
    return 1000 + k, 2000 + k + 100 * variant, 3000 + k


def kv_seed(name: str) -> int:
    return _seeds(name, 0)[2]


def make_workload(name: str, chunker: Chunker, size: str = "full", variant: int = 0,
                  slots: str = "contiguous", assembly: str = "aligned", s1_window: int = 0,
                  cdc: str = "config") -> Workload:
    """Build configuration ``name`` ("c0".."c4").

    ``assembly`` "aligned" (default): every piece of a request ends on a cut, so the request
    re-chunks into its pieces.  "unaligned": every fresh piece but the last loses 1..63 of its
    trailing tokens, so the pool chunk that follows it starts off a cut and its first chunk
    drifts (traffic whose assembly the operator does not control).  ``s1_window`` > 0 sizes the
    table for the pool's fixed windows as well (``window_registry``).

    ``cdc`` picks the chunking rule from ``CDC_RULES`` (same seeds, so the same token streams).

    ``variant`` re-draws the request batch against the same pool (used to cycle
    through several batches while timing).  ``slots`` is "contiguous" (request
    token t lands in destination row t) or "permuted" (a random permutation of
    the destination rows: worst-case scatter)."""
    spec = CONFIGS[name]
    dims = spec[size]
    pool_seed, req_seed, _ = _seeds(name, variant)
    gear = gear_table()
    (mask, min_chunk, max_chunk), carve_out = CDC_RULES[cdc], 32
    rng_pool = np.random.default_rng(pool_seed)
    rng = np.random.default_rng(req_seed)

    def chunk_stream(toks):
        off = np.array([0, len(toks)], np.uint32)
        st, ln, _ = chunker(toks, off, gear, mask, min_chunk, max_chunk)
        return np.asarray(st, np.int64), np.asarray(ln, np.int64)

    if name == "c0":
        return _make_c0(dims, chunk_stream, gear, mask, min_chunk, max_chunk, carve_out,
                        rng_pool, rng, slots)

    draw = _uniform_ids if spec["ids"] == "uniform" else _zipf_ids
    inv_freq = inv_freq_plain() if spec["rotary"] == "plain" else inv_freq_yarn()
    n_req, req_len, hit = dims["n_req"], dims["req_len"], spec["hit"]

    pool_tokens = draw(rng_pool, dims["pool"])
    p_start, p_len = chunk_stream(pool_tokens)
    usable_pool = np.arange(len(p_start) - 1)            # the stream's tail chunk is not a whole piece
    pool_p_src = rng_pool.integers(0, req_len, size=len(p_start)).astype(np.int32)

    n_fresh = int((1.0 - hit) * n_req * req_len) + n_req * 2 * max_chunk + 4 * max_chunk
    fresh_tokens = draw(rng, n_fresh)
    f_start, f_len = chunk_stream(fresh_tokens)
    fresh_next = 0
    n_fresh_usable = len(f_start) - 1
    if assembly == "unaligned":
        f_len = f_len - rng.integers(1, min_chunk, size=len(f_len))
    elif assembly != "aligned":
        raise ValueError(assembly)

    toks, piece_start, piece_len, piece_pc = [], [], [], []
    req_offsets = [0]
    cursor = 0
    for _ in range(n_req):
        # pool pieces: distinct chunks in random order up to the hit share
        order = rng.permutation(usable_pool)
        target = hit * req_len
        chosen, acc = [], 0
        for c in order:
            if acc + p_len[c] > target:
                break
            chosen.append(int(c))
            acc += int(p_len[c])
        # fresh pieces: whole chunks until the request is full; the last one is cut short
        fresh, total = [], acc
        while total < req_len:
            if fresh_next >= n_fresh_usable:
                raise RuntimeError("fresh stream exhausted")
            fresh.append(fresh_next)
            total += int(f_len[fresh_next])
            fresh_next += 1
        last_fresh = fresh.pop()
        pieces = [("p", c) for c in chosen] + [("f", c) for c in fresh]
        pieces = [pieces[k] for k in rng.permutation(len(pieces))] + [("f", last_fresh)]
        room = req_len
        for kind, c in pieces:
            if kind == "p":
                seg = pool_tokens[p_start[c]:p_start[c] + p_len[c]]
            else:
                seg = fresh_tokens[f_start[c]:f_start[c] + f_len[c]]
            seg = seg[:room]
            toks.append(seg)
            piece_start.append(cursor)
            piece_len.append(len(seg))
            piece_pc.append(c if kind == "p" else -1)
            cursor += len(seg)
            room -= len(seg)
        assert room == 0
        req_offsets.append(cursor)

    tokens = np.concatenate(toks).astype(np.int32)
    piece_start = np.array(piece_start, np.int64)
    piece_len = np.array(piece_len, np.int64)
    piece_pc = np.array(piece_pc, np.int64)
    req_offsets = np.array(req_offsets, np.uint32)
    pos_base = np.array(dims.get("pos_base", (0,) * n_req), np.int32)
    assert len(pos_base) == n_req

    limit = spec["delta_limit"]
    if limit is not None:
        # single request: each pool chunk is placed at most once, so its stored
        # position can be drawn after placement to give |delta| <= limit
        assert n_req == 1
        for s, c in zip(piece_start, piece_pc):
            if c >= 0:
                pos = int(pos_base[0]) + int(s)
                pool_p_src[c] = rng.integers(max(0, pos - limit), pos + limit + 1)

    entries = dims.get("entries")
    n_filler = max(0, entries - len(p_start)) if entries else 0
    n_entries = len(p_start) + n_filler + (len(pool_tokens) // s1_window if s1_window else 0)
    table_slots = int(np.ceil(max(n_entries, 1) / LOAD_FACTOR))

    return Workload(
        name=f"{name}-{size}", n_layers=dims["n_layers"], gear=gear, mask=mask,
        min_chunk=min_chunk, max_chunk=max_chunk, carve_out=carve_out, inv_freq=inv_freq,
        pool_tokens=pool_tokens, pool_chunk_start=p_start.astype(np.uint32),
        pool_chunk_len=p_len.astype(np.uint32), pool_p_src=pool_p_src,
        n_filler=n_filler, filler_seed=pool_seed + 7, table_slots=table_slots,
        tokens=tokens, req_offsets=req_offsets, pos_base=pos_base,
        dst_slots=_slots(len(tokens), slots, rng),
        piece_start=piece_start, piece_len=piece_len, piece_pool_chunk=piece_pc)


def _slots(n, kind, rng):
    if kind == "contiguous":
        return np.arange(n, dtype=np.int32)
    if kind == "permuted":
        return rng.permutation(n).astype(np.int32)
    raise ValueError(kind)


def _make_c0(dims, chunk_stream, gear, mask, min_chunk, max_chunk, carve_out, rng_pool, rng, slots):
    """One 4,096-token stream is both pool and request; in the request eight of
    its chunks trade places (re-drawn until every shift is within 2,048)."""
    pool_tokens = _uniform_ids(rng_pool, dims["pool"])
    p_start, p_len = chunk_stream(pool_tokens)
    n_chunks = len(p_start)
    movable = n_chunks - 1                      # the tail chunk stays last
    k = min(8, movable)
    while True:
        order = np.arange(n_chunks)
        sel = np.sort(rng.choice(movable, size=k, replace=False))
        order[sel] = sel[rng.permutation(k)]
        new_start = np.zeros(n_chunks, np.int64)
        new_start[order] = np.concatenate([[0], np.cumsum(p_len[order])[:-1]])
        if k < 2 or (np.any(order != np.arange(n_chunks)) and np.all(np.abs(new_start - p_start) <= 2048)):
            break
    tokens = np.concatenate([pool_tokens[p_start[c]:p_start[c] + p_len[c]] for c in order]).astype(np.int32)
    piece_start = np.concatenate([[0], np.cumsum(p_len[order])[:-1]]).astype(np.int64)
    return Workload(
        name="c0", n_layers=dims["n_layers"], gear=gear, mask=mask, min_chunk=min_chunk,
        max_chunk=max_chunk, carve_out=carve_out, inv_freq=inv_freq_plain(),
        pool_tokens=pool_tokens, pool_chunk_start=p_start.astype(np.uint32),
        pool_chunk_len=p_len.astype(np.uint32), pool_p_src=p_start.astype(np.int32),
        n_filler=0, filler_seed=0, table_slots=int(np.ceil(n_chunks / LOAD_FACTOR)),
        tokens=tokens, req_offsets=np.array([0, len(tokens)], np.uint32),
        pos_base=np.zeros(1, np.int32), dst_slots=_slots(len(tokens), slots, rng),
        piece_start=piece_start, piece_len=p_len[order].astype(np.int64),
        piece_pool_chunk=order.astype(np.int64))


# ---------------------------------------------------------------------------
# KV values
# ---------------------------------------------------------------------------

SENTINEL_BF16 = 0x7FC1   # a NaN pattern no rotation or copy of N(0,1) data produces


def kv_pool_torch(n_layers: int, rows: int, seed: int, device="cpu", layers_per_step: int = 1):
    """[n_layers][rows][576] bf16 ~ N(0,1), generated on ``device`` a few layers at a time."""
    import torch
    out = torch.empty((n_layers, rows, 576), dtype=torch.bfloat16, device=device)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    for l0 in range(0, n_layers, layers_per_step):
        l1 = min(n_layers, l0 + layers_per_step)
        out[l0:l1].normal_(0.0, 1.0, generator=g)
    return out


def kv_pool_fp8_torch(n_layers: int, rows: int, seed: int, device="cpu", layers_per_step: int = 1,
                      codes: str = "random"):
    """fp8 rows as [n_layers][rows][328] 16-bit words (typed bf16 like the other pools): 512 bytes of
    E4M3 codes, four fp32 block scales, then k_r as 64 bf16 ~ N(0,1).
    codes="random": uniformly random bytes (NaN codes included) and scales in [1e-3, 4): whoever
    moves the 528 bytes bit for bit can be given anything.
    codes="quantised": c_KV ~ N(0,1) quantised per block of 128 by the library type (scale =
    block maximum / 448, codes by torch's float8_e4m3fn cast): what a reader that dequantises needs."""
    import torch
    assert codes in ("random", "quantised")
    out = torch.empty((n_layers, rows, 328), dtype=torch.int16, device=device)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    for l0 in range(0, n_layers, layers_per_step):
        l1 = min(n_layers, l0 + layers_per_step)
        if codes == "random":
            c = torch.randint(0, 65536, (l1 - l0, rows, 256), generator=g, device=device, dtype=torch.int32)
            out[l0:l1, :, :256] = (c - 32768).to(torch.int16)
            scales = torch.empty((l1 - l0, rows, 4), dtype=torch.float32, device=device).uniform_(1e-3, 4.0, generator=g)
        else:
            v = torch.empty((l1 - l0, rows, 4, 128), dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=g)
            scales = v.abs().amax(dim=3) / 448.0
            q = (v / scales[..., None]).to(torch.float8_e4m3fn)
            out[l0:l1, :, :256] = q.view(torch.uint8).reshape(l1 - l0, rows, 512).view(torch.int16)
            del v, q
        out[l0:l1, :, 256:264] = scales.view(torch.int16)
        kr = torch.empty((l1 - l0, rows, 64), dtype=torch.bfloat16, device=device).normal_(0.0, 1.0, generator=g)
        out[l0:l1, :, 264:] = kr.view(torch.int16)
    return out.view(torch.bfloat16)


def sentinel_pool_torch(n_layers: int, rows: int, device="cpu", row_words: int = 576):
    import torch
    out = torch.empty((n_layers, rows, row_words), dtype=torch.int16, device=device)
    out.fill_(SENTINEL_BF16 - 0x10000 if SENTINEL_BF16 >= 0x8000 else SENTINEL_BF16)
    return out.view(torch.bfloat16)
