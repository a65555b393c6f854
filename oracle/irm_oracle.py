"""ctypes access to the plain CPU oracle (``irm_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the CPU-baseline leg
of the benchmark are the only callers.  This module does argument marshalling
and nothing else; every step of the method is in the C file.  It imports
nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "irm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

ROW_DIM = 576
# 16-bit words of a row's position-free part: bf16 rows (512 bf16 c_KV) / fp8 rows (512 e4m3 bytes
# and four fp32 block scales); the 64 bf16 elements of k_r follow
CKV_WORDS_BF16, CKV_WORDS_FP8 = 512, 264


def _ckv_words(row_words: int) -> int:
    assert row_words - KR_DIM in (CKV_WORDS_BF16, CKV_WORDS_FP8), "rows are 576 (bf16) or 328 (fp8) words"
    return row_words - KR_DIM
CKV_DIM = 512
KR_DIM = 64


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.oracle_cdc_chunk.restype = ctypes.c_int64
        L.oracle_fnv1a64_bytes.restype = ctypes.c_uint64
        L.oracle_fnv1a64_bytes.argtypes = [ctypes.c_char_p, ctypes.c_uint64]
        L.oracle_lookup.restype = ctypes.c_int
        L.oracle_reattach.restype = ctypes.c_int
        L.oracle_reattach_kr.restype = ctypes.c_int
        L.oracle_admit.restype = ctypes.c_int64
        L.oracle_s1_windows.restype = ctypes.c_int64
        L.oracle_reattach_ref.restype = ctypes.c_int
        L.oracle_bf16_to_f64.restype = ctypes.c_double
        L.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        L.oracle_f64_to_bf16.restype = ctypes.c_uint16
        L.oracle_f64_to_bf16.argtypes = [ctypes.c_double]
        _lib = L
    return _lib


def _arr(x, dtype):
    return np.ascontiguousarray(x, dtype=dtype)


def cdc_chunk(tokens, req_offsets, gear, mask, min_chunk, max_chunk):
    """-> (chunk_start u32[C], chunk_len u32[C], req_chunk_offsets u32[R+1])."""
    tokens = _arr(tokens, np.int32)
    req_offsets = _arr(req_offsets, np.uint32)
    gear = _arr(gear, np.uint32)
    assert gear.shape == (256,)
    n_req = len(req_offsets) - 1
    n_tok = int(req_offsets[-1]) if n_req >= 0 and len(req_offsets) else 0
    assert n_tok <= len(tokens)
    cap = n_tok + n_req + 1
    start = np.zeros(cap, np.uint32)
    length = np.zeros(cap, np.uint32)
    rco = np.zeros(n_req + 1, np.uint32)
    n = lib().oracle_cdc_chunk(
        _p(tokens, ctypes.c_int32), _p(req_offsets, ctypes.c_uint32), ctypes.c_uint32(n_req),
        _p(gear, ctypes.c_uint32), ctypes.c_uint32(mask), ctypes.c_uint32(min_chunk),
        ctypes.c_uint32(max_chunk), _p(start, ctypes.c_uint32), _p(length, ctypes.c_uint32),
        _p(rco, ctypes.c_uint32), ctypes.c_uint64(cap))
    if n < 0:
        raise ValueError("oracle_cdc_chunk rejected its arguments")
    return start[:n].copy(), length[:n].copy(), rco


def fnv1a64_bytes(data: bytes) -> int:
    return int(lib().oracle_fnv1a64_bytes(data, len(data)))


def chunk_hash(tokens, chunk_start, chunk_len):
    tokens = _arr(tokens, np.int32)
    chunk_start = _arr(chunk_start, np.uint32)
    chunk_len = _arr(chunk_len, np.uint32)
    out = np.zeros(len(chunk_start), np.uint64)
    lib().oracle_chunk_hash(_p(tokens, ctypes.c_int32), _p(chunk_start, ctypes.c_uint32),
                            _p(chunk_len, ctypes.c_uint32), ctypes.c_uint64(len(chunk_start)),
                            _p(out, ctypes.c_uint64))
    return out


@dataclass
class Hits:
    """Struct-of-arrays hit list, ascending chunk order."""
    src_row: np.ndarray   # u32, first row of the cached chunk in the source pool
    dst_tok: np.ndarray   # u32, first token of the request chunk (index into dst_slots)
    len: np.ndarray       # u32
    delta: np.ndarray     # i32, new position - stored position

    def __len__(self):
        return len(self.src_row)


def lookup(reg_hash, reg_src_row, reg_p_src, reg_len, reg_entry_id, chunk_hash_, chunk_start,
           chunk_len, req_chunk_offsets, req_offsets, pos_base, carve_out):
    """-> (chunk_entry i32[C], Hits, hit_tokens)."""
    reg_hash = _arr(reg_hash, np.uint64)
    reg_src_row = _arr(reg_src_row, np.uint32)
    reg_p_src = _arr(reg_p_src, np.int32)
    reg_len = _arr(reg_len, np.uint32)
    reg_entry_id = _arr(reg_entry_id, np.uint32)
    chunk_hash_ = _arr(chunk_hash_, np.uint64)
    chunk_start = _arr(chunk_start, np.uint32)
    chunk_len = _arr(chunk_len, np.uint32)
    rco = _arr(req_chunk_offsets, np.uint32)
    req_offsets = _arr(req_offsets, np.uint32)
    pos_base = _arr(pos_base, np.int32)
    n_req = len(req_offsets) - 1
    C = len(chunk_hash_)
    entry = np.full(C, -1, np.int32)
    h_src = np.zeros(C, np.uint32)
    h_dst = np.zeros(C, np.uint32)
    h_len = np.zeros(C, np.uint32)
    h_delta = np.zeros(C, np.int32)
    n_hits = ctypes.c_uint32(0)
    hit_tokens = ctypes.c_uint64(0)
    rc = lib().oracle_lookup(
        _p(reg_hash, ctypes.c_uint64), _p(reg_src_row, ctypes.c_uint32),
        _p(reg_p_src, ctypes.c_int32), _p(reg_len, ctypes.c_uint32),
        _p(reg_entry_id, ctypes.c_uint32), ctypes.c_uint64(len(reg_hash)),
        _p(chunk_hash_, ctypes.c_uint64), _p(chunk_start, ctypes.c_uint32),
        _p(chunk_len, ctypes.c_uint32), _p(rco, ctypes.c_uint32),
        _p(req_offsets, ctypes.c_uint32), _p(pos_base, ctypes.c_int32), ctypes.c_uint32(n_req),
        ctypes.c_uint32(carve_out), _p(entry, ctypes.c_int32), _p(h_src, ctypes.c_uint32),
        _p(h_dst, ctypes.c_uint32), _p(h_len, ctypes.c_uint32), _p(h_delta, ctypes.c_int32),
        ctypes.byref(n_hits), ctypes.byref(hit_tokens))
    if rc != 0:
        raise MemoryError("oracle_lookup")
    n = n_hits.value
    return entry, Hits(h_src[:n].copy(), h_dst[:n].copy(), h_len[:n].copy(), h_delta[:n].copy()), \
        int(hit_tokens.value)


def bf16_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    b = _arr(bits, np.uint16)
    with np.errstate(invalid="ignore"):          # signalling NaN patterns widen to quiet NaN
        return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bf16(x) -> np.ndarray:
    """Element-wise call of the oracle's single-rounding fp64 -> bf16."""
    x = _arr(x, np.float64)
    f = lib().oracle_f64_to_bf16
    return np.array([f(float(v)) for v in x.ravel()], np.uint16).reshape(x.shape)


def rotate_kr_f64(k, delta, inv_freq, pair_mode=0) -> np.ndarray:
    k = _arr(k, np.float64)
    inv_freq = _arr(inv_freq, np.float32)
    assert k.shape == (KR_DIM,) and inv_freq.shape == (KR_DIM // 2,)
    out = np.zeros(KR_DIM, np.float64)
    lib().oracle_rotate_kr_f64(_p(k, ctypes.c_double), ctypes.c_int64(int(delta)),
                               _p(inv_freq, ctypes.c_float), ctypes.c_uint32(pair_mode),
                               _p(out, ctypes.c_double))
    return out


def reattach_row(row_bits, delta, inv_freq, pair_mode=0) -> np.ndarray:
    row_bits = _arr(row_bits, np.uint16)
    inv_freq = _arr(inv_freq, np.float32)
    assert row_bits.ndim == 1 and inv_freq.shape == (KR_DIM // 2,)
    ckv_words = _ckv_words(len(row_bits))
    out = np.zeros(len(row_bits), np.uint16)
    lib().oracle_reattach_row(_p(row_bits, ctypes.c_uint16), ctypes.c_int32(int(delta)),
                              _p(inv_freq, ctypes.c_float), ctypes.c_uint32(pair_mode),
                              ctypes.c_uint32(ckv_words), _p(out, ctypes.c_uint16))
    return out


def reattach(src_bits, dst_bits, dst_slots, hits: Hits, inv_freq, pair_mode=0) -> None:
    """In place on ``dst_bits``.  src_bits [L][src_rows][W] u16, dst_bits [L][dst_rows][W] u16,
    W = 576 (bf16 rows) or 328 (fp8 rows)."""
    assert src_bits.dtype == np.uint16 and dst_bits.dtype == np.uint16
    assert src_bits.flags.c_contiguous and dst_bits.flags.c_contiguous
    assert src_bits.ndim == 3 and dst_bits.ndim == 3
    assert src_bits.shape[2] == dst_bits.shape[2]
    ckv_words = _ckv_words(src_bits.shape[2])
    assert src_bits.shape[0] == dst_bits.shape[0]
    dst_slots = _arr(dst_slots, np.int32)
    inv_freq = _arr(inv_freq, np.float32)
    assert inv_freq.shape == (KR_DIM // 2,)
    hs, hd = _arr(hits.src_row, np.uint32), _arr(hits.dst_tok, np.uint32)
    hl, hx = _arr(hits.len, np.uint32), _arr(hits.delta, np.int32)
    if len(hs):
        assert int((hd.astype(np.int64) + hl).max()) <= len(dst_slots)
    rc = lib().oracle_reattach(
        _p(src_bits, ctypes.c_uint16), ctypes.c_uint64(src_bits.shape[1]),
        _p(dst_bits, ctypes.c_uint16), ctypes.c_uint64(dst_bits.shape[1]),
        ctypes.c_uint32(src_bits.shape[0]), _p(dst_slots, ctypes.c_int32),
        _p(hs, ctypes.c_uint32), _p(hd, ctypes.c_uint32), _p(hl, ctypes.c_uint32),
        _p(hx, ctypes.c_int32), ctypes.c_uint32(len(hs)), _p(inv_freq, ctypes.c_float),
        ctypes.c_uint32(pair_mode), ctypes.c_uint32(ckv_words))
    if rc != 0:
        raise IndexError("oracle_reattach: a hit or slot points outside its pool")


def reattach_kr(src_bits, kr_bits, ckv_index, dst_slots, hits: Hits, inv_freq, pair_mode=0) -> None:
    """Split-pool variant, in place on ``kr_bits`` [L][kr_rows][64] u16 and ``ckv_index`` i32[kr_rows]."""
    assert src_bits.dtype == np.uint16 and kr_bits.dtype == np.uint16 and ckv_index.dtype == np.int32
    assert src_bits.flags.c_contiguous and kr_bits.flags.c_contiguous and ckv_index.flags.c_contiguous
    assert src_bits.ndim == 3 and kr_bits.ndim == 3 and kr_bits.shape[2] == KR_DIM
    ckv_words = _ckv_words(src_bits.shape[2])
    assert src_bits.shape[0] == kr_bits.shape[0] and len(ckv_index) == kr_bits.shape[1]
    dst_slots = _arr(dst_slots, np.int32)
    inv_freq = _arr(inv_freq, np.float32)
    hs, hd = _arr(hits.src_row, np.uint32), _arr(hits.dst_tok, np.uint32)
    hl, hx = _arr(hits.len, np.uint32), _arr(hits.delta, np.int32)
    if len(hs):
        assert int((hd.astype(np.int64) + hl).max()) <= len(dst_slots)
    rc = lib().oracle_reattach_kr(
        _p(src_bits, ctypes.c_uint16), ctypes.c_uint64(src_bits.shape[1]),
        _p(kr_bits, ctypes.c_uint16), ctypes.c_uint64(kr_bits.shape[1]), _p(ckv_index, ctypes.c_int32),
        ctypes.c_uint32(src_bits.shape[0]), _p(dst_slots, ctypes.c_int32),
        _p(hs, ctypes.c_uint32), _p(hd, ctypes.c_uint32), _p(hl, ctypes.c_uint32),
        _p(hx, ctypes.c_int32), ctypes.c_uint32(len(hs)), _p(inv_freq, ctypes.c_float),
        ctypes.c_uint32(pair_mode), ctypes.c_uint32(ckv_words))
    if rc != 0:
        raise IndexError("oracle_reattach_kr: a hit or slot points outside its pool")


def admit(reg_hash, chunk_hash_, chunk_start, chunk_len, req_chunk_offsets, req_offsets, pos_base,
          carve_out, chunk_entry, req_bits, slots, pool_bits, cursor):
    """Miss path, in place on ``pool_bits``.
    -> (admitted_row i32[C], new registry entries as a dict of arrays, new cursor)"""
    reg_hash = _arr(reg_hash, np.uint64)
    chunk_hash_ = _arr(chunk_hash_, np.uint64)
    chunk_start = _arr(chunk_start, np.uint32)
    chunk_len = _arr(chunk_len, np.uint32)
    rco = _arr(req_chunk_offsets, np.uint32)
    req_offsets = _arr(req_offsets, np.uint32)
    pos_base = _arr(pos_base, np.int32)
    chunk_entry = _arr(chunk_entry, np.int32)
    slots = _arr(slots, np.int32)
    assert req_bits.dtype == np.uint16 and pool_bits.dtype == np.uint16
    assert req_bits.flags.c_contiguous and pool_bits.flags.c_contiguous
    assert req_bits.ndim == 3 and pool_bits.ndim == 3 and req_bits.shape[2] == pool_bits.shape[2]
    ckv_words = _ckv_words(req_bits.shape[2])
    assert req_bits.shape[0] == pool_bits.shape[0]
    C = len(chunk_hash_)
    cur = ctypes.c_uint32(int(cursor))
    admitted = np.full(C, -1, np.int32)
    nh = np.zeros(C, np.uint64)
    ns = np.zeros(C, np.uint32)
    npos = np.zeros(C, np.int32)
    nl = np.zeros(C, np.uint32)
    n = lib().oracle_admit(
        _p(reg_hash, ctypes.c_uint64), ctypes.c_uint64(len(reg_hash)), _p(chunk_hash_, ctypes.c_uint64),
        _p(chunk_start, ctypes.c_uint32), _p(chunk_len, ctypes.c_uint32), _p(rco, ctypes.c_uint32),
        _p(req_offsets, ctypes.c_uint32), _p(pos_base, ctypes.c_int32), ctypes.c_uint32(len(req_offsets) - 1),
        ctypes.c_uint32(carve_out), _p(chunk_entry, ctypes.c_int32), _p(req_bits, ctypes.c_uint16),
        ctypes.c_uint64(req_bits.shape[1]), _p(slots, ctypes.c_int32), _p(pool_bits, ctypes.c_uint16),
        ctypes.c_uint64(pool_bits.shape[1]), ctypes.c_uint32(req_bits.shape[0]), ctypes.byref(cur),
        _p(admitted, ctypes.c_int32), _p(nh, ctypes.c_uint64), _p(ns, ctypes.c_uint32),
        _p(npos, ctypes.c_int32), _p(nl, ctypes.c_uint32), ctypes.c_uint32(ckv_words))
    if n < 0:
        raise IndexError("oracle_admit: a slot points outside the request pool")
    new = dict(hash=nh[:n].copy(), src_row=ns[:n].copy(), p_src=npos[:n].copy(), len=nl[:n].copy(),
               entry_id=ns[:n].copy())
    return admitted, new, int(cur.value)


def s1_windows(chunk_start, chunk_len, req_chunk_offsets, expand, window=128, anchor=0):
    """S1 sub-division of the chunks marked in ``expand`` into fixed windows.
    -> (win_start u32[W], win_len u32[W] (all = window), win_parent u32[W], req_win_offsets u32[R+1])"""
    chunk_start = _arr(chunk_start, np.uint32)
    chunk_len = _arr(chunk_len, np.uint32)
    rco = _arr(req_chunk_offsets, np.uint32)
    expand = np.ascontiguousarray(np.asarray(expand).astype(np.uint8))
    assert len(expand) == len(chunk_start) == len(chunk_len) and window >= 1 and anchor in (0, 1)
    cap = int((chunk_len.astype(np.int64) // window).sum()) + 1
    ws = np.zeros(cap, np.uint32)
    wp = np.zeros(cap, np.uint32)
    rwo = np.zeros(len(rco), np.uint32)
    n = lib().oracle_s1_windows(_p(chunk_start, ctypes.c_uint32), _p(chunk_len, ctypes.c_uint32),
                                _p(rco, ctypes.c_uint32), ctypes.c_uint32(len(rco) - 1),
                                _p(expand, ctypes.c_uint8), ctypes.c_uint32(window), ctypes.c_uint32(anchor),
                                _p(ws, ctypes.c_uint32), _p(wp, ctypes.c_uint32), _p(rwo, ctypes.c_uint32))
    assert 0 <= n < cap + 1
    return ws[:n].copy(), np.full(n, window, np.uint32), wp[:n].copy(), rwo


def reattach_ref(src_rows, row_index, hit_index, dst_slots, hits: Hits, inv_freq) -> np.ndarray:
    """No-materialise variant, in place on ``row_index`` / ``hit_index`` (i32[dst_rows]).
    -> trig f64[n_hits][32][2], the (cos, sin) of every hit's 32 pair angles."""
    assert row_index.dtype == np.int32 and hit_index.dtype == np.int32 and len(row_index) == len(hit_index)
    assert row_index.flags.c_contiguous and hit_index.flags.c_contiguous
    dst_slots = _arr(dst_slots, np.int32)
    inv_freq = _arr(inv_freq, np.float32)
    hs, hd = _arr(hits.src_row, np.uint32), _arr(hits.dst_tok, np.uint32)
    hl, hx = _arr(hits.len, np.uint32), _arr(hits.delta, np.int32)
    if len(hs):
        assert int((hd.astype(np.int64) + hl).max()) <= len(dst_slots)
    trig = np.zeros((len(hs), KR_DIM // 2, 2), np.float64)
    rc = lib().oracle_reattach_ref(
        ctypes.c_uint64(int(src_rows)), _p(row_index, ctypes.c_int32), _p(hit_index, ctypes.c_int32),
        ctypes.c_uint64(len(row_index)), _p(trig, ctypes.c_double), _p(dst_slots, ctypes.c_int32),
        _p(hs, ctypes.c_uint32), _p(hd, ctypes.c_uint32), _p(hl, ctypes.c_uint32), _p(hx, ctypes.c_int32),
        ctypes.c_uint32(len(hs)), _p(inv_freq, ctypes.c_float))
    if rc != 0:
        raise IndexError("oracle_reattach_ref: a hit or slot points outside its pool")
    return trig


def e4m3_to_f64(codes) -> np.ndarray:
    """The 8-bit floating-point format E4M3 in its finite-only form (the one fp8 KV caches use): one
    sign bit, four exponent bits with bias 7, three fraction bits; exponent 0 holds the subnormals
    f/8 * 2^-6; there are no infinities and only S.1111.111 is NaN, so the largest value is 448."""
    c = np.asarray(codes, np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e, f = (c >> 3) & 0xF, c & 0x7
    val = np.where(e == 0, f / 8.0 * 2.0 ** -6, (1.0 + f / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))
    val = np.where((e == 15) & (f == 7), np.nan, val)
    return sign * val


def dequant_fp8_rows(row_bits) -> np.ndarray:
    """fp8 rows [n][328] u16 (512 E4M3 codes | four fp32 scales | 64 bf16 of k_r) -> [n][576] f64:
    c_KV element d = value of code d times the scale of its block of 128, exact in fp64 (an 4-bit
    by 24-bit product); k_r widened from bf16."""
    row_bits = np.ascontiguousarray(row_bits, np.uint16)
    assert row_bits.ndim == 2 and row_bits.shape[1] == CKV_WORDS_FP8 + KR_DIM
    n = row_bits.shape[0]
    codes = row_bits[:, :256].copy().view(np.uint8).reshape(n, 512)            # little-endian byte order
    scales = row_bits[:, 256:264].copy().view(np.float32).reshape(n, 4).astype(np.float64)
    ckv = e4m3_to_f64(codes) * np.repeat(scales, 128, axis=1)
    return np.concatenate([ckv, bf16_to_f64(row_bits[:, 264:])], axis=1)


def attend_ref(q_bits, pool_bits, kv_slots, kv_offsets, row_index, hit_index, trig, scale, pair_mode=0):
    """The consumer of the no-materialise variant: MLA decode attention in the latent ("absorbed")
    form (Sec. 2 "MLA": per token a 512-dim c_KV and a 64-dim RoPE key k_r, V derived from c_KV),
    reading (c_KV, k_r_base) through the references and rotating k_r by the hit's R(delta) as it
    is loaded (Sec. 7.2; App. C).  One layer.  For request b, head h and the request's context
    slots s_0 .. s_{n-1} = kv_slots[kv_offsets[b] : kv_offsets[b+1]]:

        row_t   = row_index[s_t]                      k_t = [ c_KV(row_t) | R_t k_r_base(row_t) ]
        R_t     = rotation of hit hit_index[s_t] from ``trig`` (identity when hit_index < 0)
        score_t = scale * q[b][h] . k_t               p = softmax over t
        out[b][h] = sum_t p_t c_KV(row_t)             lse[b][h] = log sum_t exp(score_t)

    q_bits [B][H][576] and pool_bits [rows][576] are bf16 bit patterns, everything is computed in
    fp64, nothing is rounded.  A request without context gives out = 0, lse = -inf.
    pool_bits may also be [rows][328]: fp8 rows, whose c_KV is read through ``dequant_fp8_rows``.
    -> (out f64 [B][H][512], lse f64 [B][H])"""
    q = bf16_to_f64(np.asarray(q_bits, np.uint16))
    pool_bits = np.asarray(pool_bits, np.uint16)
    kv_slots = np.asarray(kv_slots, np.int64)
    kv_offsets = np.asarray(kv_offsets, np.int64)
    row_index = np.asarray(row_index, np.int64)
    hit_index = np.asarray(hit_index, np.int64)
    n_req, n_heads = q.shape[0], q.shape[1]
    assert q.shape[2] == ROW_DIM and len(kv_offsets) == n_req + 1
    fp8 = pool_bits.shape[1] == CKV_WORDS_FP8 + KR_DIM
    assert fp8 or pool_bits.shape[1] == ROW_DIM
    out = np.zeros((n_req, n_heads, CKV_DIM), np.float64)
    lse = np.full((n_req, n_heads), -np.inf, np.float64)
    half = KR_DIM // 2
    for b in range(n_req):
        slots = kv_slots[kv_offsets[b]:kv_offsets[b + 1]]
        if len(slots) == 0:
            continue
        rows = row_index[slots]
        assert rows.min() >= 0 and rows.max() < pool_bits.shape[0]
        k = dequant_fp8_rows(pool_bits[rows]) if fp8 else bf16_to_f64(pool_bits[rows])   # [n][576]
        hit = hit_index[slots]
        c = np.ones((len(slots), half))
        s = np.zeros((len(slots), half))
        on = hit >= 0
        c[on], s[on] = trig[hit[on], :, 0], trig[hit[on], :, 1]
        kr = k[:, CKV_DIM:]
        ia, ib = (np.arange(0, KR_DIM, 2), np.arange(1, KR_DIM, 2)) if pair_mode else \
            (np.arange(half), np.arange(half) + half)
        rot = np.empty_like(kr)
        rot[:, ia] = kr[:, ia] * c - kr[:, ib] * s
        rot[:, ib] = kr[:, ib] * c + kr[:, ia] * s
        keys = np.concatenate([k[:, :CKV_DIM], rot], axis=1)
        score = scale * (q[b] @ keys.T)                                # [H][n]
        top = score.max(axis=1, keepdims=True)
        e = np.exp(score - top)
        z = e.sum(axis=1, keepdims=True)
        out[b] = (e / z) @ k[:, :CKV_DIM]
        lse[b] = (top + np.log(z))[:, 0]
    return out, lse
