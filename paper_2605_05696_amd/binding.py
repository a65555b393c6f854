"""ctypes binding of ``libirm.so`` with the same names as ``include/irm.h``.

Argument marshalling only: torch supplies device memory (``tensor.data_ptr()``)
and the stream handle; every step of the path runs in the library's HIP
kernels.  There is no CPU fallback: if the library has not been built, loading
it raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libirm.so")

IRM_OK, IRM_ERR_INVALID_ARG, IRM_ERR_CAPACITY, IRM_ERR_UNSUPPORTED, IRM_ERR_DEVICE, IRM_ERR_TABLE_FULL = range(6)
STATUS_NAMES = {0: "IRM_OK", 1: "IRM_ERR_INVALID_ARG", 2: "IRM_ERR_CAPACITY", 3: "IRM_ERR_UNSUPPORTED",
                4: "IRM_ERR_DEVICE", 5: "IRM_ERR_TABLE_FULL"}
IRM_FLAG_CHUNK_OVERFLOW, IRM_FLAG_TABLE_FULL, IRM_FLAG_ROW_RANGE, IRM_FLAG_BAD_CHUNK = 1, 2, 4, 8
IRM_FLAG_WAIT_TIMEOUT = 16
IRM_ROW_BF16, IRM_ROW_FP8 = 0, 1

SYMBOLS = ("irm_ctx_create", "irm_ctx_destroy", "irm_ctx_error_flags", "irm_ctx_tune",
           "irm_ctx_profile_begin", "irm_ctx_profile_end", "irm_calibrate_copy", "irm_yardstick",
           "irm_table_create", "irm_table_destroy", "irm_table_insert",
           "irm_cdc_chunk", "irm_chunk_hash", "irm_lookup", "irm_reattach", "irm_reattach_kr", "irm_admit", "irm_table_insert_counted", "irm_s1_windows", "irm_reattach_ref", "irm_attend_ref", "irm_attend_ref_workspace_bytes",
           "irm_reattach_static")


class IrmError(RuntimeError):
    def __init__(self, call, status):
        super().__init__(f"{call} -> {STATUS_NAMES.get(status, status)}")
        self.status = status


class irm_config(ctypes.Structure):
    _fields_ = [("gear", ctypes.c_uint32 * 256), ("mask", ctypes.c_uint32),
                ("min_chunk", ctypes.c_uint32), ("max_chunk", ctypes.c_uint32),
                ("carve_out", ctypes.c_uint32), ("n_layers", ctypes.c_uint32),
                ("ckv_dim", ctypes.c_uint32), ("kr_dim", ctypes.c_uint32),
                ("pair_mode", ctypes.c_uint32), ("row_format", ctypes.c_uint32),
                ("inv_freq", ctypes.c_float * 32),
                ("max_tokens", ctypes.c_uint64), ("max_requests", ctypes.c_uint32)]


# numpy / torch views of the two record types (16 bytes each)
ENTRY_DTYPE = np.dtype([("src_row", "<u4"), ("p_src", "<i4"), ("len", "<u4"), ("entry_id", "<u4")])
HIT_DTYPE = np.dtype([("src_row", "<u4"), ("dst_tok", "<u4"), ("len", "<u4"), ("delta", "<i4")])

_lib = None


def lib():
    """Load the built library; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2605_05696_amd.build` "
                              "(or __graft_entry__.build()); there is no CPU fallback")
        import torch  # noqa: F401  -- first, so that the library binds to the HIP runtime torch uses
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
        L.irm_ctx_create.argtypes = [ctypes.POINTER(irm_config), ctypes.POINTER(vp)]
        L.irm_ctx_destroy.argtypes = [vp]
        L.irm_ctx_error_flags.argtypes = [vp, vp, ctypes.POINTER(u32)]
        L.irm_ctx_tune.argtypes = [vp, u32, u32]
        L.irm_ctx_profile_begin.argtypes = [vp, u32, u32]
        L.irm_ctx_profile_end.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(u32)]
        L.irm_calibrate_copy.argtypes = [vp, vp, u64, u32, vp]
        L.irm_yardstick.argtypes = [vp, vp, u64, u32, u32, u32, u32, vp]
        L.irm_table_create.argtypes = [vp, u64, ctypes.POINTER(vp)]
        L.irm_table_destroy.argtypes = [vp]
        L.irm_table_insert.argtypes = [vp, vp, vp, u32, vp]
        L.irm_cdc_chunk.argtypes = [vp, vp, u64, vp, u32, vp, vp, vp, vp, u32, vp]
        L.irm_chunk_hash.argtypes = [vp, vp, u64, vp, vp, vp, u32, vp, vp]
        L.irm_lookup.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, vp, u32, vp, vp, vp, vp, vp]
        L.irm_reattach.argtypes = [vp, vp, u64, u64, vp, u64, u64, vp, u64, vp, vp, u32, vp]
        L.irm_table_insert_counted.argtypes = [vp, vp, vp, vp, u32, vp]
        L.irm_reattach_static.argtypes = [ctypes.POINTER(ctypes.c_float), u32, u32, u32, vp, u64, u64, vp, u64, u64,
                                          vp, u64, vp, vp, u32, vp, vp]
        L.irm_s1_windows.argtypes = [vp, vp, vp, vp, u32, vp, u32, vp, u32, u32, u32, vp, vp, vp, vp, vp, vp, vp, u32,
                                     vp, vp]
        L.irm_reattach_ref.argtypes = [vp, u64, vp, vp, u64, vp, vp, u64, vp, vp, u32, vp]
        L.irm_attend_ref_workspace_bytes.argtypes = [u32, u32, u32]
        L.irm_attend_ref.argtypes = [vp, vp, u32, u32, vp, u64, u64, vp, vp, vp, vp, u64, vp, u32, ctypes.c_float, u32,
                                     vp, u64, vp, vp, vp]
        L.irm_admit.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, vp, u32, vp, vp, u64, u64, vp, u64, vp,
                                u64, u64, vp, vp, vp]
        L.irm_reattach_kr.argtypes = [vp, vp, u64, u64, vp, u64, u64, vp, vp, u64, vp, vp, u32, vp]
        for name in SYMBOLS:
            getattr(L, name).restype = ctypes.c_int
        L.irm_attend_ref_workspace_bytes.restype = u64       # the one call that returns a size, not a status
        _lib = L
    return _lib


def _check(call, status):
    if status != IRM_OK:
        raise IrmError(call, status)


def _dev(t, dtype, what):
    """Device pointer of a contiguous CUDA/HIP tensor of the given torch dtype."""
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{what}: need a contiguous device tensor of dtype {dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_config(gear, mask, min_chunk, max_chunk, carve_out, n_layers, inv_freq, max_tokens,
                max_requests, ckv_dim=512, kr_dim=64, pair_mode=0, row_format=0) -> irm_config:
    cfg = irm_config()
    gear = np.ascontiguousarray(gear, np.uint32)
    inv_freq = np.ascontiguousarray(inv_freq, np.float32)
    assert gear.shape == (256,) and inv_freq.shape == (32,)
    cfg.gear[:] = gear.tolist()
    cfg.inv_freq[:] = inv_freq.tolist()
    cfg.mask, cfg.min_chunk, cfg.max_chunk, cfg.carve_out = mask, min_chunk, max_chunk, carve_out
    cfg.n_layers, cfg.ckv_dim, cfg.kr_dim, cfg.pair_mode = n_layers, ckv_dim, kr_dim, pair_mode
    cfg.max_tokens, cfg.max_requests, cfg.row_format = max_tokens, max_requests, row_format
    return cfg


def irm_ctx_create(cfg: irm_config) -> ctypes.c_void_p:
    out = ctypes.c_void_p()
    _check("irm_ctx_create", lib().irm_ctx_create(ctypes.byref(cfg), ctypes.byref(out)))
    return out


def irm_ctx_destroy(ctx) -> None:
    _check("irm_ctx_destroy", lib().irm_ctx_destroy(ctx))


def irm_ctx_error_flags(ctx, stream=None) -> int:
    flags = ctypes.c_uint32(0)
    _check("irm_ctx_error_flags", lib().irm_ctx_error_flags(ctx, _stream(stream), ctypes.byref(flags)))
    return flags.value


def irm_ctx_tune(ctx, knob: int, value: int) -> None:
    _check("irm_ctx_tune", lib().irm_ctx_tune(ctx, knob, value))


def irm_ctx_profile_begin(ctx, max_samples: int, every: int = 1) -> None:
    _check("irm_ctx_profile_begin", lib().irm_ctx_profile_begin(ctx, max_samples, every))


def irm_ctx_profile_end(ctx, stream=None):
    """-> (summed milliseconds of the sampled row-kernel launches, number of samples)"""
    ms, n = ctypes.c_float(0), ctypes.c_uint32(0)
    _check("irm_ctx_profile_end", lib().irm_ctx_profile_end(ctx, _stream(stream), ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def irm_calibrate_copy(d_dst, d_src, grid: int = 0, stream=None) -> None:
    """Plain copy of one byte tensor into another of the same size (known HBM traffic)."""
    import torch
    n = d_src.numel() * d_src.element_size()
    if d_dst.numel() * d_dst.element_size() != n or not d_src.is_contiguous() or not d_dst.is_contiguous():
        raise TypeError("irm_calibrate_copy: need two contiguous device tensors of equal byte size")
    _check("irm_calibrate_copy", lib().irm_calibrate_copy(
        ctypes.c_void_p(d_dst.data_ptr()), ctypes.c_void_p(d_src.data_ptr()), n, grid, _stream(stream)))


YARDSTICK_COPY, YARDSTICK_READ, YARDSTICK_WRITE = 0, 1, 2
YARDSTICK_XCD_RANGES = 4                             # or-ed into the mode: one contiguous eighth per XCD


def irm_yardstick(d_dst, d_src, mode: int, grid: int, lanes: int, vectors_per_lane: int, stream=None) -> None:
    """A shaped read, write or copy stream over two byte tensors of equal size (see irm_measure.h)."""
    n = d_src.numel() * d_src.element_size()
    if d_dst.numel() * d_dst.element_size() != n or not d_src.is_contiguous() or not d_dst.is_contiguous():
        raise TypeError("irm_yardstick: need two contiguous device tensors of equal byte size")
    _check("irm_yardstick", lib().irm_yardstick(
        ctypes.c_void_p(d_dst.data_ptr()), ctypes.c_void_p(d_src.data_ptr()), n, mode, grid, lanes,
        vectors_per_lane, _stream(stream)))


def irm_table_create(ctx, n_slots: int) -> ctypes.c_void_p:
    out = ctypes.c_void_p()
    _check("irm_table_create", lib().irm_table_create(ctx, n_slots, ctypes.byref(out)))
    return out


def irm_table_destroy(table) -> None:
    _check("irm_table_destroy", lib().irm_table_destroy(table))


def irm_table_insert(table, d_hash, d_val, stream=None) -> None:
    """d_hash: int64 device tensor [n] (bit pattern of the uint64 hashes);
    d_val: int32 device tensor [n, 4] laid out as irm_entry."""
    import torch
    n = d_hash.numel()
    if d_val.shape != (n, 4):
        raise TypeError("d_val: need shape [n, 4]")
    _check("irm_table_insert", lib().irm_table_insert(
        table, _dev(d_hash, torch.int64, "d_hash"), _dev(d_val, torch.int32, "d_val"), n, _stream(stream)))


def irm_table_insert_counted(table, d_hash, d_val, d_n, stream=None) -> None:
    """As irm_table_insert, the number of pairs read from the device word d_n (at most len(d_hash))."""
    import torch
    cap = d_hash.numel()
    if d_val.shape != (cap, 4) or d_n.numel() != 1:
        raise TypeError("d_val: need shape [n, 4]; d_n: one element")
    _check("irm_table_insert_counted", lib().irm_table_insert_counted(
        table, _dev(d_hash, torch.int64, "d_hash"), _dev(d_val, torch.int32, "d_val"),
        _dev(d_n, torch.int32, "d_n"), cap, _stream(stream)))


S1_SELECT_NEGATIVE, S1_SELECT_NONNEGATIVE, S1_SELECT_ALL = 0, 1, 2
S1_ANCHOR_START, S1_ANCHOR_END = 0, 1


def irm_s1_windows(ctx, d_chunk_start, d_chunk_len, d_req_chunk_offsets, d_n_chunks, d_select, select_mode,
                   window, anchor, d_win_start, d_win_len, d_win_parent, d_req_win_offsets, d_n_windows,
                   d_req_offsets=None, d_pos_base=None, d_win_entry=None, stream=None) -> None:
    import torch
    i32 = torch.int32
    n_req = d_req_chunk_offsets.numel() - 1
    cap = d_win_start.numel()
    if (d_win_len.numel() != cap or d_win_parent.numel() != cap or d_req_win_offsets.numel() != n_req + 1
            or d_chunk_len.numel() != d_chunk_start.numel() or d_n_windows.numel() != 1
            or (d_select is not None and d_select.numel() != d_chunk_start.numel())
            or (d_win_entry is not None and d_win_entry.shape != (cap, 4))):
        raise TypeError("irm_s1_windows: array sizes do not match")
    opt = lambda t, name: None if t is None else _dev(t, i32, name)
    _check("irm_s1_windows", lib().irm_s1_windows(
        ctx, _dev(d_chunk_start, i32, "d_chunk_start"), _dev(d_chunk_len, i32, "d_chunk_len"),
        _dev(d_req_chunk_offsets, i32, "d_req_chunk_offsets"), n_req, _dev(d_n_chunks, i32, "d_n_chunks"),
        d_chunk_start.numel(), opt(d_select, "d_select"), select_mode, window, anchor,
        opt(d_req_offsets, "d_req_offsets"), opt(d_pos_base, "d_pos_base"), _dev(d_win_start, i32, "d_win_start"),
        _dev(d_win_len, i32, "d_win_len"), _dev(d_win_parent, i32, "d_win_parent"),
        _dev(d_req_win_offsets, i32, "d_req_win_offsets"), _dev(d_n_windows, i32, "d_n_windows"), cap,
        opt(d_win_entry, "d_win_entry"), _stream(stream)))


def irm_cdc_chunk(ctx, d_tokens, d_req_offsets, d_chunk_start, d_chunk_len, d_req_chunk_offsets,
                  d_n_chunks, stream=None) -> None:
    """uint32 arrays travel as int32 tensors (same bits)."""
    import torch
    i32 = torch.int32
    n_req = d_req_offsets.numel() - 1
    cap = d_chunk_start.numel()
    if d_chunk_len.numel() != cap or d_req_chunk_offsets.numel() != n_req + 1 or d_n_chunks.numel() != 1:
        raise TypeError("irm_cdc_chunk: output sizes do not match")
    _check("irm_cdc_chunk", lib().irm_cdc_chunk(
        ctx, _dev(d_tokens, i32, "d_tokens"), d_tokens.numel(), _dev(d_req_offsets, i32, "d_req_offsets"),
        n_req, _dev(d_chunk_start, i32, "d_chunk_start"), _dev(d_chunk_len, i32, "d_chunk_len"),
        _dev(d_req_chunk_offsets, i32, "d_req_chunk_offsets"), _dev(d_n_chunks, i32, "d_n_chunks"),
        cap, _stream(stream)))


def irm_chunk_hash(ctx, d_tokens, d_chunk_start, d_chunk_len, d_n_chunks, d_chunk_hash, stream=None) -> None:
    import torch
    i32 = torch.int32
    cap = d_chunk_hash.numel()
    if d_chunk_start.numel() < cap or d_chunk_len.numel() < cap:
        raise TypeError("irm_chunk_hash: chunk arrays shorter than the hash array")
    _check("irm_chunk_hash", lib().irm_chunk_hash(
        ctx, _dev(d_tokens, i32, "d_tokens"), d_tokens.numel(), _dev(d_chunk_start, i32, "d_chunk_start"),
        _dev(d_chunk_len, i32, "d_chunk_len"), _dev(d_n_chunks, i32, "d_n_chunks"), cap,
        _dev(d_chunk_hash, torch.int64, "d_chunk_hash"), _stream(stream)))


def irm_lookup(ctx, table, d_chunk_hash, d_chunk_start, d_chunk_len, d_req_chunk_offsets, d_req_offsets,
               d_pos_base, d_n_chunks, d_chunk_entry, d_hits, d_n_hits, d_hit_tokens, stream=None) -> None:
    """d_hits: int32 device tensor [capacity, 4] laid out as irm_hit."""
    import torch
    i32, i64 = torch.int32, torch.int64
    n_req = d_req_offsets.numel() - 1
    cap = d_chunk_entry.numel()
    if (d_hits.shape != (cap, 4) or d_chunk_hash.numel() < cap or d_chunk_start.numel() < cap
            or d_chunk_len.numel() < cap or d_pos_base.numel() != n_req
            or d_req_chunk_offsets.numel() != n_req + 1):
        raise TypeError("irm_lookup: array sizes do not match")
    _check("irm_lookup", lib().irm_lookup(
        ctx, table, _dev(d_chunk_hash, i64, "d_chunk_hash"), _dev(d_chunk_start, i32, "d_chunk_start"),
        _dev(d_chunk_len, i32, "d_chunk_len"), _dev(d_req_chunk_offsets, i32, "d_req_chunk_offsets"),
        _dev(d_req_offsets, i32, "d_req_offsets"), _dev(d_pos_base, i32, "d_pos_base"), n_req,
        _dev(d_n_chunks, i32, "d_n_chunks"), cap, _dev(d_chunk_entry, i32, "d_chunk_entry"),
        _dev(d_hits, i32, "d_hits"), _dev(d_n_hits, i32, "d_n_hits"),
        _dev(d_hit_tokens, i64, "d_hit_tokens"), _stream(stream)))


ROW_WORDS = {IRM_ROW_BF16: 576, IRM_ROW_FP8: 328}      # 16-bit words per row


def layer_pointers(pool):
    """Device array of per-layer base pointers of a pool tensor [L, rows, W] of 16-bit words
    (dtype bf16): W = 576 for bf16 rows, 328 for fp8 rows (whose first 264 words are bytes and
    scales, not bf16 values)."""
    import torch
    if pool.dim() != 3 or pool.shape[2] not in (576, 328) or pool.dtype != torch.bfloat16 or not pool.is_cuda:
        raise TypeError("pool: need a [L, rows, 576 or 328] bf16 device tensor")
    if pool.stride(2) != 1 or pool.stride(1) < pool.shape[2]:
        raise TypeError("pool: rows must be dense")
    ptrs = [pool.data_ptr() + l * pool.stride(0) * 2 for l in range(pool.shape[0])]
    return torch.tensor(ptrs, dtype=torch.int64, device=pool.device)


def irm_reattach(ctx, d_src_layer_ptrs, src_row_stride_bytes, src_rows, d_dst_layer_ptrs,
                 dst_row_stride_bytes, dst_rows, d_dst_slots, d_hits, d_n_hits, stream=None) -> None:
    import torch
    i32, i64 = torch.int32, torch.int64
    if d_hits.dim() != 2 or d_hits.shape[1] != 4:
        raise TypeError("d_hits: need shape [capacity, 4]")
    if d_src_layer_ptrs.numel() != d_dst_layer_ptrs.numel():
        raise TypeError("layer pointer arrays differ in length")
    _check("irm_reattach", lib().irm_reattach(
        ctx, _dev(d_src_layer_ptrs, i64, "d_src_layer_ptrs"), src_row_stride_bytes, src_rows,
        _dev(d_dst_layer_ptrs, i64, "d_dst_layer_ptrs"), dst_row_stride_bytes, dst_rows,
        _dev(d_dst_slots, i32, "d_dst_slots"), d_dst_slots.numel(), _dev(d_hits, i32, "d_hits"),
        _dev(d_n_hits, i32, "d_n_hits"), d_hits.shape[0], _stream(stream)))


REATTACH_STATIC_MAX_TOKENS, REATTACH_STATIC_MAX_HITS = 131072, 4096


def irm_reattach_static(inv_freq, n_layers, pair_mode, row_format, d_src_layer_ptrs, src_row_stride_bytes, src_rows,
                        d_dst_layer_ptrs, dst_row_stride_bytes, dst_rows, d_dst_slots, d_hits, d_n_hits,
                        d_error_flags=None, stream=None) -> None:
    """irm_reattach without a context: inv_freq is a host array of 32 floats; d_error_flags an
    optional int32 device tensor of one element the kernels OR their flags into."""
    import torch
    i32, i64 = torch.int32, torch.int64
    if d_hits.dim() != 2 or d_hits.shape[1] != 4:
        raise TypeError("d_hits: need shape [capacity, 4]")
    f = np.ascontiguousarray(inv_freq, np.float32)
    if f.shape != (32,):
        raise TypeError("inv_freq: need 32 floats")
    _check("irm_reattach_static", lib().irm_reattach_static(
        f.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), n_layers, pair_mode, row_format,
        _dev(d_src_layer_ptrs, i64, "d_src_layer_ptrs"), src_row_stride_bytes, src_rows,
        _dev(d_dst_layer_ptrs, i64, "d_dst_layer_ptrs"), dst_row_stride_bytes, dst_rows,
        _dev(d_dst_slots, i32, "d_dst_slots"), d_dst_slots.numel(), _dev(d_hits, i32, "d_hits"),
        _dev(d_n_hits, i32, "d_n_hits"), d_hits.shape[0],
        None if d_error_flags is None else _dev(d_error_flags, i32, "d_error_flags"), _stream(stream)))


def kr_slice_pointers(pool):
    """Per-layer pointers to the k_r slice of row 0 of a packed pool (see layer_pointers)."""
    return layer_pointers(pool) + (pool.shape[2] - 64) * 2


def kr_layer_pointers(pool):
    """Device array of per-layer base pointers of a [L, rows, 64] bf16 k_r pool tensor."""
    import torch
    if pool.dim() != 3 or pool.shape[2] != 64 or pool.dtype != torch.bfloat16 or not pool.is_cuda:
        raise TypeError("pool: need a [L, rows, 64] bf16 device tensor")
    if pool.stride(2) != 1 or pool.stride(1) < 64:
        raise TypeError("pool: rows must be dense")
    ptrs = [pool.data_ptr() + l * pool.stride(0) * 2 for l in range(pool.shape[0])]
    return torch.tensor(ptrs, dtype=torch.int64, device=pool.device)


def irm_reattach_kr(ctx, d_src_kr_layer_ptrs, src_kr_row_stride_bytes, src_rows, d_kr_layer_ptrs,
                    kr_row_stride_bytes, kr_rows, d_ckv_index, d_dst_slots, d_hits, d_n_hits,
                    stream=None) -> None:
    import torch
    i32, i64 = torch.int32, torch.int64
    if d_hits.dim() != 2 or d_hits.shape[1] != 4:
        raise TypeError("d_hits: need shape [capacity, 4]")
    if d_src_kr_layer_ptrs.numel() != d_kr_layer_ptrs.numel() or d_ckv_index.numel() < kr_rows:
        raise TypeError("irm_reattach_kr: array sizes do not match")
    _check("irm_reattach_kr", lib().irm_reattach_kr(
        ctx, _dev(d_src_kr_layer_ptrs, i64, "d_src_kr_layer_ptrs"), src_kr_row_stride_bytes, src_rows,
        _dev(d_kr_layer_ptrs, i64, "d_kr_layer_ptrs"), kr_row_stride_bytes, kr_rows,
        _dev(d_ckv_index, i32, "d_ckv_index"), _dev(d_dst_slots, i32, "d_dst_slots"), d_dst_slots.numel(),
        _dev(d_hits, i32, "d_hits"), _dev(d_n_hits, i32, "d_n_hits"), d_hits.shape[0], _stream(stream)))


def irm_admit(ctx, table, d_chunk_hash, d_chunk_start, d_chunk_len, d_req_chunk_offsets, d_req_offsets,
              d_pos_base, d_n_chunks, d_chunk_entry, d_req_layer_ptrs, req_row_stride_bytes, req_rows,
              d_slots, d_pool_layer_ptrs, pool_row_stride_bytes, pool_rows, d_cursor, d_admitted_row,
              stream=None) -> None:
    import torch
    i32, i64 = torch.int32, torch.int64
    n_req = d_req_offsets.numel() - 1
    cap = d_chunk_entry.numel()
    if (d_admitted_row.numel() != cap or d_chunk_hash.numel() < cap or d_chunk_start.numel() < cap
            or d_chunk_len.numel() < cap or d_pos_base.numel() != n_req or d_cursor.numel() != 1
            or d_req_layer_ptrs.numel() != d_pool_layer_ptrs.numel()):
        raise TypeError("irm_admit: array sizes do not match")
    _check("irm_admit", lib().irm_admit(
        ctx, table, _dev(d_chunk_hash, i64, "d_chunk_hash"), _dev(d_chunk_start, i32, "d_chunk_start"),
        _dev(d_chunk_len, i32, "d_chunk_len"), _dev(d_req_chunk_offsets, i32, "d_req_chunk_offsets"),
        _dev(d_req_offsets, i32, "d_req_offsets"), _dev(d_pos_base, i32, "d_pos_base"), n_req,
        _dev(d_n_chunks, i32, "d_n_chunks"), cap, _dev(d_chunk_entry, i32, "d_chunk_entry"),
        _dev(d_req_layer_ptrs, i64, "d_req_layer_ptrs"), req_row_stride_bytes, req_rows,
        _dev(d_slots, i32, "d_slots"), d_slots.numel(), _dev(d_pool_layer_ptrs, i64, "d_pool_layer_ptrs"),
        pool_row_stride_bytes, pool_rows, _dev(d_cursor, i32, "d_cursor"),
        _dev(d_admitted_row, i32, "d_admitted_row"), _stream(stream)))


def irm_reattach_ref(ctx, src_rows, d_row_index, d_hit_index, d_trig, d_dst_slots, d_hits, d_n_hits,
                     stream=None) -> None:
    """d_trig: float32 device tensor [hit_capacity, 32, 2]."""
    import torch
    i32 = torch.int32
    cap = d_hits.shape[0]
    if (d_hits.shape != (cap, 4) or d_trig.shape != (cap, 32, 2) or d_row_index.numel() != d_hit_index.numel()):
        raise TypeError("irm_reattach_ref: array sizes do not match")
    _check("irm_reattach_ref", lib().irm_reattach_ref(
        ctx, src_rows, _dev(d_row_index, i32, "d_row_index"), _dev(d_hit_index, i32, "d_hit_index"),
        d_row_index.numel(), _dev(d_trig, torch.float32, "d_trig"), _dev(d_dst_slots, i32, "d_dst_slots"),
        d_dst_slots.numel(), _dev(d_hits, i32, "d_hits"), _dev(d_n_hits, i32, "d_n_hits"), cap, _stream(stream)))


def irm_attend_ref(ctx, d_q, d_pool_layer, pool_row_stride_bytes, d_kv_slots, d_kv_offsets, d_row_index,
                   d_hit_index, d_trig, scale, n_splits, d_workspace, d_out, d_lse, stream=None) -> None:
    """d_q: bf16 [n_req, n_heads, 576]; d_pool_layer: one layer of the pool, [rows, >= 576] bf16
    (in an fp8 context [rows, >= 328] 16-bit words typed bf16, see layer_pointers);
    d_out: float32 [n_req, n_heads, 512]; d_lse: float32 [n_req, n_heads]; d_workspace: uint8 tensor."""
    import torch
    i32 = torch.int32
    n_req, n_heads = d_q.shape[0], d_q.shape[1]
    if (d_q.dtype != torch.bfloat16 or d_q.shape[2] != 576 or not d_q.is_contiguous() or
            d_pool_layer.dtype != torch.bfloat16 or d_out.shape != (n_req, n_heads, 512) or
            d_lse.shape != (n_req, n_heads) or d_kv_offsets.numel() != n_req + 1 or
            d_row_index.numel() != d_hit_index.numel() or d_trig.dim() != 3 or d_trig.shape[1:] != (32, 2)):
        raise TypeError("irm_attend_ref: array shapes or types do not match")
    _check("irm_attend_ref", lib().irm_attend_ref(
        ctx, d_q.data_ptr(), n_req, n_heads, d_pool_layer.data_ptr(), pool_row_stride_bytes, d_pool_layer.shape[0],
        _dev(d_kv_slots, i32, "d_kv_slots"), _dev(d_kv_offsets, i32, "d_kv_offsets"),
        _dev(d_row_index, i32, "d_row_index"), _dev(d_hit_index, i32, "d_hit_index"), d_row_index.numel(),
        _dev(d_trig, torch.float32, "d_trig"), d_trig.shape[0], float(scale), n_splits,
        d_workspace.data_ptr(), d_workspace.numel() * d_workspace.element_size(),
        _dev(d_out, torch.float32, "d_out"), _dev(d_lse, torch.float32, "d_lse"), _stream(stream)))


def irm_attend_ref_workspace_bytes(n_req, n_heads, n_splits) -> int:
    return int(lib().irm_attend_ref_workspace_bytes(n_req, n_heads, n_splits))
