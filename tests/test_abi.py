"""The C-ABI library: it loads, exports every function the header declares, and
rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_05696_amd import binding as B
from paper_2605_05696_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("irm.h", "irm_measure.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^(?:irm_status|uint64_t)\s+(irm_\w+)\s*\(", text, flags=re.M)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 21
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.SYMBOLS) == names


def test_struct_layouts_match_the_header(tmp_path):
    """Sizes and field offsets as the C compiler lays the header's structs out, against the binding's."""
    import subprocess
    fields = [f[0] for f in B.irm_config._fields_]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "irm.h"', 'int main(void) {',
            '  printf("%zu %zu %zu\\n", sizeof(irm_config), sizeof(irm_entry), sizeof(irm_hit));']
    prog += [f'  printf("%zu\\n", offsetof(irm_config, {f}));' for f in fields]
    prog += ['  return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(prog))
    exe = tmp_path / "layout"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe)], check=True)
    lines = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    sizes = [int(x) for x in lines[0].split()]
    assert sizes == [ctypes.sizeof(B.irm_config), B.ENTRY_DTYPE.itemsize, B.HIT_DTYPE.itemsize]
    assert sizes[1:] == [16, 16]
    for f, line in zip(fields, lines[1:]):
        assert getattr(B.irm_config, f).offset == int(line), f


def good_config(**over):
    kw = dict(gear=wl.gear_table(), mask=0xFF, min_chunk=64, max_chunk=1024, carve_out=32, n_layers=2,
              inv_freq=wl.inv_freq_plain(), max_tokens=4096, max_requests=4)
    kw.update(over)
    return B.make_config(**kw)


@pytest.mark.parametrize("over,status", [
    (dict(mask=0xFE), B.IRM_ERR_UNSUPPORTED),               # not 2^k - 1
    (dict(ckv_dim=256), B.IRM_ERR_UNSUPPORTED),
    (dict(kr_dim=128), B.IRM_ERR_UNSUPPORTED),
    (dict(pair_mode=2), B.IRM_ERR_UNSUPPORTED),
    (dict(min_chunk=4), B.IRM_ERR_INVALID_ARG),             # window of 8 tokens needs min >= 8
    (dict(min_chunk=0), B.IRM_ERR_INVALID_ARG),
    (dict(min_chunk=2000), B.IRM_ERR_INVALID_ARG),          # min > max
    (dict(max_chunk=1 << 20), B.IRM_ERR_INVALID_ARG),
    (dict(n_layers=0), B.IRM_ERR_INVALID_ARG),
    (dict(max_tokens=0), B.IRM_ERR_INVALID_ARG),
    (dict(max_requests=0), B.IRM_ERR_INVALID_ARG),
    (dict(inv_freq=np.full(32, np.nan, np.float32)), B.IRM_ERR_INVALID_ARG),
])
def test_ctx_create_rejects_bad_configs(over, status):
    cfg = good_config(**over)
    out = ctypes.c_void_p()
    assert B.lib().irm_ctx_create(ctypes.byref(cfg), ctypes.byref(out)) == status
    assert not out.value


def test_null_arguments_are_rejected():
    L = B.lib()
    out = ctypes.c_void_p()
    assert L.irm_ctx_create(None, ctypes.byref(out)) == B.IRM_ERR_INVALID_ARG
    assert L.irm_ctx_create(ctypes.byref(good_config()), None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_ctx_destroy(None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_table_destroy(None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_table_create(None, 16, ctypes.byref(out)) == B.IRM_ERR_INVALID_ARG
    assert L.irm_table_insert(None, None, None, 0, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_cdc_chunk(None, None, 0, None, 0, None, None, None, None, 0, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_chunk_hash(None, None, 0, None, None, None, 0, None, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_lookup(*([None] * 8), 0, None, 0, *([None] * 5)) == B.IRM_ERR_INVALID_ARG
    assert L.irm_reattach(None, None, 0, 0, None, 0, 0, None, 0, None, None, 0, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_reattach_kr(None, None, 0, 0, None, 0, 0, None, None, 0, None, None, 0, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_admit(*([None] * 8), 0, None, 0, None, None, 0, 0, None, 0, None, 0, 0, None, None, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_s1_windows(*([None] * 4), 0, None, 0, None, 0, 0, 0, *([None] * 7), 0, None, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_table_insert_counted(None, None, None, None, 0, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_reattach_ref(None, 1, None, None, 1, None, None, 1, None, None, 1, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_attend_ref(*([None] * 2), 1, 16, None, 1152, 1, *([None] * 4), 1, None, 0, ctypes.c_float(1.0), 1, None, 0,
                            None, None, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_attend_ref_workspace_bytes(2, 16, 3) == 2 * 16 * 3 * 514 * 4
    # a size beyond 32 bits must come back whole, through the raw symbol and through the binding
    big = 65535 * 8192 * 4 * 514 * 4
    assert big > 1 << 32
    assert L.irm_attend_ref_workspace_bytes(65535, 8192, 4) == big
    assert B.irm_attend_ref_workspace_bytes(65535, 8192, 4) == big
    # the entry point without a context: sizes beyond its static scratch are refused before any device call
    f32 = (ctypes.c_float * 32)(*([1.0] * 32))
    one = ctypes.c_void_p(16)
    assert L.irm_reattach_static(None, 1, 0, 0, one, 1152, 1, one, 1152, 1, one, 1, one, one, 1, None, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_reattach_static(f32, 1, 0, 0, one, 1152, 1, one, 1152, 1, one, B.REATTACH_STATIC_MAX_TOKENS + 1, one, one,
                                 1, None, None) == B.IRM_ERR_CAPACITY
    assert L.irm_reattach_static(f32, 1, 0, 0, one, 1152, 1, one, 1152, 1, one, 1, one, one,
                                 B.REATTACH_STATIC_MAX_HITS + 1, None, None) == B.IRM_ERR_CAPACITY
    flags = ctypes.c_uint32()
    assert L.irm_ctx_error_flags(None, None, ctypes.byref(flags)) == B.IRM_ERR_INVALID_ARG
    assert L.irm_ctx_tune(None, 0, 0) == B.IRM_ERR_INVALID_ARG
    assert L.irm_calibrate_copy(None, None, 0, 0, None) == B.IRM_ERR_INVALID_ARG
    assert L.irm_ctx_profile_begin(None, 4, 1) == B.IRM_ERR_INVALID_ARG
    assert L.irm_ctx_profile_end(None, None, None, None) == B.IRM_ERR_INVALID_ARG


def test_without_a_gpu_creation_fails_loudly_instead_of_falling_back():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.IrmError) as e:
        B.irm_ctx_create(good_config())
    assert e.value.status == B.IRM_ERR_DEVICE
