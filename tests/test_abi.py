"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/*.h declares, sizes its buffers sensibly and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2003_05622_amd as hps

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in ("hps.h", "hps_measure.h", "hps_mem.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(hps_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = hps.lib()
    names = _declared_symbols()
    assert set(names) == set(hps.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_strerror():
    L = hps.lib()
    seen = {L.hps_strerror(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and all(seen)


def _opt(kind=0, rng=0.01, eps=1e-8, row_format=0):
    return hps.Optimizer(kind, 0.05, eps, 0.1, rng, row_format, 0)


def test_buffer_sizes():
    L = hps.lib()
    o = _opt()
    # 1e9 keys, dim 16, row-wise: (1e9 / 0.7) slots x (8 + 64 + 4) bytes ~ 108.6 GB
    b = L.hps_table_bytes(10**9, 16, ctypes.byref(o))
    assert 108.5e9 < b < 108.7e9
    e = _opt(kind=1)
    assert L.hps_table_bytes(1 << 20, 16, ctypes.byref(e)) > L.hps_table_bytes(1 << 20, 16, ctypes.byref(o))
    assert L.hps_table_bytes(0, 16, ctypes.byref(o)) == 0
    assert L.hps_table_bytes(100, 6, ctypes.byref(o)) == 0            # dim not a multiple of 4
    assert L.hps_table_bytes(100, 2048, ctypes.byref(o)) == 0
    assert L.hps_table_bytes(1 << 32, 16, ctypes.byref(o)) == 0       # slot index would overflow
    assert L.hps_table_bytes(100, 16, None) == 0
    bad = hps.Optimizer(7, 0.05, 1e-8, 0.1, 0.01, 0, 0)
    assert L.hps_table_bytes(100, 16, ctypes.byref(bad)) == 0
    # bfloat16 rows: (1e9 / 0.7) slots x (8 + 32 + 4) bytes ~ 62.9 GB
    h = _opt(row_format=hps.ROWS_BF16)
    assert 62.8e9 < L.hps_table_bytes(10**9, 16, ctypes.byref(h)) < 63.0e9
    assert L.hps_table_bytes(100, 16, ctypes.byref(_opt(row_format=5))) == 0
    assert L.hps_workspace_bytes(1 << 31, 10, 16) == 0
    w1 = L.hps_workspace_bytes(1 << 20, 1 << 18, 16)
    w2 = L.hps_workspace_bytes(1 << 21, 1 << 18, 16)
    assert 0 < w1 < w2 < 2.2 * w1
    assert L.hps_workspace_bytes(0, 0, 16) > 0


def test_create_rejects_bad_arguments_before_touching_the_device():
    L = hps.lib()
    o = _opt()
    h = ctypes.c_void_p()
    sb = L.hps_table_bytes(1000, 8, ctypes.byref(o))
    wb = L.hps_workspace_bytes(100, 10, 8)
    ok_ptr = 1 << 20      # aligned, never dereferenced on these paths
    create = L.hps_create
    assert create(None, 1000, 8, ctypes.byref(o), ok_ptr, sb, ok_ptr, wb, 100, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 1000, 8, None, ok_ptr, sb, ok_ptr, wb, 100, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 0, 8, ctypes.byref(o), ok_ptr, sb, ok_ptr, wb, 100, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 1000, 7, ctypes.byref(o), ok_ptr, sb, ok_ptr, wb, 100, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 1000, 8, ctypes.byref(o), None, sb, ok_ptr, wb, 100, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 1000, 8, ctypes.byref(o), ok_ptr + 8, sb, ok_ptr, wb, 100, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 1000, 8, ctypes.byref(o), ok_ptr, sb, ok_ptr, wb, 1 << 31, 10, None) == hps.EINVAL
    assert create(ctypes.byref(h), 1000, 8, ctypes.byref(o), ok_ptr, sb - 1, ok_ptr, wb, 100, 10, None) == hps.ENOMEM
    assert create(ctypes.byref(h), 1000, 8, ctypes.byref(o), ok_ptr, sb, ok_ptr, wb - 1, 100, 10, None) == hps.ENOMEM
    assert not h.value
    # null handles
    assert L.hps_push(None, None, None) == hps.EINVAL
    assert L.hps_pull(None, None, 0, None, 0, 0, None, None) == hps.EINVAL
    assert L.hps_insert(None, None, 0, None, None, None) == hps.EINVAL
    assert L.hps_destroy(None) == hps.EINVAL
    assert L.hps_stats(None, None, None) == hps.EINVAL
    assert L.hps_accumulate(None, None, 0, None, None) == hps.EINVAL
    assert L.hps_accumulate_static(None, None, 0, None, None) == hps.EINVAL
    assert L.hps_probe_random_rows(None, 0, 64, 0, None, None) == hps.EINVAL


def test_no_cpu_fallback_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        hps.HpsTable(1000, 8, 100, 10)
