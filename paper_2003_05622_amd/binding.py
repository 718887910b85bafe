"""ctypes binding of the C ABI in include/hps.h (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Optional, Tuple

from .build import ensure_built

OK, EINVAL, EFULL, ERESERVED, ESTATE, EDEVICE, ENOMEM = 0, -1, -2, -3, -4, -5, -6
ADAGRAD_ROWWISE, ADAGRAD_ELEMENTWISE = 0, 1
ROWS_F32, ROWS_BF16, ROWS_F32_WIDE = 0, 1, 2

EXPORTS = ("hps_table_bytes", "hps_workspace_bytes", "hps_create", "hps_insert", "hps_pull",
           "hps_prepare", "hps_pull_prepared",
           "hps_push", "hps_set_pooling", "hps_accumulate", "hps_accumulate_static", "hps_last_unique", "hps_get", "hps_dump", "hps_dump_dirty",
           "hps_stats", "hps_probe_lengths", "hps_clear_error", "hps_clear", "hps_probe_random_rows",
           "hps_destroy", "hps_strerror", "hps_set_stage_timing", "hps_stage_times",
           "hps_mem_create", "hps_mem_fetch", "hps_mem_store", "hps_mem_complete_batch",
           "hps_mem_take_evicted", "hps_mem_list", "hps_mem_stats", "hps_mem_destroy")

STAGES = ("sort", "unique", "lookup", "pool", "push")


class Optimizer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("lr", ctypes.c_float), ("eps", ctypes.c_float),
                ("init_acc", ctypes.c_float), ("init_range", ctypes.c_float),
                ("row_format", ctypes.c_int32), ("init_seed", ctypes.c_uint64)]


class Stats(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint64), ("capacity", ctypes.c_uint64),
                ("n_slots", ctypes.c_uint64), ("last_n_keys", ctypes.c_uint64),
                ("last_n_unique", ctypes.c_uint64), ("last_n_inserted", ctypes.c_uint64),
                ("last_n_absent", ctypes.c_uint64), ("n_plain_fallbacks", ctypes.c_uint64),
                ("n_full_fallbacks", ctypes.c_uint64), ("load_factor", ctypes.c_double),
                ("error", ctypes.c_int32), ("pull_outstanding", ctypes.c_int32)]


class MemStats(ctypes.Structure):
    _fields_ = [("lru_size", ctypes.c_uint64), ("lfu_size", ctypes.c_uint64),
                ("pinned", ctypes.c_uint64), ("evicted_waiting", ctypes.c_uint64),
                ("hits", ctypes.c_uint64), ("misses", ctypes.c_uint64)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded libhps.so with argument types set.  Raises if it cannot be loaded."""
    global _lib
    if _lib is None:
        L = ctypes.CDLL(ensure_built())
        u64, u32, vp, sz = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_size_t
        st = ctypes.c_int
        L.hps_table_bytes.restype = sz
        L.hps_table_bytes.argtypes = [u64, u32, ctypes.POINTER(Optimizer)]
        L.hps_workspace_bytes.restype = sz
        L.hps_workspace_bytes.argtypes = [u64, u64, u32]
        L.hps_create.restype = st
        L.hps_create.argtypes = [ctypes.POINTER(vp), u64, u32, ctypes.POINTER(Optimizer), vp, sz,
                                 vp, sz, u64, u64, vp]
        L.hps_insert.restype = st
        L.hps_insert.argtypes = [vp, vp, u64, vp, vp, vp]
        L.hps_pull.restype = st
        L.hps_pull.argtypes = [vp, vp, u64, vp, u32, u32, vp, vp]
        L.hps_prepare.restype = st
        L.hps_prepare.argtypes = [vp, vp, u64, vp, u32, u32, vp]
        L.hps_pull_prepared.restype = st
        L.hps_pull_prepared.argtypes = [vp, vp, vp]
        L.hps_push.restype = st
        L.hps_push.argtypes = [vp, vp, vp]
        L.hps_last_unique.restype = st
        L.hps_last_unique.argtypes = [vp, vp, vp, vp]
        L.hps_get.restype = st
        L.hps_get.argtypes = [vp, vp, u64, vp, vp, vp, vp]
        L.hps_dump.restype = st
        L.hps_dump.argtypes = [vp, vp, vp, vp, u64, ctypes.POINTER(u64), vp]
        L.hps_dump_dirty.restype = st
        L.hps_dump_dirty.argtypes = [vp, vp, vp, vp, u64, ctypes.POINTER(u64), vp]
        L.hps_set_pooling.restype = st
        L.hps_set_pooling.argtypes = [vp, ctypes.c_int]
        L.hps_accumulate.restype = st
        L.hps_accumulate.argtypes = [vp, vp, u64, vp, vp]
        L.hps_accumulate_static.restype = st
        L.hps_accumulate_static.argtypes = [vp, vp, u64, vp, vp]
        L.hps_stats.restype = st
        L.hps_stats.argtypes = [vp, ctypes.POINTER(Stats), vp]
        L.hps_probe_lengths.restype = st
        L.hps_probe_lengths.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(u64), vp]
        L.hps_clear_error.restype = st
        L.hps_clear_error.argtypes = [vp, vp]
        L.hps_clear.restype = st
        L.hps_clear.argtypes = [vp, vp]
        L.hps_probe_random_rows.restype = st
        L.hps_probe_random_rows.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64, vp, vp]
        L.hps_set_stage_timing.restype = st
        L.hps_set_stage_timing.argtypes = [vp, u32]
        L.hps_stage_times.restype = st
        L.hps_stage_times.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(u32)]
        L.hps_destroy.restype = st
        L.hps_destroy.argtypes = [vp]
        L.hps_mem_create.restype = st
        L.hps_mem_create.argtypes = [ctypes.POINTER(vp), u32, u32, u64, u64]
        L.hps_mem_fetch.restype = st
        L.hps_mem_fetch.argtypes = [vp, vp, u64, u64, vp, vp, vp]
        L.hps_mem_store.restype = st
        L.hps_mem_store.argtypes = [vp, vp, u64, vp, vp, u64, ctypes.c_int]
        L.hps_mem_complete_batch.restype = st
        L.hps_mem_complete_batch.argtypes = [vp, u64]
        L.hps_mem_take_evicted.restype = st
        L.hps_mem_take_evicted.argtypes = [vp, vp, vp, vp, u64, ctypes.POINTER(u64)]
        L.hps_mem_list.restype = st
        L.hps_mem_list.argtypes = [vp, ctypes.c_int, vp, u64, ctypes.POINTER(u64)]
        L.hps_mem_stats.restype = st
        L.hps_mem_stats.argtypes = [vp, ctypes.POINTER(MemStats)]
        L.hps_mem_destroy.restype = st
        L.hps_mem_destroy.argtypes = [vp]
        L.hps_strerror.restype = ctypes.c_char_p
        L.hps_strerror.argtypes = [st]
        _lib = L
    return _lib


class HpsError(RuntimeError):
    def __init__(self, status: int, what: str):
        msg = lib().hps_strerror(status).decode()
        super().__init__("%s: %s (%d)" % (what, msg, status))
        self.status = status


def _check(status: int, what: str) -> None:
    if status != OK:
        raise HpsError(status, what)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def probe_random_rows(rows, n_accesses: int, sink) -> None:
    """Measurement aid: about n_accesses random reads of the rows of `rows` (a float32 CUDA
    tensor of shape [n_rows, 16] or [n_rows, 64]: 64- or 256-byte rows); `sink` needs 262144
    floats."""
    assert rows.dim() == 2 and rows.shape[1] in (16, 64) and sink.numel() >= 262144
    _check(lib().hps_probe_random_rows(_ptr(rows), rows.shape[0], rows.shape[1] * 4, n_accesses,
                                       _ptr(sink), _stream()), "hps_probe_random_rows")


class HpsTable:
    """One table in HBM.  Tensors are torch CUDA tensors; keys travel as int64
    tensors holding the uint64 bit patterns."""

    def __init__(self, capacity: int, dim: int, max_keys: int, max_bags: int, *,
                 opt: int = ADAGRAD_ROWWISE, lr: float = 0.05, eps: float = 1e-8,
                 init_acc: float = 0.1, init_range: float = 0.01, init_seed: int = 0,
                 row_format: int = ROWS_F32, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2003_05622_amd needs a GPU: there is no CPU path")
        self._h = None
        L = lib()
        self.capacity, self.dim, self.max_keys, self.max_bags = capacity, dim, max_keys, max_bags
        self.acc_len = dim if opt == ADAGRAD_ELEMENTWISE else 1
        self.device = torch.device(device)
        self.opt = Optimizer(opt, lr, eps, init_acc, init_range, row_format, init_seed)
        sb = L.hps_table_bytes(capacity, dim, ctypes.byref(self.opt))
        wb = L.hps_workspace_bytes(max_keys, max_bags, dim)
        if sb == 0 or wb == 0:
            raise HpsError(EINVAL, "hps_table_bytes/hps_workspace_bytes")
        with torch.cuda.device(self.device):
            self.storage = torch.empty(sb, dtype=torch.uint8, device=self.device)
            self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.device)
            h = ctypes.c_void_p()
            _check(L.hps_create(ctypes.byref(h), capacity, dim, ctypes.byref(self.opt),
                                self.storage.data_ptr(), sb, self.workspace.data_ptr(), wb,
                                max_keys, max_bags, _stream()), "hps_create")
        self._h = h
        self._last_n = 0
        self._prepared = None

    def close(self) -> None:
        if self._h:
            lib().hps_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, one method per entry point ---------------------------------------
    def insert(self, keys, weights=None, acc=None) -> None:
        _check(lib().hps_insert(self._h, _ptr(keys), keys.numel(), _ptr(weights), _ptr(acc),
                                _stream()), "hps_insert")

    def pull(self, keys, offsets, n_examples: int, n_slots: int, pooled=None):
        import torch
        n_bags = n_examples * n_slots
        assert offsets.numel() == n_bags + 1
        if pooled is None:
            pooled = torch.empty((n_bags, self.dim), dtype=torch.float32, device=self.device)
        _check(lib().hps_pull(self._h, _ptr(keys), keys.numel(), _ptr(offsets), n_examples,
                              n_slots, _ptr(pooled), _stream()), "hps_pull")
        self._last_n = keys.numel()
        return pooled

    def prepare(self, keys, offsets, n_examples: int, n_slots: int) -> None:
        assert offsets.numel() == n_examples * n_slots + 1
        import torch
        # the inputs may have been allocated on another stream than the one the dedup runs on
        cur = torch.cuda.current_stream()
        keys.record_stream(cur)
        offsets.record_stream(cur)
        _check(lib().hps_prepare(self._h, _ptr(keys), keys.numel(), _ptr(offsets), n_examples,
                                 n_slots, _stream()), "hps_prepare")
        self._prepared = (keys.numel(), n_examples * n_slots, keys, offsets)

    def pull_prepared(self, pooled=None):
        import torch
        n, n_bags, _, _ = self._prepared
        if pooled is None:
            pooled = torch.empty((n_bags, self.dim), dtype=torch.float32, device=self.device)
        _check(lib().hps_pull_prepared(self._h, _ptr(pooled), _stream()), "hps_pull_prepared")
        self._last_n = n
        return pooled

    def push(self, pooled_grads) -> None:
        _check(lib().hps_push(self._h, _ptr(pooled_grads), _stream()), "hps_push")

    def last_unique(self) -> Tuple["torch.Tensor", "torch.Tensor"]:
        import torch
        n = self._last_n
        uniq = torch.empty(max(n, 1), dtype=torch.int64, device=self.device)
        inv = torch.empty(max(n, 1), dtype=torch.int32, device=self.device)
        _check(lib().hps_last_unique(self._h, _ptr(uniq), _ptr(inv), _stream()),
               "hps_last_unique")
        u = self.stats().last_n_unique
        return uniq[:u], inv[:n]

    def get(self, keys):
        import torch
        n = keys.numel()
        w = torch.zeros((n, self.dim), dtype=torch.float32, device=self.device)
        a = torch.zeros((n, self.acc_len), dtype=torch.float32, device=self.device)
        f = torch.zeros(n, dtype=torch.uint8, device=self.device)
        _check(lib().hps_get(self._h, _ptr(keys), n, _ptr(w), _ptr(a), _ptr(f), _stream()),
               "hps_get")
        return w, a, f.bool()

    def set_pooling(self, mean: bool) -> None:
        """Bags are summed (False, the default) or averaged (True) from the next pull on."""
        _check(lib().hps_set_pooling(self._h, 1 if mean else 0), "hps_set_pooling")

    def accumulate(self, keys, values) -> None:
        """Adds values[i] onto the row of keys[i] (summed per key; absent keys are skipped)."""
        n = keys.numel()
        if n and tuple(values.shape) != (n, self.dim):
            raise ValueError("values must be [n, dim]")
        _check(lib().hps_accumulate(self._h, _ptr(keys), n, _ptr(values), _stream()),
               "hps_accumulate")

    def accumulate_static(self, keys, values) -> None:
        """accumulate() with the library's static device array as scratch (no allocation)."""
        n = keys.numel()
        if n and tuple(values.shape) != (n, self.dim):
            raise ValueError("values must be [n, dim]")
        _check(lib().hps_accumulate_static(self._h, _ptr(keys), n, _ptr(values), _stream()),
               "hps_accumulate_static")

    def dump(self, max_rows: Optional[int] = None, dirty: bool = False):
        """All rows, or with dirty=True the rows updated since the last dirty dump."""
        import torch
        if max_rows is None:
            max_rows = self.stats().size
        keys = torch.empty(max(max_rows, 1), dtype=torch.int64, device=self.device)
        w = torch.empty((max(max_rows, 1), self.dim), dtype=torch.float32, device=self.device)
        a = torch.empty((max(max_rows, 1), self.acc_len), dtype=torch.float32, device=self.device)
        n = ctypes.c_uint64(0)
        fn = lib().hps_dump_dirty if dirty else lib().hps_dump
        _check(fn(self._h, _ptr(keys), _ptr(w), _ptr(a), max_rows, ctypes.byref(n), _stream()),
               "hps_dump_dirty" if dirty else "hps_dump")
        r = int(n.value)
        return keys[:r], w[:r], a[:r]

    def stats(self) -> Stats:
        s = Stats()
        _check(lib().hps_stats(self._h, ctypes.byref(s), _stream()), "hps_stats")
        return s

    def set_stage_timing(self, stage_mask: int) -> None:
        _check(lib().hps_set_stage_timing(self._h, stage_mask), "hps_set_stage_timing")

    def stage_times(self):
        """{stage name: (sum of milliseconds, number of timed launches)} since the last call."""
        ms = (ctypes.c_double * len(STAGES))()
        cnt = (ctypes.c_uint32 * len(STAGES))()
        _check(lib().hps_stage_times(self._h, ms, cnt), "hps_stage_times")
        return {name: (ms[i], cnt[i]) for i, name in enumerate(STAGES)}

    def probe_lengths(self) -> Tuple[float, int]:
        """(mean, maximum) number of 128-byte buckets a lookup reads to find a stored key."""
        mean, most = ctypes.c_double(), ctypes.c_uint64()
        _check(lib().hps_probe_lengths(self._h, ctypes.byref(mean), ctypes.byref(most), _stream()),
               "hps_probe_lengths")
        return mean.value, most.value

    def clear(self) -> None:
        """Empties the table (settings stay)."""
        _check(lib().hps_clear(self._h, _stream()), "hps_clear")

    def clear_error(self) -> None:
        _check(lib().hps_clear_error(self._h, _stream()), "hps_clear_error")

    def check(self, what: str = "device status") -> None:
        """Raises if the sticky device status is set."""
        e = self.stats().error
        if e != 0:
            raise HpsError(e, what)


class MemTier:
    """The host-memory parameter cache behind the table (include/hps_mem.h).  numpy arrays in
    host memory; needs no GPU."""

    def __init__(self, dim: int, acc_len: int, lru_capacity: int, lfu_capacity: int):
        self.dim, self.acc_len = dim, acc_len
        self.lru_capacity, self.lfu_capacity = lru_capacity, lfu_capacity
        self._h = None
        h = ctypes.c_void_p()
        _check(lib().hps_mem_create(ctypes.byref(h), dim, acc_len, lru_capacity, lfu_capacity),
               "hps_mem_create")
        self._h = h

    def __del__(self):
        if self._h:
            lib().hps_mem_destroy(self._h)
            self._h = None

    @staticmethod
    def _keys(keys):
        import numpy as np
        return np.ascontiguousarray(np.asarray(keys, dtype=np.uint64))

    def fetch(self, keys, batch: int):
        import numpy as np
        k = self._keys(keys)
        w = np.zeros((k.size, self.dim), np.float32)
        a = np.zeros((k.size, self.acc_len), np.float32)
        f = np.zeros(k.size, np.uint8)
        _check(lib().hps_mem_fetch(self._h, k.ctypes.data, k.size, batch, w.ctypes.data, a.ctypes.data,
                                   f.ctypes.data), "hps_mem_fetch")
        return w, a, f.astype(bool)

    def store(self, keys, w, a, batch: int, visit: bool) -> None:
        import numpy as np
        k = self._keys(keys)
        w = np.ascontiguousarray(np.asarray(w, np.float32).reshape(k.size, self.dim))
        a = np.ascontiguousarray(np.asarray(a, np.float32).reshape(k.size, self.acc_len))
        _check(lib().hps_mem_store(self._h, k.ctypes.data, k.size, w.ctypes.data, a.ctypes.data, batch,
                                   1 if visit else 0), "hps_mem_store")

    def complete_batch(self, batch: int) -> None:
        _check(lib().hps_mem_complete_batch(self._h, batch), "hps_mem_complete_batch")

    def stats(self) -> MemStats:
        s = MemStats()
        _check(lib().hps_mem_stats(self._h, ctypes.byref(s)), "hps_mem_stats")
        return s

    def take_evicted_arrays(self):
        """(keys, weights, accumulators) of everything collected so far."""
        import numpy as np
        n = self.stats().evicted_waiting
        k = np.zeros(n, np.uint64)
        w = np.zeros((n, self.dim), np.float32)
        a = np.zeros((n, self.acc_len), np.float32)
        got = ctypes.c_uint64()
        _check(lib().hps_mem_take_evicted(self._h, k.ctypes.data, w.ctypes.data, a.ctypes.data, n,
                                          ctypes.byref(got)), "hps_mem_take_evicted")
        return k[:got.value], w[:got.value], a[:got.value]

    def take_evicted(self):
        k, w, a = self.take_evicted_arrays()
        return [(int(k[i]), w[i], a[i]) for i in range(k.size)]

    def _list(self, which: int):
        import numpy as np
        st = self.stats()
        n = st.lru_size if which == 0 else st.lfu_size
        k = np.zeros(max(n, 1), np.uint64)
        got = ctypes.c_uint64()
        _check(lib().hps_mem_list(self._h, which, k.ctypes.data, n, ctypes.byref(got)), "hps_mem_list")
        return [int(x) for x in k[:got.value]]

    def lru_keys(self):
        return self._list(0)

    def lfu_keys(self):
        return self._list(1)
