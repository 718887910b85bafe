"""ctypes access to the CPU oracle (oracle/hps_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module,
and this module never imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hps_oracle.cpp")
# HPS_ORACLE_LIB: use this already built library instead (the sanitizer run of the tests)
_LIB = os.environ.get("HPS_ORACLE_LIB") or os.path.join(_HERE, "libhps_oracle.so")

OK, EINVAL, EFULL, ERESERVED, ESTATE = 0, -1, -2, -3, -4
ADAGRAD_ROWWISE, ADAGRAD_ELEMENTWISE = 0, 1
ROWS_F32, ROWS_BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add contraction)."""
    if os.environ.get("HPS_ORACLE_LIB"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC",
                               "-shared", "-Wall", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u64, u32, i32, f32, vp = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32,
                                  ctypes.c_float, ctypes.c_void_p)
        L.hpo_mix.restype = u64
        L.hpo_mix.argtypes = [u64]
        L.hpo_create.restype = vp
        L.hpo_create.argtypes = [u64, u32, ctypes.c_int, f32, f32, f32, f32, u64]
        L.hpo_destroy.restype = None
        L.hpo_destroy.argtypes = [vp]
        L.hpo_size.restype = u64
        L.hpo_size.argtypes = [vp]
        L.hpo_stored_rows.restype = u64
        L.hpo_stored_rows.argtypes = [vp]
        L.hpo_acc_len.restype = u32
        L.hpo_acc_len.argtypes = [vp]
        L.hpo_init_row.restype = None
        L.hpo_init_row.argtypes = [vp, u64, vp]
        L.hpo_declare_resident.restype = i32
        L.hpo_declare_resident.argtypes = [vp, u64]
        L.hpo_materialize.restype = i32
        L.hpo_materialize.argtypes = [vp, vp, u64]
        L.hpo_insert.restype = i32
        L.hpo_insert.argtypes = [vp, vp, u64, vp, vp]
        L.hpo_dedup.restype = i32
        L.hpo_dedup.argtypes = [vp, u64, vp, vp, vp]
        L.hpo_pull.restype = i32
        L.hpo_pull.argtypes = [vp, vp, u64, vp, u64, vp, vp, vp]
        L.hpo_last_unique.restype = i32
        L.hpo_last_unique.argtypes = [vp, vp, vp]
        L.hpo_push.restype = i32
        L.hpo_push.argtypes = [vp, vp]
        L.hpo_get.restype = i32
        L.hpo_get.argtypes = [vp, vp, u64, vp, vp, vp]
        L.hpo_dump.restype = i32
        L.hpo_dump.argtypes = [vp, vp, vp, vp, u64, vp]
        L.hpo_dump_dirty.restype = i32
        L.hpo_dump_dirty.argtypes = [vp, vp, vp, vp, u64, vp]
        L.hpo_set_pooling.restype = i32
        L.hpo_set_pooling.argtypes = [vp, ctypes.c_int]
        L.hpo_accumulate.restype = i32
        L.hpo_accumulate.argtypes = [vp, vp, u64, vp, vp]
        L.hpo_clear.restype = i32
        L.hpo_clear.argtypes = [vp]
        L.hpo_set_row_format.restype = i32
        L.hpo_set_row_format.argtypes = [vp, ctypes.c_int]
        L.hpo_nearest_bf16.restype = f32
        L.hpo_nearest_bf16.argtypes = [f32]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s: oracle status %d" % (what, status))
        self.status = status


def _check(status: int, what: str) -> None:
    if status != OK:
        raise OracleError(status, what)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _keys(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


def mix(x: int) -> int:
    return int(lib().hpo_mix(ctypes.c_uint64(x & (2**64 - 1))))


def nearest_bf16(x: float) -> float:
    """The bfloat16 value nearest to the float32 x (ties to even), as a float."""
    return float(lib().hpo_nearest_bf16(ctypes.c_float(x)))


def dedup(keys) -> Tuple[np.ndarray, np.ndarray]:
    """Sorted unique keys and inverse[i] = rank of keys[i]."""
    keys = _keys(keys)
    n = keys.shape[0]
    uniq = np.empty(max(n, 1), dtype=np.uint64)
    inv = np.empty(max(n, 1), dtype=np.int32)
    nu = ctypes.c_uint64(0)
    _check(lib().hpo_dedup(_p(keys), n, _p(uniq), _p(inv), ctypes.byref(nu)), "dedup")
    return uniq[: nu.value].copy(), inv[:n].copy()


class OracleTable:
    """The reference table: create / insert / pull / push / get / dump."""

    def __init__(self, capacity: int, dim: int, *, opt: int = ADAGRAD_ROWWISE, lr: float = 0.05,
                 eps: float = 1e-8, init_acc: float = 0.1, init_range: float = 0.01,
                 init_seed: int = 0, row_format: int = ROWS_F32):
        self._h = lib().hpo_create(capacity, dim, opt, lr, eps, init_acc, init_range, init_seed)
        if not self._h:
            raise OracleError(EINVAL, "create")
        _check(lib().hpo_set_row_format(self._h, row_format), "set_row_format")
        self.capacity, self.dim = capacity, dim
        self.acc_len = int(lib().hpo_acc_len(self._h))
        self._n = 0

    def close(self) -> None:
        if self._h:
            lib().hpo_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def size(self) -> int:
        return int(lib().hpo_size(self._h))

    @property
    def stored_rows(self) -> int:
        return int(lib().hpo_stored_rows(self._h))

    def init_row(self, key: int) -> np.ndarray:
        out = np.empty(self.dim, dtype=np.float32)
        lib().hpo_init_row(self._h, ctypes.c_uint64(int(key)), _p(out))
        return out

    def declare_resident(self, n: int) -> None:
        _check(lib().hpo_declare_resident(self._h, n), "declare_resident")

    def materialize(self, keys) -> None:
        keys = _keys(keys)
        _check(lib().hpo_materialize(self._h, _p(keys), keys.shape[0]), "materialize")

    def insert(self, keys, weights=None, acc=None) -> None:
        keys = _keys(keys)
        n = keys.shape[0]
        if weights is not None:
            weights = np.ascontiguousarray(weights, dtype=np.float32).reshape(n, self.dim)
        if acc is not None:
            acc = np.ascontiguousarray(acc, dtype=np.float32).reshape(n, self.acc_len)
        _check(lib().hpo_insert(self._h, _p(keys), n, _p(weights), _p(acc)), "insert")

    def pull(self, keys, offsets) -> np.ndarray:
        keys = _keys(keys)
        offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        n_bags = offsets.shape[0] - 1
        pooled = np.zeros((n_bags, self.dim), dtype=np.float32)
        nu, ni = ctypes.c_uint64(0), ctypes.c_uint64(0)
        st = lib().hpo_pull(self._h, _p(keys), keys.shape[0], _p(offsets), n_bags, _p(pooled),
                            ctypes.byref(nu), ctypes.byref(ni))
        self.n_unique, self.n_inserted, self._n = int(nu.value), int(ni.value), keys.shape[0]
        _check(st, "pull")
        return pooled

    def last_unique(self) -> Tuple[np.ndarray, np.ndarray]:
        uniq = np.empty(max(self.n_unique, 1), dtype=np.uint64)
        inv = np.empty(max(self._n, 1), dtype=np.int32)
        _check(lib().hpo_last_unique(self._h, _p(uniq), _p(inv)), "last_unique")
        return uniq[: self.n_unique].copy(), inv[: self._n].copy()

    def push(self, grads) -> None:
        grads = np.ascontiguousarray(grads, dtype=np.float32)
        _check(lib().hpo_push(self._h, _p(grads)), "push")

    def get(self, keys) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        keys = _keys(keys)
        n = keys.shape[0]
        w = np.zeros((n, self.dim), dtype=np.float32)
        a = np.zeros((n, self.acc_len), dtype=np.float32)
        f = np.zeros(n, dtype=np.uint8)
        _check(lib().hpo_get(self._h, _p(keys), n, _p(w), _p(a), _p(f)), "get")
        return w, a, f.astype(bool)

    def set_pooling(self, mean: bool) -> None:
        _check(lib().hpo_set_pooling(self._h, 1 if mean else 0), "set_pooling")

    def clear(self) -> None:
        """Empties the table; settings stay."""
        _check(lib().hpo_clear(self._h), "clear")

    def accumulate(self, keys, values) -> int:
        """Adds the value rows onto the rows of their keys; returns the number of
        distinct keys that are not in the table (skipped)."""
        keys = _keys(keys)
        n = keys.shape[0]
        values = np.ascontiguousarray(values, dtype=np.float32).reshape(n, self.dim)
        absent = ctypes.c_uint64(0)
        _check(lib().hpo_accumulate(self._h, _p(keys), n, _p(values), ctypes.byref(absent)),
               "accumulate")
        return int(absent.value)

    def dump_dirty(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Rows changed by push/accumulate since the last call, ascending by key."""
        r = self.stored_rows
        keys = np.empty(max(r, 1), dtype=np.uint64)
        w = np.empty((max(r, 1), self.dim), dtype=np.float32)
        a = np.empty((max(r, 1), self.acc_len), dtype=np.float32)
        n = ctypes.c_uint64(0)
        _check(lib().hpo_dump_dirty(self._h, _p(keys), _p(w), _p(a), r, ctypes.byref(n)),
               "dump_dirty")
        n = int(n.value)
        return keys[:n].copy(), w[:n].copy(), a[:n].copy()

    def dump(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        r = self.stored_rows
        keys = np.empty(max(r, 1), dtype=np.uint64)
        w = np.empty((max(r, 1), self.dim), dtype=np.float32)
        a = np.empty((max(r, 1), self.acc_len), dtype=np.float32)
        n = ctypes.c_uint64(0)
        _check(lib().hpo_dump(self._h, _p(keys), _p(w), _p(a), r, ctypes.byref(n)), "dump")
        return keys[:r].copy(), w[:r].copy(), a[:r].copy()
