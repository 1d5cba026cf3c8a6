"""ctypes front end of the CPU checker (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product path never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, BF16 = 0, 1
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.cpp with the host compiler (plain -O2, one thread).
    ORACLE_SANITIZE=1 in the environment builds and loads an AddressSanitizer + UBSan variant instead
    (run the tests with libasan preloaded: LD_PRELOAD=$(g++ -print-file-name=libasan.so):$LD_PRELOAD)."""
    global _LIB
    flags = ["-O2"]
    if os.environ.get("ORACLE_SANITIZE"):
        _LIB = os.path.join(_HERE, "liboracle_san.so")
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", *flags, "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-o", _LIB, _SRC])
    return _LIB


def _p(a: Optional[np.ndarray], ct):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_table_create.restype = C.c_void_p
        L.orc_table_create.argtypes = [C.c_int, C.c_int, C.c_float]
        L.orc_table_destroy.argtypes = [C.c_void_p]
        L.orc_size.restype = C.c_int64
        L.orc_size.argtypes = [C.c_void_p]
        L.orc_dedup.restype = C.c_int64
        L.orc_evict.restype = C.c_int64
        L.orc_export.restype = C.c_int64
        L.orc_promote.restype = C.c_int64
        L.orc_export_hot.restype = C.c_int64
        L.orc_demote.restype = C.c_int64
        L.orc_put_hot.restype = C.c_int64
        L.orc_put.restype = C.c_int64
        _lib = L
    return _lib


# --------------------------------------------------------------------------- #
def plan_merge(dims, dtypes) -> Tuple[np.ndarray, int]:
    dims = np.ascontiguousarray(dims, dtype=np.int32)
    dtypes = np.ascontiguousarray(dtypes, dtype=np.int32)
    out = np.empty(len(dims), dtype=np.int32)
    n = lib().orc_plan_merge(_p(dims, C.c_int), _p(dtypes, C.c_int), C.c_int(len(dims)), _p(out, C.c_int))
    return out, int(n)


def tag_bits(m: int) -> int:
    return int(lib().orc_tag_bits(C.c_int(m)))


def tag_keys(x: np.ndarray, field_off: np.ndarray, field_tag: np.ndarray, k: int) -> Tuple[np.ndarray, int]:
    x = np.ascontiguousarray(x, dtype=np.uint64)
    field_off = np.ascontiguousarray(field_off, dtype=np.int64)
    field_tag = np.ascontiguousarray(field_tag, dtype=np.uint8)
    out = np.empty_like(x)
    err = C.c_int64(0)
    rc = lib().orc_tag_keys(_p(x, C.c_uint64), _p(field_off, C.c_int64), _p(field_tag, C.c_uint8),
                            C.c_int(len(field_tag)), C.c_int(k), _p(out, C.c_uint64), C.byref(err))
    if rc != 0:
        raise ValueError(f"orc_tag_keys rc={rc}")
    return out, int(err.value)


def dedup(key: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    key = np.ascontiguousarray(key, dtype=np.uint64)
    n = len(key)
    uniq = np.empty(n, dtype=np.uint64)
    inverse = np.empty(n, dtype=np.int32)
    counts = np.empty(n, dtype=np.int32)
    U = lib().orc_dedup(_p(key, C.c_uint64), C.c_int64(n), _p(uniq, C.c_uint64), _p(inverse, C.c_int32),
                        _p(counts, C.c_int32))
    return uniq[:U].copy(), inverse, counts[:U].copy()


def init_row(key: int, dim: int, dtype: int = F32, init_scale: float = 0.01) -> np.ndarray:
    out = np.empty(dim, dtype=np.float32)
    lib().orc_init_row(C.c_uint64(key), C.c_int(dim), C.c_int(dtype), C.c_float(init_scale), _p(out, C.c_float))
    return out


def expand(uniq_rows: np.ndarray, inverse: np.ndarray) -> np.ndarray:
    uniq_rows = np.ascontiguousarray(uniq_rows, dtype=np.float32)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    n, dim = len(inverse), uniq_rows.shape[1]
    out = np.empty((n, dim), dtype=np.float32)
    lib().orc_expand(_p(uniq_rows, C.c_float), _p(inverse, C.c_int32), C.c_int64(n), C.c_int(dim), _p(out, C.c_float))
    return out


def segment_reduce(grad: np.ndarray, inverse: np.ndarray, n_unique: int) -> np.ndarray:
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    n, dim = grad.shape
    out = np.empty((n_unique, dim), dtype=np.float32)
    rc = lib().orc_segment_reduce(_p(grad, C.c_float), _p(inverse, C.c_int32), C.c_int64(n), C.c_int64(n_unique),
                                  C.c_int(dim), _p(out, C.c_float))
    if rc != 0:
        raise ValueError("inverse index out of range")
    return out


def pool_bags(E: np.ndarray, bag_off: np.ndarray, mean: bool) -> np.ndarray:
    E = np.ascontiguousarray(E, dtype=np.float32)
    bag_off = np.ascontiguousarray(bag_off, dtype=np.int64)
    nb, dim = len(bag_off) - 1, E.shape[1]
    out = np.empty((nb, dim), dtype=np.float32)
    rc = lib().orc_pool_bags(_p(E, C.c_float), _p(bag_off, C.c_int64), C.c_int64(nb), C.c_int(dim), C.c_int(int(mean)),
                             _p(out, C.c_float))
    if rc != 0:
        raise ValueError("bag offsets must be non-decreasing")
    return out


def pool_bags_backward(d_pooled: np.ndarray, bag_off: np.ndarray, mean: bool) -> np.ndarray:
    d_pooled = np.ascontiguousarray(d_pooled, dtype=np.float32)
    bag_off = np.ascontiguousarray(bag_off, dtype=np.int64)
    nb, dim = d_pooled.shape
    G = np.empty((int(bag_off[-1]), dim), dtype=np.float32)
    lib().orc_pool_bags_backward(_p(d_pooled, C.c_float), _p(bag_off, C.c_int64), C.c_int64(nb), C.c_int(dim),
                                 C.c_int(int(mean)), _p(G, C.c_float))
    return G


def float_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    lib().orc_float_to_bf16(_p(a, C.c_float), C.c_int64(a.size), _p(out, C.c_uint16))
    return out


def bf16_bits_to_float(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.uint16)
    out = np.empty(a.shape, dtype=np.float32)
    lib().orc_bf16_to_float(_p(a, C.c_uint16), C.c_int64(a.size), _p(out, C.c_float))
    return out


class Table:
    """key -> (row, acc, last_seen, freq) map with the checker's semantics."""

    def __init__(self, dim: int, dtype: int = F32, init_scale: float = 0.01):
        self.dim, self.dtype, self.init_scale = dim, dtype, init_scale
        self._h = C.c_void_p(lib().orc_table_create(C.c_int(dim), C.c_int(dtype), C.c_float(init_scale)))
        if not self._h:
            raise ValueError("bad table description")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.orc_table_destroy(self._h)
            self._h = None

    def __len__(self) -> int:
        return int(lib().orc_size(self._h))

    @staticmethod
    def _keys(key) -> np.ndarray:
        return np.ascontiguousarray(key, dtype=np.uint64)

    def find_or_insert(self, key, step: int) -> np.ndarray:
        key = self._keys(key)
        ins = np.zeros(len(key), dtype=np.uint8)
        rc = lib().orc_find_or_insert(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), C.c_uint32(step),
                                      _p(ins, C.c_uint8))
        if rc != 0:
            raise ValueError(f"orc_find_or_insert rc={rc}")
        return ins

    def prepopulate(self, key) -> None:
        key = self._keys(key)
        rc = lib().orc_prepopulate(self._h, _p(key, C.c_uint64), C.c_int64(len(key)))
        if rc != 0:
            raise ValueError(f"orc_prepopulate rc={rc}")

    def find(self, key) -> np.ndarray:
        key = self._keys(key)
        out = np.zeros(len(key), dtype=np.uint8)
        lib().orc_find(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), _p(out, C.c_uint8))
        return out

    def lookup(self, key) -> np.ndarray:
        key = self._keys(key)
        out = np.empty((len(key), self.dim), dtype=np.float32)
        lib().orc_lookup(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), _p(out, C.c_float))
        return out

    def direct_lookup(self, key, step: int) -> np.ndarray:
        key = self._keys(key)
        out = np.empty((len(key), self.dim), dtype=np.float32)
        rc = lib().orc_direct_lookup(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), C.c_uint32(step),
                                     _p(out, C.c_float))
        if rc != 0:
            raise ValueError(f"orc_direct_lookup rc={rc}")
        return out

    def apply_adagrad(self, key, g: np.ndarray, lr: float, eps: float = 1e-8) -> None:
        key = self._keys(key)
        g = np.ascontiguousarray(g, dtype=np.float32)
        assert g.shape == (len(key), self.dim)
        lib().orc_apply_adagrad(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), _p(g, C.c_float),
                                C.c_float(lr), C.c_float(eps))

    def apply_adam(self, key, g: np.ndarray, lr: float, step: int, beta1: float = 0.9, beta2: float = 0.999,
                   eps: float = 1e-8) -> None:
        key = self._keys(key)
        g = np.ascontiguousarray(g, dtype=np.float32)
        assert g.shape == (len(key), self.dim)
        rc = lib().orc_apply_adam(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), _p(g, C.c_float), C.c_float(lr),
                                  C.c_float(beta1), C.c_float(beta2), C.c_float(eps), C.c_int64(step))
        if rc != 0:
            raise ValueError("step must be >= 1")

    def set_hot(self, capacity: int) -> None:
        """Give a 16-bit table a hot store of `capacity` fp32 masters (App. C, mixed precision)."""
        if lib().orc_set_hot(self._h, C.c_int64(capacity)) != 0:
            raise ValueError("hot rows need a bf16 table and a positive capacity")

    def promote(self, key, min_freq: int) -> int:
        key = self._keys(key)
        return int(lib().orc_promote(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), C.c_uint32(min_freq)))

    def demote(self, now: int, idle: int) -> int:
        """Hot rows untouched for `idle` steps become cold again (master rounded into the 16-bit row); how many."""
        return int(lib().orc_demote(self._h, C.c_uint32(now), C.c_uint32(idle)))

    def put(self, key, values, acc, last_seen, freq) -> int:
        """Restore dumped entries of keys that are present (rows as delivered, accumulators, last-seen steps, touch counts)."""
        key = self._keys(key)
        values = np.ascontiguousarray(values, dtype=np.float32)
        acc = np.ascontiguousarray(acc, dtype=np.float32)
        last_seen = np.ascontiguousarray(last_seen, dtype=np.uint32)
        freq = np.ascontiguousarray(freq, dtype=np.uint32)
        assert values.shape == (len(key), self.dim) and len(acc) == len(last_seen) == len(freq) == len(key)
        return int(lib().orc_put(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), _p(values, C.c_float), _p(acc, C.c_float),
                                 _p(last_seen, C.c_uint32), _p(freq, C.c_uint32)))

    def put_hot(self, key, values) -> int:
        """Masters of the listed hot keys := values (fp32 [n, dim]); absent or cold keys are skipped; how many written."""
        key = self._keys(key)
        values = np.ascontiguousarray(values, dtype=np.float32)
        assert values.shape == (len(key), self.dim)
        return int(lib().orc_put_hot(self._h, _p(key, C.c_uint64), C.c_int64(len(key)), _p(values, C.c_float)))

    def export_hot(self):
        n = int(lib().orc_export_hot(self._h, None, None))
        keys = np.empty(n, dtype=np.uint64)
        values = np.empty((n, self.dim), dtype=np.float32)
        lib().orc_export_hot(self._h, _p(keys, C.c_uint64), _p(values, C.c_float))
        return keys, values

    def evict(self, now: int, ttl: int, min_freq: int, grace: int) -> np.ndarray:
        out = np.empty(len(self), dtype=np.uint64)
        n = lib().orc_evict(self._h, C.c_uint32(now), C.c_uint32(ttl), C.c_uint32(min_freq), C.c_uint32(grace),
                            _p(out, C.c_uint64))
        return out[:n].copy()

    def export(self):
        n = len(self)
        keys = np.empty(n, dtype=np.uint64)
        values = np.empty((n, self.dim), dtype=np.float32)
        acc = np.empty(n, dtype=np.float32)
        last_seen = np.empty(n, dtype=np.uint32)
        freq = np.empty(n, dtype=np.uint32)
        lib().orc_export(self._h, _p(keys, C.c_uint64), _p(values, C.c_float), _p(acc, C.c_float),
                         _p(last_seen, C.c_uint32), _p(freq, C.c_uint32))
        return keys, values, acc, last_seen, freq

    def peek(self, key):
        key = self._keys(key)
        n = len(key)
        present = np.zeros(n, dtype=np.uint8)
        values = np.zeros((n, self.dim), dtype=np.float32)
        acc = np.zeros(n, dtype=np.float32)
        last_seen = np.zeros(n, dtype=np.uint32)
        freq = np.zeros(n, dtype=np.uint32)
        lib().orc_peek(self._h, _p(key, C.c_uint64), C.c_int64(n), _p(present, C.c_uint8), _p(values, C.c_float),
                       _p(acc, C.c_float), _p(last_seen, C.c_uint32), _p(freq, C.c_uint32))
        return present, values, acc, last_seen, freq
