"""ctypes binding of libmtgr_emb.so: same names as the C entry points, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device memory; every step of the path runs
in the library's HIP kernels.  There is no CPU fallback: if the shared library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

F32, BF16 = 0, 1
EMB_OK = 0
EMB_ERR_NO_STORAGE = -4
EMB_ERR_NEED_REHASH = -6
EMB_CHECK_STATUS = 1
EMB_ERR_TOO_LARGE = -7
EMB_DEDUP_NOALLOC_MAX_KEYS = 1 << 20
DEV_PROBE_EXHAUSTED, DEV_OUT_OF_ROWS, DEV_BAD_KEY, DEV_NEED_REHASH = 1, 2, 4, 8

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmtgr_emb.so")
_lib = None


class EmbError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class TableDesc(C.Structure):
    _fields_ = [("dim", C.c_int32), ("dtype", C.c_int32), ("init_scale", C.c_float),
                ("max_load_factor", C.c_float), ("chunk_rows_log2", C.c_int32), ("count_probes", C.c_int32)]


class HtStats(C.Structure):
    _fields_ = ([(n, C.c_uint64) for n in
                 ("live", "tombstones", "capacity", "rows_used", "rows_free", "rows_capacity", "n_rehash",
                  "n_chunks", "status", "lookups", "probes", "cas_attempts", "cas_failures", "alloc_atomics",
                  "hot_rows_used", "hot_rows_free", "hot_rows_capacity")]
                + [("probe_hist", C.c_uint64 * 8), ("refused", C.c_uint64), ("occupied", C.c_uint64)])

    def as_dict(self):
        d = {n: int(getattr(self, n)) for n, _ in self._fields_ if n != "probe_hist"}
        d["probe_hist"] = [int(v) for v in self.probe_hist]
        return d


EXPORTS = [
    "emb_tag_bits", "emb_plan_merge", "ht_probe_line", "emb_status_string", "emb_table_state_bytes",
    "emb_table_create", "emb_table_destroy", "ht_set_key_storage", "ht_add_chunk", "ht_add_chunk_adam_state", "ht_plan", "ht_rehash",
    "ht_stats", "emb_tag_keys", "emb_dedup_workspace_bytes", "emb_dedup", "ht_find_or_insert", "ht_find",
    "ht_gather", "emb_expand", "emb_expand_sorted", "grad_segment_reduce_workspace_bytes", "grad_segment_reduce",
    "ht_apply_adagrad", "ht_apply_adam", "ht_gather_expand_sorted", "emb_pool_workspace_bytes", "emb_pool_bags",
    "grad_segment_reduce_pooled", "ht_evict", "ht_export", "ht_put", "ht_set_hot_storage", "ht_promote", "ht_demote", "ht_put_hot", "ht_export_hot",
    "ht_find_or_insert_notouch", "ht_apply_adagrad_touch", "grad_reduce_apply_adagrad",
    "ht_find_or_insert_retry", "ht_clear_status", "emb_dedup_noalloc",
    "emb_tag_dedup_workspace_bytes", "emb_tag_dedup", "emb_probe_memory",
]


def load():
    """Load the built library (build it first with ``python -m paper_2505_12663_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2505_12663_amd.build` (needs hipcc)")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32, u32, u64, f32 = C.c_void_p, C.c_int64, C.c_int, C.c_uint32, C.c_uint64, C.c_float
    sig = {
        "emb_tag_bits": (C.c_int, [i32]),
        "emb_plan_merge": (C.c_int, [vp, vp, i32, vp]),
        "ht_probe_line": (u64, [u64, i32, u64]),
        "emb_status_string": (C.c_char_p, [i32]),
        "emb_table_state_bytes": (C.c_size_t, []),
        "emb_table_create": (C.c_int, [C.POINTER(vp), C.POINTER(TableDesc), vp, C.c_size_t, vp]),
        "emb_table_destroy": (C.c_int, [vp]),
        "ht_set_key_storage": (C.c_int, [vp, vp, i32, vp]),
        "ht_add_chunk": (C.c_int, [vp, vp, vp, vp, vp]),
        "ht_add_chunk_adam_state": (C.c_int, [vp, vp, vp, vp]),
        "ht_plan": (C.c_int, [vp, i64, C.POINTER(C.c_int), C.POINTER(C.c_int)]),
        "ht_rehash": (C.c_int, [vp, vp, i32, vp]),
        "ht_stats": (C.c_int, [vp, C.POINTER(HtStats), vp]),
        "emb_tag_keys": (C.c_int, [vp, vp, vp, i32, i64, i32, vp, vp, vp]),
        "emb_dedup_workspace_bytes": (C.c_size_t, [i64]),
        "emb_dedup": (C.c_int, [vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]),
        "emb_tag_dedup_workspace_bytes": (C.c_size_t, [i64, i32, i32, i32]),
        "emb_tag_dedup": (C.c_int, [vp, vp, vp, i32, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]),
        "emb_dedup_noalloc": (C.c_int, [vp, i64, vp, vp, vp, vp, vp, vp, vp, vp]),
        "emb_probe_memory": (C.c_int, [i32, vp, vp, vp, i64, vp]),
        "ht_find_or_insert": (C.c_int, [vp, vp, vp, i64, u32, vp, vp, vp]),
        "ht_find_or_insert_notouch": (C.c_int, [vp, vp, vp, i64, u32, vp, vp, vp]),
        "ht_find_or_insert_retry": (C.c_int, [vp, vp, vp, i64, u32, vp, vp, i32, vp]),
        "ht_clear_status": (C.c_int, [vp, u32, vp]),
        "ht_apply_adagrad_touch": (C.c_int, [vp, vp, vp, vp, i64, f32, f32, u32, vp]),
        "grad_reduce_apply_adagrad": (C.c_int, [vp, vp, vp, vp, i64, vp, f32, f32, i32, u32, vp, C.c_size_t, vp]),
        "ht_find": (C.c_int, [vp, vp, vp, i64, vp, vp]),
        "ht_gather": (C.c_int, [vp, vp, vp, i64, vp, vp]),
        "emb_expand": (C.c_int, [vp, vp, i64, i32, i32, vp, vp]),
        "emb_expand_sorted": (C.c_int, [vp, vp, vp, i64, i32, i32, vp, vp]),
        "grad_segment_reduce_workspace_bytes": (C.c_size_t, [i64, i32]),
        "grad_segment_reduce": (C.c_int, [vp, i32, vp, vp, i64, i32, vp, vp, C.c_size_t, vp]),
        "ht_apply_adagrad": (C.c_int, [vp, vp, vp, vp, i64, f32, f32, vp]),
        "ht_apply_adam": (C.c_int, [vp, vp, vp, vp, i64, f32, f32, f32, f32, i64, vp]),
        "ht_gather_expand_sorted": (C.c_int, [vp, vp, vp, vp, i64, vp, vp]),
        "emb_pool_workspace_bytes": (C.c_size_t, [i64, i32, i32]),
        "emb_pool_bags": (C.c_int, [vp, i32, vp, vp, i32, i64, i32, i32, vp, vp, C.c_size_t, vp]),
        "grad_segment_reduce_pooled": (C.c_int, [vp, vp, i32, vp, vp, i64, i32, i32, vp, vp, C.c_size_t, vp]),
        "ht_evict": (C.c_int, [vp, u32, u32, u32, u32, vp, i64, vp, vp]),
        "ht_export": (C.c_int, [vp, vp, vp, vp, vp, vp, i64, vp, vp]),
        "ht_put": (C.c_int, [vp, vp, vp, vp, vp, vp, i64, vp]),
        "ht_set_hot_storage": (C.c_int, [vp, vp, vp, i64, vp]),
        "ht_promote": (C.c_int, [vp, vp, vp, i64, u32, vp, vp]),
        "ht_demote": (C.c_int, [vp, u32, u32, vp, vp]),
        "ht_put_hot": (C.c_int, [vp, vp, vp, i64, vp, vp]),
        "ht_export_hot": (C.c_int, [vp, vp, vp, i64, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def status_string(status: int) -> str:
    return load().emb_status_string(status).decode()


def _check(rc: int, where: str) -> None:
    if rc != EMB_OK:
        raise EmbError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


# ------------------------------------------------------------------------------------------ host-only
def emb_tag_bits(m: int) -> int:
    return int(load().emb_tag_bits(m))


def emb_plan_merge(dims, dtypes):
    import numpy as np
    dims = np.ascontiguousarray(dims, dtype=np.int32)
    dtypes = np.ascontiguousarray(dtypes, dtype=np.int32)
    out = np.empty(len(dims), dtype=np.int32)
    n = load().emb_plan_merge(dims.ctypes.data, dtypes.ctypes.data, len(dims), out.ctypes.data)
    if n < 0:
        raise EmbError(n, "emb_plan_merge")
    return out, int(n)


def ht_probe_line(key: int, capacity_log2: int, t: int) -> int:
    return int(load().ht_probe_line(key, capacity_log2, t))


# ------------------------------------------------------------------------------------------ device calls
def emb_table_state_bytes() -> int:
    return int(load().emb_table_state_bytes())


def emb_table_create(desc: TableDesc, state: torch.Tensor, stream=None):
    h = C.c_void_p()
    _check(load().emb_table_create(C.byref(h), C.byref(desc), _ptr(state), state.numel() * state.element_size(),
                                   _stream(stream)), "emb_table_create")
    return h


def emb_table_destroy(h) -> None:
    _check(load().emb_table_destroy(h), "emb_table_destroy")


def ht_set_key_storage(h, slots, capacity_log2: int, stream=None) -> None:
    assert slots.numel() * slots.element_size() == 16 << capacity_log2
    _check(load().ht_set_key_storage(h, _ptr(slots), capacity_log2, _stream(stream)), "ht_set_key_storage")


def ht_add_chunk(h, values, meta, free_list, stream=None) -> None:
    _check(load().ht_add_chunk(h, _ptr(values), _ptr(meta), _ptr(free_list), _stream(stream)), "ht_add_chunk")


def ht_add_chunk_adam_state(h, m, v, stream=None) -> None:
    _check(load().ht_add_chunk_adam_state(h, _ptr(m), _ptr(v), _stream(stream)), "ht_add_chunk_adam_state")


def ht_plan(h, n_incoming: int):
    cap, chunks = C.c_int(0), C.c_int(0)
    _check(load().ht_plan(h, n_incoming, C.byref(cap), C.byref(chunks)), "ht_plan")
    return cap.value, chunks.value


def ht_rehash(h, new_slots, new_capacity_log2: int, stream=None) -> None:
    assert new_slots.numel() * new_slots.element_size() == 16 << new_capacity_log2
    _check(load().ht_rehash(h, _ptr(new_slots), new_capacity_log2, _stream(stream)), "ht_rehash")


def ht_stats(h, stream=None) -> dict:
    st = HtStats()
    _check(load().ht_stats(h, C.byref(st), _stream(stream)), "ht_stats")
    return st.as_dict()


def emb_tag_keys(x, field_off, field_tag, tag_bits: int, key_out, err_count, stream=None) -> None:
    _check(load().emb_tag_keys(_ptr(x), _ptr(field_off), _ptr(field_tag), field_tag.numel(), x.numel(), tag_bits,
                               _ptr(key_out), _ptr(err_count), _stream(stream)), "emb_tag_keys")


def emb_dedup_workspace_bytes(n: int) -> int:
    return int(load().emb_dedup_workspace_bytes(n))


def emb_dedup(key, n: int, uniq, inverse, counts, perm, seg_off, seg_of, n_unique, workspace, stream=None) -> None:
    _check(load().emb_dedup(_ptr(key), n, _ptr(uniq), _ptr(inverse), _ptr(counts), _ptr(perm), _ptr(seg_off),
                            _ptr(seg_of), _ptr(n_unique), _ptr(workspace), workspace.numel() * workspace.element_size(),
                            _stream(stream)), "emb_dedup")


def emb_tag_dedup_workspace_bytes(n: int, n_fields: int, tag_bits: int, id_bits: int) -> int:
    return int(load().emb_tag_dedup_workspace_bytes(n, n_fields, tag_bits, id_bits))


def emb_tag_dedup(x, field_off, field_tag, tag_bits: int, id_bits: int, key_out, uniq, inverse, counts, perm, seg_off, seg_of,
                  n_unique, err_count, workspace, stream=None) -> None:
    _check(load().emb_tag_dedup(_ptr(x), _ptr(field_off), _ptr(field_tag), field_tag.numel(), x.numel(), tag_bits, id_bits,
                                _ptr(key_out), _ptr(uniq), _ptr(inverse), _ptr(counts), _ptr(perm), _ptr(seg_off), _ptr(seg_of),
                                _ptr(n_unique), _ptr(err_count), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                _stream(stream)), "emb_tag_dedup")


def emb_dedup_noalloc(key, n: int, uniq, inverse, counts, perm, seg_off, seg_of, n_unique, stream=None) -> None:
    _check(load().emb_dedup_noalloc(_ptr(key), n, _ptr(uniq), _ptr(inverse), _ptr(counts), _ptr(perm), _ptr(seg_off),
                                    _ptr(seg_of), _ptr(n_unique), _stream(stream)), "emb_dedup_noalloc")


PROBE_READ, PROBE_WRITE, PROBE_READ_STORE_4TH, PROBE_READ_STORE_64TH = 0, 1, 2, 3


def emb_probe_memory(pattern: int, src, dst, idx, rows: int, stream=None) -> None:
    """One launch of a bare access pattern over 256-byte rows (a measuring aid, see mtgr_emb.h)."""
    _check(load().emb_probe_memory(pattern, _ptr(src), _ptr(dst), _ptr(idx), rows, _stream(stream)), "emb_probe_memory")


def ht_find_or_insert(h, key, n_dev, n_max: int, step: int, row_idx, inserted=None, stream=None, touch: bool = True) -> int:
    """Returns EMB_OK or EMB_CHECK_STATUS (launched, but new keys may have been turned away); raises on errors.
    touch=False calls ht_find_or_insert_notouch."""
    fn = load().ht_find_or_insert if touch else load().ht_find_or_insert_notouch
    rc = fn(h, _ptr(key), _ptr(n_dev), n_max, step, _ptr(row_idx), _ptr(inserted), _stream(stream))
    if rc < 0:
        raise EmbError(rc, "ht_find_or_insert" if touch else "ht_find_or_insert_notouch")
    return rc


def ht_find_or_insert_retry(h, key, n_dev, n_max: int, step: int, row_idx, inserted=None, touch: bool = True, stream=None) -> int:
    rc = load().ht_find_or_insert_retry(h, _ptr(key), _ptr(n_dev), n_max, step, _ptr(row_idx), _ptr(inserted), int(touch),
                                        _stream(stream))
    if rc < 0:
        raise EmbError(rc, "ht_find_or_insert_retry")
    return rc


def ht_clear_status(h, bits: int, stream=None) -> None:
    _check(load().ht_clear_status(h, bits, _stream(stream)), "ht_clear_status")


def ht_find(h, key, n_dev, n_max: int, row_idx, stream=None) -> None:
    _check(load().ht_find(h, _ptr(key), _ptr(n_dev), n_max, _ptr(row_idx), _stream(stream)), "ht_find")


def ht_gather(h, row_idx, n_dev, n_max: int, out, stream=None) -> None:
    _check(load().ht_gather(h, _ptr(row_idx), _ptr(n_dev), n_max, _ptr(out), _stream(stream)), "ht_gather")


def emb_expand(uniq_rows, inverse, n: int, dim: int, dtype: int, out, stream=None) -> None:
    _check(load().emb_expand(_ptr(uniq_rows), _ptr(inverse), n, dim, dtype, _ptr(out), _stream(stream)), "emb_expand")


def emb_expand_sorted(uniq_rows, seg_of, perm, n: int, dim: int, dtype: int, out, stream=None) -> None:
    _check(load().emb_expand_sorted(_ptr(uniq_rows), _ptr(seg_of), _ptr(perm), n, dim, dtype, _ptr(out), _stream(stream)),
           "emb_expand_sorted")


def grad_segment_reduce_workspace_bytes(n: int, dim: int) -> int:
    return int(load().grad_segment_reduce_workspace_bytes(n, dim))


def grad_segment_reduce(grad, grad_dtype: int, seg_of, perm, n: int, dim: int, reduced, workspace, stream=None) -> None:
    _check(load().grad_segment_reduce(_ptr(grad), grad_dtype, _ptr(seg_of), _ptr(perm), n, dim, _ptr(reduced),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "grad_segment_reduce")


def ht_apply_adagrad(h, row_idx, reduced, n_dev, n_max: int, lr: float, eps: float, stream=None) -> None:
    _check(load().ht_apply_adagrad(h, _ptr(row_idx), _ptr(reduced), _ptr(n_dev), n_max, lr, eps, _stream(stream)),
           "ht_apply_adagrad")


def ht_apply_adagrad_touch(h, row_idx, reduced, n_dev, n_max: int, lr: float, eps: float, step: int, stream=None) -> None:
    _check(load().ht_apply_adagrad_touch(h, _ptr(row_idx), _ptr(reduced), _ptr(n_dev), n_max, lr, eps, step,
                                         _stream(stream)), "ht_apply_adagrad_touch")


def ht_apply_adam(h, row_idx, reduced, n_dev, n_max: int, lr: float, beta1: float, beta2: float, eps: float, step: int,
                  stream=None) -> None:
    _check(load().ht_apply_adam(h, _ptr(row_idx), _ptr(reduced), _ptr(n_dev), n_max, lr, beta1, beta2, eps, step,
                                _stream(stream)), "ht_apply_adam")


def ht_gather_expand_sorted(h, row_idx, seg_of, perm, n: int, out, stream=None) -> None:
    _check(load().ht_gather_expand_sorted(h, _ptr(row_idx), _ptr(seg_of), _ptr(perm), n, _ptr(out), _stream(stream)),
           "ht_gather_expand_sorted")


def emb_pool_workspace_bytes(n: int, n_bags: int, dim: int) -> int:
    return int(load().emb_pool_workspace_bytes(n, n_bags, dim))


def emb_pool_bags(uniq_rows, dtype: int, inverse, bag_off, n: int, dim: int, mean: bool, pooled, workspace, stream=None) -> None:
    _check(load().emb_pool_bags(_ptr(uniq_rows), dtype, _ptr(inverse), _ptr(bag_off), bag_off.numel() - 1, n, dim,
                                int(mean), _ptr(pooled), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                _stream(stream)), "emb_pool_bags")


def grad_segment_reduce_pooled(d_pooled, bag_off, seg_of, perm, n: int, dim: int, mean: bool, reduced, workspace,
                               stream=None) -> None:
    _check(load().grad_segment_reduce_pooled(_ptr(d_pooled), _ptr(bag_off), bag_off.numel() - 1, _ptr(seg_of), _ptr(perm),
                                             n, dim, int(mean), _ptr(reduced), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)),
           "grad_segment_reduce_pooled")


def ht_evict(h, now: int, ttl: int, min_freq: int, grace: int, evicted_keys, n_evicted, stream=None) -> None:
    cap = 0 if evicted_keys is None else evicted_keys.numel()
    _check(load().ht_evict(h, now, ttl, min_freq, grace, _ptr(evicted_keys), cap, _ptr(n_evicted), _stream(stream)),
           "ht_evict")


def ht_export(h, keys, values, acc, last_seen, freq, n, stream=None) -> None:
    _check(load().ht_export(h, _ptr(keys), _ptr(values), _ptr(acc), _ptr(last_seen), _ptr(freq), keys.numel(), _ptr(n),
                            _stream(stream)), "ht_export")


def ht_put(h, row_idx, values, acc, last_seen, freq, n: int, stream=None) -> None:
    _check(load().ht_put(h, _ptr(row_idx), _ptr(values), _ptr(acc), _ptr(last_seen), _ptr(freq), n, _stream(stream)),
           "ht_put")


def ht_set_hot_storage(h, hot_values, hot_free, hot_rows: int, stream=None) -> None:
    _check(load().ht_set_hot_storage(h, _ptr(hot_values), _ptr(hot_free), hot_rows, _stream(stream)), "ht_set_hot_storage")


def ht_promote(h, row_idx, n_dev, n_max: int, min_freq: int, n_promoted=None, stream=None) -> None:
    _check(load().ht_promote(h, _ptr(row_idx), _ptr(n_dev), n_max, min_freq, _ptr(n_promoted), _stream(stream)),
           "ht_promote")


def ht_demote(h, now: int, idle: int, n_demoted=None, stream=None) -> None:
    _check(load().ht_demote(h, now, idle, _ptr(n_demoted), _stream(stream)), "ht_demote")


def ht_put_hot(h, row_idx, masters, n: int, n_written=None, stream=None) -> None:
    _check(load().ht_put_hot(h, _ptr(row_idx), _ptr(masters), n, _ptr(n_written), _stream(stream)), "ht_put_hot")


def ht_export_hot(h, keys, values, n, stream=None) -> None:
    _check(load().ht_export_hot(h, _ptr(keys), _ptr(values), keys.numel(), _ptr(n), _stream(stream)), "ht_export_hot")


def grad_reduce_apply_adagrad(h, grad, seg_of, perm, n: int, row_idx, lr: float, eps: float, touch_step, ws, stream=None) -> None:
    """touch_step None: plain update; an int: the update also stamps last_seen = touch_step and counts a touch."""
    _check(load().grad_reduce_apply_adagrad(h, _ptr(grad), _ptr(seg_of), _ptr(perm), n, _ptr(row_idx), lr, eps,
                                            0 if touch_step is None else 1, 0 if touch_step is None else touch_step,
                                            _ptr(ws), ws.numel(), _stream(stream)), "grad_reduce_apply_adagrad")
