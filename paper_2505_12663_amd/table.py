"""Storage owner for one merged hash table and the buffers of one lookup step.

The C library allocates nothing; this module keeps the torch tensors that back the key
structure, the value chunks and the per-step buffers alive, and applies the capacity policy the
library plans (``ht_plan``): rehash the key structure when the device turned new keys away at the
load-factor limit, keep a spare value chunk registered (dual-chunk rule of Sec. 3.1).  All arithmetic of the path
runs in the library's kernels.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as B


def _np_to_dev_i64(a: np.ndarray, device) -> torch.Tensor:
    """uint64 numpy keys -> int64 device tensor holding the same bits."""
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return torch.from_numpy(a.view(np.int64)).to(device)


class EmbeddingTable:
    """One dynamic hash table (possibly holding several merged logical tables)."""

    def __init__(self, dim: int, dtype: int = B.F32, capacity_log2: int = 18, chunk_rows_log2: int = 16,
                 init_scale: float = 0.01, max_load_factor: float = 0.75, count_probes: bool = False,
                 device: str = "cuda:0", initial_chunks: int = 2, adam_state: bool = False, hot_rows: int = 0):
        self.device = torch.device(device)
        self.dim, self.dtype = dim, dtype
        self.chunk_rows_log2 = chunk_rows_log2
        self.adam_state = adam_state
        self.torch_dtype = torch.float32 if dtype == B.F32 else torch.bfloat16
        self.state = torch.empty(B.emb_table_state_bytes(), dtype=torch.uint8, device=self.device)
        desc = B.TableDesc(dim, dtype, init_scale, max_load_factor, chunk_rows_log2, int(count_probes))
        self.h = B.emb_table_create(desc, self.state)
        self._refused_seen = 0
        self.peak_load = 0.0          # highest (live + deleted) / capacity any counter read-back has shown
        self.capacity_log2 = capacity_log2
        self.slots = torch.empty((1 << capacity_log2, 2), dtype=torch.int64, device=self.device)   # 16 B per slot
        B.ht_set_key_storage(self.h, self.slots, capacity_log2)
        self.chunks: List[tuple] = []
        for _ in range(initial_chunks):
            self.add_chunk()
        self.hot_rows = hot_rows
        if hot_rows > 0:   # fp32 masters for frequently used keys of a 16-bit table
            self.hot_values = torch.empty((hot_rows, dim), dtype=torch.float32, device=self.device)
            self.hot_free = torch.empty(hot_rows, dtype=torch.int32, device=self.device)
            B.ht_set_hot_storage(self.h, self.hot_values, self.hot_free, hot_rows)

    def close(self) -> None:
        if self.h is not None:
            torch.cuda.synchronize(self.device)
            B.emb_table_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- storage ------------------------------------------------------------------------------
    def add_chunk(self) -> None:
        n = 1 << self.chunk_rows_log2
        values = torch.empty((n, self.dim), dtype=self.torch_dtype, device=self.device)
        meta = torch.empty((n, 4), dtype=torch.int32, device=self.device)        # 16 bytes per row
        free_list = torch.empty(n, dtype=torch.int32, device=self.device)
        B.ht_add_chunk(self.h, values, meta, free_list)
        chunk = (values, meta, free_list)
        if self.adam_state:
            m = torch.empty((n, self.dim), dtype=torch.float32, device=self.device)
            v = torch.empty((n, self.dim), dtype=torch.float32, device=self.device)
            B.ht_add_chunk_adam_state(self.h, m, v)
            chunk += (m, v)
        self.chunks.append(chunk)

    def rehash(self, new_capacity_log2: int) -> None:
        new_slots = torch.empty((1 << new_capacity_log2, 2), dtype=torch.int64, device=self.device)
        B.ht_rehash(self.h, new_slots, new_capacity_log2)
        # torch's caching allocator is stream-ordered: dropping the old array here is safe for
        # work queued on the current stream.
        self.slots, self.capacity_log2 = new_slots, new_capacity_log2

    def stats(self) -> dict:
        st = B.ht_stats(self.h)
        self.peak_load = max(self.peak_load, (st["live"] + st["tombstones"]) / max(st["capacity"], 1))
        return st

    def make_room(self, n_incoming: int) -> None:
        """Room for n_incoming more keys, from the exact counters (synchronises): add value chunks, and expand or
        clean the key structure if live + deleted + n_incoming slots would pass the load-factor limit."""
        self.stats()                       # exact counts replace the running upper bounds
        cap, chunks = B.ht_plan(self.h, n_incoming)
        for _ in range(chunks):
            self.add_chunk()
        if cap:
            self.rehash(cap)

    def _keep_spare_chunk(self, st: dict, n_next: int) -> None:
        """Dual-chunk rule of Sec. 3.1: besides the rows the next call may need, one whole chunk stays unused."""
        free_rows = st["rows_capacity"] - (st["rows_used"] - st["rows_free"])
        per = 1 << self.chunk_rows_log2
        while free_rows < n_next + per:
            self.add_chunk()
            free_rows += per

    # -- calls --------------------------------------------------------------------------------
    def find_or_insert(self, key, n_dev, n_max: int, step: int, row_idx, inserted=None, touch: bool = True) -> None:
        """touch=False: the step's update call (apply_adagrad with touch_step) counts the touch.
        The library admits new keys on the device up to the load-factor limit.  While its host-side bounds prove
        that everything fits, nothing here waits for the GPU; otherwise the counters are read back after the
        call and, if keys were turned away, room is made (rehash, chunks) and the call is issued again for them."""
        rc = B.ht_find_or_insert(self.h, key, n_dev, n_max, step, row_idx, inserted, touch=touch)
        if rc == B.EMB_OK:
            return
        for _ in range(4):
            st = self.stats()
            turned_away = st["refused"] - self._refused_seen
            self._refused_seen = st["refused"]
            if turned_away == 0:
                self._keep_spare_chunk(st, n_max)
                return
            # the bits the turned-away elements raised (a table filled to its last slot by claims that were
            # still being counted shows as an exhausted probe sequence); the retry must end with none of them
            B.ht_clear_status(self.h, B.DEV_NEED_REHASH | B.DEV_OUT_OF_ROWS | B.DEV_PROBE_EXHAUSTED)
            self.make_room(turned_away)
            B.ht_find_or_insert_retry(self.h, key, n_dev, n_max, step, row_idx, inserted, touch=touch)
        raise B.EmbError(B.EMB_ERR_NEED_REHASH, "ht_find_or_insert: keys still turned away after making room")

    def find(self, key, n_dev, n_max: int, row_idx) -> None:
        B.ht_find(self.h, key, n_dev, n_max, row_idx)

    def gather(self, row_idx, n_dev, n_max: int, out) -> None:
        B.ht_gather(self.h, row_idx, n_dev, n_max, out)

    def apply_adagrad(self, row_idx, reduced, n_dev, n_max: int, lr: float, eps: float = 1e-8,
                      touch_step: Optional[int] = None) -> None:
        if touch_step is None:
            B.ht_apply_adagrad(self.h, row_idx, reduced, n_dev, n_max, lr, eps)
        else:
            B.ht_apply_adagrad_touch(self.h, row_idx, reduced, n_dev, n_max, lr, eps, touch_step)

    def apply_adam(self, row_idx, reduced, n_dev, n_max: int, lr: float, step: int, beta1: float = 0.9,
                   beta2: float = 0.999, eps: float = 1e-8) -> None:
        B.ht_apply_adam(self.h, row_idx, reduced, n_dev, n_max, lr, beta1, beta2, eps, step)

    def evict(self, now: int, ttl: int, min_freq: int, grace: int, want_keys: bool = True):
        live = self.stats()["live"]
        n_ev = torch.zeros(1, dtype=torch.int64, device=self.device)
        keys = torch.empty(max(live, 1), dtype=torch.int64, device=self.device) if want_keys else None
        B.ht_evict(self.h, now, ttl, min_freq, grace, keys, n_ev)
        n = int(n_ev.item())
        self.stats()
        return (keys[:n] if want_keys else None), n

    def export(self):
        """Dump (keys, values, acc, last_seen, freq) sorted by key, as numpy arrays."""
        live = self.stats()["live"]
        cap = max(live, 1)
        keys = torch.empty(cap, dtype=torch.int64, device=self.device)
        values = torch.empty((cap, self.dim), dtype=self.torch_dtype, device=self.device)
        acc = torch.empty(cap, dtype=torch.float32, device=self.device)
        last_seen = torch.empty(cap, dtype=torch.int32, device=self.device)
        freq = torch.empty(cap, dtype=torch.int32, device=self.device)
        n = torch.zeros(1, dtype=torch.int64, device=self.device)
        B.ht_export(self.h, keys, values, acc, last_seen, freq, n)
        cnt = int(n.item())
        assert cnt == live, (cnt, live)
        k = keys[:cnt].cpu().numpy().view(np.uint64)
        order = np.argsort(k, kind="stable")
        vals = values[:cnt].float().cpu().numpy()
        return (k[order], vals[order], acc[:cnt].cpu().numpy()[order],
                last_seen[:cnt].cpu().numpy().view(np.uint32)[order], freq[:cnt].cpu().numpy().view(np.uint32)[order])

    def promote(self, row_idx, n_dev, n_max: int, min_freq: int, n_promoted=None) -> None:
        B.ht_promote(self.h, row_idx, n_dev, n_max, min_freq, n_promoted)

    def demote(self, now: int, idle: int, n_demoted=None) -> None:
        B.ht_demote(self.h, now, idle, n_demoted)

    def import_hot(self, keys, masters) -> int:
        """Restore dumped masters (keys int64 device tensor, masters fp32 [n, dim]): the keys must be in the table; each
        gets a master (while the store has room) holding the dumped values.  Returns how many masters were written."""
        n = keys.numel()
        if n == 0:
            return 0
        row_idx = torch.empty(n, dtype=torch.int32, device=self.device)
        self.find(keys.contiguous(), None, n, row_idx)
        self.promote(row_idx, None, n, 0)
        cnt = torch.zeros(1, dtype=torch.int64, device=self.device)
        B.ht_put_hot(self.h, row_idx, masters.contiguous(), n, cnt)
        return int(cnt.item())

    def export_hot(self):
        """Host copy of the fp32 masters, sorted by key: (keys uint64, values float32 [n, dim])."""
        cap = max(self.hot_rows, 1)
        keys = torch.empty(cap, dtype=torch.int64, device=self.device)
        values = torch.empty((cap, self.dim), dtype=torch.float32, device=self.device)
        n = torch.zeros(1, dtype=torch.int64, device=self.device)
        B.ht_export_hot(self.h, keys, values, n)
        cnt = int(n.item())
        k = keys[:cnt].cpu().numpy().view(np.uint64)
        order = np.argsort(k, kind="stable")
        return k[order], values[:cnt].cpu().numpy()[order]

    def export_device(self, values: bool = True):
        """Unordered dump as device tensors (keys int64, values or None, acc, last_seen, freq), trimmed to the live count."""
        live = self.stats()["live"]
        cap = max(live, 1)
        keys = torch.empty(cap, dtype=torch.int64, device=self.device)
        values = torch.empty((cap, self.dim), dtype=self.torch_dtype, device=self.device) if values else None
        acc = torch.empty(cap, dtype=torch.float32, device=self.device)
        last_seen = torch.empty(cap, dtype=torch.int32, device=self.device)
        freq = torch.empty(cap, dtype=torch.int32, device=self.device)
        n = torch.zeros(1, dtype=torch.int64, device=self.device)
        B.ht_export(self.h, keys, values, acc, last_seen, freq, n)
        cnt = int(n.item())
        return keys[:cnt], (values[:cnt] if values is not None else None), acc[:cnt], last_seen[:cnt], freq[:cnt]

    def import_rows(self, keys, values, acc, last_seen, freq, step: int = 0) -> None:
        """Restore dumped entries: create the keys, then overwrite row contents and records."""
        n = keys.numel()
        if n == 0:
            return
        row_idx = torch.empty(n, dtype=torch.int32, device=self.device)
        self.find_or_insert(keys.contiguous(), None, n, step, row_idx)
        B.ht_put(self.h, row_idx, values.contiguous(), acc.contiguous(), last_seen.contiguous(), freq.contiguous(), n)


class StepBuffers:
    """Device buffers of one forward+backward step over at most n_max IDs of one merged table."""

    def __init__(self, n_max: int, dim: int, dtype: int = B.F32, device: str = "cuda:0", with_grad: bool = True):
        dev = torch.device(device)
        tdt = torch.float32 if dtype == B.F32 else torch.bfloat16
        self.n_max, self.dim, self.dtype = n_max, dim, dtype
        self.key = torch.empty(n_max, dtype=torch.int64, device=dev)
        self.uniq = torch.empty(n_max, dtype=torch.int64, device=dev)
        self.inverse = torch.empty(n_max, dtype=torch.int32, device=dev)
        self.perm = torch.empty(n_max, dtype=torch.int32, device=dev)
        self.seg_off = torch.empty(n_max + 1, dtype=torch.int32, device=dev)
        self.seg_of = torch.empty(n_max, dtype=torch.int32, device=dev)
        self.counts = torch.empty(n_max, dtype=torch.int32, device=dev)
        self.n_unique = torch.zeros(1, dtype=torch.int64, device=dev)
        self.err_count = torch.zeros(1, dtype=torch.int64, device=dev)
        self.row_idx = torch.empty(n_max, dtype=torch.int32, device=dev)
        self.inserted = torch.empty(n_max, dtype=torch.uint8, device=dev)
        self.dedup_ws = torch.empty(B.emb_dedup_workspace_bytes(n_max), dtype=torch.uint8, device=dev)
        # emb_tag_dedup: the larger of its two internal forms (8-byte records / tag, then deduplicate)
        self.tag_dedup_ws = torch.empty(max(B.emb_tag_dedup_workspace_bytes(n_max, 1, 0, 32),
                                            B.emb_tag_dedup_workspace_bytes(n_max, 1, 0, 63)), dtype=torch.uint8, device=dev)
        self.uniq_rows = torch.empty((n_max, dim), dtype=tdt, device=dev)
        self.out = torch.empty((n_max, dim), dtype=tdt, device=dev)
        if with_grad:
            self.reduced = torch.empty((n_max, dim), dtype=torch.float32, device=dev)
            self.reduce_ws = torch.empty(B.grad_segment_reduce_workspace_bytes(n_max, dim), dtype=torch.uint8, device=dev)


def forward(table: EmbeddingTable, buf: StepBuffers, x, field_off, field_tag, tag_bits: int, step: int,
            touch: bool = True, id_bits: Optional[int] = None, want_keys: bool = True) -> None:
    """tag + dedup (one call) -> find-or-insert -> gather -> expand (in sorted order); results in buf.out[:n].
    id_bits: declared width of the raw IDs (default: everything Eq. 8 leaves, 63 - tag_bits).
    want_keys: also write the tagged keys to buf.key.
    touch=False leaves the rows' touch records to the update of the same step (backward with touch_step)."""
    n = x.numel()
    B.emb_tag_dedup(x, field_off, field_tag, tag_bits, (63 - tag_bits) if id_bits is None else id_bits,
                    buf.key if want_keys else None, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of,
                    buf.n_unique, buf.err_count, buf.tag_dedup_ws)
    table.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted, touch=touch)
    table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
    B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, table.dim, table.dtype, buf.out)


def forward_two_call(table: EmbeddingTable, buf: StepBuffers, x, field_off, field_tag, tag_bits: int, step: int,
                     touch: bool = True) -> None:
    """The same with emb_tag_keys and emb_dedup as separate calls (the tagged keys are materialised)."""
    n = x.numel()
    B.emb_tag_keys(x, field_off, field_tag, tag_bits, buf.key, buf.err_count)
    B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of, buf.n_unique,
                buf.dedup_ws)
    table.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted, touch=touch)
    table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
    B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, table.dim, table.dtype, buf.out)


def backward(table: EmbeddingTable, buf: StepBuffers, grad, n: int, lr: float, eps: float = 1e-8,
             touch_step: Optional[int] = None) -> None:
    """segment-reduce the upstream gradient per distinct key, then row-wise Adagrad (which also counts
    the step's touch when touch_step is given)."""
    B.grad_segment_reduce(grad, table.dtype, buf.seg_of, buf.perm, n, table.dim, buf.reduced, buf.reduce_ws)
    table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, lr, eps, touch_step)


def backward_fused(table: EmbeddingTable, buf: StepBuffers, grad, n: int, lr: float, eps: float = 1e-8,
                   touch_step: Optional[int] = None) -> None:
    """segment-reduce and row-wise Adagrad in one pass (buf.reduced is not written)."""
    B.grad_reduce_apply_adagrad(table.h, grad, buf.seg_of, buf.perm, n, buf.row_idx, lr, eps, touch_step, buf.reduce_ws)


def forward_fused(table: EmbeddingTable, buf: StepBuffers, x, field_off, field_tag, tag_bits: int, step: int) -> None:
    """tag -> dedup -> find-or-insert -> gather+expand in one kernel; results in buf.out[:n]
    (buf.uniq_rows is not written)."""
    n = x.numel()
    B.emb_tag_keys(x, field_off, field_tag, tag_bits, buf.key, buf.err_count)
    B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of, buf.n_unique,
                buf.dedup_ws)
    table.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted)
    B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n, buf.out)

