#!/usr/bin/env python3
"""Benchmark of the sparse-embedding step on one MI355X.

A step = tag -> dedup -> find-or-insert -> gather -> expand -> (upstream gradient already in HBM)
-> gradient segment-reduce -> row-wise Adagrad over one batch of the long-sequence lookup
configuration (batch 512, lengths U{256..4096}, 8 fields, dim 64 fp32, 50 M-key table, Zipf 1.05).
Inputs are resident in HBM when the timed region starts.  Prints ONE JSON line on stdout.

    python bench.py [--gpus 1] [--steps 20] [--warmup 3] [--config 2] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

HBM_PEAK_GBPS = 8000.0


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(n: int, u: int, u_new: int, v_row: int, v_grad: int, dim: int) -> dict:
    """Bytes the method itself must move per step (sort passes, probe overshoot and workspace
    traffic are overhead, not credit).  v_row / v_grad = bytes of a table row / a gradient row."""
    red_row = 4 * dim
    b = {
        "tag_dedup": 8 * n + 8 * u + 4 * n,
        "find_or_insert": (8 + 12 + 8) * u + (4 + 8) * u + u_new * (12 + v_row + 4 + 8 + 8),
        "gather": 4 * u + 2 * v_row * u,
        "expand": 4 * n + v_row * u + v_row * n,
        "reduce": v_grad * n + 4 * n + red_row * u,
        "adagrad": 4 * u + red_row * u + v_row * u + 4 * u + v_row * u + 4 * u,
    }
    b["total"] = sum(b.values())
    return b


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, choices=[2, 5])
    ap.add_argument("--batches", type=int, default=4, help="distinct pre-generated batches cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--touch-in-lookup", action="store_true",
                    help="ht_find_or_insert + ht_apply_adagrad (two updates of every row record per step) instead of "
                         "ht_find_or_insert_notouch + ht_apply_adagrad_touch (one)")
    ap.add_argument("--literal-zipf", action="store_true",
                    help="extra line: config 2 with ranks Zipf-distributed over the whole 2^40 key space (about a quarter "
                         "of the IDs miss the pre-populated table, so it grows by ~2 M keys per step); runs last, "
                         "takes ~30 s more")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the fused-lookup and pooled-lookup extra lines (profiling runs: only the step's own kernels)")
    ap.add_argument("--count-probes", action="store_true", help="maintain probe/CAS counters (small overhead)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run plain device-to-device copies of this many MiB (reference kernel of known "
                         "size for scaling hardware counters; reports the copy rate)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share of the embedding path; run it with --gpus 1 "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2

    from paper_2505_12663_amd import binding as B
    from paper_2505_12663_amd import EmbeddingTable, StepBuffers
    from workloads import make_config, merged_inputs

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = make_config(args.config)
    dims = [w.table_dim(t) for t in range(w.n_tables)]
    dtypes = [0 if w.table_dtype(t) == "f32" else 1 for t in range(w.n_tables)]
    merged, n_merged = B.emb_plan_merge(dims, dtypes)
    assert n_merged == 1
    tag_bits = B.emb_tag_bits(w.n_tables)
    dim, dtype = dims[0], dtypes[0]
    v_row = dim * (4 if dtype == 0 else 2)
    n_keys = sum(w.prepopulated)
    cap_log2 = 27 if args.config == 2 else 29
    chunk_log2 = 24 if args.config == 2 else 26
    n_chunks = (n_keys >> chunk_log2) + 2

    t0 = time.time()
    table = EmbeddingTable(dim, dtype, capacity_log2=cap_log2, chunk_rows_log2=chunk_log2, max_load_factor=0.75,
                           count_probes=args.count_probes, initial_chunks=n_chunks)
    # ---- bulk load of the pre-existing keys (step 0), in slices
    slice_n = 1 << 22
    dk = torch.empty(slice_n, dtype=torch.int64, device=dev)
    rows = torch.empty(slice_n, dtype=torch.int32, device=dev)
    err = torch.zeros(1, dtype=torch.int64, device=dev)
    for t in range(w.n_tables):
        P = w.prepopulated[t]
        tag = torch.tensor([t], dtype=torch.uint8, device=dev)
        for lo in range(0, P, slice_n):
            hi = min(P, lo + slice_n)
            x = torch.from_numpy(w.prepopulated_ids(t, lo, hi).view(np.int64)).to(dev)
            off = torch.tensor([0, hi - lo], dtype=torch.int64, device=dev)
            B.emb_tag_keys(x, off, tag, tag_bits, dk, err)
            table.find_or_insert(dk, None, hi - lo, 0, rows)
        log(f"bulk load: logical table {t} done ({P} keys, {time.time() - t0:.1f}s)")
    st = table.stats()
    assert st["live"] == n_keys and st["status"] == 0, st
    log(f"table ready: live={st['live']} capacity=2^{cap_log2} load={st['live'] / st['capacity']:.3f}")

    # ---- pre-generate the batches and put them in HBM
    batches = []
    lengths_of = []
    n_max = 0
    for s in range(args.batches):
        b = w.next_step(s)
        x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
        batches.append((torch.from_numpy(x.view(np.int64)).to(dev), torch.from_numpy(off).to(dev),
                        torch.from_numpy(tags).to(dev), len(x), (x, off, tags)))
        n_max = max(n_max, len(x))
        lengths_of.append(b.lengths)
        log(f"batch {s}: N={len(x)} ({time.time() - t0:.1f}s)")
    buf = StepBuffers(n_max, dim, dtype)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    grad = torch.randn((n_max, dim), generator=gen, device=dev, dtype=torch.float32)
    if dtype == 1:
        grad = grad.to(torch.bfloat16)
    v_grad = v_row

    phases = ["tag", "dedup", "find_or_insert", "gather", "expand", "reduce", "adagrad"]
    touch = args.touch_in_lookup   # False: the update writes the row record once per step (touch + accumulator)

    def one_step(step: int, ev=None):
        dx, doff, dtag, n, _ = batches[step % len(batches)]
        rec = (lambda i: ev[i].record()) if ev is not None else (lambda i: None)
        rec(0)
        B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
        rec(1)
        B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
        rec(2)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=touch)
        rec(3)
        table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
        rec(4)
        B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, dim, dtype, buf.out)
        rec(5)
        B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
        rec(6)
        table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, None if touch else step + 1)
        rec(7)
        return n

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(phases) + 1)] for _ in range(args.steps)]
    uniques, news, ids = [], [], 0
    st_before = table.stats()
    live_before = st_before["live"]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        ids += one_step(args.warmup + k, events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    st_after = table.stats()
    live_after = st_after["live"]

    phase_ms = {p: float(np.mean([events[k][i].elapsed_time(events[k][i + 1]) for k in range(args.steps)]))
                for i, p in enumerate(phases)}
    # U per batch (not on the timed path)
    u_of = {}
    for s in range(len(batches)):
        one_step(s)
        u_of[s] = int(buf.n_unique.item())
    n_avg = ids / args.steps
    u_avg = float(np.mean([u_of[(args.warmup + k) % len(batches)] for k in range(args.steps)]))
    u_new = (live_after - live_before) / args.steps
    ab = algorithmic_bytes(int(n_avg), int(u_avg), int(u_new), v_row, v_grad, dim)
    achieved = ab["total"] / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the expand (one kernel = one phase): its own algorithmic bytes over its own time,
    # both measured here; `traffic` = HBM bytes per launch from the committed counter summary (FETCH_SIZE and
    # WRITE_SIZE runs of this same command, scaled by a 1 GiB copy), valid for the default configuration only
    dom = "expand"
    dom_gbps = ab[dom] / (phase_ms[dom] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_copy_rows<16,false,true,true> (emb_expand_sorted)", "achieved": round(dom_gbps, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4),
                "traffic": profiled_traffic("k_copy_rows<16, false, true, true>") if args.config == 2 else None,
                "bytes_per_launch": ab[dom], "avg_ms": round(phase_ms[dom], 4)}

    result = {
        "metric": "embedding IDs/sec fwd+bwd",
        "value": round(ids / wall, 1),
        "unit": "IDs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if dtype == 0 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"config{args.config}:{w.name}", "batch": w.batch, "fields": len(w.features), "dim": dim,
                   "table_keys": n_keys, "capacity_log2": cap_log2, "ids_per_step": int(n_avg),
                   "unique_per_step": int(u_avg), "new_keys_per_step": round(u_new, 1),
                   "row_record_updates_per_step": 2 if touch else 1},
        "unique_ids_per_sec": round(u_avg * args.steps / wall, 1),
        "algorithmic_bytes_per_step": ab["total"],
        "achieved_hbm_gbps": round(achieved, 1),
        "hbm_frac_of_8TBps": round(achieved / HBM_PEAK_GBPS, 4),
        "phase_ms": {k: round(v, 4) for k, v in phase_ms.items()},
        "phase_gbps": {p: round(ab[q] / (phase_ms[p] * 1e-3) / 1e9, 1) for p, q in
                       [("dedup", "tag_dedup"), ("find_or_insert", "find_or_insert"), ("gather", "gather"),
                        ("expand", "expand"), ("reduce", "reduce"), ("adagrad", "adagrad")]},
        "roofline": roofline,
    }
    if args.count_probes:
        pc = {k: st_after[k] - st_before[k] for k in ("lookups", "probes", "cas_attempts", "cas_failures", "alloc_atomics")}
        pc["lines_per_lookup"] = round(pc["probes"] / max(pc["lookups"], 1), 4)
        result["probe_counters_timed_region"] = pc

    # ---- the same step with the fused lookup (no distinct-row matrix), as an extra line
    def one_step_fused(step: int):
        dx, doff, dtag, n, _ = batches[step % len(batches)]
        B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
        B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=touch)
        B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n, buf.out)
        B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
        table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, None if touch else step + 1)
        return n

    base = args.warmup + args.steps + len(batches)
    if not args.no_extras:
        for s in range(2):
            one_step_fused(base + s)
        torch.cuda.synchronize()
        t_f = time.perf_counter()
        ids_f = 0
        for k in range(args.steps):
            ids_f += one_step_fused(base + 2 + k)
        torch.cuda.synchronize()
        wall_f = time.perf_counter() - t_f
        result["fused_lookup"] = {"ms_per_step": round(wall_f * 1e3 / args.steps, 4), "ids_per_sec": round(ids_f / wall_f, 1),
                                  "note": "ht_gather_expand_sorted replaces ht_gather + emb_expand_sorted: same result, "
                                          "2 x rowbytes x unique fewer bytes moved"}

    # ---- the leanest form that still delivers every output of the step on one GPU: no position-ordered inverse
    # (the sorted-order pair perm / seg_of carries the mapping) and the fused lookup, as an extra line
    if not args.no_extras:
        def one_step_lean(step: int):
            dx, doff, dtag, n, _ = batches[step % len(batches)]
            B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
            B.emb_dedup(buf.key, n, buf.uniq, None, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
            table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=touch)
            B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n, buf.out)
            B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
            table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, None if touch else step + 1)
            return n

        base_l = base + 3 * (2 + args.steps)
        for s in range(2):
            one_step_lean(base_l + s)
        torch.cuda.synchronize()
        t_l = time.perf_counter()
        ids_l = 0
        for k in range(args.steps):
            ids_l += one_step_lean(base_l + 2 + k)
        torch.cuda.synchronize()
        wall_l = time.perf_counter() - t_l
        result["lean_step"] = {"ms_per_step": round(wall_l * 1e3 / args.steps, 4), "ids_per_sec": round(ids_l / wall_l, 1),
                               "note": "emb_dedup without the position-ordered inverse array + ht_gather_expand_sorted: "
                                       "same embeddings out, same table after the step"}

    # ---- both fusions of the no-communication case: fused lookup and fused backward (no distinct-row matrix, no
    # reduced-gradient matrix), as an extra line
    if not args.no_extras:
        def one_step_fused2(step: int):
            dx, doff, dtag, n, _ = batches[step % len(batches)]
            B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
            B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
            table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=touch)
            B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n, buf.out)
            B.grad_reduce_apply_adagrad(table.h, grad, buf.seg_of, buf.perm, n, buf.row_idx, w.lr, w.eps,
                                        None if touch else step + 1, buf.reduce_ws)
            return n

        base2 = base + 2 + args.steps
        for s in range(2):
            one_step_fused2(base2 + s)
        torch.cuda.synchronize()
        ev0, ev1, ev2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        t_f2 = time.perf_counter()
        ids_f2 = 0
        for k in range(args.steps):
            ids_f2 += one_step_fused2(base2 + 2 + k)
        torch.cuda.synchronize()
        wall_f2 = time.perf_counter() - t_f2
        # the fused backward alone
        ev0.record()
        for k in range(5):
            B.grad_reduce_apply_adagrad(table.h, grad, buf.seg_of, buf.perm, batches[0][3], buf.row_idx, w.lr, w.eps, None,
                                        buf.reduce_ws)
        ev1.record()
        torch.cuda.synchronize()
        result["fused_step"] = {"ms_per_step": round(wall_f2 * 1e3 / args.steps, 4), "ids_per_sec": round(ids_f2 / wall_f2, 1),
                                "fused_backward_ms": round(ev0.elapsed_time(ev1) / 5, 4),
                                "note": "ht_gather_expand_sorted + grad_reduce_apply_adagrad: neither the distinct-row "
                                        "matrix nor the reduced-gradient matrix is written"}

    # ---- pooled variant (one vector per sample and field instead of one per position), as an extra line
    if args.config == 2 and not args.no_extras:
        lens0 = np.concatenate(lengths_of[0]).astype(np.int64)
        bag_off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens0)]).astype(np.int64)).to(dev)
        nb = len(lens0)
        pws = torch.empty(B.emb_pool_workspace_bytes(n_max, nb, dim), dtype=torch.uint8, device=dev)
        pooled = torch.empty((nb, dim), dtype=torch.float32, device=dev)
        d_pooled = torch.randn((nb, dim), generator=gen, device=dev, dtype=torch.float32)

        def one_step_pooled(step: int):
            dx, doff, dtag, n, _ = batches[0]
            B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
            B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
            table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=touch)
            table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
            B.emb_pool_bags(buf.uniq_rows, dtype, buf.inverse, bag_off, n, dim, True, pooled, pws)
            B.grad_segment_reduce_pooled(d_pooled, bag_off, buf.seg_of, buf.perm, n, dim, True, buf.reduced, pws)
            table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, None if touch else step + 1)
            return n

        base = base + 2 * (2 + args.steps)
        for s in range(2):
            one_step_pooled(base + s)
        torch.cuda.synchronize()
        t_p = time.perf_counter()
        ids_p = 0
        for k in range(args.steps):
            ids_p += one_step_pooled(base + 2 + k)
        torch.cuda.synchronize()
        wall_p = time.perf_counter() - t_p
        result["pooled_lookup"] = {"ms_per_step": round(wall_p * 1e3 / args.steps, 4), "ids_per_sec": round(ids_p / wall_p, 1),
                                   "bags": nb, "mode": "mean",
                                   "note": "emb_pool_bags / grad_segment_reduce_pooled replace expand / reduce: one "
                                           "fp32 vector per (sample, field) instead of one row per position"}

    # ---- same shape with realistic per-field vocabularies (a few fields with a handful of values): segments of
    # 10^5..10^6 positions; table-free phases only (dedup, expand, reduce), as an extra line
    if args.config == 2 and not args.no_extras:
        wl = make_config(2, field_vocab=[6_250_000, 20_000, 6_250_000, 500_000, 100, 24, 8, 50])
        bl = wl.next_step(0)
        xl, offl, tagl, _ = merged_inputs(wl.features, bl.ids, merged, 0)
        nl = len(xl)
        if nl <= n_max:
            dxl = torch.from_numpy(xl.view(np.int64)).to(dev)
            B.emb_tag_keys(dxl, torch.from_numpy(offl).to(dev), torch.from_numpy(tagl).to(dev), tag_bits, buf.key, buf.err_count)

            def timed(fn, reps=10):
                fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps

            t_d = timed(lambda: B.emb_dedup(buf.key, nl, buf.uniq, buf.inverse, buf.counts, buf.perm, None, buf.seg_of,
                                            buf.n_unique, buf.dedup_ws))
            ul = int(buf.n_unique.item())
            longest = int(buf.counts[:ul].max().item())
            t_e = timed(lambda: B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, nl, dim, dtype, buf.out))
            t_r = timed(lambda: B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, nl, dim, buf.reduced, buf.reduce_ws))
            result["low_cardinality_fields"] = {
                "ids": nl, "unique": ul, "longest_segment": longest, "dedup_ms": round(t_d, 4),
                "expand_ms": round(t_e, 4), "reduce_ms": round(t_r, 4),
                "note": "field vocabularies 6.25M, 20k, 6.25M, 500k, 100, 24, 8, 50: worst case for the segmented "
                        "reduction (one segment spans thousands of spans)"}

    # ---- literal reading of "Zipf over a 2^40 key space": the table keeps growing (inserts, new chunks, rehash)
    if args.config == 2 and args.literal_zipf:
        wz = make_config(2, field_vocab=[2 ** 40] * 8)
        wz.prepopulated = list(w.prepopulated)
        k_steps = min(args.steps, 10)
        zb = []
        for s_ in range(k_steps + 1):
            bz = wz.next_step(s_)
            xz, offz, tagz, _ = merged_inputs(wz.features, bz.ids, merged, 0)
            if len(xz) <= n_max:
                zb.append((torch.from_numpy(xz.view(np.int64)).to(dev), torch.from_numpy(offz).to(dev),
                           torch.from_numpy(tagz).to(dev), len(xz)))
        st0 = table.stats()

        def one_step_z(i: int, step: int):
            dx, doff, dtag, n = zb[i]
            B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
            B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
            table.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted, touch=touch)
            table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
            B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, dim, dtype, buf.out)
            B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
            table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, None if touch else step)
            return n

        base_z = 10_000
        one_step_z(0, base_z)                       # warm-up on a batch of its own
        torch.cuda.synchronize()
        st1 = table.stats()
        t_z = time.perf_counter()
        ids_z = 0
        for k in range(1, len(zb)):
            ids_z += one_step_z(k, base_z + k)
        torch.cuda.synchronize()
        wall_z = time.perf_counter() - t_z
        st2 = table.stats()
        nz = len(zb) - 1
        result["literal_zipf"] = {
            "steps": nz, "ms_per_step": round(wall_z * 1e3 / nz, 4), "ids_per_sec": round(ids_z / wall_z, 1),
            "new_keys_per_step": round((st2["live"] - st1["live"]) / nz, 1), "live_after": st2["live"],
            "chunks_added": st2["n_chunks"] - st0["n_chunks"], "rehashes": st2["n_rehash"] - st0["n_rehash"],
            "status": st2["status"],
            "note": "ranks Zipf(1.05) over 2^40, top 6.25 M ranks per field pre-populated: every step creates rows "
                    "for about a quarter of its IDs; host-side capacity planning (chunk registration, rehash) included"}

    if args.copy_probe_mib > 0:
        nbytes = args.copy_probe_mib << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src)
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        result["copy_probe"] = {"bytes_read": nbytes, "bytes_written": nbytes, "avg_ms": round(ms, 4),
                                "gbps_read_plus_write": round(2 * nbytes / (ms * 1e-3) / 1e9, 1)}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, batches[0][4], tag_bits, dim, dtype, n_keys)
    print(json.dumps(result), flush=True)
    table.close()
    return 0


def profiled_traffic(kernel: str):
    """HBM bytes per dispatch of `kernel` from profiles/hbm_traffic_config2_step.txt (None if absent)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_config2_step.txt")
    try:
        for line in open(path):
            parts = [p.strip() for p in line.split("|")]
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_dispatch" and parts[1] == kernel:
                return int(float(parts[2]))
    except OSError:
        pass
    return None


def cpu_baseline(w, batch0, tag_bits, dim, dtype, n_keys) -> dict:
    """The CPU checker as it stands, one thread, timed on one full step of the first batch.
    Pre-existing keys the step touches are materialised first (untimed), as the lazy checker does."""
    import oracle
    x, off, tags = batch0
    log("cpu baseline: preparing (untimed)")
    key, _ = oracle.tag_keys(x, off, tags, tag_bits)
    uniq, _, _ = oracle.dedup(key)
    t = oracle.Table(dim, dtype)
    t.prepopulate(uniq)
    rng = np.random.Generator(np.random.Philox(key=1234))
    G = rng.standard_normal((len(x), dim), dtype=np.float32)
    log("cpu baseline: timing one step")
    t0 = time.perf_counter()
    key, _ = oracle.tag_keys(x, off, tags, tag_bits)
    uniq, inverse, _ = oracle.dedup(key)
    t.find_or_insert(uniq, 1)
    E_u = t.lookup(uniq)
    E = oracle.expand(E_u, inverse)
    g = oracle.segment_reduce(G, inverse, len(uniq))
    t.apply_adagrad(uniq, g, w.lr, w.eps)
    dt = time.perf_counter() - t0
    assert E.shape == (len(x), dim)
    return {"value": round(len(x) / dt, 1), "unit": "IDs/s", "cores": 1, "kind": "oracle",
            "sample": f"one full step of batch 0 ({len(x)} IDs, {len(uniq)} unique), touched keys pre-materialised",
            "seconds": round(dt, 2), "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    sys.exit(main())
