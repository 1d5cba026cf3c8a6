#!/usr/bin/env python3
"""Benchmark of the sparse-embedding step on one MI355X.

A step = tag + dedup -> find-or-insert -> gather -> expand -> (upstream gradient already in HBM)
-> gradient segment-reduce -> row-wise Adagrad over one batch of the long-sequence lookup
configuration (batch 512, lengths U{256..4096}, 8 fields, dim 64 fp32, 50 M-key table, Zipf 1.05).
Every output of the step is materialised (distinct keys, the mapping between positions and distinct keys in
sorted order (perm, seg_of), distinct rows, expanded rows, reduced gradients).  Inputs are resident in HBM when
the timed region starts.  Prints ONE JSON line on stdout.

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


def timed_loop(step_fn, first_step: int, steps: int, warmup: int = 2):
    """warmup untimed calls, then `steps` calls bracketed by synchronisations; (wall seconds, total IDs)."""
    for s in range(warmup):
        step_fn(first_step + s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ids = 0
    for k in range(steps):
        ids += step_fn(first_step + warmup + k)
    torch.cuda.synchronize()
    return time.perf_counter() - t0, ids


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5],
                    help="2: long-sequence lookup (the headline); 5: large bf16 table; 3: table merging - the step over 32 "
                         "logical tables merged into 4 hash tables against the same step over 32 separate tables; "
                         "4: the streaming insert / evict / rehash configuration from an empty table (--steps of its "
                         "1000 steps, default 200)")
    ap.add_argument("--batches", type=int, default=0,
                    help="distinct pre-generated batches cycled through (default: 4 for the long-sequence configuration, "
                         "which brings no new keys; warmup + steps for the large one, so that every step brings its "
                         "share of keys never seen before)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--literal-zipf", action="store_true",
                    help="extra line literal_zipf (config 2 with ranks Zipf-distributed over the whole 2^40 key space: "
                         "about a quarter of the IDs miss the pre-populated table, so it grows by ~2 M keys per "
                         "step) over 10 steps instead of 4")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the extra lines (profiling runs: only the step's own kernels)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run plain device-to-device copies of this many MiB (reference kernel of known "
                         "size for scaling hardware counters; reports the copy rate)")
    ap.add_argument("--ceiling-probes", action="store_true",
                    help="extra line: what the memory system delivers to streaming and random-row kernels of this "
                         "library's access shapes (2 GiB buffers): the yardstick next to the nominal 8 TB/s")
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
    if args.config == 3:
        print(json.dumps(table_merging_line(args, B, EmbeddingTable, StepBuffers, make_config, merged_inputs, dev)), flush=True)
        return 0
    if args.config == 4:
        print(json.dumps(streaming_line(args, B, EmbeddingTable, StepBuffers, make_config, merged_inputs, dev)), flush=True)
        return 0
    w = make_config(args.config)
    dims = [w.table_dim(t) for t in range(w.n_tables)]
    dtypes = [0 if w.table_dtype(t) == "f32" else 1 for t in range(w.n_tables)]
    merged, n_merged = B.emb_plan_merge(dims, dtypes)
    assert n_merged == 1
    tag_bits = B.emb_tag_bits(w.n_tables)
    id_bits = w.id_bits
    dim, dtype = dims[0], dtypes[0]
    v_row = dim * (4 if dtype == 0 else 2)
    n_keys = sum(w.prepopulated)
    cap_log2 = 27 if args.config == 2 else 29
    chunk_log2 = 24 if args.config == 2 else 26
    n_chunks = (n_keys >> chunk_log2) + 2
    n_batches = args.batches or (4 if args.config == 2 else args.warmup + args.steps)

    t0 = time.time()
    table = EmbeddingTable(dim, dtype, capacity_log2=cap_log2, chunk_rows_log2=chunk_log2, max_load_factor=0.75,
                           count_probes=False, initial_chunks=n_chunks)
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
    for s in range(n_batches):
        b = w.next_step(s)
        x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
        keep_host = (x, off, tags) if s == 0 else None
        batches.append((torch.from_numpy(x.view(np.int64)).to(dev), torch.from_numpy(off).to(dev),
                        torch.from_numpy(tags).to(dev), len(x), keep_host))
        n_max = max(n_max, len(x))
        lengths_of.append(b.lengths if s == 0 else None)
        log(f"batch {s}: N={len(x)} ({time.time() - t0:.1f}s)")
    buf = StepBuffers(n_max, dim, dtype)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    grad = torch.randn((n_max, dim), generator=gen, device=dev, dtype=torch.float32)
    if dtype == 1:
        grad = grad.to(torch.bfloat16)
    v_grad = v_row

    phases = ["tag_dedup", "find_or_insert", "gather", "expand", "reduce", "adagrad"]

    # The step this library recommends for one GPU: tag + dedup in one call (8-byte sort records, no tagged-key
    # array), one row-record update per step (the lookup leaves the touch to the update).  Same outputs and the same
    # table afterwards as the step of the named calls below.
    # The mapping positions <-> distinct keys is written in sorted order (perm, seg_of), which is what the expand
    # and the reduce read; the position-ordered `inverse` (a random 4-byte scatter no call of this step reads) is
    # left out here and written by the step of the named calls below.
    def one_step(step: int, ev=None, only=None):
        dx, doff, dtag, n, _ = batches[step % len(batches)]
        rec = (lambda i: ev[i].record() if only is None or i in only else None) if ev is not None else (lambda i: None)
        rec(0)
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        rec(1)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=False)
        rec(2)
        table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
        rec(3)
        B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, dim, dtype, buf.out)
        rec(4)
        B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
        rec(5)
        table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, step + 1)
        rec(6)
        return n

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(phases) + 1)] for _ in range(args.steps)]
    # An event between two calls costs the stream about 4 us (7 per step: 25 us, 1.1 % of the long-sequence step).
    # Where no step changes the table's key set (the long-sequence configuration) the timed region therefore carries
    # only the two events around the dominant kernel, and the per-phase breakdown comes from a second pass of the
    # same number of steps with an event after every call; the large configuration, whose steps differ (new keys,
    # capacity expansion), keeps all events in its timed region so that the breakdown is of the very steps timed.
    dom_i = phases.index("expand")
    lean = args.config == 2
    ids = 0
    live_before = table.stats()["live"]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        ids += one_step(args.warmup + k, events[k], only=(dom_i, dom_i + 1) if lean else None)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    st_after = table.stats()
    live_after = st_after["live"]
    next_step = args.warmup + args.steps
    dom_ms_timed = float(np.mean([events[k][dom_i].elapsed_time(events[k][dom_i + 1]) for k in range(args.steps)]))
    if lean:
        for k in range(args.steps):
            one_step(next_step + k, events[k])
        torch.cuda.synchronize()
        next_step += args.steps

    per_step = {p: [events[k][i].elapsed_time(events[k][i + 1]) for k in range(args.steps)] for i, p in enumerate(phases)}
    phase_ms = {p: float(np.mean(v)) for p, v in per_step.items()}
    step_ms = [events[k][0].elapsed_time(events[k][len(phases)]) for k in range(args.steps)]
    # U of the timed batches (read back outside the timed region)
    u_of = {}
    for s in sorted({(args.warmup + k) % len(batches) for k in range(args.steps)}):
        dx, doff, dtag, n, _ = batches[s]
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        u_of[s] = int(buf.n_unique.item())
    n_avg = ids / args.steps
    u_avg = float(np.mean([u_of[(args.warmup + k) % len(batches)] for k in range(args.steps)]))
    u_new = (live_after - live_before) / args.steps
    ab = algorithmic_bytes(int(n_avg), int(u_avg), int(u_new), v_row, v_grad, dim)
    achieved = ab["total"] / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the expand (one kernel = one phase): its own algorithmic bytes over its own time,
    # both measured here; `traffic` = HBM bytes per launch from the committed counter summary (FETCH_SIZE and
    # WRITE_SIZE runs of this same command, scaled by a 1 GiB copy) of the configuration
    dom = "expand"
    dom_gbps = ab[dom] / (dom_ms_timed * 1e-3) / 1e9        # from the events of the timed region
    lpr = max(1, v_row // 16)
    kname = f"k_copy_rows<{lpr}, false, true, true>"
    roofline = {"bound": "hbm", "kernel": f"{kname} (emb_expand_sorted)", "achieved": round(dom_gbps, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4),
                "traffic": profiled_traffic(kname, args.config),
                "bytes_per_launch": ab[dom], "avg_ms": round(dom_ms_timed, 4),
                "whole_step": {"algorithmic_bytes": ab["total"], "achieved": round(achieved, 1),
                               "frac": round(achieved / HBM_PEAK_GBPS, 4)}}

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
                   "unique_per_step": int(u_avg), "new_keys_per_step": round(u_new, 1), "distinct_batches": len(batches),
                   "calls": "emb_tag_dedup (mapping as perm + seg_of), ht_find_or_insert_notouch, ht_gather, "
                            "emb_expand_sorted, grad_segment_reduce, ht_apply_adagrad_touch"},
        "unique_ids_per_sec": round(u_avg * args.steps / wall, 1),
        "algorithmic_bytes_per_step": ab["total"],
        "achieved_hbm_gbps": round(achieved, 1),
        "hbm_frac_of_8TBps": round(achieved / HBM_PEAK_GBPS, 4),
        "step_ms_median": round(float(np.median(step_ms)), 4),
        "phase_timing": ("second pass of the same number of steps with an event after every call (the timed region carries "
                         "only the two events around the dominant kernel)") if lean else "events of the timed region",
        "phase_ms": {k: round(v, 4) for k, v in phase_ms.items()},
        "phase_gbps": {p: round(ab[p] / (phase_ms[p] * 1e-3) / 1e9, 1) for p in phases},
        "roofline": roofline,
    }
    if st_after["n_rehash"] or st_after["refused"]:
        # the table crossed its load-factor limit inside the timed region: the step that expands the key structure
        # is in ms_per_step (and in the mean phase times); the medians show the ordinary step
        slow = int(np.argmax(step_ms))
        result["capacity_expansion"] = {
            "rehashes_in_run": st_after["n_rehash"], "keys_turned_away_at_the_limit": st_after["refused"],
            "capacity_log2_after": int(np.log2(st_after["capacity"])),
            "slowest_step_ms": round(step_ms[slow], 3), "slowest_step_find_or_insert_ms": round(per_step["find_or_insert"][slow], 3),
            "median_step_ms": round(float(np.median(step_ms)), 4),
            "phase_ms_median": {p: round(float(np.median(v)), 4) for p, v in per_step.items()},
            "note": "find_or_insert of the slowest step includes reading the counters back, the key-only rehash into a "
                    "structure of twice the size and the second attempt for the keys that had been turned away"}

    # ---- the step spelled with the calls the problem statement names, as an extra line: emb_tag_keys + emb_dedup,
    # ht_find_or_insert (touches every row record), ht_gather, emb_expand by `inverse`, grad_segment_reduce,
    # ht_apply_adagrad (updates the record again)
    def one_step_named(step: int):
        dx, doff, dtag, n, _ = batches[step % len(batches)]
        B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
        B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of, buf.n_unique, buf.dedup_ws)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=True)
        table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
        B.emb_expand(buf.uniq_rows, buf.inverse, n, dim, dtype, buf.out)
        B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
        table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, None)
        return n

    extras_ok = not args.no_extras and args.config == 2      # the extra lines reuse batches; only where no step brings new keys
    if extras_ok:
        wall_n, ids_n = timed_loop(one_step_named, next_step, args.steps)
        next_step += args.steps + 2
        result["named_calls_step"] = {
            "ms_per_step": round(wall_n * 1e3 / args.steps, 4), "ids_per_sec": round(ids_n / wall_n, 1),
            "hbm_frac_of_8TBps": round(ab["total"] * args.steps / wall_n / 1e9 / HBM_PEAK_GBPS, 4),
            "calls": "emb_tag_keys, emb_dedup, ht_find_or_insert, ht_gather, emb_expand, grad_segment_reduce, ht_apply_adagrad"}

    # ---- probe and atomic counts of the lookup, from a counted pass outside the timed region
    if not args.no_extras:
        result["probe_counts"] = probe_counts(B, table, batches, buf, tag_bits, id_bits, dim, dtype, cap_log2, chunk_log2)

    # ---- first stage of a hash-based deduplication, measured for comparison with the sort
    if extras_ok:
        result["hash_front_end_probe"] = hash_front_end_probe(B, batches, buf, tag_bits, id_bits, phase_ms["tag_dedup"])

    # ---- the same step with the fused lookup (no distinct-row matrix), as an extra line
    def one_step_fused(step: int):
        dx, doff, dtag, n, _ = batches[step % len(batches)]
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=False)
        B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n, buf.out)
        B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
        table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, step + 1)
        return n

    if extras_ok:
        wall_f, ids_f = timed_loop(one_step_fused, next_step, args.steps)
        next_step += args.steps + 2
        result["fused_lookup"] = {"ms_per_step": round(wall_f * 1e3 / args.steps, 4), "ids_per_sec": round(ids_f / wall_f, 1),
                                  "note": "ht_gather_expand_sorted replaces ht_gather + emb_expand_sorted: same result, "
                                          "2 x rowbytes x unique fewer bytes moved"}

    # ---- the same calls as a two-stage pipeline over two streams (the paper's training pipeline overlaps the ID
    # dispatch of the next batch with the computation of the current one): tag + dedup of batch i+1 touches no table
    # state, so it runs on a second stream (default priority) while batch i looks up, gathers, expands, reduces and
    # updates.  Two sets of dedup outputs; every timed step issues one dedup and one lookup-to-update chain
    if extras_ok:
        main_s, side_s = torch.cuda.current_stream(), torch.cuda.Stream()
        sets = [(buf.uniq, buf.perm, buf.seg_of, buf.n_unique, buf.err_count, buf.tag_dedup_ws),
                tuple(torch.empty_like(t) for t in (buf.uniq, buf.perm, buf.seg_of, buf.n_unique, buf.err_count, buf.tag_dedup_ws))]
        ev_dedup = [torch.cuda.Event(), torch.cuda.Event()]
        ev_free = [torch.cuda.Event(), torch.cuda.Event()]

        def dedup_ahead(step: int):
            dx, doff, dtag, n, _ = batches[step % len(batches)]
            uq, pm, so, nu, er, ws = sets[step & 1]
            side_s.wait_event(ev_free[step & 1])            # the step that last read this set has finished
            B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, uq, None, None, pm, None, so, nu, er, ws, stream=side_s)
            ev_dedup[step & 1].record(side_s)

        def one_step_piped(step: int):
            dedup_ahead(step + 1)
            dx, doff, dtag, n, _ = batches[step % len(batches)]
            uq, pm, so, nu, er, ws = sets[step & 1]
            main_s.wait_event(ev_dedup[step & 1])
            table.find_or_insert(uq, nu, n, step + 1, buf.row_idx, buf.inserted, touch=False)
            table.gather(buf.row_idx, nu, n, buf.uniq_rows)
            B.emb_expand_sorted(buf.uniq_rows, so, pm, n, dim, dtype, buf.out)
            B.grad_segment_reduce(grad, dtype, so, pm, n, dim, buf.reduced, buf.reduce_ws)
            table.apply_adagrad(buf.row_idx, buf.reduced, nu, n, w.lr, w.eps, step + 1)
            ev_free[step & 1].record(main_s)
            return n

        torch.cuda.synchronize()
        ev_free[0].record(main_s)
        ev_free[1].record(main_s)
        dedup_ahead(next_step)                               # prologue: the first batch's dedup, untimed
        wall_2, ids_2 = timed_loop(one_step_piped, next_step, args.steps)
        side_s.synchronize()
        next_step += args.steps + 3
        result["two_stream_pipeline"] = {
            "ms_per_step": round(wall_2 * 1e3 / args.steps, 4), "ids_per_sec": round(ids_2 / wall_2, 1),
            "hbm_frac_of_8TBps": round(ab["total"] * args.steps / wall_2 / 1e9 / HBM_PEAK_GBPS, 4),
            "note": "every timed step issues emb_tag_dedup of the next batch on a second stream and find-or-insert, gather, "
                    "expand, reduce, Adagrad of the current batch on the first: the same calls and the same work per step "
                    "as the headline, which runs them back to back on one stream; the sort's own traffic competes with "
                    "the row kernels for memory bandwidth, so only its latency-bound share is hidden"}

    # ---- no position-ordered inverse (the sorted-order pair perm / seg_of carries the mapping), fused lookup and
    # fused backward: nothing is written that one GPU does not read again, as an extra line
    def one_step_lean(step: int):
        dx, doff, dtag, n, _ = batches[step % len(batches)]
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=False)
        B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n, buf.out)
        B.grad_reduce_apply_adagrad(table.h, grad, buf.seg_of, buf.perm, n, buf.row_idx, w.lr, w.eps, step + 1, buf.reduce_ws)
        return n

    if extras_ok:
        wall_l, ids_l = timed_loop(one_step_lean, next_step, args.steps)
        next_step += args.steps + 2
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for k in range(5):
            B.grad_reduce_apply_adagrad(table.h, grad, buf.seg_of, buf.perm, batches[0][3], buf.row_idx, w.lr, w.eps, None,
                                        buf.reduce_ws)
        ev1.record()
        torch.cuda.synchronize()
        result["no_intermediates_step"] = {
            "ms_per_step": round(wall_l * 1e3 / args.steps, 4), "ids_per_sec": round(ids_l / wall_l, 1),
            "hbm_frac_of_8TBps_by_the_unfused_byte_count": round(ab["total"] * args.steps / wall_l / 1e9 / HBM_PEAK_GBPS, 4),
            "fused_backward_ms": round(ev0.elapsed_time(ev1) / 5, 4),
            "note": "emb_tag_dedup + ht_gather_expand_sorted + grad_reduce_apply_adagrad: same embeddings out, same "
                    "table after the step; distinct-row matrix and reduced-gradient matrix are not written"}

    # ---- the fused calls on their own (any configuration): the buffers still hold the last timed step's batch
    if not args.no_extras and not extras_ok:
        dx, doff, dtag, n_last, _ = batches[(args.warmup + args.steps - 1) % len(batches)]
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        table.find_or_insert(buf.uniq, buf.n_unique, n_last, next_step, buf.row_idx, buf.inserted, touch=False)
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        reps = 3
        e0.record()
        for _ in range(reps):
            B.ht_gather_expand_sorted(table.h, buf.row_idx, buf.seg_of, buf.perm, n_last, buf.out)
        e1.record()
        for _ in range(reps):
            B.grad_reduce_apply_adagrad(table.h, grad, buf.seg_of, buf.perm, n_last, buf.row_idx, w.lr, w.eps, None, buf.reduce_ws)
        e2.record()
        torch.cuda.synchronize()
        result["fused_calls"] = {
            "ht_gather_expand_sorted_ms": round(e0.elapsed_time(e1) / reps, 4),
            "against_gather_plus_expand_ms": round(phase_ms["gather"] + phase_ms["expand"], 4),
            "grad_reduce_apply_adagrad_ms": round(e1.elapsed_time(e2) / reps, 4),
            "against_reduce_plus_adagrad_ms": round(phase_ms["reduce"] + phase_ms["adagrad"], 4),
            "note": "same results without the distinct-row matrix / the reduced-gradient matrix (which, with fp32 sums of "
                    "bf16 gradients, is twice the size of the rows it updates)"}

    # ---- pooled variant (one vector per sample and field instead of one per position), as an extra line
    if extras_ok:
        lens0 = np.concatenate(lengths_of[0]).astype(np.int64)
        bag_off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens0)]).astype(np.int64)).to(dev)
        nb = len(lens0)
        pws = torch.empty(B.emb_pool_workspace_bytes(n_max, nb, dim), dtype=torch.uint8, device=dev)
        pooled = torch.empty((nb, dim), dtype=torch.float32, device=dev)
        d_pooled = torch.randn((nb, dim), generator=gen, device=dev, dtype=torch.float32)

        def one_step_pooled(step: int):
            dx, doff, dtag, n, _ = batches[0]
            B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of,
                            buf.n_unique, buf.err_count, buf.tag_dedup_ws)
            table.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=False)
            table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
            B.emb_pool_bags(buf.uniq_rows, dtype, buf.inverse, bag_off, n, dim, True, pooled, pws)
            B.grad_segment_reduce_pooled(d_pooled, bag_off, buf.seg_of, buf.perm, n, dim, True, buf.reduced, pws)
            table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, step + 1)
            return n

        wall_p, ids_p = timed_loop(one_step_pooled, next_step, args.steps)
        next_step += args.steps + 2
        result["pooled_lookup"] = {"ms_per_step": round(wall_p * 1e3 / args.steps, 4), "ids_per_sec": round(ids_p / wall_p, 1),
                                   "bags": nb, "mode": "mean",
                                   "note": "emb_pool_bags / grad_segment_reduce_pooled replace expand / reduce: one "
                                           "fp32 vector per (sample, field) instead of one row per position"}

    def timed(fn, reps=10):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # ---- same shape with realistic per-field vocabularies (a few fields with a handful of values): segments of
    # 10^5..10^6 positions; table-free phases only (dedup, expand, reduce), as an extra line
    if extras_ok:
        wl = make_config(2, field_vocab=[6_250_000, 20_000, 6_250_000, 500_000, 100, 24, 8, 50])
        bl = wl.next_step(0)
        xl, offl, tagl, _ = merged_inputs(wl.features, bl.ids, merged, 0)
        nl = len(xl)
        if nl <= n_max:
            dxl, doffl, dtagl = torch.from_numpy(xl.view(np.int64)).to(dev), torch.from_numpy(offl).to(dev), torch.from_numpy(tagl).to(dev)
            t_d = timed(lambda: B.emb_tag_dedup(dxl, doffl, dtagl, tag_bits, id_bits, None, buf.uniq, buf.inverse, buf.counts,
                                                buf.perm, buf.seg_off, buf.seg_of, buf.n_unique, buf.err_count, buf.tag_dedup_ws))
            ul = int(buf.n_unique.item())
            longest = int(buf.counts[:ul].max().item())
            t_e = timed(lambda: B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, nl, dim, dtype, buf.out))
            t_r = timed(lambda: B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, nl, dim, buf.reduced, buf.reduce_ws))
            result["low_cardinality_fields"] = {
                "ids": nl, "unique": ul, "longest_segment": longest, "tag_dedup_ms": round(t_d, 4),
                "expand_ms": round(t_e, 4), "reduce_ms": round(t_r, 4),
                "note": "field vocabularies 6.25M, 20k, 6.25M, 500k, 100, 24, 8, 50: worst case for the segmented "
                        "reduction (one segment spans thousands of spans)"}

    # ---- literal reading of "Zipf over a 2^40 key space": the table keeps growing (inserts, new chunks, rehash)
    # (4 steps by default, 10 with --literal-zipf; the only line of the default run in which every step inserts)
    if extras_ok:
        wz = make_config(2, field_vocab=[2 ** 40] * 8)
        wz.prepopulated = list(w.prepopulated)
        k_steps = min(args.steps, 10) if args.literal_zipf else 4
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
            B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                            buf.n_unique, buf.err_count, buf.tag_dedup_ws)
            table.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted, touch=False)
            table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
            B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, dim, dtype, buf.out)
            B.grad_segment_reduce(grad, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
            table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, step)
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

    # ---- eviction scan and key-structure migration on the benchmark's own table (last GPU work of the run)
    if extras_ok:
        result["table_maintenance"] = table_maintenance(B, table, next_step + 20_000)

    if args.copy_probe_mib > 0:
        nbytes = args.copy_probe_mib << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        ms = timed(lambda: dst.copy_(src))
        result["copy_probe"] = {"bytes_read": nbytes, "bytes_written": nbytes, "avg_ms": round(ms, 4),
                                "gbps_read_plus_write": round(2 * nbytes / (ms * 1e-3) / 1e9, 1)}
        del src, dst
    if args.ceiling_probes:
        result["ceiling_probes"] = ceiling_probes(B, timed, dev)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, batches[0][4], tag_bits, dim, dtype, n_keys)
    print(json.dumps(result), flush=True)
    table.close()
    return 0


def streaming_line(args, B, EmbeddingTable, StepBuffers, make_config, merged_inputs, dev) -> dict:
    """Dynamic insert / delete configuration (Sec. 3.1): batch 512 x 1024 x 4 fields, 20 % of a step's keys never seen
    before, keys evicted every 20 steps (unseen for 200 steps, or touched fewer than 3 times and unseen for 20), load-factor
    limit 0.85, the table empty and at 2^22 slots at step 0.  The timed region is the stream itself: every step's
    forward + backward calls, the eviction scans, and whatever the capacity protocol costs when the device turns keys
    away at the limit (counter read-back, key-only rehash, second attempt)."""
    w = make_config(4)
    steps = args.steps if args.steps != 20 else 200         # 20 is the command line's default for the other lines
    merged, _ = B.emb_plan_merge([64] * 4, [0] * 4)
    tag_bits, id_bits, dim = B.emb_tag_bits(4), w.id_bits, 64
    t0 = time.time()
    batches, n_max = [], 1
    for s_ in range(steps):
        b = w.next_step(s_)
        x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
        batches.append((torch.from_numpy(x.view(np.int64)).to(dev), torch.from_numpy(off).to(dev), torch.from_numpy(tags).to(dev), len(x)))
        n_max = max(n_max, len(x))
        if s_ % 50 == 49:
            log(f"batches generated: {s_ + 1} ({time.time() - t0:.1f}s)")
    table = EmbeddingTable(dim, 0, capacity_log2=22, chunk_rows_log2=21, max_load_factor=w.max_load_factor, count_probes=False)
    buf = StepBuffers(n_max, dim)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    grad = torch.randn((n_max, dim), generator=gen, device=dev, dtype=torch.float32)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    evict_ms, evicted, ids = [], 0, 0
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for step in range(steps):
        dx, doff, dtag, n = batches[step]
        ev[step][0].record()
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        table.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted, touch=False)
        table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
        B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, dim, 0, buf.out)
        B.grad_segment_reduce(grad, 0, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
        table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, step)
        ev[step][1].record()
        ids += n
        if (step + 1) % w.evict_every == 0:
            te = time.perf_counter()
            _, n_ev = table.evict(step, w.ttl, w.min_freq, w.grace, want_keys=False)     # reads the count back
            evict_ms.append((time.perf_counter() - te) * 1e3)
            evicted += n_ev
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    st = table.stats()
    step_ms = [a.elapsed_time(b_) for a, b_ in ev]
    out = {
        "metric": "embedding IDs/sec fwd+bwd", "value": round(ids / wall, 1), "unit": "IDs/s", "n_gpus": 1, "steps": steps,
        "warmup": 0, "ms_per_step": round(wall * 1e3 / steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config4:{w.name}", "batch": w.batch, "fields": len(w.features), "dim": dim,
                   "ids_per_step": ids // steps, "evict_every": w.evict_every, "ttl": w.ttl, "min_freq": w.min_freq,
                   "grace": w.grace, "max_load_factor": w.max_load_factor, "capacity_log2_at_start": 22},
        "step_ms_median": round(float(np.median(step_ms)), 4), "step_ms_max": round(float(np.max(step_ms)), 3),
        "evictions": {"scans": len(evict_ms), "keys_evicted": evicted,
                      "ms_per_scan_with_count_read_back": round(float(np.mean(evict_ms)), 3) if evict_ms else None},
        "table_after": {"live": st["live"], "deleted_markers": st["tombstones"], "capacity_log2": int(np.log2(st["capacity"])),
                        "load_factor": round((st["live"] + st["tombstones"]) / st["capacity"], 3), "rehashes": st["n_rehash"],
                        "keys_turned_away_and_reissued": st["refused"], "peak_load_factor_seen": round(table.peak_load, 3),
                        "status": st["status"]},
        "note": "the whole stream from an empty table: every step's calls, the eviction scans and the capacity protocol "
                "(keys turned away at the limit, counters read back, key-only rehash, second attempt) are inside the wall "
                "time; step_ms_median is the ordinary step between such events"}
    table.close()
    return out


def table_merging_line(args, B, EmbeddingTable, StepBuffers, make_config, merged_inputs, dev) -> dict:
    """Table-merging configuration (Sec. 3.2): 32 logical tables with dims from {16, 32, 64, 128}, batch 1024 x 40 fields,
    1-200 IDs per field.  The same forward+backward step over (a) the 4 hash tables the merge plan gives (one per dim, IDs
    tagged with their logical table, Eq. 8) and (b) 32 separate hash tables, one per logical table: what merging buys on
    this GPU is fewer, larger launches.  Tables start empty and fill during the warm-up steps."""
    w = make_config(3)
    dims = [w.table_dim(t) for t in range(w.n_tables)]
    merged, n_merged = B.emb_plan_merge(dims, [0] * w.n_tables)
    tag_bits, id_bits = w.tag_bits, w.id_bits
    n_steps = args.warmup + args.steps
    raw = [w.next_step(s) for s in range(n_steps)]

    def build(plan, n_groups):
        """tables, buffers and device inputs of every step for a grouping of the logical tables"""
        group_dim = [dims[list(plan).index(g)] for g in range(n_groups)]
        per_step = []
        n_max = [1] * n_groups
        for b in raw:
            groups = []
            for g in range(n_groups):
                x, off, tags, _ = merged_inputs(w.features, b.ids, plan, g)
                n_max[g] = max(n_max[g], len(x))
                groups.append((torch.from_numpy(x.view(np.int64)).to(dev), torch.from_numpy(off).to(dev),
                               torch.from_numpy(tags).to(dev), len(x)))
            per_step.append(groups)
        cap = 22 if n_groups == n_merged else 20
        tables = [EmbeddingTable(group_dim[g], 0, capacity_log2=cap, chunk_rows_log2=cap - 2, initial_chunks=2)
                  for g in range(n_groups)]
        bufs = [StepBuffers(n_max[g], group_dim[g]) for g in range(n_groups)]
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed)
        grads = [torch.randn((n_max[g], group_dim[g]), generator=gen, device=dev, dtype=torch.float32) for g in range(n_groups)]
        return tables, bufs, grads, per_step, group_dim

    def group_step(t, buf, grad, inp, step, stream=None):
        dx, doff, dtag, n = inp
        if n == 0:
            return 0
        B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                        buf.n_unique, buf.err_count, buf.tag_dedup_ws)
        t.find_or_insert(buf.uniq, buf.n_unique, n, step + 1, buf.row_idx, buf.inserted, touch=False)
        t.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
        B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, t.dim, 0, buf.out)
        B.grad_segment_reduce(grad, 0, buf.seg_of, buf.perm, n, t.dim, buf.reduced, buf.reduce_ws)
        t.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, w.lr, w.eps, step + 1)
        return n

    def run(plan, n_groups, streams=None):
        tables, bufs, grads, per_step, group_dim = build(plan, n_groups)
        main = torch.cuda.current_stream()

        def step_fn(step):
            ids = 0
            if streams is None:
                for g in range(n_groups):
                    ids += group_step(tables[g], bufs[g], grads[g], per_step[step][g], step)
            else:
                for g in range(n_groups):
                    st = streams[g % len(streams)]
                    st.wait_stream(main)
                    with torch.cuda.stream(st):
                        ids += group_step(tables[g], bufs[g], grads[g], per_step[step][g], step)
                for st in streams:
                    main.wait_stream(st)
            return ids
        for s_ in range(args.warmup):
            step_fn(s_)
        torch.cuda.synchronize()
        live0 = sum(t.stats()["live"] for t in tables)
        t0 = time.perf_counter()
        ids = 0
        for k in range(args.steps):
            ids += step_fn(args.warmup + k)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        stats = [t.stats() for t in tables]
        out = {"tables": n_groups, "ms_per_step": round(wall * 1e3 / args.steps, 4), "ids_per_sec": round(ids / wall, 1),
               "ids_per_step": ids // args.steps, "live_keys_after": sum(s_["live"] for s_ in stats),
               "new_keys_per_step": round((sum(s_["live"] for s_ in stats) - live0) / args.steps, 1),
               "status": max(s_["status"] for s_ in stats)}
        for t in tables:
            t.close()
        del tables, bufs, grads, per_step
        torch.cuda.empty_cache()
        return out, wall, ids

    m, wall_m, ids_m = run(merged, n_merged)
    log(f"merged: {m}")
    m4, _, _ = run(merged, n_merged, [torch.cuda.Stream() for _ in range(n_merged)])
    log(f"merged, one stream per table: {m4}")
    u, _, _ = run(np.arange(w.n_tables, dtype=np.int32), w.n_tables)
    log(f"unmerged: {u}")
    return {
        "metric": "embedding IDs/sec fwd+bwd", "value": m["ids_per_sec"], "unit": "IDs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config3:{w.name}", "logical_tables": w.n_tables, "merged_tables": int(n_merged),
                   "fields": len(w.features), "batch": w.batch, "tag_bits": tag_bits, "ids_per_step": m["ids_per_step"]},
        "merged": m, "merged_one_stream_per_table": m4, "separate_tables": u,
        "speedup_from_merging": round(u["ms_per_step"] / m["ms_per_step"], 2),
        "note": "the same forward+backward step over the 4 merged hash tables of the merge plan (one per dim, IDs tagged with "
                "their logical table) and over 32 separate hash tables; tables start empty and keep inserting new keys",
    }


def probe_counts(B, table, batches, buf, tag_bits, id_bits, dim, dtype, cap_log2, chunk_log2) -> dict:
    """Probe and atomic counts of the hash table from instrumented calls outside the timed region (the counters
    cost a few atomics per wave, so the timed table runs without them): a 3.9 M-key bulk insert into a fresh table
    of 2^23 slots (load factor 0 -> 0.47) with its compare-and-swap, admission and allocator counts, then a lookup
    of the same keys and a lookup of as many absent keys at that load, each with its histogram of distinct slot
    lines inspected per key."""
    from paper_2505_12663_amd import EmbeddingTable
    dx, doff, dtag, n, _ = batches[0]
    B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, None, None, buf.perm, None, buf.seg_of,
                    buf.n_unique, buf.err_count, buf.tag_dedup_ws)
    u = int(buf.n_unique.item())
    out = {}
    dev = buf.uniq.device
    t2 = EmbeddingTable(dim, dtype, capacity_log2=23, chunk_rows_log2=22, max_load_factor=0.75, count_probes=True,
                        initial_chunks=2)
    g = torch.Generator(device=dev).manual_seed(3)
    keys = torch.randint(0, 1 << 40, (1 << 22,), generator=g, device=dev, dtype=torch.int64)
    keys = torch.unique(keys)[: (1 << 22) - (1 << 18)].contiguous()             # distinct, a little under 4 M
    k = keys.numel()
    rows = torch.empty(k, dtype=torch.int32, device=dev)
    s0 = t2.stats()
    table_ms = time.perf_counter()
    t2.find_or_insert(keys, None, k, 1, rows)
    torch.cuda.synchronize()
    table_ms = (time.perf_counter() - table_ms) * 1e3
    s1 = t2.stats()
    d = lambda a, b, f: b[f] - a[f]
    out["bulk_insert"] = {
        "keys": k, "load_factor_after": round(s1["live"] / s1["capacity"], 3),
        "lines_per_key": round(d(s0, s1, "probes") / max(d(s0, s1, "lookups"), 1), 4),
        "distinct_lines_per_key_histogram_1_to_8plus": [b - a for a, b in zip(s0["probe_hist"], s1["probe_hist"])],
        "cas_attempts": d(s0, s1, "cas_attempts"), "cas_failures": d(s0, s1, "cas_failures"),
        "admission_and_allocator_atomics": d(s0, s1, "alloc_atomics"), "wall_ms_with_sync": round(table_ms, 3)}
    B.ht_find(t2.h, keys, None, k, rows)
    s2 = t2.stats()
    out["lookup_at_load_0.5"] = {
        "keys": k, "lines_per_key": round(d(s1, s2, "probes") / max(d(s1, s2, "lookups"), 1), 4),
        "distinct_lines_per_key_histogram_1_to_8plus": [b - a for a, b in zip(s1["probe_hist"], s2["probe_hist"])]}
    # absent keys at that load (a miss ends at the first line with a never-used slot)
    miss = keys + (1 << 41)
    B.ht_find(t2.h, miss, None, k, rows)
    s3 = t2.stats()
    out["miss_at_load_0.5"] = {
        "keys": k, "lines_per_key": round(d(s2, s3, "probes") / max(d(s2, s3, "lookups"), 1), 4),
        "distinct_lines_per_key_histogram_1_to_8plus": [b - a for a, b in zip(s2["probe_hist"], s3["probe_hist"])]}
    t2.close()
    # the same at the stress configuration's load-factor limit: a table filled to floor(0.85 * 2^22) slots
    t3 = EmbeddingTable(dim, dtype, capacity_log2=22, chunk_rows_log2=22, max_load_factor=0.85, count_probes=True,
                        initial_chunks=1)
    k3 = int(np.float32(0.85) * (1 << 22))
    keys3 = keys[:k3].contiguous()
    rows3 = torch.empty(k3, dtype=torch.int32, device=dev)
    a0 = t3.stats()
    t3.find_or_insert(keys3, None, k3, 1, rows3)
    a1 = t3.stats()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    B.ht_find(t3.h, keys3, None, k3, rows3)
    e1.record()
    a2 = t3.stats()
    B.ht_find(t3.h, miss[:k3].contiguous(), None, k3, rows3)
    a3 = t3.stats()
    out["at_load_0.85"] = {
        "keys": k3, "load_factor": round((a1["live"] + a1["tombstones"]) / a1["capacity"], 4), "turned_away": a1["refused"],
        "insert_lines_per_key": round(d(a0, a1, "probes") / max(d(a0, a1, "lookups"), 1), 4),
        "insert_cas_attempts": d(a0, a1, "cas_attempts"), "insert_cas_failures": d(a0, a1, "cas_failures"),
        "hit_lines_per_key": round(d(a1, a2, "probes") / max(d(a1, a2, "lookups"), 1), 4),
        "hit_distinct_lines_histogram_1_to_8plus": [b - a for a, b in zip(a1["probe_hist"], a2["probe_hist"])],
        "hit_lookup_ms": round(e0.elapsed_time(e1), 4),
        "miss_lines_per_key": round(d(a2, a3, "probes") / max(d(a2, a3, "lookups"), 1), 4),
        "miss_distinct_lines_histogram_1_to_8plus": [b - a for a, b in zip(a2["probe_hist"], a3["probe_hist"])]}
    t3.close()
    stb = table.stats()
    out["benchmark_table"] = {"load_factor": round((stb["live"] + stb["tombstones"]) / stb["capacity"], 4),
                              "distinct_keys_looked_up_per_step": u,
                              "atomics_per_lookup_step": "none for keys that are present (admission and allocation "
                                                         "atomics are per block of 512 keys that brings new keys)"}
    return out


def table_maintenance(B, table, now: int) -> dict:
    """Eviction and rehash timed on the table the benchmark has just used (HIP events, one call each): a scan that
    evicts nothing, the migration into a key structure of twice the size, an eviction of every key no step has
    touched since the bulk load, and the same-size migration that purges the deleted markers.  GB/s = the bytes the
    operation must move (16 per slot read, 16 per slot of the new structure written, 16 per live key's record) over
    its time."""
    dev = table.device
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def once(fn):
        torch.cuda.synchronize()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    out = {}
    n_ev = torch.zeros(1, dtype=torch.int64, device=dev)
    st = table.stats()
    cap, live = st["capacity"], st["live"]
    ms = once(lambda: B.ht_evict(table.h, now, 1 << 30, 0, 0, None, n_ev))
    out["evict_scan_nothing_evicted"] = {"slots": cap, "live": live, "ms": round(ms, 3),
                                         "gbps": round((16 * cap + 16 * live) / ms / 1e6, 1)}
    log2 = table.capacity_log2
    new_slots = torch.empty((1 << (log2 + 1), 2), dtype=torch.int64, device=dev)
    ms = once(lambda: B.ht_rehash(table.h, new_slots, log2 + 1))
    table.slots, table.capacity_log2 = new_slots, log2 + 1
    out["rehash_to_twice_the_size"] = {"slots_before": cap, "live": live, "ms": round(ms, 3),
                                       "gbps": round((16 * cap + 32 * cap) / ms / 1e6, 1)}
    cap *= 2
    ms = once(lambda: B.ht_evict(table.h, now, now, 0, 0, None, n_ev))      # last seen at step 0 = never touched since the load
    gone = int(n_ev.item())
    out["evict_untouched_keys"] = {"slots": cap, "live_before": live, "evicted": gone, "ms": round(ms, 3)}
    st = table.stats()
    purge = torch.empty((1 << (log2 + 1), 2), dtype=torch.int64, device=dev)
    ms = once(lambda: B.ht_rehash(table.h, purge, log2 + 1))
    table.slots = purge
    st2 = table.stats()
    out["rehash_same_size_purge"] = {"slots": cap, "live": st2["live"], "deleted_markers_before": st["tombstones"],
                                     "deleted_markers_after": st2["tombstones"], "ms": round(ms, 3),
                                     "gbps": round((16 * cap + 16 * cap) / ms / 1e6, 1)}
    out["status"] = st2["status"]
    return out


def hash_front_end_probe(B, batches, buf, tag_bits, id_bits, sort_ms) -> dict:
    """What the first stage of a hash-based deduplication costs on this batch, measured with the library's own
    table: every ID of the batch, duplicates included, goes through find-or-insert into an empty table with
    16-byte rows (the row index a key receives is its dense number, i.e. an inverse in arrival order).  A hash
    front end would still have to clear the table, bring the distinct keys into ascending order, renumber, and
    sort (number, position) pairs for the backward pass's segments; the sort-based call delivers all of that."""
    from paper_2505_12663_amd import EmbeddingTable
    dx, doff, dtag, n, _ = batches[0]
    B.emb_tag_keys(dx, doff, dtag, tag_bits, buf.key, buf.err_count)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ms, distinct, rcs = [], 0, []
    for rep in range(3):
        t = EmbeddingTable(4, 0, capacity_log2=23, chunk_rows_log2=22, max_load_factor=1.0, initial_chunks=1)
        torch.cuda.synchronize()
        e0.record()
        rcs.append(B.ht_find_or_insert(t.h, buf.key, None, n, 1, buf.row_idx, None, touch=False))
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
        st = t.stats()
        distinct, refused = st["live"], st["refused"]
        t.close()
    e0.record()
    B.emb_tag_dedup(dx, doff, dtag, tag_bits, id_bits, None, buf.uniq, buf.inverse, None, buf.perm, None, buf.seg_of,
                    buf.n_unique, buf.err_count, buf.tag_dedup_ws)
    e1.record()
    torch.cuda.synchronize()
    return {"ids": n, "distinct": distinct, "turned_away": refused, "table_slots_log2": 23,
            "insert_all_ids_ms": round(float(np.median(ms)), 4), "insert_all_ids_ms_all": [round(m, 4) for m in ms],
            "emb_tag_dedup_ms": round(sort_ms, 4), "emb_tag_dedup_with_position_ordered_inverse_ms": round(e0.elapsed_time(e1), 4),
            "note": "find-or-insert of all IDs of one batch (duplicates included) into an empty table with 16-byte rows: "
                    "stage one of a hash-based deduplication (dense numbers in arrival order), next to the whole "
                    "sort-based call, which also delivers ascending distinct keys, perm and segments"}


def ceiling_probes(B, timed, dev) -> dict:
    """What the part delivers to kernels of this library's access shapes, measured with the library's own row
    movers on synthetic indices (2 GiB of 256-byte rows) and with the runtime's fill / copy for comparison."""
    rows = 1 << 23                                     # 8 M rows x 256 B = 2 GiB
    dim = 64
    src = torch.empty((rows, dim), dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    nbytes = src.numel() * 4
    ident = torch.arange(rows, dtype=torch.int32, device=dev)
    g = torch.Generator(device=dev).manual_seed(1)
    rnd = torch.randperm(rows, generator=g, device=dev).to(torch.int32)
    quarter = (ident // 4).contiguous()
    out = {"buffer_bytes": nbytes}
    ms = timed(lambda: dst.fill_(2.0))
    out["runtime_fill_write_gbps"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    ms = timed(lambda: dst.copy_(src))
    out["runtime_copy_read_plus_write_gbps"] = round(2 * nbytes / (ms * 1e-3) / 1e9, 1)
    ms = timed(lambda: B.emb_expand(src, ident, rows, dim, 0, dst))
    out["row_copy_sequential_read_plus_write_gbps"] = round((2 * nbytes + 4 * rows) / (ms * 1e-3) / 1e9, 1)
    ms = timed(lambda: B.emb_expand(src, rnd, rows, dim, 0, dst))
    out["random_row_read_sequential_write_gbps"] = round((2 * nbytes + 4 * rows) / (ms * 1e-3) / 1e9, 1)
    ms = timed(lambda: B.emb_expand_sorted(src, quarter, rnd, rows, dim, 0, dst))
    out["quarter_read_random_row_write_gbps"] = round((nbytes // 4 + nbytes + 8 * rows) / (ms * 1e-3) / 1e9, 1)
    # reads only: the segment reduction over one giant segment (every row is read once, one row is written)
    zeros = torch.zeros(rows, dtype=torch.int32, device=dev)
    red = torch.empty((1, dim), dtype=torch.float32, device=dev)
    rws = torch.empty(B.grad_segment_reduce_workspace_bytes(rows, dim), dtype=torch.uint8, device=dev)
    ms = timed(lambda: B.grad_segment_reduce(src, 0, zeros, ident, rows, dim, red, rws))
    out["row_read_sequential_gbps"] = round((nbytes + 8 * rows) / (ms * 1e-3) / 1e9, 1)
    ms = timed(lambda: B.grad_segment_reduce(src, 0, zeros, rnd, rows, dim, red, rws))
    out["row_read_random_gbps"] = round((nbytes + 8 * rows) / (ms * 1e-3) / 1e9, 1)
    # bare access patterns (emb_probe_memory): what the memory system gives kernels that only read, only write, or
    # store one row per 4 / per 64 rows read; 256-byte rows, 16 lanes per row, loads overlapped as in the row kernels
    quarter_rows = torch.empty((rows // 4, dim), dtype=torch.float32, device=dev)
    for name, pattern, idx, moved in (
            ("bare_read_sequential_gbps", B.PROBE_READ, None, nbytes),
            ("bare_read_random_rows_gbps", B.PROBE_READ, rnd, nbytes + 4 * rows),
            ("bare_write_sequential_gbps", B.PROBE_WRITE, None, nbytes),
            ("bare_write_random_rows_gbps", B.PROBE_WRITE, rnd, nbytes + 4 * rows),
            ("bare_read_random_rows_store_every_64th_gbps", B.PROBE_READ_STORE_64TH, rnd, nbytes + 4 * rows + nbytes // 64),
            ("bare_read_random_rows_store_every_4th_gbps", B.PROBE_READ_STORE_4TH, rnd, nbytes + 4 * rows + nbytes // 4)):
        target = dst if pattern == B.PROBE_WRITE else quarter_rows
        ms = timed(lambda: B.emb_probe_memory(pattern, src, target, idx, rows))
        out[name] = round(moved / (ms * 1e-3) / 1e9, 1)
    del quarter_rows
    out["note"] = ("kernels of this library on synthetic indices: row mover with identity index (streaming copy), with a "
                   "random permutation as source index (the gather's shape), with one source row per four positions and a "
                   "random destination permutation (the sorted expand's shape); segment reduction of all rows into one "
                   "segment in sequential and in random row order (the reduce's shape: reads only); bare_*: "
                   "emb_probe_memory, kernels that do nothing but the named accesses over the same 256-byte rows")
    return out


def profiled_traffic(kernel: str, config: int):
    """HBM bytes per dispatch of `kernel` from profiles/hbm_traffic_config<config>_step.txt (None if absent)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_config{config}_step.txt")
    try:
        for line in open(path):
            parts = [p.strip() for p in line.split("|")]
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_dispatch" and parts[1] == kernel:
                return int(float(parts[2]))
    except OSError:
        pass
    return None


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, batch0, tag_bits, dim, dtype, n_keys) -> dict:
    """The CPU checker as it stands, one thread, timed on one whole step of the first batch, three repetitions,
    median (about 15 s of CPU work).  Pre-existing keys the step touches are materialised first (untimed), as the
    lazy checker does."""
    import oracle
    x, off, tags = batch0
    n_fields = len(tags)
    n = int(off[n_fields])
    x, off, tags = x[:n], off[:n_fields + 1], tags[:n_fields]
    log("cpu baseline: preparing (untimed)")
    key, _ = oracle.tag_keys(x, off, tags, tag_bits)
    uniq, _, _ = oracle.dedup(key)
    rng = np.random.Generator(np.random.Philox(key=1234))
    G = rng.standard_normal((len(x), dim), dtype=np.float32)
    times = []
    for rep in range(3):
        t = oracle.Table(dim, dtype)
        t.prepopulate(uniq)
        log(f"cpu baseline: timing repetition {rep + 1} of 3")
        t0 = time.perf_counter()
        key, _ = oracle.tag_keys(x, off, tags, tag_bits)
        uniq, inverse, _ = oracle.dedup(key)
        t.find_or_insert(uniq, 1)
        E_u = t.lookup(uniq)
        E = oracle.expand(E_u, inverse)
        g = oracle.segment_reduce(G, inverse, len(uniq))
        t.apply_adagrad(uniq, g, w.lr, w.eps)
        times.append(time.perf_counter() - t0)
        assert E.shape == (len(x), dim)
        del t, E, E_u, g
    dt = float(np.median(times))
    return {"value": round(len(x) / dt, 1), "unit": "IDs/s", "cores": 1, "kind": "oracle",
            "sample": f"one full step over the first {n_fields} of {len(batch0[2])} fields of batch 0 ({len(x)} IDs, "
                      f"{len(uniq)} unique), touched keys pre-materialised, median of 3 repetitions",
            "seconds": round(dt, 2), "seconds_all": [round(v, 2) for v in times], "host_cpus": os.cpu_count(),
            "cpu_model": cpu_model()}


if __name__ == "__main__":
    sys.exit(main())
