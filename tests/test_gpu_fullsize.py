"""Parity at the published sizes, in the launch configuration bench.py times (needs an MI355X).

The integer work (tagged keys, distinct keys, inverse indices, counts) is compared in full; row
contents, exact integer-valued reduced gradients, updated rows and insert flags are compared on a
sample of distinct keys that always contains the longest segments.  Pre-existing keys are
materialised in the checker only when touched (an untouched row is a pure function of its key).
"""
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import make_config, merged_inputs

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2505_12663_amd import binding as B
    from paper_2505_12663_amd import EmbeddingTable, StepBuffers
    from harness import Pair, run_step_sampled, tracked_subset, dev_keys, host_keys, check_reduce_normal_sampled


def _bulk_load(pair, w, tag_bits, slice_n=1 << 23):
    """Insert ranks [0, P) of every logical table at step 0; returns per-table sorted arrays of the
    pre-existing raw IDs (for the lazy membership test)."""
    dk = torch.empty(slice_n, dtype=torch.int64, device="cuda")
    rows = torch.empty(slice_n, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int64, device="cuda")
    for t in range(w.n_tables):
        P = w.prepopulated[t]
        tag = torch.tensor([t], dtype=torch.uint8, device="cuda")
        for lo in range(0, P, slice_n):
            hi = min(P, lo + slice_n)
            x = dev_keys(w.prepopulated_ids(t, lo, hi))
            off = torch.tensor([0, hi - lo], dtype=torch.int64, device="cuda")
            B.emb_tag_keys(x, off, tag, tag_bits, dk, err)
            pair.gpu.find_or_insert(dk, None, hi - lo, 0, rows)
        print(f"  bulk load: table {t} ({P} keys)", flush=True)


def _membership(w, tag_bits):
    """tagged key -> was it loaded at step 0?  Uses the workload's rank <-> ID bijection."""
    from workloads import unscramble_bits
    shift = 63 - tag_bits

    def is_pre(keys):
        tags = (keys >> np.uint64(shift)).astype(np.int64)
        raw = keys & np.uint64((1 << shift) - 1)
        out = np.zeros(len(keys), dtype=bool)
        for t in range(w.n_tables):
            m = tags == t
            if m.any():
                out[m] = unscramble_bits(raw[m], w.id_bits, w.table_seed(t)) < np.uint64(w.prepopulated[t])
        return out
    return is_pre


def _hot_keys(w, tag_bits, per_table=2):
    """Tagged keys of the most popular ranks of every logical table (the longest segments)."""
    shift = 63 - tag_bits
    ks = [w.raw_ids_of_ranks(t, np.arange(per_table, dtype=np.uint64)) | np.uint64(t << shift) for t in range(w.n_tables)]
    return np.concatenate(ks)


def test_config2_full_size_two_steps():
    w = make_config(2)
    merged, n_merged = B.emb_plan_merge([64] * 8, [0] * 8)
    tag_bits = B.emb_tag_bits(8)
    pair = Pair(64, 0, capacity_log2=27, chunk_rows_log2=24, count_probes=True)
    _bulk_load(pair, w, tag_bits)
    st = pair.gpu.stats()
    assert st["live"] == 50_000_000 and st["status"] == 0
    buf = StepBuffers(512 * 4096 * 8, 64)
    is_pre = _membership(w, tag_bits)
    tracked = tracked_subset(_hot_keys(w, tag_bits))
    for step in (1, 2):
        b = w.next_step(step - 1)
        x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
        n, U, n_new = run_step_sampled(pair, buf, x, off, tags, tag_bits, step, w.lr, w.eps, 11 + step, is_pre, tracked,
                                       id_bits=w.id_bits)
        print(f"  step {step}: N={n} U={U} new={n_new}", flush=True)
        assert n_new == 0 and 0.15 < U / n < 0.35
    # the same segments with N(0,1) gradients: fp32 sums in the kernel's fixed order against fp64 sums in input order
    okey, _ = oracle.tag_keys(x, off, tags, tag_bits)
    n_seg = check_reduce_normal_sampled(buf, okey, 64, 0, tracked, 99)
    print(f"  N(0,1) reduce: {n_seg} tracked segments within 1e-5", flush=True)
    assert n_seg > 3000
    st = pair.gpu.stats()
    assert st["live"] == 50_000_000 and st["status"] == 0 and st["n_rehash"] == 0
    pair.gpu.close()


def test_config2_low_cardinality_fields_segments_of_hundreds_of_thousands():
    """The long-sequence shape with realistic per-field vocabularies: action, scene, hour fields with a handful of
    values give segments of 10^5..10^6 positions, the worst case for the segmented reduction (many levels of
    partial rows for one segment) and the best case for the sorted expand.  Dedup, expand and reduce are compared
    with the checker in full (integer-valued gradients: one correct fp32 answer)."""
    from workloads import small_int_grads
    w = make_config(2, field_vocab=[6_250_000, 20_000, 6_250_000, 500_000, 100, 24, 8, 50])
    merged, n_merged = B.emb_plan_merge([64] * 8, [0] * 8)
    tag_bits = B.emb_tag_bits(8)
    b = w.next_step(0)
    x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
    n, dim = len(x), 64
    okey, _ = oracle.tag_keys(x, off, tags, tag_bits)
    ouniq, oinv, ocnt = oracle.dedup(okey)
    U = len(ouniq)
    assert ocnt.max() > 300_000 and U < n // 8
    buf = StepBuffers(n, dim)
    B.emb_tag_keys(dev_keys(x), torch.from_numpy(off).cuda(), torch.from_numpy(tags).cuda(), tag_bits, buf.key, buf.err_count)
    B.emb_dedup(buf.key, n, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of, buf.n_unique, buf.dedup_ws)
    assert int(buf.n_unique.item()) == U
    assert np.array_equal(host_keys(buf.uniq[:U]), ouniq)
    assert np.array_equal(buf.inverse[:n].cpu().numpy(), oinv)
    assert np.array_equal(buf.counts[:U].cpu().numpy(), ocnt)
    print(f"  dedup: N={n} U={U} longest segment {int(ocnt.max())}", flush=True)
    # expand, both forms, against the definition
    gen = torch.Generator(device="cuda").manual_seed(5)
    buf.uniq_rows[:U].normal_(generator=gen)
    inv_dev = buf.inverse[:n].long()
    B.emb_expand_sorted(buf.uniq_rows, buf.seg_of, buf.perm, n, dim, 0, buf.out)
    assert torch.equal(buf.out[:n], buf.uniq_rows[:U][inv_dev])
    buf.out.zero_()
    B.emb_expand(buf.uniq_rows, buf.inverse, n, dim, 0, buf.out)
    assert torch.equal(buf.out[:n], buf.uniq_rows[:U][inv_dev])
    # reduce: integers in [-8, 8]; the longest segment sums 4e5 of them, exact in fp32 in any order
    G = small_int_grads(n, dim, 21, "cuda")
    B.grad_segment_reduce(G, 0, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
    og = oracle.segment_reduce(G.cpu().numpy(), oinv, U)
    assert np.array_equal(buf.reduced[:U].cpu().numpy(), og)
    print("  expand and reduce exact", flush=True)


def test_config3_full_size_merged_tables():
    w = make_config(3)
    dims = [w.table_dim(t) for t in range(w.n_tables)]
    merged, n_merged = B.emb_plan_merge(dims, [0] * w.n_tables)
    om, on = oracle.plan_merge(dims, [0] * w.n_tables)
    assert n_merged == on == 4 and np.array_equal(merged, om)
    sig = [dims[list(merged).index(g)] for g in range(n_merged)]
    pairs = [Pair(d, 0, capacity_log2=22, chunk_rows_log2=20) for d in sig]
    bufs = [StepBuffers(1024 * 200 * 14, d) for d in sig]
    nobody = lambda keys: np.zeros(len(keys), dtype=bool)        # tables start empty
    tracked = tracked_subset(_hot_keys(w, 8, per_table=1))
    for step in range(3):
        b = w.next_step(step)
        tot = 0
        for g in range(n_merged):
            x, off, tags, sel = merged_inputs(w.features, b.ids, merged, g)
            assert len(x) <= bufs[g].n_max
            n, U, n_new = run_step_sampled(pairs[g], bufs[g], x, off, tags, 8, step, w.lr, w.eps, 5 + g, nobody,
                                           tracked, id_bits=w.id_bits)
            tot += n
        print(f"  step {step}: total IDs {tot}", flush=True)
        assert 3_000_000 < tot < 5_500_000
    for p in pairs:
        assert p.gpu.stats()["status"] == 0
        p.gpu.close()


def test_config4_full_batch_insert_evict_rehash():
    """Full batch (512 x 1024 x 4 = 2.1 M IDs per step) with the configuration's own eviction clock (unseen for 200
    steps, or touched fewer than 3 times and unseen for 20; every 20 steps; load-factor limit 0.85), for the first
    260 of the 1000 streaming steps: long enough for several limit-driven rehashes and for the 200-step rule to fire.
    The checker mirrors the tracked subset of keys (a fixed 1/512 of the key space plus the hottest keys) exactly
    through every step and every eviction: insert flags, touch records, exact integer-valued reduced gradients,
    updated rows, eviction sets.  On all keys: the distinct keys and inverse indices (in full against the checker
    every tenth step, by properties otherwise), the eviction predicate on a dump of the records, the counters."""
    from harness import small_int_rows, close_rows
    from paper_2505_12663_amd import forward, backward
    from workloads import small_int_grads
    w = make_config(4)
    assert (w.ttl, w.min_freq, w.grace, w.evict_every, w.max_load_factor) == (200, 3, 20, 20, 0.85)
    merged, _ = B.emb_plan_merge([64] * 4, [0] * 4)
    tag_bits = B.emb_tag_bits(4)
    # 260 steps by default (about 95 s); MTGR_CONFIG4_STEPS=1000 runs the configuration's whole stream (about 6 minutes)
    dim, steps = 64, int(os.environ.get("MTGR_CONFIG4_STEPS", "260"))
    pair = Pair(dim, 0, capacity_log2=22, chunk_rows_log2=21, max_load_factor=w.max_load_factor, count_probes=True)
    buf = StepBuffers(512 * 1024 * 4, dim)
    tracked = tracked_subset(_hot_keys(w, tag_bits))
    rehash_at, lf_at_refusal, evicted_total = [], [], 0
    for step in range(steps):
        b = w.next_step(step)
        x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
        n = len(x)
        okey, _ = oracle.tag_keys(x, off, tags, tag_bits)
        refused_before, rehash_before = pair.gpu._refused_seen, pair.gpu.stats()["n_rehash"]
        pair.gpu.peak_load = 0.0
        forward(pair.gpu, buf, dev_keys(x), torch.from_numpy(off).cuda(), torch.from_numpy(tags).cuda(), tag_bits, step,
                id_bits=w.id_bits)
        U = int(buf.n_unique.item())
        if pair.gpu._refused_seen > refused_before:
            lf_at_refusal.append(pair.gpu.peak_load)       # what the counters showed when keys were turned away
        # ---- all keys: distinct keys and inverse
        assert np.array_equal(host_keys(buf.key[:n]), okey)
        if step % 10 == 0:
            ou, oi, oc = oracle.dedup(okey)
            assert U == len(ou) and np.array_equal(host_keys(buf.uniq[:U]), ou)
            assert np.array_equal(buf.inverse[:n].cpu().numpy(), oi) and np.array_equal(buf.counts[:U].cpu().numpy(), oc)
        else:
            u = buf.uniq[:U]
            assert bool((u[1:] > u[:-1]).all()) and torch.equal(u[buf.inverse[:n].long()], buf.key[:n])
        assert bool((buf.row_idx[:U] >= 0).all())
        # ---- tracked subset through the checker
        pos = np.flatnonzero(tracked(okey))
        skeys, sinv = np.unique(okey[pos], return_inverse=True)
        oins = pair.orc.find_or_insert(skeys, step)
        sidx = torch.from_numpy(np.searchsorted(host_keys(buf.uniq[:U]), skeys)).cuda()
        assert np.array_equal(host_keys(buf.uniq[sidx]), skeys)
        assert np.array_equal(buf.inserted[sidx].cpu().numpy(), oins), "insert flags (tracked keys)"
        E_u = buf.uniq_rows[sidx].cpu().numpy()
        oE_u = pair.orc.lookup(skeys)
        never = pair.orc.peek(skeys)[2] == 0
        assert np.array_equal(E_u[never], oE_u[never]) and close_rows(E_u, oE_u.astype(np.float64), w.lr, pair.rtol)
        assert torch.equal(buf.out[torch.from_numpy(pos).cuda()], buf.uniq_rows[sidx][torch.from_numpy(sinv).cuda()])
        backward(pair.gpu, buf, small_int_grads(n, dim, step, "cuda"), n, w.lr, w.eps)
        og = np.zeros((len(skeys), dim), dtype=np.float64)
        np.add.at(og, sinv, small_int_rows(pos, dim, step).astype(np.float64))
        og = og.astype(np.float32)
        assert np.array_equal(buf.reduced[sidx].cpu().numpy(), og), "reduced gradients (tracked keys, exact)"
        pair.orc.apply_adagrad(skeys, og, w.lr, w.eps)
        rows_after = torch.empty((len(skeys), dim), dtype=torch.float32, device="cuda")
        pair.gpu.gather(buf.row_idx[sidx].contiguous(), None, len(skeys), rows_after)
        assert close_rows(rows_after.cpu().numpy(), pair.orc.lookup(skeys).astype(np.float64), w.lr, pair.rtol)
        # ---- eviction
        if (step + 1) % w.evict_every == 0:
            gk, _, ga, gl, gf = pair.gpu.export_device(values=False)
            age = step - gl.long()
            go = (age >= w.ttl) | ((gf < w.min_freq) & (age >= w.grace))
            expect = torch.sort(gk[go]).values
            # the tracked keys' records against the checker's, bit for bit (accumulators within the bound)
            hk = host_keys(gk)
            sel = np.flatnonzero(tracked(hk))
            order = sel[np.argsort(hk[sel], kind="stable")]
            ok, ov, oa, ol, of = pair.orc.export()
            assert np.array_equal(hk[order], ok), "tracked key set"
            d_order = torch.from_numpy(order).cuda()
            assert np.array_equal(gl[d_order].cpu().numpy().view(np.uint32), ol)
            assert np.array_equal(gf[d_order].cpu().numpy().view(np.uint32), of)
            assert np.allclose(ga[d_order].cpu().numpy(), oa, rtol=1e-5, atol=1e-12)
            ev, n_ev = pair.gpu.evict(step, w.ttl, w.min_freq, w.grace)
            assert n_ev == expect.numel() and torch.equal(torch.sort(ev).values, expect)
            oev = pair.orc.evict(step, w.ttl, w.min_freq, w.grace)
            hev = host_keys(ev)
            assert np.array_equal(np.sort(hev[tracked(hev)]), oev), "eviction set (tracked keys)"
            if n_ev:
                found = torch.empty(n_ev, dtype=torch.int32, device="cuda")
                pair.gpu.find(ev.contiguous(), None, n_ev, found)
                assert bool((found == -1).all())
            evicted_total += n_ev
        st = pair.gpu.stats()
        lf = (st["live"] + st["tombstones"]) / st["capacity"]
        assert st["status"] == 0 and st["rows_free"] + st["live"] == st["rows_used"] and lf <= float(np.float32(w.max_load_factor))
        if st["n_rehash"] > rehash_before:
            rehash_at.append(step)
        if step % 10 == 9 or st["n_rehash"] > rehash_before:
            print(f"  step {step}: U={U} live={st['live']} deleted={st['tombstones']} cap=2^{int(np.log2(st['capacity']))} "
                  f"load={lf:.3f} rehash={st['n_rehash']} turned away so far={st['refused']} evicted so far={evicted_total}", flush=True)
    st = pair.gpu.stats()
    print(f"  rehashes at steps {rehash_at}; load factor when keys were turned away: {[round(v, 4) for v in lf_at_refusal]}; "
          f"lines per lookup {st['probes'] / st['lookups']:.3f}, CAS failures {st['cas_failures']} of {st['cas_attempts']}", flush=True)
    # the key structure was expanded only when the device had turned keys away at the limit (Sec. 3.1)
    assert len(rehash_at) >= 2 and len(lf_at_refusal) == len(rehash_at)
    assert all(0.84 <= v <= float(np.float32(w.max_load_factor)) for v in lf_at_refusal)      # the limit is a float32
    assert evicted_total > 1_000_000
    pair.gpu.close()


def test_config5_full_size_bf16_400m_keys():
    w = make_config(5)
    merged, _ = B.emb_plan_merge([128] * 4, [1] * 4)
    tag_bits = B.emb_tag_bits(4)
    pair = Pair(128, 1, capacity_log2=29, chunk_rows_log2=26, max_load_factor=0.75)
    for _ in range(6):                       # 8 chunks of 2^26 rows = 537 M rows (~137 GB of bf16 rows)
        pair.gpu.add_chunk()
    _bulk_load(pair, w, tag_bits, slice_n=1 << 24)
    st = pair.gpu.stats()
    assert st["live"] == 400_000_000 and st["status"] == 0
    print(f"  table: load {st['live'] / st['capacity']:.3f}", flush=True)
    buf = StepBuffers(2048 * 2048 * 4, 128, 1)
    is_pre = _membership(w, tag_bits)
    b = w.next_step(0)
    x, off, tags, _ = merged_inputs(w.features, b.ids, merged, 0)
    n, U, n_new = run_step_sampled(pair, buf, x, off, tags, tag_bits, 1, w.lr, w.eps, 3, is_pre,
                                   tracked_subset(_hot_keys(w, tag_bits)), id_bits=w.id_bits)
    print(f"  step 1: N={n} U={U} new={n_new}", flush=True)
    okey, _ = oracle.tag_keys(x, off, tags, tag_bits)
    n_seg = check_reduce_normal_sampled(buf, okey, 128, 1, tracked_subset(_hot_keys(w, tag_bits)), 98)   # bf16 N(0,1) gradients
    print(f"  N(0,1) bf16 reduce: {n_seg} tracked segments within 1e-5", flush=True)
    st = pair.gpu.stats()
    assert n == 2048 * 2048 * 4 and 0.02 < n_new / U < 0.09          # ~5 % of the distinct keys are new
    assert st["live"] == 400_000_000 + n_new and st["status"] == 0
    assert st["n_rehash"] == 0 and st["capacity"] == 1 << 29 and st["refused"] == 0   # 0.7458 < 0.75: still fits
    # 3 M keys never issued before push the table over the limit: the device admits keys up to
    # floor(0.75 * 2^29) slots, the owner expands the key structure (values do not move) and re-issues the call
    fresh = w.raw_ids_of_ranks(0, np.arange(w._issued[0], w._issued[0] + 3_000_000, dtype=np.uint64))
    rows = torch.empty(len(fresh), dtype=torch.int32, device="cuda")
    pair.gpu.peak_load = 0.0
    pair.gpu.find_or_insert(dev_keys(fresh), None, len(fresh), 2, rows)       # tag 0: the raw ID is the key
    st = pair.gpu.stats()
    print(f"  +3 M keys: turned away at load {pair.gpu.peak_load:.4f}: {st['refused']}, capacity 2^{int(np.log2(st['capacity']))}", flush=True)
    assert st["live"] == 400_000_000 + n_new + 3_000_000 and st["status"] == 0 and bool((rows >= 0).all())
    assert st["n_rehash"] == 1 and st["capacity"] == 1 << 30 and st["refused"] > 0 and 0.7499 < pair.gpu.peak_load <= 0.75
    pick = np.arange(0, len(fresh), 300_007)
    got = torch.empty((len(pick), 128), dtype=torch.bfloat16, device="cuda")
    pair.gpu.gather(rows[torch.from_numpy(pick).cuda()].contiguous(), None, len(pick), got)
    ref = np.stack([oracle.init_row(int(k), 128, dtype=1) for k in fresh[pick]])
    assert np.array_equal(got.float().cpu().numpy(), ref)             # new rows are the key-seeded initial rows
    pair.gpu.close()


def test_dedup_beyond_2_pow_30_keys():
    """Largest sizes: n just above 2^30 (the entry point takes n < 2^31).  Checked by properties that hold at any
    size: distinct keys strictly ascending, uniq[inverse] == key, the sorted order is a stable sort of the keys,
    segment offsets and counts agree with it."""
    n = (1 << 30) + 12345
    g = torch.Generator(device="cuda").manual_seed(7)
    key = torch.randint(0, 1 << 40, (n,), generator=g, device="cuda", dtype=torch.int64)
    key[: n // 2] &= (1 << 22) - 1                       # half of the keys from a 4 M-key vocabulary: long segments
    key |= torch.randint(0, 26, (n,), generator=g, device="cuda", dtype=torch.int64) << 55
    key[-5:] = key[0].clone()
    uniq = torch.empty(n, dtype=torch.int64, device="cuda")
    inverse = torch.empty(n, dtype=torch.int32, device="cuda")
    perm = torch.empty(n, dtype=torch.int32, device="cuda")
    seg_off = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    seg_of = torch.empty(n, dtype=torch.int32, device="cuda")
    n_unique = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.emb_dedup_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    print(f"  n={n}, workspace {ws.numel() / 2**30:.1f} GiB", flush=True)
    B.emb_dedup(key, n, uniq, inverse, None, perm, seg_off, seg_of, n_unique, ws)
    U = int(n_unique.item())
    del ws
    print(f"  U={U}", flush=True)
    assert 0 < U < n
    u = uniq[:U]
    assert bool((u[1:] > u[:-1]).all())                                   # strictly ascending, hence distinct
    assert bool((inverse >= 0).all()) and int(inverse.max().item()) == U - 1
    step = 1 << 28                                                        # check in slices to bound temporaries
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        assert torch.equal(u[inverse[lo:hi].long()], key[lo:hi])          # every key maps to its own distinct key
        p = perm[lo:hi].long()
        sk = key[p]
        assert torch.equal(u[seg_of[lo:hi].long()], sk)                   # sorted order carries the right segment
        assert bool((sk[1:] >= sk[:-1]).all())
        assert bool(((sk[1:] != sk[:-1]) | (p[1:] > p[:-1])).all())       # equal keys keep their input order
    assert int(seg_off[0].item()) == 0 and int(seg_off[U].item()) == n
    so = seg_off[: U + 1].long()
    assert bool((so[1:] > so[:-1]).all())
    assert torch.equal(seg_of[so[:-1]].long(), torch.arange(U, device="cuda"))   # a segment starts where seg_off says
    # perm is a permutation: every position appears once
    seen = torch.zeros(n, dtype=torch.uint8, device="cuda")
    seen[perm.long()] = 1
    assert bool(seen.all())


def test_tag_dedup_of_forty_million_ids_equals_tag_then_dedup():
    """The fused call on more IDs than its smallest-launch layout covers (above 8192 sort tiles the per-tile counts
    of distinct keys go through their own prefix-sum launch): every output must equal, bit for bit, that of the
    unfused pair emb_tag_keys + emb_dedup, which shares no kernel with it; the properties that hold at any size are
    checked on top (Eq. 8 keys, ascending distinct keys, stable order inside a segment)."""
    n_fields, tag_bits, id_bits = 6, 4, 26
    lens = [9_000_001, 3, 12_345_678, 0, 18_000_000, 654_321]
    n = sum(lens)
    assert n > 8192 * 4096
    g = torch.Generator(device="cuda").manual_seed(11)
    x = torch.randint(0, 1 << id_bits, (n,), generator=g, device="cuda", dtype=torch.int64)
    x[: lens[0] // 2] &= (1 << 12) - 1                                    # long segments in the first field
    x[-7:] = x[-8].clone()
    off = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64, device="cuda")
    tags = torch.tensor([5, 0, 9, 3, 15, 1], dtype=torch.uint8, device="cuda")

    def outputs():
        return dict(key=torch.empty(n, dtype=torch.int64, device="cuda"), uniq=torch.empty(n, dtype=torch.int64, device="cuda"),
                    inverse=torch.empty(n, dtype=torch.int32, device="cuda"), counts=torch.empty(n, dtype=torch.int32, device="cuda"),
                    perm=torch.empty(n, dtype=torch.int32, device="cuda"), seg_off=torch.empty(n + 1, dtype=torch.int32, device="cuda"),
                    seg_of=torch.empty(n, dtype=torch.int32, device="cuda"), n_unique=torch.zeros(1, dtype=torch.int64, device="cuda"),
                    err=torch.zeros(1, dtype=torch.int64, device="cuda"))
    a, b = outputs(), outputs()
    ws = torch.empty(B.emb_tag_dedup_workspace_bytes(n, n_fields, tag_bits, id_bits), dtype=torch.uint8, device="cuda")
    print(f"  n={n}", flush=True)
    B.emb_tag_dedup(x, off, tags, tag_bits, id_bits, a["key"], a["uniq"], a["inverse"], a["counts"], a["perm"], a["seg_off"],
                    a["seg_of"], a["n_unique"], a["err"], ws)
    U = int(a["n_unique"].item())
    print(f"  fused: U={U}", flush=True)
    del ws
    B.emb_tag_keys(x, off, tags, tag_bits, b["key"], b["err"])
    ws = torch.empty(B.emb_dedup_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    B.emb_dedup(b["key"], n, b["uniq"], b["inverse"], b["counts"], b["perm"], b["seg_off"], b["seg_of"], b["n_unique"], ws)
    assert int(b["n_unique"].item()) == U and int(a["err"].item()) == int(b["err"].item()) == 0
    print("  unfused pair done", flush=True)
    assert torch.equal(a["key"], b["key"])
    for name, m in (("uniq", U), ("inverse", n), ("counts", U), ("perm", n), ("seg_off", U + 1), ("seg_of", n)):
        assert torch.equal(a[name][:m], b[name][:m]), name
    # properties
    field = torch.repeat_interleave(tags.long(), torch.tensor(lens, device="cuda"))
    assert torch.equal(a["key"], (field << (63 - tag_bits)) | x)          # Eq. 8, bit 63 stays clear
    u = a["uniq"][:U]
    assert bool((u[1:] > u[:-1]).all())
    assert torch.equal(u[a["inverse"].long()], a["key"])
    p = a["perm"].long()
    sk = a["key"][p]
    assert bool(((sk[1:] > sk[:-1]) | ((sk[1:] == sk[:-1]) & (p[1:] > p[:-1]))).all())
    assert int(a["seg_off"][U].item()) == n and int(a["counts"][:U].long().sum().item()) == n
