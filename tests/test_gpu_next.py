"""Compositions of the entry points that the paper describes around the single-device path (needs an MI355X):
two-stage deduplication over the ID lists of several emulated peers (Sec. 3.3) and sparse gradient
accumulation over micro-batches (App. C), both checked against the CPU checker's plain definitions."""
import numpy as np
import pytest
import torch

import oracle
from workloads import make_config, merged_inputs, normal_grads

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2505_12663_amd import binding as B
    from paper_2505_12663_amd import EmbeddingTable, StepBuffers
    from harness import dev_keys, host_keys, close_reduce, close_rows, RTOL_F32, RTOL_BF16


def _dedup(buf, keys_dev, n):
    B.emb_dedup(keys_dev, n, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of, buf.n_unique, buf.dedup_ws)
    return int(buf.n_unique.item())


def test_two_stage_dedup_over_emulated_peers():
    """Each of P peers deduplicates its own IDs (stage 1) and sends the distinct ones; the owner
    deduplicates what it received (stage 2), looks the distinct keys up once, returns one row per
    received ID, and every peer expands.  The result must equal looking every ID up directly."""
    P, dim = 4, 32
    w = make_config(1, batch=128)
    b = w.next_step(0)
    x, off, tags, _ = merged_inputs(w.features, b.ids, [0], 0)
    key, _ = oracle.tag_keys(x, off, tags, 1)
    parts = np.array_split(key, P)
    table, ot = EmbeddingTable(dim, 0, capacity_log2=16, chunk_rows_log2=13), oracle.Table(dim)
    # stage 1 on every peer
    peer = []
    for p in range(P):
        n = len(parts[p])
        buf = StepBuffers(n, dim, with_grad=False)
        U = _dedup(buf, dev_keys(parts[p]), n)
        ou, oi, _ = oracle.dedup(parts[p])
        assert np.array_equal(host_keys(buf.uniq[:U]), ou) and np.array_equal(buf.inverse[:n].cpu().numpy(), oi)
        peer.append((buf, n, U))
    # "all-to-all" of IDs: the owner receives the concatenation of the peers' distinct keys
    received = torch.cat([buf.uniq[:U] for buf, n, U in peer])
    R = received.numel()
    own = StepBuffers(R, dim, with_grad=False)
    U2 = _dedup(own, received, R)                                   # stage 2: duplicates across peers
    assert U2 == len(np.unique(key)) and U2 < R
    table.find_or_insert(own.uniq, own.n_unique, R, 0, own.row_idx)
    table.gather(own.row_idx, own.n_unique, R, own.uniq_rows)
    B.emb_expand(own.uniq_rows, own.inverse, R, dim, 0, own.out)     # one row per received ID, in received order
    # "all-to-all" of rows back, then every peer expands with its stage-1 inverse
    outs, lo = [], 0
    for buf, n, U in peer:
        rows_for_peer = own.out[lo:lo + U].contiguous()
        lo += U
        B.emb_expand(rows_for_peer, buf.inverse, n, dim, 0, buf.out)
        outs.append(buf.out[:n])
    E = torch.cat(outs).cpu().numpy()
    assert np.array_equal(E, ot.direct_lookup(key, 0))              # dedup only removes repeated transmission
    assert table.stats()["live"] == len(ot) == U2
    table.close()


def test_sparse_gradient_accumulation_over_micro_batches():
    """Gradients of identical IDs across K micro-batches are accumulated and applied once (App. C):
    recorded (ID, gradient) pairs are concatenated, reduced per ID, and only activated rows are updated."""
    K, dim = 3, 64
    w = make_config(1, batch=96)
    table, ot = EmbeddingTable(dim, 0, capacity_log2=16, chunk_rows_log2=13), oracle.Table(dim)
    keys, grads = [], []
    for k in range(K):                                   # forward passes of the micro-batches: lookups only
        b = w.next_step(k)
        x, off, tags, _ = merged_inputs(w.features, b.ids, [0], 0)
        key, _ = oracle.tag_keys(x, off, tags, 1)
        n = len(key)
        buf = StepBuffers(n, dim, with_grad=False)
        U = _dedup(buf, dev_keys(key), n)
        table.find_or_insert(buf.uniq, buf.n_unique, n, k, buf.row_idx)
        ot.find_or_insert(np.unique(key), k)
        keys.append(key)
        grads.append(normal_grads(77, k, n, dim))
    allk, allg = np.concatenate(keys), np.concatenate(grads)
    n = len(allk)
    buf = StepBuffers(n, dim)
    U = _dedup(buf, dev_keys(allk), n)                   # merge the recorded IDs
    ou, oi, _ = oracle.dedup(allk)
    B.grad_segment_reduce(torch.from_numpy(allg).cuda(), 0, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
    og = oracle.segment_reduce(allg, oi, len(ou))
    sabs = oracle.segment_reduce(np.abs(allg), oi, len(ou)).astype(np.float64)
    assert close_reduce(buf.reduced[:U].cpu().numpy(), og.astype(np.float64), sabs, RTOL_F32)
    table.find(buf.uniq, buf.n_unique, n, buf.row_idx)   # rows of the activated keys (no touch: not a lookup step)
    table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, 0.01, 1e-8)
    ot.apply_adagrad(ou, og, 0.01, 1e-8)
    gk, gv, ga, gl, gf = table.export()
    ok, ov, oa, ol, of = ot.export()
    assert np.array_equal(gk, ok) and np.array_equal(gl, ol) and np.array_equal(gf, of)
    assert close_rows(gv, ov.astype(np.float64), 0.01, RTOL_F32) and np.allclose(ga, oa, rtol=1e-5)
    table.close()


@pytest.mark.parametrize("dim,dtype,mean", [(64, 0, False), (64, 0, True), (32, 0, True), (128, 1, False), (128, 1, True), (16, 0, False),
                                            (256, 0, True), (24, 0, False), (4, 0, True), (40, 1, True), (256, 1, False)])
def test_pooled_lookup_forward_and_backward(dim, dtype, mean):
    """Sum / mean pooling of every (sample, field) bag and its backward pass, against the checker
    (which is pinned to torch's EmbeddingBag): forward within 1e-5 of the float64 sums, backward with
    integer-valued output gradients bit-exact for the sum and within 1e-5 for the mean."""
    w = make_config(1, batch=200)
    b = w.next_step(0)
    x, off, tags, _ = merged_inputs(w.features, b.ids, [0], 0)
    lens = np.concatenate(b.lengths).astype(np.int64)            # field-major, sample-major: one bag per entry
    lens[5] += lens[6]; lens[6] = 0                              # make one bag empty (positions stay the same)
    bag_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n, nb = len(x), len(lens)
    assert bag_off[-1] == n
    key, _ = oracle.tag_keys(x, off, tags, 1)
    ou, oi, oc = oracle.dedup(key)
    table, ot = EmbeddingTable(dim, dtype, capacity_log2=16, chunk_rows_log2=13), oracle.Table(dim, dtype)
    buf = StepBuffers(n, dim, dtype)
    B.emb_dedup(dev_keys(key), n, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of, buf.n_unique, buf.dedup_ws)
    U = int(buf.n_unique.item())
    table.find_or_insert(buf.uniq, buf.n_unique, n, 0, buf.row_idx)
    table.gather(buf.row_idx, buf.n_unique, n, buf.uniq_rows)
    ot.find_or_insert(ou, 0)
    oE = oracle.expand(ot.lookup(ou), oi)
    d_off = torch.from_numpy(bag_off).cuda()
    ws = torch.empty(B.emb_pool_workspace_bytes(n, nb, dim), dtype=torch.uint8, device="cuda")
    pooled = torch.full((nb, dim), 5.0, device="cuda")
    B.emb_pool_bags(buf.uniq_rows, dtype, buf.inverse, d_off, n, dim, mean, pooled, ws)
    ref = oracle.pool_bags(oE, bag_off, mean).astype(np.float64)
    sabs = oracle.pool_bags(np.abs(oE), bag_off, mean).astype(np.float64)
    got = pooled.cpu().numpy()
    assert close_reduce(got, ref, sabs, RTOL_F32)
    assert (got[6] == 0).all()
    # backward
    rng = np.random.default_rng(4)
    dY = rng.integers(-4, 5, size=(nb, dim)).astype(np.float32)
    B.grad_segment_reduce_pooled(torch.from_numpy(dY).cuda(), d_off, buf.seg_of, buf.perm, n, dim, mean, buf.reduced, ws)
    G = oracle.pool_bags_backward(dY, bag_off, mean)
    og = oracle.segment_reduce(G, oi, U)
    g = buf.reduced[:U].cpu().numpy()
    if not mean:
        assert np.array_equal(g, og)                                         # integer sums: one correct answer
    else:
        sabs_g = oracle.segment_reduce(np.abs(G), oi, U).astype(np.float64)
        assert close_reduce(g, og.astype(np.float64), sabs_g, RTOL_F32)
    table.apply_adagrad(buf.row_idx, buf.reduced, buf.n_unique, n, 0.01, 1e-8)
    ot.apply_adagrad(ou, og, 0.01, 1e-8)
    gk, gv, ga, _, _ = table.export()
    ok, ov, oa, _, _ = ot.export()
    assert np.array_equal(gk, ok)
    assert close_rows(gv, ov.astype(np.float64), 0.01, RTOL_F32 if dtype == 0 else 1e-2)
    table.close()


@pytest.mark.parametrize("dim,dtype", [(64, 0), (32, 0), (128, 1), (16, 0), (256, 0), (24, 0), (4, 0), (40, 1)])
def test_sparse_adam_matches_checker(dim, dtype):
    """Lazy Adam on the activated rows only, several steps with new keys arriving and an eviction in
    between (moment rows of recycled rows must restart from zero)."""
    rtol = RTOL_F32 if dtype == 0 else 1e-2
    table = EmbeddingTable(dim, dtype, capacity_log2=13, chunk_rows_log2=10, adam_state=True, initial_chunks=2)
    ot = oracle.Table(dim, dtype)
    rng = np.random.default_rng(dim)
    pool = np.arange(1, 3001, dtype=np.uint64) * np.uint64(104729)
    for step in range(1, 9):
        ks = np.unique(pool[rng.integers(0, 300 * step, size=500)])
        n = len(ks)
        row_idx = torch.empty(n, dtype=torch.int32, device="cuda")
        table.find_or_insert(dev_keys(ks), None, n, step, row_idx)
        ot.find_or_insert(ks, step)
        g = normal_grads(3, step, n, dim)
        table.apply_adam(row_idx, torch.from_numpy(g).cuda(), None, n, 1e-3, step)
        ot.apply_adam(ks, g, 1e-3, step)
        if step == 5:
            ev, n_ev = table.evict(step, 3, 0, 0)            # drop keys unseen for 3 steps; their rows get reused
            oev = ot.evict(step, 3, 0, 0)
            assert np.array_equal(np.sort(host_keys(ev)), oev) and n_ev > 0
        gk, gv, ga, gl, gf = table.export()
        ok, ov, oa, ol, of = ot.export()
        assert np.array_equal(gk, ok) and np.array_equal(gl, ol) and np.array_equal(gf, of)
        assert close_rows(gv, ov.astype(np.float64), 1e-3, rtol), float(np.abs(gv - ov).max())
    st = table.stats()
    assert st["status"] == 0 and st["n_chunks"] >= 2
    table.close()
    # without moment rows the call is refused
    plain = EmbeddingTable(dim, dtype, capacity_log2=10, chunk_rows_log2=8)
    r = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(B.EmbError):
        plain.apply_adam(r, torch.zeros((4, dim), device="cuda"), None, 4, 1e-3, 1)
    plain.close()


def test_checkpoint_dump_restores_and_reshards_by_modulo():
    """Each device saves its own shard; a job resized from 1 to 2 devices reads the dump of rank
    r mod 1 and keeps the keys it owns (App. C).  Restored tables must hold exactly the dumped state."""
    dim = 32
    src = EmbeddingTable(dim, 0, capacity_log2=14, chunk_rows_log2=11)
    ot = oracle.Table(dim)
    rng = np.random.default_rng(2)
    pool = np.arange(1, 5001, dtype=np.uint64) * np.uint64(2654435761)
    for step in range(4):
        ks = np.unique(pool[rng.integers(0, 5000, size=1500)])
        row_idx = torch.empty(len(ks), dtype=torch.int32, device="cuda")
        src.find_or_insert(dev_keys(ks), None, len(ks), step, row_idx)
        g = normal_grads(1, step, len(ks), dim)
        src.apply_adagrad(row_idx, torch.from_numpy(g).cuda(), None, len(ks), 0.01, 1e-8)
        ot.find_or_insert(ks, step)
        ot.apply_adagrad(ks, g, 0.01, 1e-8)
    dump = src.export_device()
    ref = src.export()
    # same world size, different capacity: everything comes back bit for bit
    same = EmbeddingTable(dim, 0, capacity_log2=15, chunk_rows_log2=12)
    same.import_rows(*dump)
    for a, b in zip(ref, same.export()):
        assert np.array_equal(a, b)
    # two devices: owner(key) = key mod 2 stands in for the sharding function
    k = host_keys(dump[0])
    shards = []
    for r in range(2):
        m = torch.from_numpy((k % np.uint64(2)) == r).cuda()
        t = EmbeddingTable(dim, 0, capacity_log2=13, chunk_rows_log2=11)
        t.import_rows(dump[0][m], dump[1][m], dump[2][m], dump[3][m], dump[4][m])
        shards.append(t)
    parts = [t.export() for t in shards]
    assert sum(len(p[0]) for p in parts) == len(ref[0])
    merged = [np.concatenate([p[i] for p in parts]) for i in range(5)]
    order = np.argsort(merged[0], kind="stable")
    for i in range(5):
        assert np.array_equal(merged[i][order], ref[i])
    # and the checker agrees with what was restored (keys, counters; rows within tolerance)
    ok, ov, oa, ol, of = ot.export()
    assert np.array_equal(ref[0], ok) and np.array_equal(ref[3], ol) and np.array_equal(ref[4], of)
    assert close_rows(ref[1], ov.astype(np.float64), 0.01, RTOL_F32)
    for t in [src, same] + shards:
        t.close()


# --------------------------------------------------------------------------- hot / cold rows
def _bf16_rows(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def _mixed_pair(dim, hot_rows, cap_log2=14):
    from harness import RTOL_BF16  # noqa: F401
    table = EmbeddingTable(dim, B.BF16, capacity_log2=cap_log2, chunk_rows_log2=11, hot_rows=hot_rows)
    ot = oracle.Table(dim, oracle.BF16)
    ot.set_hot(hot_rows)
    return table, ot


def _insert(table, ot, ks, step):
    row_idx = torch.empty(len(ks), dtype=torch.int32, device="cuda")
    table.find_or_insert(dev_keys(ks), None, len(ks), step, row_idx)
    ot.find_or_insert(ks, step)
    return row_idx


@pytest.mark.parametrize("dim", [64, 24, 256])
def test_hot_cold_rows_match_checker(dim):
    """App. C mixed precision: keys touched often get an fp32 master, the rest stay 16-bit.  Promotion set, masters,
    delivered rows and the store's bookkeeping must follow the checker; a hot row's master to fp32 accuracy."""
    from harness import RTOL_BF16
    lr, eps = 0.05, 1e-8
    table, ot = _mixed_pair(dim, hot_rows=3000)
    rng = np.random.default_rng(dim)
    pool = (np.arange(1, 3001, dtype=np.uint64) * np.uint64(0x9E3779B1)) & np.uint64((1 << 40) - 1)
    # popularity: key i is drawn with weight 1/(i+1)
    wts = 1.0 / np.arange(1, 3001)
    wts /= wts.sum()
    for step in range(6):
        ks = np.unique(pool[rng.choice(3000, size=900, p=wts)])
        _insert(table, ot, ks, step)
    allk = np.sort(pool)
    row_idx = torch.empty(len(allk), dtype=torch.int32, device="cuda")
    table.find(dev_keys(allk), None, len(allk), row_idx)
    present = row_idx.cpu().numpy() >= 0
    n_prom = torch.zeros(1, dtype=torch.int64, device="cuda")
    table.promote(row_idx, None, len(allk), 4, n_prom)
    want = ot.promote(allk[present], 4)
    assert 0 < want < 3000 and int(n_prom.item()) == want
    hk, hv = table.export_hot()
    ok, ov = ot.export_hot()
    assert np.array_equal(hk, ok) and np.array_equal(hv, ov)          # a fresh master is the 16-bit row, exactly
    table.promote(row_idx, None, len(allk), 4, n_prom)
    assert int(n_prom.item()) == 0                                     # nothing is promoted twice
    st = table.stats()
    assert st["hot_rows_used"] == want and st["hot_rows_capacity"] == 3000
    # optimizer steps on random subsets, hot and cold rows mixed
    for step in range(6, 14):
        ks = np.unique(pool[rng.choice(3000, size=700, p=wts)])
        ri = _insert(table, ot, ks, step)
        g = normal_grads(3, step, len(ks), dim)
        table.apply_adagrad(ri, torch.from_numpy(g).cuda(), None, len(ks), lr, eps)
        ot.apply_adagrad(ks, g, lr, eps)
    hk, hv = table.export_hot()
    ok, ov = ot.export_hot()
    assert np.array_equal(hk, ok)
    assert close_rows(hv, ov.astype(np.float64), lr, RTOL_F32)        # masters: fp32 accuracy
    # delivered rows: gather and the fused lookup agree with each other and with the checker
    keys_now, vals_now, acc_now, _, freq_now = ot.export()
    row_idx = torch.empty(len(keys_now), dtype=torch.int32, device="cuda")
    table.find(dev_keys(keys_now), None, len(keys_now), row_idx)
    out = torch.empty((len(keys_now), dim), dtype=torch.bfloat16, device="cuda")
    table.gather(row_idx, None, len(keys_now), out)
    got = _bf16_rows(out)
    assert close_rows(got, vals_now.astype(np.float64), lr, RTOL_BF16)
    never = acc_now == 0
    assert never.any() and np.array_equal(got[never], vals_now[never])
    ident = torch.arange(len(keys_now), dtype=torch.int32, device="cuda")
    fused = torch.empty_like(out)
    B.ht_gather_expand_sorted(table.h, row_idx, ident, ident, len(keys_now), fused)
    assert torch.equal(fused.view(torch.int16), out.view(torch.int16))
    ek, ev, ea, _, ef = table.export()
    assert np.array_equal(ek, keys_now) and np.array_equal(ef, freq_now)
    assert np.array_equal(ev, got)                                      # the dump delivers what a lookup delivers
    # eviction returns masters to the store; re-promotion reuses them before taking new ones
    gone, n_gone = table.evict(14, 6, 0, 0)
    assert n_gone > 0 and np.array_equal(np.sort(host_keys(gone)), ot.evict(14, 6, 0, 0))
    hk2, _ = table.export_hot()
    ok2, _ = ot.export_hot()
    assert np.array_equal(hk2, ok2)
    st = table.stats()
    assert st["hot_rows_free"] == len(ok) - len(ok2) and st["hot_rows_used"] == want
    keys_now = ot.export()[0]
    row_idx = torch.empty(len(keys_now), dtype=torch.int32, device="cuda")
    table.find(dev_keys(keys_now), None, len(keys_now), row_idx)
    table.promote(row_idx, None, len(keys_now), 2, n_prom)
    want2 = ot.promote(keys_now, 2)
    assert int(n_prom.item()) == want2
    st = table.stats()
    reused = min(want2, len(ok) - len(ok2))
    assert st["hot_rows_free"] == len(ok) - len(ok2) - reused and st["hot_rows_used"] == want + want2 - reused
    assert np.array_equal(table.export_hot()[0], ot.export_hot()[0])
    assert st["status"] == 0
    table.close()


@pytest.mark.parametrize("dim", [64, 24, 256])
def test_demotion_by_idle_time_matches_checker(dim):
    """The hot set follows the access pattern both ways: hot rows no lookup has touched for `idle` steps become cold
    again.  The demoted key set, the remaining masters, the delivered rows (unchanged by a demotion, bit for bit), the
    store's bookkeeping and a further update of hot, demoted and cold rows must follow the checker."""
    from harness import RTOL_BF16
    lr, eps = 0.05, 1e-8
    table, ot = _mixed_pair(dim, hot_rows=600)
    rng = np.random.default_rng(100 + dim)
    pool = (np.arange(1, 2001, dtype=np.uint64) * np.uint64(0x9E3779B1)) & np.uint64((1 << 40) - 1)
    for step in range(3):
        _insert(table, ot, pool, step)
    _insert(table, ot, pool[:600], 3)                            # 600 keys reach four touches: exactly the store's size
    allk = np.sort(pool)
    row_idx = torch.empty(len(allk), dtype=torch.int32, device="cuda")
    table.find(dev_keys(allk), None, len(allk), row_idx)
    n_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    table.promote(row_idx, None, len(allk), 4, n_dev)
    assert int(n_dev.item()) == 600 and ot.promote(allk, 4) == 600
    hot_keys = table.export_hot()[0]
    assert np.array_equal(hot_keys, ot.export_hot()[0]) and np.array_equal(hot_keys, np.sort(pool[:600]))
    # a drifting working set: keys 300 .. 1499 of the pool stay in use, so half of the hot keys fall idle
    for step in range(4, 12):
        ks = np.unique(pool[rng.integers(300, 1500, size=900)])
        ri = _insert(table, ot, ks, step)
        g = normal_grads(9, step, len(ks), dim)
        table.apply_adagrad(ri, torch.from_numpy(g).cuda(), None, len(ks), lr, eps)
        ot.apply_adagrad(ks, g, lr, eps)
    out = torch.empty((len(allk), dim), dtype=torch.bfloat16, device="cuda")
    table.gather(row_idx, None, len(allk), out)
    before = out.clone()
    table.demote(12, 6, n_dev)
    want = ot.demote(12, 6)
    assert 0 < want < 600 and int(n_dev.item()) == want
    hk, hv = table.export_hot()
    ok, ov = ot.export_hot()
    assert np.array_equal(hk, ok)                                 # who stays hot is unique
    assert close_rows(hv, ov.astype(np.float64), lr, RTOL_F32)
    table.gather(row_idx, None, len(allk), out)
    assert torch.equal(out.view(torch.int16), before.view(torch.int16))   # a demotion changes no delivered bit
    st = table.stats()
    assert st["hot_rows_free"] == want and st["hot_rows_used"] == 600 and st["status"] == 0
    table.demote(12, 6, n_dev)
    assert int(n_dev.item()) == 0                                 # nothing is demoted twice
    # hot, demoted and never-hot rows take one more update each; the freed masters serve other keys
    ri = _insert(table, ot, allk, 12)
    g = normal_grads(9, 12, len(allk), dim)
    table.apply_adagrad(ri, torch.from_numpy(g).cuda(), None, len(allk), lr, eps)
    ot.apply_adagrad(allk, g, lr, eps)
    ek, ev, ea, el, ef = table.export()
    kk, kv, ka, kl, kf = ot.export()
    assert np.array_equal(ek, kk) and np.array_equal(el, kl) and np.array_equal(ef, kf)
    # A demoted row has been rounded to 16 bits twice since its master was last compared (once by the demotion, once by
    # this update), each time from values that agree with the checker's only to fp32 accuracy: two 16-bit roundings can
    # differ by two spacings, so these rows get twice the 16-bit tolerance; all other rows the usual one.
    was_demoted = np.isin(ek, np.setdiff1d(hot_keys, hk))
    assert was_demoted.sum() == want
    assert close_rows(ev[~was_demoted], kv[~was_demoted].astype(np.float64), lr, RTOL_BF16)
    assert close_rows(ev[was_demoted], kv[was_demoted].astype(np.float64), lr, 2 * RTOL_BF16)
    assert np.allclose(ea, ka, rtol=RTOL_F32, atol=1e-12)
    table.promote(ri, None, len(allk), 5, n_dev)
    assert int(n_dev.item()) == want                              # exactly the freed masters are handed out again
    st = table.stats()
    assert st["hot_rows_free"] == 0 and st["hot_rows_used"] == 600
    table.close()


def test_checkpoint_of_a_table_with_hot_rows_restores_its_masters():
    """Dump = the 16-bit view of every row (ht_export) plus the fp32 masters (ht_export_hot).  A table restored from both
    (ht_put, then ht_promote with min_freq 0 and ht_put_hot for the dumped masters) holds the dumped state bit for bit,
    agrees with the checker restored the same way, and keeps following the original through further updates."""
    from harness import RTOL_BF16
    dim, lr, eps = 64, 0.05, 1e-8
    table, ot = _mixed_pair(dim, hot_rows=400)
    rng = np.random.default_rng(77)
    pool = (np.arange(1, 1201, dtype=np.uint64) * np.uint64(0x9E3779B1)) & np.uint64((1 << 40) - 1)
    for step in range(3):
        _insert(table, ot, pool, step)
    ri = _insert(table, ot, pool[:300], 3)
    n_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    table.promote(ri, None, 300, 4, n_dev)
    assert int(n_dev.item()) == 300 and ot.promote(pool[:300], 4) == 300
    for step in range(4, 9):
        ks = np.unique(pool[rng.integers(0, 1200, size=700)])
        ri = _insert(table, ot, ks, step)
        g = normal_grads(21, step, len(ks), dim)
        table.apply_adagrad(ri, torch.from_numpy(g).cuda(), None, len(ks), lr, eps)
        ot.apply_adagrad(ks, g, lr, eps)
    dump = table.export_device()
    ref = table.export()
    hk, hv = table.export_hot()
    # ---- restore on both sides
    t2 = EmbeddingTable(dim, B.BF16, capacity_log2=13, chunk_rows_log2=10, hot_rows=400)
    t2.import_rows(*dump)
    assert t2.import_hot(dev_keys(hk), torch.from_numpy(hv).cuda()) == len(hk)
    o2 = oracle.Table(dim, oracle.BF16)
    ok_, ov_, oa_, ol_, of_ = ot.export()
    o2.find_or_insert(ok_, 0)
    assert o2.put(ok_, ov_, oa_, ol_, of_) == len(ok_)
    o2.set_hot(400)
    ohk, ohv = ot.export_hot()
    assert o2.promote(ohk, 0) == len(ohk) and o2.put_hot(ohk, ohv) == len(ohk)
    for a, b in zip(ref, t2.export()):
        assert np.array_equal(a, b)                                     # rows as delivered, accumulators, counters
    hk2, hv2 = t2.export_hot()
    assert np.array_equal(hk2, hk) and np.array_equal(hv2, hv)          # masters bit for bit
    assert np.array_equal(hk2, o2.export_hot()[0])
    st = t2.stats()
    assert st["hot_rows_used"] == len(hk) and st["status"] == 0
    # ---- original and restored table take the same further updates
    for step in range(9, 12):
        ks = np.unique(pool[rng.integers(0, 1200, size=700)])
        g = torch.from_numpy(normal_grads(21, step, len(ks), dim)).cuda()
        for t in (table, t2):
            r = torch.empty(len(ks), dtype=torch.int32, device="cuda")
            t.find_or_insert(dev_keys(ks), None, len(ks), step, r)
            t.apply_adagrad(r, g, None, len(ks), lr, eps)
        for o in (ot, o2):
            o.find_or_insert(ks, step)
            o.apply_adagrad(ks, g.cpu().numpy(), lr, eps)
    for a, b in zip(table.export(), t2.export()):
        assert np.array_equal(a, b)
    assert np.array_equal(table.export_hot()[1], t2.export_hot()[1])
    assert close_rows(t2.export_hot()[1], o2.export_hot()[1].astype(np.float64), lr, RTOL_F32)
    assert close_rows(t2.export()[1], o2.export()[1].astype(np.float64), lr, RTOL_BF16)
    table.close()
    t2.close()


def test_hot_store_full_keeps_the_rest_cold():
    dim = 32
    table, ot = _mixed_pair(dim, hot_rows=5)
    ks = np.arange(1, 41, dtype=np.uint64) * np.uint64(1000003)
    for step in range(3):
        ri = _insert(table, ot, ks, step)
    n_prom = torch.zeros(1, dtype=torch.int64, device="cuda")
    table.promote(ri, None, len(ks), 3, n_prom)
    assert int(n_prom.item()) == 5 == ot.promote(ks, 3)                # which five is not specified
    hk, hv = table.export_hot()
    assert len(hk) == 5 and np.all(np.isin(hk, ks))
    st = table.stats()
    assert st["hot_rows_used"] == 5 and st["hot_rows_free"] == 0
    # every row still updates: the hot ones in fp32, the others in 16-bit
    g = normal_grads(4, 0, len(ks), dim)
    w0 = torch.empty((len(ks), dim), dtype=torch.bfloat16, device="cuda")
    table.gather(ri, None, len(ks), w0)
    table.apply_adagrad(ri, torch.from_numpy(g).cuda(), None, len(ks), 0.05, 1e-8)
    w1 = torch.empty_like(w0)
    table.gather(ri, None, len(ks), w1)
    ss = (g.astype(np.float64) ** 2).mean(axis=1)
    want = _bf16_rows(w0).astype(np.float64) - 0.05 * g / (np.sqrt(ss) + 1e-8)[:, None]
    from harness import RTOL_BF16
    assert close_rows(_bf16_rows(w1), want, 0.05, RTOL_BF16)
    hk1, hv1 = table.export_hot()
    sel = np.searchsorted(ks, hk1)
    assert close_rows(hv1, want[sel], 0.05, RTOL_F32)
    table.close()


def test_hot_rows_keep_small_updates_on_device():
    """The property the hot store exists for: a stream of updates, each below half a 16-bit spacing, moves a hot
    row by their sum and leaves a cold row where it was."""
    dim, T, lr = 64, 400, 1e-4
    table = EmbeddingTable(dim, B.BF16, capacity_log2=10, chunk_rows_log2=6, init_scale=1.0, hot_rows=4)
    ks = np.array([21, 22], dtype=np.uint64)
    ri = torch.empty(2, dtype=torch.int32, device="cuda")
    table.find_or_insert(dev_keys(ks), None, 2, 0, ri)
    table.find_or_insert(dev_keys(ks[:1]), None, 1, 1, ri[:1].clone())
    table.promote(ri, None, 2, 2)
    w0 = torch.empty((2, dim), dtype=torch.bfloat16, device="cuda")
    table.gather(ri, None, 2, w0)
    g = torch.ones((2, dim), dtype=torch.float32, device="cuda")
    for _ in range(T):
        table.apply_adagrad(ri, g, None, 2, lr, 0.0)
    w1 = torch.empty_like(w0)
    table.gather(ri, None, 2, w1)
    a, b = _bf16_rows(w0).astype(np.float64), _bf16_rows(w1).astype(np.float64)
    shift = lr * np.sum(1.0 / np.sqrt(np.arange(1, T + 1, dtype=np.float64)))      # acc after s steps is s
    big = np.abs(a) > 0.25
    assert np.array_equal(b[1][big[1]], a[1][big[1]])                               # cold: unchanged
    _, hv = table.export_hot()
    assert np.allclose(hv[0], a[0] - shift, rtol=0, atol=T * 2.0 ** -24)            # hot: the full sum arrived
    assert np.all(np.abs(b[0] - (a[0] - shift)) <= 2.0 ** -8)
    table.close()


def test_hot_store_argument_checks():
    t32 = EmbeddingTable(32, B.F32, capacity_log2=10, chunk_rows_log2=6)
    hv = torch.empty((4, 32), dtype=torch.float32, device="cuda")
    hf = torch.empty(4, dtype=torch.int32, device="cuda")
    with pytest.raises(B.EmbError):
        B.ht_set_hot_storage(t32.h, hv, hf, 4)                     # fp32 tables have no 16-bit form
    ri = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.EmbError):
        B.ht_promote(t32.h, ri, None, 1, 1)                        # no hot store
    tb = EmbeddingTable(32, B.BF16, capacity_log2=10, chunk_rows_log2=6, hot_rows=4, adam_state=True)
    with pytest.raises(B.EmbError):
        B.ht_set_hot_storage(tb.h, hv, hf, 4)                      # only once
    t32.close()
    tb.close()


def test_sparse_adam_moves_the_masters_of_hot_rows():
    """Adam on a 16-bit table with hot rows: a hot row's master takes the update in fp32, a cold row rounds as before.
    Masters to fp32 accuracy against the checker, delivered rows to 16-bit accuracy; moments identical for both kinds."""
    from harness import RTOL_BF16
    dim, lr = 64, 1e-3
    table = EmbeddingTable(dim, B.BF16, capacity_log2=13, chunk_rows_log2=10, adam_state=True, initial_chunks=2, hot_rows=500)
    ot = oracle.Table(dim, oracle.BF16)
    ot.set_hot(500)
    rng = np.random.default_rng(31)
    pool = (np.arange(1, 1501, dtype=np.uint64) * np.uint64(0x9E3779B1)) & np.uint64((1 << 40) - 1)
    for step in range(3):
        _insert(table, ot, pool, step)
    ri = _insert(table, ot, pool[:400], 3)
    n_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    table.promote(ri, None, 400, 4, n_dev)
    assert int(n_dev.item()) == 400 and ot.promote(pool[:400], 4) == 400
    for step in range(1, 7):
        ks = np.unique(pool[rng.integers(0, 1500, size=800)])
        r = _insert(table, ot, ks, 3 + step)
        g = normal_grads(17, step, len(ks), dim)
        table.apply_adam(r, torch.from_numpy(g).cuda(), None, len(ks), lr, step)
        ot.apply_adam(ks, g, lr, step)
    hk, hv = table.export_hot()
    ok, ov = ot.export_hot()
    assert np.array_equal(hk, ok) and len(hk) == 400
    assert close_rows(hv, ov.astype(np.float64), lr, RTOL_F32)                 # masters: fp32 accuracy
    moved = np.abs(hv - np.float32(torch.from_numpy(hv).to(torch.bfloat16).float().numpy())) > 0
    assert moved.mean() > 0.5                                                  # masters really hold more than 16 bits
    gk, gv, _, _, gf = table.export()
    kk, kv, _, _, kf = ot.export()
    assert np.array_equal(gk, kk) and np.array_equal(gf, kf)
    assert close_rows(gv, kv.astype(np.float64), lr, RTOL_BF16)
    assert table.stats()["status"] == 0
    table.close()


# --------------------------------------------------------------------------- one record update per step
@pytest.mark.parametrize("dtype,hot", [(0, 0), (1, 0), (1, 1500)])
def test_notouch_lookup_plus_touching_update_equals_the_plain_pair(dtype, hot):
    """ht_find_or_insert_notouch + ht_apply_adagrad_touch must leave the table exactly where ht_find_or_insert +
    ht_apply_adagrad leave it (bit for bit: same kernels' arithmetic), and keys without an update keep their record."""
    dim, lr, eps = 64, 0.05, 1e-8
    ta = EmbeddingTable(dim, dtype, capacity_log2=13, chunk_rows_log2=10, hot_rows=hot)
    tb = EmbeddingTable(dim, dtype, capacity_log2=13, chunk_rows_log2=10, hot_rows=hot)
    rng = np.random.default_rng(11)
    pool = np.arange(1, 1501, dtype=np.uint64) * np.uint64(48271)
    for step in range(1, 9):
        ks = np.unique(pool[rng.integers(0, 1500, size=600)])
        n = len(ks)
        dk = dev_keys(ks)
        g = torch.from_numpy(normal_grads(9, step, n, dim)).cuda()
        ra = torch.empty(n, dtype=torch.int32, device="cuda")
        rb = torch.empty(n, dtype=torch.int32, device="cuda")
        ia = torch.empty(n, dtype=torch.uint8, device="cuda")
        ib = torch.empty(n, dtype=torch.uint8, device="cuda")
        ta.find_or_insert(dk, None, n, step, ra, ia)
        ta.apply_adagrad(ra, g, None, n, lr, eps)
        tb.find_or_insert(dk, None, n, step, rb, ib, touch=False)
        assert torch.equal(ia, ib)
        tb.apply_adagrad(rb, g, None, n, lr, eps, touch_step=step)
        if hot and step == 4:
            ta.promote(ra, None, n, 2)
            tb.promote(rb, None, n, 2)
        for a, b in zip(ta.export(), tb.export()):
            assert np.array_equal(a, b)
    if hot:
        for a, b in zip(ta.export_hot(), tb.export_hot()):
            assert np.array_equal(a, b)
        assert ta.stats()["hot_rows_used"] > 0
    # a key that is looked up without an update keeps its record
    k = dev_keys(pool[:5])
    r = torch.empty(5, dtype=torch.int32, device="cuda")
    before = tb.export()
    tb.find_or_insert(k, None, 5, 99, r, None, touch=False)
    for a, b in zip(before, tb.export()):
        assert np.array_equal(a, b)
    # a key created by the quiet lookup starts with touch count 0 and the step as last_seen
    newk = np.array([0x7FFF0001], dtype=np.uint64)
    r1 = torch.empty(1, dtype=torch.int32, device="cuda")
    tb.find_or_insert(dev_keys(newk), None, 1, 123, r1, None, touch=False)
    ek, _, ea, el, ef = tb.export()
    i = int(np.searchsorted(ek, newk[0]))
    assert ek[i] == newk[0] and ef[i] == 0 and el[i] == 123 and ea[i] == 0
    ta.close()
    tb.close()


def test_notouch_lookup_with_duplicate_new_keys_resolves_every_element():
    """Duplicates of a key that is being created in the same call meet an unpublished row and are resolved by the
    follow-up kernel; in the quiet form that kernel must still hand out the row, only without counting."""
    dim = 32
    t = EmbeddingTable(dim, 0, capacity_log2=12, chunk_rows_log2=10)
    rng = np.random.default_rng(3)
    distinct = np.arange(1, 301, dtype=np.uint64) * np.uint64(7919)
    ks = distinct[rng.integers(0, 300, size=20000)]                 # ~67 copies of each key, all new
    r = torch.empty(len(ks), dtype=torch.int32, device="cuda")
    t.find_or_insert(dev_keys(ks), None, len(ks), 5, r, None, touch=False)
    rows = r.cpu().numpy()
    assert (rows >= 0).all()
    first = {}
    for k, row in zip(ks.tolist(), rows.tolist()):
        assert first.setdefault(k, row) == row                       # one row per key
    assert len(set(first.values())) == len(first) == len(np.unique(ks))
    ek, _, _, el, ef = t.export()
    assert np.array_equal(ek, np.unique(ks)) and (ef == 0).all() and (el == 5).all()
    assert t.stats()["status"] == 0
    t.close()


# --------------------------------------------------------------------------- fused backward
@pytest.mark.parametrize("dim,dtype", [(64, 0), (128, 1), (32, 0), (16, 0), (256, 0), (24, 0), (4, 0), (40, 1), (8, 1)])
@pytest.mark.parametrize("touch", [False, True])
def test_fused_backward_equals_reduce_then_adagrad(dim, dtype, touch):
    """grad_reduce_apply_adagrad against the checker (fp64 segment sums in input order, then the row-wise Adagrad
    update; updated rows and accumulators within the bounds of R16, touch records exact), and bit-identical to
    grad_segment_reduce + ht_apply_adagrad(_touch): same summation tree, same update arithmetic; long segments
    (several levels), single rows and skipped rows included."""
    from paper_2505_12663_amd import backward, backward_fused
    lr, eps = 0.05, 1e-8
    ta = EmbeddingTable(dim, dtype, capacity_log2=14, chunk_rows_log2=11)
    tb = EmbeddingTable(dim, dtype, capacity_log2=14, chunk_rows_log2=11)
    ot = oracle.Table(dim, dtype)
    rtol = RTOL_F32 if dtype == 0 else RTOL_BF16
    rng = np.random.default_rng(dim + 7 * dtype)
    vocab = np.arange(1, 4001, dtype=np.uint64) * np.uint64(2654435761)
    n = 64 * 64 * 3 + 77
    bufa, bufb = StepBuffers(n, dim, dtype), StepBuffers(n, dim, dtype)
    for step in range(1, 5):
        wts = 1.0 / np.arange(1, 4001) ** 1.2
        ks = vocab[rng.choice(4000, size=n, p=wts / wts.sum())]
        ks[: n // 3] = vocab[0]                                     # one segment of thousands of positions
        dk = dev_keys(ks)
        G = torch.from_numpy(normal_grads(5, step, n, dim)).cuda()
        if dtype == 1:
            G = G.to(torch.bfloat16)
        for t, buf in ((ta, bufa), (tb, bufb)):
            B.emb_dedup(dk, n, buf.uniq, buf.inverse, buf.counts, buf.perm, buf.seg_off, buf.seg_of, buf.n_unique, buf.dedup_ws)
            t.find_or_insert(buf.uniq, buf.n_unique, n, step, buf.row_idx, buf.inserted, touch=not touch)
        U = int(bufa.n_unique.item())
        if step == 3:                                               # a segment without a row is skipped by both forms
            bufa.row_idx[5] = -1
            bufb.row_idx[5] = -1
        backward(ta, bufa, G, n, lr, eps, touch_step=step if touch else None)
        backward_fused(tb, bufb, G, n, lr, eps, touch_step=step if touch else None)
        for a, b in zip(ta.export(), tb.export()):
            assert np.array_equal(a, b)
        # the checker's step: every distinct key is touched once, every segment but the skipped one is updated
        ouniq, oinv, _ = oracle.dedup(ks)
        assert U == len(ouniq)
        ot.find_or_insert(ouniq, step)
        og = oracle.segment_reduce(G.float().cpu().numpy(), oinv, U)
        upd = np.ones(U, dtype=bool)
        if step == 3:
            upd[5] = False
            skipped_key = ouniq[5]     # its record depends on which call counts the touch: left out from here on
        ot.apply_adagrad(ouniq[upd], og[upd], lr, eps)
        gk, gv, ga, gl, gf = tb.export()
        ok, ov, oa, ol, of = ot.export()
        assert np.array_equal(gk, ok)
        m = np.ones(len(gk), dtype=bool) if step < 3 else gk != skipped_key
        assert np.array_equal(gl[m], ol[m]) and np.array_equal(gf[m], of[m])
        assert close_rows(gv[m], ov[m].astype(np.float64), lr, rtol), float(np.abs(gv[m] - ov[m]).max())
        assert np.allclose(ga[m], oa[m], rtol=1e-5, atol=1e-12), float(np.abs(ga[m] - oa[m]).max())
    assert ta.stats()["status"] == 0 and tb.stats()["status"] == 0
    # hot-store tables take the two-call form
    if dtype == 1:
        th = EmbeddingTable(dim, dtype, capacity_log2=10, chunk_rows_log2=6, hot_rows=4)
        with pytest.raises(B.EmbError):
            backward_fused(th, bufb, G, n, lr, eps)
        th.close()
    ta.close()
    tb.close()
