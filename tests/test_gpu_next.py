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
    from harness import dev_keys, host_keys, close_reduce, close_rows, RTOL_F32


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
    assert close_rows(gv, ov.astype(np.float64), 0.01, RTOL_F32) and np.allclose(ga, oa, rtol=4e-5)
    table.close()


@pytest.mark.parametrize("dim,dtype,mean", [(64, 0, False), (64, 0, True), (32, 0, True), (128, 1, False), (128, 1, True), (16, 0, False)])
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


@pytest.mark.parametrize("dim,dtype", [(64, 0), (32, 0), (128, 1), (16, 0)])
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
