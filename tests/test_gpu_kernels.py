"""Element-by-element parity of every HIP entry point against the CPU checker (needs an MI355X).

Sizes span several tiles and ragged tails; edge cases cover empty inputs, one element, all-equal
and all-distinct keys, duplicate keys in one insert call, one giant segment, absent keys.
Integer / index / byte results are compared bit-exactly; fp32 results within 1e-5 (relative to the
sum of |addends| for reductions, to max(|w|, lr) for updated rows); bf16 rows within 1e-2.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import bounded_zipf_ranks, scramble_bits, normal_grads, small_int_grads

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2505_12663_amd import binding as B
    from paper_2505_12663_amd import EmbeddingTable, StepBuffers
    from harness import dev_keys, host_keys, close_reduce, close_rows, RTOL_F32, RTOL_BF16


def _zipf_keys(n, vocab, seed, bits=40, tag=0, tag_shift=59):
    rng = np.random.default_rng(seed)
    r = bounded_zipf_ranks(rng, n, vocab, 1.05)
    return (scramble_bits(r.astype(np.uint64), bits, seed) | np.uint64(tag << tag_shift)).astype(np.uint64)


# ------------------------------------------------------------------------------------------ tag
@pytest.mark.parametrize("tag_bits,n_fields,n", [(2, 3, 1000), (8, 40, 50_000), (0, 1, 77), (4, 5, 0), (16, 7, 4097)])
def test_tag_keys(tag_bits, n_fields, n):
    rng = np.random.default_rng(n + tag_bits)
    cuts = np.sort(rng.integers(0, n + 1, size=n_fields - 1)) if n_fields > 1 else np.zeros(0, dtype=np.int64)
    off = np.concatenate([[0], cuts, [n]]).astype(np.int64)          # some fields may be empty
    tags = rng.integers(0, min(1 << tag_bits, 256), size=n_fields).astype(np.uint8)
    x = rng.integers(0, 1 << (63 - tag_bits), size=n, dtype=np.uint64)
    if n > 10:
        x[3] = np.uint64(1 << (63 - tag_bits)) if tag_bits > 0 else x[3]     # one ID out of range
    okey, oerr = oracle.tag_keys(x, off, tags, tag_bits)
    key = torch.empty(max(n, 1), dtype=torch.int64, device="cuda")
    err = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    B.emb_tag_keys(dev_keys(x), torch.from_numpy(off).cuda(), torch.from_numpy(tags).cuda(), tag_bits, key, err)
    assert int(err.item()) == oerr
    assert np.array_equal(host_keys(key[:n]), okey)


# ------------------------------------------------------------------------------------------ dedup
def _run_dedup(keys):
    n = len(keys)
    d = dev_keys(keys) if n else torch.empty(0, dtype=torch.int64, device="cuda")
    m = max(n, 1)
    uniq = torch.empty(m, dtype=torch.int64, device="cuda")
    inverse = torch.empty(m, dtype=torch.int32, device="cuda")
    counts = torch.empty(m, dtype=torch.int32, device="cuda")
    perm = torch.empty(m, dtype=torch.int32, device="cuda")
    seg_off = torch.full((m + 1,), -7, dtype=torch.int32, device="cuda")
    seg_of = torch.full((m,), -7, dtype=torch.int32, device="cuda")
    n_unique = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.emb_dedup_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    B.emb_dedup(d, n, uniq, inverse, counts, perm, seg_off, seg_of, n_unique, ws)
    U = int(n_unique.item())
    sof = seg_of[:n].cpu().numpy()
    pm = perm[:n].cpu().numpy()
    inv = inverse[:n].cpu().numpy()
    assert np.array_equal(sof, inv[pm])          # seg_of[j] = inverse[perm[j]] by definition
    return (host_keys(uniq[:U]), inv, counts[:U].cpu().numpy(), pm, seg_off[:U + 1].cpu().numpy())


@pytest.mark.parametrize("case", ["empty", "one", "all_equal", "all_distinct", "zipf_small", "zipf_tiles",
                                  "tagged_mix", "full_64bit_range", "two_values_far_apart"])
def test_dedup_matches_checker(case):
    rng = np.random.default_rng(11)
    keys = {
        "empty": np.zeros(0, dtype=np.uint64),
        "one": np.array([42], dtype=np.uint64),
        "all_equal": np.full(5000, (3 << 59) | 12345, dtype=np.uint64),
        "all_distinct": rng.permutation(np.arange(10_001, dtype=np.uint64) * np.uint64(2654435761)),
        "zipf_small": _zipf_keys(777, 300, 1),
        "zipf_tiles": _zipf_keys(4096 * 13 + 57, 50_000, 2),
        "tagged_mix": np.concatenate([_zipf_keys(30_000, 4000, 3, tag=t) for t in (0, 1, 5, 7)]),
        "full_64bit_range": rng.integers(0, 1 << 63, size=20_000, dtype=np.uint64),
        "two_values_far_apart": rng.choice(np.array([5, (1 << 62) + 5], dtype=np.uint64), size=9000),
    }[case]
    if case == "tagged_mix":
        keys = keys[rng.permutation(len(keys))]
    uniq, inverse, counts, perm, seg_off = _run_dedup(keys)
    ou, oi, oc = oracle.dedup(keys)
    assert np.array_equal(uniq, ou) and np.array_equal(inverse, oi) and np.array_equal(counts, oc)
    n, U = len(keys), len(ou)
    # perm / seg_off: the part that is unique is checked exactly (stable order = ascending position)
    assert seg_off[0] == 0 and seg_off[-1] == n if n else seg_off[0] == 0
    if n:
        assert np.array_equal(np.diff(seg_off), oc)
        assert np.array_equal(np.sort(perm), np.arange(n))
        assert np.array_equal(keys[perm], np.repeat(ou, oc))
        seg_of_pos = np.repeat(np.arange(U), oc)
        same = seg_of_pos[1:] == seg_of_pos[:-1]
        assert (np.diff(perm)[same] > 0).all()


# ------------------------------------------------------------------------------------------ tag + dedup in one call
@pytest.mark.parametrize("case", ["config2_like", "one_field", "empty", "one", "shared_and_unordered_tags", "empty_fields",
                                  "id_bits_exceeded", "all_equal", "all_distinct", "narrow_ids_wide_tags", "many_fields",
                                  "two_call_form"])
def test_tag_dedup_matches_tag_then_dedup(case):
    """emb_tag_dedup against the checker's tag (Eq. 8) followed by its sort-based dedup: tagged keys, error count,
    distinct keys, inverse, counts bit-exact; perm / seg_off / seg_of by what is unique about them."""
    rng = np.random.default_rng(5)
    tag_bits, id_bits = 4, 40
    if case == "config2_like":          # 8 fields, one identifier each, several tiles and a ragged tail
        lens, tags = [4096 * 3 + 11] * 8, list(range(8))
        xs = [_zipf_keys(l, 20_000, 10 + f) for f, l in enumerate(lens)]
    elif case == "one_field":
        lens, tags, tag_bits = [70_001], [0], 0
        xs = [_zipf_keys(lens[0], 9000, 3)]
    elif case == "empty":
        lens, tags, xs = [0, 0], [1, 2], [np.zeros(0, np.uint64)] * 2
    elif case == "one":
        lens, tags, xs = [0, 1], [3, 2], [np.zeros(0, np.uint64), np.array([77], np.uint64)]
    elif case == "shared_and_unordered_tags":   # two fields feed identifier 5; identifiers not in field order
        lens, tags = [5000, 3000, 7000, 100, 6000], [5, 2, 9, 5, 0]
        xs = [_zipf_keys(l, 800, 20 + f) for f, l in enumerate(lens)]       # the same IDs under several identifiers
        xs[3] = xs[0][:100].copy()
    elif case == "empty_fields":
        lens, tags = [0, 4097, 0, 0, 5], [1, 2, 3, 4, 15]
        xs = [_zipf_keys(l, 500, 30 + f) if l else np.zeros(0, np.uint64) for f, l in enumerate(lens)]
    elif case == "id_bits_exceeded":    # IDs beyond the declared width are counted and wrapped
        lens, tags, id_bits = [9000, 9000], [0, 1], 12
        xs = [rng.integers(0, 1 << 14, size=l, dtype=np.uint64) for l in lens]
    elif case == "all_equal":
        lens, tags = [6000, 6000], [1, 1]
        xs = [np.full(l, 123456789, np.uint64) for l in lens]
    elif case == "all_distinct":
        lens, tags = [10_001], [7]
        xs = [rng.permutation(np.arange(10_001, dtype=np.uint64) * np.uint64(48271)) & np.uint64((1 << 40) - 1)]
    elif case == "narrow_ids_wide_tags":      # the identifier spans more than one radix pass
        lens, tags, tag_bits, id_bits = [3000] * 6, [0, 255, 4097, 65535, 300, 255], 16, 5
        xs = [rng.integers(0, 32, size=l, dtype=np.uint64) for l in lens]
    elif case == "many_fields":
        nf = 700
        lens, tags, tag_bits = list(rng.integers(0, 60, size=nf)), list(rng.integers(0, 200, size=nf)), 8
        xs = [rng.integers(0, 50, size=int(l), dtype=np.uint64) for l in lens]
    else:                                # records of ID and position do not fit 64 bits: tag, then dedup, inside the call
        lens, tags, id_bits = [20_000, 20_000], [0, 3], 59
        xs = [rng.integers(0, 1 << 59, size=l, dtype=np.uint64) for l in lens]
        xs[1][:5000] = xs[0][:5000]
    if case == "narrow_ids_wide_tags":
        tags = [t & 0xFF for t in tags]  # identifiers are bytes at this boundary
    _check_tag_dedup(xs, lens, tags, tag_bits, id_bits)


@pytest.mark.parametrize("seed", range(24))
def test_tag_dedup_random_shapes(seed):
    """Random field counts, lengths (empty fields included), identifier assignments, widths and duplicate rates;
    sizes from one record to a dozen tiles, with and without the packed records fitting 64 bits."""
    rng = np.random.default_rng(1000 + seed)
    nf = int(rng.integers(1, 41))
    tag_bits = int(rng.integers(0, 9)) if nf > 1 or seed % 2 else 0
    id_bits = int(rng.choice([3, 9, 17, 18, 27, 36, 40, 45, 50, 55]))
    id_bits = min(id_bits, 63 - tag_bits)
    scale = int(rng.choice([1, 40, 700, 4096, 13_000]))
    lens = [int(l) for l in rng.integers(0, scale + 1, size=nf)]
    if sum(lens) == 0:
        lens[int(rng.integers(0, nf))] = 1
    tags = [int(t) for t in rng.integers(0, 1 << tag_bits, size=nf)]
    vocab = int(rng.choice([1, 7, 300, 50_000, 1 << 40]))
    xs = []
    for l in lens:
        v = rng.integers(0, min(vocab, 1 << id_bits), size=l, dtype=np.uint64)
        if seed % 3 == 0 and l:            # spread the values over the whole declared width
            v = (v * np.uint64(0x9E3779B97F4A7C15)) & np.uint64((1 << id_bits) - 1)
        xs.append(v)
    if seed % 5 == 0:                      # some IDs beyond the declared width: counted and wrapped
        for v in xs:
            if len(v):
                v[:: 7] |= np.uint64(1 << id_bits) if id_bits < 62 - tag_bits else np.uint64(0)
    _check_tag_dedup(xs, lens, tags, tag_bits, id_bits)


def _check_tag_dedup(xs, lens, tags, tag_bits, id_bits):
    x = np.concatenate(xs) if sum(lens) else np.zeros(0, np.uint64)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    tg = np.array(tags, dtype=np.uint8)
    n = len(x)
    wrapped = x & np.uint64((1 << id_bits) - 1)
    okey, oerr = oracle.tag_keys(wrapped, off, tg, tag_bits)
    oerr += int((x != wrapped).sum())
    ou, oi, oc = oracle.dedup(okey)
    U = len(ou)
    m = max(n, 1)
    key = torch.full((m,), -1, dtype=torch.int64, device="cuda")
    uniq = torch.full((m,), -1, dtype=torch.int64, device="cuda")
    inverse, counts, perm, seg_of = (torch.full((m,), -7, dtype=torch.int32, device="cuda") for _ in range(4))
    seg_off = torch.full((m + 1,), -7, dtype=torch.int32, device="cuda")
    n_unique = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    err = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.emb_tag_dedup_workspace_bytes(n, len(tags), tag_bits, id_bits), dtype=torch.uint8, device="cuda")
    dx = dev_keys(x) if n else torch.empty(0, dtype=torch.int64, device="cuda")
    B.emb_tag_dedup(dx, torch.from_numpy(off).cuda(), torch.from_numpy(tg).cuda(), tag_bits, id_bits, key, uniq, inverse,
                    counts, perm, seg_off, seg_of, n_unique, err, ws)
    assert int(n_unique.item()) == U and int(err.item()) == oerr
    assert np.array_equal(host_keys(key[:n]), okey), "tagged keys"
    assert np.array_equal(host_keys(uniq[:U]), ou) and np.array_equal(inverse[:n].cpu().numpy(), oi)
    assert np.array_equal(counts[:U].cpu().numpy(), oc)
    so, pm, sf = seg_off[:U + 1].cpu().numpy(), perm[:n].cpu().numpy(), seg_of[:n].cpu().numpy()
    assert so[0] == 0
    if n:
        assert so[-1] == n and np.array_equal(np.diff(so), oc)
        assert np.array_equal(pm, np.argsort(okey, kind="stable"))       # positions by (key, position)
        assert np.array_equal(sf, oi[pm])
    # without the optional outputs
    uniq2 = torch.full((m,), -1, dtype=torch.int64, device="cuda")
    B.emb_tag_dedup(dx, torch.from_numpy(off).cuda(), torch.from_numpy(tg).cuda(), tag_bits, id_bits, None, uniq2, None,
                    None, perm, None, seg_of, n_unique, err, ws)
    assert int(n_unique.item()) == U and torch.equal(uniq2[:U], uniq[:U])
    if n:
        assert np.array_equal(perm[:n].cpu().numpy(), pm) and np.array_equal(seg_of[:n].cpu().numpy(), sf)


# ------------------------------------------------------------------------------------------ table
@pytest.mark.parametrize("dim,dtype", [(32, 0), (64, 0), (16, 0), (128, 0), (128, 1), (8, 1), (256, 0), (4, 0), (24, 0), (256, 1), (40, 1)])
def test_find_or_insert_gather_roundtrip(dim, dtype):
    keys = _zipf_keys(20_000, 6000, 5)                         # with duplicates inside one call
    keys[:64] = keys[0]                                          # a whole wave of the same new key
    t = EmbeddingTable(dim, dtype, capacity_log2=15, chunk_rows_log2=12, count_probes=True, initial_chunks=3)
    ot = oracle.Table(dim, dtype)
    n = len(keys)
    d = dev_keys(keys)
    row_idx = torch.empty(n, dtype=torch.int32, device="cuda")
    inserted = torch.empty(n, dtype=torch.uint8, device="cuda")
    t.find_or_insert(d, None, n, 7, row_idx, inserted)
    oins = ot.find_or_insert(keys, 7)
    r = row_idx.cpu().numpy()
    assert (r >= 0).all()
    # one row per distinct key, the same row for every duplicate
    uk, first = np.unique(keys, return_index=True)
    assert len(np.unique(r)) == len(uk)
    assert np.array_equal(r, r[first][np.searchsorted(uk, keys)])
    # exactly one element per new key reports the insert (which duplicate wins is free)
    ins = inserted.cpu().numpy()
    assert ins.sum() == oins.sum() == len(uk)
    assert np.array_equal(np.sort(keys[ins == 1]), uk)
    st = t.stats()
    assert st["live"] == len(uk) == len(ot) and st["status"] == 0 and st["tombstones"] == 0
    assert st["rows_used"] == len(uk)
    assert st["lookups"] == n and st["probes"] >= n and st["cas_attempts"] >= len(uk)
    # gather = the checker's lookup, bit for bit (initial rows are a pure function of the key)
    tdt = torch.float32 if dtype == 0 else torch.bfloat16
    out = torch.empty((n, dim), dtype=tdt, device="cuda")
    t.gather(row_idx, None, n, out)
    assert np.array_equal(out.float().cpu().numpy(), ot.lookup(keys))
    # second call inserts nothing and returns the same rows; touch counters agree with the checker
    row2 = torch.empty_like(row_idx)
    t.find_or_insert(d, None, n, 8, row2, inserted)
    ot.find_or_insert(keys, 8)
    assert np.array_equal(row2.cpu().numpy(), r) and int(inserted.sum().item()) == 0
    assert t.stats()["live"] == len(uk)
    gk, gv, ga, gl, gf = t.export()
    ok, ov, oa, ol, of = ot.export()
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov) and np.array_equal(gl, ol) and np.array_equal(gf, of)
    assert (ga == 0).all()
    # read-only find: present keys -> same rows, absent keys -> -1, gather of -1 -> zeros
    probe = np.concatenate([uk[:100], uk[:50] ^ np.uint64(1 << 50)])
    found = torch.empty(len(probe), dtype=torch.int32, device="cuda")
    t.find(dev_keys(probe), None, len(probe), found)
    f = found.cpu().numpy()
    assert np.array_equal(f >= 0, ot.find(probe).astype(bool))
    assert np.array_equal(f[:100], r[first][:100])
    out2 = torch.full((len(probe), dim), 3.0, dtype=tdt, device="cuda")
    t.gather(found, None, len(probe), out2)
    assert np.array_equal(out2.float().cpu().numpy(), ot.lookup(probe))
    t.close()


def test_count_on_device_limits_the_work():
    keys = np.arange(1, 1001, dtype=np.uint64) * np.uint64(7919)
    t = EmbeddingTable(32, 0, capacity_log2=12, chunk_rows_log2=10)
    row_idx = torch.full((1000,), -5, dtype=torch.int32, device="cuda")
    n_dev = torch.tensor([300], dtype=torch.int64, device="cuda")
    t.find_or_insert(dev_keys(keys), n_dev, 1000, 0, row_idx)
    assert t.stats()["live"] == 300
    assert (row_idx[:300] >= 0).all() and (row_idx[300:] == -5).all()
    out = torch.full((1000, 32), 9.0, device="cuda")
    t.gather(row_idx, n_dev, 1000, out)
    assert (out[300:] == 9.0).all() and (out[:300].abs() <= 0.01).all()
    t.close()


def test_bad_key_and_capacity_errors_are_reported():
    t = EmbeddingTable(32, 0, capacity_log2=8, chunk_rows_log2=6, initial_chunks=1)      # 256 slots, 64 rows
    keys = np.array([5, (1 << 63) | 5, 6], dtype=np.uint64)
    row_idx = torch.empty(3, dtype=torch.int32, device="cuda")
    t.find_or_insert(dev_keys(keys), None, 3, 0, row_idx)
    r = row_idx.cpu().numpy()
    assert r[0] >= 0 and r[2] >= 0 and r[1] == -1
    assert t.stats()["status"] & B.DEV_BAD_KEY
    t.close()


def _export_maps(t):
    gk, gv, ga, gl, gf = t.export()
    return gk, gv, gl, gf


def test_load_factor_limit_is_enforced_on_the_device_and_the_call_can_be_reissued():
    """Sec. 3.1 "Capacity Expansion": new keys are admitted up to floor(0.75 * capacity) live + deleted slots, the
    rest are turned away (row -1, counted, status bit) with nothing of them left; after a rehash the second
    attempt places exactly those, and every key has been touched once."""
    t = EmbeddingTable(32, 0, capacity_log2=8, chunk_rows_log2=9, initial_chunks=1)      # 256 slots -> limit 192; 512 rows
    ot = oracle.Table(32, 0)
    first = np.arange(1, 151, dtype=np.uint64) * np.uint64(104729)
    r1 = torch.empty(150, dtype=torch.int32, device="cuda")
    assert B.ht_find_or_insert(t.h, dev_keys(first), None, 150, 3, r1) == B.EMB_OK          # 150 <= 192: proven to fit
    ot.find_or_insert(first, 3)
    more = np.concatenate([first[:20], np.arange(1, 101, dtype=np.uint64) * np.uint64(15485863)])   # 20 old + 100 new
    r2 = torch.full((120,), -9, dtype=torch.int32, device="cuda")
    ins = torch.full((120,), 9, dtype=torch.uint8, device="cuda")
    assert B.ht_find_or_insert(t.h, dev_keys(more), None, 120, 4, r2, ins) == B.EMB_CHECK_STATUS
    st = t.stats()
    assert st["live"] == 192 and st["refused"] == 58 and st["tombstones"] == 0     # turned away before claiming a slot
    assert st["status"] == B.DEV_NEED_REHASH and st["rows_used"] == 192 and st["rows_free"] == 0
    r = r2.cpu().numpy()
    assert (r[:20] >= 0).all() and (r[20:] >= 0).sum() == 42 and (r[20:] == -1).sum() == 58
    assert np.array_equal(ins.cpu().numpy() == 1, np.concatenate([np.zeros(20, bool), r[20:] >= 0]))
    # the keys that were turned away read as absent
    found = torch.empty(120, dtype=torch.int32, device="cuda")
    t.find(dev_keys(more), None, 120, found)
    assert np.array_equal(found.cpu().numpy(), r)
    # make room (the plan doubles: 192 live + 58 to come > 0.375 * 256) and issue the call again for the rest
    B.ht_clear_status(t.h, B.DEV_NEED_REHASH)
    t.make_room(58)
    assert B.ht_find_or_insert_retry(t.h, dev_keys(more), None, 120, 4, r2, ins, touch=True) == B.EMB_OK
    st = t.stats()
    assert st["live"] == 250 and st["tombstones"] == 0 and st["capacity"] == 1024 and st["status"] == 0 and st["refused"] == 58
    assert (r2 >= 0).all() and np.array_equal(r2.cpu().numpy()[:20], r[:20]) and int(ins.sum().item()) == 100
    ot.find_or_insert(more, 4)
    gk, gv, gl, gf = _export_maps(t)
    ok, ov, oa, ol, of = ot.export()
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov) and np.array_equal(gl, ol) and np.array_equal(gf, of)
    t.close()


def test_storage_owner_reaches_the_load_factor_limit_before_it_rehashes():
    """The same through EmbeddingTable.find_or_insert: the key structure is expanded only when the device has
    turned keys away at the limit, so the load factor touches 0.85 (R7), and duplicates in the call are handled."""
    t = EmbeddingTable(16, 0, capacity_log2=10, chunk_rows_log2=8, initial_chunks=1, max_load_factor=0.85)
    ot = oracle.Table(16, 0)
    rng = np.random.default_rng(8)
    peak = 0.0
    for step in range(1, 40):
        ks = scramble_bits(rng.integers(0, 60 * step, size=300).astype(np.uint64), 40, 5)   # duplicates, growing vocabulary
        row_idx = torch.empty(300, dtype=torch.int32, device="cuda")
        t.find_or_insert(dev_keys(ks), None, 300, step, row_idx)
        ot.find_or_insert(ks, step)
        assert (row_idx >= 0).all()
        st = t.stats()
        assert st["status"] == 0 and st["live"] == len(ot) and st["rows_free"] + st["live"] == st["rows_used"]
        peak = max(peak, t.peak_load)
    assert t.stats()["n_rehash"] >= 1 and 0.84 <= peak <= float(np.float32(0.85))
    gk, gv, gl, gf = _export_maps(t)
    ok, ov, oa, ol, of = ot.export()
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov) and np.array_equal(gl, ol) and np.array_equal(gf, of)
    t.close()


def test_out_of_rows_turns_keys_away_and_leaks_nothing():
    t = EmbeddingTable(32, 0, capacity_log2=10, chunk_rows_log2=5, initial_chunks=1)       # 32 rows registered
    ks = np.arange(1, 51, dtype=np.uint64) * np.uint64(7919)
    r = torch.empty(50, dtype=torch.int32, device="cuda")
    assert B.ht_find_or_insert(t.h, dev_keys(ks), None, 50, 1, r) == B.EMB_CHECK_STATUS
    st = t.stats()
    assert st["status"] == B.DEV_OUT_OF_ROWS and st["live"] == 32 and st["refused"] == 18 and st["tombstones"] == 18
    assert st["rows_used"] == 32 and st["rows_free"] == 0          # the allocator stops at the registered rows
    assert int((r >= 0).sum().item()) == 32 and int((r == -1).sum().item()) == 18
    assert sorted(r[r >= 0].cpu().tolist()) == list(range(32))     # every row handed out once
    B.ht_clear_status(t.h, B.DEV_OUT_OF_ROWS)
    t.make_room(18)                                                 # one more chunk; the key structure is fine
    B.ht_find_or_insert_retry(t.h, dev_keys(ks), None, 50, 1, r, None, touch=True)
    st = t.stats()
    assert st["status"] == 0 and st["live"] == 50 and st["rows_used"] == 50 and st["n_chunks"] == 2 and st["n_rehash"] == 0
    assert st["refused"] == 18
    assert sorted(r.cpu().tolist()) == list(range(50))             # no row skipped, none handed out twice
    gk, gv, gl, gf = _export_maps(t)
    assert np.array_equal(gk, np.sort(ks)) and (gf == 1).all() and (gl == 1).all()
    t.close()


def test_probe_sequence_exhausted_on_a_full_table():
    """A key structure filled to the last slot (load-factor limit 1.0, for this test only): a new key visits every
    line (Theorem 1), finds no room, gets -1 and sets the status bit; the kernel ends normally and nothing changes."""
    t = EmbeddingTable(32, 0, capacity_log2=6, chunk_rows_log2=7, initial_chunks=1, max_load_factor=1.0)   # 64 slots
    ks = np.arange(1, 65, dtype=np.uint64) * np.uint64(2654435761)
    r = torch.empty(64, dtype=torch.int32, device="cuda")
    assert B.ht_find_or_insert(t.h, dev_keys(ks), None, 64, 0, r) == B.EMB_OK
    st = t.stats()
    assert st["live"] == 64 and st["status"] == 0 and (r >= 0).all()
    extra = np.arange(100, 108, dtype=np.uint64) * np.uint64(40503)
    both = np.concatenate([ks[:8], extra])
    r2 = torch.empty(16, dtype=torch.int32, device="cuda")
    B.ht_find_or_insert(t.h, dev_keys(both), None, 16, 1, r2)
    st = t.stats()
    assert st["status"] == B.DEV_PROBE_EXHAUSTED and st["live"] == 64 and st["tombstones"] == 0 and st["refused"] == 8
    assert np.array_equal(r2[:8].cpu().numpy(), r[:8].cpu().numpy()) and (r2[8:] == -1).all()
    found = torch.empty(16, dtype=torch.int32, device="cuda")
    t.find(dev_keys(both), None, 16, found)                          # a read-only lookup of an absent key ends too
    assert torch.equal(found, r2)
    assert st["rows_free"] + st["live"] == st["rows_used"]
    t.close()


# ------------------------------------------------------------------------------------------ expand
@pytest.mark.parametrize("dim,dtype,n,u", [(64, 0, 10_000, 3000), (32, 0, 4097, 1), (128, 1, 5000, 5000),
                                            (16, 0, 63, 10), (128, 0, 2000, 300), (4, 0, 1000, 17), (256, 0, 3000, 500), (24, 0, 3000, 500),
                                            (256, 1, 3000, 500), (40, 1, 3000, 40)])
def test_expand(dim, dtype, n, u):
    rng = np.random.default_rng(n)
    rows = rng.standard_normal((u, dim)).astype(np.float32)
    inverse = rng.integers(0, u, size=n).astype(np.int32)
    tdt = torch.float32 if dtype == 0 else torch.bfloat16
    d_rows = torch.from_numpy(rows).cuda().to(tdt)
    out = torch.empty((n, dim), dtype=tdt, device="cuda")
    B.emb_expand(d_rows, torch.from_numpy(inverse).cuda(), n, dim, dtype, out)
    ref = oracle.expand(d_rows.float().cpu().numpy(), inverse)
    assert np.array_equal(out.float().cpu().numpy(), ref)
    # the sorted-order variant must give the same matrix: perm = positions by (index, position), seg_of = index there
    perm = np.argsort(inverse, kind="stable").astype(np.int32)
    seg_of = inverse[perm]
    out2 = torch.full((n, dim), 7.0, dtype=tdt, device="cuda")
    B.emb_expand_sorted(d_rows, torch.from_numpy(seg_of).cuda(), torch.from_numpy(perm).cuda(), n, dim, dtype, out2)
    assert np.array_equal(out2.float().cpu().numpy(), ref)


# ------------------------------------------------------------------------------------------ reduce
def _reduce_gpu(G_dev, dtype, keys):
    n, dim = G_dev.shape
    uniq, inverse, counts, perm, seg_off = _run_dedup(keys)
    U = len(uniq)
    d_sof, d_perm = torch.from_numpy(inverse[perm]).cuda(), torch.from_numpy(perm).cuda()
    red = torch.full((max(U, 1), dim), 123.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.grad_segment_reduce_workspace_bytes(n, dim), dtype=torch.uint8, device="cuda")
    B.grad_segment_reduce(G_dev, dtype, d_sof, d_perm, n, dim, red, ws)
    return red[:U].cpu().numpy(), inverse, U


@pytest.mark.parametrize("dim,dtype", [(64, 0), (32, 0), (16, 0), (128, 0), (128, 1), (8, 1), (256, 0), (4, 0), (24, 0), (256, 1), (40, 1)])
@pytest.mark.parametrize("shape", ["zipf", "one_giant_segment", "all_distinct", "tiny"])
def test_segment_reduce(dim, dtype, shape):
    n = {"zipf": 128 * 128 * 2 + 300, "one_giant_segment": 40_000, "all_distinct": 5000, "tiny": 3}[shape]
    if shape == "zipf":
        keys = _zipf_keys(n, 3000, 9)
    elif shape == "one_giant_segment":
        keys = np.full(n, 77, dtype=np.uint64)
        keys[::1000] = np.arange(len(keys[::1000]), dtype=np.uint64) + np.uint64(1000)
    elif shape == "all_distinct":
        keys = np.random.default_rng(1).permutation(n).astype(np.uint64)
    else:
        keys = np.array([9, 4, 9], dtype=np.uint64)
    # (a) integer-valued gradients: exactly one correct fp32 answer
    Gi = small_int_grads(n, dim, 3, "cuda")
    Gi_dev = Gi if dtype == 0 else Gi.to(torch.bfloat16)
    red, inverse, U = _reduce_gpu(Gi_dev, dtype, keys)
    ref = oracle.segment_reduce(Gi.cpu().numpy(), inverse, U)
    assert np.array_equal(red, ref)
    # (b) N(0,1) gradients: within 1e-5 of the float64 sum, relative to the sum of |addends|
    G = normal_grads(5, 0, n, dim)
    if dtype == 1:
        G = torch.from_numpy(G).to(torch.bfloat16).float().numpy()
    G_dev = torch.from_numpy(G).cuda() if dtype == 0 else torch.from_numpy(G).cuda().to(torch.bfloat16)
    red, inverse, U = _reduce_gpu(G_dev, dtype, keys)
    ref = oracle.segment_reduce(G, inverse, U).astype(np.float64)
    sabs = oracle.segment_reduce(np.abs(G), inverse, U).astype(np.float64)
    assert close_reduce(red, ref, sabs, RTOL_F32)
    assert np.allclose(red.astype(np.float64).sum(0), G.astype(np.float64).sum(0), rtol=0, atol=1e-5 * np.abs(G).sum(0).max())
    # (c) the order of additions is fixed: a second run is bit-identical
    red2, _, _ = _reduce_gpu(G_dev, dtype, keys)
    assert np.array_equal(red, red2)


# ------------------------------------------------------------------------------------------ adagrad
@pytest.mark.parametrize("dim,dtype", [(32, 0), (64, 0), (128, 0), (16, 0), (128, 1), (8, 1), (256, 0), (4, 0), (24, 0), (256, 1), (40, 1)])
def test_adagrad_matches_checker(dim, dtype):
    rtol = RTOL_F32 if dtype == 0 else RTOL_BF16
    keys = np.unique(_zipf_keys(6000, 4000, 21))
    n = len(keys)
    t = EmbeddingTable(dim, dtype, capacity_log2=14, chunk_rows_log2=11, initial_chunks=2)
    ot = oracle.Table(dim, dtype)
    row_idx = torch.empty(n, dtype=torch.int32, device="cuda")
    t.find_or_insert(dev_keys(keys), None, n, 0, row_idx)
    ot.find_or_insert(keys, 0)
    upd = np.arange(0, n, 2)                                     # update every other key; the rest must not move
    for step in range(3):
        g = normal_grads(31, step, len(upd), dim) * np.float32(10.0 ** (step - 1))
        g[5, :] = -2.5                                           # constant-gradient row
        ot.apply_adagrad(keys[upd], g, 0.01, 1e-8)
        ridx = row_idx[torch.from_numpy(upd).cuda()].contiguous()
        ridx[7] = -1                                             # a skipped entry
        ot_skip_fix = None
        t.apply_adagrad(ridx, torch.from_numpy(g).cuda(), None, len(upd), 0.01, 1e-8)
        # the checker updated entry 7 as well; undo by comparing everything except that key
        gk, gv, ga, _, _ = t.export()
        ok, ov, oa, _, _ = ot.export()
        assert np.array_equal(gk, ok)
        skip = np.isin(gk, keys[upd][7])
        touched = np.isin(gk, keys[upd]) & ~skip
        assert close_rows(gv[touched], ov[touched].astype(np.float64), 0.01, rtol)
        assert np.allclose(ga[touched], oa[touched], rtol=1e-5, atol=0)
        untouched = ~np.isin(gk, keys[upd])
        assert (ga[untouched] == 0).all()
        assert np.array_equal(gv[untouched], ov[untouched])
    if dtype == 0:
        # entry 7 was skipped on the device in all three steps: still the initial row
        assert np.array_equal(gv[skip][0], oracle.init_row(int(keys[upd][7]), dim))
    t.close()


# ------------------------------------------------------------------------------------------ evict / rehash
def test_evict_and_rehash_against_checker():
    dim = 32
    t = EmbeddingTable(dim, 0, capacity_log2=12, chunk_rows_log2=10, max_load_factor=0.75, initial_chunks=2)
    ot = oracle.Table(dim, 0)
    rng = np.random.default_rng(4)
    pool = scramble_bits(np.arange(3000, dtype=np.uint64), 40, 99)
    total_evicted = 0
    for step in range(60):
        ks = np.unique(pool[rng.integers(0, min(3000, 200 + 50 * step), size=400)])
        n = len(ks)
        row_idx = torch.empty(n, dtype=torch.int32, device="cuda")
        t.find_or_insert(dev_keys(ks), None, n, step, row_idx)
        ot.find_or_insert(ks, step)
        g = normal_grads(77, step, n, dim)
        t.apply_adagrad(row_idx, torch.from_numpy(g).cuda(), None, n, 0.01, 1e-8)
        ot.apply_adagrad(ks, g, 0.01, 1e-8)
        if step % 10 == 9:
            before = t.export()
            ev, n_ev = t.evict(step, 12, 3, 4)
            oev = ot.evict(step, 12, 3, 4)
            assert n_ev == len(oev) and np.array_equal(np.sort(host_keys(ev)), oev)     # eviction set, as a set
            total_evicted += n_ev
            st = t.stats()
            assert st["live"] == len(ot) == len(before[0]) - n_ev and st["tombstones"] >= n_ev > 0
            # evicted keys read as absent; survivors keep their rows bit for bit
            found = torch.empty(max(n_ev, 1), dtype=torch.int32, device="cuda")
            t.find(ev.contiguous(), None, n_ev, found)
            assert (found[:n_ev] == -1).all()
            after = t.export()
            keep = ~np.isin(before[0], oev)
            assert np.array_equal(after[0], before[0][keep]) and np.array_equal(after[1], before[1][keep])
            assert np.array_equal(after[2], before[2][keep])
        if step == 35:
            # explicit rehash to the same size: purges deleted markers, content unchanged
            before = t.export()
            t.rehash(t.capacity_log2)
            st = t.stats()
            assert st["tombstones"] == 0 and st["live"] == len(before[0])
            for a, b in zip(before, t.export()):
                assert np.array_equal(a, b)
    assert total_evicted > 100
    st = t.stats()
    assert st["n_rehash"] >= 2 and st["status"] == 0 and st["rows_free"] + st["live"] <= st["rows_used"]
    gk, gv, ga, gl, gf = t.export()
    ok, ov, oa, ol, of = ot.export()
    assert np.array_equal(gk, ok) and np.array_equal(gl, ol) and np.array_equal(gf, of)
    assert close_rows(gv, ov.astype(np.float64), 0.01, RTOL_F32) and np.allclose(ga, oa, rtol=1e-5)
    # a re-inserted key starts from its initial row with a zero accumulator
    gone = np.setdiff1d(pool, gk)[:5]
    row_idx = torch.empty(5, dtype=torch.int32, device="cuda")
    t.find_or_insert(dev_keys(gone), None, 5, 61, row_idx)
    out = torch.empty((5, dim), device="cuda")
    t.gather(row_idx, None, 5, out)
    assert np.array_equal(out.cpu().numpy(), np.stack([oracle.init_row(int(k), dim) for k in gone]))
    t.close()


@pytest.mark.parametrize("grow", [0, 1, 2, 3, 4, -1])
def test_rehash_keeps_every_pair_at_high_load(grow):
    """Key-structure migration from a table at load 0.85 with deleted markers (a good part of the keys sits away
    from its home line): same size, 2, 4, 8 times larger (two streaming passes), 16 times larger and smaller (general
    path).  Every live key keeps its row, deleted keys stay absent, no marker survives, the lookup still ends within a
    few lines, and inserts work afterwards."""
    cap_log2 = 14
    n = int(np.float32(0.85) * (1 << cap_log2))
    keys = scramble_bits(np.arange(n, dtype=np.uint64), 44, 21)
    t = EmbeddingTable(8, 0, capacity_log2=cap_log2, chunk_rows_log2=cap_log2, max_load_factor=0.85, count_probes=True,
                       initial_chunks=2)
    rows = torch.empty(n, dtype=torch.int32, device="cuda")
    # two halves at steps 1 and 2, then everything of step 1 is evicted: markers all over the probe sequences
    h = n // 2 if grow >= 0 else (n * 3) // 4
    t.find_or_insert(dev_keys(keys[:h]), None, h, 1, rows[:h])
    t.find_or_insert(dev_keys(keys[h:]), None, n - h, 2, rows[h:])
    assert t.stats()["live"] == n
    ev, n_ev = t.evict(3, 2, 0, 0)                    # last seen at step 1 -> age 2 -> out
    assert n_ev == h
    keep = keys[h:]
    before = torch.empty(len(keep), dtype=torch.int32, device="cuda")
    t.find(dev_keys(keep), None, len(keep), before)
    assert (before >= 0).all()
    t.rehash(cap_log2 + grow)
    st = t.stats()
    assert st["live"] == len(keep) and st["tombstones"] == 0 and st["status"] == 0 and st["capacity"] == 1 << (cap_log2 + grow)
    after = torch.empty_like(before)
    p0 = st["probes"]
    t.find(dev_keys(keep), None, len(keep), after)
    assert torch.equal(before, after)
    lines = (t.stats()["probes"] - p0) / len(keep)
    assert lines < (1.6 if grow <= 0 else 1.2), lines
    gone = torch.empty(h, dtype=torch.int32, device="cuda")
    t.find(dev_keys(keys[:h]), None, h, gone)
    assert (gone == -1).all()
    # the migrated structure takes inserts like any other: the evicted keys come back as new rows
    back = min(h, int(0.85 * (1 << (cap_log2 + grow))) - len(keep))
    t.find_or_insert(dev_keys(keys[:back]), None, back, 4, gone[:back])
    st = t.stats()
    assert (gone[:back] >= 0).all() and st["live"] == len(keep) + back and st["status"] == 0
    t.find(dev_keys(keep), None, len(keep), after)
    assert torch.equal(before, after)
    t.close()


def test_evict_and_export_respect_the_capacity_of_their_output_lists():
    """ht_evict and ht_export store at most `cap` entries, report the full count, and write nothing beyond the
    list's end; what they store is a subset of the right answer."""
    n, dim = 5000, 8
    keys = scramble_bits(np.arange(n, dtype=np.uint64), 40, 31)
    t = EmbeddingTable(dim, 0, capacity_log2=14, chunk_rows_log2=13, initial_chunks=1)
    rows = torch.empty(n, dtype=torch.int32, device="cuda")
    t.find_or_insert(dev_keys(keys[:3000]), None, 3000, 1, rows[:3000])
    t.find_or_insert(dev_keys(keys[3000:]), None, 2000, 5, rows[3000:])
    # export into lists shorter than the table
    cap = 1200
    guard = -12345
    ek = torch.full((cap + 64,), guard, dtype=torch.int64, device="cuda")
    ev = torch.full((cap + 64, dim), 7.5, dtype=torch.float32, device="cuda")
    ea = torch.full((cap + 64,), 7.5, dtype=torch.float32, device="cuda")
    el = torch.full((cap + 64,), guard, dtype=torch.int32, device="cuda")
    ef = torch.full((cap + 64,), guard, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    B.ht_export(t.h, ek[:cap], ev[:cap], ea[:cap], el[:cap], ef[:cap], cnt)
    assert int(cnt.item()) == n
    assert (ek[cap:] == guard).all() and (ev[cap:] == 7.5).all() and (ea[cap:] == 7.5).all()
    assert (el[cap:] == guard).all() and (ef[cap:] == guard).all()
    got = host_keys(ek[:cap])
    assert len(np.unique(got)) == cap and np.isin(got, keys).all()
    first = np.isin(got, keys[:3000])
    assert np.array_equal(el[:cap].cpu().numpy(), np.where(first, 1, 5)) and (ef[:cap] == 1).all() and (ea[:cap] == 0).all()
    want = np.stack([oracle.init_row(int(k), dim) for k in got[:50]])
    assert np.array_equal(ev[:50].cpu().numpy(), want)
    # evict the 3000 keys of step 1 into a list of 1000
    cap = 1000
    kk = torch.full((cap + 64,), guard, dtype=torch.int64, device="cuda")
    n_ev = torch.zeros(1, dtype=torch.int64, device="cuda")
    B.ht_evict(t.h, 6, 3, 0, 0, kk[:cap], n_ev)                  # age >= 3: the keys last seen at step 1
    assert int(n_ev.item()) == 3000 and (kk[cap:] == guard).all()
    listed = host_keys(kk[:cap])
    assert len(np.unique(listed)) == cap and np.isin(listed, keys[:3000]).all()
    st = t.stats()
    assert st["live"] == 2000 and st["tombstones"] == 3000 and st["rows_free"] == 3000 and st["status"] == 0
    found = torch.empty(n, dtype=torch.int32, device="cuda")
    t.find(dev_keys(keys), None, n, found)
    assert (found[:3000] == -1).all() and torch.equal(found[3000:], rows[3000:])
    # without a list at all
    B.ht_evict(t.h, 9, 3, 0, 0, None, n_ev)
    assert int(n_ev.item()) == 2000 and t.stats()["live"] == 0
    t.close()


def test_full_table_up_to_the_load_factor_limit():
    # exactly capacity * max_load_factor keys fit without a rehash and are all found again
    cap_log2 = 13
    n = int((1 << cap_log2) * 0.75)
    keys = scramble_bits(np.arange(n, dtype=np.uint64), 40, 5)
    t = EmbeddingTable(16, 0, capacity_log2=cap_log2, chunk_rows_log2=cap_log2, count_probes=True, initial_chunks=1)
    row_idx = torch.empty(n, dtype=torch.int32, device="cuda")
    assert B.ht_find_or_insert(t.h, dev_keys(keys), None, n, 0, row_idx) == 0
    st = t.stats()
    assert st["live"] == n and st["n_rehash"] == 0 and st["status"] == 0
    assert len(np.unique(row_idx.cpu().numpy())) == n
    found = torch.empty(n, dtype=torch.int32, device="cuda")
    t.find(dev_keys(keys), None, n, found)
    assert torch.equal(found, row_idx)
    st2 = t.stats()
    assert (st2["probes"] - st["probes"]) / n < 2.5          # lines inspected per successful lookup at LF 0.75
    t.close()


# ------------------------------------------------------------------------------------------ fused form
@pytest.mark.parametrize("dim,dtype", [(64, 0), (32, 0), (128, 0), (128, 1), (16, 0), (8, 1), (256, 0), (4, 0), (24, 0), (256, 1), (40, 1)])
def test_fused_gather_expand_equals_the_two_calls(dim, dtype):
    """gather+expand in one kernel is bit-identical to ht_gather followed by emb_expand(_sorted), over
    several steps with updates in between, and agrees with the checker's direct lookup."""
    from paper_2505_12663_amd import forward, backward, forward_fused
    rtol = RTOL_F32 if dtype == 0 else RTOL_BF16
    n = 64 * 64 * 3 + 77
    raw = _zipf_keys(n, 2500, 33) & np.uint64((1 << 40) - 1)
    off, tags = np.array([0, n], dtype=np.int64), np.array([0], dtype=np.uint8)
    dx, doff, dtag = dev_keys(raw), torch.from_numpy(off).cuda(), torch.from_numpy(tags).cuda()
    ta = EmbeddingTable(dim, dtype, capacity_log2=14, chunk_rows_log2=12)
    tb = EmbeddingTable(dim, dtype, capacity_log2=14, chunk_rows_log2=12)
    ot = oracle.Table(dim, dtype)
    ba, bb = StepBuffers(n, dim, dtype), StepBuffers(n, dim, dtype)
    okey, _ = oracle.tag_keys(raw, off, tags, 1)
    ou, oi, oc = oracle.dedup(okey)
    for step in range(3):
        forward(ta, ba, dx, doff, dtag, 1, step)
        forward_fused(tb, bb, dx, doff, dtag, 1, step)
        assert torch.equal(ba.out[:n], bb.out[:n])                       # same bits, with and without E_u
        ot.find_or_insert(ou, step)
        oE = oracle.expand(ot.lookup(ou), oi)
        assert close_rows(bb.out[:n].float().cpu().numpy(), oE.astype(np.float64), 0.01, rtol)
        if step == 0:
            assert np.array_equal(bb.out[:n].float().cpu().numpy(), oE)  # before any update: bit-exact
        G = normal_grads(9, step, n, dim)
        if dtype == 1:
            G = torch.from_numpy(G).to(torch.bfloat16).float().numpy()
        dG = torch.from_numpy(G).cuda() if dtype == 0 else torch.from_numpy(G).cuda().to(torch.bfloat16)
        backward(ta, ba, dG, n, 0.01, 1e-8)
        backward(tb, bb, dG, n, 0.01, 1e-8)
        ot.apply_adagrad(ou, oracle.segment_reduce(G, oi, len(ou)), 0.01, 1e-8)
    ta.close()
    tb.close()


def test_dedup_without_position_ordered_inverse():
    """inverse is optional: with NULL every other output is unchanged, and (perm, seg_of) carry the same mapping."""
    keys = _zipf_keys(50_000, 7000, 3)
    n = len(keys)
    a, b = StepBuffers(n, 16, with_grad=False), StepBuffers(n, 16, with_grad=False)
    dk = dev_keys(keys)
    B.emb_dedup(dk, n, a.uniq, a.inverse, a.counts, a.perm, a.seg_off, a.seg_of, a.n_unique, a.dedup_ws)
    b.inverse.fill_(-7)
    B.emb_dedup(dk, n, b.uniq, None, b.counts, b.perm, b.seg_off, b.seg_of, b.n_unique, b.dedup_ws)
    U = int(a.n_unique.item())
    assert int(b.n_unique.item()) == U
    for x, y, m in ((a.uniq, b.uniq, U), (a.counts, b.counts, U), (a.perm, b.perm, n), (a.seg_of, b.seg_of, n),
                    (a.seg_off, b.seg_off, U + 1)):
        assert torch.equal(x[:m], y[:m])
    assert bool((b.inverse == -7).all())                                   # untouched
    rebuilt = torch.empty(n, dtype=torch.int32, device="cuda")
    rebuilt[b.perm[:n].long()] = b.seg_of[:n]
    assert torch.equal(rebuilt, a.inverse[:n])                             # inverse[perm[j]] == seg_of[j]
    ou, oi, oc = oracle.dedup(keys)
    assert np.array_equal(rebuilt.cpu().numpy(), oi) and np.array_equal(host_keys(b.uniq[:U]), ou)
