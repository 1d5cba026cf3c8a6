"""Pins of the CPU checker against things other than itself.

Each test ties one function of ``oracle/`` to what the paper or plain
mathematics fixes: the paper's worked tagging example, brute force on tiny
inputs, library routines on special cases (``torch.unique``,
``torch.optim.Adagrad`` at dim 1, ``numpy.add.at``, torch's bfloat16 cast),
closed forms and invariants.  None of them needs a GPU.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import make_config, normal_grads


def _read_rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# --------------------------------------------------------------------------- #
# tagging (Sec. 3.2, Eq. 8)
# --------------------------------------------------------------------------- #
def test_tag_bits_paper_example_and_formula(golden_dir):
    m, k, shift, row_bits, max_rows_log2 = map(int, _read_rows(os.path.join(golden_dir, "eq8_table_tag_example.txt"))[0])
    assert oracle.tag_bits(m) == k
    assert 63 - k == shift == row_bits == max_rows_log2
    for m_, k_ in _read_rows(os.path.join(golden_dir, "tag_bits_formula.txt")):
        assert oracle.tag_bits(int(m_)) == int(k_)


def test_tag_keys_bit_layout():
    # three tables, two identifier bits: table i sits at bit 61 (Eq. 8 with k = 2)
    x = np.array([0, 1, 5, (1 << 61) - 1, 7, 7, 7], dtype=np.uint64)
    off = np.array([0, 3, 4, 7], dtype=np.int64)
    tags = np.array([0, 1, 2], dtype=np.uint8)
    key, errs = oracle.tag_keys(x, off, tags, 2)
    assert errs == 0
    assert key.tolist() == [0, 1, 5, (1 << 61) | ((1 << 61) - 1), (2 << 61) | 7, (2 << 61) | 7, (2 << 61) | 7]
    assert (key >> np.uint64(63) == 0).all()                       # offset stays a positive int64
    assert ((key >> np.uint64(61)).astype(np.int64) == [0, 0, 0, 1, 2, 2, 2]).all()   # tag round trip
    assert ((key & np.uint64((1 << 61) - 1)) == x).all()           # raw ID round trip
    # same raw ID in two tables -> two different keys
    assert key[4] != (1 << 61) | 7


def test_tag_keys_range_error_is_counted():
    x = np.array([1 << 61, 3], dtype=np.uint64)     # first ID needs 62 bits, only 61 available
    key, errs = oracle.tag_keys(x, np.array([0, 2], dtype=np.int64), np.array([1], dtype=np.uint8), 2)
    assert errs == 1
    assert key.tolist() == [(1 << 61) | 0, (1 << 61) | 3]
    with pytest.raises(ValueError):   # table index 4 does not fit in 2 bits
        oracle.tag_keys(x, np.array([0, 2], dtype=np.int64), np.array([4], dtype=np.uint8), 2)


def test_tag_keys_eight_bit_tags_and_empty_fields():
    rng = np.random.default_rng(1)
    x = rng.integers(0, 1 << 55, size=100, dtype=np.uint64)
    off = np.array([0, 0, 40, 40, 100], dtype=np.int64)
    tags = np.array([9, 200, 3, 31], dtype=np.uint8)
    key, errs = oracle.tag_keys(x, off, tags, 8)
    assert errs == 0
    expect_tag = np.array([200] * 40 + [31] * 60, dtype=np.uint64)
    assert ((key >> np.uint64(55)) == expect_tag).all()
    assert ((key & np.uint64((1 << 55) - 1)) == x).all()


def test_plan_merge_groups_by_dim_and_dtype():
    merged_of, n = oracle.plan_merge([64, 16, 64, 128, 16, 64], [0, 0, 0, 0, 1, 0])
    assert n == 4
    assert merged_of.tolist() == [0, 1, 0, 2, 3, 0]     # order of first appearance; (16,bf16) != (16,f32)


# --------------------------------------------------------------------------- #
# deduplication (Sec. 3.3)
# --------------------------------------------------------------------------- #
def _brute_dedup(keys):
    keys = [int(k) for k in keys]
    uniq = []
    for k in keys:                     # O(N^2): no sort, no hashing
        if all(k != u for u in uniq):
            uniq.append(k)
    for i in range(len(uniq)):         # selection sort
        for j in range(i + 1, len(uniq)):
            if uniq[j] < uniq[i]:
                uniq[i], uniq[j] = uniq[j], uniq[i]
    inverse = [next(p for p, u in enumerate(uniq) if u == k) for k in keys]
    counts = [sum(1 for k in keys if k == u) for u in uniq]
    return uniq, inverse, counts


@pytest.mark.parametrize("case", ["random", "all_equal", "all_distinct", "empty", "single", "big_values"])
def test_dedup_brute_force(case):
    rng = np.random.default_rng(7)
    keys = {
        "random": rng.integers(0, 20, size=64),
        "all_equal": np.full(33, 12345),
        "all_distinct": rng.permutation(50) * 3 + 1,
        "empty": np.zeros(0),
        "single": np.array([9]),
        "big_values": rng.integers(0, 4, size=40) * ((1 << 61) + 12345) + (1 << 59),
    }[case].astype(np.uint64)
    uniq, inverse, counts = oracle.dedup(keys)
    bu, bi, bc = _brute_dedup(keys)
    assert uniq.tolist() == bu and inverse.tolist() == bi and counts.tolist() == bc


def test_dedup_matches_torch_unique_and_invariants():
    w = make_config(1)
    b = w.next_step(0)
    keys = np.concatenate(b.ids)
    uniq, inverse, counts = oracle.dedup(keys)
    tu, ti, tc = torch.unique(torch.from_numpy(keys.astype(np.int64)), sorted=True, return_inverse=True,
                              return_counts=True)
    assert np.array_equal(uniq.astype(np.int64), tu.numpy())
    assert np.array_equal(inverse.astype(np.int64), ti.numpy())
    assert np.array_equal(counts.astype(np.int64), tc.numpy())
    assert np.array_equal(uniq[inverse], keys)                  # every inverse index maps back to its key
    assert (np.diff(uniq.astype(np.int64)) > 0).all()           # strictly increasing
    assert counts.sum() == len(keys) and len(uniq) == len(set(keys.tolist()))


# --------------------------------------------------------------------------- #
# row initialisation (reading A2: key-seeded splitmix64 stream -> U[-s, s))
# --------------------------------------------------------------------------- #
def test_init_row_from_published_splitmix_vector(golden_dir):
    outs = [int(r[0], 16) for r in _read_rows(os.path.join(golden_dir, "splitmix64_seed0.txt"))]
    row = oracle.init_row(0, len(outs), oracle.F32, 0.01)
    for j, z in enumerate(outs):
        q = (z >> 40) - (1 << 23)                                  # top 24 bits, centred
        expect = np.float32(np.float32(q) * (np.float32(0.01) * np.float32(2.0 ** -23)))
        assert row[j] == expect
    # a different scale only rescales by an exact power-of-two-free constant: check 1.0 -> q * 2^-23 exactly
    row1 = oracle.init_row(0, len(outs), oracle.F32, 1.0)
    for j, z in enumerate(outs):
        assert float(row1[j]) == ((z >> 40) - (1 << 23)) / float(1 << 23)


def test_init_row_distribution_and_determinism():
    rows = np.stack([oracle.init_row(int(k), 64) for k in range(1000, 3000)])
    assert rows.min() >= -0.01 and rows.max() < 0.01
    assert abs(rows.mean()) < 2e-4
    assert abs(rows.var() - 0.01 ** 2 / 3) < 0.02 * (0.01 ** 2 / 3)     # variance of U(-s, s) is s^2/3
    assert np.array_equal(oracle.init_row(77, 64), oracle.init_row(77, 64))
    assert not np.array_equal(oracle.init_row(77, 64), oracle.init_row(78, 64))
    # a prefix of a longer row is the shorter row: element j depends on (key, j) only
    assert np.array_equal(oracle.init_row(77, 128)[:64], oracle.init_row(77, 64))
    # the tag takes part: same raw ID in tables 0 and 1 gives different rows
    assert not np.array_equal(oracle.init_row(5, 16), oracle.init_row((1 << 61) | 5, 16))
    # columns are uncorrelated across keys
    c = np.corrcoef(rows[:, 0], rows[:, 1])[0, 1]
    assert abs(c) < 0.08


def test_bf16_rounding_matches_torch_cast():
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 0.01,
                        np.array([1.0, 1.00390625, 1.001953125, 1.005859375, -1.001953125], dtype=np.float32)])
    bits = oracle.float_to_bf16_bits(a)
    t = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.astype(np.int16), t.view(torch.int16).numpy())
    assert np.array_equal(oracle.bf16_bits_to_float(bits), t.to(torch.float32).numpy())
    r = oracle.init_row(123, 128, oracle.BF16)
    assert np.array_equal(r, torch.from_numpy(oracle.init_row(123, 128, oracle.F32)).to(torch.bfloat16).float().numpy())


# --------------------------------------------------------------------------- #
# dynamic table: insert / lookup (Sec. 3.1)
# --------------------------------------------------------------------------- #
def test_find_or_insert_lookup_and_counters():
    t = oracle.Table(32)
    keys = np.array([11, 5, 11, 99, 5, 11], dtype=np.uint64)
    ins = t.find_or_insert(keys, step=4)
    assert ins.tolist() == [1, 1, 0, 1, 0, 0] and len(t) == 3
    rows = t.lookup(keys)
    for i, k in enumerate(keys):
        assert np.array_equal(rows[i], oracle.init_row(int(k), 32))     # lookup after insert = initial row
    ins2 = t.find_or_insert(np.array([5, 11, 99], dtype=np.uint64), step=5)
    assert ins2.sum() == 0 and len(t) == 3                             # second call inserts nothing
    k, v, acc, last_seen, freq = t.export()
    assert k.tolist() == [5, 11, 99]
    assert freq.tolist() == [3, 4, 2] and last_seen.tolist() == [5, 5, 5] and (acc == 0).all()
    assert t.find(np.array([5, 6], dtype=np.uint64)).tolist() == [1, 0]
    assert (t.lookup(np.array([6], dtype=np.uint64)) == 0).all()        # absent key reads as zeros
    with pytest.raises(ValueError):
        t.find_or_insert(np.array([1 << 63], dtype=np.uint64), 0)       # top bit must stay clear


def test_prepopulate_equals_one_touch_at_step_zero():
    a, b = oracle.Table(8), oracle.Table(8)
    keys = np.array([3, 1, 2], dtype=np.uint64)
    a.find_or_insert(keys, step=0)
    b.prepopulate(keys)
    b.prepopulate(keys[:2])                                            # idempotent
    for x, y in zip(a.export(), b.export()):
        assert np.array_equal(x, y)


def test_dedup_lookup_expand_equals_direct_lookup():
    # Sec. 3.3: deduplication only removes repeated transmission; the forward result is unchanged.
    w = make_config(1)
    b = w.next_step(0)
    off = np.concatenate([[0], np.cumsum([len(i) for i in b.ids])]).astype(np.int64)
    key, _ = oracle.tag_keys(np.concatenate(b.ids), off, np.zeros(4, dtype=np.uint8), oracle.tag_bits(1))
    t1, t2 = oracle.Table(32), oracle.Table(32)
    uniq, inverse, _ = oracle.dedup(key)
    t1.find_or_insert(uniq, 0)
    E = oracle.expand(t1.lookup(uniq), inverse)
    E_direct = t2.direct_lookup(key, 0)
    assert np.array_equal(E, E_direct)
    assert np.array_equal(t1.export()[0], t2.export()[0]) and np.array_equal(t1.export()[1], t2.export()[1])


# --------------------------------------------------------------------------- #
# gradient aggregation (Sec. 2 "Backward Update")
# --------------------------------------------------------------------------- #
def test_segment_reduce_exact_cases_and_conservation():
    rng = np.random.default_rng(5)
    n, U, D = 3000, 37, 8
    inverse = rng.integers(0, U, size=n).astype(np.int32)
    counts = np.bincount(inverse, minlength=U)
    ones = oracle.segment_reduce(np.ones((n, D), dtype=np.float32), inverse, U)
    assert np.array_equal(ones, np.repeat(counts[:, None], D, 1).astype(np.float32))     # G == 1 -> counts
    gi = rng.integers(-8, 9, size=(n, D)).astype(np.float32)
    ref = np.zeros((U, D), dtype=np.float64)
    np.add.at(ref, inverse, gi.astype(np.float64))
    assert np.array_equal(oracle.segment_reduce(gi, inverse, U), ref.astype(np.float32))  # integers: exact
    g = normal_grads(1, 0, n, D)
    red = oracle.segment_reduce(g, inverse, U)
    ref = np.zeros((U, D), dtype=np.float64)
    np.add.at(ref, inverse, g.astype(np.float64))
    assert np.array_equal(red, ref.astype(np.float32))                # float64 accumulate, one rounding
    assert np.allclose(red.astype(np.float64).sum(0), g.astype(np.float64).sum(0), rtol=0, atol=1e-3)  # conserved
    # a transposed or mis-indexed operand shows up here: segment u must only see its own rows
    one_hot = np.zeros((n, D), dtype=np.float32)
    one_hot[17, 3] = 2.0
    r = oracle.segment_reduce(one_hot, inverse, U)
    assert r[inverse[17], 3] == 2.0 and r.sum() == 2.0
    with pytest.raises(ValueError):
        oracle.segment_reduce(g, inverse, int(inverse.max()))     # one segment too few


# --------------------------------------------------------------------------- #
# row-wise Adagrad (reading A1)
# --------------------------------------------------------------------------- #
def test_adagrad_dim1_equals_torch_optim_adagrad():
    # With one element per row, row-wise Adagrad is the element-wise Adagrad of the library.
    keys = np.arange(1, 41, dtype=np.uint64)
    t = oracle.Table(1)
    t.find_or_insert(keys, 0)
    p = torch.nn.Parameter(torch.from_numpy(t.lookup(keys).astype(np.float64)).clone())
    opt = torch.optim.Adagrad([p], lr=float(np.float32(0.01)), eps=float(np.float32(1e-8)),
                              initial_accumulator_value=0.0)
    rng = np.random.default_rng(11)
    for step in range(5):
        g = rng.standard_normal((40, 1)).astype(np.float32)
        t.apply_adagrad(keys, g, 0.01, 1e-8)
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
        # library result in float64 vs checker (float64 math, stored in float32 each step)
        assert np.allclose(t.lookup(keys), p.detach().numpy(), rtol=2e-6, atol=1e-9)


def test_adagrad_first_step_closed_form_and_untouched_rows():
    D = 16
    keys = np.array([10, 20, 30, 40], dtype=np.uint64)
    t = oracle.Table(D)
    t.find_or_insert(keys, 0)
    w0 = t.lookup(keys).astype(np.float64)
    rng = np.random.default_rng(2)
    g = rng.standard_normal((2, D)).astype(np.float32)
    g[1, :] = -3.0                                               # constant-gradient row
    t.apply_adagrad(keys[[0, 2]], g, 0.01, 1e-8)
    k, v, acc, _, _ = t.export()
    # independent recomputation with torch float64 tensor ops
    gt = torch.from_numpy(g).double()
    acc_t = (gt * gt).mean(dim=1)
    w_t = torch.from_numpy(w0[[0, 2]]) - float(np.float32(0.01)) * gt / (acc_t.sqrt() + float(np.float32(1e-8)))[:, None]
    assert np.array_equal(acc[[0, 2]], acc_t.float().numpy())                 # acc = mean(g^2) on the first step
    assert np.array_equal(v[[0, 2]], w_t.float().numpy())
    assert np.allclose(v[2], w0[2] + 0.01, rtol=0, atol=1e-8)                  # w - lr * sign(c), c < 0
    assert np.array_equal(v[[1, 3]], w0[[1, 3]].astype(np.float32)) and (acc[[1, 3]] == 0).all()   # rows not listed
    # absent key is skipped, table unchanged in size
    t.apply_adagrad(np.array([999], dtype=np.uint64), g[:1], 0.01, 1e-8)
    assert len(t) == 4
    # second step accumulates: acc = mean(g1^2) + mean(g2^2)
    t.apply_adagrad(keys[[0]], g[:1], 0.01, 1e-8)
    assert np.isclose(t.export()[2][0], 2 * float(acc_t[0]), rtol=1e-6)


def test_adagrad_bf16_rows_round_once_to_nearest_even():
    D = 8
    keys = np.array([7], dtype=np.uint64)
    t = oracle.Table(D, oracle.BF16)
    t.find_or_insert(keys, 0)
    w0 = t.lookup(keys).astype(np.float64)
    g = (np.arange(D, dtype=np.float32).reshape(1, D) - 3.5) * 0.25
    t.apply_adagrad(keys, g, 0.01, 1e-8)
    acc = (g.astype(np.float64) ** 2).mean()
    w = w0 - float(np.float32(0.01)) * g.astype(np.float64) / (np.sqrt(acc) + float(np.float32(1e-8)))
    # nearest bf16 neighbours of the exact value: the stored value must be the closer one
    got = t.lookup(keys).astype(np.float64)
    lo = torch.from_numpy(w).float()
    cand = torch.stack([lo.to(torch.bfloat16).double(),
                        (lo * (1 + 2 ** -7)).to(torch.bfloat16).double(),
                        (lo * (1 - 2 ** -7)).to(torch.bfloat16).double()])
    best = cand.gather(0, (cand - torch.from_numpy(w)).abs().argmin(0, keepdim=True))[0].numpy()
    assert np.array_equal(got, best)
    assert np.array_equal(oracle.float_to_bf16_bits(got.astype(np.float32)).astype(np.uint32) << 16,
                          got.astype(np.float32).view(np.uint32))          # stored values are bf16-representable


# --------------------------------------------------------------------------- #
# eviction (reading A9)
# --------------------------------------------------------------------------- #
def test_evict_brute_force_predicate_and_reinsert():
    t = oracle.Table(4)
    rng = np.random.default_rng(9)
    for step in range(0, 40):
        ks = rng.integers(0, 60, size=8).astype(np.uint64)
        t.find_or_insert(np.unique(ks), step)
    t.apply_adagrad(np.array([1, 2, 3], dtype=np.uint64), np.ones((3, 4), dtype=np.float32), 0.01)
    keys, vals, acc, last_seen, freq = t.export()
    now, ttl, min_freq, grace = 40, 15, 3, 5
    expect = sorted(int(k) for k, ls, fq in zip(keys, last_seen, freq)
                    if (now - int(ls) >= ttl) or (int(fq) < min_freq and now - int(ls) >= grace))
    assert 0 < len(expect) < len(keys)
    gone = t.evict(now, ttl, min_freq, grace)
    assert gone.tolist() == expect                                        # ascending, exactly the predicate
    assert len(t) == len(keys) - len(expect)
    assert t.find(gone).sum() == 0                                        # evicted keys read as absent
    k2, v2, a2, _, _ = t.export()
    keep = ~np.isin(keys, gone)
    assert np.array_equal(k2, keys[keep]) and np.array_equal(v2, vals[keep]) and np.array_equal(a2, acc[keep])
    # a later re-insert is a fresh insert
    ins = t.find_or_insert(gone[:1], 41)
    assert ins.tolist() == [1]
    p, v, a, ls, fq = t.peek(gone[:1])
    assert p[0] == 1 and np.array_equal(v[0], oracle.init_row(int(gone[0]), 4)) and a[0] == 0 and fq[0] == 1
    # rules are switched off by a zero threshold
    assert len(t.evict(1000, 0, 0, 0)) == 0
    n = len(t)
    assert len(t.evict(1000, 1, 0, 0)) == n and len(t) == 0


def test_three_steps_of_tiny_config_conserve_and_stay_finite():
    """Whole-step sanity on configuration 1: sizes, conservation, monotone accumulator."""
    w = make_config(1)
    t = oracle.Table(32)
    prev_acc = {}
    for step in range(3):
        b = w.next_step(step)
        off = np.concatenate([[0], np.cumsum([len(i) for i in b.ids])]).astype(np.int64)
        key, _ = oracle.tag_keys(np.concatenate(b.ids), off, np.zeros(4, dtype=np.uint8), 1)
        uniq, inverse, counts = oracle.dedup(key)
        t.find_or_insert(uniq, step)
        G = normal_grads(w.seed, step, len(key), 32)
        g = oracle.segment_reduce(G, inverse, len(uniq))
        assert np.allclose(g.sum(0), G.astype(np.float64).sum(0), atol=1e-2)
        t.apply_adagrad(uniq, g, w.lr, w.eps)
        keys, vals, acc, last_seen, freq = t.export()
        assert np.isfinite(vals).all() and (acc >= 0).all()
        touched = np.isin(keys, uniq)
        assert (last_seen[touched] == step).all() and (last_seen[~touched] < step).all()
        for k, a in zip(keys.tolist(), acc.tolist()):
            assert a >= prev_acc.get(k, 0.0)
            prev_acc[k] = a


# --------------------------------------------------------------------------- #
# pooling (Sec. 3.2): the library routine for pooled lookups is torch's EmbeddingBag
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_pooling_forward_backward_equal_torch_embedding_bag(mode):
    rng = np.random.default_rng(21)
    U, D = 50, 8
    lens = np.array([3, 0, 1, 7, 2, 0, 5, 4], dtype=np.int64)          # two empty bags
    bag_off = np.concatenate([[0], np.cumsum(lens)])
    n = int(bag_off[-1])
    inverse = rng.integers(0, U, size=n).astype(np.int32)
    W = rng.standard_normal((U, D)).astype(np.float32)
    E = oracle.expand(W, inverse)
    pooled = oracle.pool_bags(E, bag_off, mode == "mean")
    Wt = torch.from_numpy(W.astype(np.float64)).requires_grad_(True)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(inverse.astype(np.int64)), Wt,
                                            torch.from_numpy(bag_off[:-1]), mode=mode)
    assert np.array_equal(pooled, ref.detach().float().numpy())                       # float64 sums, one rounding
    assert (pooled[[1, 5]] == 0).all()                                                 # empty bags
    # backward: d(loss)/dW from autograd == per-key reduction of the per-position gradients
    dY = rng.integers(-4, 5, size=(len(lens), D)).astype(np.float32)
    ref.backward(torch.from_numpy(dY.astype(np.float64)))
    G = oracle.pool_bags_backward(dY, bag_off, mode == "mean")
    g = oracle.segment_reduce(G, inverse, U)
    assert np.allclose(g, Wt.grad.numpy(), rtol=1e-6, atol=1e-6)
    if mode == "sum":
        assert np.array_equal(g, Wt.grad.float().numpy())                             # integers: exact
        assert np.array_equal(G, np.repeat(dY, lens, axis=0))


# --------------------------------------------------------------------------- #
# sparse Adam (Sec. 4.1 trains with Adam): the library routine is torch.optim.SparseAdam
# --------------------------------------------------------------------------- #
def test_sparse_adam_equals_torch_sparse_adam():
    D, n_keys = 6, 30
    keys = np.arange(100, 100 + n_keys, dtype=np.uint64)
    t = oracle.Table(D)
    t.find_or_insert(keys, 0)
    W0 = t.lookup(keys).astype(np.float64)
    p = torch.nn.Parameter(torch.from_numpy(W0).clone())
    lr, b1, b2, eps = float(np.float32(1e-3)), float(np.float32(0.9)), float(np.float32(0.999)), float(np.float32(1e-8))
    opt = torch.optim.SparseAdam([p], lr=lr, betas=(b1, b2), eps=eps)
    rng = np.random.default_rng(8)
    for step in range(1, 7):
        rows = np.sort(rng.choice(n_keys, size=11, replace=False))            # only these rows are activated
        g = rng.standard_normal((len(rows), D)).astype(np.float32)
        t.apply_adam(keys[rows], g, lr, step, b1, b2, eps)
        p.grad = torch.sparse_coo_tensor(torch.from_numpy(rows[None, :]), torch.from_numpy(g.astype(np.float64)),
                                         size=(n_keys, D))
        opt.step()
        # float64 library result vs checker (float64 math, fp32 state between steps)
        assert np.allclose(t.lookup(keys), p.detach().numpy(), rtol=3e-6, atol=1e-9)
    untouched_row = oracle.Table(D)
    untouched_row.find_or_insert(np.array([7], dtype=np.uint64), 0)
    untouched_row.apply_adam(np.array([9], dtype=np.uint64), np.ones((1, D), dtype=np.float32), lr, 1)   # absent key: skipped
    assert np.array_equal(untouched_row.lookup(np.array([7], dtype=np.uint64))[0], oracle.init_row(7, D))
    with pytest.raises(ValueError):
        t.apply_adam(keys[:1], np.ones((1, D), dtype=np.float32), lr, 0)


def test_sparse_adam_first_step_closed_form():
    # t = 1: m = (1-b1) g, v = (1-b2) g^2  =>  w -= lr * g / (|g| + eps * sqrt(1-b2)) ~ lr * sign(g)
    D = 4
    t = oracle.Table(D)
    k = np.array([5], dtype=np.uint64)
    t.find_or_insert(k, 0)
    w0 = t.lookup(k).astype(np.float64)
    g = np.array([[2.0, -3.0, 0.5, -0.25]], dtype=np.float32)
    t.apply_adam(k, g, 0.01, 1)
    assert np.allclose(t.lookup(k), w0 - 0.01 * np.sign(g), rtol=0, atol=2e-8)


# --------------------------------------------------------------------------- #
# hot / cold rows (App. C "Mixed Precision Training"): frequently used keys of a 16-bit table keep an
# fp32 vector so that repeated small updates are not lost to 16-bit rounding
# --------------------------------------------------------------------------- #
def test_hot_rows_keep_small_updates_that_cold_rows_lose():
    D, T, lr = 8, 1000, 1e-4      # total shift 6.2e-3, more than one 16-bit spacing below 1 (3.9e-3)
    t = oracle.Table(D, oracle.BF16, init_scale=1.0)
    keys = np.array([11, 12], dtype=np.uint64)
    t.find_or_insert(keys, 0)
    t.find_or_insert(keys[:1], 1)                      # key 11 touched twice, key 12 once
    t.set_hot(4)
    assert t.promote(keys, 2) == 1                     # only key 11 qualifies
    assert np.array_equal(t.export_hot()[0], keys[:1])
    w0 = t.lookup(keys).astype(np.float64)
    assert np.array_equal(t.export_hot()[1][0], w0[0].astype(np.float32))   # the master starts as the 16-bit values
    g = np.ones((2, D), dtype=np.float32)
    for _ in range(T):
        t.apply_adagrad(keys, g, lr, 0.0)
    # constant unit gradient: acc after s steps = s, so the total shift is lr * sum_s 1/sqrt(s)
    shift = lr * np.sum(1.0 / np.sqrt(np.arange(1, T + 1, dtype=np.float64)))
    master = t.export_hot()[1][0].astype(np.float64)
    assert np.allclose(master, w0[0] - shift, rtol=0, atol=T * 2.0 ** -25)  # T fp32 roundings of values below 1
    got = t.lookup(keys).astype(np.float64)
    big = np.abs(w0) > 0.25                             # there a step of at most 1e-4 is below half a 16-bit spacing
    assert big[0].any() and big[1].any()
    assert np.array_equal(got[1][big[1]], w0[1][big[1]])                    # cold: every single update rounds away
    assert np.all(np.abs(got[0][big[0]] - (w0[0][big[0]] - shift)) <= 2.0 ** -9)   # hot: delivered = rounded master
    assert np.all(got[0][big[0]] != w0[0][big[0]])
    assert np.array_equal(got[0], torch.from_numpy(master.astype(np.float32)).to(torch.bfloat16).float().numpy())


def test_hot_and_cold_updates_equal_torch_casts():
    D, n_keys, lr, eps = 16, 12, 0.05, 1e-8
    keys = np.arange(1, n_keys + 1, dtype=np.uint64) * np.uint64(7919)
    t = oracle.Table(D, oracle.BF16)
    t.find_or_insert(keys, 0)
    t.find_or_insert(keys[::2], 1)
    t.set_hot(n_keys)
    assert t.promote(keys, 2) == n_keys // 2
    hot = np.zeros(n_keys, dtype=bool)
    hot[::2] = True
    w = torch.from_numpy(t.lookup(keys)).double()
    acc = torch.zeros(n_keys, dtype=torch.float64)
    rng = np.random.default_rng(5)
    for _ in range(6):
        g = rng.standard_normal((n_keys, D)).astype(np.float32)
        t.apply_adagrad(keys, g, lr, eps)
        gd = torch.from_numpy(g).double()
        acc_new = acc + (gd * gd).mean(dim=1)             # used unrounded within the step, stored as fp32
        new = w - float(np.float32(lr)) * gd / (acc_new.sqrt() + float(np.float32(eps)))[:, None]
        acc = acc_new.float().double()
        as_f32 = new.float()
        w = torch.where(torch.from_numpy(hot)[:, None], as_f32.double(), new.to(torch.bfloat16).double())
    assert np.array_equal(t.export_hot()[1], w[torch.from_numpy(hot)].float().numpy())
    assert np.array_equal(t.lookup(keys), w.float().to(torch.bfloat16).float().numpy())


def test_hot_store_capacity_and_release_on_eviction():
    t = oracle.Table(4, oracle.BF16)
    keys = np.arange(1, 9, dtype=np.uint64)
    t.find_or_insert(keys, 0)
    t.find_or_insert(keys, 1)
    t.set_hot(3)
    assert t.promote(keys, 2) == 3 and np.array_equal(t.export_hot()[0], keys[:3])   # in the order given
    assert t.promote(keys, 2) == 0                                                    # full
    t.find_or_insert(keys[1:], 50)
    assert np.array_equal(t.evict(60, 20, 0, 0), keys[:1])                            # key 1 is stale; its master is released
    assert t.promote(keys, 2) == 1 and np.array_equal(t.export_hot()[0], keys[1:4])
    with pytest.raises(ValueError):
        oracle.Table(4).set_hot(3)                                                    # fp32 tables have no cold form


def test_demotion_keeps_what_lookups_deliver_and_frees_the_master():
    """Demotion by idle time (App. C: the hot set follows the access pattern).  Pins: the demoted set is the brute-force
    predicate over the dump; a lookup delivers the same bits before and after (a hot row is delivered as its rounded
    master, which is exactly what the 16-bit row becomes); the master returns to the store; and from then on the row
    rounds like any cold row - one more update equals torch's bf16 arithmetic on the delivered values."""
    D, lr, eps = 16, 0.05, 1e-8
    keys = np.arange(1, 13, dtype=np.uint64) * np.uint64(104729)
    t = oracle.Table(D, oracle.BF16, init_scale=1.0)
    for s in range(3):
        t.find_or_insert(keys, s)
    t.set_hot(8)
    assert t.promote(keys, 3) == 8                       # the first eight, in the order given
    rng = np.random.default_rng(5)
    for s in range(3, 9):                                # keys[::2] stay in use, the others fall idle after step 2
        t.find_or_insert(keys[::2], s)
        t.apply_adagrad(keys, rng.standard_normal((len(keys), D)).astype(np.float32), lr, eps)
    hot_before = t.export_hot()[0]
    assert np.array_equal(hot_before, keys[:8])
    _, _, _, last_seen, _ = t.export()
    before = t.lookup(keys)
    now, idle = 9, 5
    want = np.array([k for k, ls in zip(np.sort(keys), last_seen) if k in set(hot_before) and now - int(ls) >= idle])
    assert t.demote(now, idle) == len(want) == 4         # keys[1], [3], [5], [7]
    assert np.array_equal(t.export_hot()[0], np.setdiff1d(hot_before, want))
    assert np.array_equal(t.lookup(keys), before)        # delivered bits unchanged
    assert t.demote(now, idle) == 0                      # nothing is demoted twice
    assert t.promote(keys[8:], 3) == 4                   # the freed masters serve other keys
    # a demoted row now updates in 16-bit arithmetic: torch casts as the independent statement
    k = want[:1]
    w = torch.from_numpy(t.lookup(k)[0].copy())
    _, _, acc0, _, _ = t.peek(k)
    g = rng.standard_normal((1, D)).astype(np.float32)
    t.apply_adagrad(k, g, lr, eps)
    acc = np.float64(acc0[0]) + np.mean(g[0].astype(np.float64) ** 2)
    ref = (w.double() - lr * torch.from_numpy(g[0]).double() / (np.sqrt(np.float32(acc).astype(np.float64)) + eps))
    assert torch.equal(torch.from_numpy(t.lookup(k)[0]), ref.float().to(torch.bfloat16).float())


def test_restored_masters_continue_where_the_dump_left_off():
    """Checkpoint of a table with hot rows (App. C): the dump holds the 16-bit view of every row and the fp32 masters.
    Pins: a table restored with its masters delivers the same bits and then follows the original bit for bit through
    many small updates; restored without them (all rows cold) it loses those updates to 16-bit rounding, which is the
    closed form of the hot/cold pin above (constant unit gradient: shift = lr * sum 1/sqrt(s))."""
    D, T, lr = 8, 400, 1e-4
    keys = np.array([21, 22, 23], dtype=np.uint64)
    a = oracle.Table(D, oracle.BF16, init_scale=1.0)
    a.find_or_insert(keys, 0)
    a.find_or_insert(keys[:2], 1)
    a.set_hot(4)
    assert a.promote(keys, 2) == 2
    g = np.ones((3, D), dtype=np.float32)
    for _ in range(T):
        a.apply_adagrad(keys, g, lr, 0.0)
    dk, dv, dacc, dls, dfq = a.export()
    hk, hv = a.export_hot()

    def restore(with_masters: bool):
        b = oracle.Table(D, oracle.BF16, init_scale=1.0)
        b.find_or_insert(dk, 0)
        b.put(dk, dv, dacc, dls, dfq)
        b.set_hot(4)
        if with_masters:
            assert b.promote(hk, 0) == len(hk) and b.put_hot(hk, hv) == len(hk)
            assert b.put_hot(keys[2:], hv[:1]) == 0          # a cold key is skipped
        return b

    full, cold = restore(True), restore(False)
    assert np.array_equal(full.export_hot()[1], hv) and np.array_equal(full.lookup(keys), a.lookup(keys))
    assert np.array_equal(cold.lookup(keys), a.lookup(keys))  # the 16-bit view is what the dump delivered
    for _ in range(T):
        for t in (a, full, cold):
            t.apply_adagrad(keys, g, lr, 0.0)
    assert np.array_equal(full.export_hot()[1], a.export_hot()[1]) and np.array_equal(full.lookup(keys), a.lookup(keys))
    steps = np.arange(T + 1, 2 * T + 1, dtype=np.float64)
    shift = lr * np.sum(1.0 / np.sqrt(steps))                # what the second T steps move a value by
    w_mid = hv.astype(np.float64)
    assert np.allclose(a.export_hot()[1], w_mid - shift, rtol=0, atol=T * 2.0 ** -25)
    big = np.abs(dv[:2]) > 0.25                              # there every single step is below half a 16-bit spacing
    assert big.any() and np.array_equal(cold.lookup(keys[:2])[big], dv[:2][big])   # without masters nothing moves


def test_adam_on_a_hot_row_is_the_fp32_update():
    """A hot row of a 16-bit table under Adam: its master must move exactly like the row of an fp32 table that starts
    from the same (16-bit representable) values - the fp32 table's Adam is pinned to torch.optim.SparseAdam above -
    while a cold row of the same table ends on 16-bit values."""
    D, lr = 16, 1e-2
    keys = np.array([5, 6], dtype=np.uint64)
    tb = oracle.Table(D, oracle.BF16, init_scale=1.0)
    tb.find_or_insert(keys, 0)
    tb.find_or_insert(keys[:1], 1)
    tb.set_hot(2)
    assert tb.promote(keys, 2) == 1                                  # key 5 hot, key 6 cold
    start = tb.lookup(keys)
    t32 = oracle.Table(D, oracle.F32, init_scale=1.0)
    t32.find_or_insert(keys, 0)
    _, _, acc, ls, fq = t32.export()
    assert t32.put(np.sort(keys), start[np.argsort(keys)], acc, ls, fq) == 2
    rng = np.random.default_rng(8)
    for step in range(1, 6):
        g = rng.standard_normal((2, D)).astype(np.float32)
        tb.apply_adam(keys, g, lr, step)
        t32.apply_adam(keys, g, lr, step)
    assert np.array_equal(tb.export_hot()[1][0], t32.lookup(keys[:1])[0])          # master == fp32 row, bit for bit
    cold = tb.lookup(keys[1:])[0]
    assert np.array_equal(cold, torch.from_numpy(cold).to(torch.bfloat16).float().numpy())   # cold row: 16-bit values
    assert not np.array_equal(cold, t32.lookup(keys[1:])[0])                        # and it did round on the way
