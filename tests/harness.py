"""Side-by-side driver: the same seeded step through the HIP library and through the CPU checker."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2505_12663_amd import binding as B
from paper_2505_12663_amd import EmbeddingTable, StepBuffers, forward, forward_two_call, backward

RTOL_F32 = 1e-5     # reduced gradients and updated rows, fp32 tables
RTOL_BF16 = 1e-2    # bf16 tables


def dev_keys(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()


def host_keys(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def close_reduce(got: np.ndarray, ref: np.ndarray, sabs: np.ndarray, rtol: float) -> bool:
    """|a-b| <= rtol*|b| + rtol*sum|addends|: a plain relative error is meaningless for sums that cancel."""
    return bool((np.abs(got.astype(np.float64) - ref) <= rtol * np.abs(ref) + rtol * sabs).all())


def close_rows(got: np.ndarray, ref: np.ndarray, lr: float, rtol: float) -> bool:
    """|a-b| <= rtol*max(|b|, lr): one optimizer step moves an element by at most ~lr."""
    return bool((np.abs(got.astype(np.float64) - ref) <= rtol * np.maximum(np.abs(ref), lr)).all())


class Pair:
    """One merged table on both sides."""

    def __init__(self, dim, dtype=B.F32, capacity_log2=18, chunk_rows_log2=16, max_load_factor=0.75,
                 count_probes=True, init_scale=0.01):
        self.dim, self.dtype = dim, dtype
        self.gpu = EmbeddingTable(dim, dtype, capacity_log2, chunk_rows_log2, init_scale, max_load_factor, count_probes)
        self.orc = oracle.Table(dim, dtype, init_scale)
        self.rtol = RTOL_F32 if dtype == B.F32 else RTOL_BF16

    def compare_tables(self, lr, exact_rows_when_untouched=True):
        gk, gv, ga, gl, gf = self.gpu.export()
        ok, ov, oa, ol, of = self.orc.export()
        assert np.array_equal(gk, ok), "key sets differ"
        assert np.array_equal(gl, ol), "last_seen differs"
        assert np.array_equal(gf, of), "freq differs"
        assert close_rows(gv, ov.astype(np.float64), lr, self.rtol), float(np.abs(gv - ov).max())
        assert np.allclose(ga, oa, rtol=RTOL_F32, atol=1e-12), float(np.abs(ga - oa).max())   # the accumulator is fp32 whatever the table dtype
        if exact_rows_when_untouched:
            never = oa == 0
            assert np.array_equal(gv[never], ov[never]), "rows never updated must be bit-identical"
            assert (ga[never] == 0).all()
        return len(gk)


def run_step(pair: Pair, buf: StepBuffers, x: np.ndarray, field_off: np.ndarray, field_tag: np.ndarray,
             tag_bits: int, step: int, G: np.ndarray, lr: float, eps: float, prepopulated_keys=None,
             one_record_update: bool = False, id_bits=None, two_call: bool = False):
    """One forward+backward on both sides; asserts the parity bar and returns (N, U).
    one_record_update: the HIP side looks keys up without touching them and lets the update count the
    touch; the checker keeps touching in the lookup - after the step both must be in the same state."""
    n = len(x)
    # ---- checker
    okey, oerr = oracle.tag_keys(x, field_off, field_tag, tag_bits)
    ouniq, oinv, ocnt = oracle.dedup(okey)
    if prepopulated_keys is not None:
        pair.orc.prepopulate(prepopulated_keys(ouniq))
    oins = pair.orc.find_or_insert(ouniq, step)
    oE_u = pair.orc.lookup(ouniq)
    _, _, oacc_before, _, _ = pair.orc.peek(ouniq)
    oE = oracle.expand(oE_u, oinv)
    og = oracle.segment_reduce(G, oinv, len(ouniq))
    osabs = oracle.segment_reduce(np.abs(G), oinv, len(ouniq)).astype(np.float64)
    pair.orc.apply_adagrad(ouniq, og, lr, eps)
    # ---- HIP path
    dx, doff, dtag = dev_keys(x), torch.from_numpy(field_off).cuda(), torch.from_numpy(field_tag).cuda()
    if two_call:
        forward_two_call(pair.gpu, buf, dx, doff, dtag, tag_bits, step, touch=not one_record_update)
    else:
        forward(pair.gpu, buf, dx, doff, dtag, tag_bits, step, touch=not one_record_update, id_bits=id_bits)
    U = int(buf.n_unique.item())
    assert int(buf.err_count.item()) == oerr
    assert np.array_equal(host_keys(buf.key[:n]), okey), "tagged keys"
    assert U == len(ouniq), (U, len(ouniq))
    assert np.array_equal(host_keys(buf.uniq[:U]), ouniq), "unique keys"
    assert np.array_equal(buf.inverse[:n].cpu().numpy(), oinv), "inverse"
    assert np.array_equal(buf.counts[:U].cpu().numpy(), ocnt), "counts"
    assert np.array_equal(buf.inserted[:U].cpu().numpy(), oins), "inserted flags"
    E_u = buf.uniq_rows[:U].float().cpu().numpy()
    E = buf.out[:n].float().cpu().numpy()
    assert np.array_equal(E, E_u[oinv]), "expand must copy rows bit for bit"
    never = oacc_before == 0                       # rows no optimizer step has touched yet
    assert np.array_equal(E_u[never], oE_u[never]), "rows never updated must be bit-identical"
    assert close_rows(E_u, oE_u.astype(np.float64), lr, pair.rtol), "gathered rows"
    assert close_rows(E, oE.astype(np.float64), lr, pair.rtol), "forward embeddings"
    if pair.dtype == B.F32:
        dG = torch.from_numpy(G).cuda()
    else:
        dG = torch.from_numpy(G).cuda().to(torch.bfloat16)     # G is bf16-representable: exact
    backward(pair.gpu, buf, dG, n, lr, eps, touch_step=step if one_record_update else None)
    g = buf.reduced[:U].cpu().numpy()
    assert close_reduce(g, og.astype(np.float64), osabs, RTOL_F32), "reduced gradients"
    return n, U


def small_int_rows(pos: np.ndarray, dim: int, seed: int) -> np.ndarray:
    """Rows `pos` of workloads.small_int_grads(n, dim, seed) without materialising the whole matrix
    (same integer formula, evaluated with numpy on the requested rows only)."""
    i = pos.astype(np.int64)[:, None]
    j = np.arange(dim, dtype=np.int64)[None, :]
    h = (i * 2654435761 + j * 40503 + (seed & 0xFFFF) * 97) & 0x7FFFFFFF
    h = ((h ^ (h >> 13)) * 1274126177) & 0x7FFFFFFF
    return ((h >> 9) % 17 - 8).astype(np.float32)


def tracked_subset(hot_keys: np.ndarray):
    """Predicate choosing the keys the checker mirrors at full size: a fixed 1/512 of the key space
    (by a multiplicative hash of the key, so the choice is the same in every step) plus a given set
    of hot keys.  Because membership depends on the key alone, the checker's table is an exact mirror
    of the device table restricted to these keys, across any number of steps."""
    hot = np.sort(np.asarray(hot_keys, dtype=np.uint64))

    def tracked(keys: np.ndarray) -> np.ndarray:
        h = (keys * np.uint64(0x9E3779B97F4A7C15)) >> np.uint64(55)
        return (h == 0) | np.isin(keys, hot)
    return tracked


def run_step_sampled(pair: Pair, buf: StepBuffers, x, field_off, field_tag, tag_bits, step, lr, eps, grad_seed,
                     is_prepopulated, tracked, rng_seed=0, id_bits=None):
    """One full-size forward+backward on the GPU; the checker does the integer work in full (tag, dedup)
    and the row work on the tracked subset of distinct keys: insert flags, gathered rows, expanded rows,
    exact integer-valued reduced gradients, updated rows."""
    from workloads import small_int_grads
    n = len(x)
    okey, oerr = oracle.tag_keys(x, field_off, field_tag, tag_bits)
    ouniq, oinv, ocnt = oracle.dedup(okey)
    U = len(ouniq)
    rng = np.random.default_rng(rng_seed + step)
    pick = np.flatnonzero(tracked(ouniq))
    skeys = ouniq[pick]
    pre = is_prepopulated(skeys)
    pair.orc.prepopulate(skeys[pre])
    # ---- HIP path, forward
    dx, doff, dtag = dev_keys(x), torch.from_numpy(field_off).cuda(), torch.from_numpy(field_tag).cuda()
    forward(pair.gpu, buf, dx, doff, dtag, tag_bits, step, id_bits=id_bits)
    assert int(buf.n_unique.item()) == U and int(buf.err_count.item()) == oerr
    assert np.array_equal(host_keys(buf.uniq[:U]), ouniq), "unique keys"
    assert np.array_equal(buf.inverse[:n].cpu().numpy(), oinv), "inverse"
    assert np.array_equal(buf.counts[:U].cpu().numpy(), ocnt), "counts"
    ins = buf.inserted[:U].cpu().numpy()
    oins = pair.orc.find_or_insert(skeys, step)
    assert np.array_equal(ins[pick], oins), "inserted flags (sample)"
    dpick = torch.from_numpy(pick).cuda()
    oE_u = pair.orc.lookup(skeys)
    _, _, oacc_before, _, _ = pair.orc.peek(skeys)
    E_u = buf.uniq_rows[dpick].float().cpu().numpy()
    never = oacc_before == 0
    assert np.array_equal(E_u[never], oE_u[never]), "rows never updated must be bit-identical"
    assert close_rows(E_u, oE_u.astype(np.float64), lr, pair.rtol), "gathered rows (sample)"
    pos = rng.integers(0, n, size=20000)
    E = buf.out[torch.from_numpy(pos).cuda()].cpu()
    assert torch.equal(E, buf.uniq_rows[torch.from_numpy(oinv[pos].astype(np.int64)).cuda()].cpu()), "expand (sample)"
    # ---- backward with integer-valued gradients: exactly one correct fp32 sum per element
    dG = small_int_grads(n, pair.dim, grad_seed, "cuda")
    if pair.dtype != B.F32:
        dG = dG.to(torch.bfloat16)
    backward(pair.gpu, buf, dG, n, lr, eps)
    order = np.argsort(oinv, kind="stable")
    seg_off = np.concatenate([[0], np.cumsum(ocnt)])
    og = np.zeros((len(pick), pair.dim), dtype=np.float32)
    for s, u in enumerate(pick):
        p = order[seg_off[u]:seg_off[u + 1]]
        og[s] = small_int_rows(p, pair.dim, grad_seed).astype(np.float64).sum(0).astype(np.float32)
    g = buf.reduced[dpick].cpu().numpy()
    assert np.array_equal(g, og), "reduced gradients (sample, exact)"
    pair.orc.apply_adagrad(skeys, og, lr, eps)
    rows_after = torch.empty((len(pick), pair.dim), dtype=buf.uniq_rows.dtype, device="cuda")
    pair.gpu.gather(buf.row_idx[dpick].contiguous(), None, len(pick), rows_after)
    assert close_rows(rows_after.float().cpu().numpy(), pair.orc.lookup(skeys).astype(np.float64), lr, pair.rtol), "updated rows"
    return n, U, int(ins.sum())


def check_reduce_normal_sampled(buf: StepBuffers, okey: np.ndarray, dim: int, dtype: int, tracked, seed: int) -> int:
    """Full-size gradient reduction of N(0,1) gradients (rounded to bf16 for bf16 tables) over the segments that
    buf.seg_of / buf.perm describe, compared on the tracked distinct keys with the checker's fp64 sums in input
    order, within the bound for reductions (1e-5 of |sum| plus 1e-5 of the sum of |addends|).  Returns the number
    of segments compared.  The gradient matrix is drawn on the device (an input, not part of the method)."""
    n = len(okey)
    gen = torch.Generator(device="cuda").manual_seed(seed)
    G = torch.randn((n, dim), generator=gen, device="cuda", dtype=torch.float32)
    if dtype != B.F32:
        G = G.to(torch.bfloat16)
    B.grad_segment_reduce(G, dtype, buf.seg_of, buf.perm, n, dim, buf.reduced, buf.reduce_ws)
    U = int(buf.n_unique.item())
    pos = np.flatnonzero(tracked(okey))
    skeys, sinv = np.unique(okey[pos], return_inverse=True)
    sidx = np.searchsorted(host_keys(buf.uniq[:U]), skeys)
    Gs = G[torch.from_numpy(pos).cuda()].float().cpu().numpy()
    ref = oracle.segment_reduce(Gs, sinv.astype(np.int32), len(skeys))
    sabs = oracle.segment_reduce(np.abs(Gs), sinv.astype(np.int32), len(skeys)).astype(np.float64)
    got = buf.reduced[torch.from_numpy(sidx).cuda()].cpu().numpy()
    assert close_reduce(got, ref.astype(np.float64), sabs, RTOL_F32), "reduced N(0,1) gradients (tracked segments)"
    return len(skeys)
