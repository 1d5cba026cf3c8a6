"""The allocation-free entry point emb_dedup_noalloc against emb_dedup (needs an MI355X): same results bit for bit,
on two calls in a row, the second with a smaller input; sizes beyond its fixed scratch are refused."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2505_12663_amd import binding as B
    from harness import dev_keys


def _both(keys):
    n = len(keys)
    d = dev_keys(keys)
    outs = []
    for noalloc in (False, True):
        uniq = torch.full((n,), -1, dtype=torch.int64, device="cuda")
        inverse = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        counts = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        seg_off = torch.full((n + 1,), -1, dtype=torch.int32, device="cuda")
        seg_of = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        n_unique = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        if noalloc:
            B.emb_dedup_noalloc(d, n, uniq, inverse, counts, perm, seg_off, seg_of, n_unique)
        else:
            ws = torch.empty(B.emb_dedup_workspace_bytes(n), dtype=torch.uint8, device="cuda")
            B.emb_dedup(d, n, uniq, inverse, counts, perm, seg_off, seg_of, n_unique, ws)
        U = int(n_unique.item())
        outs.append((U, uniq[:U].cpu(), inverse.cpu(), counts[:U].cpu(), perm.cpu(), seg_off[:U + 1].cpu(), seg_of.cpu()))
    return outs


def test_noalloc_dedup_equals_dedup_on_two_calls_in_a_row():
    rng = np.random.default_rng(12)
    for n, vocab in ((300_000, 70_000), (9_001, 2_500)):          # several tiles and a ragged tail, then a smaller input
        keys = (rng.zipf(1.2, size=n) % vocab).astype(np.uint64) * np.uint64(0x9E3779B1) | np.uint64(3 << 59)
        a, b = _both(keys)
        assert a[0] == b[0] and 0 < a[0] < n
        for x, y in zip(a[1:], b[1:]):
            assert torch.equal(x, y)


def test_noalloc_dedup_refuses_sizes_beyond_its_scratch():
    n = B.EMB_DEDUP_NOALLOC_MAX_KEYS + 1
    key = torch.zeros(n, dtype=torch.int64, device="cuda")
    out = torch.empty(n, dtype=torch.int64, device="cuda")
    i32 = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    nu = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(B.EmbError) as e:
        B.emb_dedup_noalloc(key, n, out, i32, None, i32, None, i32, nu)
    assert e.value.status == B.EMB_ERR_TOO_LARGE
    # the largest admitted size works
    n = B.EMB_DEDUP_NOALLOC_MAX_KEYS
    B.emb_dedup_noalloc(key[:n], n, out, i32, None, None, None, None, nu)
    assert int(nu.item()) == 1 and int(out[0].item()) == 0 and bool((i32[:n] == 0).all())
