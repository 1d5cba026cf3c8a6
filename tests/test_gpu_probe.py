"""The memory-probe entry point (a measuring aid): its stores are what the header says, so that the rates bench.py
derives from it are rates of the stated access patterns."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2505_12663_amd import binding as B      # noqa: E402


@pytest.mark.parametrize("with_index", [False, True])
def test_probe_patterns_store_what_the_header_says(with_index):
    rows = 64 * 37
    g = torch.Generator(device="cuda").manual_seed(3)
    src = torch.randint(-8, 9, (rows, 64), generator=g, device="cuda").to(torch.float32)     # integer-valued: sums are exact
    idx = torch.randperm(rows, generator=g, device="cuda").to(torch.int32) if with_index else None
    order = idx.long() if with_index else torch.arange(rows, device="cuda")
    # write-only: row idx[r] holds r
    dst = torch.full((rows, 64), -1.0, device="cuda")
    B.emb_probe_memory(B.PROBE_WRITE, None, dst, idx, rows)
    want = torch.empty_like(dst)
    want[order] = torch.arange(rows, device="cuda", dtype=torch.float32)[:, None].expand(rows, 64)
    assert torch.equal(dst, want)
    # reads with one stored row per 4 and per 64 read
    for pattern, every in ((B.PROBE_READ_STORE_4TH, 4), (B.PROBE_READ_STORE_64TH, 64)):
        out = torch.full((rows // every, 64), -1.0, device="cuda")
        B.emb_probe_memory(pattern, src, out, idx, rows)
        assert torch.equal(out, src[order].view(rows // every, every, 64).sum(dim=1))
    # reads only: nothing is written
    guard = torch.full((4, 64), 7.0, device="cuda")
    B.emb_probe_memory(B.PROBE_READ, src, guard, idx, rows)
    torch.cuda.synchronize()
    assert bool((guard == 7.0).all())


def test_probe_rejects_bad_arguments():
    buf = torch.zeros((64, 64), device="cuda")
    for rows in (0, 63, -64):
        with pytest.raises(B.EmbError):
            B.emb_probe_memory(B.PROBE_WRITE, None, buf, None, rows)
    with pytest.raises(B.EmbError):
        B.emb_probe_memory(9, buf, buf, None, 64)
    with pytest.raises(B.EmbError):
        B.emb_probe_memory(B.PROBE_READ, None, buf, None, 64)
