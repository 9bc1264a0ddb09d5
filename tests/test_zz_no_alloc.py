"""The entry point that allocates nothing (mar_rank_metrics_static: partial sums in an array built into the
library) against the entry point it is a variant of (mar_rank_metrics: partial sums in the context's
workspace), through the C ABI: equal bits, two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar

pytestmark = pytest.mark.gpu


def test_static_scratch_metrics_equal_the_workspace_metrics():
    dev = torch.device("cuda:0")
    tr = mar.Trainer(100, 2, 8, mar.MODEL_DISTMULT, 16, 2, 8, device=dev)        # any context: it only lends its workspace
    rng = np.random.default_rng(11)
    ks = [1, 3, 10, 50]
    big = torch.from_numpy(rng.integers(1, 1001, 300_000).astype(np.int32)).to(dev)      # 74 partial records, ragged last tile
    small = torch.from_numpy(rng.integers(1, 60, 5_000).astype(np.int32)).to(dev)        # 2 records: stale ones stay behind
    for ranks in (big, small):
        want = torch.full((1 + len(ks),), -1.0, dtype=torch.float64, device=dev)
        got = torch.full((1 + len(ks),), -2.0, dtype=torch.float64, device=dev)
        mar.mar_rank_metrics(tr.ctx, ranks, ranks.numel(), ks, want)
        mar.mar_rank_metrics_static(ranks, ranks.numel(), ks, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (got, want)
        # and both are the plain definition
        r = ranks.cpu().numpy().astype(np.float64)
        ref = np.array([np.mean(1.0 / r)] + [np.mean(r <= k) for k in ks])
        assert np.allclose(got.cpu().numpy(), ref, rtol=1e-12, atol=0)
    # empty input writes zeros; sizes beyond the built-in array are refused before anything is enqueued
    out = torch.full((2,), 7.0, dtype=torch.float64, device=dev)
    mar.mar_rank_metrics_static(None, 0, [5], out)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [0.0, 0.0]
    with pytest.raises(mar.MarError) as ei:
        mar.mar_rank_metrics_static(big, 4096 * 4096 + 1, ks, out)
    assert ei.value.code == -2 and "scratch" in str(ei.value)
    tr.close()
