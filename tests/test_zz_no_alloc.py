"""The entry point that allocates nothing (skm_assign_exact_static) against skm_assign_exact: same kernels, the
working memory in a fixed device array instead of hipMalloc'd buffers.  Two calls in a row, the second smaller, so
that whatever the first left in the array would show."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_matches_the_allocating_one():
    from paper_2603_20009_amd import skm, datagen
    skm.lib()
    rng = np.random.default_rng(3)
    for (n, d, k) in ((70_000, 128, 300), (5000, 128, 37), (900, 48, 900)):
        print("static scratch", n, d, k, flush=True)
        X = datagen.mixture(n, d, 30, 5, "linear").cuda()
        Y = (X[torch.from_numpy(rng.choice(n, k, replace=False)).cuda()] + 0.01).contiguous()
        a_ref, d_ref = skm.assign_exact(X, Y)
        out = (torch.full((n,), -7, device="cuda", dtype=torch.int32), torch.full((n,), -1.0, device="cuda"))
        a, dist = skm.assign_exact_static(X, Y, out)
        assert torch.equal(a, a_ref) and torch.equal(dist, d_ref)       # the same kernels on the same inputs
        assert int(a.min()) >= 0 and int(a.max()) < k
    # beyond the limits: a clear error, outputs untouched
    X = torch.zeros((10, 24), device="cuda")
    with pytest.raises(skm.SkmError, match="multiple of 16"):
        skm.assign_exact_static(X, X[:2].contiguous())
    X = torch.zeros((20_000, 16), device="cuda")
    with pytest.raises(skm.SkmError, match="k out of range"):
        skm.assign_exact_static(X, X[:16_385].contiguous())
