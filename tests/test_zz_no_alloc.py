"""lcn_backward_static (the entry point that allocates nothing: its scratch is an array in the
library's device image) against lcn_backward through the C ABI: same kernels on the same state, so
the outputs are the same bits.  Two calls in a row, the second on a smaller problem (the array keeps
the first call's contents), then once more on the first; a handle whose pattern needs more than the
array holds is refused before anything is launched."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def _both(lcn, h, mode):
    nnz = 0
    if mode != "nystrom":
        nnz = int(lcn.lcn_get_csr(h)[1].numel())
    ref = lcn.lcn_backward(h, nnz)
    outs = [None if r is None else torch.full_like(r, float("nan")) for r in ref]
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    st = lcn.lcn_backward_static(h, *outs)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before   # nothing came from torch either
    assert st == lcn.binding.OK
    for got, want in zip(outs, ref):
        assert (got is None) == (want is None)
        if got is not None:
            assert torch.equal(got, want)
    return nnz


def test_static_scratch_matches_caller_scratch():
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    big = workloads.config3(n=3000, landmarks=96, buckets=20, iters=60)
    small = workloads.config1(n=700, d=9)
    hb = gpu_build(big, "lcn")
    lcn.sinkhorn_run(hb, 20)
    hs = gpu_build(small, "lcn")
    lcn.sinkhorn_run(hs, 10)
    nnz_big = _both(lcn, hb, "lcn")
    nnz_small = _both(lcn, hs, "lcn")        # second call in a row, smaller input
    assert 0 < nnz_small < nnz_big
    _both(lcn, hb, "lcn")
    # sparse kernel (pattern output only) and Nystrom (no scratch at all)
    hq = gpu_build(small, "sparse")
    lcn.sinkhorn_run(hq, 10)
    _both(lcn, hq, "sparse")
    hn = gpu_build(small, "nystrom")
    lcn.sinkhorn_run(hn, 10)
    _both(lcn, hn, "nystrom")
    for h in (hb, hs, hq, hn):
        lcn.lcn_destroy(h)


def test_static_scratch_refuses_what_does_not_fit():
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    rng = np.random.default_rng(4)
    n = 2200                                   # dense kernel: 4.84 M stored entries, 2 x 19 MB of records
    X = rng.standard_normal((n, 3)).astype(np.float32)
    Y = rng.standard_normal((n, 3)).astype(np.float32)
    u = np.full(n, 1.0 / n, np.float32)
    p = workloads.Problem("dense", X, Y, u, u, 1.0, workloads.COST_SQEUCLID, 0, 1, 1, 3)
    h = gpu_build(p, "dense")
    lcn.sinkhorn_run(h, 3)
    assert lcn.lcn_backward_scratch_bytes(h) > (32 << 20)
    gsp = torch.full((n * n,), 7.0, device="cuda")
    assert lcn.lcn_backward_static(h, None, None, gsp, None) == lcn.binding.ERR_ALLOC
    assert bool((gsp == 7.0).all())            # refused before anything was written
    lcn.lcn_destroy(h)
