"""Analytic derivatives of the distance (Prop. 1) from the HIP library against
the oracle, element by element: the factor parts (n x l and m x l) and the
pattern parts in the order of the canonical CSR.  Both sides differentiate at
their own scalings after the same number of iterations; the scalings agree to
1e-4 in the logs (the parity bound), so products u_i v_j agree to about twice
that: |g_gpu - g_oracle| <= 2e-4 |g_oracle| + 1e-5 max |g_oracle|."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


def _close(g_gpu, g_or, what):
    g_gpu = g_gpu.cpu().numpy().astype(np.float64)
    assert g_gpu.shape == g_or.shape, what
    scale = np.abs(g_or).max()
    err = np.abs(g_gpu - g_or) - 2e-4 * np.abs(g_or)
    assert err.max() <= 1e-5 * scale, "%s: worst %g of scale %g" % (what, err.max(), scale)
    return float(np.abs(g_gpu - g_or).max() / scale)


def _run(p, mode, iters):
    import paper_2107_06876_amd as lcn
    from parity import gpu_build, oracle_run
    B, st, *_ = oracle_run(p, mode, iters=iters)
    op = B.op
    ksp = knys = None
    if mode in ("sparse", "lcn"):
        ksp = oracle.pattern_values(p.X, p.Y, p.cost, p.lam, op.rowptr, op.colidx)
    if mode == "lcn":
        knys = oracle.pattern_values(p.X, p.Y, p.cost, p.lam, op.rowptr, op.colidx, op.U, op.W, nystrom_only=True)
    if mode == "dense":   # the dense kernel as a full pattern
        n, m = op.n, op.m
        rowptr = (np.arange(n + 1) * m).astype(np.int64)
        colidx = np.tile(np.arange(m), n).astype(np.int32)
        ksp = op.Kd.ravel()
        op = oracle.Operator(n, m, rowptr=rowptr, colidx=colidx, val=ksp)
    gU, gW, gsp, gnys = oracle.backward(op, p.lam, st, ksp, knys)
    h = gpu_build(p, mode)
    lcn.sinkhorn_run(h, iters)
    nnz = 0
    if mode != "nystrom":
        rowptr_g, colidx_g, _ = lcn.lcn_get_csr(h)
        np.testing.assert_array_equal(colidx_g.cpu().numpy(), op.colidx)
        nnz = int(colidx_g.numel())
    hU, hWt, hsp, hnys = lcn.lcn_backward(h, nnz)
    out = {}
    if gU is not None:
        out["gU"] = _close(hU, gU, "gU")
        out["gW"] = _close(hWt, np.ascontiguousarray(gW.T), "gW^T")
    else:
        assert hU is None and hWt is None
    if gsp is not None:
        out["gsp"] = _close(hsp, gsp, "gsp")
    if gnys is not None:
        out["gnys"] = _close(hnys, gnys, "gnys")
        assert float(hnys.min()) >= 0.0 or float(hnys.abs().max()) > 0   # present and signed as derived
    else:
        assert hnys is None
    lcn.lcn_destroy(h)
    print(p.name, mode, out, flush=True)
    return out


@pytest.mark.parametrize("mode", ["lcn", "nystrom", "sparse", "dense"])
def test_backward_config1(mode):
    _run(workloads.config1(), mode, 50)


def test_backward_three_rounds_with_long_segments():
    p = workloads.config3(n=3000, d=48, landmarks=96, buckets=12, rounds=3, iters=40, name="C3 reduced")
    _run(p, "lcn", 40)


def test_backward_requests_that_do_not_exist_are_refused():
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    h = gpu_build(workloads.config1(), "nystrom")
    lcn.sinkhorn_run(h, 3)
    g = torch.empty(16, dtype=torch.float32, device="cuda:0")
    lib = lcn.load_library()
    import ctypes
    st = lib.lcn_backward(h.raw, None, None, ctypes.c_void_p(g.data_ptr()), None, None, 0)
    assert st == lcn.binding.ERR_STATE
    lcn.lcn_destroy(h)


@pytest.mark.parametrize("shape,mode", [((300, 200, 5, 7, 3, 6), "lcn"), ((300, 200, 5, 7, 3, 6), "sparse"),
                                        ((1, 1, 1, 1, 1, 1), "lcn"), ((1, 1, 1, 1, 1, 1), "dense"),
                                        ((40, 2600, 4, 5, 1, 1), "lcn"), ((129, 127, 64, 33, 5, 5), "lcn"),
                                        ((2, 130, 2, 3, 1, 8), "sparse")])
def test_backward_edge_shapes(shape, mode):
    """Derivatives and the CSR export behind them on the smallest and most ragged shapes: a single
    pair, six and eight hash rounds, and rows of 2600 entries (longer than the 2048 a wavefront
    ranks in LDS, so the serial merge takes them)."""
    from test_gpu_parity import _edge_problem
    _run(_edge_problem(*shape), mode, 15)
