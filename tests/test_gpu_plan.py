"""Rows of the transport plan from the HIP library (lcn_plan_rows): element by
element against the oracle's materialised plan, and the plan-quality measures of
the paper's accuracy table on its synthetic workload (uniform in the d-ball)."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["lcn", "nystrom", "sparse", "dense"])
def test_plan_rows_match_the_oracle(mode):
    import paper_2107_06876_amd as lcn
    from parity import gpu_build, oracle_run
    p = workloads.config1()
    iters = 30
    B, st, *_ = oracle_run(p, mode, iters=iters)
    K = B.op.dense()
    with np.errstate(over="ignore"):
        P = np.exp(st.log_u)[:, None] * K * np.exp(st.log_v)[None, :]
    h = gpu_build(p, mode)
    lcn.sinkhorn_run(h, iters)
    i0, nrows = 37, 613                      # a ragged block of rows
    got = lcn.lcn_plan_rows(h, i0, nrows).cpu().numpy().astype(np.float64)
    want = P[i0:i0 + nrows]
    scale = np.abs(want).max()
    err = np.abs(got - want) - 2e-4 * np.abs(want)
    assert err.max() <= 1e-6 * scale, (mode, err.max(), scale)
    full = lcn.lcn_plan_rows(h, 0, p.n)
    np.testing.assert_allclose(float(full.double().sum()), P.sum(), rtol=1e-5)
    lcn.lcn_destroy(h)


def _plan_metrics(h_approx, h_exact, n):
    """Pearson correlation of all plan entries and overlap (IoU) of the 0.1 % largest ones."""
    import torch
    import paper_2107_06876_amd as lcn
    Pa = lcn.lcn_plan_rows(h_approx, 0, n).flatten()
    Pe = lcn.lcn_plan_rows(h_exact, 0, n).flatten()
    x, y = Pa.double(), Pe.double()
    xm, ym = x.mean(), y.mean()
    pcc = float(((x - xm) * (y - ym)).sum() / torch.sqrt(((x - xm) ** 2).sum() * ((y - ym) ** 2).sum()))
    k = Pa.numel() // 1000
    ta = torch.topk(Pa, k).indices
    te = torch.topk(Pe, k).indices
    inter = int(torch.isin(ta, te).sum())
    return pcc, inter / (2 * k - inter)


def test_accuracy_table_on_the_dball_workload():
    """Sec. 8, Table 1, uniform in the d-ball (d = 16, n = 10^4, lambda = 0.05, 40 neighbours or
    landmarks in total): the paper reports, as relative error of the distance / PCC / IoU,
    Nystrom 1.837 / 0.073 / 0.018, sparse 0.241 / 0.341 / 0.090, LCN 0.435 / 0.328 / 0.079.
    Samples, landmarks and buckets differ from the paper's runs, so the plan measures are
    asserted to lie near those figures (measured here: 0.092 / 0.022, 0.407 / 0.116,
    0.402 / 0.103).  The relative error of the distance is only compared in its ORDER: the exact
    distance is a near-cancellation of transport cost and lambda H (0.069 for the unit ball), so its
    relative error scales with the radius of the ball, which the paper does not state."""
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    res = {}
    p = workloads.dball()
    hd = gpu_build(p, "dense")
    lcn.sinkhorn_run(hd, p.iters)
    d_exact = lcn.transport_cost(hd)
    for name, mode, kw in (("nystrom", "nystrom", dict(landmarks=40)), ("sparse", "sparse", dict(buckets=250)),
                           ("lcn", "lcn", dict())):
        q = workloads.dball(**kw)
        try:
            h = gpu_build(q, mode)
            lcn.sinkhorn_run(h, q.iters)
            status = "ok"
        except lcn.LcnError as e:   # Nystrom alone may produce non-positive sums (App. "Limitations")
            status = str(e)
            res[name] = (status,)
            continue
        d = lcn.transport_cost(h)
        pcc, iou = _plan_metrics(h, hd, q.n)
        res[name] = (abs(d - d_exact) / abs(d_exact), pcc, iou)
        lcn.lcn_destroy(h)
    print("d-ball accuracy (rel. err., PCC, IoU):", res, "exact distance", d_exact, flush=True)
    rel, pcc, iou = res["lcn"]
    assert 0.2 < pcc < 0.55 and 0.05 < iou < 0.16
    rel_s, pcc_s, iou_s = res["sparse"]
    assert 0.2 < pcc_s < 0.55 and 0.05 < iou_s < 0.16
    assert rel_s < rel
    if len(res["nystrom"]) == 3:   # Nystrom alone: far behind on the plan, worst on the distance
        rel_n, pcc_n, iou_n = res["nystrom"]
        assert 0.03 < pcc_n < 0.15 and 0.008 < iou_n < 0.04
        assert rel < rel_n
    lcn.lcn_destroy(hd)


@pytest.mark.parametrize("name", ["config1", "config2"])
def test_plan_measures_on_configs_1_and_2(name):
    """PCC and IoU of the 0.1 % largest entries of the LCN plan against the dense plan (the other two
    columns of the accuracy table, Sec. 8) on configurations 1 and 2, through lcn_plan_rows.  Config 2
    at 0.5 x median (at its own lambda the LCN path reports non-positive sums).  Measured: config 1
    0.966 / 0.41, config 2 0.991 / 0.65; the clustered inputs are what the approximation is made for
    (Sec. 4, Thm. 2), so both sit far above the d-ball figures."""
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    p = workloads.config1() if name == "config1" else workloads.config2(lam_factor=0.5)
    hd = gpu_build(p, "dense")
    lcn.sinkhorn_run(hd, p.iters)
    hl = gpu_build(p, "lcn")
    lcn.sinkhorn_run(hl, p.iters)
    pcc, iou = _plan_metrics(hl, hd, p.n)
    rel = abs(lcn.transport_cost(hl) - lcn.transport_cost(hd)) / abs(lcn.transport_cost(hd))
    print("plan measures", name, "rel. err.", rel, "PCC", pcc, "IoU", iou, flush=True)
    assert pcc > 0.93 and iou > 0.3 and rel < 0.01
    lcn.lcn_destroy(hl)
    lcn.lcn_destroy(hd)
