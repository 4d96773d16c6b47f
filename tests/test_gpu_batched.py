"""GPU parity of the batched small-problem path (config 4: many graph-pair
sized problems with deletion rows/columns, Sec. 6) against the oracle, pair by
pair."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu


def _oracle_pair(B, p, mode, bp=True):
    Xp = B.X[B.x_off[p]:B.x_off[p + 1]]
    Yp = B.Y[B.y_off[p]:B.y_off[p + 1]]
    n, m = len(Xp), len(Yp)
    lam = float(B.lam[p])
    Bl = oracle.build_problem(Xp, Yp, B.cost, lam, mode, B.num_landmarks, B.landmark_seed + p, B.kmeans_iters,
                              B.ridge, 0, B.num_buckets, 1, B.lsh_seed + p)
    if bp:
        kpe = np.exp(-B.del_x[B.x_off[p]:B.x_off[p + 1]].astype(np.float64) / lam)
        keq = np.exp(-B.del_y[B.y_off[p]:B.y_off[p + 1]].astype(np.float64) / lam)
        a = np.full(n + m, 1.0 / (n + m))
        st = oracle.sinkhorn_bp(Bl.op, kpe, keq, a, a, B.iters)
        _, _, dist, resid = oracle.marginals_bp(Bl.op, kpe, keq, a, a, lam, st)
    else:
        a, b = np.full(n, 1.0 / n), np.full(m, 1.0 / m)
        st = oracle.sinkhorn(Bl.op, a, b, B.iters)
        _, _, dist, resid = oracle.marginals(Bl.op, a, b, lam, st)
    return Bl, st, dist, resid


def _run_gpu(B, mode, bp=True):
    import paper_2107_06876_amd as lcn
    dev = "cuda:0"
    modes = {"dense": lcn.MODE_DENSE, "sparse": lcn.MODE_SPARSE, "nystrom": lcn.MODE_NYSTROM, "lcn": lcn.MODE_LCN}
    X = torch.from_numpy(B.X).to(dev)
    Y = torch.from_numpy(B.Y).to(dev)
    dx = torch.from_numpy(B.del_x).to(dev) if bp else None
    dy = torch.from_numpy(B.del_y).to(dev) if bp else None
    lm = dict(num_landmarks=B.num_landmarks, kmeans_iters=B.kmeans_iters, seed=B.landmark_seed, ridge=B.ridge)
    lsh = dict(num_buckets=B.num_buckets, num_rounds=1, kmeans_iters=B.kmeans_iters, seed=B.lsh_seed)
    h = lcn.lcn_build_batched(X, Y, B.x_off, B.y_off, B.lam, B.cost, modes[mode], dx, dy,
                              landmarks=lm if mode in ("lcn", "nystrom") else None,
                              lsh=lsh if mode in ("lcn", "sparse") else None)
    lcn.sinkhorn_run(h, B.iters)
    dist, resid = lcn.lcn_batched_results(h)
    st = lcn.lcn_batched_get(h)
    return h, dist, resid, {k: v.cpu().numpy() for k, v in st.items()}


@pytest.mark.parametrize("mode,bp", [("lcn", True), ("dense", True), ("lcn", False), ("nystrom", True)])
def test_config4(mode, bp):
    B = workloads.config4(pairs=192 if mode == "lcn" and bp else 64)
    h, dist, resid, st = _run_gpu(B, mode, bp)
    worst = dict(log=0.0, cost=0.0, resid=0.0)
    for p in range(B.num_problems):
        Bl, so, dist_o, resid_o = _oracle_pair(B, p, mode, bp)
        n = int(B.x_off[p + 1] - B.x_off[p])
        m = int(B.y_off[p + 1] - B.y_off[p])
        z0 = int(B.x_off[p] + B.y_off[p])
        lu = st["log_u"][z0:z0 + (n + m if bp else n)]
        lv = st["log_v"][z0:z0 + (n + m if bp else m)]
        assert so.nonpositive == 0
        if mode in ("lcn", "nystrom"):
            np.testing.assert_array_equal(st["landmarks"][p], Bl.landmarks)
        if mode == "lcn":
            np.testing.assert_array_equal(st["buckets"][z0:z0 + n + m], Bl.buckets[0])
        np.testing.assert_allclose(st["kernel"][p][:n, :m], Bl.op.dense(), rtol=2e-6, atol=1e-30)
        worst["log"] = max(worst["log"], np.abs(lu - so.log_u).max(), np.abs(lv - so.log_v).max())
        worst["cost"] = max(worst["cost"], abs(dist[p] - dist_o) / abs(dist_o))
        worst["resid"] = max(worst["resid"], abs(resid[p] - resid_o))
    print("C4", mode, bp, worst, flush=True)
    assert worst["log"] <= 1e-4 and worst["cost"] <= 1e-4 and worst["resid"] <= 1e-5, worst
