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
    status = lcn.sinkhorn_run(h, B.iters, check=False)
    dist, resid = lcn.lcn_batched_results(h)
    st = lcn.lcn_batched_get(h)
    st = {k: v.cpu().numpy() for k, v in st.items()}
    st["status"] = status
    st["counts"] = lcn.lcn_last_error_counts(h)
    return h, dist, resid, st


@pytest.mark.parametrize("mode,bp", [("lcn", True), ("dense", True), ("lcn", False), ("nystrom", True),
                                     ("sparse", True), ("sparse", False), ("dense", False)])
def test_config4(mode, bp):
    """All 1024 pairs of the configuration (Sec. 6 workload), every pair against the oracle's run of
    the same pair.  Without deletion entries the sparse kernel of a pair often has points whose
    bucket holds no point of the other set (4 buckets over 16..64 points): those get scaling 0 on
    both sides, are counted, and the call returns the warning status (App. "Limitations")."""
    import paper_2107_06876_amd as lcn
    B = workloads.config4()
    assert B.num_problems == 1024
    h, dist, resid, st = _run_gpu(B, mode, bp)
    worst = dict(log=0.0, cost=0.0, resid=0.0)
    counts_o = np.zeros(3, dtype=np.int64)
    for p in range(B.num_problems):
        Bl, so, dist_o, resid_o = _oracle_pair(B, p, mode, bp)
        n = int(B.x_off[p + 1] - B.x_off[p])
        m = int(B.y_off[p + 1] - B.y_off[p])
        z0 = int(B.x_off[p] + B.y_off[p])
        lu = st["log_u"][z0:z0 + (n + m if bp else n)]
        lv = st["log_v"][z0:z0 + (n + m if bp else m)]
        assert so.nonpositive == 0
        counts_o += (so.nonpositive, so.empty_rows, so.empty_cols)
        if mode in ("lcn", "nystrom"):
            np.testing.assert_array_equal(st["landmarks"][p], Bl.landmarks)
        if mode in ("lcn", "sparse"):
            np.testing.assert_array_equal(st["buckets"][z0:z0 + n + m], Bl.buckets[0])
        np.testing.assert_allclose(st["kernel"][p][:n, :m], Bl.op.dense(), rtol=2e-6, atol=1e-30)
        fu, fv = np.isfinite(so.log_u), np.isfinite(so.log_v)
        np.testing.assert_array_equal(np.isfinite(lu), fu)       # unsupported points: -infinity on both sides
        np.testing.assert_array_equal(np.isfinite(lv), fv)
        assert np.all(lu[~fu] == -np.inf) and np.all(lv[~fv] == -np.inf)
        worst["log"] = max(worst["log"], np.abs(lu - so.log_u)[fu].max(initial=0.0),
                           np.abs(lv - so.log_v)[fv].max(initial=0.0))
        worst["cost"] = max(worst["cost"], abs(dist[p] - dist_o) / abs(dist_o))
        worst["resid"] = max(worst["resid"], abs(resid[p] - resid_o))
    print("C4", mode, bp, worst, "status", st["status"], "counts", st["counts"], flush=True)
    assert worst["log"] <= 1e-4 and worst["cost"] <= 1e-4 and worst["resid"] <= 1e-5, worst
    assert st["counts"] == tuple(int(c) for c in counts_o)
    want = lcn.binding.WARN_NO_SUPPORT if counts_o[1] + counts_o[2] else lcn.binding.OK
    assert st["status"] == want
    if mode == "sparse" and not bp:
        assert counts_o[1] > 0 and counts_o[2] > 0    # the case this configuration exists to cover


def test_deletion_costs_bitwise():
    """c_i = || alpha .* x_i ||_2 (Sec. 6): same fp64 operations in the same order on both sides."""
    import paper_2107_06876_amd as lcn
    rng = np.random.default_rng(11)
    for total, d in ((1, 1), (257, 32), (5000, 64), (300, 301)):
        X = rng.standard_normal((total, d)).astype(np.float32)
        alpha = rng.uniform(0.5, 1.5, d).astype(np.float32)
        got = lcn.lcn_deletion_costs(torch.from_numpy(X).cuda(), torch.from_numpy(alpha).cuda()).cpu().numpy()
        np.testing.assert_array_equal(got, oracle.deletion_costs(X, alpha))
    empty = lcn.lcn_deletion_costs(torch.empty((0, 8), device="cuda"), torch.ones(8, device="cuda"))
    assert empty.numel() == 0


def test_multi_head_unbalanced():
    """Multi-head OT with learnable deletion costs (Sec. 6): every (pair, head) is a problem of
    the batch with lambda_k = 2^(k - K/2) lambda and c = || alpha_k .* x ||_2; the K distances
    of every pair against the oracle's."""
    import paper_2107_06876_amd as lcn
    H = workloads.config4_heads(pairs=40, heads=4)
    B, K = H.batch, H.heads
    P = B.num_problems
    dev = "cuda:0"
    X = torch.from_numpy(B.X).to(dev)
    Y = torch.from_numpy(B.Y).to(dev)
    lam = np.concatenate([lcn.lcn_head_lambdas(float(l0), K) for l0 in H.base_lam])
    dx = torch.empty(X.shape[0], dtype=torch.float32, device=dev)
    dy = torch.empty(Y.shape[0], dtype=torch.float32, device=dev)
    for q in range(P):                                    # one head's rows at a time
        a = torch.from_numpy(H.alpha[H.head_of[q]]).to(dev)
        lcn.lcn_deletion_costs(X[B.x_off[q]:B.x_off[q + 1]], a, out=dx[B.x_off[q]:B.x_off[q + 1]])
        lcn.lcn_deletion_costs(Y[B.y_off[q]:B.y_off[q + 1]], a, out=dy[B.y_off[q]:B.y_off[q + 1]])
    lm = dict(num_landmarks=B.num_landmarks, kmeans_iters=B.kmeans_iters, seed=B.landmark_seed, ridge=B.ridge)
    lsh = dict(num_buckets=B.num_buckets, num_rounds=1, kmeans_iters=B.kmeans_iters, seed=B.lsh_seed)
    h = lcn.lcn_build_batched(X, Y, B.x_off, B.y_off, lam, B.cost, lcn.MODE_LCN, dx, dy, landmarks=lm, lsh=lsh)
    lcn.sinkhorn_run(h, B.iters)
    dist, resid = lcn.lcn_batched_results(h)
    st = {k: v.cpu().numpy() for k, v in lcn.lcn_batched_get(h).items()}

    # the oracle's side: its own lambdas and deletion costs
    B.lam = np.concatenate([oracle.head_lambdas(float(l0), K) for l0 in H.base_lam])
    np.testing.assert_array_equal(lam, B.lam)
    B.del_x = np.concatenate([oracle.deletion_costs(B.X[B.x_off[q]:B.x_off[q + 1]], H.alpha[H.head_of[q]])
                              for q in range(P)])
    B.del_y = np.concatenate([oracle.deletion_costs(B.Y[B.y_off[q]:B.y_off[q + 1]], H.alpha[H.head_of[q]])
                              for q in range(P)])
    np.testing.assert_array_equal(dx.cpu().numpy(), B.del_x)
    np.testing.assert_array_equal(dy.cpu().numpy(), B.del_y)
    worst = dict(log=0.0, cost=0.0, resid=0.0)
    dist_o = np.empty(P)
    for q in range(P):
        Bl, so, dist_o[q], resid_o = _oracle_pair(B, q, "lcn", True)
        n = int(B.x_off[q + 1] - B.x_off[q])
        m = int(B.y_off[q + 1] - B.y_off[q])
        z0 = int(B.x_off[q] + B.y_off[q])
        assert so.nonpositive == 0
        np.testing.assert_array_equal(st["landmarks"][q], Bl.landmarks)
        np.testing.assert_array_equal(st["buckets"][z0:z0 + n + m], Bl.buckets[0])
        worst["log"] = max(worst["log"], np.abs(st["log_u"][z0:z0 + n + m] - so.log_u).max(),
                           np.abs(st["log_v"][z0:z0 + n + m] - so.log_v).max())
        worst["cost"] = max(worst["cost"], abs(dist[q] - dist_o[q]) / abs(dist_o[q]))
        worst["resid"] = max(worst["resid"], abs(resid[q] - resid_o))
    print("C4 heads", worst, flush=True)
    assert worst["log"] <= 1e-4 and worst["cost"] <= 1e-4 and worst["resid"] <= 1e-5, worst
    # d in R^K per pair: heads of a pair differ (their lambdas do)
    d_pk = dist.reshape(-1, K)
    assert np.all(np.ptp(d_pk, axis=1) > 0)


def test_batched_runs_resume():
    """sinkhorn_run(20) then sinkhorn_run(30) equals sinkhorn_run(50): the state between runs is
    the stored log scalings."""
    import paper_2107_06876_amd as lcn
    B = workloads.config4(pairs=64)
    dev = "cuda:0"
    X, Y = torch.from_numpy(B.X).to(dev), torch.from_numpy(B.Y).to(dev)
    dx, dy = torch.from_numpy(B.del_x).to(dev), torch.from_numpy(B.del_y).to(dev)
    lm = dict(num_landmarks=B.num_landmarks, kmeans_iters=B.kmeans_iters, seed=B.landmark_seed, ridge=B.ridge)
    lsh = dict(num_buckets=B.num_buckets, num_rounds=1, kmeans_iters=B.kmeans_iters, seed=B.lsh_seed)
    out = []
    for parts in ((50,), (20, 30)):
        h = lcn.lcn_build_batched(X, Y, B.x_off, B.y_off, B.lam, B.cost, lcn.MODE_LCN, dx, dy, landmarks=lm, lsh=lsh)
        for it in parts:
            lcn.sinkhorn_run(h, it)
        dist, resid = lcn.lcn_batched_results(h)
        dist2, _ = lcn.lcn_batched_results(h)                 # a query leaves the state alone
        np.testing.assert_array_equal(dist, dist2)
        st = lcn.lcn_batched_get(h)
        out.append((dist, st["log_u"].cpu().numpy(), st["log_v"].cpu().numpy()))
        lcn.lcn_destroy(h)
    np.testing.assert_allclose(out[0][0], out[1][0], rtol=1e-10)
    np.testing.assert_allclose(out[0][1], out[1][1], rtol=0, atol=1e-11)
    np.testing.assert_allclose(out[0][2], out[1][2], rtol=0, atol=1e-11)


def _edge_batch(sizes, d, l, b, rounds=1, seed=3):
    """A hand-made batch: sizes = [(n_p, m_p), ...]."""
    rng = np.random.default_rng(seed)
    ns = np.array([s[0] for s in sizes])
    ms = np.array([s[1] for s in sizes])
    x_off = np.concatenate([[0], np.cumsum(ns)]).astype(np.int64)
    y_off = np.concatenate([[0], np.cumsum(ms)]).astype(np.int64)
    X = rng.standard_normal((int(x_off[-1]), d)).astype(np.float32)
    Y = (rng.standard_normal((int(y_off[-1]), d)) + 0.2).astype(np.float32)
    lam = np.full(len(sizes), 0.5 * d, dtype=np.float32)
    B = workloads.Batch("edge", X, Y, x_off, y_off, lam,
                        rng.uniform(0.5, 2.0, X.shape[0]).astype(np.float32),
                        rng.uniform(0.5, 2.0, Y.shape[0]).astype(np.float32),
                        workloads.COST_EUCLID, num_landmarks=l, num_buckets=b, iters=30)
    return B


@pytest.mark.parametrize("d,l,b", [(1, 1, 1), (64, 2, 2), (7, 2, 1)])
@pytest.mark.parametrize("mode,bp", [("lcn", True), ("lcn", False), ("sparse", True), ("dense", False)])
def test_batched_edge_shapes(d, l, b, mode, bp):
    """Pairs of 1 x 1, 64 x 64 (the largest), 1 x 64 and 64 x 1 points and ragged ones in one batch;
    one dimension and 64; one landmark, one bucket; per-point deletion costs."""
    sizes = [(1, 1), (64, 64), (1, 64), (64, 1), (17, 33), (2, 2), (63, 64)]
    B = _edge_batch(sizes, d, l, b)
    h, dist, resid, st = _run_gpu(B, mode, bp)
    worst = dict(log=0.0, cost=0.0, resid=0.0)
    for p in range(B.num_problems):
        Bl, so, dist_o, resid_o = _oracle_pair(B, p, mode, bp)
        n, m = sizes[p]
        z0 = int(B.x_off[p] + B.y_off[p])
        if so.nonpositive:
            continue   # the Nystrom part went negative on this pair: the batch reports it (checked below)
        lu = st["log_u"][z0:z0 + (n + m if bp else n)]
        lv = st["log_v"][z0:z0 + (n + m if bp else m)]
        if mode == "lcn":
            np.testing.assert_array_equal(st["landmarks"][p], Bl.landmarks)
        if mode in ("lcn", "sparse"):
            np.testing.assert_array_equal(st["buckets"][z0:z0 + n + m], Bl.buckets[0])
        fin = np.isfinite(so.log_u)
        worst["log"] = max(worst["log"], np.abs(lu - so.log_u)[fin].max(initial=0.0),
                           np.abs(lv - so.log_v)[np.isfinite(so.log_v)].max(initial=0.0))
        worst["cost"] = max(worst["cost"], abs(dist[p] - dist_o) / abs(dist_o))
        worst["resid"] = max(worst["resid"], abs(resid[p] - resid_o))
    print("C4 edge", d, l, b, mode, bp, worst, flush=True)
    assert worst["log"] <= 1e-4 and worst["cost"] <= 1e-4 and worst["resid"] <= 1e-5, worst
