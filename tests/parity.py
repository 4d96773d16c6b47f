"""Shared driver of the GPU parity tests: runs one problem through the oracle
and through the HIP library (C ABI via the ctypes binding) and compares them
element by element.

Tolerances (fp32 state, fp64 oracle):
  bucket ids, CSR structure, landmarks     bit-exact
  log u, log v                             max abs difference <= 1e-4
      (to first order the relative error of u, v; safe for scalings that span
       many orders of magnitude)
  Sinkhorn distance                        relative error <= 1e-4
  L1 marginal residual                     absolute error <= 1e-5
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2107_06876_amd as lcn
import workloads

MODES = {"dense": lcn.MODE_DENSE, "sparse": lcn.MODE_SPARSE, "nystrom": lcn.MODE_NYSTROM, "lcn": lcn.MODE_LCN}

TOL_LOG = 1e-4
TOL_COST_REL = 1e-4
TOL_RESID = 1e-5
NONPOS_SLACK = 4


def oracle_run(p: workloads.Problem, mode: str, hash_kind=workloads.HASH_KMEANS, iters=None):
    B = oracle.build_problem(p.X, p.Y, p.cost, p.lam, mode, p.num_landmarks, p.landmark_seed, p.kmeans_iters, p.ridge,
                             hash_kind, p.num_buckets, p.num_rounds, p.lsh_seed, p.projections,
                             landmark_init=p.landmark_init, landmark_iters=p.landmark_iters,
                             branching=p.branching, and_width=p.and_width)
    st = oracle.sinkhorn(B.op, p.a, p.b, p.iters if iters is None else iters)
    r, c, dist, resid = oracle.marginals(B.op, p.a, p.b, p.lam, st)
    return B, st, r, c, dist, resid


def gpu_build(p: workloads.Problem, mode: str, hash_kind=workloads.HASH_KMEANS, device="cuda:0"):
    dt = torch.bfloat16 if p.bf16_inputs else torch.float32
    X = torch.from_numpy(p.X).to(device).to(dt)
    Y = torch.from_numpy(p.Y).to(device).to(dt)
    a = torch.from_numpy(p.a).to(device)
    b = torch.from_numpy(p.b).to(device)
    lm = dict(num_landmarks=p.num_landmarks, seed=p.landmark_seed, ridge=p.ridge,
              kmeans_iters=p.kmeans_iters if p.landmark_iters is None else p.landmark_iters)
    if isinstance(p.landmark_init, str):
        lm["init"] = {"sample": lcn.INIT_SAMPLE, "kmeans++": lcn.INIT_KMEANSPP}[p.landmark_init]
    else:
        lm["init_centroids"] = torch.from_numpy(np.ascontiguousarray(p.landmark_init, dtype=np.float32)).to(device)
    lsh = dict(hash=hash_kind, num_buckets=p.num_buckets, num_rounds=p.num_rounds, kmeans_iters=p.kmeans_iters,
               seed=p.lsh_seed, branching=p.branching, and_width=p.and_width)
    if hash_kind == workloads.HASH_CROSSPOLYTOPE:
        lsh["projections"] = torch.from_numpy(np.ascontiguousarray(p.projections)).to(device)
    return lcn.lcn_build(X, Y, a, b, p.lam, p.cost, MODES[mode],
                         landmarks=lm if mode in ("nystrom", "lcn") else None,
                         lsh=lsh if mode in ("sparse", "lcn") else None)


def compare(p: workloads.Problem, mode: str, hash_kind=workloads.HASH_KMEANS, iters=None, check_structure=True):
    """Runs both sides and asserts parity.  Returns a dict of the observed
    differences (for reporting)."""
    iters = p.iters if iters is None else iters
    B, st, r_o, c_o, dist_o, resid_o = oracle_run(p, mode, hash_kind, iters)
    h = gpu_build(p, mode, hash_kind)
    out = {}
    if check_structure and mode in ("nystrom", "lcn"):
        L = lcn.lcn_get_landmarks(h).cpu().numpy()
        np.testing.assert_array_equal(L, B.landmarks)
        U, Wt = lcn.lcn_get_factors(h)
        U, Wt = U.cpu().numpy().astype(np.float64), Wt.cpu().numpy().astype(np.float64)
        big = B.op.U > 1e-30                      # below that fp32 storage runs into subnormals
        out["U_rel"] = float(np.max(np.abs(U[big] - B.op.U[big]) / B.op.U[big]))
        assert out["U_rel"] < 1e-6
        scale = np.abs(B.op.W).max()
        out["W_abs_over_max"] = float(np.max(np.abs(Wt.T - B.op.W)) / scale)
        assert out["W_abs_over_max"] < 1e-6
    if check_structure and mode in ("sparse", "lcn"):
        bk = lcn.lcn_get_buckets(h).cpu().numpy()
        np.testing.assert_array_equal(bk, B.buckets)
        rowptr, colidx, val = lcn.lcn_get_csr(h)
        np.testing.assert_array_equal(rowptr.cpu().numpy(), B.op.rowptr)
        np.testing.assert_array_equal(colidx.cpu().numpy(), B.op.colidx)
        info = lcn.lcn_get_info(h)
        assert info.nnz_unique == B.op.colidx.size
        v = val.cpu().numpy().astype(np.float64)
        scale = np.abs(B.op.val).max() if B.op.val.size else 1.0
        if mode == "lcn" and v.size:
            # the correction is K - U W with the factors as stored (fp32): where it is a small difference
            # of two larger numbers, the rounding of the factors (2^-24 each) is what limits it
            scale = max(scale, 0.1 * float((np.abs(B.op.U) @ np.abs(B.op.W)).max()))
        out["val_abs_over_max"] = float(np.max(np.abs(v - B.op.val)) / scale) if v.size else 0.0
        assert out["val_abs_over_max"] < 2e-6
    if st.nonpositive > 0:
        # The Nystrom part went negative (App. "Limitations"): both sides must say so.  Once one sum
        # is non-positive its scaling is NaN, the next sweep's accumulator is NaN and every later sum
        # counts, identically on both sides; only the first failing sweep's count can differ, by the
        # sums that are zero to within the rounding of the stored factors (a relative 1e-7 of their
        # terms): at most NONPOS_SLACK of them here, none on any configuration of this suite so far.
        status = lcn.sinkhorn_run(h, iters, check=False)
        nonpos, _, _ = lcn.lcn_last_error_counts(h)
        out.update(status=status, nonpositive_gpu=nonpos, nonpositive_oracle=st.nonpositive)
        assert status == lcn.binding.ERR_NONPOSITIVE, out
        assert abs(nonpos - st.nonpositive) <= NONPOS_SLACK, out
        lcn.lcn_destroy(h)
        return out
    status = lcn.sinkhorn_run(h, iters, check=False)
    want = lcn.binding.WARN_NO_SUPPORT if (st.empty_rows or st.empty_cols) else lcn.binding.OK
    assert status == want, (status, want, st.empty_rows, st.empty_cols)
    lu, lv = lcn.lcn_get_scalings(h)
    lu, lv = lu.cpu().numpy().astype(np.float64), lv.cpu().numpy().astype(np.float64)
    fin_u, fin_v = np.isfinite(st.log_u), np.isfinite(st.log_v)
    np.testing.assert_array_equal(np.isfinite(lu), fin_u)
    np.testing.assert_array_equal(np.isfinite(lv), fin_v)
    out["log_u"] = float(np.max(np.abs(lu[fin_u] - st.log_u[fin_u])))
    out["log_v"] = float(np.max(np.abs(lv[fin_v] - st.log_v[fin_v])))
    dist = lcn.transport_cost(h)
    r, c, resid = lcn.plan_marginals(h)
    out["cost_rel"] = abs(dist - dist_o) / abs(dist_o)
    out["resid_abs"] = abs(resid - resid_o)
    out["marg_abs"] = float(max(np.max(np.abs(r.cpu().numpy() - r_o)), np.max(np.abs(c.cpu().numpy() - c_o))))
    info = lcn.lcn_get_info(h)
    out["status"] = status
    out["empty_rows"], out["empty_cols"] = info.empty_rows, info.empty_cols
    # counted per sweep on both sides: a point without support is counted once per iteration
    assert (info.empty_rows, info.empty_cols) == (st.empty_rows, st.empty_cols), out
    assert lcn.lcn_last_error_counts(h) == (0, st.empty_rows, st.empty_cols)
    assert info.nonpositive == 0 and st.nonpositive == 0
    assert out["log_u"] <= TOL_LOG and out["log_v"] <= TOL_LOG, out
    assert out["cost_rel"] <= TOL_COST_REL, out
    assert out["resid_abs"] <= TOL_RESID, out
    assert out["marg_abs"] <= 1e-6, out
    lcn.lcn_destroy(h)
    return out
