"""Configuration 5 (n = m = 200 000, d = 300, bf16-stored inputs, 512
landmarks, 1024 buckets x 3 rounds, 200 iterations) against the oracle results
stored by tests/golden/make_c5_golden.py: digests of the full structure, and
scalings / marginals on the seeded 5000-point subsample."""
import hashlib
import os

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "c5_oracle.npz")


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def test_config5_against_stored_oracle_results():
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build, TOL_LOG, TOL_COST_REL, TOL_RESID
    g = np.load(GOLDEN)
    p = workloads.config5()
    assert int(g["n"]) == p.n
    h = gpu_build(p, "lcn")
    assert digest(lcn.lcn_get_landmarks(h).cpu().numpy()) == str(g["landmarks_sha256"])
    assert digest(lcn.lcn_get_buckets(h).cpu().numpy()) == str(g["buckets_sha256"])
    rowptr, colidx, _ = lcn.lcn_get_csr(h, values=False)
    assert digest(rowptr.cpu().numpy()) == str(g["rowptr_sha256"])
    assert digest(colidx.cpu().numpy()) == str(g["colidx_sha256"])
    info = lcn.lcn_get_info(h)
    assert info.nnz_unique == int(g["nnz"])
    del rowptr, colidx
    lcn.sinkhorn_run(h, int(g["iters"]))
    lu, lv = lcn.lcn_get_scalings(h)
    lu = lu.cpu().numpy().astype(np.float64)[g["rows"]]
    lv = lv.cpu().numpy().astype(np.float64)[g["cols"]]
    dist = lcn.transport_cost(h)
    r, c, resid = lcn.plan_marginals(h)
    out = dict(log_u=float(np.abs(lu - g["log_u"]).max()), log_v=float(np.abs(lv - g["log_v"]).max()),
               cost_rel=abs(dist - float(g["dist"])) / abs(float(g["dist"])), resid_abs=abs(resid - float(g["resid"])),
               marg=float(max(np.abs(r.cpu().numpy()[g["rows"]] - g["r"]).max(),
                              np.abs(c.cpu().numpy()[g["cols"]] - g["c"]).max())),
               undecided_last=info.undecided_last)
    print("C5", out, flush=True)
    assert out["log_u"] <= TOL_LOG and out["log_v"] <= TOL_LOG
    assert out["cost_rel"] <= TOL_COST_REL and out["resid_abs"] <= TOL_RESID and out["marg"] <= 1e-8
    lcn.lcn_destroy(h)
