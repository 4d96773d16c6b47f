"""Writes tests/golden/c5_oracle.npz: the CPU oracle's results for configuration 5
(n = m = 200 000, d = 300, bf16-stored inputs, 512 landmarks, 1024 buckets x 3
rounds, 200 iterations) on a seeded 5000-point subsample, plus digests of the
full structure.  Calls only oracle/ and workloads/; takes tens of minutes on
8 cores.  Run from the repository root:  python tests/golden/make_c5_golden.py
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle      # noqa: E402
import workloads   # noqa: E402


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def main(out_path, scale=None):
    t0 = time.time()
    p = workloads.config5() if scale is None else workloads.config5(n=scale)
    print("inputs", time.time() - t0, flush=True)
    B = oracle.build_problem(p.X, p.Y, p.cost, p.lam, "lcn", p.num_landmarks, p.landmark_seed, p.kmeans_iters,
                             p.ridge, 0, p.num_buckets, p.num_rounds, p.lsh_seed)
    print("build", time.time() - t0, "nnz", B.op.colidx.size, flush=True)
    st = None
    done = 0
    for chunk in (1, 4, 45, 50, 100):
        st = oracle.sinkhorn(B.op, p.a, p.b, chunk, st)
        done += chunk
        print("iterations", done, time.time() - t0, "nonpositive", st.nonpositive, flush=True)
    r, c, dist, resid = oracle.marginals(B.op, p.a, p.b, p.lam, st)
    rng = np.random.Generator(np.random.PCG64([workloads.BASE_SEED + 5, 99]))
    rows = np.sort(rng.choice(p.n, size=min(5000, p.n), replace=False))
    cols = np.sort(rng.choice(p.m, size=min(5000, p.m), replace=False))
    np.savez(out_path, n=p.n, rows=rows, cols=cols, log_u=st.log_u[rows], log_v=st.log_v[cols], r=r[rows], c=c[cols],
             dist=dist, resid=resid, nnz=B.op.colidx.size, iters=done, nonpositive=st.nonpositive,
             landmarks_sha256=digest(B.landmarks), buckets_sha256=digest(B.buckets),
             rowptr_sha256=digest(B.op.rowptr), colidx_sha256=digest(B.op.colidx))
    print("done", time.time() - t0, "dist", dist, "resid", resid, flush=True)


if __name__ == "__main__":
    scale = int(sys.argv[1]) if len(sys.argv) > 1 else None
    name = "c5_oracle.npz" if scale is None else "c5_oracle_n%d.npz" % scale
    main(os.path.join(os.path.dirname(os.path.abspath(__file__)), name), scale)
