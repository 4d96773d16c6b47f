"""Pins for the CPU oracle: closed forms, invariants, special cases and brute
force that the paper and the mathematics fix.  None of these compares the
oracle with itself or with the HIP path."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.cluster.vq
import scipy.optimize
import scipy.spatial.distance

import oracle
from oracle import COST_COSINE, COST_EUCLID, COST_SQEUCLID, Operator

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def plan(op_dense, st):
    return np.exp(st.log_u)[:, None] * op_dense * np.exp(st.log_v)[None, :]


# ------------------------------------------------------------------ costs --

def test_cost_hand_values():
    x = np.array([[3.0, 4.0]], dtype=np.float32)
    o = np.zeros((1, 2), dtype=np.float32)
    assert oracle.cost_matrix(x, o + 0.0, COST_SQEUCLID)[0, 0] == 25.0
    assert oracle.cost_matrix(x, o, COST_EUCLID)[0, 0] == 5.0
    e1 = np.array([[1.0, 0.0]], dtype=np.float32)
    e2 = np.array([[0.0, 7.0]], dtype=np.float32)
    assert oracle.cost_matrix(e1, e2, COST_COSINE)[0, 0] == 1.0
    assert abs(oracle.cost_matrix(e1, 3 * e1, COST_COSINE)[0, 0]) < 1e-15
    assert abs(oracle.cost_matrix(e1, -2 * e1, COST_COSINE)[0, 0] - 2.0) < 1e-15


@pytest.mark.parametrize("cost,metric", [(COST_SQEUCLID, "sqeuclidean"), (COST_EUCLID, "euclidean"),
                                          (COST_COSINE, "cosine")])
def test_cost_matches_library_cdist(cost, metric):
    r = rng(1)
    X = r.standard_normal((13, 7)).astype(np.float32)
    Y = r.standard_normal((5, 7)).astype(np.float32)
    ref = scipy.spatial.distance.cdist(X.astype(np.float64), Y.astype(np.float64), metric)
    np.testing.assert_allclose(oracle.cost_matrix(X, Y, cost), ref, rtol=1e-12, atol=1e-13)
    # asymmetric shapes catch a transposed operand
    assert oracle.cost_matrix(X, Y, cost).shape == (13, 5)


def test_gibbs_kernel_is_exp_of_minus_cost_over_lambda():
    r = rng(2)
    X = r.standard_normal((4, 3)).astype(np.float32)
    Y = r.standard_normal((6, 3)).astype(np.float32)
    C = scipy.spatial.distance.cdist(X.astype(np.float64), Y.astype(np.float64), "euclidean")
    np.testing.assert_allclose(oracle.gibbs_kernel(X, Y, COST_EUCLID, 0.3), np.exp(-C / 0.3), rtol=1e-12)


# -------------------------------------------------------- dense Sinkhorn --

def test_dense_2x2_closed_form():
    """Uniform marginals on a 2x2 kernel: the scaled matrix keeps the cross
    ratio rho = K11 K22 / (K12 K21), so P11 = P22 = sqrt(rho) / (2 (1 + sqrt(rho)))."""
    K = np.array([[0.9, 0.2], [0.05, 0.6]])
    op = Operator(2, 2, Kd=K)
    a = np.array([0.5, 0.5])
    st = oracle.sinkhorn(op, a, a, 200)
    P = plan(K, st)
    rho = K[0, 0] * K[1, 1] / (K[0, 1] * K[1, 0])
    p = 0.5 * math.sqrt(rho) / (1 + math.sqrt(rho))
    np.testing.assert_allclose(P, [[p, 0.5 - p], [0.5 - p, p]], rtol=1e-12)


def test_first_iteration_by_hand():
    """Eq. 2 from t = 1: s = p ./ (K 1), then t = q ./ (K^T s); a 2x3 case
    written out by hand catches a swapped update order or a transposed K."""
    K = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    a = np.array([0.25, 0.75])
    b = np.array([0.2, 0.3, 0.5])
    st = oracle.sinkhorn(Operator(2, 3, Kd=K), a, b, 1)
    u = np.array([0.25 / 6.0, 0.75 / 15.0])
    v = np.array([0.2 / (1 * u[0] + 4 * u[1]), 0.3 / (2 * u[0] + 5 * u[1]), 0.5 / (3 * u[0] + 6 * u[1])])
    np.testing.assert_allclose(np.exp(st.log_u), u, rtol=1e-13)
    np.testing.assert_allclose(np.exp(st.log_v), v, rtol=1e-13)


def test_converged_plan_satisfies_both_marginals_and_iteration_bound():
    """Fixed point of eq. 2 <=> P 1 = p and P^T 1 = q (eq. 1); Thm. 4 bounds
    the iterations needed for an L1 residual of eps."""
    r = rng(3)
    n = 12
    X = r.standard_normal((n, 3)).astype(np.float32)
    Y = r.standard_normal((n, 3)).astype(np.float32)
    K = oracle.gibbs_kernel(X, Y, COST_EUCLID, 0.5)
    a = r.random(n) + 0.5
    a /= a.sum()
    b = r.random(n) + 0.5
    b /= b.sum()
    op = Operator(n, n, Kd=K)
    eps = 0.05
    bound = 2 + (-4 * math.log(K.min() * min(a.min(), b.min()))) / eps
    st = oracle.sinkhorn(op, a, b, int(math.ceil(bound)))
    _, _, _, resid = oracle.marginals(op, a, b, 0.5, st)
    assert resid <= eps
    st = oracle.sinkhorn(op, a, b, 5000, st)
    rr, cc, _, resid = oracle.marginals(op, a, b, 0.5, st)
    P = plan(K, st)
    np.testing.assert_allclose(P.sum(1), a, atol=1e-13)
    np.testing.assert_allclose(P.sum(0), b, atol=1e-13)
    np.testing.assert_allclose(rr, P.sum(1), atol=1e-14)
    np.testing.assert_allclose(cc, P.sum(0), atol=1e-14)
    assert resid < 1e-12


def test_resumable():
    r = rng(4)
    K = r.random((5, 7)) + 0.1
    a = np.full(5, 0.2)
    b = np.full(7, 1 / 7)
    op = Operator(5, 7, Kd=K)
    s1 = oracle.sinkhorn(op, a, b, 7)
    s2 = oracle.sinkhorn(op, a, b, 3)
    s2 = oracle.sinkhorn(op, a, b, 4, s2)
    np.testing.assert_array_equal(s1.log_u, s2.log_u)
    np.testing.assert_array_equal(s1.log_v, s2.log_v)


def test_distance_formula_equals_cost_minus_entropy():
    """Eq. 1, <P, C> - lambda H(P), against the log-scaling form of eq. 5, on
    a materialised plan that has NOT converged (the identity holds for any
    scalings when the plan's own marginals are used)."""
    r = rng(5)
    n, m, lam = 9, 14, 0.7
    X = r.standard_normal((n, 4)).astype(np.float32)
    Y = r.standard_normal((m, 4)).astype(np.float32)
    C = scipy.spatial.distance.cdist(X.astype(np.float64), Y.astype(np.float64), "sqeuclidean")
    K = oracle.gibbs_kernel(X, Y, COST_SQEUCLID, lam)
    a = np.full(n, 1 / n)
    b = np.full(m, 1 / m)
    op = Operator(n, m, Kd=K)
    st = oracle.sinkhorn(op, a, b, 3)
    rr, cc, dist, resid = oracle.marginals(op, a, b, lam, st)
    P = plan(np.exp(-C / lam), st)
    H = -(P * np.log(P)).sum()
    assert abs(dist - ((P * C).sum() - lam * H)) < 1e-12
    assert abs(resid - (np.abs(P.sum(1) - a).sum() + np.abs(P.sum(0) - b).sum())) < 1e-13
    assert resid > 1e-6  # really not converged


@pytest.mark.parametrize("n", [5, 7])
def test_small_lambda_approaches_exact_assignment(n):
    """As lambda -> 0 the entropic plan's transport cost approaches exact OT,
    here brute-forced over all permutations (uniform marginals): the gap lies
    in [0, lambda log n]."""
    r = rng(60 + n)
    X = r.random((n, 2)).astype(np.float32)
    Y = r.random((n, 2)).astype(np.float32)
    C = scipy.spatial.distance.cdist(X.astype(np.float64), Y.astype(np.float64), "euclidean")
    best = min(sum(C[i, s[i]] for i in range(n)) for s in itertools.permutations(range(n))) / n
    ri, ci = scipy.optimize.linear_sum_assignment(C)
    assert abs(best - C[ri, ci].sum() / n) < 1e-13
    a = np.full(n, 1 / n)
    lam = 0.01
    op = Operator(n, n, Kd=oracle.gibbs_kernel(X, Y, COST_EUCLID, lam))
    st = oracle.sinkhorn(op, a, a, 50000)
    _, _, dist, resid = oracle.marginals(op, a, a, lam, st)
    assert resid < 1e-4
    P = plan(np.exp(-C / lam), st)
    gap = (P * C).sum() - best
    slack = 2 * resid * C.max()      # the plan is feasible only up to the residual
    assert -slack <= gap <= lam * math.log(n) + slack
    # and the distance with entropy sits between OT - lambda*2 log n and OT
    assert best - lam * 2 * math.log(n) - slack <= dist <= best + slack


# --------------------------------------------------------------- Nystrom --

def test_spd_inverse_closed_form():
    """(b 1 1^T + (a - b) I)^{-1} = -b / ((a - b)(a + (n - 1) b)) 1 1^T + I / (a - b)
    (proof of Lemma B)."""
    n, a, b = 9, 1.0, 0.37
    A = b * np.ones((n, n)) + (a - b) * np.eye(n)
    ref = -b / ((a - b) * (a + (n - 1) * b)) * np.ones((n, n)) + np.eye(n) / (a - b)
    np.testing.assert_allclose(oracle.spd_inverse(A), ref, rtol=1e-12, atol=1e-14)


def test_spd_inverse_against_library_and_failure():
    r = rng(7)
    B = r.standard_normal((11, 11))
    A = B @ B.T + 0.5 * np.eye(11)
    np.testing.assert_allclose(oracle.spd_inverse(A) @ A, np.eye(11), atol=1e-10)
    with pytest.raises(np.linalg.LinAlgError):
        oracle.spd_inverse(np.array([[1.0, 2.0], [2.0, 1.0]]))


@pytest.mark.parametrize("l", [2, 5])
def test_nystrom_lemma_b_closed_form(l):
    """Lemma B: l landmarks at mutual L2 distance Delta, points at distance
    r_i (resp. r_j) from all of them => K~_ij = l exp(-(r_i + r_j)/lambda) /
    (1 + (l - 1) exp(-Delta/lambda)).  Landmarks: scaled unit vectors of R^l (a
    regular simplex); equidistant points lie on the axis through its centre,
    at distance sqrt(R^2 + t^2) with R = sqrt((l-1)/(2l)) Delta the
    circumradius quoted after Thm. 2's proof."""
    Delta, lam = 1.3, 0.8
    L = (np.eye(l) * Delta / math.sqrt(2)).astype(np.float64)
    centre = L.mean(0)
    axis = np.ones(l) / math.sqrt(l)
    tx = np.array([0.0, 0.4, -1.1])
    ty = np.array([0.25, 2.0, -0.3, 0.9])
    X = centre + tx[:, None] * axis
    Y = centre + ty[:, None] * axis
    U, W = oracle.nystrom(X, Y, L, COST_EUCLID, lam)
    Rc = math.sqrt((l - 1) / (2 * l)) * Delta
    ri = np.sqrt(Rc ** 2 + tx ** 2)
    rj = np.sqrt(Rc ** 2 + ty ** 2)
    ref = l * np.exp(-(ri[:, None] + rj[None, :]) / lam) / (1 + (l - 1) * math.exp(-Delta / lam))
    # inputs pass through float32, so the landmarks are equidistant to ~1e-7
    np.testing.assert_allclose(U @ W, ref, rtol=2e-6)


def test_nystrom_two_landmark_collinear_closed_form_and_cluster_errors():
    """Proof of Thm. 2: landmarks at 0 and D on a line, x_i at r, x_j at D - r
    => K_Nys,ij = exp(-D/lam) (2 - exp(-2r/lam) - exp(-(2D-2r)/lam)) / (1 - exp(-2D/lam)).
    With one bucket per cluster this pair is off the sparse pattern, so LCN has
    the same value there and the three maximum errors of Thm. 2 follow."""
    Dd, r, lam = 4.0, 0.5, 0.75
    L = np.array([[0.0], [Dd]])
    X = np.array([[r], [-r], [Dd + r]])
    Y = np.array([[Dd - r], [r], [Dd - r / 2]])
    U, W = oracle.nystrom(X, Y, L, COST_EUCLID, lam)
    e = math.exp
    ref = e(-Dd / lam) * (2 - e(-2 * r / lam) - e(-(2 * Dd - 2 * r) / lam)) / (1 - e(-2 * Dd / lam))
    assert abs((U @ W)[0, 0] - ref) < 1e-14
    # LCN with buckets = clusters {x0, x1, y1} and {x2, y0, y2}
    buckets = np.array([[0, 0, 1, 1, 0, 1]], dtype=np.int32)
    rowptr, colidx = oracle.pattern(buckets, 3, 3)
    val = oracle.pattern_values(X, Y, COST_EUCLID, lam, rowptr, colidx, U, W)
    Klcn = Operator(3, 3, U=U, W=W, rowptr=rowptr, colidx=colidx, val=val).dense()
    K = oracle.gibbs_kernel(X, Y, COST_EUCLID, lam)
    # closest pair between clusters: distance D - 2r
    err_lcn = K[0, 0] - Klcn[0, 0]
    lead = e(-(Dd - 2 * r) / lam) * (1 - e(-2 * r / lam) * (2 - e(-2 * r / lam)))
    assert abs(err_lcn - lead) < 5 * e(-(Dd - 2 * r) / lam) * e(-2 * Dd / lam) + 1e-15
    # sparse error for that pair is the whole entry exp(-(D-2r)/lam)
    assert abs(K[0, 0] - e(-(Dd - 2 * r) / lam)) < 1e-15
    # Nystrom error for two coincident points at the cluster boundary: 1 - exp(-2r/lam) - O(.)
    assert abs((K[0, 1] - (U @ W)[0, 1]) - (1 - e(-2 * r / lam))) < 5 * e(-2 * (Dd - r) / lam)


def test_nystrom_exact_when_landmarks_are_the_points():
    """U A^{-1} V with landmarks = X gives A A^{-1} V = V = K(X, Y)."""
    r = rng(8)
    X = r.standard_normal((10, 3)).astype(np.float32)
    Y = r.standard_normal((17, 3)).astype(np.float32)
    for cost, lam in [(COST_EUCLID, 0.6), (COST_SQEUCLID, 0.8)]:
        U, W = oracle.nystrom(X, Y, X, cost, lam)
        K = oracle.gibbs_kernel(X, Y, cost, lam)
        np.testing.assert_allclose(U @ W, K, rtol=1e-7, atol=1e-10)
        assert U.shape == (10, 10) and W.shape == (10, 17)
    # same with landmarks = Y: U A^{-1} V = U A^{-1} A = U = K
    U, W = oracle.nystrom(X, Y, Y, COST_EUCLID, 0.6)
    np.testing.assert_allclose(U @ W, oracle.gibbs_kernel(X, Y, COST_EUCLID, 0.6), rtol=1e-7, atol=1e-10)


def test_ridge_is_added_to_the_landmark_kernel():
    r = rng(9)
    X = r.standard_normal((6, 2)).astype(np.float32)
    Y = r.standard_normal((4, 2)).astype(np.float32)
    L = r.standard_normal((3, 2)).astype(np.float32)
    lam, ridge = 0.9, 0.25
    A = oracle.gibbs_kernel(L, L, COST_EUCLID, lam) + ridge * np.eye(3)
    ref = oracle.gibbs_kernel(X, L, COST_EUCLID, lam) @ np.linalg.solve(A, oracle.gibbs_kernel(L, Y, COST_EUCLID, lam))
    U, W = oracle.nystrom(X, Y, L, COST_EUCLID, lam, ridge)
    np.testing.assert_allclose(U @ W, ref, rtol=1e-11)


# ------------------------------------------------------------------- LCN --

def _small_problem(seed, n=40, m=55, d=5):
    r = rng(seed)
    cx = r.standard_normal((4, d)) * 2
    X = (cx[r.integers(0, 4, n)] + 0.4 * r.standard_normal((n, d))).astype(np.float32)
    Y = (cx[r.integers(0, 4, m)] + 0.4 * r.standard_normal((m, d))).astype(np.float32)
    return X, Y


def test_lcn_is_exact_on_the_pattern_and_nystrom_off_it():
    """K_LCN = K_Nys - K^sp_Nys + K^sp: exact where the sparse pattern has an
    entry, plain Nystrom elsewhere (Sec. 4)."""
    X, Y = _small_problem(10)
    lam = 1.5
    B = oracle.build_problem(X, Y, COST_SQEUCLID, lam, "lcn", num_landmarks=6, num_buckets=5, num_rounds=2,
                             kmeans_iters=4)
    K = oracle.gibbs_kernel(X, Y, COST_SQEUCLID, lam)
    Klcn = B.op.dense()
    Knys = B.op.U @ B.op.W
    mask = np.zeros_like(K, dtype=bool)
    for i in range(X.shape[0]):
        mask[i, B.op.colidx[B.op.rowptr[i]:B.op.rowptr[i + 1]]] = True
    assert mask.any() and (~mask).any()
    np.testing.assert_allclose(Klcn[mask], K[mask], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(Klcn[~mask], Knys[~mask], rtol=0, atol=0)
    # the sparse path on the same pattern keeps K there and 0 elsewhere (eq. 3)
    Bs = oracle.build_problem(X, Y, COST_SQEUCLID, lam, "sparse", num_buckets=5, num_rounds=2, kmeans_iters=4)
    Ksp = Bs.op.dense()
    np.testing.assert_array_equal(Bs.op.colidx, B.op.colidx)
    np.testing.assert_allclose(Ksp[mask], K[mask], rtol=1e-14)
    assert (Ksp[~mask] == 0).all()


def test_nystrom_values_on_the_pattern_are_the_materialised_product():
    """K^sp_Nys (Sec. 4: the Nystrom approximation restricted to the pattern) against the
    materialised U W with n != m and l != n, m (a transposed or mis-strided operand fails), and
    the decomposition K^sp_Delta = K^sp - K^sp_Nys of the three value modes."""
    X, Y = _small_problem(12, n=23, m=17)
    lam = 1.3
    B = oracle.build_problem(X, Y, COST_SQEUCLID, lam, "lcn", num_landmarks=7, num_buckets=4, num_rounds=2,
                             kmeans_iters=4)
    rowptr, colidx = B.op.rowptr, B.op.colidx
    assert 0 < colidx.size < 23 * 17
    rows = np.repeat(np.arange(23), np.diff(rowptr))
    UW = B.op.U @ B.op.W
    knys = oracle.pattern_values(X, Y, COST_SQEUCLID, lam, rowptr, colidx, B.op.U, B.op.W, nystrom_only=True)
    np.testing.assert_allclose(knys, UW[rows, colidx], rtol=1e-13, atol=1e-300)
    # W read with the stride of its transpose is a different matrix, so the comparison can tell
    wrong = B.op.U @ np.ascontiguousarray(B.op.W).reshape(17, 7).T
    assert np.abs(knys - wrong[rows, colidx]).max() > 1e-3 * np.abs(knys).max()
    ksp = oracle.pattern_values(X, Y, COST_SQEUCLID, lam, rowptr, colidx)
    kdelta = oracle.pattern_values(X, Y, COST_SQEUCLID, lam, rowptr, colidx, B.op.U, B.op.W)
    np.testing.assert_allclose(ksp - knys, kdelta, rtol=0, atol=1e-15)
    np.testing.assert_allclose(ksp, oracle.gibbs_kernel(X, Y, COST_SQEUCLID, lam)[rows, colidx], rtol=1e-14)
    # a pattern of one entry per row (no bucket structure) picks the same entries
    rp = np.arange(24, dtype=np.int64)
    ci = ((5 * np.arange(23) + 3) % 17).astype(np.int32)
    one = oracle.pattern_values(X, Y, COST_SQEUCLID, lam, rp, ci, B.op.U, B.op.W, nystrom_only=True)
    np.testing.assert_allclose(one, UW[np.arange(23), ci], rtol=1e-13, atol=1e-300)


def test_single_bucket_makes_sparse_and_lcn_equal_dense():
    X, Y = _small_problem(11, n=30, m=30)
    lam = 2.0
    a = np.full(30, 1 / 30)
    dense = oracle.build_problem(X, Y, COST_SQEUCLID, lam, "dense")
    sd = oracle.sinkhorn(dense.op, a, a, 25)
    for mode in ("sparse", "lcn"):
        B = oracle.build_problem(X, Y, COST_SQEUCLID, lam, mode, num_landmarks=5, num_buckets=1, num_rounds=1,
                                 kmeans_iters=3)
        assert B.op.colidx.size == 900
        st = oracle.sinkhorn(B.op, a, a, 25)
        np.testing.assert_allclose(st.log_u, sd.log_u, atol=1e-10)
        np.testing.assert_allclose(st.log_v, sd.log_v, atol=1e-10)
        d0 = oracle.marginals(dense.op, a, a, lam, sd)[2]
        d1 = oracle.marginals(B.op, a, a, lam, st)[2]
        assert abs(d0 - d1) < 1e-10


def test_operator_products_match_materialised_matrix():
    """U (W t) + S t and its transpose against the materialised K_LCN, with
    n != m so a transposed operand cannot pass."""
    X, Y = _small_problem(12, n=23, m=37)
    lam = 1.2
    B = oracle.build_problem(X, Y, COST_SQEUCLID, lam, "lcn", num_landmarks=4, num_buckets=3, num_rounds=2,
                             kmeans_iters=3)
    Kt = B.op.dense()
    r = rng(13)
    a = r.random(23) + 0.1
    a /= a.sum()
    b = r.random(37) + 0.1
    b /= b.sum()
    st = oracle.sinkhorn(B.op, a, b, 4)
    ref = oracle.sinkhorn(Operator(23, 37, Kd=Kt), a, b, 4)
    np.testing.assert_allclose(st.log_u, ref.log_u, atol=1e-11)
    np.testing.assert_allclose(st.log_v, ref.log_v, atol=1e-11)
    m1 = oracle.marginals(B.op, a, b, lam, st)
    m2 = oracle.marginals(Operator(23, 37, Kd=Kt), a, b, lam, ref)
    for x, y in zip(m1, m2):
        np.testing.assert_allclose(x, y, atol=1e-11)


def test_sparse_rows_without_support_carry_no_mass():
    """App. "Limitations": a sparse kernel may have rows/columns without any
    entry; they are ignored (log scaling -inf, zero mass) and counted."""
    K = np.array([[1.0, 0.5, 0.0], [0.0, 0.0, 0.0], [0.2, 0.0, 0.0]])
    rowptr = np.array([0, 2, 2, 3], dtype=np.int64)
    colidx = np.array([0, 1, 0], dtype=np.int32)
    val = np.array([1.0, 0.5, 0.2])
    op = Operator(3, 3, rowptr=rowptr, colidx=colidx, val=val)
    a = np.full(3, 1 / 3)
    st = oracle.sinkhorn(op, a, a, 2)
    assert st.empty_rows == 2 and st.empty_cols == 2 and st.nonpositive == 0
    assert np.isneginf(st.log_u[1]) and np.isneginf(st.log_v[2])
    rr, cc, dist, resid = oracle.marginals(op, a, a, 1.0, st)
    assert rr[1] == 0 and cc[2] == 0 and np.isfinite(dist)
    P = plan(K, st)
    np.testing.assert_allclose(rr, P.sum(1), atol=1e-15)
    np.testing.assert_allclose(cc, P.sum(0), atol=1e-15)


def test_negative_row_sum_is_reported():
    """App. "Limitations": the Nystrom part is not guaranteed non-negative."""
    U = np.array([[1.0], [1.0]])
    W = np.array([[1.0, -3.0]])
    st = oracle.sinkhorn(Operator(2, 2, U=U, W=W), np.array([0.5, 0.5]), np.array([0.5, 0.5]), 1)
    assert st.nonpositive > 0


# ------------------------------------------------------------- structure --

def test_pattern_matches_brute_force_sets():
    r = rng(14)
    n, m, R, b = 37, 29, 3, 6
    buckets = r.integers(0, b, size=(R, n + m)).astype(np.int32)
    rowptr, colidx = oracle.pattern(buckets, n, m)
    pairs = set()
    for rr in range(R):
        for beta in range(b):
            xs = [i for i in range(n) if buckets[rr, i] == beta]
            ys = [j for j in range(m) if buckets[rr, n + j] == beta]
            pairs.update(itertools.product(xs, ys))
    got = [(i, int(j)) for i in range(n) for j in colidx[rowptr[i]:rowptr[i + 1]]]
    assert len(got) == len(set(got)) == len(pairs) and set(got) == pairs
    for i in range(n):
        seg = colidx[rowptr[i]:rowptr[i + 1]]
        assert (np.diff(seg) > 0).all()
    # one round: nnz = sum over buckets of n_b * m_b
    rp1, ci1 = oracle.pattern(buckets[:1], n, m)
    cx = np.bincount(buckets[0, :n], minlength=b)
    cy = np.bincount(buckets[0, n:], minlength=b)
    assert ci1.size == int((cx * cy).sum())


def test_expected_neighbours_per_point():
    """App. "Complexity analysis": about m / b neighbours per point for b
    buckets (one hash per band)."""
    r = rng(15)
    n = m = 4000
    b = 16
    Z = r.standard_normal((n + m, 24)).astype(np.float32)
    R = r.standard_normal((24, b // 2)).astype(np.float32)
    bk = oracle.crosspolytope(Z, R, b)[None, :]
    rowptr, _ = oracle.pattern(bk, n, m)
    assert abs(rowptr[-1] / n - m / b) < 0.15 * m / b


def _exact_sqdist(z, c):
    return sum((Fraction(float(a)) - Fraction(float(b))) ** 2 for a, b in zip(z, c))


def test_assign_matches_exact_rational_argmin_and_tie_rule():
    r = rng(16)
    Z = r.standard_normal((25, 6)).astype(np.float32)
    Cn = r.standard_normal((7, 6)).astype(np.float32)
    got = oracle.assign(Z, Cn)
    for p in range(25):
        d = [_exact_sqdist(Z[p], Cn[c]) for c in range(7)]
        assert got[p] == d.index(min(d))
    # exact ties: duplicate centroids, and a point midway between two centroids
    Cn2 = np.array([[1.0, 0.0], [-1.0, 0.0], [1.0, 0.0], [0.0, 5.0]], dtype=np.float32)
    Z2 = np.array([[2.0, 0.0], [0.0, 0.0], [-3.0, 1.0], [0.0, 4.0]], dtype=np.float32)
    np.testing.assert_array_equal(oracle.assign(Z2, Cn2), [0, 0, 1, 3])


def test_crosspolytope_definition_and_sign_symmetry():
    r = rng(17)
    N, d, b = 200, 9, 10
    Z = r.standard_normal((N, d)).astype(np.float32)
    R = r.standard_normal((d, b // 2)).astype(np.float32)
    h = oracle.crosspolytope(Z, R, b)
    g = Z.astype(np.float64) @ R.astype(np.float64)
    np.testing.assert_array_equal(h, np.argmax(np.concatenate([g, -g], axis=1), axis=1))
    hneg = oracle.crosspolytope(-Z, R, b)
    np.testing.assert_array_equal(hneg, (h + b // 2) % b)
    assert h.min() >= 0 and h.max() < b
    # zero vector: every projection ties at 0 -> lowest index
    assert oracle.crosspolytope(np.zeros((1, d), np.float32), R, b)[0] == 0


def test_seeded_indices_follow_published_generator():
    with open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")) as f:
        outs = [int(line) for line in f if line.strip() and not line.startswith("#")]
    N, k = 1000, 5
    perm = list(range(N))
    want = []
    for t in range(k):
        j = t + outs[t] % (N - t)
        perm[t], perm[j] = perm[j], perm[t]
        want.append(perm[t])
    np.testing.assert_array_equal(oracle.seeded_indices(1234567, N, k), want)
    full = oracle.seeded_indices(99, 257, 257)
    assert sorted(full.tolist()) == list(range(257))
    assert not np.array_equal(oracle.seeded_indices(1, 1000, 20), oracle.seeded_indices(2, 1000, 20))
    with pytest.raises(ValueError):
        oracle.seeded_indices(1, 5, 6)


def test_kmeans_against_library_lloyd():
    """scipy's kmeans2 started from the same centroids runs the same Lloyd
    iteration (assign, then means); its labels are those of the last assign
    step and its code book the means of those clusters."""
    r = rng(18)
    cx = r.standard_normal((6, 8)) * 4
    Z = (cx[r.integers(0, 6, 600)] + 0.5 * r.standard_normal((600, 8))).astype(np.float32)
    k, T, seed = 6, 5, 3
    cent, asg = oracle.kmeans(Z, k, T, seed)
    init = Z[oracle.seeded_indices(seed, 600, k)].astype(np.float64)
    ref_c, ref_l = scipy.cluster.vq.kmeans2(Z.astype(np.float64), init, iter=T, minit="matrix")
    np.testing.assert_array_equal(asg, ref_l)
    np.testing.assert_allclose(cent, ref_c, rtol=2e-7, atol=1e-7)
    # the assignment is w.r.t. the centroids before the last update
    prev, _ = oracle.kmeans(Z, k, T - 1, seed)
    np.testing.assert_array_equal(asg, oracle.assign(Z, prev))


def test_kmeans_objective_never_increases():
    r = rng(19)
    Z = r.standard_normal((500, 5)).astype(np.float32)
    prev = None
    for T in range(1, 8):
        cent, _ = oracle.kmeans(Z, 9, T, 5)
        lab = oracle.assign(Z, cent)
        obj = ((Z.astype(np.float64) - cent[lab].astype(np.float64)) ** 2).sum()
        if prev is not None:
            assert obj <= prev * (1 + 1e-7)
        prev = obj


def test_kmeans_mean_is_fixed_point_mean_and_empty_cluster_keeps_centroid():
    # two distinct points only, three clusters: two start centroids coincide, the
    # higher-numbered of them never wins a tie, stays empty and must keep its start
    Z = np.array([[0.5, 1.25]] * 6 + [[-2.0, 0.125]] * 4, dtype=np.float32)
    for seed in range(6):
        idx = oracle.seeded_indices(seed, 10, 3)
        start = Z[idx]
        T = 3 if len({tuple(x) for x in start}) == 2 else 1
        cent, asg = oracle.kmeans(Z, 3, T, seed)
        firsts = {}
        for c in range(3):
            firsts.setdefault(tuple(start[c]), c)
        for c in range(3):
            owner = firsts[tuple(start[c])]
            if owner != c:      # a duplicate start: never wins a tie, stays empty, keeps its start
                assert (asg != c).all()
                np.testing.assert_array_equal(cent[c], start[c])
        if len(firsts) == 2:    # both distinct points are starts: each owner keeps exactly its point
            for p in range(10):
                assert asg[p] == firsts[tuple(Z[p])]
            for pt, c in firsts.items():
                np.testing.assert_array_equal(cent[c], np.array(pt, dtype=np.float32))
        else:                   # one distinct start: cluster 0 takes every point
            assert (asg == 0).all()
            np.testing.assert_array_equal(cent[0], Z.astype(np.float64).mean(0).astype(np.float32))
    # means of values that are exact in 2^-32 fixed point are exact rational means, rounded once
    r = rng(20)
    Zi = (r.integers(-2 ** 12, 2 ** 12, size=(64, 3)) / 2.0 ** 10).astype(np.float32)
    cent, asg = oracle.kmeans(Zi, 4, 2, 11)
    for c in range(4):
        mem = Zi[asg == c]
        if len(mem):
            exact = [float(sum(Fraction(float(v)) for v in mem[:, j]) / len(mem)) for j in range(3)]
            np.testing.assert_array_equal(cent[c], np.array(exact, dtype=np.float32))


# -------------------------------------------------- bipartite matching BP --

def _bp_matrix(K, kpe, keq):
    n, m = K.shape
    top = np.concatenate([K, np.diag(kpe)], axis=1)
    bot = np.concatenate([np.diag(keq), np.ones((m, n))], axis=1)
    return np.concatenate([top, bot], axis=0)


def test_bp_block_products_match_materialised_matrix():
    """Sec. 6: K_BP = exp(-C_BP / lambda) with diagonal (p, eps) and (eps, q)
    blocks and an all-ones (eps, eps) block; n != m."""
    r = rng(21)
    n, m, lam = 5, 8, 0.9
    X = r.standard_normal((n, 3)).astype(np.float32)
    Y = r.standard_normal((m, 3)).astype(np.float32)
    K = oracle.gibbs_kernel(X, Y, COST_EUCLID, lam)
    kpe = np.exp(-(r.random(n) + 0.5) / lam)
    keq = np.exp(-(r.random(m) + 0.5) / lam)
    N = n + m
    a = np.full(N, 1 / N)
    st = oracle.sinkhorn_bp(Operator(n, m, Kd=K), kpe, keq, a, a, 6)
    Kbp = _bp_matrix(K, kpe, keq)
    ref = oracle.sinkhorn(Operator(N, N, Kd=Kbp), a, a, 6)
    np.testing.assert_allclose(st.log_u, ref.log_u, atol=1e-12)
    np.testing.assert_allclose(st.log_v, ref.log_v, atol=1e-12)
    m1 = oracle.marginals_bp(Operator(n, m, Kd=K), kpe, keq, a, a, lam, st)
    m2 = oracle.marginals(Operator(N, N, Kd=Kbp), a, a, lam, ref)
    for x, y in zip(m1, m2):
        np.testing.assert_allclose(x, y, atol=1e-12)


def test_bp_single_pair_closed_form_and_infinite_deletion_cost():
    # n = m = 1: K_BP = [[K, kpe], [keq, 1]], uniform marginals -> 2x2 closed form
    K = np.array([[0.3]])
    kpe, keq = np.array([0.6]), np.array([0.2])
    a = np.array([0.5, 0.5])
    st = oracle.sinkhorn_bp(Operator(1, 1, Kd=K), kpe, keq, a, a, 300)
    P = plan(_bp_matrix(K, kpe, keq), st)
    rho = 0.3 * 1.0 / (0.6 * 0.2)
    p = 0.5 * math.sqrt(rho) / (1 + math.sqrt(rho))
    np.testing.assert_allclose(P, [[p, 0.5 - p], [0.5 - p, p]], rtol=1e-12)
    # deletion cost -> infinity (kernel 0): the point block decouples into balanced OT
    r = rng(22)
    n = 6
    X = r.standard_normal((n, 2)).astype(np.float32)
    Y = r.standard_normal((n, 2)).astype(np.float32)
    Kxy = oracle.gibbs_kernel(X, Y, COST_EUCLID, 1.0)
    z = np.zeros(n)
    abp = np.full(2 * n, 1 / (2 * n))
    sbp = oracle.sinkhorn_bp(Operator(n, n, Kd=Kxy), z, z, abp, abp, 40)
    bal = oracle.sinkhorn(Operator(n, n, Kd=Kxy), abp[:n], abp[:n], 40)
    np.testing.assert_allclose(sbp.log_u[:n], bal.log_u, atol=1e-12)
    np.testing.assert_allclose(sbp.log_v[:n], bal.log_v, atol=1e-12)


def test_log_domain_path_survives_diverging_scalings_and_matches_library_logsumexp():
    """A sparse kernel without support (App. "Limitations": non-square blocks)
    makes the scalings drift without bound; the log-sum-exp form (App.
    "Implementational details") must keep working far beyond the range of
    exp(), and agree with the same iteration written with the library's
    logsumexp."""
    import scipy.special
    r = rng(23)
    n, m = 7, 5
    K = np.zeros((n, m))
    K[:5, :2] = r.random((5, 2)) + 0.1      # block with 5 rows, 2 columns
    K[5:, 2:] = r.random((2, 3)) + 0.1      # block with 2 rows, 3 columns
    rows, cols = np.nonzero(K)
    rowptr = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=n))]).astype(np.int64)
    op = Operator(n, m, rowptr=rowptr, colidx=cols.astype(np.int32), val=K[rows, cols])
    a = np.full(n, 1 / n)
    b = np.full(m, 1 / m)
    iters = 3000
    st = oracle.sinkhorn(op, a, b, iters)
    with np.errstate(divide="ignore"):
        logK = np.log(K)
    lu, lv = np.zeros(n), np.zeros(m)
    for _ in range(iters):
        lu = np.log(a) - scipy.special.logsumexp(logK + lv[None, :], axis=1)
        lv = np.log(b) - scipy.special.logsumexp(logK + lu[:, None], axis=0)
    assert np.abs(lu).max() > 800          # far outside what exp() can represent
    np.testing.assert_allclose(st.log_u, lu, rtol=1e-10, atol=1e-8)
    np.testing.assert_allclose(st.log_v, lv, rtol=1e-10, atol=1e-8)
    assert st.nonpositive == 0 and st.empty_rows == 0
    rr, cc, dist, resid = oracle.marginals(op, a, b, 1.0, st)
    assert np.isfinite(dist) and np.isfinite(resid)
    np.testing.assert_allclose(cc, b, atol=1e-12)   # columns were scaled last


# ---- analytic derivatives (Prop. 1) ------------------------------------------

def _small_lcn(seed=31):
    """A small decomposed kernel with every entry positive, its four parts separate."""
    r = rng(seed)
    n, m, d, l = 9, 11, 3, 3
    X = (0.4 * r.standard_normal((n, d))).astype(np.float32)
    Y = (0.4 * r.standard_normal((m, d))).astype(np.float32)
    lam = 1.5
    L = np.concatenate([X, Y])[[0, 7, 15]]
    U, W = oracle.nystrom(X, Y, L, COST_SQEUCLID, lam, 0.0)
    bucket = np.concatenate([np.arange(n) % 2, np.arange(m) % 2]).astype(np.int32)[None, :]
    rowptr, colidx = oracle.pattern(bucket, n, m)
    ksp = oracle.pattern_values(X, Y, COST_SQEUCLID, lam, rowptr, colidx)
    knys = oracle.pattern_values(X, Y, COST_SQEUCLID, lam, rowptr, colidx, U, W, nystrom_only=True)
    a = r.random(n) + 0.5
    b = r.random(m) + 0.5
    return n, m, lam, U, W, rowptr, colidx, ksp, knys, a / a.sum(), b / b.sum()


def _converged(n, m, lam, U, W, rowptr, colidx, ksp, knys, a, b, iters=3000):
    op = Operator(n, m, U=U, W=W, rowptr=rowptr, colidx=colidx, val=ksp - knys)
    assert op.dense().min() > 0
    st = oracle.sinkhorn(op, a, b, iters)
    _, _, dist, resid = oracle.marginals(op, a, b, lam, st)
    assert resid < 1e-13
    return op, st, dist


def test_backward_matches_finite_differences_of_the_converged_distance():
    """Prop. 1 with U, W, log K^sp and log K^sp_Nys as independent variables:
    central differences of the converged distance reproduce every derivative,
    including the sign of the K^sp_Nys term (which enters the kernel negatively)."""
    n, m, lam, U, W, rowptr, colidx, ksp, knys, a, b = _small_lcn()
    op, st, d0 = _converged(n, m, lam, U, W, rowptr, colidx, ksp, knys, a, b)
    gU, gW, gsp, gnys = oracle.backward(op, lam, st, ksp, knys)
    h = 1e-5

    def dist(U_=U, W_=W, ksp_=ksp, knys_=knys):
        return _converged(n, m, lam, U_, W_, rowptr, colidx, ksp_, knys_, a, b)[2]

    for (i, k) in [(0, 0), (4, 2), (8, 1)]:
        E = np.zeros_like(U)
        E[i, k] = h
        fd = (dist(U_=U + E) - dist(U_=U - E)) / (2 * h)
        np.testing.assert_allclose(gU[i, k], fd, rtol=2e-5)
    for (k, j) in [(0, 0), (2, 10), (1, 5)]:      # n != m: a transposed result would not even fit
        E = np.zeros_like(W)
        E[k, j] = h
        fd = (dist(W_=W + E) - dist(W_=W - E)) / (2 * h)
        np.testing.assert_allclose(gW[k, j], fd, rtol=2e-5)
    for e in [0, 17, len(colidx) - 1]:
        f = np.ones_like(ksp)
        f[e] = math.exp(h)
        fd = (dist(ksp_=ksp * f) - dist(ksp_=ksp / f)) / (2 * h)
        np.testing.assert_allclose(gsp[e], fd, rtol=2e-5)
        fd = (dist(knys_=knys * f) - dist(knys_=knys / f)) / (2 * h)
        np.testing.assert_allclose(gnys[e], fd, rtol=2e-5)
        assert gsp[e] < 0 < gnys[e]


def test_backward_mass_identity():
    """sum U o gU = sum W o gW = -lambda (mass of the Nystrom part), sum gsp = -lambda (mass of
    the K^sp part), sum gnys = +lambda (mass of the K^sp_Nys part); the plan's mass is 1, so
    sum U o gU + sum gsp + sum gnys = -lambda."""
    n, m, lam, U, W, rowptr, colidx, ksp, knys, a, b = _small_lcn(32)
    op, st, _ = _converged(n, m, lam, U, W, rowptr, colidx, ksp, knys, a, b)
    gU, gW, gsp, gnys = oracle.backward(op, lam, st, ksp, knys)
    u, v = np.exp(st.log_u), np.exp(st.log_v)
    mass_nys = u @ (U @ W) @ v
    np.testing.assert_allclose((U * gU).sum(), -lam * mass_nys, rtol=1e-12)
    np.testing.assert_allclose((W * gW).sum(), -lam * mass_nys, rtol=1e-12)
    np.testing.assert_allclose((U * gU).sum() + gsp.sum() + gnys.sum(), -lam, rtol=1e-11)


def test_backward_dense_gives_the_plan():
    """First line of Prop. 1: d d / d C = P for plain entropic OT (K = K^sp on the full pattern),
    against the materialised plan and against a central difference in one cost entry."""
    r = rng(33)
    n, m = 6, 8
    C = r.random((n, m))
    lam = 0.7
    a = np.full(n, 1 / n)
    b = np.full(m, 1 / m)
    rowptr = (np.arange(n + 1) * m).astype(np.int64)
    colidx = np.tile(np.arange(m), n).astype(np.int32)

    def solve(Cm):
        K = np.exp(-Cm / lam)
        op = Operator(n, m, rowptr=rowptr, colidx=colidx, val=K.ravel())
        st = oracle.sinkhorn(op, a, b, 3000)
        return op, st, K, oracle.marginals(op, a, b, lam, st)[2]

    op, st, K, d0 = solve(C)
    _, _, gsp, _ = oracle.backward(op, lam, st, ksp=K.ravel())
    P = plan(K, st)
    np.testing.assert_allclose(-gsp.reshape(n, m) / lam, P, rtol=1e-12)
    h = 1e-5
    E = np.zeros_like(C)
    E[2, 5] = h
    fd = (solve(C + E)[3] - solve(C - E)[3]) / (2 * h)
    np.testing.assert_allclose(P[2, 5], fd, rtol=2e-5)


# ---------------------------------------------------- multi-head / deletion costs --

def test_deletion_costs_special_cases():
    """Sec. 6, learnable deletion cost: alpha = 1 is the Euclidean norm, a unit
    alpha picks |x_j|, and the 3-4-5 triangle."""
    rng = np.random.default_rng(5)
    X = rng.standard_normal((37, 19)).astype(np.float32)
    alpha = rng.uniform(0.5, 1.5, 19).astype(np.float32)
    c = oracle.deletion_costs(X, alpha)
    assert c.dtype == np.float32
    ref = np.linalg.norm(X.astype(np.float64) * alpha.astype(np.float64), axis=1)
    np.testing.assert_allclose(c, ref, rtol=1e-7)
    np.testing.assert_allclose(oracle.deletion_costs(X, np.ones(19, np.float32)),
                               np.linalg.norm(X.astype(np.float64), axis=1), rtol=1e-7)
    e = np.zeros(19, np.float32)
    e[7] = 2.0
    np.testing.assert_array_equal(oracle.deletion_costs(X, e), np.abs(2.0 * X[:, 7]))
    np.testing.assert_array_equal(oracle.deletion_costs(np.array([[3.0, 4.0]], np.float32),
                                                        np.ones(2, np.float32)), [5.0])
    # homogeneous of degree one in alpha
    np.testing.assert_allclose(oracle.deletion_costs(X, 2 * alpha), 2 * c, rtol=1e-7)


def test_head_lambdas_closed_form():
    """Sec. 6, multi-head OT: consecutive heads differ by a factor of two and
    K = 2 gives (lambda, 2 lambda); the geometric mean is sqrt(2) lambda."""
    np.testing.assert_array_equal(oracle.head_lambdas(0.25, 2), np.array([0.25, 0.5], np.float32))
    lam8 = oracle.head_lambdas(0.1, 8).astype(np.float64)
    np.testing.assert_allclose(lam8[1:] / lam8[:-1], 2.0, rtol=1e-6)
    np.testing.assert_allclose(np.exp(np.log(lam8).mean()), np.sqrt(2.0) * np.float32(0.1), rtol=1e-6)
    np.testing.assert_allclose(lam8[3], np.float32(0.1), rtol=1e-7)   # k = K/2


# ------------------------------------------------------------ k-means++ sampling --

def test_kmeanspp_second_pick_follows_squared_distances():
    """Sec. 4, landmarks sampled via k-means++: given the first point, the second is
    drawn with probability D^2 / sum D^2.  Four points on a line, 40 000 seeds: the
    empirical law of (first, second) against the closed form (first uniform)."""
    Z = np.array([[0.0], [1.0], [3.0], [7.0]], dtype=np.float32)
    N, S = 4, 40000
    counts = np.zeros((N, N))
    for seed in range(S):
        i, j = oracle.kmeanspp(Z, 2, seed)
        counts[i, j] += 1
    D2 = (Z - Z.T) ** 2
    expect = (D2 / D2.sum(axis=1, keepdims=True)) / N
    assert np.all(np.diag(counts) == 0)
    sigma = np.sqrt(expect * (1 - expect) / S)
    assert np.all(np.abs(counts / S - expect) <= 4.5 * sigma + 1e-12), (counts / S, expect)


def test_kmeanspp_structure():
    """Distinct picks; a copy of a chosen point is never drawn while other points are left;
    far-apart tight clusters each receive one of k = (number of clusters) picks; scaling
    the points by a power of two changes nothing (the weights are relative to the largest norm);
    more picks than distinct points falls back to the lowest unused index."""
    rng = np.random.default_rng(3)
    Z = rng.standard_normal((400, 5)).astype(np.float32)
    for seed in range(5):
        idx = oracle.kmeanspp(Z, 50, seed)
        assert len(set(idx.tolist())) == 50 and idx.min() >= 0 and idx.max() < 400
        np.testing.assert_array_equal(oracle.kmeanspp(4.0 * Z, 50, seed), idx)
        np.testing.assert_array_equal(oracle.kmeanspp(Z, 20, seed), idx[:20])        # a prefix of the longer run
    centres = 100.0 * np.eye(6, 5)
    label = np.arange(300) % 6
    C = (centres[label] + 0.01 * rng.standard_normal((300, 5))).astype(np.float32)
    for seed in range(20):
        assert sorted(label[oracle.kmeanspp(C, 6, seed)].tolist()) == list(range(6))
    Zd = np.concatenate([Z[:7], Z[:7], Z[:7]])                                       # 7 distinct points, 3 copies each
    for seed in range(10):
        idx = oracle.kmeanspp(Zd, 10, seed)
        assert sorted((idx[:7] % 7).tolist()) == list(range(7))                      # first the 7 distinct ones
        left = sorted(set(range(21)) - set(idx[:7].tolist()))
        np.testing.assert_array_equal(idx[7:], left[:3])                             # then lowest unused indices
    idx = oracle.kmeanspp(np.zeros((5, 3), np.float32), 3, 1)                       # all points equal
    np.testing.assert_array_equal(idx[1:], sorted(set(range(5)) - {int(idx[0])})[:2])


def test_kmeanspp_first_pick_uniform_and_potential():
    """First pick uniform over the points; the D^2 potential after k-means++ seeding is, on
    clustered data, far below that of a uniform sample (the reason the paper prefers it)."""
    Z = np.arange(10, dtype=np.float32).reshape(10, 1)
    first = np.bincount([int(oracle.kmeanspp(Z, 1, s)[0]) for s in range(20000)], minlength=10) / 20000.0
    assert np.all(np.abs(first - 0.1) < 4.5 * np.sqrt(0.09 / 20000))
    rng = np.random.default_rng(8)
    centres = 10.0 * rng.standard_normal((12, 4))
    sizes = (2000 * np.arange(1, 13) / 78).astype(int)                               # unbalanced clusters
    P = np.concatenate([c + 0.1 * rng.standard_normal((s, 4)) for c, s in zip(centres, sizes)]).astype(np.float32)

    def potential(idx):
        return ((P[:, None, :].astype(np.float64) - P[idx][None].astype(np.float64)) ** 2).sum(-1).min(1).sum()

    pp = np.median([potential(oracle.kmeanspp(P, 12, s)) for s in range(15)])
    un = np.median([potential(oracle.seeded_indices(s, len(P), 12)) for s in range(15)])
    assert pp < 0.2 * un, (pp, un)


def test_lloyd_from_given_start():
    """k-means from caller-supplied centroids: the true means of well separated clusters are a
    fixed point, and the seeded start passed in by hand reproduces the seeded run."""
    rng = np.random.default_rng(4)
    centres = 20.0 * np.eye(4, 3)
    label = np.arange(200) % 4
    Z = (centres[label] + rng.standard_normal((200, 3))).astype(np.float32)
    means = np.stack([Z[label == c].astype(np.float64).mean(0) for c in range(4)])
    cent, asg = oracle.kmeans(Z, 4, 3, 0, init=means.astype(np.float32))
    np.testing.assert_array_equal(asg, label)
    np.testing.assert_allclose(cent, means, rtol=0, atol=1e-6)
    a = oracle.kmeans(Z, 4, 5, 9)
    b = oracle.kmeans(Z, 4, 5, 9, init=Z[oracle.seeded_indices(9, 200, 4)])
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    c0, a0 = oracle.kmeans(Z, 4, 0, 9, init="kmeans++")
    np.testing.assert_array_equal(c0, Z[oracle.kmeanspp(Z, 4, 9)])
    np.testing.assert_array_equal(a0, oracle.assign(Z, c0))


# ----------------------------------------- hierarchical k-means, AND construction --

def test_hierarchical_kmeans_structure():
    """App. "Choosing LSH neighbors and Nystrom landmarks" (hierarchical k-means): one level is flat
    k-means; a trailing branching factor 1 changes nothing; the upper level of a two-level hash IS
    the flat hash with the same seed; every lower-level run only sees its parent's members."""
    rng = np.random.default_rng(12)
    Z = rng.standard_normal((600, 6)).astype(np.float32)
    _, flat = oracle.kmeans(Z, 7, 5, 33)
    np.testing.assert_array_equal(oracle.hierarchical_kmeans(Z, [7], 5, 33), flat)
    np.testing.assert_array_equal(oracle.hierarchical_kmeans(Z, [7, 1], 5, 33), flat)
    two = oracle.hierarchical_kmeans(Z, [7, 4], 5, 33)
    np.testing.assert_array_equal(two // 4, flat)
    assert two.min() >= 0 and two.max() < 28
    three = oracle.hierarchical_kmeans(Z, [3, 2, 4], 5, 33)
    np.testing.assert_array_equal(three // 4, oracle.hierarchical_kmeans(Z, [3, 2], 5, 33))
    # a parent with fewer members than children: one bucket per member, ids below the branching factor
    tiny = np.concatenate([[[0, 0], [1, 0], [0, 1]], 100 + rng.standard_normal((50, 2))]).astype(np.float32)
    h = oracle.hierarchical_kmeans(tiny, [2, 5], 10, 1)
    lone = h[:3]
    assert len(set(lone.tolist())) == 3 and len(set((lone // 5).tolist())) == 1
    assert set((h[3:] // 5).tolist()) == {1 - int(lone[0] // 5)}


def test_hierarchical_kmeans_fixed_point():
    """Run to convergence, every point is nearer (or as near) to the mean of its own bucket than to
    the mean of any sibling bucket -- Lloyd's fixed point, inside every parent."""
    rng = np.random.default_rng(13)
    centres = 6.0 * rng.standard_normal((12, 3))
    Z = (centres[rng.integers(0, 12, 900)] + 0.5 * rng.standard_normal((900, 3))).astype(np.float32)
    b1, b2 = 4, 3
    h = oracle.hierarchical_kmeans(Z, [b1, b2], 200, 5)
    Zd = Z.astype(np.float64)
    for parent in range(b1):
        kids = [c for c in range(parent * b2, (parent + 1) * b2) if np.any(h == c)]
        means = np.stack([Zd[h == c].mean(0) for c in kids])
        mem = np.flatnonzero(h // b2 == parent)
        D = ((Zd[mem][:, None, :] - means[None]) ** 2).sum(-1)
        own = np.array([kids.index(c) for c in h[mem]])
        assert np.all(D[np.arange(len(mem)), own] <= D.min(1) + 1e-9)


def test_crosspolytope_and_construction():
    """AND construction: two points share a band's bucket iff all r hashes of the band agree; one
    hash is the plain cross-polytope hash."""
    rng = np.random.default_rng(14)
    Z = rng.standard_normal((500, 10)).astype(np.float32)
    P = rng.standard_normal((3, 10, 4)).astype(np.float32)
    b = 8
    hs = [oracle.crosspolytope(Z, P[j], b) for j in range(3)]
    np.testing.assert_array_equal(oracle.crosspolytope_and(Z, P[:1], b), hs[0])
    band = oracle.crosspolytope_and(Z, P, b)
    assert band.max() < b ** 3
    same = band[:, None] == band[None, :]
    allsame = np.ones_like(same)
    for hj in hs:
        allsame &= hj[:, None] == hj[None, :]
    np.testing.assert_array_equal(same, allsame)
    # fewer neighbours than a single hash: the pattern of the band is the intersection
    n = 250
    B1 = oracle.hash_rounds(Z, 1, b, 1, 0, 0, projections=P[:1])
    B3 = oracle.hash_rounds(Z, 1, b, 1, 0, 0, projections=P, and_width=3)
    r1, c1 = oracle.pattern(B1, n, n)
    r3, c3 = oracle.pattern(B3, n, n)
    s1 = {(i, j) for i in range(n) for j in c1[r1[i]:r1[i + 1]]}
    s3 = {(i, j) for i in range(n) for j in c3[r3[i]:r3[i + 1]]}
    assert s3 <= s1 and len(s3) < len(s1)
