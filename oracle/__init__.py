"""ctypes front end of the CPU oracle (oracle/lcn_oracle.c).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and the cpu_baseline
leg of bench.py may import this package.  It shares nothing with the HIP
library and never imports it.  The functions here only marshal numpy arrays
into the C routines and chain them in the order of the method (Secs. 2-4, 6).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lcn_oracle.c")
_LIB = os.path.join(_HERE, "liblcn_oracle.so")

COST_SQEUCLID, COST_EUCLID, COST_COSINE = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_cost.restype = ctypes.c_double
        _lib.orc_pattern.restype = ctypes.c_int64
    return _lib


def _p(arr, ctype):
    if arr is None:
        return ctypes.POINTER(ctype)()
    return arr.ctypes.data_as(ctypes.POINTER(ctype))


def _f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def _f64(x):
    return None if x is None else np.ascontiguousarray(x, dtype=np.float64)


F, D, I32, I64 = ctypes.c_float, ctypes.c_double, ctypes.c_int32, ctypes.c_int64


def cost_matrix(X, Y, cost):
    X, Y = _f32(X), _f32(Y)
    C = np.empty((X.shape[0], Y.shape[0]))
    lib().orc_cost_matrix(_p(X, F), I64(X.shape[0]), _p(Y, F), I64(Y.shape[0]), X.shape[1], cost, _p(C, D))
    return C


def gibbs_kernel(X, Y, cost, lam):
    X, Y = _f32(X), _f32(Y)
    K = np.empty((X.shape[0], Y.shape[0]))
    lib().orc_gibbs_kernel(_p(X, F), I64(X.shape[0]), _p(Y, F), I64(Y.shape[0]), X.shape[1], cost, D(lam), _p(K, D))
    return K


def seeded_indices(seed, N, k):
    idx = np.empty(k, dtype=np.int64)
    rc = lib().orc_seeded_indices(ctypes.c_uint64(seed), I64(N), k, _p(idx, I64))
    if rc:
        raise ValueError("seeded_indices: bad arguments")
    return idx


def assign(Z, cent):
    Z, cent = _f32(Z), _f32(cent)
    out = np.empty(Z.shape[0], dtype=np.int32)
    lib().orc_assign(_p(Z, F), I64(Z.shape[0]), Z.shape[1], _p(cent, F), cent.shape[0], _p(out, I32))
    return out


def kmeanspp(Z, k, seed):
    """Indices (int64, k) of the points k-means++ seeding picks (D^2 sampling)."""
    Z = _f32(Z)
    idx = np.empty(k, dtype=np.int64)
    rc = lib().orc_kmeanspp(_p(Z, F), I64(Z.shape[0]), Z.shape[1], k, ctypes.c_uint64(seed), _p(idx, I64))
    if rc:
        raise ValueError("kmeanspp: bad arguments")
    return idx


def kmeans(Z, k, T, seed, init="sample"):
    """Returns (centroids float32 (k, d), assignment int32 (N,)).  init: "sample"
    (k seeded distinct points), "kmeans++" (D^2 sampling; T may be 0: the sampled
    points themselves) or an array of k start centroids."""
    Z = _f32(Z)
    cent = np.empty((k, Z.shape[1]), dtype=np.float32)
    asg = np.empty(Z.shape[0], dtype=np.int32)
    if isinstance(init, str) and init == "sample" and T >= 1:
        rc = lib().orc_kmeans(_p(Z, F), I64(Z.shape[0]), Z.shape[1], k, T, ctypes.c_uint64(seed), _p(cent, F),
                              _p(asg, I32))
    else:
        if isinstance(init, str):
            idx = {"sample": seeded_indices, "kmeans++": lambda s, N, kk: kmeanspp(Z, kk, s)}[init](seed, Z.shape[0], k)
            cent[:] = Z[idx]
        else:
            cent[:] = _f32(init).reshape(k, Z.shape[1])
        rc = lib().orc_lloyd(_p(Z, F), I64(Z.shape[0]), Z.shape[1], k, T, _p(cent, F), _p(asg, I32))
    if rc:
        raise ValueError("kmeans: bad arguments")
    return cent, asg


def crosspolytope(Z, R, b):
    Z, R = _f32(Z), _f32(R)
    assert R.shape == (Z.shape[1], b // 2) and b % 2 == 0
    out = np.empty(Z.shape[0], dtype=np.int32)
    lib().orc_crosspolytope(_p(Z, F), I64(Z.shape[0]), Z.shape[1], _p(R, F), b, _p(out, I32))
    return out


def pattern(buckets, n, m):
    """buckets: (R, n+m) int32.  Returns CSR (rowptr int64, colidx int32)."""
    buckets = np.ascontiguousarray(buckets, dtype=np.int32).reshape(-1, n + m)
    R = buckets.shape[0]
    rowptr = np.zeros(n + 1, dtype=np.int64)
    nnz = lib().orc_pattern(_p(buckets, I32), R, I64(n), I64(m), _p(rowptr, I64), _p(None, I32))
    colidx = np.empty(max(nnz, 1), dtype=np.int32)
    lib().orc_pattern(_p(buckets, I32), R, I64(n), I64(m), _p(rowptr, I64), _p(colidx, I32))
    return rowptr, colidx[:nnz]


def spd_inverse(A):
    A = _f64(A)
    out = np.empty_like(A)
    rc = lib().orc_spd_inverse(_p(A, D), A.shape[0], _p(out, D))
    if rc:
        raise np.linalg.LinAlgError("matrix is not positive definite")
    return out


def nystrom(X, Y, L, cost, lam, ridge=0.0):
    """Returns (U (n, l), W (l, m)) in fp64."""
    X, Y, L = _f32(X), _f32(Y), _f32(L)
    n, m, l = X.shape[0], Y.shape[0], L.shape[0]
    U = np.empty((n, l))
    W = np.empty((l, m))
    rc = lib().orc_nystrom(_p(X, F), I64(n), _p(Y, F), I64(m), X.shape[1], _p(L, F), l, cost, D(lam), D(ridge),
                           _p(U, D), _p(W, D))
    if rc:
        raise np.linalg.LinAlgError("landmark kernel matrix is not positive definite")
    return U, W


def pattern_values(X, Y, cost, lam, rowptr, colidx, U=None, W=None, nystrom_only=False):
    """K^sp on the pattern, or the LCN correction K^sp - (U W) when U, W are given
    (nystrom_only: (U W) on the pattern alone)."""
    X, Y = _f32(X), _f32(Y)
    n, m = X.shape[0], Y.shape[0]
    val = np.empty(max(colidx.shape[0], 1))
    mode = 0 if U is None else (2 if nystrom_only else 1)
    l = 0 if U is None else U.shape[1]
    lib().orc_pattern_values(_p(X, F), _p(Y, F), X.shape[1], cost, D(lam), I64(n), I64(m), _p(rowptr, I64),
                             _p(colidx, I32), mode, _p(_f64(U), D), _p(_f64(W), D), l, _p(val, D))
    return val[:colidx.shape[0]]


@dataclass
class Operator:
    """K~ = Kd + U W + S, any part optional (see orc_op in the C source)."""
    n: int
    m: int
    Kd: Optional[np.ndarray] = None
    U: Optional[np.ndarray] = None
    W: Optional[np.ndarray] = None
    rowptr: Optional[np.ndarray] = None
    colidx: Optional[np.ndarray] = None
    val: Optional[np.ndarray] = None

    def __post_init__(self):
        self.Kd, self.U, self.W, self.val = _f64(self.Kd), _f64(self.U), _f64(self.W), _f64(self.val)

    @property
    def l(self):
        return 0 if self.U is None else self.U.shape[1]

    def _args(self):
        return (I64(self.n), I64(self.m), self.l, _p(self.Kd, D), _p(self.U, D), _p(self.W, D),
                _p(self.rowptr, I64), _p(self.colidx, I32), _p(self.val, D))

    def dense(self):
        """Materialise K~ (small problems only; used by the pins)."""
        K = np.zeros((self.n, self.m))
        if self.Kd is not None:
            K += self.Kd
        if self.U is not None:
            K += self.U @ self.W
        if self.rowptr is not None:
            for i in range(self.n):
                s, e = self.rowptr[i], self.rowptr[i + 1]
                K[i, self.colidx[s:e]] += self.val[s:e]
        return K


@dataclass
class SinkhornState:
    log_u: np.ndarray
    log_v: np.ndarray
    nonpositive: int = 0
    empty_rows: int = 0
    empty_cols: int = 0


def sinkhorn(op: Operator, a, b, iters, state: Optional[SinkhornState] = None) -> SinkhornState:
    a, b = _f64(a), _f64(b)
    if state is None:
        state = SinkhornState(np.zeros(op.n), np.zeros(op.m))
    counts = np.zeros(3, dtype=np.int64)
    lib().orc_sinkhorn(*op._args(), _p(a, D), _p(b, D), int(iters), _p(state.log_u, D), _p(state.log_v, D),
                       _p(counts, I64))
    state.nonpositive += int(counts[0])
    state.empty_rows += int(counts[1])
    state.empty_cols += int(counts[2])
    return state


def backward(op: Operator, lam, state: SinkhornState, ksp=None, knys=None):
    """Derivatives of the distance at the (converged) scalings of `state` (Prop. 1):
    returns (gU n x l, gW l x m, gsp, gnys), entries None where the part is absent.
    ksp / knys: K^sp and K^sp_Nys on the pattern of `op`."""
    l = op.l
    gU = np.empty((op.n, l)) if l else None
    gW = np.empty((l, op.m)) if l else None
    nnz = 0 if op.colidx is None else op.colidx.shape[0]
    ksp, knys = _f64(ksp), _f64(knys)
    gsp = np.empty(max(nnz, 1)) if ksp is not None else None
    gnys = np.empty(max(nnz, 1)) if knys is not None else None
    lib().orc_backward(I64(op.n), I64(op.m), l, _p(op.U, D), _p(op.W, D), _p(op.rowptr, I64), _p(op.colidx, I32),
                       _p(ksp, D), _p(knys, D), D(lam), _p(state.log_u, D), _p(state.log_v, D), _p(gU, D), _p(gW, D),
                       _p(gsp, D), _p(gnys, D))
    return gU, gW, None if gsp is None else gsp[:nnz], None if gnys is None else gnys[:nnz]


def marginals(op: Operator, a, b, lam, state: SinkhornState):
    """Returns (r, c, distance, l1_residual)."""
    a, b = _f64(a), _f64(b)
    r, c = np.empty(op.n), np.empty(op.m)
    dist, resid = D(0.0), D(0.0)
    lib().orc_marginals(*op._args(), _p(a, D), _p(b, D), D(lam), _p(state.log_u, D), _p(state.log_v, D),
                        _p(r, D), _p(c, D), ctypes.byref(dist), ctypes.byref(resid))
    return r, c, dist.value, resid.value


def sinkhorn_bp(op: Operator, kpe, keq, a, b, iters, state: Optional[SinkhornState] = None) -> SinkhornState:
    kpe, keq, a, b = _f64(kpe), _f64(keq), _f64(a), _f64(b)
    N = op.n + op.m
    if state is None:
        state = SinkhornState(np.zeros(N), np.zeros(N))
    counts = np.zeros(3, dtype=np.int64)
    lib().orc_sinkhorn_bp(*op._args(), _p(kpe, D), _p(keq, D), _p(a, D), _p(b, D), int(iters),
                          _p(state.log_u, D), _p(state.log_v, D), _p(counts, I64))
    state.nonpositive += int(counts[0])
    return state


def marginals_bp(op: Operator, kpe, keq, a, b, lam, state: SinkhornState):
    kpe, keq, a, b = _f64(kpe), _f64(keq), _f64(a), _f64(b)
    N = op.n + op.m
    r, c = np.empty(N), np.empty(N)
    dist, resid = D(0.0), D(0.0)
    lib().orc_marginals_bp(*op._args(), _p(kpe, D), _p(keq, D), _p(a, D), _p(b, D), D(lam), _p(state.log_u, D),
                           _p(state.log_v, D), _p(r, D), _p(c, D), ctypes.byref(dist), ctypes.byref(resid))
    return r, c, dist.value, resid.value


def deletion_costs(X, alpha):
    """Deletion cost of every point for learnable unbalanced OT (Sec. 6):
    c_i = || alpha .* x_i ||_2, as float32.  The squares are added in fp64 in
    the order of the dimensions."""
    X, alpha = _f32(X), _f32(alpha)
    s = np.zeros(X.shape[0])
    for k in range(X.shape[1]):
        t = X[:, k].astype(np.float64) * np.float64(alpha[k])
        s = s + t * t
    return np.sqrt(s).astype(np.float32)


def head_lambdas(lam, num_heads):
    """Regularisation of the K heads of multi-head OT (Sec. 6):
    lambda_k = 2^(k - K/2) * lambda for k = 1 .. K, as float32."""
    K = int(num_heads)
    return np.array([np.float32(2.0 ** (k - K / 2.0) * float(np.float32(lam))) for k in range(1, K + 1)],
                    dtype=np.float32)


# ------------------------------------------------------------ whole paths --

@dataclass
class Built:
    """Everything the build stage produces for one problem."""
    mode: str
    op: Operator
    landmarks: Optional[np.ndarray] = None      # (l, d) float32
    buckets: Optional[np.ndarray] = None        # (R, n+m) int32
    extras: dict = field(default_factory=dict)


def hierarchical_kmeans(Z, branching, T, seed):
    """Hierarchical k-means hashing (App. "Choosing LSH neighbors and Nystrom
    landmarks": used instead of flat k-means for large inputs).  Level 0 is
    k-means with branching[0] clusters on all points; level j >= 1 runs a
    separate k-means with branching[j] clusters inside every cluster of level
    j-1 (on its members in index order; with fewer members than branching[j],
    one cluster per member).  bucket = parent * branching[j] + child.  Seeds
    (this build's reading): level 0 uses `seed`, cluster `parent` of level j uses
    seed + j * 2^32 + parent.  Returns int32 bucket ids < prod(branching)."""
    Z = _f32(Z)
    ids = np.zeros(Z.shape[0], dtype=np.int64)
    parents = 1
    for level, b in enumerate(branching):
        new = np.empty_like(ids)
        for parent in range(parents):
            members = np.flatnonzero(ids == parent)
            if members.size == 0:
                continue
            k = min(int(b), members.size)
            s = seed if level == 0 else seed + (level << 32) + parent
            _, asg = kmeans(Z[members], k, T, s)
            new[members] = parent * int(b) + asg
        ids = new
        parents *= int(b)
    return ids.astype(np.int32)


def crosspolytope_and(Z, projections, b):
    """AND construction (App. "Choosing LSH neighbors and Nystrom landmarks"):
    a band of r cross-polytope hashes matches only if all r do, i.e. the band's
    bucket is the tuple (h_1 .. h_r), numbered h_1 * b^(r-1) + .. + h_r.
    projections: (r, d, b/2)."""
    out = np.zeros(Z.shape[0], dtype=np.int64)
    for j in range(projections.shape[0]):
        out = out * b + crosspolytope(Z, projections[j], b)
    return out.astype(np.int32)


def hash_rounds(Z, hash_kind, num_buckets, num_rounds, kmeans_iters, seed, projections=None, branching=None,
                and_width=1):
    """Bucket ids of every point of Z = [X; Y] for each hash round (Sec. 3).
    Round r of k-means LSH is a fresh (hierarchical, if `branching` is given)
    k-means run seeded with seed + r; round r of cross-polytope LSH uses
    projections[r] (with the AND construction projections[r*w : (r+1)*w] and
    num_buckets is the bucket count of ONE hash)."""
    out = np.empty((num_rounds, Z.shape[0]), dtype=np.int32)
    for r in range(num_rounds):
        if hash_kind == 0:
            if branching:
                out[r] = hierarchical_kmeans(Z, branching, kmeans_iters, seed + r)
            else:
                _, out[r] = kmeans(Z, num_buckets, kmeans_iters, seed + r)
        elif and_width > 1:
            out[r] = crosspolytope_and(Z, projections[r * and_width:(r + 1) * and_width], num_buckets)
        else:
            out[r] = crosspolytope(Z, projections[r], num_buckets)
    return out


def build_problem(X, Y, cost, lam, mode, num_landmarks=0, landmark_seed=1, kmeans_iters=10, ridge=0.0,
                  hash_kind=0, num_buckets=0, num_rounds=0, lsh_seed=101, projections=None,
                  landmark_init="sample", landmark_iters=None, branching=None, and_width=1) -> Built:
    """The build stage of one path: mode in {"dense", "sparse", "nystrom", "lcn"}."""
    X, Y = _f32(X), _f32(Y)
    n, m = X.shape[0], Y.shape[0]
    Z = np.concatenate([X, Y], axis=0)
    if mode == "dense":
        return Built(mode, Operator(n, m, Kd=gibbs_kernel(X, Y, cost, lam)))
    L = U = W = None
    buckets = rowptr = colidx = val = None
    if mode in ("nystrom", "lcn"):
        L, _ = kmeans(Z, num_landmarks, kmeans_iters if landmark_iters is None else landmark_iters, landmark_seed,
                      init=landmark_init)
        U, W = nystrom(X, Y, L, cost, lam, ridge)
    if mode in ("sparse", "lcn"):
        buckets = hash_rounds(Z, hash_kind, num_buckets, num_rounds, kmeans_iters, lsh_seed, projections,
                              branching=branching, and_width=and_width)
        rowptr, colidx = pattern(buckets, n, m)
        val = pattern_values(X, Y, cost, lam, rowptr, colidx, U, W)
    return Built(mode, Operator(n, m, U=U, W=W, rowptr=rowptr, colidx=colidx, val=val), L, buckets)
