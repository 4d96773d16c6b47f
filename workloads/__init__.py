"""Seeded synthetic inputs for the five benchmark configurations.

This module only *draws inputs* (point sets, marginals, the regularisation
value handed to both sides, random projections for cross-polytope hashing).
It holds none of the method's arithmetic: no hashing, no k-means, no Nystrom
factors, no Sinkhorn updates.  The oracle and the HIP path both consume what
is produced here and never import each other.

The inputs stand in for the paper's workloads (word-embedding alignment at
N = 20 000, d = 300, lambda = 0.05 -- Sec. 7 "Approximating Sinkhorn" and
"Embedding alignment"; batches of small graph pairs -- Sec. 6); none of the
paper's datasets is reproduced here.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

BASE_SEED = 210706876

COST_SQEUCLID = 0
COST_EUCLID = 1
COST_COSINE = 2

HASH_KMEANS = 0
HASH_CROSSPOLYTOPE = 1


@dataclasses.dataclass
class Problem:
    """One optimal-transport problem plus the approximation budget."""
    name: str
    X: np.ndarray            # (n, d) float32
    Y: np.ndarray            # (m, d) float32
    a: np.ndarray            # (n,) float32, sums to 1
    b: np.ndarray            # (m,) float32, sums to 1
    lam: float               # regularisation, already rounded to float32
    cost: int
    num_landmarks: int
    num_buckets: int
    num_rounds: int
    iters: int
    kmeans_iters: int = 10
    landmark_seed: int = 1
    lsh_seed: int = 101
    ridge: float = 0.0
    bf16_inputs: bool = False
    # cross-polytope projections, (rounds, d, buckets/2) float32
    projections: Optional[np.ndarray] = None
    # start of the landmark k-means: "sample", "kmeans++" or an (l, d) float32 array; its
    # iteration count if it differs from kmeans_iters (0: the start itself is the landmark set)
    landmark_init: object = "sample"
    landmark_iters: Optional[int] = None
    # hierarchical k-means hashing: branching factors per level (their product is num_buckets)
    branching: Optional[tuple] = None
    # cross-polytope hashing: hashes per band (AND construction); num_buckets is then the bucket
    # count of ONE hash and projections holds num_rounds * and_width matrices
    and_width: int = 1

    @property
    def n(self):
        return self.X.shape[0]

    @property
    def m(self):
        return self.Y.shape[0]

    @property
    def d(self):
        return self.X.shape[1]


def _rng(config_index: int, stream: int = 0):
    return np.random.Generator(np.random.PCG64([BASE_SEED + config_index, stream]))


def _f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def _sq_costs(X, Y):
    X = X.astype(np.float64)
    Y = Y.astype(np.float64)
    return (X * X).sum(1)[:, None] + (Y * Y).sum(1)[None, :] - 2.0 * X @ Y.T


def _random_orthogonal(rng, d):
    q, r = np.linalg.qr(rng.standard_normal((d, d)))
    return q * np.sign(np.diag(r))[None, :]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned
    as float32 holding exactly representable values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def projections(config_index: int, rounds: int, d: int, buckets: int) -> np.ndarray:
    """Gaussian projection matrices for cross-polytope hashing (App. "Choosing
    LSH neighbors and Nystrom landmarks"), one d x b/2 matrix per round."""
    rng = _rng(config_index, 7)
    return _f32(rng.standard_normal((rounds, d, buckets // 2)))


def gaussian_mixture(config_index: int, n: int, d: int, comps: int, sigma: float):
    rng = _rng(config_index, 1)
    centres = rng.standard_normal((comps, d))
    which = rng.integers(0, comps, size=n)
    return centres[which] + sigma * rng.standard_normal((n, d)), centres, rng


def config1(n: int = 1024, d: int = 16) -> Problem:
    """Tiny clustered problem: 8 isotropic Gaussians, squared Euclidean cost."""
    rng = _rng(1, 1)
    centres = rng.standard_normal((8, d))
    X = centres[rng.integers(0, 8, size=n)] + 0.3 * rng.standard_normal((n, d))
    Y = centres[rng.integers(0, 8, size=n)] + 0.3 * rng.standard_normal((n, d))
    Y[:, 0] += 0.5
    X, Y = _f32(X), _f32(Y)
    lam = np.float32(0.05 * np.median(_sq_costs(X, Y)))
    a = _f32(np.full(n, 1.0 / n))
    return Problem("C1", X, Y, a, a.copy(), float(lam), COST_SQEUCLID,
                   num_landmarks=64, num_buckets=16, num_rounds=1, iters=50)


def config2(n: int = 10000, d: int = 64, landmarks: int = 128, buckets: int = 64,
            lam_factor: float = 0.05) -> Problem:
    """Mid-size: 32-component mixture, Y = rotated X plus noise; lambda =
    lam_factor * median cost (0.05 in the benchmark configuration)."""
    rng = _rng(2, 1)
    centres = rng.standard_normal((32, d))
    X = centres[rng.integers(0, 32, size=n)] + 0.5 * rng.standard_normal((n, d))
    Q = _random_orthogonal(rng, d)
    Y = X @ Q + 0.05 * rng.standard_normal((n, d))
    X, Y = _f32(X), _f32(Y)
    # lambda = 0.05 * median cost, the median taken over a seeded sample of pairs
    ns = min(1 << 20, n * n)
    ii = rng.integers(0, n, size=ns)
    jj = rng.integers(0, n, size=ns)
    diff = X[ii].astype(np.float64) - Y[jj].astype(np.float64)
    lam = np.float32(lam_factor * np.median((diff * diff).sum(1)))
    a = _f32(np.full(n, 1.0 / n))
    return Problem("C2", X, Y, a, a.copy(), float(lam), COST_SQEUCLID,
                   num_landmarks=landmarks, num_buckets=buckets, num_rounds=2, iters=100)


def _embedding_like(rng, n, d):
    w = np.arange(1, d + 1, dtype=np.float64) ** -0.5
    g = rng.standard_normal((n, d)) * np.sqrt(w)[None, :]
    return g / np.linalg.norm(g, axis=1, keepdims=True)


def config3(n: int = 20000, d: int = 300, landmarks: int = 256, buckets: int = 128,
            rounds: int = 3, iters: int = 200, config_index: int = 3,
            bf16: bool = False, name: str = "C3", prealigned: bool = False) -> Problem:
    """Embedding-alignment shape: unit vectors with a decaying spectrum,
    Y = X Q + noise with a tenth of the rows replaced, cost 1 - cosine.
    prealigned: Y is rotated back (Y Q^T), so that matched rows are close, as
    after the Procrustes pre-alignment of the paper's word-embedding runs
    (Sec. 8); not one of the benchmark configurations, an accuracy variant."""
    rng = _rng(config_index, 1)
    X = _embedding_like(rng, n, d)
    Q = _random_orthogonal(rng, d)
    Y = X @ Q + 0.02 * rng.standard_normal((n, d))
    repl = rng.choice(n, size=n // 10, replace=False)
    Y[repl] = _embedding_like(rng, repl.size, d)
    if prealigned:
        Y = Y @ Q.T
    Y = Y / np.linalg.norm(Y, axis=1, keepdims=True)
    X, Y = _f32(X), _f32(Y)
    if bf16:
        X, Y = round_to_bf16(X), round_to_bf16(Y)
    a = _f32(np.full(n, 1.0 / n))
    return Problem(name, X, Y, a, a.copy(), float(np.float32(0.05)), COST_COSINE,
                   num_landmarks=landmarks, num_buckets=buckets, num_rounds=rounds,
                   iters=iters, bf16_inputs=bf16,
                   projections=projections(config_index, rounds, d, buckets))


def dball(n: int = 10000, d: int = 16, landmarks: int = 20, buckets: int = 500, iters: int = 300,
          stream: int = 1) -> Problem:
    """Two independent samples, uniform in the unit d-ball, Euclidean cost,
    lambda = 0.05: the one synthetic workload of the paper's accuracy table
    (Sec. 8, Table 1, last column group: 20 landmarks and on average 20
    neighbours for LCN).  Not a benchmark configuration."""
    rng = _rng(7, stream)

    def sample():
        g = rng.standard_normal((n, d))
        g /= np.linalg.norm(g, axis=1, keepdims=True)
        return g * rng.random((n, 1)) ** (1.0 / d)

    X, Y = _f32(sample()), _f32(sample())
    a = _f32(np.full(n, 1.0 / n))
    return Problem("d-ball", X, Y, a, a.copy(), float(np.float32(0.05)), COST_EUCLID,
                   num_landmarks=landmarks, num_buckets=buckets, num_rounds=1, iters=iters)


def config5(n: int = 200000, d: int = 300, landmarks: int = 512, buckets: int = 1024) -> Problem:
    """Large log-linear-only problem; inputs are stored in bfloat16."""
    return config3(n=n, d=d, landmarks=landmarks, buckets=buckets, rounds=3, iters=200,
                   config_index=5, bf16=True, name="C5")


@dataclasses.dataclass
class Batch:
    """A ragged batch of small problems for the bipartite-matching (deletion
    row/column) form of Sec. 6."""
    name: str
    X: np.ndarray            # (sum n_p, d) float32
    Y: np.ndarray            # (sum m_p, d) float32
    x_off: np.ndarray        # (P+1,) int64
    y_off: np.ndarray        # (P+1,) int64
    lam: np.ndarray          # (P,) float32
    del_x: np.ndarray        # (sum n_p,) float32 deletion cost of each X point
    del_y: np.ndarray        # (sum m_p,) float32 deletion cost of each Y point
    cost: int
    num_landmarks: int
    num_buckets: int
    iters: int
    kmeans_iters: int = 10
    landmark_seed: int = 1
    lsh_seed: int = 101
    ridge: float = 0.0

    @property
    def num_problems(self):
        return self.lam.shape[0]


def config4(pairs: int = 1024, d: int = 32, lo: int = 16, hi: int = 64) -> Batch:
    """Many small pairs: node embeddings from a fixed random two-layer tanh
    network, Euclidean cost, deletion cost 1 on both sides."""
    rng = _rng(4, 1)
    W1 = rng.standard_normal((d, d)) / np.sqrt(d)
    W2 = rng.standard_normal((d, d)) / np.sqrt(d)
    b1 = 0.1 * rng.standard_normal(d)
    b2 = 0.1 * rng.standard_normal(d)
    ns = rng.integers(lo, hi + 1, size=pairs)
    ms = rng.integers(lo, hi + 1, size=pairs)
    x_off = np.concatenate([[0], np.cumsum(ns)]).astype(np.int64)
    y_off = np.concatenate([[0], np.cumsum(ms)]).astype(np.int64)

    def embed(count):
        raw = rng.standard_normal((count, d))
        return _f32(np.tanh(np.tanh(raw @ W1 + b1) @ W2 + b2))

    X = embed(int(x_off[-1]))
    Y = embed(int(y_off[-1]))
    lam = np.empty(pairs, dtype=np.float32)
    for p in range(pairs):
        C = np.sqrt(np.maximum(_sq_costs(X[x_off[p]:x_off[p + 1]], Y[y_off[p]:y_off[p + 1]]), 0.0))
        lam[p] = np.float32(0.05 * np.median(C))
    return Batch("C4", X, Y, x_off, y_off, lam,
                 np.ones(X.shape[0], dtype=np.float32), np.ones(Y.shape[0], dtype=np.float32),
                 COST_EUCLID, num_landmarks=8, num_buckets=4, iters=50)


@dataclasses.dataclass
class HeadBatch:
    """Multi-head OT over a ragged batch (Sec. 6): every pair is solved by K
    heads, each on its own linear map of the pair's node embeddings.  Pair p,
    head k (k = 0 .. K-1) is problem p*K + k of `batch`, whose lam, del_x and
    del_y are left for the caller to fill (they are part of the method: the
    head's lambda_k and the learnable deletion costs)."""
    batch: Batch
    heads: int
    base_lam: np.ndarray     # (pairs,) float32
    alpha: np.ndarray        # (K, d) float32 deletion weights of each head
    head_of: np.ndarray      # (P*K,) int32 head index of every problem


def config4_heads(pairs: int = 48, heads: int = 4, d: int = 32) -> HeadBatch:
    """config4's pairs seen through `heads` seeded random linear layers."""
    base = config4(pairs=pairs, d=d)
    rng = _rng(4, 2)
    Wk = rng.standard_normal((heads, d, d)) / np.sqrt(d)
    alpha = _f32(rng.uniform(0.5, 1.5, size=(heads, d)))
    Xs, Ys, xo, yo, head_of = [], [], [0], [0], []
    for p in range(pairs):
        Xp = base.X[base.x_off[p]:base.x_off[p + 1]].astype(np.float64)
        Yp = base.Y[base.y_off[p]:base.y_off[p + 1]].astype(np.float64)
        for k in range(heads):
            Xs.append(_f32(Xp @ Wk[k]))
            Ys.append(_f32(Yp @ Wk[k]))
            xo.append(xo[-1] + len(Xp))
            yo.append(yo[-1] + len(Yp))
            head_of.append(k)
    X, Y = np.concatenate(Xs), np.concatenate(Ys)
    batch = Batch("C4-heads", X, Y, np.asarray(xo, dtype=np.int64), np.asarray(yo, dtype=np.int64),
                  np.zeros(pairs * heads, dtype=np.float32), None, None, COST_EUCLID,
                  num_landmarks=8, num_buckets=4, iters=50)
    # base lambda chosen so that the sharpest head (k = 1) has config4's lambda
    base_lam = _f32(base.lam.astype(np.float64) * 2.0 ** (heads / 2.0 - 1.0))
    return HeadBatch(batch, heads, base_lam, alpha, np.asarray(head_of, dtype=np.int32))


def get(index: int, **kw):
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[index](**kw)
