"""GPU parity: the HIP path against the CPU oracle, element by element, on the
same seeded inputs.  Everything goes through the C ABI.  Sizes are those the
oracle finishes in seconds; they span several 64-wide tiles and ragged tails
(n, m, d, l and bucket sizes that are not multiples of 64)."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["lcn", "nystrom", "sparse", "dense"])
def test_config1(mode):
    from parity import compare
    p = workloads.config1()
    out = compare(p, mode)
    print("C1", mode, out, flush=True)


@pytest.mark.parametrize("mode,lam_factor", [("lcn", 0.5), ("nystrom", 0.5), ("sparse", 0.05), ("dense", 0.05),
                                             ("lcn", 0.05)])
def test_config2_reduced(mode, lam_factor):
    """Config 2's recipe (rotated mixture, two hash rounds) at n = m = 1500,
    l = 100, 24 buckets: ragged everywhere.  At the configuration's own
    lambda = 0.05 * median the X and Y clusters are disjoint, the true kernel
    between them is ~e^-20 and the Nystrom error (which has both signs)
    dominates it: the oracle reports non-positive sums and the HIP path must
    report the same.  Numerical parity of the Nystrom/LCN paths on this shape is
    therefore checked at lambda = 0.5 * median."""
    from parity import compare
    p = workloads.config2(n=1500, landmarks=100, buckets=24, lam_factor=lam_factor)
    p.iters = 40
    out = compare(p, mode)
    print("C2r", mode, lam_factor, out, flush=True)


@pytest.mark.parametrize("mode,hash_kind", [("lcn", workloads.HASH_KMEANS), ("sparse", workloads.HASH_CROSSPOLYTOPE),
                                            ("sparse", workloads.HASH_KMEANS), ("nystrom", workloads.HASH_KMEANS)])
def test_config3_reduced(mode, hash_kind):
    """Config 3's recipe (unit vectors, cosine cost, three hash rounds; sparse
    Sinkhorn with cross-polytope hashing as in the paper's word-embedding
    runs) at n = m = 3000, d = 300, l = 96, 20 buckets."""
    from parity import compare
    p = workloads.config3(n=3000, landmarks=96, buckets=20, iters=60)
    out = compare(p, mode, hash_kind)
    print("C3r", mode, hash_kind, out, flush=True)


def test_unequal_sizes_and_marginals():
    """n != m, non-uniform marginals, Euclidean cost, one hash round."""
    from parity import compare
    rng = np.random.default_rng(5)
    p = workloads.config1(n=700, d=9)
    p.Y = p.Y[:450].copy()
    a = rng.random(700) + 0.2
    b = rng.random(450) + 0.2
    p.a = (a / a.sum()).astype(np.float32)
    p.b = (b / b.sum()).astype(np.float32)
    p.cost = workloads.COST_EUCLID
    p.lam = float(np.float32(0.4))
    p.num_landmarks, p.num_buckets, p.iters = 37, 7, 30
    for mode in ("lcn", "sparse", "dense", "nystrom"):
        out = compare(p, mode)
        print("uneq", mode, out, flush=True)


def test_resumable_and_set_scalings():
    """N then M iterations equal N + M bit for bit; restarting from exported
    scalings continues within fp32 rounding of the state."""
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    p = workloads.config1()
    h1 = gpu_build(p, "lcn")
    lcn.sinkhorn_run(h1, 12)
    u1, v1 = lcn.lcn_get_scalings(h1)
    h2 = gpu_build(p, "lcn")
    lcn.sinkhorn_run(h2, 5)
    lcn.sinkhorn_run(h2, 7)
    u2, v2 = lcn.lcn_get_scalings(h2)
    assert torch.equal(u1, u2) and torch.equal(v1, v2)
    h3 = gpu_build(p, "lcn")
    lcn.sinkhorn_run(h3, 5)
    u5, v5 = lcn.lcn_get_scalings(h3)
    h4 = gpu_build(p, "lcn")
    lcn.lcn_set_scalings(h4, u5, v5)
    lcn.sinkhorn_run(h4, 7)
    u4, v4 = lcn.lcn_get_scalings(h4)
    assert (u4 - u1).abs().max().item() < 1e-5 and (v4 - v1).abs().max().item() < 1e-5
    # the build is deterministic: same landmarks, buckets and factors bit for bit
    assert torch.equal(lcn.lcn_get_landmarks(h1), lcn.lcn_get_landmarks(h2))
    assert torch.equal(lcn.lcn_get_buckets(h1), lcn.lcn_get_buckets(h2))
    U1, W1 = lcn.lcn_get_factors(h1)
    U2, W2 = lcn.lcn_get_factors(h2)
    assert torch.equal(U1, U2) and torch.equal(W1, W2)


def test_fused_reduction_matches_separate_launches(monkeypatch):
    """A sweep that adds up its predecessor's partial sums itself gives the
    same bits as a sweep followed by the separate reduction launch, also when
    the iterations are split into runs of 1, 2 and 3 (first, inner and last
    sweep of a run take different paths) and with unequal sides."""
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    r = np.random.default_rng(5)
    pu = workloads.config1()
    pu.X = np.ascontiguousarray(pu.X[:700])
    pu.a = (r.random(700) + 0.5).astype(np.float32)
    pu.a /= pu.a.sum()
    for p in (workloads.config1(), pu,
              workloads.config3(n=3000, d=48, landmarks=96, buckets=12, rounds=3, iters=6, name="C3 reduced")):
        res = {}
        for fused in ("1", "0"):
            monkeypatch.setenv("LCN_FUSED_REDUCE", fused)
            h = gpu_build(p, "lcn")
            lcn.sinkhorn_run(h, 6)
            res[fused] = lcn.lcn_get_scalings(h) + (lcn.transport_cost(h),)
            lcn.lcn_destroy(h)
        assert torch.equal(res["1"][0], res["0"][0]) and torch.equal(res["1"][1], res["0"][1])
        assert res["1"][2] == res["0"][2]
        monkeypatch.setenv("LCN_FUSED_REDUCE", "1")
        h = gpu_build(p, "lcn")
        for k in (1, 2, 3):
            lcn.sinkhorn_run(h, k)
        u, v = lcn.lcn_get_scalings(h)
        assert torch.equal(u, res["1"][0]) and torch.equal(v, res["1"][1])
        lcn.lcn_destroy(h)


def test_filter_plus_exact_rule_equals_exact_rule_everywhere(monkeypatch):
    """Buckets and landmarks decided by the matrix-core filter plus the exact
    rule on the undecided points (over two candidates or over all centroids)
    are those of the exact rule applied to every point; 300 buckets exercise
    the two-candidate path (more than 256 centroids), bf16 input the two-product
    filter, bf16 input with more than 128 centroids its variant with resident points."""
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    cases = (workloads.config1(),
             workloads.config3(n=3000, d=48, landmarks=96, buckets=300, rounds=2, iters=2, name="C3 reduced"),
             workloads.config3(n=2500, d=70, landmarks=64, buckets=24, rounds=2, iters=2, bf16=True,
                               name="C5 reduced"),
             # bf16 input against more than 128 centroids: the filter that keeps the points on chip, with
             # a last group of centroids, a last pass and a last workgroup that are all partly empty
             workloads.config3(n=2500, d=70, landmarks=200, buckets=300, rounds=2, iters=2, bf16=True,
                               name="C5 reduced, many centroids"))
    for p in cases:
        got = {}
        for exact in ("0", "1"):
            monkeypatch.setenv("LCN_EXACT_ASSIGN_ONLY", exact)
            h = gpu_build(p, "lcn")
            got[exact] = (lcn.lcn_get_landmarks(h), lcn.lcn_get_buckets(h), lcn.lcn_get_info(h).undecided_last)
            lcn.lcn_destroy(h)
        assert torch.equal(got["0"][0], got["1"][0]) and torch.equal(got["0"][1], got["1"][1]), p.name
        assert got["1"][2] == 0


@pytest.mark.parametrize("n,d,landmarks,buckets", [
    (70, 8, 129, 130),        # one step of 16 dimensions, one point group past the first workgroup, 129 and 130 centroids
    (129, 24, 140, 200),      # two workgroups, the second with one point
    (1000, 304, 160, 512),    # the widest rows the resident kernel takes (19 steps), two-candidate path
    (1000, 305, 160, 300),    # one dimension more: back to the kernel that streams the points
    (3000, 100, 500, 1000),   # many passes, a last pass with one group of 8 centroids
])
def test_filter_with_resident_points_on_edge_shapes(monkeypatch, n, d, landmarks, buckets):
    """bf16 points against more than 128 centroids (the filter that keeps a workgroup's points in
    LDS): landmarks and buckets equal those of the exact rule applied to every point, on shapes with
    partly empty point groups, centroid groups and passes, and on both sides of its width limit."""
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    p = workloads.config3(n=n, d=d, landmarks=landmarks, buckets=buckets, rounds=1, iters=1, bf16=True,
                          name="bf16 %dx%d" % (n, d))
    got = {}
    for exact in ("0", "1"):
        monkeypatch.setenv("LCN_EXACT_ASSIGN_ONLY", exact)
        h = gpu_build(p, "lcn")
        got[exact] = (lcn.lcn_get_landmarks(h), lcn.lcn_get_buckets(h))
        lcn.lcn_destroy(h)
    assert torch.equal(got["0"][0], got["1"][0]) and torch.equal(got["0"][1], got["1"][1])


def test_config3_full_size():
    """The benchmark configuration itself (n = m = 20 000, d = 300, l = 256,
    128 buckets x 3 rounds, 200 iterations), in the launch configuration
    bench.py times: every landmark, bucket id, CSR entry and scaling is
    compared with the oracle."""
    from parity import compare
    p = workloads.config3()
    out = compare(p, "lcn")
    print("C3 full", out, flush=True)


def test_config2_full_size_dense_and_sparse():
    """Config 2 at full size: the dense 10k x 10k path (the accuracy reference)
    and sparse Sinkhorn against the oracle on a reduced iteration count (the
    dense oracle costs seconds per iteration); LCN at this lambda reports
    non-positive sums on both sides (see test_config2_reduced)."""
    from parity import compare
    p = workloads.config2()
    out = compare(p, "sparse", iters=20)
    print("C2 full sparse", out, flush=True)
    out = compare(p, "lcn", iters=3)
    print("C2 full lcn", out, flush=True)
    out = compare(p, "dense", iters=4)
    print("C2 full dense", out, flush=True)


@pytest.mark.parametrize("iters_l", [0, 3])
def test_landmarks_by_kmeanspp_sampling(iters_l):
    """Landmarks sampled via k-means++ (Sec. 4; the paper's choice for word embeddings), alone
    (0 Lloyd iterations) and as the start of k-means: same points picked on both sides, then
    the usual parity.  Sizes leave ragged tails in the sweep (N = 6000 = 23.4 workgroups of
    256 points, d = 300 = 9.4 chunks of 32)."""
    from parity import compare
    p = workloads.config3(n=3000, landmarks=96, buckets=20, iters=40)
    p.landmark_init, p.landmark_iters = "kmeans++", iters_l
    out = compare(p, "lcn")
    print("C3r kmeans++", iters_l, out, flush=True)
    p = workloads.config1(n=700, d=9)
    p.landmark_init, p.landmark_iters = "kmeans++", iters_l
    out = compare(p, "nystrom")
    print("C1 kmeans++", iters_l, out, flush=True)


def test_kmeanspp_with_repeated_points():
    """More landmarks than distinct points on one side of the draw: once every remaining
    point coincides with a chosen one the lowest unused index is taken.  Checked on the
    picked landmarks only (A is singular by construction, so the build reports that)."""
    import torch
    import oracle
    import paper_2107_06876_amd as lcn
    rng = np.random.default_rng(2)
    base = rng.standard_normal((9, 7)).astype(np.float32)
    X = np.concatenate([base, base, base[:4]])             # 22 points, 9 distinct
    Y = np.concatenate([base[::-1], base[:3]])             # 12 points
    Z = np.concatenate([X, Y])
    for seed in (1, 2, 3):
        want = Z[oracle.kmeanspp(Z, 12, seed)]
        a = torch.full((len(X),), 1.0 / len(X), device="cuda")
        b = torch.full((len(Y),), 1.0 / len(Y), device="cuda")
        lm = dict(num_landmarks=12, kmeans_iters=0, seed=seed, init=lcn.INIT_KMEANSPP, ridge=1e-3)
        h = lcn.lcn_build(torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), a, b, 1.0, lcn.COST_SQEUCLID,
                          lcn.MODE_NYSTROM, landmarks=lm)
        np.testing.assert_array_equal(lcn.lcn_get_landmarks(h).cpu().numpy(), want)
        lcn.lcn_destroy(h)


def test_landmarks_from_given_start():
    """Caller-supplied start centroids for the landmark k-means."""
    from parity import compare
    p = workloads.config1(n=900, d=16)
    rng = np.random.default_rng(9)
    half = p.num_landmarks // 2
    start = np.concatenate([p.X[:half], p.Y[:p.num_landmarks - half]])
    p.landmark_init = (start + 0.05 * rng.standard_normal(start.shape)).astype(np.float32)
    out = compare(p, "lcn")
    print("C1 given start", out, flush=True)


@pytest.mark.parametrize("branching", [(6, 4), (3, 2, 4), (2, 32)])
def test_hierarchical_kmeans_hashing(branching):
    """Hierarchical k-means LSH (App. "Choosing LSH neighbors and Nystrom landmarks"): same bucket
    of every point in every round, then the usual parity.  (2, 32) on 1400 points leaves parents
    whose chunks of 64 members are ragged; config 1 with (3, 2, 4) has three levels."""
    from parity import compare
    p = workloads.config3(n=2000, d=70, landmarks=64, buckets=int(np.prod(branching)), rounds=2, iters=30,
                          name="C3 reduced")
    p.branching = branching
    out = compare(p, "lcn")
    print("C3r hierarchical", branching, out, flush=True)
    p = workloads.config1(n=700, d=9)
    p.num_buckets, p.branching = int(np.prod(branching)), branching
    out = compare(p, "sparse")
    print("C1 hierarchical", branching, out, flush=True)


def test_hierarchical_kmeans_parent_smaller_than_branching():
    """A parent with fewer members than children: one bucket per member."""
    import torch
    import oracle
    import paper_2107_06876_amd as lcn
    rng = np.random.default_rng(6)
    X = np.concatenate([[[0, 0, 0], [1, 0, 0], [0, 1, 0]], 50 + rng.standard_normal((90, 3))]).astype(np.float32)
    Y = (50 + rng.standard_normal((70, 3))).astype(np.float32)
    want = oracle.hash_rounds(np.concatenate([X, Y]), 0, 10, 2, 6, 11, branching=(2, 5))
    a = torch.full((len(X),), 1.0 / len(X), device="cuda")
    b = torch.full((len(Y),), 1.0 / len(Y), device="cuda")
    lsh = dict(num_buckets=10, num_rounds=2, kmeans_iters=6, seed=11, branching=(2, 5))
    h = lcn.lcn_build(torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), a, b, 5.0, lcn.COST_SQEUCLID,
                      lcn.MODE_SPARSE, lsh=lsh)
    np.testing.assert_array_equal(lcn.lcn_get_buckets(h).cpu().numpy(), want)
    lcn.lcn_destroy(h)


@pytest.mark.parametrize("width", [2, 3])
def test_crosspolytope_and_construction(width):
    """AND construction for cross-polytope hashing: a band of `width` hashes, bucket = the tuple."""
    from parity import compare
    p = workloads.config3(n=3000, landmarks=96, buckets=8 if width == 2 else 4, rounds=3, iters=40)
    p.and_width = width
    p.projections = workloads.projections(3, p.num_rounds * width, p.d, p.num_buckets)
    out = compare(p, "sparse", workloads.HASH_CROSSPOLYTOPE)
    print("C3r AND", width, out, flush=True)


def test_landmarks_by_uniform_sampling():
    """Zero Lloyd iterations from the seeded sample: uniform landmark sampling, the baseline the
    paper compares its landmark choices with (Sec. 4)."""
    from parity import compare
    p = workloads.config1(n=700, d=9)
    p.landmark_iters = 0
    out = compare(p, "nystrom")
    print("C1 uniform landmarks", out, flush=True)


def _edge_problem(n, m, d, l, b, R, iters=15):
    rng = np.random.default_rng(0)
    X = rng.standard_normal((n, d)).astype(np.float32)
    Y = (rng.standard_normal((m, d)) + 0.3).astype(np.float32)
    C = ((X[:, None, :].astype(np.float64) - Y[None].astype(np.float64)) ** 2).sum(-1)
    lam = float(np.float32(max(0.5 * np.median(C), 0.1)))
    return workloads.Problem("edge", X, Y, np.full(n, 1.0 / n, np.float32), np.full(m, 1.0 / m, np.float32), lam,
                             workloads.COST_SQEUCLID, l, b, R, iters)


@pytest.mark.parametrize("shape", [(300, 200, 5, 7, 3, 6), (1, 1, 1, 1, 1, 1), (65, 1, 3, 2, 2, 2),
                                   (2, 130, 2, 3, 1, 8), (129, 127, 64, 33, 5, 5)])
@pytest.mark.parametrize("mode", ["lcn", "sparse", "nystrom", "dense"])
def test_edge_shapes(shape, mode):
    """Smallest and most ragged shapes: a single point per side, one landmark, one bucket, a side of
    one point against 65 (the Nystrom part goes negative there: both sides must say so), more
    than four hash rounds (the eight-round code path), sizes one off a multiple of 64."""
    from parity import compare
    out = compare(_edge_problem(*shape), mode)
    print("edge", shape, mode, out, flush=True)


@pytest.mark.parametrize("shape,mode", [((200, 150, 8192, 9, 4, 2), "lcn"), ((2100, 2100, 3, 5, 4096, 1), "lcn"),
                                        ((2100, 2100, 3, 5, 4096, 1), "sparse"), ((300, 300, 1, 3, 2, 1), "lcn")])
def test_limits_of_the_parameters(shape, mode):
    """The largest dimension (8192), the largest bucket count (4096, most of them empty) and a
    single dimension."""
    from parity import compare
    out = compare(_edge_problem(*shape), mode)
    print("limits", shape, mode, out, flush=True)


def test_new_structure_options_on_tiny_inputs():
    """k-means++ picking every point (l = n + m), hierarchical hashing with more leaves than
    points, an AND band on a handful of points."""
    from parity import compare
    p = _edge_problem(3, 2, 4, 5, 1, 1)
    p.landmark_init, p.landmark_iters = "kmeans++", 0
    print("tiny kmeans++", compare(p, "nystrom"), flush=True)
    p = _edge_problem(6, 5, 2, 2, 6, 3)
    p.branching = (2, 3)
    print("tiny hierarchical", compare(p, "sparse"), flush=True)
    p = _edge_problem(9, 7, 3, 2, 2, 2)
    p.and_width = 3
    p.projections = workloads.projections(1, p.num_rounds * 3, p.d, p.num_buckets)
    print("tiny AND", compare(p, "sparse", workloads.HASH_CROSSPOLYTOPE), flush=True)


def test_overlapped_build_gives_the_same_bits(monkeypatch):
    """The build with its k-means runs on streams and host threads of their own against the build
    that keeps everything on the caller's stream: landmarks, buckets, pattern, values, factors and
    the scalings after a few iterations, bit for bit; five builds in a row of the former."""
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    cases = [(workloads.config3(n=3000, d=48, landmarks=96, buckets=12, rounds=3, iters=6, name="C3 reduced"), "lcn", {}),
             (workloads.config1(), "sparse", {}),
             (workloads.config3(n=2000, d=70, landmarks=64, buckets=24, rounds=5, iters=6, name="C3 reduced"), "lcn",
              dict(branching=(6, 4), landmark_init="kmeans++", landmark_iters=2))]
    for p, mode, opts in cases:
        for k, v in opts.items():
            setattr(p, k, v)

        def snapshot():
            h = gpu_build(p, mode)
            lcn.sinkhorn_run(h, 4)
            out = [x.clone() for x in lcn.lcn_get_scalings(h)]
            out.append(lcn.lcn_get_buckets(h).clone())
            out.extend(x.clone() for x in lcn.lcn_get_csr(h))
            if mode == "lcn":
                out.append(lcn.lcn_get_landmarks(h).clone())
                out.extend(x.clone() for x in lcn.lcn_get_factors(h))
            lcn.lcn_destroy(h)
            return out

        monkeypatch.setenv("LCN_BUILD_OVERLAP", "0")
        ref = snapshot()
        monkeypatch.setenv("LCN_BUILD_OVERLAP", "1")
        for _ in range(5):
            got = snapshot()
            assert len(got) == len(ref)
            for a, b in zip(got, ref):
                assert torch.equal(a, b)


def test_build_on_a_stream_of_the_callers_own():
    """A handle built and run on a stream the caller made (the build uses that stream as one of its
    lanes, with a host thread of the library enqueuing on it) against one on the default stream:
    buckets, pattern, factors and scalings bit for bit."""
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    p = workloads.config3(n=3000, d=48, landmarks=96, buckets=12, rounds=3, iters=6, name="C3 reduced")

    def snapshot():
        h = gpu_build(p, "lcn")
        lcn.sinkhorn_run(h, 4)
        out = [x.clone() for x in lcn.lcn_get_scalings(h)]
        out.append(lcn.lcn_get_buckets(h).clone())
        out.extend(x.clone() for x in lcn.lcn_get_csr(h))
        out.append(lcn.lcn_get_landmarks(h).clone())
        out.extend(x.clone() for x in lcn.lcn_get_factors(h))
        d = lcn.transport_cost(h)
        lcn.lcn_destroy(h)
        return out, d

    ref, dref = snapshot()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        got, dgot = snapshot()
    side.synchronize()
    torch.cuda.synchronize()
    assert dgot == dref
    assert len(got) == len(ref)
    for a, b in zip(got, ref):
        assert torch.equal(a, b)


def test_coinciding_landmarks_with_a_ridge():
    """Two landmarks on top of each other make the landmark kernel matrix singular (what either side
    does with it unregularised depends on rounding in the last place); with a ridge both sides invert
    it and the factors agree.  The coinciding pair's distance is exactly zero on both sides."""
    import torch
    import oracle
    import paper_2107_06876_amd as lcn
    rng = np.random.default_rng(11)
    X = rng.standard_normal((40, 6)).astype(np.float32)
    Y = rng.standard_normal((30, 6)).astype(np.float32)
    L = np.concatenate([X[:5], X[2:3], Y[:4]]).astype(np.float32)   # landmark 5 repeats landmark 2
    a = torch.full((len(X),), 1.0 / len(X), device="cuda")
    b = torch.full((len(Y),), 1.0 / len(Y), device="cuda")
    for cost, ocost in ((lcn.COST_SQEUCLID, workloads.COST_SQEUCLID), (lcn.COST_EUCLID, workloads.COST_EUCLID)):
        lm = dict(num_landmarks=len(L), kmeans_iters=0, seed=1, init=lcn.INIT_GIVEN,
                  init_centroids=torch.from_numpy(L).cuda(), ridge=1e-3)
        Uo, Wo = oracle.nystrom(X, Y, L, ocost, 2.0, 1e-3)
        h = lcn.lcn_build(torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), a, b, 2.0, cost, lcn.MODE_NYSTROM,
                          landmarks=lm)
        U, Wt = lcn.lcn_get_factors(h)
        np.testing.assert_allclose(U.cpu().numpy(), Uo, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(Wt.cpu().numpy().T, Wo, rtol=0, atol=1e-6 * np.abs(Wo).max())
        lcn.lcn_destroy(h)


def _two_clusters(counts_x, counts_y, gap, sigma, d=4, seed=7):
    rng = np.random.default_rng(seed)

    def pts(counts):
        out = []
        for c, k in enumerate(counts):
            x = sigma * rng.standard_normal((k, d))
            x[:, 0] += c * gap
            out.append(x)
        return np.concatenate(out).astype(np.float32)

    return pts(counts_x), pts(counts_y)


def test_scalings_spread_beyond_single_precision_range():
    """Scalings that span more than single precision's e^87 and matter (App. "Implementational
    details": log stabilisation).  Two clusters 200 lambda apart: every stored factor and value
    between them is zero, so the kernel is two independent blocks that share only the exponent
    taken out of each scaling vector.  The small block carries marginals of 2e-38 per point and
    starts from log v = 30: its u settles e^110 below the large block's, and the sums of its
    columns consist of such entries only.  The linear sweeps gather single-precision copies
    exp(log x - max) * 2^64, which hold entries down to e^-131 below the largest; unscaled copies
    (floor e^-87, nothing left below e^-103) would leave these sums at zero."""
    import oracle
    import torch
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    X0, Y0 = _two_clusters((64,), (64,), gap=0.0, sigma=0.25, seed=1)
    X1, Y1 = _two_clusters((192,), (192,), gap=0.0, sigma=1.0, seed=2)
    X1[:, 0] += 20.0
    Y1[:, 0] += 20.0
    a = np.concatenate([np.full(64, 2e-38), np.full(192, 1 / 192)]).astype(np.float32)
    p = workloads.Problem("two blocks", np.concatenate([X0, X1]), np.concatenate([Y0, Y1]), a, a.copy(), 2.0,
                          workloads.COST_SQEUCLID, 16, 2, 2, 30)
    lv0 = np.zeros(256, dtype=np.float32)
    lv0[:64] = 30.0
    B = oracle.build_problem(p.X, p.Y, p.cost, p.lam, "lcn", p.num_landmarks, p.landmark_seed, p.kmeans_iters,
                             p.ridge, 0, p.num_buckets, p.num_rounds, p.lsh_seed, None)
    st = oracle.sinkhorn(B.op, p.a, p.b, p.iters, oracle.SinkhornState(np.zeros(256), lv0.astype(np.float64)))
    r_o, c_o, dist_o, resid_o = oracle.marginals(B.op, p.a, p.b, p.lam, st)
    assert st.nonpositive == 0
    spread = np.ptp(st.log_u)
    assert 105.0 < spread < 125.0
    h = gpu_build(p, "lcn")
    np.testing.assert_array_equal(lcn.lcn_get_buckets(h).cpu().numpy(), B.buckets)
    lcn.lcn_set_scalings(h, torch.zeros(256, device="cuda"), torch.from_numpy(lv0).cuda())
    assert lcn.sinkhorn_run(h, p.iters, check=False) == lcn.binding.OK
    lu, lv = (t.cpu().numpy().astype(np.float64) for t in lcn.lcn_get_scalings(h))
    out = dict(spread=spread, log_u=np.abs(lu - st.log_u).max(), log_v=np.abs(lv - st.log_v).max())
    dist = lcn.transport_cost(h)
    r, c, resid = lcn.plan_marginals(h)
    out["cost_rel"] = abs(dist - dist_o) / abs(dist_o)
    out["resid_abs"] = abs(resid - resid_o)
    print("spread", out, flush=True)
    assert out["log_u"] <= 1e-4 and out["log_v"] <= 1e-4 and out["cost_rel"] <= 1e-4 and out["resid_abs"] <= 1e-5, out
    # the small block's marginals are met to their own scale, not only to the large block's
    np.testing.assert_allclose(c.cpu().numpy()[:64], c_o[:64], rtol=1e-4, atol=0)
    np.testing.assert_allclose(r.cpu().numpy()[:64], r_o[:64], rtol=1e-4, atol=0)
    lcn.lcn_destroy(h)


def test_first_sweeps_of_a_fresh_state(monkeypatch):
    """From u = v = 1 the first u is of the order of 1 / (K 1): with a kernel that is e^-60
    everywhere (two tight clusters far apart, one bucket, one landmark -- a rank-one Nystrom part is
    positive) that is e^50 above the exponent the state starts with, more than the copies hold.
    The library runs each side's first sweep of a fresh state twice (first for the exponent);
    with that switched off from the host the same run reports LCN_ERR_RANGE."""
    import paper_2107_06876_amd as lcn
    from parity import compare, gpu_build
    X, Y = _two_clusters((128,), (0, 128), gap=7.75, sigma=0.1)
    u = np.full(128, 1 / 128, np.float32)
    p = workloads.Problem("far apart", X, Y, u, u, 1.0, workloads.COST_SQEUCLID, 1, 1, 1, 12)
    # the landmark lies e^-40 from either cluster, so the Nystrom part (e^-80) stays below the kernel (e^-60)
    p.landmark_init, p.landmark_iters = np.array([[3.875, 5.0, 0.0, 0.0]], dtype=np.float32), 0
    out = compare(p, "lcn")
    print("far apart", out, flush=True)
    assert out["status"] == lcn.binding.OK
    monkeypatch.setenv("LCN_DOUBLE_FIRST_SWEEP", "0")
    h = gpu_build(p, "lcn")
    assert lcn.sinkhorn_run(h, 3, check=False) == lcn.binding.ERR_RANGE
    lcn.lcn_destroy(h)
    monkeypatch.setenv("LCN_DOUBLE_FIRST_SWEEP", "1")
    h = gpu_build(p, "lcn")
    assert lcn.sinkhorn_run(h, 3, check=False) == lcn.binding.OK
    lcn.lcn_destroy(h)


def test_coinciding_landmarks_without_a_ridge_are_singular():
    """The first two landmarks on top of each other and no ridge: A_00 = A_10 = A_11 = exp(0) = 1
    exactly, so the second Cholesky pivot is 1 - 1 * 1 = 0 whatever the order of operations, and
    both sides refuse (App. "Limitations"; LCN_ERR_SINGULAR from the build).  (A repeated landmark
    further down leaves a pivot that is zero only up to rounding: see the test with a ridge.)"""
    import torch
    import oracle
    import paper_2107_06876_amd as lcn
    rng = np.random.default_rng(11)
    X = rng.standard_normal((40, 6)).astype(np.float32)
    Y = rng.standard_normal((30, 6)).astype(np.float32)
    L = np.concatenate([X[:1], X[:1], X[1:5], Y[:4]]).astype(np.float32)   # landmark 1 repeats landmark 0
    a = torch.full((len(X),), 1.0 / len(X), device="cuda")
    b = torch.full((len(Y),), 1.0 / len(Y), device="cuda")
    for cost, ocost in ((lcn.COST_SQEUCLID, workloads.COST_SQEUCLID), (lcn.COST_EUCLID, workloads.COST_EUCLID)):
        with pytest.raises(np.linalg.LinAlgError):
            oracle.nystrom(X, Y, L, ocost, 2.0, 0.0)
        lm = dict(num_landmarks=len(L), kmeans_iters=0, seed=1, init=lcn.INIT_GIVEN,
                  init_centroids=torch.from_numpy(L).cuda(), ridge=0.0)
        with pytest.raises(lcn.LcnError) as err:
            lcn.lcn_build(torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), a, b, 2.0, cost, lcn.MODE_NYSTROM,
                          landmarks=lm)
        assert err.value.status == lcn.binding.ERR_SINGULAR


def test_a_sweep_that_gives_up_its_wait_reports_a_device_error(monkeypatch):
    """The hand-over of a sweep's totals between workgroups is a bounded wait.  With the bound set to
    zero ticks from the host, a workgroup that finds its totals still pending gives up at once:
    every kernel still runs to its end, the run reports LCN_ERR_DEVICE, and the handle stays failed
    (later calls on it keep saying so) while a fresh handle works."""
    import paper_2107_06876_amd as lcn
    from parity import gpu_build
    p = workloads.config3(n=3000, d=48, landmarks=96, buckets=12, rounds=3, iters=6, name="C3 reduced")
    monkeypatch.setenv("LCN_WAIT_TICKS", "0")
    h = gpu_build(p, "lcn")
    assert lcn.sinkhorn_run(h, 20, check=False) == lcn.binding.ERR_DEVICE
    assert lcn.sinkhorn_run(h, 1, check=False) == lcn.binding.ERR_DEVICE
    with pytest.raises(lcn.LcnError) as err:
        lcn.lcn_last_error_counts(h)
    assert err.value.status == lcn.binding.ERR_DEVICE
    lcn.lcn_destroy(h)
    monkeypatch.delenv("LCN_WAIT_TICKS")
    h = gpu_build(p, "lcn")
    assert lcn.sinkhorn_run(h, 20, check=False) == lcn.binding.OK
    lcn.lcn_destroy(h)


def test_a_sweep_grid_larger_than_what_is_resident(monkeypatch):
    """By default a sweep's grid is capped at the workgroups that are resident together.  Raised
    above that from the host (LCN_PASS_GRID), the workgroups beyond start as others finish; the
    hand-over of the totals needs only the first few workgroups of a launch, which are dispatched
    first and wait for nothing, so the bounded wait still ends and the results are the oracle's."""
    from parity import compare
    import paper_2107_06876_amd as lcn
    p = workloads.config3(n=6000, d=64, landmarks=128, buckets=32, rounds=2, iters=20, name="C3 reduced")
    monkeypatch.setenv("LCN_PASS_GRID", "4096")   # 375 workgroups per sweep of 6000 rows
    out = compare(p, "lcn")
    assert out["status"] == lcn.binding.OK
    print("grid above residency", out, flush=True)


@pytest.mark.parametrize("mode,lam_factor", [("lcn", 0.5), ("nystrom", 0.5), ("lcn", 0.1), ("nystrom", 0.1),
                                             ("lcn", 0.075)])
def test_config2_full_size_lcn_and_nystrom(mode, lam_factor):
    """Config 2 at its own size (n = m = 10 000, d = 64, l = 128, 64 buckets x 2 rounds, 100
    iterations) with numbers: at the configuration's lambda = 0.05 * median both sides end in
    non-positive sums (test_config2_full_size_dense_and_sparse), so the Nystrom and LCN paths are
    compared where the oracle stays positive: 0.5 and 0.1 * median for both, and 0.075 * median for
    LCN alone (there the Nystrom part by itself already fails; the correction keeps the sums
    positive)."""
    from parity import compare
    p = workloads.config2(lam_factor=lam_factor)
    out = compare(p, mode)
    print("C2 full", mode, lam_factor, out, flush=True)


@pytest.mark.parametrize("case", ["config1", "config2 reduced", "config3 reduced", "unequal sides", "five rounds",
                                  "ragged", "one by one", "long buckets"])
def test_bucket_shapes(case):
    """More shapes of the bucket blocks against the oracle: blocks of fewer and more than 64 rows,
    more than four hash rounds, a single point per side, buckets of more than 256 members of the
    other side (record segments far longer than a wavefront), empty buckets."""
    from parity import compare
    if case == "config1":
        p = workloads.config1()
    elif case == "config2 reduced":
        p = workloads.config2(n=1500, landmarks=100, buckets=24, lam_factor=0.5)
        p.iters = 40
    elif case == "config3 reduced":
        p = workloads.config3(n=3000, landmarks=96, buckets=20, iters=60)
    elif case == "unequal sides":
        rng = np.random.default_rng(5)
        p = workloads.config1(n=700, d=9)
        p.Y = p.Y[:450].copy()
        b = rng.random(450) + 0.2
        p.b = (b / b.sum()).astype(np.float32)
        p.num_landmarks, p.num_buckets, p.iters = 37, 7, 30
    elif case == "five rounds":
        p = _edge_problem(129, 127, 64, 33, 5, 5)
    elif case == "ragged":
        p = _edge_problem(300, 200, 5, 7, 3, 6)
    elif case == "one by one":
        p = _edge_problem(1, 1, 1, 1, 1, 1)
    else:
        p = workloads.config3(n=2500, d=40, landmarks=64, buckets=3, rounds=2, iters=20, name="C3 reduced")
    out = compare(p, "lcn")
    print("bucket shapes", case, out, flush=True)
