/*
 * lcn.h -- C ABI of the MI355X LCN-Sinkhorn library.
 *
 * Entropy-regularised optimal transport between two point sets X (n x d) and
 * Y (m x d) with marginals a, b (Sec. 2 of Gasteiger, Lienen & Guennemann,
 * "Scalable Optimal Transport in High Dimensions ...", ICML 2021), where the
 * Gibbs kernel K = exp(-C / lambda) is replaced by one of
 *     dense    K itself                                   (Sec. 2, eq. 2)
 *     sparse   K^sp: K on pairs that share an LSH bucket  (Sec. 3, eq. 3)
 *     nystrom  K_Nys = U A^{-1} V from l landmarks        (Sec. 4)
 *     lcn      K_LCN = K_Nys + (K^sp - K^sp_Nys)          (Sec. 4)
 * and Sinkhorn's scaling iteration is run on that kernel without ever forming
 * it ("LCN-Sinkhorn", Sec. 4).
 *
 * General conventions
 *   - "device" pointers are HIP device memory on the current device, "host"
 *     pointers ordinary host memory.  All matrices are row-major and dense.
 *   - The caller owns every buffer it passes in, including the workspace, and
 *     must keep the workspace alive and untouched until lcn_destroy.  X, Y, a,
 *     b, the projections and init_centroids are read during lcn_build only
 *     (the build synchronises the stream before it returns, also on error).
 *   - All work is ordered on the HIP stream given to lcn_build (a
 *     hipStream_t passed as void*; NULL = the default stream); during a build
 *     parts of it run on streams of the library's own that fork from and
 *     join that stream through events, enqueued by short-lived host threads
 *     (one of which enqueues on the given stream itself) that end before
 *     lcn_build returns: enqueue nothing on that stream from another thread
 *     while lcn_build runs.  Calls that return host scalars
 *     synchronise that stream.
 *   - Every function returns an lcn_status and never throws or aborts.  On
 *     LCN_ERR_INVALID_ARG nothing has been written or launched, with one
 *     exception: whether the points are finite and inside the range k-means
 *     needs (see lcn_build) is only known once the device has read them, so
 *     that INVALID_ARG comes after the build has used the workspace (no handle
 *     is returned and the caller's inputs are never written).
 *   - Same inputs and seeds give bit-identical landmarks, buckets, block
 *     structure, factors and scalings.
 *   - A handle must not be used from two threads at once.
 */
#ifndef LCN_H
#define LCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lcn_handle_s *lcn_handle; /* opaque; host memory owned by the library */

typedef enum {
    LCN_OK = 0,
    LCN_ERR_INVALID_ARG = 1, /* null pointer, non-positive size/lambda, l > n + m, odd bucket count ... */
    LCN_ERR_ALLOC = 2,       /* workspace too small; *bytes_needed says how much is required */
    LCN_ERR_DEVICE = 3,      /* a HIP call failed, or a sweep gave up its bounded wait for another workgroup's
                                totals; the latter is remembered: every later sinkhorn_run, lcn_get_info and
                                lcn_last_error_counts on the handle returns LCN_ERR_DEVICE, its scalings are
                                not to be used, and only lcn_destroy and a fresh lcn_build recover */
    LCN_ERR_STATE = 4,       /* handle is null, destroyed, or of the wrong kind for this call */
    LCN_ERR_SINGULAR = 5,    /* A (+ ridge I) is not positive definite (App. "Limitations") */
    LCN_ERR_NONPOSITIVE = 6, /* some (K~ v)_i or (K~^T u)_j was <= 0: the Nystrom part is not
                                guaranteed non-negative (App. "Limitations") */
    LCN_WARN_NO_SUPPORT = 7, /* sparse kernel only: some row/column has no entry at all; such points
                                get scaling 0 and carry no mass (App. "Limitations") -- the results
                                are still valid */
    LCN_ERR_RANGE = 8        /* nystrom / lcn: between two iterations some scaling grew by more than e^43
                                relative to its vector's largest entry (the vectors are held as
                                exp(log x - max log x) with the maximum of one iteration earlier, App.
                                "Implementational details"; the sparse part reads single-precision copies
                                that cover e^-131 .. e^43 around that maximum): the results are invalid */
} lcn_status;

typedef enum { LCN_COST_SQEUCLID = 0, LCN_COST_EUCLID = 1, LCN_COST_COSINE = 2 } lcn_cost;
typedef enum { LCN_MODE_DENSE = 0, LCN_MODE_SPARSE = 1, LCN_MODE_NYSTROM = 2, LCN_MODE_LCN = 3 } lcn_mode;
typedef enum { LCN_HASH_KMEANS = 0, LCN_HASH_CROSSPOLYTOPE = 1 } lcn_hash;
typedef enum { LCN_F32 = 0, LCN_BF16 = 1 } lcn_dtype; /* storage type of X and Y only */

typedef enum {
    LCN_INIT_SAMPLE = 0,   /* num_landmarks distinct points by a splitmix64-driven partial Fisher-Yates shuffle */
    LCN_INIT_KMEANSPP = 1, /* k-means++ seeding: D^2 sampling, see below */
    LCN_INIT_GIVEN = 2     /* the caller's init_centroids */
} lcn_landmark_init;

/* Landmarks of the Nystrom part (Sec. 4): Lloyd's k-means on X u Y with a fixed
 * iteration count (App. "Complexity analysis") from the start `init` names;
 * kmeans_iters = 0 takes the start itself -- with LCN_INIT_KMEANSPP that is
 * the paper's "sampling via k-means++" (Sec. 4; App. "Choosing LSH neighbors
 * and Nystrom landmarks"), with LCN_INIT_SAMPLE uniform sampling.
 * LCN_INIT_KMEANSPP: first point r_0 mod (n+m); then, with w_i the squared
 * distance (fp64, dimensions left to right) of point i to the nearest chosen
 * point and q_i = floor(w_i 2^(38-e)) where 4 max|z|^2 = f 2^e, 1/2 <= f < 1,
 * the lowest i with q_0 + .. + q_i > r_t mod (sum q); r_t is the t-th output of
 * splitmix64 from `seed`; if all q are 0 the lowest index not yet chosen.
 * ridge: A + ridge*I is inverted; 0 is the paper's plain inverse.
 * lcn_build_batched supports LCN_INIT_SAMPLE with kmeans_iters >= 1 only. */
typedef struct {
    int32_t num_landmarks; /* l, 1 .. 512, <= n + m */
    int32_t kmeans_iters;  /* >= 0 */
    uint64_t seed;
    double ridge;          /* >= 0 */
    int32_t init;          /* lcn_landmark_init */
    const float *init_centroids; /* device, l x d fp32, read during lcn_build; LCN_INIT_GIVEN only, else NULL */
} lcn_landmark_params;

/* Locality-sensitive hashing of X u Y (Sec. 3; App. "Choosing LSH neighbors
 * and Nystrom landmarks").  Two points are neighbours if they share a bucket
 * in at least one of num_rounds independent hash rounds (OR construction with
 * one hash per band, App. "Complexity analysis").
 *   LCN_HASH_KMEANS: round r = a k-means run with num_buckets clusters and
 *     seed + r; bucket = cluster.  With branching[0] > 0 the run is hierarchical
 *     (used for large inputs): up to three levels whose factors multiply to
 *     num_buckets; level 0 is a k-means with branching[0] clusters on all points,
 *     level j >= 1 runs inside every cluster of level j-1 its own k-means with
 *     branching[j] <= 32 clusters on that cluster's members (in index order;
 *     with fewer members, one cluster per member) seeded with
 *     seed + r + j * 2^32 + parent; bucket = parent * branching[j] + child.
 *   LCN_HASH_CROSSPOLYTOPE: round r = argmax([x^T R_r || -x^T R_r]) with
 *     R_r = projections + r*d*(num_buckets/2), a d x num_buckets/2 row-major
 *     device matrix supplied by the caller; num_buckets must be even.
 *     AND construction (and_width = w > 1): a round is a band of w hashes that
 *     matches only if all w do; hash j of round r uses matrix r*w + j, the
 *     band's bucket is h_0 * b^(w-1) + .. + h_(w-1) with b = num_buckets, and
 *     b^w <= 4096.  The paper advises against it for k-means hashing; it is
 *     rejected there.
 * Ties go to the lowest bucket index. */
typedef struct {
    int32_t hash;         /* lcn_hash */
    int32_t num_buckets;  /* b, 1 .. 4096 (cross-polytope with and_width w: b^w <= 4096) */
    int32_t num_rounds;   /* R, 1 .. 8 */
    int32_t kmeans_iters; /* >= 1 (k-means hashing only) */
    uint64_t seed;
    const float *projections; /* device; cross-polytope only, else NULL */
    int32_t branching[3];     /* hierarchical k-means: factors per level, unused levels 0; all 0: flat */
    int32_t and_width;        /* cross-polytope: hashes per band; 0 or 1: one */
} lcn_lsh_params;

/* Size of a workspace that is certainly enough for everything except the
 * sparse values, plus room for `nnz_guess` sparse entries (pass 0 to get a
 * balanced-bucket guess).  The exact need is only known once the buckets have
 * been built: if lcn_build returns LCN_ERR_ALLOC, call it again with a
 * workspace of at least the *bytes_needed it reported.
 * landmarks / lsh may be NULL for modes that do not use them. */
lcn_status lcn_workspace_bytes(int64_t n, int64_t m, int32_t d, int32_t mode, const lcn_landmark_params *landmarks,
                               const lcn_lsh_params *lsh, int64_t nnz_guess, size_t *bytes);

/* Build the approximate kernel for one problem (Secs. 2-4).
 *   X, Y       device, n x d and m x d (d <= 8192), of type `dtype` (bf16 is widened to fp32 on load)
 *   a, b       device, fp32 marginals of length n and m (positive)
 *   lambda     entropic regularisation (> 0); K = exp(-c / lambda)
 *   cost       lcn_cost; k-means always uses the Euclidean rule on the vectors as given
 *   mode       lcn_mode; landmarks is required for NYSTROM/LCN, lsh for SPARSE/LCN
 *   workspace  device, 256-byte aligned; everything the handle needs lives in it
 *   bytes_needed  host, nullable; set on LCN_OK and on LCN_ERR_ALLOC
 *   out        host; receives the handle (NULL on error)
 * The scalings start at v = 1 (eq. 2).  Points must satisfy |x| < 2^10 and
 * n + m <= 2^20 when k-means is used (its means are summed in 2^-32 fixed
 * point so that they do not depend on summation order).
 * Errors: INVALID_ARG, ALLOC, DEVICE, SINGULAR. */
lcn_status lcn_build(const void *X, int64_t n, const void *Y, int64_t m, int32_t d, int32_t dtype, const float *a,
                     const float *b, float lambda, int32_t cost, int32_t mode, const lcn_landmark_params *landmarks,
                     const lcn_lsh_params *lsh, void *workspace, size_t workspace_bytes, void *hip_stream,
                     size_t *bytes_needed, lcn_handle *out);

/* A ragged batch of small problems (the graph-pair workloads of Sec. 6), all
 * built by one launch (one workgroup per problem) and iterated by one launch
 * (one wavefront per problem).  Problem p owns rows
 * x_off[p] .. x_off[p+1] of X and y_off[p] .. y_off[p+1] of Y (at most 64 each).
 * With deletion costs the problem is the bipartite-matching form of Sec. 6:
 *   C_BP = [[C, diag(c_{p,eps})], [diag(c_{eps,q}), 0]]   ((n+m) x (m+n)),
 * uniform marginals 1/(n+m); without them plain OT with marginals 1/n, 1/m.
 * The LSH / Nystrom approximation applies to the n x m block only. */
typedef struct {
    int32_t num_problems;
    const int64_t *x_off;     /* host, num_problems + 1, x_off[0] = 0 */
    const int64_t *y_off;     /* host, num_problems + 1 */
    const float *lambda;      /* host, one regularisation per problem (> 0) */
    const float *del_cost_x;  /* device, deletion cost c_{i,eps} of every X point, or NULL (both or neither) */
    const float *del_cost_y;  /* device, deletion cost c_{eps,j} of every Y point, or NULL */
} lcn_batch_desc;

/* Build all problems of a batch.  X, Y: device fp32, (sum n_p) x d and
 * (sum m_p) x d, d <= 64; they must stay valid until the build returns.
 * landmarks: l <= 16, problem p uses seed + p; lsh: flat k-means hashing only,
 * buckets <= 16, rounds <= 4, problem p round r uses seed + p*rounds + r.
 * The handle works with sinkhorn_run, transport_cost (writes num_problems
 * doubles), lcn_last_run_timing and lcn_destroy; results per problem come from
 * lcn_batched_results / lcn_batched_get.  Errors as lcn_build. */
lcn_status lcn_build_batched(const float *X, const float *Y, int32_t d, const lcn_batch_desc *desc, int32_t cost,
                             int32_t mode, const lcn_landmark_params *landmarks, const lcn_lsh_params *lsh,
                             void *workspace, size_t workspace_bytes, void *hip_stream, size_t *bytes_needed,
                             lcn_handle *out);
/* Sinkhorn distance and L1 marginal residual of every problem (host arrays of
 * num_problems doubles, nullable) and the plan marginals (device fp32, nullable,
 * problem p at offset x_off[p] + y_off[p], n+m entries with deletion rows). */
lcn_status lcn_batched_results(lcn_handle h, double *dist_host, double *resid_host, float *row_dev, float *col_dev);
/* Per-problem state and structure (device outputs, each nullable): log scalings
 * as fp64 (problem p at offset x_off[p] + y_off[p]), landmarks
 * [num_problems][l][d], bucket ids (problem p: [rounds][n_p + m_p] at
 * rounds * (x_off[p] + y_off[p])), and the 64 x 64 kernel tiles. */
lcn_status lcn_batched_get(lcn_handle h, double *log_u_dev, double *log_v_dev, float *landmarks_dev,
                           int32_t *buckets_dev, float *kernel_dev);

/* Deletion costs of learnable unbalanced OT (Sec. 6): out[i] = || alpha .* x_i ||_2
 * for the `total` rows of X (device fp32, total x d, d >= 1), alpha a device
 * fp32 vector of d weights, out device fp32 of `total` entries (the arrays
 * lcn_batch_desc takes as del_cost_x / del_cost_y).  The squares are added in
 * fp64 in the order of the dimensions, the root is taken in fp64 and rounded
 * to fp32.  Asynchronous on hip_stream; nothing is allocated.  total == 0 is a
 * no-op that reads no pointer; INVALID_ARG for null pointers, total < 0 or d < 1. */
lcn_status lcn_deletion_costs(const float *X, int64_t total, int32_t d, const float *alpha, float *out,
                              void *hip_stream);
/* Regularisation parameters of multi-head OT (Sec. 6): K heads solve the same
 * pair, each on its own embeddings, with lambda_k = 2^(k - K/2) * lambda.
 * Writes out_host[k-1] for k = 1 .. K (host array of K floats).  The heads of a
 * batch are ordinary problems of lcn_build_batched: pair p, head k is problem
 * p*K + (k-1) with its own rows of X and Y, its own lambda and deletion costs.
 * INVALID_ARG unless lambda > 0, 1 <= K <= 64 and every lambda_k is finite and > 0. */
lcn_status lcn_head_lambdas(float lambda, int32_t num_heads, float *out_host);

/* Run `iters` Sinkhorn iterations u = a ./ (K~ v), v = b ./ (K~^T u) (eq. 2),
 * continuing from the current scalings: N then M iterations equal N + M.
 * Returns after the work has finished.  NONPOSITIVE is reported if any sum
 * was <= 0 (the affected scalings are NaN); WARN_NO_SUPPORT if the sparse
 * kernel has empty rows/columns. */
lcn_status sinkhorn_run(lcn_handle h, int32_t iters);

/* Sinkhorn distance of the current plan P = diag(u) K~ diag(v):
 *   d = <P, C> - lambda H(P) = lambda (sum_i r_i log u_i + sum_j c_j log v_j),
 * r = P 1, c = P^T 1 (eq. 1; eq. 5 for the decomposed plan).  Entropy is
 * included, so d may be negative.  d_host: host double. */
lcn_status transport_cost(lcn_handle h, double *d_host);

/* Marginals of the current plan: row_dev (n) = u .* (K~ v), col_dev (m) =
 * v .* (K~^T u) as fp32 device vectors (either may be NULL), and the stopping
 * quantity ||r - a||_1 + ||c - b||_1 of Thm. 3/4 (host double, nullable). */
lcn_status plan_marginals(lcn_handle h, float *row_dev, float *col_dev, double *l1_residual_host);

/* Natural logs of the scalings, fp32 device vectors of length n and m. */
lcn_status lcn_get_scalings(lcn_handle h, float *log_u_dev, float *log_v_dev);
/* Restart from given log v (log u is recomputed by the next iteration; it is
 * stored so that queries see it).  Both device fp32. */
lcn_status lcn_set_scalings(lcn_handle h, const float *log_u_dev, const float *log_v_dev);

/* Structure queries (device outputs). */
lcn_status lcn_get_landmarks(lcn_handle h, float *L_dev /* l x d */);
lcn_status lcn_get_buckets(lcn_handle h, int32_t *bucket_dev /* R x (n + m): x_i at [r][i], y_j at [r][n + j] */);
/* Canonical CSR of the sparse part (pairs sharing a bucket in any round, each
 * once; columns ascending).  Call with colidx_dev == NULL to get *nnz_host and
 * rowptr_dev (n + 1, int64) only.  val_dev (nullable) receives K^sp (sparse,
 * dense modes) or K^sp - K^sp_Nys (lcn mode). */
lcn_status lcn_get_csr(lcn_handle h, int64_t *nnz_host, int64_t *rowptr_dev, int32_t *colidx_dev, float *val_dev);
/* Nystrom factors as stored: U (n x l) and W^T (m x l), fp32 device. */
lcn_status lcn_get_factors(lcn_handle h, float *U_dev, float *Wt_dev);

/* Analytic derivatives of the distance with respect to the parts of the
 * decomposed kernel K_LCN = U W + K^sp - K^sp_Nys, taken as independent
 * variables, at the current scalings (Prop. 1; exact at convergence):
 *   gU_dev   (n x l)   -lambda u_i (W v)_k
 *   gWt_dev  (m x l)   -lambda (U^T u)_k v_j   (the l x m derivative, transposed like W^T in lcn_get_factors)
 *   gsp_dev            -lambda u_i K^sp_ij v_j      w.r.t. log K^sp      (= -lambda P^sp)
 *   gnys_dev           +lambda u_i K^sp_Nys,ij v_j  w.r.t. log K^sp_Nys  (the term enters the kernel negatively)
 * gsp_dev / gnys_dev hold one value per entry of the pattern in the order of
 * lcn_get_csr.  Which outputs exist depends on the mode: lcn all four, nystrom
 * gU and gWt, sparse and dense gsp (for those d d / d C = -gsp / lambda is the
 * plan itself); asking for one that does not exist is LCN_ERR_STATE.  Outputs
 * are device fp32, any may be NULL.  scratch_dev: device memory of at least
 * lcn_backward_scratch_bytes() bytes (0 if no pattern output is requested),
 * 256-byte aligned; too small is LCN_ERR_ALLOC.  Synchronises the stream. */
lcn_status lcn_backward_scratch_bytes(lcn_handle h, size_t *bytes);
lcn_status lcn_backward(lcn_handle h, float *gU_dev, float *gWt_dev, float *gsp_dev, float *gnys_dev,
                        void *scratch_dev, size_t scratch_bytes);

/* lcn_backward for callers that cannot allocate device memory or hand over a
 * scratch buffer: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same outputs, same kernels, same results as
 * lcn_backward; the scratch is an array of LCN_STATIC_SCRATCH_BYTES that the
 * library's device image holds on every GPU it runs on until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine) and still synchronises the handle's stream.  A handle that needs
 * more than the array holds (lcn_backward_scratch_bytes: 8 (n + 1) +
 * 8 (nnz_stored + 64) bytes, rounded up) gets LCN_ERR_ALLOC and nothing is
 * launched.  All calls on one GPU share that GPU's array, whatever their handle
 * or stream, and it keeps the last call's contents: two calls that overlap on
 * one GPU race and corrupt each other's pattern outputs -- serialise them. */
#define LCN_STATIC_SCRATCH_BYTES (32u << 20)
lcn_status lcn_backward_static(lcn_handle h, float *gU_dev, float *gWt_dev, float *gsp_dev, float *gnys_dev);

/* Rows i0 .. i0 + nrows - 1 of the current transport plan P = diag(u) K~ diag(v)
 * (Sec. 2; for the lcn mode the decomposed plan of Sec. 4 eq. 4 written out),
 * as a dense nrows x m block, row-major, device fp32.  For inspection and for
 * plan-quality measures (Sec. 8: correlation and overlap of the largest entries
 * with the exact plan); costs O(nrows m l).  Synchronises the stream. */
lcn_status lcn_plan_rows(lcn_handle h, int64_t i0, int64_t nrows, float *out_dev);

/* Sizes and counters: stored sparse entries (tiles, including pairs that a
 * later round repeats and that are stored as zero), unique pairs, and the
 * numeric-fault counters accumulated since the build. */
typedef struct {
    int64_t n, m;
    int32_t d, l, rounds, buckets;
    int64_t nnz_stored, nnz_unique;
    int64_t nonpositive, empty_rows, empty_cols;
    size_t workspace_used;
    int64_t undecided_last; /* points the MFMA filter left to the exact rule in the last k-means assignment */
} lcn_info;
lcn_status lcn_get_info(lcn_handle h, lcn_info *info_host);

/* The failure modes of App. "Limitations" as counts, accumulated over every
 * sweep since the build (a point that stays unsupported for N iterations is
 * counted N times): sums (K~ v)_i or (K~^T u)_j that were <= 0 although the
 * kernel has signed parts (Nystrom, LCN, or deletion entries: the scaling is
 * NaN and sinkhorn_run returns LCN_ERR_NONPOSITIVE), and rows / columns of a
 * kernel without signed parts (sparse, dense) whose sum was exactly zero
 * because no stored entry reaches them (scaling 0, no mass,
 * LCN_WARN_NO_SUPPORT).  Host outputs, each nullable.  Works on handles of
 * lcn_build and of lcn_build_batched (there: totals over all problems).
 * Synchronises the stream. */
lcn_status lcn_last_error_counts(lcn_handle h, int64_t *nonpositive, int64_t *empty_rows, int64_t *empty_cols);

/* Elapsed GPU time in milliseconds of the kernels of the last sinkhorn_run on
 * this handle, measured with HIP events on the handle's stream, and the
 * number of half-iteration launches it covered (2 per iteration, plus 2 for the
 * first run after a build or lcn_set_scalings, whose first sweep over each side
 * runs twice: once to learn the exponent of its result). */
lcn_status lcn_last_run_timing(lcn_handle h, float *ms_host, int32_t *launches_host);

/* What this part reaches, measured in place (the roofline's practical ceilings;
 * no part of the method).  `what`:
 *   LCN_CAL_COPY_GBS          device-to-device copy of half the workspace into the
 *                             other half, read + write bytes per second, GB/s
 *   LCN_CAL_READ_GBS          read-only sweep over the workspace, GB/s
 *   LCN_CAL_MFMA_BF16_TFLOPS  independent v_mfma_f32_32x32x16_bf16 on registers
 *   LCN_CAL_MFMA_F64_TFLOPS   independent v_mfma_f64_16x16x4_f64 on registers
 *   LCN_CAL_LAUNCH_US         microseconds per launch of an empty kernel in a
 *                             stream of 2000 dependent launches
 * workspace: device, 256-byte aligned, at least 64 MiB, overwritten (larger is
 * better for the two memory figures: what fits the 256 MB last-level cache is
 * served from there).  Runs on the given stream and synchronises it; allocates
 * no device memory.  value_host receives the figure.
 * Errors: INVALID_ARG, DEVICE. */
typedef enum {
    LCN_CAL_COPY_GBS = 0,
    LCN_CAL_READ_GBS = 1,
    LCN_CAL_MFMA_BF16_TFLOPS = 2,
    LCN_CAL_MFMA_F64_TFLOPS = 3,
    LCN_CAL_LAUNCH_US = 4
} lcn_calibration;
lcn_status lcn_calibrate(int32_t what, void *workspace, size_t workspace_bytes, void *hip_stream, double *value_host);

void lcn_destroy(lcn_handle h); /* frees host memory only; the workspace is the caller's */
const char *lcn_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* LCN_H */
