/*
 * CPU oracle for dense, sparse (LSH), Nystrom and LCN Sinkhorn.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 restatement of what
 * the method computes, written from the paper, and it shares no code with the
 * HIP library.  Only the tests, the smoke check and the cpu_baseline leg of
 * the benchmark may call it; the product never does.
 *
 * Every loop follows the definition it cites; there is no blocking, fusion or
 * reordering.  OpenMP is used over independent rows only.
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC  (no fast-math: the
 * bucket rule below depends on IEEE evaluation in the written order).
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py to
 * closed forms, invariants or brute force, except the values that a fixed
 * number of Sinkhorn iterations reaches on the synthetic workloads, which the
 * paper does not print ("parity unpinned" by the paper for those values; the
 * iteration itself is pinned through its fixed point and closed forms).
 *
 * Conventions (paper notation -> here): X_p,X_q -> X (n x d), Y (m x d);
 * p,q -> a,b; s,t -> u,v (kept as natural logs); U,A,V as in Sec. 4 with
 * W = A^{-1} V.  All matrices are row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { COST_SQEUCLID = 0, COST_EUCLID = 1, COST_COSINE = 2 };

/* ---------------------------------------------------------------- costs -- */

/* Ground cost c(x, y) (Sec. 2; the costs the experiments use: L2 and its
 * square, and cosine for word embeddings, App. "Choosing LSH neighbors and
 * Nystrom landmarks"). */
double orc_cost(const float *x, const float *y, int d, int cost)
{
    if (cost == COST_COSINE) {
        double xy = 0.0, xx = 0.0, yy = 0.0;
        for (int k = 0; k < d; ++k) {
            xy += (double)x[k] * (double)y[k];
            xx += (double)x[k] * (double)x[k];
            yy += (double)y[k] * (double)y[k];
        }
        return 1.0 - xy / (sqrt(xx) * sqrt(yy));
    }
    double s = 0.0;
    for (int k = 0; k < d; ++k) {
        double t = (double)x[k] - (double)y[k];
        s += t * t;
    }
    return cost == COST_EUCLID ? sqrt(s) : s;
}

/* C_ij = c(x_i, y_j) (Sec. 2). */
void orc_cost_matrix(const float *X, int64_t n, const float *Y, int64_t m, int d, int cost, double *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            C[i * m + j] = orc_cost(X + i * d, Y + j * d, d, cost);
}

/* Gibbs kernel K_ij = exp(-C_ij / lambda) (Sec. 2). */
void orc_gibbs_kernel(const float *X, int64_t n, const float *Y, int64_t m, int d, int cost, double lambda, double *K)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            K[i * m + j] = exp(-orc_cost(X + i * d, Y + j * d, d, cost) / lambda);
}

/* ------------------------------------------------- seeded index choice -- */

/* splitmix64 (Steele, Lea & Flood 2014), the counter-based generator both
 * sides implement for the k-means start. */
static uint64_t splitmix64(uint64_t *state)
{
    uint64_t z = (*state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* k distinct indices out of 0..N-1: the first k steps of a Fisher-Yates
 * shuffle of the identity, step t swapping slot t with slot
 * t + (next() mod (N - t)).  The paper only says "k-means"; this start is this
 * build's reading and is integer-only so both sides agree exactly. */
int orc_seeded_indices(uint64_t seed, int64_t N, int k, int64_t *idx)
{
    if (k > N || k < 0) return 1;
    int64_t *perm = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    if (!perm) return 2;
    for (int64_t i = 0; i < N; ++i) perm[i] = i;
    uint64_t s = seed;
    for (int t = 0; t < k; ++t) {
        int64_t j = t + (int64_t)(splitmix64(&s) % (uint64_t)(N - t));
        int64_t tmp = perm[t];
        perm[t] = perm[j];
        perm[j] = tmp;
        idx[t] = perm[t];
    }
    free(perm);
    return 0;
}

/* ------------------------------------------------------------- k-means -- */

/* Squared distance used to decide a bucket: fp64, dimensions added left to
 * right, multiply and add as separate IEEE operations. */
static double bucket_sqdist(const float *z, const float *c, int d)
{
    double s = 0.0;
    for (int k = 0; k < d; ++k) {
        double t = (double)z[k] - (double)c[k];
        double t2 = t * t;
        s = s + t2;
    }
    return s;
}

/* Nearest centroid of every point; ties go to the lowest centroid index. */
void orc_assign(const float *Z, int64_t N, int d, const float *cent, int k, int32_t *assign)
{
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < N; ++p) {
        int best = 0;
        double bestD = bucket_sqdist(Z + p * d, cent, d);
        for (int c = 1; c < k; ++c) {
            double D = bucket_sqdist(Z + p * d, cent + (int64_t)c * d, d);
            if (D < bestD) {
                bestD = D;
                best = c;
            }
        }
        assign[p] = best;
    }
}

/* Lloyd's k-means with a fixed number of iterations (Sec. 4 "k-means
 * Nystrom"; Sec. 3 / App. "Choosing LSH neighbors..." "k-means LSH"; App.
 * "Complexity analysis": "k-means with a fixed number of iterations").
 * One iteration = assign every point to its nearest centroid, then move every
 * non-empty cluster's centroid to the mean of its members (an empty cluster
 * keeps its centroid).  The mean is taken from 2^-32 fixed-point sums so that
 * it does not depend on summation order.  Outputs: the centroids after T
 * iterations and the assignment made in iteration T (the clusters whose means
 * those centroids are).  Requires |z| < 2^10, N <= 2^20, T >= 1. */
int orc_lloyd(const float *Z, int64_t N, int d, int k, int T, float *cent, int32_t *assign);

int orc_kmeans(const float *Z, int64_t N, int d, int k, int T, uint64_t seed, float *cent, int32_t *assign)
{
    if (T < 1 || k < 1 || k > N) return 1;
    int64_t *idx = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    if (!idx) return 2;
    if (orc_seeded_indices(seed, N, k, idx)) return 1;
    for (int c = 0; c < k; ++c)
        memcpy(cent + (int64_t)c * d, Z + idx[c] * d, sizeof(float) * (size_t)d);
    free(idx);
    return orc_lloyd(Z, N, d, k, T, cent, assign);
}

/* T Lloyd iterations from the centroids `cent` holds on entry (T = 0 leaves
 * them as they are and only makes the assignment). */
int orc_lloyd(const float *Z, int64_t N, int d, int k, int T, float *cent, int32_t *assign)
{
    if (T < 0 || k < 1) return 1;
    int64_t *sums = (int64_t *)malloc(sizeof(int64_t) * (size_t)k * (size_t)d);
    int64_t *counts = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    if (!sums || !counts) return 2;
    if (T == 0) orc_assign(Z, N, d, cent, k, assign);
    for (int it = 0; it < T; ++it) {
        orc_assign(Z, N, d, cent, k, assign);
        memset(sums, 0, sizeof(int64_t) * (size_t)k * (size_t)d);
        memset(counts, 0, sizeof(int64_t) * (size_t)k);
        for (int64_t p = 0; p < N; ++p) {
            int c = assign[p];
            counts[c] += 1;
            for (int j = 0; j < d; ++j)
                sums[(int64_t)c * d + j] += llrint(ldexp((double)Z[p * d + j], 32));
        }
        for (int c = 0; c < k; ++c) {
            if (counts[c] == 0) continue;
            for (int j = 0; j < d; ++j)
                cent[(int64_t)c * d + j] =
                    (float)(ldexp((double)sums[(int64_t)c * d + j], -32) / (double)counts[c]);
        }
    }
    free(sums);
    free(counts);
    return 0;
}

/* k-means++ seeding ("sampling via k-means++", Sec. 4): the first point is
 * uniform, every further point is drawn with probability proportional to its
 * squared distance w_i to the nearest point chosen so far.  The paper names the
 * method only; this build's reading makes the draw exact integer work so that
 * both sides agree on every index:
 *   - distances by the fp64 bucket rule (left to right, separate multiply and add);
 *   - weights q_i = floor(w_i * 2^(38 - e)), with 4 * max_i |z_i|^2 = f * 2^e,
 *     1/2 <= f < 1 (no distance exceeds that bound, so q_i < 2^39 and the total
 *     of 2^20 points fits 64 bits); a chosen point has weight 0;
 *   - step t takes the t-th output r_t of splitmix64(seed): the first index is
 *     r_0 mod N, later ones the lowest i whose running total q_0 + .. + q_i
 *     exceeds r_t mod (total);
 *   - if the total is 0 (every remaining point coincides with a chosen one) the
 *     lowest index not chosen yet is taken. */
int orc_kmeanspp(const float *Z, int64_t N, int d, int k, uint64_t seed, int64_t *idx)
{
    if (k < 1 || k > N) return 1;
    double *w = (double *)malloc(sizeof(double) * (size_t)N);
    char *chosen = (char *)calloc((size_t)N, 1);
    float *zero = (float *)calloc((size_t)d, sizeof(float));
    if (!w || !chosen || !zero) return 2;
    double m2 = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        double s = bucket_sqdist(Z + i * d, zero, d);
        if (s > m2) m2 = s;
    }
    int e = 0;
    (void)frexp(4.0 * m2, &e);
    const int shift = 38 - e;
    uint64_t st = seed;
    for (int t = 0; t < k; ++t) {
        const uint64_t r = splitmix64(&st);
        int64_t pick = -1;
        if (t == 0) {
            pick = (int64_t)(r % (uint64_t)N);
        } else {
            uint64_t total = 0;
            for (int64_t i = 0; i < N; ++i)
                if (!chosen[i]) total += (uint64_t)floor(ldexp(w[i], shift));
            if (total == 0) {
                for (int64_t i = 0; i < N && pick < 0; ++i)
                    if (!chosen[i]) pick = i;
            } else {
                const uint64_t target = r % total;
                uint64_t run = 0;
                for (int64_t i = 0; i < N && pick < 0; ++i) {
                    if (chosen[i]) continue;
                    run += (uint64_t)floor(ldexp(w[i], shift));
                    if (run > target) pick = i;
                }
            }
        }
        idx[t] = pick;
        chosen[pick] = 1;
        for (int64_t i = 0; i < N; ++i) {
            double s = bucket_sqdist(Z + i * d, Z + pick * d, d);
            if (t == 0 || s < w[i]) w[i] = s;
        }
    }
    free(w);
    free(chosen);
    free(zero);
    return 0;
}

/* Cross-polytope hash h(x) = argmax([x^T R || -x^T R]) with R of shape
 * d x b/2 (App. "Choosing LSH neighbors and Nystrom landmarks").  Projections
 * in fp64, left to right, separate multiply and add; ties to the lowest
 * index. */
void orc_crosspolytope(const float *Z, int64_t N, int d, const float *R, int b, int32_t *bucket)
{
    int h = b / 2;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < N; ++p) {
        int best = -1;
        double bestG = 0.0;
        for (int half = 0; half < 2; ++half) {
            for (int c = 0; c < h; ++c) {
                double g = 0.0;
                for (int k = 0; k < d; ++k) {
                    double t = (double)Z[p * d + k] * (double)R[(int64_t)k * h + c];
                    g = g + t;
                }
                if (half) g = -g;
                if (best < 0 || g > bestG) {
                    bestG = g;
                    best = half * h + c;
                }
            }
        }
        bucket[p] = best;
    }
}

/* ------------------------------------------------------ sparse pattern -- */

/* Pattern of K^sp (Sec. 3): (i, j) is kept iff x_i and y_j share a bucket in
 * at least one of the R hash rounds (the OR over bands of the AND-OR
 * construction with one hash per band, App. "Complexity analysis").
 * bucket is R x (n + m): entry [r][i] for x_i, [r][n + j] for y_j.
 * With colidx == NULL only rowptr is filled.  Returns nnz.  Column indices
 * are ascending within a row. */
int64_t orc_pattern(const int32_t *bucket, int R, int64_t n, int64_t m, int64_t *rowptr, int32_t *colidx)
{
    int64_t N = n + m;
    if (!colidx) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            int64_t cnt = 0;
            for (int64_t j = 0; j < m; ++j) {
                int near = 0;
                for (int r = 0; r < R; ++r)
                    if (bucket[r * N + i] == bucket[r * N + n + j]) near = 1;
                cnt += near;
            }
            rowptr[i + 1] = cnt;
        }
        rowptr[0] = 0;
        for (int64_t i = 0; i < n; ++i) rowptr[i + 1] += rowptr[i];
        return rowptr[n];
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t pos = rowptr[i];
        for (int64_t j = 0; j < m; ++j) {
            int near = 0;
            for (int r = 0; r < R; ++r)
                if (bucket[r * N + i] == bucket[r * N + n + j]) near = 1;
            if (near) colidx[pos++] = (int32_t)j;
        }
    }
    return rowptr[n];
}

/* ----------------------------------------------------- Nystrom factors -- */

/* Inverse of a symmetric positive definite matrix through its Cholesky factor
 * (App. "Implementational details": A^{-1} in double precision; the paper
 * saw no difference between an explicit inverse, Cholesky or a solve).
 * A is l x l and is left untouched.  Returns 1 if a pivot is not positive. */
int orc_spd_inverse(const double *A, int l, double *Ainv)
{
    double *L = (double *)calloc((size_t)l * (size_t)l, sizeof(double));
    double *Li = (double *)calloc((size_t)l * (size_t)l, sizeof(double));
    if (!L || !Li) return 2;
    for (int j = 0; j < l; ++j) {
        double s = A[(int64_t)j * l + j];
        for (int k = 0; k < j; ++k) s -= L[(int64_t)j * l + k] * L[(int64_t)j * l + k];
        if (!(s > 0.0)) {
            free(L);
            free(Li);
            return 1;
        }
        double ljj = sqrt(s);
        L[(int64_t)j * l + j] = ljj;
        for (int i = j + 1; i < l; ++i) {
            double t = A[(int64_t)i * l + j];
            for (int k = 0; k < j; ++k) t -= L[(int64_t)i * l + k] * L[(int64_t)j * l + k];
            L[(int64_t)i * l + j] = t / ljj;
        }
    }
    /* Li = L^{-1} by forward substitution, column by column */
    for (int c = 0; c < l; ++c) {
        for (int i = c; i < l; ++i) {
            double t = (i == c) ? 1.0 : 0.0;
            for (int k = c; k < i; ++k) t -= L[(int64_t)i * l + k] * Li[(int64_t)k * l + c];
            Li[(int64_t)i * l + c] = t / L[(int64_t)i * l + i];
        }
    }
    /* A^{-1} = L^{-T} L^{-1} */
    for (int i = 0; i < l; ++i)
        for (int j = 0; j < l; ++j) {
            double t = 0.0;
            int k0 = i > j ? i : j;
            for (int k = k0; k < l; ++k) t += Li[(int64_t)k * l + i] * Li[(int64_t)k * l + j];
            Ainv[(int64_t)i * l + j] = t;
        }
    free(L);
    free(Li);
    return 0;
}

/* Nystrom factors (Sec. 4): U_ik = k(x_i, l_k), A_kk' = k(l_k, l_k'),
 * V_kj = k(l_k, y_j) with k = exp(-c / lambda); W = (A + ridge I)^{-1} V
 * (App. "Implementational details": W precomputed).  ridge = 0 is the paper;
 * a positive ridge is this build's option for near-singular A.
 * U is n x l, W is l x m.  Returns nonzero if A is not positive definite. */
int orc_nystrom(const float *X, int64_t n, const float *Y, int64_t m, int d, const float *L, int l, int cost,
                double lambda, double ridge, double *U, double *W)
{
    double *A = (double *)malloc(sizeof(double) * (size_t)l * (size_t)l);
    double *Ainv = (double *)malloc(sizeof(double) * (size_t)l * (size_t)l);
    double *V = (double *)malloc(sizeof(double) * (size_t)l * (size_t)m);
    if (!A || !Ainv || !V) return 2;
    for (int i = 0; i < l; ++i)
        for (int j = 0; j < l; ++j)
            A[(int64_t)i * l + j] =
                exp(-orc_cost(L + (int64_t)i * d, L + (int64_t)j * d, d, cost) / lambda) + (i == j ? ridge : 0.0);
    int rc = orc_spd_inverse(A, l, Ainv);
    if (rc) {
        free(A);
        free(Ainv);
        free(V);
        return rc;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int k = 0; k < l; ++k) U[i * l + k] = exp(-orc_cost(X + i * d, L + (int64_t)k * d, d, cost) / lambda);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < l; ++k)
        for (int64_t j = 0; j < m; ++j) V[(int64_t)k * m + j] = exp(-orc_cost(L + (int64_t)k * d, Y + j * d, d, cost) / lambda);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < l; ++k)
        for (int64_t j = 0; j < m; ++j) {
            double t = 0.0;
            for (int q = 0; q < l; ++q) t += Ainv[(int64_t)k * l + q] * V[(int64_t)q * m + j];
            W[(int64_t)k * m + j] = t;
        }
    free(A);
    free(Ainv);
    free(V);
    return 0;
}

/* ------------------------------------------------- sparse kernel values -- */

/* mode 0: K^sp_ij = exp(-c(x_i, y_j) / lambda) on the pattern (Sec. 3).
 * mode 1: the LCN correction K^sp_ij - (U W)_ij on the pattern (Sec. 4,
 * K_LCN = K_Nys + K^sp_Delta).
 * mode 2: the Nystrom value K^sp_Nys,ij = (U W)_ij on the pattern alone. */
void orc_pattern_values(const float *X, const float *Y, int d, int cost, double lambda, int64_t n, int64_t m,
                        const int64_t *rowptr, const int32_t *colidx, int mode, const double *U, const double *W,
                        int l, double *val)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int64_t j = colidx[e];
            double kij = mode == 2 ? 0.0 : exp(-orc_cost(X + i * d, Y + j * d, d, cost) / lambda);
            if (mode >= 1) {
                double nys = 0.0;
                for (int k = 0; k < l; ++k) nys += U[i * l + k] * W[(int64_t)k * m + j];
                kij = mode == 1 ? kij - nys : nys;
            }
            val[e] = kij;
        }
}

/* ------------------------------------------------------------ operator -- */

/* The approximate kernel every Sinkhorn variant multiplies with:
 *   K~ = Kd (dense, Sec. 2)  +  U W (Nystrom, Sec. 4)  +  S (sparse values on
 * a CSR pattern: K^sp for sparse Sinkhorn, K^sp_Delta for LCN).
 * Any of the three parts may be absent (NULL / l = 0). */
typedef struct {
    int64_t n, m;
    int l;
    const double *Kd;
    const double *U, *W;
    const int64_t *rowptr;
    const int32_t *colidx;
    const double *val;
} orc_op;

/* out = K~ t, evaluated as U (W t) + S t, never forming K~ (Sec. 4,
 * "LCN-Sinkhorn"). */
static void op_apply(const orc_op *op, const double *t, double *out)
{
    int64_t n = op->n, m = op->m;
    int l = op->l;
    double *y = (double *)calloc((size_t)(l > 0 ? l : 1), sizeof(double));
    for (int k = 0; k < l; ++k) {
        double s = 0.0;
        for (int64_t j = 0; j < m; ++j) s += op->W[(int64_t)k * m + j] * t[j];
        y[k] = s;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        if (op->Kd)
            for (int64_t j = 0; j < m; ++j) s += op->Kd[i * m + j] * t[j];
        for (int k = 0; k < l; ++k) s += op->U[i * l + k] * y[k];
        if (op->rowptr)
            for (int64_t e = op->rowptr[i]; e < op->rowptr[i + 1]; ++e) s += op->val[e] * t[op->colidx[e]];
        out[i] = s;
    }
    free(y);
}

/* out = K~^T s, evaluated as W^T (U^T s) + S^T s. */
static void op_apply_t(const orc_op *op, const double *s, double *out)
{
    int64_t n = op->n, m = op->m;
    int l = op->l;
    double *z = (double *)calloc((size_t)(l > 0 ? l : 1), sizeof(double));
    for (int64_t i = 0; i < n; ++i)
        for (int k = 0; k < l; ++k) z[k] += op->U[i * l + k] * s[i];
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j) {
        double acc = 0.0;
        if (op->Kd)
            for (int64_t i = 0; i < n; ++i) acc += op->Kd[i * m + j] * s[i];
        for (int k = 0; k < l; ++k) acc += op->W[(int64_t)k * m + j] * z[k];
        out[j] = acc;
    }
    if (op->rowptr)
        for (int64_t i = 0; i < n; ++i)
            for (int64_t e = op->rowptr[i]; e < op->rowptr[i + 1]; ++e) out[op->colidx[e]] += op->val[e] * s[i];
    free(z);
}

static double vec_max(const double *x, int64_t n)
{
    double mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i)
        if (x[i] > mx) mx = x[i];
    return isfinite(mx) ? mx : 0.0;
}

/* log of (K~ exp(log_in)) per row (or of the transpose per column) for a
 * kernel without signed parts (dense K or sparse K^sp): the log-sum-exp
 * trick of App. "Implementational details", log sum_j exp(x_j) = max_j x_j +
 * log sum_j exp(x_j - max_j x_j) with x_j = log K_ij + log_in_j, so that
 * nothing over- or underflows however far the scalings drift.  A row/column
 * without any non-zero term gives -inf. */
static void lse_apply(const orc_op *op, int transpose, const double *log_in, double *out)
{
    int64_t n = op->n, m = op->m;
    int64_t n_out = transpose ? m : n;
    double *mx = (double *)malloc(sizeof(double) * (size_t)n_out);
    double *sm = (double *)malloc(sizeof(double) * (size_t)n_out);
    for (int64_t o = 0; o < n_out; ++o) {
        mx[o] = -INFINITY;
        sm[o] = 0.0;
    }
    /* pass 0 finds max_j x_j of every output, pass 1 adds exp(x_j - max) */
    for (int pass = 0; pass < 2; ++pass) {
        if (op->Kd) {
#pragma omp parallel for schedule(static)
            for (int64_t o = 0; o < n_out; ++o) {
                int64_t cnt = transpose ? n : m;
                for (int64_t q = 0; q < cnt; ++q) {
                    double k = transpose ? op->Kd[q * m + o] : op->Kd[o * m + q];
                    if (!(k > 0.0)) continue;
                    double x = log(k) + log_in[q];
                    if (pass == 0) {
                        if (x > mx[o]) mx[o] = x;
                    } else if (x > -INFINITY) {
                        sm[o] += exp(x - mx[o]);
                    }
                }
            }
        }
        if (op->rowptr) {
            for (int64_t i = 0; i < n; ++i)
                for (int64_t e = op->rowptr[i]; e < op->rowptr[i + 1]; ++e) {
                    double k = op->val[e];
                    if (!(k > 0.0)) continue;
                    int64_t j = op->colidx[e];
                    int64_t o = transpose ? j : i;
                    double x = log(k) + log_in[transpose ? i : j];
                    if (pass == 0) {
                        if (x > mx[o]) mx[o] = x;
                    } else if (x > -INFINITY) {
                        sm[o] += exp(x - mx[o]);
                    }
                }
        }
    }
    for (int64_t o = 0; o < n_out; ++o) out[o] = sm[o] > 0.0 ? mx[o] + log(sm[o]) : -INFINITY;
    free(mx);
    free(sm);
}

/* One scaling update in log form: out_i = log(marg_i) - log(sum_i) where
 * sum = K~ exp(log_in) (or its transpose).
 * Kernels without signed parts (dense, sparse) go through lse_apply.  With a
 * Nystrom part (Nystrom, LCN) K~ has signed entries and cannot itself be kept
 * as logs (App. "Limitations": A^{-1} cannot be done in log space); there the
 * max-shift of the log-sum-exp trick is applied once per vector: the largest
 * exponent of log_in is taken out before the products are formed.
 * A row/column of the sparse kernel without any entry (App. "Limitations")
 * gives log scaling -inf, i.e. the point carries no mass, and is counted in
 * *empty.  A non-positive sum (possible for Nystrom/LCN, App. "Limitations")
 * is counted in *nonpos and yields NaN. */
static void scaling_update(const orc_op *op, int transpose, const double *log_in, int64_t n_in, const double *marg,
                           int64_t n_out, double *log_out, int64_t *nonpos, int64_t *empty)
{
    if (op->l == 0) {
        double *ls = (double *)malloc(sizeof(double) * (size_t)n_out);
        lse_apply(op, transpose, log_in, ls);
        for (int64_t i = 0; i < n_out; ++i) {
            if (ls[i] > -INFINITY) {
                log_out[i] = log(marg[i]) - ls[i];
            } else {
                log_out[i] = -INFINITY;
                *empty += 1;
            }
        }
        free(ls);
        return;
    }
    double M = vec_max(log_in, n_in);
    double *lin = (double *)malloc(sizeof(double) * (size_t)n_in);
    double *sum = (double *)malloc(sizeof(double) * (size_t)n_out);
    for (int64_t j = 0; j < n_in; ++j) lin[j] = exp(log_in[j] - M);
    if (transpose)
        op_apply_t(op, lin, sum);
    else
        op_apply(op, lin, sum);
    for (int64_t i = 0; i < n_out; ++i) {
        if (sum[i] > 0.0) {
            log_out[i] = log(marg[i]) - log(sum[i]) - M;
        } else {
            log_out[i] = NAN;
            *nonpos += 1;
        }
    }
    free(lin);
    free(sum);
}

static orc_op make_op(int64_t n, int64_t m, int l, const double *Kd, const double *U, const double *W,
                      const int64_t *rowptr, const int32_t *colidx, const double *val)
{
    orc_op op;
    op.n = n;
    op.m = m;
    op.l = l;
    op.Kd = Kd;
    op.U = U;
    op.W = W;
    op.rowptr = rowptr;
    op.colidx = colidx;
    op.val = val;
    return op;
}

/* Sinkhorn iterations (Sec. 2, eq. 2): starting from the given log v (the
 * paper starts at t = 1, i.e. log v = 0), repeat iters times
 *     u = a ./ (K~ v),   v = b ./ (K~^T u).
 * log_u, log_v are in/out (log_u is overwritten before it is read).
 * counts[0] accumulates non-positive sums, counts[1] rows and counts[2]
 * columns without any kernel entry, over all iterations. */
void orc_sinkhorn(int64_t n, int64_t m, int l, const double *Kd, const double *U, const double *W,
                  const int64_t *rowptr, const int32_t *colidx, const double *val, const double *a, const double *b,
                  int iters, double *log_u, double *log_v, int64_t *counts)
{
    orc_op op = make_op(n, m, l, Kd, U, W, rowptr, colidx, val);
    for (int it = 0; it < iters; ++it) {
        scaling_update(&op, 0, log_v, m, a, n, log_u, &counts[0], &counts[1]);
        scaling_update(&op, 1, log_u, n, b, m, log_v, &counts[0], &counts[2]);
    }
}

/* Marginals of the current plan P = diag(u) K~ diag(v):  r = u .* (K~ v),
 * c = v .* (K~^T u); the Sinkhorn distance
 *     d = <P, C> - lambda H(P) = lambda (sum_i r_i log u_i + sum_j c_j log v_j)
 * (Sec. 2 eq. 1 rewritten with C_ij = lambda (log u_i + log v_j - log P_ij);
 * Sec. 4 eq. 5 is this expression for the decomposed plan, its s and t read
 * as the log scalings the implementation stores); and the stopping quantity
 * ||r - a||_1 + ||c - b||_1 of Thm. 3 / Thm. 4.  Points with log scaling -inf
 * carry no mass and contribute nothing. */
void orc_marginals(int64_t n, int64_t m, int l, const double *Kd, const double *U, const double *W,
                   const int64_t *rowptr, const int32_t *colidx, const double *val, const double *a, const double *b,
                   double lambda, const double *log_u, const double *log_v, double *r, double *c, double *dist,
                   double *resid)
{
    orc_op op = make_op(n, m, l, Kd, U, W, rowptr, colidx, val);
    double D = 0.0, E = 0.0;
    if (l == 0) { /* kernels without signed parts: everything stays in logs */
        double *lr = (double *)malloc(sizeof(double) * (size_t)n);
        double *lc = (double *)malloc(sizeof(double) * (size_t)m);
        lse_apply(&op, 0, log_v, lr);
        lse_apply(&op, 1, log_u, lc);
        for (int64_t i = 0; i < n; ++i) {
            r[i] = (isinf(log_u[i]) || isinf(lr[i])) ? 0.0 : exp(log_u[i] + lr[i]);
            if (r[i] != 0.0) D += r[i] * log_u[i];
            E += fabs(r[i] - a[i]);
        }
        for (int64_t j = 0; j < m; ++j) {
            c[j] = (isinf(log_v[j]) || isinf(lc[j])) ? 0.0 : exp(log_v[j] + lc[j]);
            if (c[j] != 0.0) D += c[j] * log_v[j];
            E += fabs(c[j] - b[j]);
        }
        free(lr);
        free(lc);
        *dist = lambda * D;
        *resid = E;
        return;
    }
    double Mu = vec_max(log_u, n), Mv = vec_max(log_v, m);
    double *ul = (double *)malloc(sizeof(double) * (size_t)n);
    double *vl = (double *)malloc(sizeof(double) * (size_t)m);
    for (int64_t i = 0; i < n; ++i) ul[i] = exp(log_u[i] - Mu);
    for (int64_t j = 0; j < m; ++j) vl[j] = exp(log_v[j] - Mv);
    op_apply(&op, vl, r);
    op_apply_t(&op, ul, c);
    for (int64_t i = 0; i < n; ++i) {
        r[i] = isinf(log_u[i]) ? 0.0 : exp(log_u[i] + Mv) * r[i];
        if (r[i] != 0.0) D += r[i] * log_u[i];
        E += fabs(r[i] - a[i]);
    }
    for (int64_t j = 0; j < m; ++j) {
        c[j] = isinf(log_v[j]) ? 0.0 : exp(log_v[j] + Mu) * c[j];
        if (c[j] != 0.0) D += c[j] * log_v[j];
        E += fabs(c[j] - b[j]);
    }
    free(ul);
    free(vl);
    *dist = lambda * D;
    *resid = E;
}

/* ------------------------------------------------- analytic derivatives -- */

/* Derivatives of the distance at converged scalings (Prop. 1; App. "Proof of
 * Prop. 1"), with the four parts of the decomposed kernel
 *     K_LCN = U W + K^sp - K^sp_Nys   (last two on the pattern)
 * taken as independent variables.  From d d / d C_ij = P_ij (Danskin) and
 * C_ij = -lambda log K_ij:  d d / d K_ij = -lambda P_ij / K_ij = -lambda u_i v_j, so
 *     gU_ik   = -lambda u_i (W v)_k                       (n x l)
 *     gW_kj   = -lambda (U^T u)_k v_j                     (l x m)
 *     gsp_e   = -lambda u_i K^sp_ij v_j      = -lambda P^sp_ij      (w.r.t. log K^sp)
 *     gnys_e  = +lambda u_i K^sp_Nys,ij v_j                (w.r.t. log K^sp_Nys)
 * K^sp_Nys enters K_LCN with a minus sign, hence the plus; the proposition prints a
 * minus there as well, which the finite-difference pin contradicts.
 * ksp / knys: kernel values on the pattern (NULL: that output is skipped).
 * With l = 0 (dense or sparse Sinkhorn: K = K^sp) only gsp is produced, and
 * d d / d C = -gsp / lambda = P is the first line of the proposition. */
void orc_backward(int64_t n, int64_t m, int l, const double *U, const double *W, const int64_t *rowptr,
                  const int32_t *colidx, const double *ksp, const double *knys, double lambda, const double *log_u,
                  const double *log_v, double *gU, double *gW, double *gsp, double *gnys)
{
    if (l > 0) {
        double *y = (double *)calloc((size_t)l, sizeof(double));
        double *z = (double *)calloc((size_t)l, sizeof(double));
        for (int k = 0; k < l; ++k)
            for (int64_t j = 0; j < m; ++j) y[k] += W[(int64_t)k * m + j] * exp(log_v[j]);
        for (int64_t i = 0; i < n; ++i)
            for (int k = 0; k < l; ++k) z[k] += U[i * l + k] * exp(log_u[i]);
        for (int64_t i = 0; i < n; ++i)
            for (int k = 0; k < l; ++k) gU[i * l + k] = -lambda * exp(log_u[i]) * y[k];
        for (int k = 0; k < l; ++k)
            for (int64_t j = 0; j < m; ++j) gW[(int64_t)k * m + j] = -lambda * z[k] * exp(log_v[j]);
        free(y);
        free(z);
    }
    if (rowptr) {
        for (int64_t i = 0; i < n; ++i)
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const double uv = exp(log_u[i] + log_v[colidx[e]]);
                if (ksp) gsp[e] = -lambda * uv * ksp[e];
                if (knys) gnys[e] = lambda * uv * knys[e];
            }
    }
}

/* -------------------------------------- bipartite-matching augmentation -- */

/* Unbalanced OT through the bipartite-matching cost matrix C_BP (Sec. 6): the
 * n x m block is the (approximated) kernel K~; the (p, eps) block is diagonal
 * with kernel values kpe_i = exp(-c_{i,eps} / lambda), the (eps, q) block is
 * diagonal with keq_j = exp(-c_{eps,j} / lambda), and the (eps, eps) block has
 * cost 0, i.e. kernel 1 everywhere.  Rows: n points then m deletion rows;
 * columns: m points then n deletion columns. */
static void bp_apply(const orc_op *op, const double *kpe, const double *keq, const double *t, double *out)
{
    int64_t n = op->n, m = op->m;
    op_apply(op, t, out); /* K t_hat */
    double tail = 0.0;
    for (int64_t i = 0; i < n; ++i) tail += t[m + i];
    for (int64_t i = 0; i < n; ++i) out[i] += kpe[i] * t[m + i];
    for (int64_t j = 0; j < m; ++j) out[n + j] = keq[j] * t[j] + tail;
}

static void bp_apply_t(const orc_op *op, const double *kpe, const double *keq, const double *s, double *out)
{
    int64_t n = op->n, m = op->m;
    op_apply_t(op, s, out); /* K^T s_hat */
    double tail = 0.0;
    for (int64_t j = 0; j < m; ++j) tail += s[n + j];
    for (int64_t j = 0; j < m; ++j) out[j] += keq[j] * s[n + j];
    for (int64_t i = 0; i < n; ++i) out[m + i] = kpe[i] * s[i] + tail;
}

/* Sinkhorn on K_BP.  a, b, log_u, log_v all have length n + m. */
void orc_sinkhorn_bp(int64_t n, int64_t m, int l, const double *Kd, const double *U, const double *W,
                     const int64_t *rowptr, const int32_t *colidx, const double *val, const double *kpe,
                     const double *keq, const double *a, const double *b, int iters, double *log_u, double *log_v,
                     int64_t *counts)
{
    orc_op op = make_op(n, m, l, Kd, U, W, rowptr, colidx, val);
    int64_t N = n + m;
    double *lin = (double *)malloc(sizeof(double) * (size_t)N);
    double *sum = (double *)malloc(sizeof(double) * (size_t)N);
    for (int it = 0; it < iters; ++it) {
        for (int half = 0; half < 2; ++half) {
            const double *lin_log = half ? log_u : log_v;
            double *out_log = half ? log_v : log_u;
            const double *marg = half ? b : a;
            double M = vec_max(lin_log, N);
            for (int64_t j = 0; j < N; ++j) lin[j] = exp(lin_log[j] - M);
            if (half)
                bp_apply_t(&op, kpe, keq, lin, sum);
            else
                bp_apply(&op, kpe, keq, lin, sum);
            for (int64_t i = 0; i < N; ++i) {
                if (sum[i] > 0.0) {
                    out_log[i] = log(marg[i]) - log(sum[i]) - M;
                } else {
                    out_log[i] = NAN;
                    counts[0] += 1;
                }
            }
        }
    }
    free(lin);
    free(sum);
}

/* Marginals, distance and residual of the K_BP plan (as orc_marginals). */
void orc_marginals_bp(int64_t n, int64_t m, int l, const double *Kd, const double *U, const double *W,
                      const int64_t *rowptr, const int32_t *colidx, const double *val, const double *kpe,
                      const double *keq, const double *a, const double *b, double lambda, const double *log_u,
                      const double *log_v, double *r, double *c, double *dist, double *resid)
{
    orc_op op = make_op(n, m, l, Kd, U, W, rowptr, colidx, val);
    int64_t N = n + m;
    double Mu = vec_max(log_u, N), Mv = vec_max(log_v, N);
    double *ul = (double *)malloc(sizeof(double) * (size_t)N);
    double *vl = (double *)malloc(sizeof(double) * (size_t)N);
    for (int64_t i = 0; i < N; ++i) ul[i] = exp(log_u[i] - Mu);
    for (int64_t j = 0; j < N; ++j) vl[j] = exp(log_v[j] - Mv);
    bp_apply(&op, kpe, keq, vl, r);
    bp_apply_t(&op, kpe, keq, ul, c);
    double D = 0.0, E = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        r[i] = exp(log_u[i] + Mv) * r[i];
        D += r[i] * log_u[i];
        E += fabs(r[i] - a[i]);
    }
    for (int64_t j = 0; j < N; ++j) {
        c[j] = exp(log_v[j] + Mu) * c[j];
        D += c[j] * log_v[j];
        E += fabs(c[j] - b[j]);
    }
    *dist = lambda * D;
    *resid = E;
    free(ul);
    free(vl);
}
