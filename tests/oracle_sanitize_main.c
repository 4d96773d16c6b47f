/*
 * Memory-safety run of the CPU oracle: compiles oracle/lcn_oracle.c into this
 * program with AddressSanitizer and UndefinedBehaviorSanitizer and walks every
 * exported routine through one small problem whose sizes are ragged on purpose
 * (n != m, d odd, landmarks and buckets that do not divide anything), the way
 * oracle/__init__.py chains them.  It checks no numbers -- the pins in
 * test_oracle_pins.py do that -- only that no routine reads or writes outside
 * what its caller sized, leaks, or trips undefined behaviour.  Built and run
 * by tests/test_oracle_sanitizers.py (CPU only).
 */
#include "../oracle/lcn_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 88172645463325252ull;
static double unit_random(void)
{ /* xorshift64: inputs only, none of the method's arithmetic */
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}

#define NEW(type, count) ((type *)malloc(sizeof(type) * (size_t)((count) > 0 ? (count) : 1)))

static int run_problem(int64_t n, int64_t m, int d, int l, int b, int R, int cost)
{
    const int64_t N = n + m;
    float *Z = NEW(float, N * d);
    for (int64_t i = 0; i < N * d; ++i) Z[i] = (float)(2.0 * unit_random() - 1.0 + (i / d >= n ? 0.25 : 0.0));
    const float *X = Z, *Y = Z + n * d;
    const double lambda = 0.8;
    int rc = 0;

    double *C = NEW(double, n * m), *K = NEW(double, n * m);
    orc_cost_matrix(X, n, Y, m, d, cost, C);
    orc_gibbs_kernel(X, n, Y, m, d, cost, lambda, K);

    /* landmarks: seeded sample + Lloyd, k-means++ start, a Lloyd run from given centroids */
    float *L = NEW(float, (int64_t)l * d);
    int32_t *assign = NEW(int32_t, N);
    rc |= orc_kmeans(Z, N, d, l, 3, 5, L, assign);
    int64_t *picks = NEW(int64_t, l);
    rc |= orc_kmeanspp(Z, N, d, l, 9, picks);
    float *L2 = NEW(float, (int64_t)l * d);
    for (int k = 0; k < l; ++k) memcpy(L2 + (int64_t)k * d, Z + picks[k] * d, sizeof(float) * (size_t)d);
    rc |= orc_lloyd(Z, N, d, l, 0, L2, assign);
    rc |= orc_lloyd(Z, N, d, l, 2, L2, assign);
    int64_t *idx = NEW(int64_t, l);
    rc |= orc_seeded_indices(1234567, N, l, idx);

    /* buckets: round 0 by k-means, later rounds by cross-polytope (b even there) */
    int32_t *bucket = NEW(int32_t, (int64_t)R * N);
    float *cent = NEW(float, (int64_t)b * d);
    rc |= orc_kmeans(Z, N, d, b, 2, 101, cent, bucket);
    const int bc = b + (b & 1);
    float *proj = NEW(float, (int64_t)d * (bc / 2));
    for (int r = 1; r < R; ++r) {
        for (int64_t i = 0; i < (int64_t)d * (bc / 2); ++i) proj[i] = (float)(unit_random() - 0.5);
        orc_crosspolytope(Z, N, d, proj, bc, bucket + (int64_t)r * N);
    }
    int64_t *rowptr = NEW(int64_t, n + 1);
    const int64_t nnz = orc_pattern(bucket, R, n, m, rowptr, NULL);
    int32_t *colidx = NEW(int32_t, nnz);
    if (orc_pattern(bucket, R, n, m, rowptr, colidx) != nnz) rc |= 2;

    /* factors, values in the three modes */
    double *U = NEW(double, n * l), *W = NEW(double, (int64_t)l * m);
    rc |= orc_nystrom(X, n, Y, m, d, L, l, cost, lambda, 1e-6, U, W);
    double *A = NEW(double, (int64_t)l * l), *Ainv = NEW(double, (int64_t)l * l);
    for (int p = 0; p < l; ++p)
        for (int q = 0; q < l; ++q)
            A[p * l + q] = exp(-orc_cost(L + (int64_t)p * d, L + (int64_t)q * d, d, cost) / lambda) + (p == q ? 1e-3 : 0.0);
    rc |= orc_spd_inverse(A, l, Ainv);
    A[0] = -1.0; /* not positive definite: must be refused, not crash */
    if (orc_spd_inverse(A, l, Ainv) == 0) rc |= 4;
    double *ksp = NEW(double, nnz), *kdelta = NEW(double, nnz), *knys = NEW(double, nnz);
    orc_pattern_values(X, Y, d, cost, lambda, n, m, rowptr, colidx, 0, NULL, NULL, 0, ksp);
    orc_pattern_values(X, Y, d, cost, lambda, n, m, rowptr, colidx, 1, U, W, l, kdelta);
    orc_pattern_values(X, Y, d, cost, lambda, n, m, rowptr, colidx, 2, U, W, l, knys);

    /* the four operators: dense, sparse, Nystrom, LCN */
    double *a = NEW(double, N), *bm = NEW(double, N);
    for (int64_t i = 0; i < n; ++i) a[i] = 1.0 / (double)n;
    for (int64_t j = 0; j < m; ++j) bm[j] = 1.0 / (double)m;
    double *lu = NEW(double, N), *lv = NEW(double, N), *r = NEW(double, N), *c = NEW(double, N);
    double dist, resid;
    int64_t counts[3];
    for (int mode = 0; mode < 4; ++mode) {
        const double *Kd = mode == 0 ? K : NULL;
        const int ll = mode >= 2 ? l : 0;
        const double *Uo = mode >= 2 ? U : NULL, *Wo = mode >= 2 ? W : NULL;
        const int64_t *rp = (mode == 1 || mode == 3) ? rowptr : NULL;
        const int32_t *ci = (mode == 1 || mode == 3) ? colidx : NULL;
        const double *val = mode == 1 ? ksp : (mode == 3 ? kdelta : NULL);
        memset(lu, 0, sizeof(double) * (size_t)N);
        memset(lv, 0, sizeof(double) * (size_t)N);
        memset(counts, 0, sizeof(counts));
        orc_sinkhorn(n, m, ll, Kd, Uo, Wo, rp, ci, val, a, bm, 4, lu, lv, counts);
        orc_marginals(n, m, ll, Kd, Uo, Wo, rp, ci, val, a, bm, lambda, lu, lv, r, c, &dist, &resid);
        if (mode == 3 && counts[0] == 0) {
            double *gU = NEW(double, n * l), *gW = NEW(double, (int64_t)l * m), *gsp = NEW(double, nnz),
                   *gnys = NEW(double, nnz);
            orc_backward(n, m, l, U, W, rowptr, colidx, ksp, knys, lambda, lu, lv, gU, gW, gsp, gnys);
            free(gU);
            free(gW);
            free(gsp);
            free(gnys);
        }
        if (mode == 1) {
            double *gsp = NEW(double, nnz);
            orc_backward(n, m, 0, NULL, NULL, rowptr, colidx, ksp, NULL, lambda, lu, lv, NULL, NULL, gsp, NULL);
            free(gsp);
        }
        /* the bipartite-matching form of the same operator (Sec. 6) */
        double *kpe = NEW(double, n), *keq = NEW(double, m);
        for (int64_t i = 0; i < n; ++i) kpe[i] = exp(-(0.5 + unit_random()) / lambda);
        for (int64_t j = 0; j < m; ++j) keq[j] = exp(-(0.5 + unit_random()) / lambda);
        for (int64_t i = 0; i < N; ++i) a[i] = bm[i] = 1.0 / (double)N;
        memset(lu, 0, sizeof(double) * (size_t)N);
        memset(lv, 0, sizeof(double) * (size_t)N);
        memset(counts, 0, sizeof(counts));
        orc_sinkhorn_bp(n, m, ll, Kd, Uo, Wo, rp, ci, val, kpe, keq, a, bm, 3, lu, lv, counts);
        orc_marginals_bp(n, m, ll, Kd, Uo, Wo, rp, ci, val, kpe, keq, a, bm, lambda, lu, lv, r, c, &dist, &resid);
        for (int64_t i = 0; i < n; ++i) a[i] = 1.0 / (double)n;
        for (int64_t j = 0; j < m; ++j) bm[j] = 1.0 / (double)m;
        free(kpe);
        free(keq);
    }

    free(Z); free(C); free(K); free(L); free(assign); free(picks); free(L2); free(idx); free(bucket); free(cent);
    free(proj); free(rowptr); free(colidx); free(U); free(W); free(A); free(Ainv); free(ksp); free(kdelta); free(knys);
    free(a); free(bm); free(lu); free(lv); free(r); free(c);
    return rc;
}

int main(void)
{
    int rc = 0;
    rc |= run_problem(37, 29, 5, 6, 4, 2, COST_SQEUCLID);
    rc |= run_problem(29, 41, 3, 5, 3, 3, COST_EUCLID);
    rc |= run_problem(17, 17, 7, 4, 2, 1, COST_COSINE);
    rc |= run_problem(1, 1, 1, 1, 1, 1, COST_SQEUCLID);
    rc |= run_problem(2, 65, 2, 2, 1, 2, COST_SQEUCLID);
    printf("oracle sanitizer run: rc=%d\n", rc);
    return rc;
}
