// Many small transport problems in one launch (the graph-pair workloads of
// Sec. 6): one workgroup per pair, everything in LDS.
//
// Build: the same method as the large path, per pair -- k-means landmarks and
// k-means LSH buckets on X_p u Y_p by the exact bucket rule, Nystrom factors in
// fp64, exact kernel values on pairs that share a bucket (Secs. 3-4).  At these
// sizes (at most 64 points per side) the approximated kernel K~ = U A^{-1} V +
// (K^sp - K^sp_Nys) is written out as a dense 64 x 64 fp32 tile, which is what
// the iteration then keeps in LDS.
//
// Iteration: Sinkhorn on the bipartite-matching matrix of Sec. 6,
//   K_BP = [[K~, diag(k_p,eps)], [diag(k_eps,q), 1]],
// using its block formulas (only the two diagonals are stored), with the
// log-sum-exp max-shift taken out per vector (App. "Implementational details").
// Without deletion costs it is plain Sinkhorn on K~.
//
// Compiled with -ffp-contract=off: the bucket rule needs separate multiply and add.
#include <cmath>
#include <new>
#include <vector>

#include "lcn_internal.h"

#pragma clang fp contract(off)

namespace lcn {

constexpr int BMAX = 64;   // points per side
constexpr int BD = 64;     // dimensions
constexpr int BL = 16;     // landmarks, buckets
constexpr int BR = 4;      // hash rounds
constexpr uint32_t BATCH_MAGIC = 0x4C434E42u;  // "LCNB"

struct BatchDev {
    int P, d, cost, mode, l, b, R, T_l, T_b, bp;
    unsigned long long seed_l, seed_b;
    double ridge;
    const float *X, *Y;           // caller's points (fp32 copies in the workspace)
    const long long *x_off, *y_off;
    const float *lambda;
    const float *del_x, *del_y;   // deletion costs or null
    float *Kt;                    // [P][64][64]
    double *kpe, *keq;            // exp(-del / lambda)
    float *landmarks;             // [P][l][d]
    int *buckets;                 // per pair [R][n_p + m_p], pairs back to back at R * (x_off + y_off)
    double *log_u, *log_v;        // per pair at x_off + y_off, length n + m each (n resp. m without BP)
    double *dist, *resid;         // [P]
    unsigned long long *counters; // [0] non-positive sums
    int *fail;
};

__device__ inline unsigned long long splitmix64_dev(unsigned long long &state)
{
    unsigned long long z = (state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__device__ inline double pair_cost(const float *x, const float *y, int d, int cost)
{
    if (cost == LCN_COST_COSINE) {
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
    return cost == LCN_COST_EUCLID ? sqrt(s) : s;
}

// Lloyd's k-means on the N points in Z (LDS) by the whole workgroup; same
// definition as the large path: seeded distinct start, exact-rule assignment,
// fixed-point means, empty clusters keep their centroid.
__device__ void block_kmeans(const float (*Z)[BD + 1], int N, int d, int k, int T, unsigned long long seed,
                             float (*cent)[BD + 1], int *assign, int *perm)
{
    const int tid = threadIdx.x;
    if (tid == 0) {
        for (int i = 0; i < N; ++i) perm[i] = i;
        unsigned long long s = seed;
        for (int t = 0; t < k; ++t) {
            int j = t + (int)(splitmix64_dev(s) % (unsigned long long)(N - t));
            int tmp = perm[t];
            perm[t] = perm[j];
            perm[j] = tmp;
        }
    }
    __syncthreads();
    for (int e = tid; e < k * d; e += blockDim.x) cent[e / d][e % d] = Z[perm[e / d]][e % d];
    __syncthreads();
    for (int it = 0; it < T; ++it) {
        if (tid < N) {
            int best = 0;
            double bestD = 0.0;
            for (int c = 0; c < k; ++c) {
                double s = 0.0;
                for (int j = 0; j < d; ++j) {
                    double t = (double)Z[tid][j] - (double)cent[c][j];
                    double t2 = t * t;
                    s = s + t2;
                }
                if (c == 0 || s < bestD) {
                    bestD = s;
                    best = c;
                }
            }
            assign[tid] = best;
        }
        __syncthreads();
        for (int e = tid; e < k * d; e += blockDim.x) {
            const int c = e / d, j = e % d;
            long long sum = 0, cnt = 0;
            for (int p = 0; p < N; ++p)
                if (assign[p] == c) {
                    sum += __double2ll_rn((double)Z[p][j] * 4294967296.0);
                    ++cnt;
                }
            if (cnt > 0) cent[c][j] = (float)(((double)sum * (1.0 / 4294967296.0)) / (double)cnt);
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void batched_build_kernel(BatchDev B)
{
    __shared__ float Z[2 * BMAX][BD + 1];
    __shared__ float cent[BL][BD + 1];
    __shared__ double Uf[BMAX][BL];     // U, then U A^{-1}
    __shared__ double Vf[BL][BMAX];
    __shared__ double Am[BL][BL], Lm[BL][BL], Li[BL][BL];
    __shared__ int assign[2 * BMAX];
    __shared__ int bucket[BR][2 * BMAX];
    __shared__ int perm[2 * BMAX];
    __shared__ int fail_sh;

    const int p = blockIdx.x, tid = threadIdx.x;
    const long long x0 = B.x_off[p], y0 = B.y_off[p];
    const int n = (int)(B.x_off[p + 1] - x0), m = (int)(B.y_off[p + 1] - y0);
    const int N = n + m, d = B.d;
    const double lam = (double)B.lambda[p];
    if (tid == 0) fail_sh = 0;
    for (int e = tid; e < N * d; e += 256) {
        const int i = e / d, j = e % d;
        Z[i][j] = i < n ? B.X[(x0 + i) * d + j] : B.Y[(y0 + i - n) * d + j];
    }
    __syncthreads();
    const bool low_rank = B.mode == LCN_MODE_NYSTROM || B.mode == LCN_MODE_LCN;
    const bool hashed = B.mode == LCN_MODE_SPARSE || B.mode == LCN_MODE_LCN;
    const int l = low_rank ? B.l : 0;

    if (low_rank) {
        block_kmeans(Z, N, d, l, B.T_l, B.seed_l + (unsigned long long)p, cent, assign, perm);
        for (int e = tid; e < l * d; e += 256) B.landmarks[((long long)p * l + e / d) * d + e % d] = cent[e / d][e % d];
        // factors in fp64
        for (int e = tid; e < n * l; e += 256) Uf[e / l][e % l] = exp(-pair_cost(Z[e / l], cent[e % l], d, B.cost) / lam);
        for (int e = tid; e < l * m; e += 256) Vf[e / m][e % m] = exp(-pair_cost(cent[e / m], Z[n + e % m], d, B.cost) / lam);
        for (int e = tid; e < l * l; e += 256)
            Am[e / l][e % l] = exp(-pair_cost(cent[e / l], cent[e % l], d, B.cost) / lam) + (e / l == e % l ? B.ridge : 0.0);
        __syncthreads();
        if (tid == 0) {  // Cholesky of the l x l landmark kernel
            for (int j = 0; j < l; ++j) {
                double s = Am[j][j];
                for (int k = 0; k < j; ++k) s -= Lm[j][k] * Lm[j][k];
                if (!(s > 0.0)) {
                    fail_sh = 1;
                    s = 1.0;
                }
                const double ljj = sqrt(s);
                Lm[j][j] = ljj;
                for (int i = j + 1; i < l; ++i) {
                    double t = Am[i][j];
                    for (int k = 0; k < j; ++k) t -= Lm[i][k] * Lm[j][k];
                    Lm[i][j] = t / ljj;
                }
            }
        }
        __syncthreads();
        if (tid < l) {  // column tid of L^{-1}
            const int c = tid;
            for (int i = 0; i < l; ++i) {
                double v = 0.0;
                if (i >= c) {
                    double t = (i == c) ? 1.0 : 0.0;
                    for (int k = c; k < i; ++k) t -= Lm[i][k] * Li[k][c];
                    v = t / Lm[i][i];
                }
                Li[i][c] = v;
            }
        }
        __syncthreads();
        for (int e = tid; e < l * l; e += 256) {  // A^{-1} = L^{-T} L^{-1}
            const int i = e / l, j = e % l;
            double t = 0.0;
            for (int k = (i > j ? i : j); k < l; ++k) t += Li[k][i] * Li[k][j];
            Am[i][j] = t;
        }
        __syncthreads();
        // U <- U A^{-1}: every thread first reads the whole row it rewrites
        for (int i = tid; i < n; i += 256) {
            double row[BL];
            for (int k = 0; k < l; ++k) row[k] = Uf[i][k];
            for (int q = 0; q < l; ++q) {
                double t = 0.0;
                for (int k = 0; k < l; ++k) t += row[k] * Am[k][q];
                Uf[i][q] = t;
            }
        }
        __syncthreads();
    }
    if (hashed) {
        for (int r = 0; r < B.R; ++r) {
            block_kmeans(Z, N, d, B.b, B.T_b, B.seed_b + (unsigned long long)p * B.R + r, cent, assign, perm);
            for (int i = tid; i < N; i += 256) {
                bucket[r][i] = assign[i];
                B.buckets[(x0 + y0) * B.R + (long long)r * N + i] = assign[i];
            }
            __syncthreads();
        }
    }
    // K~_ij: exact where x_i and y_j share a bucket, Nystrom elsewhere (0 without a Nystrom part)
    float *Kt = B.Kt + (long long)p * BMAX * BMAX;
    for (int e = tid; e < n * m; e += 256) {
        const int i = e / m, j = e % m;
        bool near = B.mode == LCN_MODE_DENSE;
        if (hashed)
            for (int r = 0; r < B.R; ++r) near |= bucket[r][i] == bucket[r][n + j];
        double v = 0.0;
        if (near) {
            v = exp(-pair_cost(Z[i], Z[n + j], d, B.cost) / lam);
        } else if (low_rank) {
            for (int k = 0; k < l; ++k) v += Uf[i][k] * Vf[k][j];
        }
        Kt[i * BMAX + j] = (float)v;
    }
    if (B.bp) {
        for (int i = tid; i < n; i += 256) B.kpe[x0 + i] = exp(-(double)B.del_x[x0 + i] / lam);
        for (int j = tid; j < m; j += 256) B.keq[y0 + j] = exp(-(double)B.del_y[y0 + j] / lam);
    }
    const int len_u = B.bp ? N : n, len_v = B.bp ? N : m;
    for (int i = tid; i < len_u; i += 256) B.log_u[x0 + y0 + i] = 0.0;
    for (int i = tid; i < len_v; i += 256) B.log_v[x0 + y0 + i] = 0.0;
    __syncthreads();
    if (tid == 0 && fail_sh) *B.fail = 1;
}

// block-wide maximum / sum of one value per thread (256 threads = 4 wavefronts), result to all:
// butterfly inside each wavefront, then the four results through LDS (sh: at least 4 doubles)
__device__ inline double block_max(double v, double *sh)
{
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const double r = fmax(fmax(sh[0], sh[1]), fmax(sh[2], sh[3]));
    __syncthreads();
    return r;
}

__device__ inline double block_sum(double v, double *sh)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const double r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    __syncthreads();
    return r;
}

// iters Sinkhorn iterations per pair (iters == 0: only the query part), then the
// pair's distance and marginal residual.
__global__ __launch_bounds__(256) void batched_run_kernel(BatchDev B, int iters, float *row_marg, float *col_marg)
{
    __shared__ float K[BMAX][BMAX + 1];
    __shared__ double lu[2 * BMAX], lv[2 * BMAX], xin[2 * BMAX], sums[2 * BMAX];
    __shared__ double kpe[BMAX], keq[BMAX];
    __shared__ double red[256];

    const int p = blockIdx.x, tid = threadIdx.x;
    const long long x0 = B.x_off[p], y0 = B.y_off[p];
    const int n = (int)(B.x_off[p + 1] - x0), m = (int)(B.y_off[p + 1] - y0);
    const int N = n + m;
    const int len_u = B.bp ? N : n, len_v = B.bp ? N : m;
    const float *Kt = B.Kt + (long long)p * BMAX * BMAX;
    for (int e = tid; e < n * m; e += 256) K[e / m][e % m] = Kt[(e / m) * BMAX + e % m];
    for (int i = tid; i < n; i += 256) kpe[i] = B.bp ? B.kpe[x0 + i] : 0.0;
    for (int j = tid; j < m; j += 256) keq[j] = B.bp ? B.keq[y0 + j] : 0.0;
    for (int i = tid; i < len_u; i += 256) lu[i] = B.log_u[x0 + y0 + i];
    for (int i = tid; i < len_v; i += 256) lv[i] = B.log_v[x0 + y0 + i];
    __syncthreads();
    const double log_a = -log((double)len_u), log_b = -log((double)len_v);  // uniform marginals
    unsigned long long nonpos = 0;

    // sums[i] = (K_BP x)_i for x = exp(lin - M) (transpose: K_BP^T); 4 threads share an output
    auto apply = [&](bool transpose, const double *logs_in, int len_in, int len_out) -> double {
        const double M = block_max(tid < len_in ? logs_in[tid] : -INFINITY, red);
        const double Ms = (M > -INFINITY && M < INFINITY) ? M : 0.0;
        const double x = tid < len_in ? exp(logs_in[tid] - Ms) : 0.0;
        if (tid < len_in) xin[tid] = x;
        const int pts_in = transpose ? n : m;    // point part of the input vector
        const int pts_out = transpose ? m : n;
        double tail = 0.0;                       // sum of the deletion part of the input
        if (B.bp)
            tail = block_sum(tid >= pts_in ? x : 0.0, red);   // its barrier also publishes xin
        else
            __syncthreads();
        const int o = tid >> 2, part = tid & 3;
        double s = 0.0;
        if (o < pts_out) {
            for (int q = part; q < pts_in; q += 4) s = fma(transpose ? (double)K[q][o] : (double)K[o][q], xin[q], s);
        }
        s += __shfl_xor(s, 1, 64);
        s += __shfl_xor(s, 2, 64);
        if (part == 0 && o < pts_out) {
            if (B.bp) s += (transpose ? keq[o] : kpe[o]) * xin[pts_in + o];
            sums[o] = s;
        }
        if (B.bp && tid < pts_in) sums[pts_out + tid] = (transpose ? kpe[tid] : keq[tid]) * xin[tid] + tail;
        __syncthreads();
        (void)len_out;
        return Ms;
    };

    for (int it = 0; it < iters; ++it) {
        double M = apply(false, lv, len_v, len_u);
        if (tid < len_u) {
            const double s = sums[tid];
            if (s > 0.0) {
                lu[tid] = log_a - log(s) - M;
            } else {
                lu[tid] = NAN;
                ++nonpos;
            }
        }
        __syncthreads();
        M = apply(true, lu, len_u, len_v);
        if (tid < len_v) {
            const double s = sums[tid];
            if (s > 0.0) {
                lv[tid] = log_b - log(s) - M;
            } else {
                lv[tid] = NAN;
                ++nonpos;
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < len_u; i += 256) B.log_u[x0 + y0 + i] = lu[i];
    for (int i = tid; i < len_v; i += 256) B.log_v[x0 + y0 + i] = lv[i];
    if (nonpos) atomicAdd(&B.counters[0], nonpos);

    // marginals r = u .* (K_BP v), c = v .* (K_BP^T u); distance and residual
    double Mv = apply(false, lv, len_v, len_u);
    double dsum = 0.0, esum = 0.0;
    if (tid < len_u) {
        const double r = exp(lu[tid] + Mv) * sums[tid];
        dsum += r * lu[tid];
        esum += fabs(r - exp(log_a));
        if (row_marg) row_marg[x0 + y0 + tid] = (float)r;
    }
    __syncthreads();
    double Mu = apply(true, lu, len_u, len_v);
    if (tid < len_v) {
        const double c = exp(lv[tid] + Mu) * sums[tid];
        dsum += c * lv[tid];
        esum += fabs(c - exp(log_b));
        if (col_marg) col_marg[x0 + y0 + tid] = (float)c;
    }
    __syncthreads();
    const double D = block_sum(dsum, red);
    const double E = block_sum(esum, red);
    if (tid == 0) {
        B.dist[p] = (double)B.lambda[p] * D;
        B.resid[p] = E;
    }
}

// c_i = || alpha .* x_i ||_2 (Sec. 6, learnable deletion cost); one thread per
// point, squares added in fp64 in the order of the dimensions.
__global__ __launch_bounds__(256) void deletion_cost_kernel(const float *X, long long total, int d, const float *alpha,
                                                            float *out)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const float *x = X + i * d;
    double s = 0.0;
    for (int k = 0; k < d; ++k) {
        const double t = (double)x[k] * (double)alpha[k];
        s += t * t;
    }
    out[i] = (float)sqrt(s);
}

struct BatchHandle {
    uint32_t magic;
    BatchDev dev;
    hipStream_t stream;
    long long total_x, total_y;
    size_t ws_used;
    hipEvent_t ev0, ev1;
    float last_ms;
};

}  // namespace lcn

using namespace lcn;

#define BHIPCHK(expr)                 \
    do {                              \
        hipError_t e_ = (expr);       \
        if (e_ != hipSuccess) {       \
            (void)hipGetLastError();  \
            return LCN_ERR_DEVICE;    \
        }                             \
    } while (0)

namespace lcn {
bool is_batched_handle(const void *h) { return h && *(const uint32_t *)h == BATCH_MAGIC; }

lcn_status batched_run(void *hh, int iters)
{
    BatchHandle &h = *(BatchHandle *)hh;
    BHIPCHK(hipEventRecord(h.ev0, h.stream));
    hipLaunchKernelGGL(batched_run_kernel, dim3(h.dev.P), dim3(256), 0, h.stream, h.dev, iters, (float *)nullptr,
                       (float *)nullptr);
    BHIPCHK(hipGetLastError());
    BHIPCHK(hipEventRecord(h.ev1, h.stream));
    unsigned long long c = 0;
    BHIPCHK(hipMemcpyAsync(&c, h.dev.counters, sizeof(c), hipMemcpyDeviceToHost, h.stream));
    BHIPCHK(hipStreamSynchronize(h.stream));
    BHIPCHK(hipEventElapsedTime(&h.last_ms, h.ev0, h.ev1));
    return c ? LCN_ERR_NONPOSITIVE : LCN_OK;
}

lcn_status batched_query(void *hh, double *dist_host, double *resid_host, float *row_dev, float *col_dev)
{
    BatchHandle &h = *(BatchHandle *)hh;
    hipLaunchKernelGGL(batched_run_kernel, dim3(h.dev.P), dim3(256), 0, h.stream, h.dev, 0, row_dev, col_dev);
    BHIPCHK(hipGetLastError());
    if (dist_host)
        BHIPCHK(hipMemcpyAsync(dist_host, h.dev.dist, sizeof(double) * h.dev.P, hipMemcpyDeviceToHost, h.stream));
    if (resid_host)
        BHIPCHK(hipMemcpyAsync(resid_host, h.dev.resid, sizeof(double) * h.dev.P, hipMemcpyDeviceToHost, h.stream));
    BHIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status batched_timing(void *hh, float *ms, int *launches)
{
    BatchHandle &h = *(BatchHandle *)hh;
    if (ms) *ms = h.last_ms;
    if (launches) *launches = 1;
    return LCN_OK;
}

void batched_destroy(void *hh)
{
    BatchHandle *h = (BatchHandle *)hh;
    (void)hipStreamSynchronize(h->stream);
    (void)hipEventDestroy(h->ev0);
    (void)hipEventDestroy(h->ev1);
    h->magic = 0;
    delete h;
}
}  // namespace lcn

extern "C" {

lcn_status lcn_build_batched(const float *X, const float *Y, int32_t d, const lcn_batch_desc *desc, int32_t cost,
                             int32_t mode, const lcn_landmark_params *lm, const lcn_lsh_params *lsh, void *workspace,
                             size_t workspace_bytes, void *hip_stream, size_t *bytes_needed, lcn_handle *out)
{
    if (!out) return LCN_ERR_INVALID_ARG;
    *out = nullptr;
    if (!X || !Y || !desc || !desc->x_off || !desc->y_off || !desc->lambda || !workspace ||
        ((uintptr_t)workspace & 255))
        return LCN_ERR_INVALID_ARG;
    const int P = desc->num_problems;
    if (P < 1 || d < 1 || d > BD) return LCN_ERR_INVALID_ARG;
    if (cost < LCN_COST_SQEUCLID || cost > LCN_COST_COSINE || mode < LCN_MODE_DENSE || mode > LCN_MODE_LCN)
        return LCN_ERR_INVALID_ARG;
    const bool low_rank = mode == LCN_MODE_NYSTROM || mode == LCN_MODE_LCN;
    const bool hashed = mode == LCN_MODE_SPARSE || mode == LCN_MODE_LCN;
    if (low_rank && (!lm || lm->num_landmarks < 1 || lm->num_landmarks > BL || lm->kmeans_iters < 1 || lm->init != LCN_INIT_SAMPLE ||
                     !(lm->ridge >= 0.0)))
        return LCN_ERR_INVALID_ARG;
    if (hashed && (!lsh || lsh->hash != LCN_HASH_KMEANS || lsh->num_buckets < 1 || lsh->num_buckets > BL ||
                   lsh->num_rounds < 1 || lsh->num_rounds > BR || lsh->kmeans_iters < 1 || lsh->branching[0] != 0 ||
                   lsh->and_width > 1))
        return LCN_ERR_INVALID_ARG;
    if ((desc->del_cost_x == nullptr) != (desc->del_cost_y == nullptr)) return LCN_ERR_INVALID_ARG;
    for (int p = 0; p < P; ++p) {
        const long long n = desc->x_off[p + 1] - desc->x_off[p], m = desc->y_off[p + 1] - desc->y_off[p];
        if (n < 1 || m < 1 || n > BMAX || m > BMAX) return LCN_ERR_INVALID_ARG;
        if (low_rank && lm->num_landmarks > n + m) return LCN_ERR_INVALID_ARG;
        if (hashed && lsh->num_buckets > n + m) return LCN_ERR_INVALID_ARG;
        if (!(desc->lambda[p] > 0.f)) return LCN_ERR_INVALID_ARG;
    }
    if (desc->x_off[0] != 0 || desc->y_off[0] != 0) return LCN_ERR_INVALID_ARG;
    const long long tx = desc->x_off[P], ty = desc->y_off[P];

    BatchHandle *hp = new (std::nothrow) BatchHandle{};
    if (!hp) return LCN_ERR_ALLOC;
    BatchHandle &h = *hp;
    struct Guard {
        BatchHandle *p;
        ~Guard()
        {
            if (p) {
                if (p->ev0) (void)hipEventDestroy(p->ev0);
                if (p->ev1) (void)hipEventDestroy(p->ev1);
                delete p;
            }
        }
    } guard{hp};
    h.stream = (hipStream_t)hip_stream;
    h.total_x = tx;
    h.total_y = ty;
    BatchDev &D = h.dev;
    D.P = P;
    D.d = d;
    D.cost = cost;
    D.mode = mode;
    D.l = low_rank ? lm->num_landmarks : 0;
    D.b = hashed ? lsh->num_buckets : 1;
    D.R = hashed ? lsh->num_rounds : 0;
    D.T_l = low_rank ? lm->kmeans_iters : 0;
    D.T_b = hashed ? lsh->kmeans_iters : 0;
    D.seed_l = low_rank ? lm->seed : 0;
    D.seed_b = hashed ? lsh->seed : 0;
    D.ridge = low_rank ? lm->ridge : 0.0;
    D.bp = desc->del_cost_x ? 1 : 0;
    D.X = X;
    D.Y = Y;
    D.del_x = desc->del_cost_x;
    D.del_y = desc->del_cost_y;

    char *base = (char *)workspace;
    size_t used = 0;
    auto take = [&](size_t bytes) -> void * {
        bytes = (bytes + 255) & ~(size_t)255;
        void *ptr = base + used;
        used += bytes;
        return ptr;
    };
    long long *xo = (long long *)take(sizeof(long long) * (P + 1));
    long long *yo = (long long *)take(sizeof(long long) * (P + 1));
    float *lam = (float *)take(sizeof(float) * P);
    D.Kt = (float *)take(sizeof(float) * (size_t)P * BMAX * BMAX);
    D.kpe = (double *)take(sizeof(double) * (size_t)tx);
    D.keq = (double *)take(sizeof(double) * (size_t)ty);
    D.landmarks = (float *)take(sizeof(float) * (size_t)P * (D.l > 0 ? D.l : 1) * d);
    D.buckets = (int *)take(sizeof(int) * (size_t)(D.R > 0 ? D.R : 1) * (tx + ty));
    D.log_u = (double *)take(sizeof(double) * (size_t)(tx + ty));
    D.log_v = (double *)take(sizeof(double) * (size_t)(tx + ty));
    D.dist = (double *)take(sizeof(double) * P);
    D.resid = (double *)take(sizeof(double) * P);
    D.counters = (unsigned long long *)take(64);
    D.fail = (int *)take(64);
    h.ws_used = used;
    if (bytes_needed) *bytes_needed = used + 256;
    if (used > workspace_bytes) return LCN_ERR_ALLOC;
    D.x_off = xo;
    D.y_off = yo;
    D.lambda = lam;

    BHIPCHK(hipEventCreate(&h.ev0));
    BHIPCHK(hipEventCreate(&h.ev1));
    BHIPCHK(hipMemcpyAsync(xo, desc->x_off, sizeof(long long) * (P + 1), hipMemcpyHostToDevice, h.stream));
    BHIPCHK(hipMemcpyAsync(yo, desc->y_off, sizeof(long long) * (P + 1), hipMemcpyHostToDevice, h.stream));
    BHIPCHK(hipMemcpyAsync(lam, desc->lambda, sizeof(float) * P, hipMemcpyHostToDevice, h.stream));
    BHIPCHK(hipMemsetAsync(D.counters, 0, 64, h.stream));
    BHIPCHK(hipMemsetAsync(D.fail, 0, 64, h.stream));
    hipLaunchKernelGGL(batched_build_kernel, dim3(P), dim3(256), 0, h.stream, D);
    BHIPCHK(hipGetLastError());
    int fail = 0;
    BHIPCHK(hipMemcpyAsync(&fail, D.fail, sizeof(int), hipMemcpyDeviceToHost, h.stream));
    BHIPCHK(hipStreamSynchronize(h.stream));
    if (fail) return LCN_ERR_SINGULAR;
    h.magic = BATCH_MAGIC;
    guard.p = nullptr;
    *out = (lcn_handle)hp;
    return LCN_OK;
}

lcn_status lcn_batched_results(lcn_handle hh, double *dist_host, double *resid_host, float *row_dev, float *col_dev)
{
    if (!is_batched_handle(hh)) return LCN_ERR_STATE;
    return batched_query(hh, dist_host, resid_host, row_dev, col_dev);
}

lcn_status lcn_batched_get(lcn_handle hh, double *log_u_dev, double *log_v_dev, float *landmarks_dev,
                           int32_t *buckets_dev, float *kernel_dev)
{
    if (!is_batched_handle(hh)) return LCN_ERR_STATE;
    BatchHandle &h = *(BatchHandle *)hh;
    const BatchDev &D = h.dev;
    const size_t tz = (size_t)(h.total_x + h.total_y);
    if (log_u_dev) BHIPCHK(hipMemcpyAsync(log_u_dev, D.log_u, sizeof(double) * tz, hipMemcpyDeviceToDevice, h.stream));
    if (log_v_dev) BHIPCHK(hipMemcpyAsync(log_v_dev, D.log_v, sizeof(double) * tz, hipMemcpyDeviceToDevice, h.stream));
    if (landmarks_dev && D.l > 0)
        BHIPCHK(hipMemcpyAsync(landmarks_dev, D.landmarks, sizeof(float) * (size_t)D.P * D.l * D.d,
                               hipMemcpyDeviceToDevice, h.stream));
    if (buckets_dev && D.R > 0)
        BHIPCHK(hipMemcpyAsync(buckets_dev, D.buckets, sizeof(int) * (size_t)D.R * tz, hipMemcpyDeviceToDevice,
                               h.stream));
    if (kernel_dev)
        BHIPCHK(hipMemcpyAsync(kernel_dev, D.Kt, sizeof(float) * (size_t)D.P * BMAX * BMAX, hipMemcpyDeviceToDevice,
                               h.stream));
    BHIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_deletion_costs(const float *X, int64_t total, int32_t d, const float *alpha, float *out,
                              void *hip_stream)
{
    if (total < 0 || d < 1) return LCN_ERR_INVALID_ARG;
    if (total == 0) return LCN_OK;
    if (!X || !alpha || !out) return LCN_ERR_INVALID_ARG;
    const long long groups = (total + 255) / 256;
    if (groups > 0x7FFFFFFFLL) return LCN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(deletion_cost_kernel, dim3((unsigned)groups), dim3(256), 0, (hipStream_t)hip_stream, X,
                       (long long)total, d, alpha, out);
    BHIPCHK(hipGetLastError());
    return LCN_OK;
}

lcn_status lcn_head_lambdas(float lambda, int32_t num_heads, float *out_host)
{
    if (!out_host || !(lambda > 0.f) || num_heads < 1 || num_heads > 64) return LCN_ERR_INVALID_ARG;
    for (int k = 1; k <= num_heads; ++k) {
        const float v = (float)(std::exp2((double)k - 0.5 * (double)num_heads) * (double)lambda);
        if (!(v > 0.f) || !std::isfinite(v)) return LCN_ERR_INVALID_ARG;
        out_host[k - 1] = v;
    }
    return LCN_OK;
}

}  // extern "C"
