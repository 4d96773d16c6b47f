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

#include "iter_common.h"   // cross-lane sums and maxima through the DPP data path
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
    unsigned long long *counters; // [0] non-positive sums, [1] / [2] sums of exactly zero without signed terms (rows / columns), per sweep
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

// A row-major matrix in LDS whose row length is only known at launch: M[i][j].
template <typename T>
struct Rows {
    T *base;
    int stride;
    __device__ T *operator[](int i) const { return base + i * stride; }
};

// LDS of the build kernel, sized by the batch's d, l and bucket count (not by their upper
// limits): doubles first, then floats, then integers.
struct BuildLds {
    int zs, ls, kmax;   // row length of the points / centroids, of U, and the larger of l and b
    size_t uf, vf, am, lm, li, sums, z, cent, assign, bucket, perm, cnts, fail, bytes;
};

__host__ __device__ inline BuildLds build_lds(int d, int l, int b)
{
    BuildLds L;
    L.zs = d + 1;
    L.ls = l > 0 ? l : 1;
    L.kmax = l > b ? l : b;
    if (L.kmax < 1) L.kmax = 1;
    size_t at = 0;
    auto take = [&](size_t bytes) {
        const size_t here = at;
        at += (bytes + 15) & ~(size_t)15;
        return here;
    };
    L.uf = take(sizeof(double) * BMAX * L.ls);
    L.vf = take(sizeof(double) * L.ls * BMAX);
    L.am = take(sizeof(double) * L.ls * L.ls);
    L.lm = take(sizeof(double) * L.ls * L.ls);
    L.li = take(sizeof(double) * L.ls * L.ls);
    L.sums = take(sizeof(unsigned long long) * L.kmax * d);
    L.z = take(sizeof(float) * 2 * BMAX * L.zs);
    L.cent = take(sizeof(float) * L.kmax * L.zs);
    L.assign = take(sizeof(int) * 2 * BMAX);
    L.bucket = take(sizeof(int) * BR * 2 * BMAX);
    L.perm = take(sizeof(int) * 2 * BMAX);
    L.cnts = take(sizeof(int) * L.kmax);
    L.fail = take(sizeof(int));
    L.bytes = at;
    return L;
}

// Lloyd's k-means on the N points in Z (LDS) by the whole workgroup; same
// definition as the large path: seeded distinct start, exact-rule assignment,
// fixed-point means, empty clusters keep their centroid.
__device__ void block_kmeans(Rows<float> Z, int N, int d, int k, int T, unsigned long long seed, Rows<float> cent,
                             int *assign, int *perm, Rows<unsigned long long> sums, int *cnts)
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
    // kp lanes share a point, one candidate centroid each (k <= 16)
    const int kp = k <= 1 ? 1 : k <= 2 ? 2 : k <= 4 ? 4 : k <= 8 ? 8 : 16;
    const int per_pass = (int)blockDim.x / kp;
    for (int it = 0; it < T; ++it) {
        for (int base = 0; base < N; base += per_pass) {   // same trip count in every lane
            const int pt = base + tid / kp;
            int bc = tid % kp;
            double s = INFINITY;
            if (pt < N && bc < k) {
                s = 0.0;
                for (int j = 0; j < d; ++j) {
                    double t = (double)Z[pt][j] - (double)cent[bc][j];
                    double t2 = t * t;
                    s = s + t2;
                }
            }
            for (int o = 1; o < kp; o <<= 1) {   // smallest distance, lowest index among equals
                const double os = __shfl_xor(s, o, 64);
                const int oc = __shfl_xor(bc, o, 64);
                if (os < s || (os == s && oc < bc)) {
                    s = os;
                    bc = oc;
                }
            }
            if (pt < N && tid % kp == 0) assign[pt] = bc;
        }
        for (int e = tid; e < k * d; e += blockDim.x) sums[e / d][e % d] = 0ull;
        if (tid < k) cnts[tid] = 0;
        __syncthreads();
        // member sums in 2^-32 fixed point (integer addition: any order gives the same sum):
        // lane j of a 64-lane group adds dimension j of the group's share of the points
        {
            const int j = tid & 63, grp = tid >> 6, groups = (int)blockDim.x >> 6;
            for (int p = grp; p < N; p += groups) {
                const int c = assign[p];
                if (j < d)
                    atomicAdd(&sums[c][j], (unsigned long long)__double2ll_rn((double)Z[p][j] * 4294967296.0));
                if (j == 0) atomicAdd(&cnts[c], 1);
            }
        }
        __syncthreads();
        for (int e = tid; e < k * d; e += blockDim.x) {
            const int c = e / d, j = e % d;
            const int cnt = cnts[c];
            if (cnt > 0) cent[c][j] = (float)(((double)(long long)sums[c][j] * (1.0 / 4294967296.0)) / (double)cnt);
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void batched_build_kernel(BatchDev B)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const BuildLds L = build_lds(B.d, B.l, B.b);
    const Rows<float> Z{(float *)(lds + L.z), L.zs};            // the pair's points, X then Y
    const Rows<float> cent{(float *)(lds + L.cent), L.zs};
    const Rows<double> Uf{(double *)(lds + L.uf), L.ls};        // U, then U A^{-1}
    const Rows<double> Vf{(double *)(lds + L.vf), BMAX};
    const Rows<double> Am{(double *)(lds + L.am), L.ls}, Lm{(double *)(lds + L.lm), L.ls}, Li{(double *)(lds + L.li), L.ls};
    const Rows<unsigned long long> sums{(unsigned long long *)(lds + L.sums), B.d};   // k-means: member sums
    const Rows<int> bucket{(int *)(lds + L.bucket), 2 * BMAX};
    int *assign = (int *)(lds + L.assign), *perm = (int *)(lds + L.perm), *cnts = (int *)(lds + L.cnts);
    int &fail_sh = *(int *)(lds + L.fail);

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
        block_kmeans(Z, N, d, l, B.T_l, B.seed_l + (unsigned long long)p, cent, assign, perm, sums, cnts);
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
            block_kmeans(Z, N, d, B.b, B.T_b, B.seed_b + (unsigned long long)p * B.R + r, cent, assign, perm, sums,
                         cnts);
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

__device__ inline double lane_value(double v, int src_lane)   // src_lane: a constant
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src_lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src_lane);
    return __hiloint2double(hi, lo);
}

__device__ inline double rcp64(double x)   // 1 / x for a positive finite x, to about one unit in the last place
{
    double r = __builtin_amdgcn_rcp(x);
    r = fma(fma(-x, r, 1.0), r, r);
    r = fma(fma(-x, r, 1.0), r, r);
    return r;
}

// iters Sinkhorn iterations per pair (iters == 0: only the query part), then the
// pair's distance and marginal residual.
//
// One wavefront per pair, no workgroup-wide step and no LDS anywhere.  Lane l keeps in registers row l
// and column l of the pair's kernel tile (zero beyond n x m) and the entries of index l of
// the scaling vectors u = [u^ (n); u~ (m)], v = [v^ (m); v~ (n)] (point part; deletion part,
// Sec. 6).  Inside the loop a vector is held as x * 2^E with one integer E for the whole
// vector, chosen after every update so that the largest entry lies in [1, 2): the max-shift of
// App. "Implementational details" with the shift restricted to powers of two, which costs an
// exponent extraction instead of an exp and a log per entry and half-iteration.  Logs are
// formed once, when the state is stored.  In a half-iteration every lane multiplies its row
// (or column) with the point part of the input vector, whose entries it reads from the other
// lanes' registers one by one (lane reads, no LDS, no barrier):
//   (K_BP v)_i     = sum_j K_ij v^_j + k_{i,eps} v~_i          (K_BP v)_{n+j}     = k_{eps,j} v^_j + sum v~
//   (K_BP^T u)_j   = sum_i K_ij u^_i + k_{eps,j} u~_j          (K_BP^T u)_{m+i}   = k_{i,eps} u^_i + sum u~
__global__ __launch_bounds__(64) void batched_run_kernel(BatchDev B, int iters, float *row_marg, float *col_marg)
{
    const double LN2 = 0.69314718055994530942;
    const int p = blockIdx.x, lane = threadIdx.x;
    const long long x0 = B.x_off[p], y0 = B.y_off[p];
    const int n = (int)(B.x_off[p + 1] - x0), m = (int)(B.y_off[p + 1] - y0);
    const bool bp = B.bp != 0;
    const int len_u = bp ? n + m : n, len_v = bp ? n + m : m;
    const float *Kt = B.Kt + (long long)p * BMAX * BMAX;
    float Kr[BMAX], Kc[BMAX];
#pragma unroll
    for (int j = 0; j < BMAX; ++j) {
        Kr[j] = (lane < n && j < m) ? Kt[lane * BMAX + j] : 0.f;
        Kc[j] = (j < n && lane < m) ? Kt[j * BMAX + lane] : 0.f;
    }
    const double kpe = (bp && lane < n) ? B.kpe[x0 + lane] : 0.0;
    const double keq = (bp && lane < m) ? B.keq[y0 + lane] : 0.0;
    const bool has_up = lane < n, has_ud = bp && lane < m;   // this lane's entries of u (point, deletion part)
    const bool has_vp = lane < m, has_vd = bp && lane < n;   // ... and of v
    double *gu = B.log_u + x0 + y0, *gv = B.log_v + x0 + y0;
    const double a_each = 1.0 / (double)len_u, b_each = 1.0 / (double)len_v;   // uniform marginals
    unsigned long long nonpos = 0, empty_u = 0, empty_v = 0;
    // A kernel without a Nystrom part and without deletion entries has no signed terms: a sum of
    // exactly zero means the point shares no bucket with any point of the other set (or only
    // vanished entries).  Such a point gets scaling 0 (log = -infinity), carries no mass and is
    // counted apart from the non-positive sums (App. "Limitations": ignored, not a failure).
    const bool unsupported_is_zero = !bp && B.l == 0;

    // stored logs -> x * 2^E
    auto load_vec = [&](double lp, bool hp, double ld, bool hd, double &xp, double &xd) -> int {
        const double M = wave_max(fmax(hp ? lp : -INFINITY, hd ? ld : -INFINITY));
        const double Ms = (M > -INFINITY && M < INFINITY) ? M : 0.0;
        const double Ef = floor(Ms * 1.4426950408889634074);
        xp = hp ? exp(lp - Ef * LN2) : 0.0;
        xd = hd ? exp(ld - Ef * LN2) : 0.0;
        return (int)Ef;
    };
    // largest entry into [1, 2); returns the exponent taken out (NaN entries are ignored by fmax)
    auto renorm = [&](double &xp, double &xd) -> int {
        const double mx = wave_max(fmax(xp, xd));
        if (!(mx > 0.0) || !(mx < INFINITY)) return 0;
        const int e = ilogb(mx);
        xp = ldexp(xp, -e);
        xd = ldexp(xd, -e);
        return e;
    };
    // One product with K_BP (Kreg = rows) or its transpose (Kreg = columns) for the input held in
    // (xp, xd): k_p / k_d is the deletion kernel value that enters this lane's point / deletion output.
    // len_in: length of the input's point part (the tile is zero beyond it; whole sixteens are skipped).
    auto product = [&](const float (&Kreg)[BMAX], int len_in, double xp, double xd, double k_p, double k_d,
                       double &s_p, double &s_d) {
        const double tail = bp ? wave_sum(xd) : 0.0;
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int j0 = 0; j0 < BMAX; j0 += 16) {
            if (j0 < len_in) {   // the same in every lane
#pragma unroll
                for (int j = j0; j < j0 + 16; ++j) acc[j & 3] = fma((double)Kreg[j], lane_value(xp, j), acc[j & 3]);
            }
        }
        s_p = (acc[0] + acc[1]) + (acc[2] + acc[3]) + k_p * xd;
        s_d = k_d * xp + tail;
    };
    auto scale = [&](double marg, double s, bool exists, unsigned long long &empty) -> double {
        if (!exists) return 0.0;
        if (s > 0.0) return marg * rcp64(s);
        if (unsupported_is_zero && s == 0.0) {
            ++empty;
            return 0.0;
        }
        ++nonpos;
        return NAN;
    };

    double xu_p = 0.0, xu_d = 0.0, xv_p, xv_d, s_p, s_d;
    int Eu = 0;
    int Ev = load_vec(has_vp ? gv[lane] : 0.0, has_vp, has_vd ? gv[m + lane] : 0.0, has_vd, xv_p, xv_d);
    if (iters == 0) Eu = load_vec(has_up ? gu[lane] : 0.0, has_up, has_ud ? gu[n + lane] : 0.0, has_ud, xu_p, xu_d);
    for (int it = 0; it < iters; ++it) {
        product(Kr, m, xv_p, xv_d, kpe, keq, s_p, s_d);        // u = a ./ (K_BP v), eq. 2
        xu_p = scale(a_each, s_p, has_up, empty_u);
        xu_d = scale(a_each, s_d, has_ud, empty_u);
        Eu = -Ev + renorm(xu_p, xu_d);
        product(Kc, n, xu_p, xu_d, keq, kpe, s_p, s_d);        // v = b ./ (K_BP^T u)
        xv_p = scale(b_each, s_p, has_vp, empty_v);
        xv_d = scale(b_each, s_d, has_vd, empty_v);
        Ev = -Eu + renorm(xv_p, xv_d);
    }
    const double lu_p = log(xu_p) + (double)Eu * LN2, lu_d = log(xu_d) + (double)Eu * LN2;
    const double lv_p = log(xv_p) + (double)Ev * LN2, lv_d = log(xv_d) + (double)Ev * LN2;
    if (iters > 0) {
        if (has_up) gu[lane] = lu_p;
        if (has_ud) gu[n + lane] = lu_d;
        if (has_vp) gv[lane] = lv_p;
        if (has_vd) gv[m + lane] = lv_d;
        nonpos = (unsigned long long)wave_sum((double)nonpos);
        empty_u = (unsigned long long)wave_sum((double)empty_u);
        empty_v = (unsigned long long)wave_sum((double)empty_v);
        if (lane == 0 && nonpos) atomicAdd(&B.counters[0], nonpos);
        if (lane == 0 && empty_u) atomicAdd(&B.counters[1], empty_u);
        if (lane == 0 && empty_v) atomicAdd(&B.counters[2], empty_v);
    }

    // marginals r = u .* (K_BP v), c = v .* (K_BP^T u); distance and residual
    double dsum = 0.0, esum = 0.0;
    product(Kr, m, xv_p, xv_d, kpe, keq, s_p, s_d);
    if (has_up) {
        const double r = ldexp(xu_p * s_p, Eu + Ev);
        if (r != 0.0) dsum += r * lu_p;   // a point without mass (log u = -infinity) adds nothing
        esum += fabs(r - a_each);
        if (row_marg) row_marg[x0 + y0 + lane] = (float)r;
    }
    if (has_ud) {
        const double r = ldexp(xu_d * s_d, Eu + Ev);
        dsum += r * lu_d;
        esum += fabs(r - a_each);
        if (row_marg) row_marg[x0 + y0 + n + lane] = (float)r;
    }
    product(Kc, n, xu_p, xu_d, keq, kpe, s_p, s_d);
    if (has_vp) {
        const double c = ldexp(xv_p * s_p, Eu + Ev);
        if (c != 0.0) dsum += c * lv_p;
        esum += fabs(c - b_each);
        if (col_marg) col_marg[x0 + y0 + lane] = (float)c;
    }
    if (has_vd) {
        const double c = ldexp(xv_d * s_d, Eu + Ev);
        dsum += c * lv_d;
        esum += fabs(c - b_each);
        if (col_marg) col_marg[x0 + y0 + m + lane] = (float)c;
    }
    const double D = wave_sum(dsum);
    const double E = wave_sum(esum);
    if (lane == 0) {
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
    hipLaunchKernelGGL(batched_run_kernel, dim3(h.dev.P), dim3(64), 0, h.stream, h.dev, iters, (float *)nullptr,
                       (float *)nullptr);
    BHIPCHK(hipGetLastError());
    BHIPCHK(hipEventRecord(h.ev1, h.stream));
    unsigned long long c[3] = {0, 0, 0};
    BHIPCHK(hipMemcpyAsync(c, h.dev.counters, sizeof(c), hipMemcpyDeviceToHost, h.stream));
    BHIPCHK(hipStreamSynchronize(h.stream));
    BHIPCHK(hipEventElapsedTime(&h.last_ms, h.ev0, h.ev1));
    if (c[0]) return LCN_ERR_NONPOSITIVE;
    return (c[1] | c[2]) ? LCN_WARN_NO_SUPPORT : LCN_OK;
}

lcn_status batched_query(void *hh, double *dist_host, double *resid_host, float *row_dev, float *col_dev)
{
    BatchHandle &h = *(BatchHandle *)hh;
    hipLaunchKernelGGL(batched_run_kernel, dim3(h.dev.P), dim3(64), 0, h.stream, h.dev, 0, row_dev, col_dev);
    BHIPCHK(hipGetLastError());
    if (dist_host)
        BHIPCHK(hipMemcpyAsync(dist_host, h.dev.dist, sizeof(double) * h.dev.P, hipMemcpyDeviceToHost, h.stream));
    if (resid_host)
        BHIPCHK(hipMemcpyAsync(resid_host, h.dev.resid, sizeof(double) * h.dev.P, hipMemcpyDeviceToHost, h.stream));
    BHIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status batched_counts(void *hh, unsigned long long c[3])
{
    BatchHandle &h = *(BatchHandle *)hh;
    BHIPCHK(hipMemcpyAsync(c, h.dev.counters, 3 * sizeof(unsigned long long), hipMemcpyDeviceToHost, h.stream));
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
    const size_t lds_bytes = build_lds(D.d, D.l, D.b).bytes;
    BHIPCHK(hipFuncSetAttribute((const void *)batched_build_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes));
    hipLaunchKernelGGL(batched_build_kernel, dim3(P), dim3(256), lds_bytes, h.stream, D);
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
