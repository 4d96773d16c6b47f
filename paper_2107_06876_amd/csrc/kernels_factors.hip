// Factor build: Nystrom factors U = k(X, L), V = k(L, Y), A = k(L, L) with
// k = exp(-c / lambda) (Sec. 4), the fp64 inverse of A and W = A^{-1} V (App.
// "Implementational details"), and the sparse values per bucket block:
// K^sp for sparse Sinkhorn (Sec. 3, eq. 3) or the correction K^sp - K^sp_Nys of
// K_LCN (Sec. 4).  Everything that feeds the inverse or a difference of nearly
// equal numbers is accumulated in fp64; only the stored factors are fp32.
#include "lcn_internal.h"

namespace lcn {

constexpr int TILE = 64;
constexpr int KCH = 32;
constexpr int LDT = TILE + 4;

// ------------------------------------------------------------ row norms --

__global__ void sqnorm_kernel(const float *__restrict__ P, long long rows, int d, double *__restrict__ out)
{
    long long row = (long long)blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    double s = 0.0;
    for (int k = lane; k < d; k += 64) {
        double v = (double)P[row * d + k];
        s = fma(v, v, s);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) out[row] = s;
}

hipError_t launch_sqnorms(const float *P, long long rows, int d, double *out, hipStream_t s)
{
    hipLaunchKernelGGL(sqnorm_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, P, rows, d, out);
    return hipGetLastError();
}

// ------------------------------------------------ pairwise tile machinery --
//
// 256 threads hold a 64 x 64 tile of fp64 accumulators, 4 x 4 per thread.
// Rows of both operands may be gathered through index lists held in LDS.

struct TileAcc {
    double v[4][4];
};

// stage 64 rows x KCH features of a row-major matrix into dst[k][row]
__device__ inline void stage_rows(float (*dst)[LDT], const float *__restrict__ base, long long ld,
                                  const long long *rowidx /* LDS, 64 entries, -1 = absent */, int k0, int kmax)
{
    const int tid = threadIdx.x;
    const int kk = tid & 31;
    const int r0 = tid >> 5;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
        int r = r0 + pass * 8;
        long long src = rowidx[r];
        float v = 0.f;
        if (src >= 0 && k0 + kk < kmax) v = base[src * ld + k0 + kk];
        dst[kk][r] = v;
    }
}

template <bool SQDIFF>
__device__ inline void tile_fma(TileAcc &acc, const float (*Ps)[LDT], const float (*Cs)[LDT])
{
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll 4
    for (int kk = 0; kk < KCH; ++kk) {
        const float4 pz = *(const float4 *)&Ps[kk][ty * 4];
        const float4 cz = *(const float4 *)&Cs[kk][tx * 4];
        const double pv[4] = {(double)pz.x, (double)pz.y, (double)pz.z, (double)pz.w};
        const double cv[4] = {(double)cz.x, (double)cz.y, (double)cz.z, (double)cz.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (SQDIFF) {
                    double t = pv[i] - cv[j];
                    acc.v[i][j] = fma(t, t, acc.v[i][j]);
                } else {
                    acc.v[i][j] = fma(pv[i], cv[j], acc.v[i][j]);
                }
            }
    }
}

__device__ inline void tile_zero(TileAcc &acc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc.v[i][j] = 0.0;
}

// cost from the accumulated quantity (squared distance, or dot product for cosine)
__device__ inline double cost_from_acc(double acc, int cost, double pn, double qn)
{
    if (cost == LCN_COST_COSINE) return 1.0 - acc / (sqrt(pn) * sqrt(qn));
    if (cost == LCN_COST_EUCLID) return sqrt(acc);
    return acc;
}

// ----------------------------------------------------- kernel matrix k(P, Q) --

__global__ __launch_bounds__(256) void kernel_matrix_kernel(const float *__restrict__ P, long long rows,
                                                            const float *__restrict__ Q, int cols, int d, int cost,
                                                            double inv_lambda, const double *__restrict__ pn,
                                                            const double *__restrict__ qn, float *out32,
                                                            double *out64, int ldo)
{
    __shared__ float Ps[KCH][LDT];
    __shared__ float Cs[KCH][LDT];
    __shared__ long long pidx[TILE], qidx[TILE];
    const int tid = threadIdx.x;
    const long long p0 = (long long)blockIdx.x * TILE;
    const int q0 = blockIdx.y * TILE;
    if (tid < TILE) {
        pidx[tid] = p0 + tid < rows ? p0 + tid : -1;
        qidx[tid] = q0 + tid < cols ? q0 + tid : -1;
    }
    TileAcc acc;
    tile_zero(acc);
    for (int k0 = 0; k0 < d; k0 += KCH) {
        __syncthreads();
        stage_rows(Ps, P, d, pidx, k0, d);
        stage_rows(Cs, Q, d, qidx, k0, d);
        __syncthreads();
        if (cost == LCN_COST_COSINE)
            tile_fma<false>(acc, Ps, Cs);
        else
            tile_fma<true>(acc, Ps, Cs);
    }
    const int tx = tid & 15, ty = tid >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        long long p = p0 + ty * 4 + i;
        if (p >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int q = q0 + tx * 4 + j;
            if (q >= cols) continue;
            double c = cost_from_acc(acc.v[i][j], cost, pn ? pn[p] : 0.0, qn ? qn[q] : 0.0);
            double kv = exp(-c * inv_lambda);
            if (out32) out32[p * ldo + q] = (float)kv;
            if (out64) out64[p * cols + q] = kv;
        }
    }
}

hipError_t launch_kernel_matrix(const float *P, long long rows, const float *Q, int cols, int d, int cost,
                                double lambda, const double *pn, const double *qn, float *out32, double *out64,
                                int ldo, hipStream_t s)
{
    dim3 grid((unsigned)((rows + TILE - 1) / TILE), (unsigned)((cols + TILE - 1) / TILE));
    hipLaunchKernelGGL(kernel_matrix_kernel, grid, dim3(256), 0, s, P, rows, Q, cols, d, cost, 1.0 / lambda, pn, qn,
                       out32, out64, ldo);
    return hipGetLastError();
}

// ----------------------------------------------------------- fp64 inverse --
//
// A is symmetric positive definite (a PSD kernel matrix, plus the ridge).
// One workgroup factors A = L L^T column by column (Lt holds L^T, so that a
// column of L is contiguous), then inverts L by forward substitution; A^{-1} =
// L^{-T} L^{-1} is formed by the GEMM kernel below.

__global__ __launch_bounds__(1024) void cholesky_kernel(const double *__restrict__ A, int l, double ridge,
                                                        double *Lt, int *fail_flag)
{
    __shared__ double red[4][512];
    __shared__ double pivot;
    const int tid = threadIdx.x;
    const int ti = tid & 255, tg = tid >> 8;
    for (int j = 0; j < l; ++j) {
        // partial sums over k = tg, tg + 4, ... < j of Lt[k][i] * Lt[k][j], i = j .. l-1
        for (int i = j + ti; i < l; i += 256) {
            double s = 0.0;
            for (int k = tg; k < j; k += 4) s = fma(Lt[(long long)k * l + i], Lt[(long long)k * l + j], s);
            red[tg][i] = s;
        }
        __syncthreads();
        if (tid == 0) {
            double s = A[(long long)j * l + j] + ridge - (red[0][j] + red[1][j] + red[2][j] + red[3][j]);
            if (!(s > 0.0)) {
                *fail_flag = 1;
                s = 1.0;
            }
            pivot = sqrt(s);
        }
        __syncthreads();
        const double piv = pivot;
        if (tg == 0) {
            for (int i = j + ti; i < l; i += 256) {
                double v;
                if (i == j)
                    v = piv;
                else
                    v = (A[(long long)i * l + j] - (red[0][i] + red[1][i] + red[2][i] + red[3][i])) / piv;
                Lt[(long long)j * l + i] = v;
            }
        }
        __syncthreads();
    }
}

// Li = L^{-1} (lower triangular, row-major, zero above the diagonal); one thread per column
__global__ __launch_bounds__(512) void tri_inverse_kernel(const double *__restrict__ Lt, int l, double *Li)
{
    const int c = threadIdx.x;
    if (c >= l) return;
    for (int i = 0; i < l; ++i) {
        double v = 0.0;
        if (i >= c) {
            double t = (i == c) ? 1.0 : 0.0;
            for (int k = c; k < i; ++k) t = fma(-Lt[(long long)k * l + i], Li[(long long)k * l + c], t);
            v = t / Lt[(long long)i * l + i];
        }
        Li[(long long)i * l + c] = v;
    }
}

// C (M x N) = op(A) * B with fp64 operands; op(A) = A (M x K) or A^T with A stored K x M.
template <bool TRANSA>
__global__ __launch_bounds__(256) void gemm_f64_kernel(const double *__restrict__ A, const double *__restrict__ B,
                                                       long long M, int N, int K, float *C32, double *C64, int ldc)
{
    constexpr int KC = 16;
    __shared__ double As[KC][TILE + 2];
    __shared__ double Bs[KC][TILE + 2];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const long long r0 = (long long)blockIdx.x * TILE;
    const int c0 = blockIdx.y * TILE;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    for (int k0 = 0; k0 < K; k0 += KC) {
        __syncthreads();
        if (TRANSA) {
            const int rr = tid & 63, kq = tid >> 6;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                int kk = kq + pass * 4;
                double v = 0.0;
                if (r0 + rr < M && k0 + kk < K) v = A[(long long)(k0 + kk) * M + r0 + rr];
                As[kk][rr] = v;
            }
        } else {
            const int kk = tid & 15, rq = tid >> 4;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                int rr = rq + pass * 16;
                double v = 0.0;
                if (r0 + rr < M && k0 + kk < K) v = A[(r0 + rr) * K + k0 + kk];
                As[kk][rr] = v;
            }
        }
        {
            const int cc = tid & 63, kq = tid >> 6;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                int kk = kq + pass * 4;
                double v = 0.0;
                if (c0 + cc < N && k0 + kk < K) v = B[(long long)(k0 + kk) * N + c0 + cc];
                Bs[kk][cc] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
            double av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(av[i], bv[j], acc[i][j]);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        long long r = r0 + ty * 4 + i;
        if (r >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = c0 + tx * 4 + j;
            if (c >= N) continue;
            if (C32) C32[r * ldc + c] = (float)acc[i][j];
            if (C64) C64[r * ldc + c] = acc[i][j];
        }
    }
}

hipError_t launch_gemm_f64(const double *A, const double *B, long long M, int N, int K, float *C32, int ldc,
                           hipStream_t s)
{
    dim3 grid((unsigned)((M + TILE - 1) / TILE), (unsigned)((N + TILE - 1) / TILE));
    hipLaunchKernelGGL(gemm_f64_kernel<false>, grid, dim3(256), 0, s, A, B, M, N, K, C32, (double *)nullptr, ldc);
    return hipGetLastError();
}

hipError_t launch_spd_inverse(double *A, int l, double ridge, double *Lt, double *Li, double *Ainv, int *fail_flag,
                              hipStream_t s)
{
    hipError_t e = hipMemsetAsync(Lt, 0, sizeof(double) * (size_t)l * l, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cholesky_kernel, dim3(1), dim3(1024), 0, s, A, l, ridge, Lt, fail_flag);
    hipLaunchKernelGGL(tri_inverse_kernel, dim3(1), dim3(512), 0, s, Lt, l, Li);
    dim3 grid((unsigned)((l + TILE - 1) / TILE), (unsigned)((l + TILE - 1) / TILE));
    // A^{-1} = Li^T Li
    hipLaunchKernelGGL(gemm_f64_kernel<true>, grid, dim3(256), 0, s, Li, Li, (long long)l, l, l, (float *)nullptr,
                       Ainv, l);
    return hipGetLastError();
}

// ------------------------------------------------- sparse values per block --
//
// One workgroup per 64 x 64 piece of a bucket block (round r, bucket beta):
// rows are the X members of the bucket, columns its Y members.  The exact
// kernel value and (LCN mode) the Nystrom value U_i . W_:j are accumulated in
// fp64 from the gathered rows; a pair that an earlier round already holds is
// stored as zero so that the union over rounds counts it once.

__global__ __launch_bounds__(256) void correction_kernel(SortBuffers B, const float *__restrict__ Z, int d, int cost,
                                                         double inv_lambda, const double *__restrict__ zn,
                                                         const float *__restrict__ U, const float *__restrict__ Wt,
                                                         int lp, int log_values, float *vals_x, float *vals_y,
                                                         unsigned long long *unique_counter)
{
    __shared__ float Ps[KCH][LDT];
    __shared__ float Cs[KCH][LDT];
    __shared__ float vals[TILE][TILE + 1];
    __shared__ long long xi[TILE], yj[TILE];
    __shared__ long long xdst[TILE], ydst[TILE];  // where each row's / column's slice of this block starts
    __shared__ int bx[8][TILE], by[8][TILE];
    __shared__ unsigned cnt_sh;

    const int tid = threadIdx.x;
    const int nb = B.R * B.b;
    // which block does this build tile belong to: last blk with tile_off[blk] <= blockIdx.x
    int lo = 0, hi = nb;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (B.tile_off[mid] <= (int)blockIdx.x)
            lo = mid;
        else
            hi = mid;
    }
    const int blk = lo;
    const int r = blk / B.b, beta = blk - r * B.b;
    const int *offx = B.off + (0 * B.R + r) * (B.b + 1);
    const int *offy = B.off + (1 * B.R + r) * (B.b + 1);
    const int nx = offx[beta + 1] - offx[beta];
    const int ny = offy[beta + 1] - offy[beta];
    const int tiles_y = (ny + 63) / 64;
    const int t_in = blockIdx.x - B.tile_off[blk];
    const int ti = t_in / tiles_y, tj = t_in - ti * tiles_y;
    const int *xperm = B.perm + (long long)r * B.n + offx[beta];
    const int *yperm = B.perm + (long long)B.R * B.n + (long long)r * B.m + offy[beta];
    const long long N = B.n + B.m;

    if (tid < TILE) {
        int li = ti * 64 + tid;
        long long gi = li < nx ? xperm[li] : -1;
        xi[tid] = gi;
        long long dst = -1;
        if (gi >= 0) {
            dst = B.rowbase_x[gi];
            for (int q = 0; q < r; ++q) dst += B.seg_x[(long long)q * B.n + gi].len;
        }
        xdst[tid] = dst;
        for (int q = 0; q < r; ++q) bx[q][tid] = gi >= 0 ? B.bucket[(long long)q * N + gi] : -1;
    } else if (tid < 2 * TILE) {
        int t = tid - TILE;
        int lj = tj * 64 + t;
        long long gj = lj < ny ? yperm[lj] : -1;
        yj[t] = gj >= 0 ? B.n + gj : -1;  // row of Z
        long long dst = -1;
        if (gj >= 0) {
            dst = B.rowbase_y[gj];
            for (int q = 0; q < r; ++q) dst += B.seg_y[(long long)q * B.m + gj].len;
        }
        ydst[t] = dst;
        for (int q = 0; q < r; ++q) by[q][t] = gj >= 0 ? B.bucket[(long long)q * N + B.n + gj] : -2;
    }
    if (tid == 0) cnt_sh = 0;

    TileAcc acc;
    tile_zero(acc);
    for (int k0 = 0; k0 < d; k0 += KCH) {
        __syncthreads();
        stage_rows(Ps, Z, d, xi, k0, d);
        stage_rows(Cs, Z, d, yj, k0, d);
        __syncthreads();
        if (cost == LCN_COST_COSINE)
            tile_fma<false>(acc, Ps, Cs);
        else
            tile_fma<true>(acc, Ps, Cs);
    }
    const int tx = tid & 15, ty = tid >> 4;
    double kv[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            long long gi = xi[ty * 4 + i], gj = yj[tx * 4 + j];
            double v = 0.0;
            if (gi >= 0 && gj >= 0) {
                double c = cost_from_acc(acc.v[i][j], cost, zn ? zn[gi] : 0.0, zn ? zn[gj] : 0.0);
                v = log_values ? -c * inv_lambda : exp(-c * inv_lambda);
            }
            kv[i][j] = v;
        }
    if (U) {
        // Nystrom value on the same pairs: sum_k U[i][k] * Wt[j][k]
        __syncthreads();
        if (tid < TILE) {
            if (yj[tid] >= 0) yj[tid] -= B.n;  // back to a row of Wt
        }
        tile_zero(acc);
        for (int k0 = 0; k0 < lp; k0 += KCH) {
            __syncthreads();
            stage_rows(Ps, U, lp, xi, k0, lp);
            stage_rows(Cs, Wt, lp, yj, k0, lp);
            __syncthreads();
            tile_fma<false>(acc, Ps, Cs);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) kv[i][j] -= acc.v[i][j];
    }
    // drop pairs an earlier round owns, count the rest
    unsigned mine = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int li = ty * 4 + i, lj = tx * 4 + j;
            bool present = xi[li] >= 0 && yj[lj] >= 0;
            bool dup = false;
            for (int q = 0; q < r; ++q) dup |= bx[q][li] == by[q][lj];
            if (!present || dup) kv[i][j] = log_values ? -INFINITY : 0.0;
            if (present && !dup) ++mine;
            vals[li][lj] = (float)kv[i][j];
        }
    atomicAdd(&cnt_sh, mine);
    __syncthreads();
    if (tid == 0) atomicAdd(unique_counter, (unsigned long long)cnt_sh);
    // write the piece into the row records of X and of Y, coalesced along each record
    const int lane = tid & 63, w = tid >> 6;
    for (int rr = w; rr < TILE; rr += 4) {
        const int lj = tj * 64 + lane;
        if (xdst[rr] >= 0 && lj < ny) vals_x[xdst[rr] + lj] = vals[rr][lane];
        const int li = ti * 64 + lane;
        if (ydst[rr] >= 0 && li < nx) vals_y[ydst[rr] + li] = vals[lane][rr];
    }
}

hipError_t launch_correction(const Handle &h, int ntiles, hipStream_t s)
{
    if (ntiles <= 0) return hipSuccess;
    const bool lcn_mode = h.mode == LCN_MODE_LCN;
    hipLaunchKernelGGL(correction_kernel, dim3(ntiles), dim3(256), 0, s, h.sort, h.Z, h.d, h.cost, 1.0 / h.lambda,
                       h.cost == LCN_COST_COSINE ? h.zn : (const double *)nullptr,
                       lcn_mode ? h.U : (const float *)nullptr, lcn_mode ? h.Wt : (const float *)nullptr, h.lp,
                       h.log_domain, h.vals_x, h.vals_y, h.counters + 3);
    return hipGetLastError();
}

}  // namespace lcn
