// Factor build: Nystrom factors U = k(X, L), V = k(L, Y), A = k(L, L) with
// k = exp(-c / lambda) (Sec. 4), the fp64 inverse of A and W = A^{-1} V (App.
// "Implementational details"), and the sparse values per bucket block:
// K^sp for sparse Sinkhorn (Sec. 3, eq. 3) or the correction K^sp - K^sp_Nys of
// K_LCN (Sec. 4).  Everything that feeds the inverse or a difference of nearly
// equal numbers is accumulated in fp64; only the stored factors are fp32.
// The contractions (point . landmark, point . point within a bucket, U . W, and
// the GEMMs of the inverse) run on the fp64 matrix instruction, 64 x 64 output
// tiles per workgroup, operands staged through LDS with the next chunks' global
// loads in flight; costs are formed from the dot product and fp64 squared norms.
#include "lcn_internal.h"

namespace lcn {

constexpr int TILE = 64;
constexpr int KCH = 32;
constexpr int LDK = KCH + 4;   // row stride of a staged chunk: rows 36 words apart put a wave's 64 operand reads on 64 banks

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
// 256 threads (4 wavefronts) hold a 64 x 64 tile of fp64 accumulators of a product P Q^T, built by
// the fp64 matrix instruction v_mfma_f64_16x16x4_f64: wavefront w owns the 32 x 32 quarter at rows
// 32 (w / 2), columns 32 (w % 2), as 2 x 2 instruction tiles of 16 x 16.  Operand layout of the
// instruction: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16] (one fp64 each, 4 deep) and
// receives D[4 v + l / 16][l % 16], v = 0..3.  A thread's 16 accumulators are numbered
// e = 4 (2 ti + tj) + v; tile_row / tile_col give their place in the 64 x 64 tile.
// Rows of both operands may be gathered through index lists held in LDS.

typedef double double4_t __attribute__((ext_vector_type(4)));

struct TileAcc {
    double4_t t[4];   // [2 ti + tj]
    __device__ inline double get(int e) const { return t[e >> 2][e & 3]; }
};

__device__ inline int tile_row(int e)
{
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    return 32 * (w >> 1) + 16 * (e >> 3) + 4 * (e & 3) + (l >> 4);
}

__device__ inline int tile_col(int e)
{
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    return 32 * (w & 1) + 16 * ((e >> 2) & 1) + (l & 15);
}

// stage 64 rows x KCH features of a row-major matrix into dst[row][k]
__device__ inline void stage_rows(float (*dst)[LDK], const float *__restrict__ base, long long ld,
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
        dst[r][kk] = v;
    }
}

// The same in two halves, so that a chunk's loads are in flight while the chunk before it is
// multiplied: 64 rows x KCH features into registers (row index + rowoff, absent if negative) ...
__device__ inline void fetch_rows(float (&v)[8], const float *__restrict__ base, long long ld,
                                  const long long *rowidx, long long rowoff, int k0, int kmax)
{
    const int kk = threadIdx.x & 31, r0 = threadIdx.x >> 5;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
        const long long src = rowidx[r0 + pass * 8];
        v[pass] = (src >= 0 && k0 + kk < kmax) ? base[(src + rowoff) * ld + k0 + kk] : 0.f;
    }
}

// ... and from the registers into dst[row][k]
__device__ inline void store_rows(float (*dst)[LDK], const float (&v)[8])
{
    const int kk = threadIdx.x & 31, r0 = threadIdx.x >> 5;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) dst[r0 + pass * 8][kk] = v[pass];
}

// The same for rows whose chunks start on 16-byte boundaries (ld a multiple of 4): thread t takes
// floats 4 (t % 8) .. + 3 of rows t / 8 and t / 8 + 32, one 16-byte load each.
typedef float float4_t __attribute__((ext_vector_type(4)));

__device__ inline void fetch_rows4(float (&v)[8], const float *__restrict__ base, long long ld,
                                   const long long *rowidx, long long rowoff, int k0, int kmax)
{
    const int q = threadIdx.x & 7, r = threadIdx.x >> 3;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const long long src = rowidx[r + 32 * hh];
        float4_t x = {0.f, 0.f, 0.f, 0.f};
        if (src >= 0 && k0 + 4 * q < kmax) x = *(const float4_t *)(base + (src + rowoff) * ld + k0 + 4 * q);
        v[4 * hh + 0] = x.x, v[4 * hh + 1] = x.y, v[4 * hh + 2] = x.z, v[4 * hh + 3] = x.w;
    }
}

__device__ inline void store_rows4(float (*dst)[LDK], const float (&v)[8])
{
    const int q = threadIdx.x & 7, r = threadIdx.x >> 3;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const float4_t x = {v[4 * hh + 0], v[4 * hh + 1], v[4 * hh + 2], v[4 * hh + 3]};
        *(float4_t *)&dst[r + 32 * hh][4 * q] = x;
    }
}

// acc += P_chunk Q_chunk^T for the KCH staged features (dot products; the staged values are fp32,
// products and sums fp64).  Only the first `rows` rows and `cols` columns of the tile hold points:
// an instruction tile of 16 x 16 that lies wholly outside is skipped (its accumulators stay zero).
__device__ inline void tile_mma(TileAcc &acc, const float (*Ps)[LDK], const float (*Cs)[LDK], int rows = TILE,
                                int cols = TILE)
{
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int rw = 32 * (w >> 1), cw = 32 * (w & 1);
    const int r0 = rw + (l & 15), c0 = cw + (l & 15), kq = l >> 4;
    const bool ra = rw < rows, rb = rw + 16 < rows, ca = cw < cols, cb = cw + 16 < cols;   // wave-uniform
    if (!ra || !ca) return;
    // Lane quarter kq feeds features 8 kq .. 8 kq + 7 of the chunk, one per instruction (the order
    // in which a dot product's terms are added is free): eight consecutive floats per operand row.
    typedef float f4 __attribute__((ext_vector_type(4)));
    auto row8 = [&](const float (*M)[LDK], int r, float (&o)[8]) {
        const f4 lo = *(const f4 *)&M[r][8 * kq], hi = *(const f4 *)&M[r][8 * kq + 4];
        o[0] = lo.x, o[1] = lo.y, o[2] = lo.z, o[3] = lo.w, o[4] = hi.x, o[5] = hi.y, o[6] = hi.z, o[7] = hi.w;
    };
    float a0[8], b0[8], a1[8] = {}, b1[8] = {};
    row8(Ps, r0, a0);
    row8(Cs, c0, b0);
    if (rb) row8(Ps, r0 + 16, a1);
    if (cb) row8(Cs, c0 + 16, b1);
#pragma unroll
    for (int ks = 0; ks < KCH / 4; ++ks) {
        acc.t[0] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a0[ks], (double)b0[ks], acc.t[0], 0, 0, 0);
        if (cb) acc.t[1] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a0[ks], (double)b1[ks], acc.t[1], 0, 0, 0);
        if (rb) acc.t[2] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a1[ks], (double)b0[ks], acc.t[2], 0, 0, 0);
        if (rb && cb) acc.t[3] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a1[ks], (double)b1[ks], acc.t[3], 0, 0, 0);
    }
}

__device__ inline void tile_zero(TileAcc &acc)
{
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc.t[q][v] = 0.0;
}

// cost from the dot product and the squared norms of the two points; the squared distance is
// |p|^2 + |q|^2 - 2 p.q in fp64 (rounding can leave it a hair below zero for coinciding points)
// For the cosine cost the callers pass, instead of the squared norms, their inverse roots (taken once
// per row and column of a tile, not once per pair): 1 - p.q / (|p| |q|).
__device__ inline double cost_from_dot(double dot, int cost, double pn, double qn)
{
    if (cost == LCN_COST_COSINE) return 1.0 - dot * pn * qn;
    const double sq = fmax(pn + qn - 2.0 * dot, 0.0);
    return cost == LCN_COST_EUCLID ? sqrt(sq) : sq;
}

// what cost_from_dot wants of a point's squared norm
__device__ inline double norm_term(double sqnorm, int cost)
{
    return cost == LCN_COST_COSINE ? 1.0 / sqrt(sqnorm) : sqnorm;
}

// Which 64 x 64 tile of a (row tiles x col_tiles) grid a workgroup of a one-dimensional launch takes.
// Workgroups go to the eight dies in turn, each die with a cache of its own: die x takes the row tiles
// x, x + 8, ... and runs through all column tiles of one row tile back to back, so the rows of the tall
// operand are fetched from memory once instead of once per column tile.  (A different dealing of
// workgroups to dies costs bandwidth, not correctness.)
__device__ inline void die_tile(int col_tiles, long long &row_tile, int &col_tile)
{
    const unsigned w = blockIdx.x, s = w >> 3;
    col_tile = (int)(s % (unsigned)col_tiles);
    row_tile = (long long)(s / (unsigned)col_tiles) * 8 + (w & 7);
}

static unsigned die_grid(long long rows, int cols)
{
    const long long rt = (rows + TILE - 1) / TILE, ct = (cols + TILE - 1) / TILE;
    return (unsigned)((rt + 7) / 8 * 8 * ct);
}

// ----------------------------------------------------- kernel matrix k(P, Q) --

__global__ __launch_bounds__(256) void kernel_matrix_kernel(const float *__restrict__ P, long long rows,
                                                            const float *__restrict__ Q, int cols, int d, int cost,
                                                            double inv_lambda, const double *__restrict__ pn,
                                                            const double *__restrict__ qn, float *out32,
                                                            double *out64, int ldo)
{
    __shared__ __align__(16) float Ps[TILE][LDK];
    __shared__ __align__(16) float Cs[TILE][LDK];
    __shared__ long long pidx[TILE], qidx[TILE];
    __shared__ double pterm[TILE], qterm[TILE];   // per row / column of the tile: see norm_term
    const int tid = threadIdx.x;
    long long ptile;
    int qtile;
    die_tile((cols + TILE - 1) / TILE, ptile, qtile);
    const long long p0 = ptile * TILE;
    const int q0 = qtile * TILE;
    if (p0 >= rows) return;   // padding of the launch to a multiple of eight row tiles
    if (tid < TILE) {
        pidx[tid] = p0 + tid < rows ? p0 + tid : -1;
        qidx[tid] = q0 + tid < cols ? q0 + tid : -1;
        pterm[tid] = p0 + tid < rows ? norm_term(pn[p0 + tid], cost) : 0.0;
    } else if (tid < 2 * TILE) {
        const int t = tid - TILE;
        qterm[t] = q0 + t < cols ? norm_term(qn[q0 + t], cost) : 0.0;
    }
    TileAcc acc;
    tile_zero(acc);
    // the loads of two chunks are in flight while a chunk is multiplied
    const int nd = (d + KCH - 1) / KCH;
    const bool vec = (d & 3) == 0 && (((size_t)P | (size_t)Q) & 15) == 0;   // rows start on 16-byte boundaries
    struct Chunk {
        float p[8], c[8];
    };
    auto fetch = [&](Chunk &C, int c) {
        if (c >= nd) return;
        if (vec) {
            fetch_rows4(C.p, P, d, pidx, 0, c * KCH, d);
            fetch_rows4(C.c, Q, d, qidx, 0, c * KCH, d);
        } else {
            fetch_rows(C.p, P, d, pidx, 0, c * KCH, d);
            fetch_rows(C.c, Q, d, qidx, 0, c * KCH, d);
        }
    };
    auto step = [&](Chunk &C, int c) {
        __syncthreads();
        if (vec) {
            store_rows4(Ps, C.p);
            store_rows4(Cs, C.c);
        } else {
            store_rows(Ps, C.p);
            store_rows(Cs, C.c);
        }
        __syncthreads();
        fetch(C, c + 2);
        tile_mma(acc, Ps, Cs);
    };
    Chunk ch[2] = {};
    __syncthreads();   // pidx, qidx
    fetch(ch[0], 0);
    fetch(ch[1], 1);
    for (int c = 0; c < nd; c += 2) {
        step(ch[0], c);
        if (c + 1 < nd) step(ch[1], c + 1);
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const long long p = p0 + tile_row(e);
        const int q = q0 + tile_col(e);
        if (p >= rows || q >= cols) continue;
        // a point against itself (the diagonal of the landmarks' matrix) is at cost zero exactly
        double c = (P == Q && p == q) ? 0.0 : cost_from_dot(acc.get(e), cost, pterm[tile_row(e)], qterm[tile_col(e)]);
        const double sq_est = cost == LCN_COST_EUCLID ? c * c : c;
        if (P == Q && p != q && cost != LCN_COST_COSINE && sq_est <= 1e-9 * (pn[p] + qn[q])) {
            // two landmarks (nearly) on top of each other: the norms cancel, so the squared distance is
            // taken from the differences; coinciding landmarks give exactly zero and a singular matrix
            double sq = 0.0;
            for (int kk = 0; kk < d; ++kk) {
                const double df = (double)P[p * d + kk] - (double)Q[(long long)q * d + kk];
                sq = fma(df, df, sq);
            }
            c = cost == LCN_COST_EUCLID ? sqrt(sq) : sq;
        }
        const double kv = exp(-c * inv_lambda);
        if (out32) out32[p * ldo + q] = (float)kv;
        if (out64) out64[p * cols + q] = kv;
    }
}

hipError_t launch_kernel_matrix(const float *P, long long rows, const float *Q, int cols, int d, int cost,
                                double lambda, const double *pn, const double *qn, float *out32, double *out64,
                                int ldo, hipStream_t s)
{
    if (rows <= 0 || cols <= 0) return hipSuccess;
    hipLaunchKernelGGL(kernel_matrix_kernel, dim3(die_grid(rows, cols)), dim3(256), 0, s, P, rows, Q, cols, d, cost, 1.0 / lambda, pn, qn,
                       out32, out64, ldo);
    return hipGetLastError();
}

// ----------------------------------------------------------- fp64 inverse --
//
// A is symmetric positive definite (a PSD kernel matrix, plus the ridge).
// Blocked right-looking Cholesky A = L L^T with 64-wide panels: the diagonal
// block is factored and inverted in LDS by one workgroup, the panel below and
// the trailing matrix are updated by tiled fp64 GEMMs.  Then X = L^{-1} is
// built block row by block row from the inverted diagonal blocks, and
// A^{-1} = X^T X.

constexpr int NB = 64;

// C (M x N, ld ldc) = beta * C + alpha * op(A) * op(B); op = transpose when the flag is set.
// A is M x K (lda) or, transposed, stored K x M; B is K x N (ldb) or, transposed, stored N x K.
// Optional fp32 copy of the result (ld ldc32).
__global__ __launch_bounds__(256) void gemm64_kernel(const double *A, int lda, int transA, const double *B, int ldb,
                                                     int transB, double *C,
                                                     int ldc, long long M, int N, int K, double alpha, double beta,
                                                     float *C32, int ldc32)
{
    constexpr int KC = 16;
    __shared__ double As[KC][TILE + 2];
    __shared__ double Bs[KC][TILE + 2];
    const int tid = threadIdx.x;
    long long rtile;
    int ctile;
    die_tile((N + TILE - 1) / TILE, rtile, ctile);
    const long long r0 = rtile * TILE;
    const int c0 = ctile * TILE;
    if (r0 >= M) return;   // padding of the launch to a multiple of eight row tiles
    const int wv = tid >> 6, ln = tid & 63;
    const int ar = 32 * (wv >> 1) + (ln & 15), bc = 32 * (wv & 1) + (ln & 15), kq4 = ln >> 4;
    TileAcc acc;
    tile_zero(acc);
    // a chunk's loads are requested before the chunk ahead of it is multiplied
    double ra[4], rb[4];
    auto fetch = [&](int k0) {
        if (transA) {
            const int rr = tid & 63, kq = tid >> 6;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int kk = kq + pass * 4;
                ra[pass] = (r0 + rr < M && k0 + kk < K) ? A[(long long)(k0 + kk) * lda + r0 + rr] : 0.0;
            }
        } else {
            const int kk = tid & 15, rq = tid >> 4;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int rr = rq + pass * 16;
                ra[pass] = (r0 + rr < M && k0 + kk < K) ? A[(r0 + rr) * lda + k0 + kk] : 0.0;
            }
        }
        if (transB) {
            const int kk = tid & 15, cq = tid >> 4;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int cc = cq + pass * 16;
                rb[pass] = (c0 + cc < N && k0 + kk < K) ? B[(long long)(c0 + cc) * ldb + k0 + kk] : 0.0;
            }
        } else {
            const int cc = tid & 63, kq = tid >> 6;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int kk = kq + pass * 4;
                rb[pass] = (c0 + cc < N && k0 + kk < K) ? B[(long long)(k0 + kk) * ldb + c0 + cc] : 0.0;
            }
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += KC) {
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            if (transA)
                As[(tid >> 6) + pass * 4][tid & 63] = ra[pass];
            else
                As[tid & 15][(tid >> 4) + pass * 16] = ra[pass];
            if (transB)
                Bs[tid & 15][(tid >> 4) + pass * 16] = rb[pass];
            else
                Bs[(tid >> 6) + pass * 4][tid & 63] = rb[pass];
        }
        __syncthreads();
        if (k0 + KC < K) fetch(k0 + KC);
#pragma unroll
        for (int ks = 0; ks < KC / 4; ++ks) {
            const int k = 4 * ks + kq4;
            const double a0 = As[k][ar], a1 = As[k][ar + 16];
            const double b0 = Bs[k][bc], b1 = Bs[k][bc + 16];
            acc.t[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc.t[0], 0, 0, 0);
            acc.t[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc.t[1], 0, 0, 0);
            acc.t[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc.t[2], 0, 0, 0);
            acc.t[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc.t[3], 0, 0, 0);
        }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const long long r = r0 + tile_row(e);
        const int c = c0 + tile_col(e);
        if (r >= M || c >= N) continue;
        double v = alpha * acc.get(e);
        if (beta != 0.0) v += beta * C[r * ldc + c];
        if (C) C[r * ldc + c] = v;
        if (C32) C32[r * ldc32 + c] = (float)v;
    }
}

static void gemm64(const double *A, int lda, bool tA, const double *B, int ldb, bool tB, double *C, int ldc,
                   long long M, int N, int K, double alpha, double beta, float *C32, int ldc32, hipStream_t s)
{
    if (M <= 0 || N <= 0) return;
    hipLaunchKernelGGL(gemm64_kernel, dim3(die_grid(M, N)), dim3(256), 0, s, A, lda, tA ? 1 : 0, B, ldb, tB ? 1 : 0, C, ldc, M, N, K,
                       alpha, beta, C32, ldc32);
}

hipError_t launch_gemm_f64(const double *A, const double *B, long long M, int N, int K, float *C32, int ldc,
                           hipStream_t s)
{
    gemm64(A, K, false, B, N, false, nullptr, 0, M, N, K, 1.0, 0.0, C32, ldc, s);
    return hipGetLastError();
}

// One workgroup of 256 threads: Cholesky factor of the nb x nb diagonal block at (j0, j0) of Lm
// (ridge added to its diagonal), written back into Lm's lower triangle, and the inverse of that
// triangular factor into Dinv (NB x NB, zero above the diagonal and outside nb).
// A block smaller than NB is padded with the identity.  The block is worked through in panels of
// PB columns: one wavefront factors the panel's PB x PB diagonal part with a row per lane (the
// pivot column is passed on by lane reads, no barrier), a thread per row below solves against it,
// and all threads update the columns to the right, which they hold as 4 x 4 register patches
// (thread (ty, tx): rows 4 ty.., columns 4 tx..).  Three barriers per panel.  The inverse is built
// from the inverses of the 16 x 16 diagonal parts (a thread per column, forward substitution) and
// three rounds of 16 x 16 block products, X_ij = -X_ii sum_k L_ik X_kj.
constexpr int PB = 8;            // panel width
constexpr int CB = 16;           // block size of the inverse
constexpr int CLD = NB + 1;      // row stride of the LDS copies
constexpr size_t CHOL_LDS = sizeof(double) * (2 * NB * CLD + 3 * CB * CB + NB);

__device__ inline double lane_read64(double v, int lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// 1 / sqrt(x) to fp64 rounding for positive normal x: hardware estimate and two Newton steps
__device__ inline double rsqrt64(double x)
{
    double r = __builtin_amdgcn_rsq(x);
    r = fma(0.5 * r, fma(-x * r, r, 1.0), r);
    r = fma(0.5 * r, fma(-x * r, r, 1.0), r);
    return r;
}

__global__ __launch_bounds__(256) void chol_diag_kernel(double *Lm, int l, int j0, int nb, double ridge, double *Dinv,
                                                        int *fail_flag)
{
    extern __shared__ double chol_lds[];
    double (*As)[CLD] = reinterpret_cast<double (*)[CLD]>(chol_lds);                 // the block, then L
    double (*Xs)[CLD] = reinterpret_cast<double (*)[CLD]>(chol_lds + NB * CLD);      // L^{-1}
    double (*Ts)[CB][CB] = reinterpret_cast<double (*)[CB][CB]>(chol_lds + 2 * NB * CLD);
    double *rs_sh = chol_lds + 2 * NB * CLD + 3 * CB * CB;                           // 1 / L_jj
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    double p[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = 4 * ty + a, k = 4 * tx + b;
            double v = (i == k) ? 1.0 : 0.0;
            if (i < nb && k < nb) v = Lm[(long long)(j0 + i) * l + j0 + k] + (i == k ? ridge : 0.0);
            p[a][b] = v;
            Xs[i][k] = 0.0;
        }
    bool fail = false;
    for (int sb = 0; sb < NB / PB; ++sb) {
        const int c0 = PB * sb;
        // the panel's columns leave the registers (rows above the panel are not needed any more)
        if ((4 * tx) / PB == sb && ty >= tx) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) As[4 * ty + a][4 * tx + b] = p[a][b];
        }
        __syncthreads();
        if (tid < 64) {
            // lane r < 16 holds row c0 + r of the diagonal part; entries right of the diagonal are never used
            const int r = tid & (PB - 1);
            double a[PB];
#pragma unroll
            for (int k = 0; k < PB; ++k) a[k] = As[c0 + r][c0 + k];
#pragma unroll
            for (int c = 0; c < PB; ++c) {
                double dd = lane_read64(a[c], c);
                if (!(dd > 0.0)) {
                    fail = true;
                    dd = 1.0;
                }
                const double rs = rsqrt64(dd);
                if (tid == 0) rs_sh[c0 + c] = rs;
                a[c] *= rs;
#pragma unroll
                for (int k = c + 1; k < PB; ++k) a[k] = fma(-a[c], lane_read64(a[c], k), a[k]);
            }
            if (tid < PB) {
#pragma unroll
                for (int k = 0; k < PB; ++k) As[c0 + r][c0 + k] = a[k];
            }
        }
        __syncthreads();
        // rows below the diagonal part: x L11^T = a, a thread per row
        const int below = NB - c0 - PB;
        if (tid < below) {
            const int r = c0 + PB + tid;
            double x[PB];
#pragma unroll
            for (int k = 0; k < PB; ++k) x[k] = As[r][c0 + k];
#pragma unroll
            for (int q = 0; q < PB; ++q) {   // column q is final: take it out of the columns to its right
                x[q] *= rs_sh[c0 + q];
#pragma unroll
                for (int k = q + 1; k < PB; ++k) x[k] = fma(-x[q], As[c0 + k][c0 + q], x[k]);
            }
#pragma unroll
            for (int k = 0; k < PB; ++k) As[r][c0 + k] = x[k];
        }
        __syncthreads();
        // columns to the right of the panel, on or below the diagonal
        if (4 * tx >= c0 + PB && tx <= ty) {
#pragma unroll
            for (int kk = 0; kk < PB; ++kk) {
                double li[4], lk[4];
#pragma unroll
                for (int a = 0; a < 4; ++a) li[a] = As[4 * ty + a][c0 + kk];
#pragma unroll
                for (int b = 0; b < 4; ++b) lk[b] = As[4 * tx + b][c0 + kk];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) p[a][b] = fma(-li[a], lk[b], p[a][b]);
            }
        }
    }
    if (fail && tid == 0) *fail_flag = 1;
    // As holds L on and below the diagonal
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = 4 * ty + a, k = 4 * tx + b;
            if (i < nb && k <= i) Lm[(long long)(j0 + i) * l + j0 + k] = As[i][k];
        }
    // inverses of the four diagonal parts: thread c takes column c % 16 of part c / 16
    if (tid < NB) {
        const int base = tid & ~(CB - 1), cc = tid & (CB - 1);
        double x[CB];
#pragma unroll
        for (int r = 0; r < CB; ++r) x[r] = (r == cc) ? 1.0 : 0.0;
#pragma unroll
        for (int k = 0; k < CB; ++k) {   // x[k] is final (zero above row cc): take it out of the rows below
            x[k] *= rs_sh[base + k];
#pragma unroll
            for (int r = k + 1; r < CB; ++r) x[r] = fma(-As[base + r][base + k], x[k], x[r]);
        }
#pragma unroll
        for (int r = 0; r < CB; ++r) Xs[base + r][base + cc] = x[r];
    }
    __syncthreads();
    // parts further and further below the diagonal
    const int er = tid >> 4, ec = tid & 15;
    for (int dist = 1; dist < NB / CB; ++dist) {
        for (int i = dist; i < NB / CB; ++i) {
            const int j = i - dist;
            double t = 0.0;
            for (int kb = j; kb < i; ++kb) {
#pragma unroll
                for (int k = 0; k < CB; ++k) t = fma(As[CB * i + er][CB * kb + k], Xs[CB * kb + k][CB * j + ec], t);
            }
            Ts[i - dist][er][ec] = t;
        }
        __syncthreads();
        for (int i = dist; i < NB / CB; ++i) {
            const int j = i - dist;
            double t = 0.0;
#pragma unroll
            for (int k = 0; k < CB; ++k) t = fma(Xs[CB * i + er][CB * i + k], Ts[i - dist][k][ec], t);
            Xs[CB * i + er][CB * j + ec] = -t;
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = 4 * ty + a, k = 4 * tx + b;
            Dinv[i * NB + k] = (i < nb && k < nb) ? Xs[i][k] : 0.0;
        }
}

__global__ void copy_f64_kernel(const double *src, double *dst, long long count)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = src[i];
}

// dst (rows x cols, ld ldd) = src (ld lds)
__global__ void copy_block_kernel(const double *src, int lds, double *dst, int ldd, int rows, int cols)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows * cols) return;
    const int i = e / cols, j = e % cols;
    dst[(long long)i * ldd + j] = src[(long long)i * lds + j];
}

// Lm: work copy that ends up holding L in its lower triangle; Xm: L^{-1};
// Dinv: the inverted diagonal blocks, ceil(l / 64) of NB x NB; Tm: NB x l scratch;
// Ainv: the result.
hipError_t launch_spd_inverse(double *A, int l, double ridge, double *Lm, double *Xm, double *Ainv, double *Dinv,
                              double *Tm, int *fail_flag, hipStream_t s)
{
    const long long ll = (long long)l * l;
    hipLaunchKernelGGL(copy_f64_kernel, dim3((unsigned)((ll + 255) / 256)), dim3(256), 0, s, A, Lm, ll);
    hipError_t e = hipMemsetAsync(Xm, 0, sizeof(double) * (size_t)ll, s);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)chol_diag_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)CHOL_LDS);
    if (e != hipSuccess) return e;
    const int panels = (l + NB - 1) / NB;
    for (int p = 0; p < panels; ++p) {
        const int j0 = p * NB;
        const int nb = l - j0 < NB ? l - j0 : NB;
        double *Dp = Dinv + (long long)p * NB * NB;
        hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(256), CHOL_LDS, s, Lm, l, j0, nb, ridge, Dp, fail_flag);
        const int below = l - j0 - nb;
        if (below > 0) {
            double *A21 = Lm + (long long)(j0 + nb) * l + j0;
            double *A22 = Lm + (long long)(j0 + nb) * l + j0 + nb;
            // L21 = A21 * L11^{-T}, in place: nb <= 64 columns, so one workgroup owns a row tile and
            // has read all of it before it writes
            gemm64(A21, l, false, Dp, NB, true, A21, l, below, nb, nb, 1.0, 0.0, nullptr, 0, s);
            // A22 -= L21 * L21^T
            gemm64(A21, l, false, A21, l, true, A22, l, below, below, nb, -1.0, 1.0, nullptr, 0, s);
        }
    }
    // X = L^{-1}, block row i:  X_ii = L_ii^{-1},  X_i,<i = -L_ii^{-1} (L_i,<i X_<i,<i)
    for (int p = 0; p < panels; ++p) {
        const int i0 = p * NB;
        const int nb = l - i0 < NB ? l - i0 : NB;
        double *Dp = Dinv + (long long)p * NB * NB;
        hipLaunchKernelGGL(copy_block_kernel, dim3((nb * nb + 255) / 256), dim3(256), 0, s, Dp, NB,
                           Xm + (long long)i0 * l + i0, l, nb, nb);
        if (i0 > 0) {
            gemm64(Lm + (long long)i0 * l, l, false, Xm, l, false, Tm, l, nb, i0, i0, -1.0, 0.0, nullptr, 0, s);
            gemm64(Dp, NB, false, Tm, l, false, Xm + (long long)i0 * l, l, nb, i0, nb, 1.0, 0.0, nullptr, 0, s);
        }
    }
    // A^{-1} = X^T X
    gemm64(Xm, l, true, Xm, l, false, Ainv, l, l, l, l, 1.0, 0.0, nullptr, 0, s);
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
                                                         unsigned long long *unique_counter, BackwardArgs bw)
{
    __shared__ __align__(16) float Ps[TILE][LDK];
    __shared__ __align__(16) float Cs[TILE][LDK];
    __shared__ float vals[TILE][TILE + 1];
    __shared__ long long xi[TILE], yj[TILE];
    __shared__ double xterm[TILE], yterm[TILE];   // per row / column of the tile: see norm_term
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
        xterm[tid] = gi >= 0 ? norm_term(zn[gi], cost) : 0.0;
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
        yterm[t] = gj >= 0 ? norm_term(zn[B.n + gj], cost) : 0.0;
        long long dst = -1;
        if (gj >= 0) {
            dst = B.rowbase_y[gj];
            for (int q = 0; q < r; ++q) dst += B.seg_y[(long long)q * B.m + gj].len;
        }
        ydst[t] = dst;
        for (int q = 0; q < r; ++q) by[q][t] = gj >= 0 ? B.bucket[(long long)q * N + B.n + gj] : -2;
    }
    if (tid == 0) cnt_sh = 0;
    const int rows_here = nx - ti * 64 < 64 ? nx - ti * 64 : 64;   // members of the bucket in this piece
    const int cols_here = ny - tj * 64 < 64 ? ny - tj * 64 : 64;

    // One run of chunks: the features of the points (exact cost), then, in the lcn mode, the
    // Nystrom value on the same pairs, sum_k U[i][k] Wt[j][k].  The loads of a chunk are requested
    // before the chunk ahead of it is multiplied.
    const int nd = (d + KCH - 1) / KCH, nl = U ? (lp + KCH - 1) / KCH : 0;
    constexpr int DEPTH = 2;          // chunks whose loads are in flight (3 measured slower: registers)
    const bool vecz = (d & 3) == 0;   // rows of Z start on 16-byte boundaries (lp is a multiple of 64)
    struct Chunk {
        float p[8], c[8];
    };
    auto fetch = [&](Chunk &C, int c) {
        if (c >= nd + nl) return;
        if (c >= nd) {
            fetch_rows4(C.p, U, lp, xi, 0, (c - nd) * KCH, lp);
            fetch_rows4(C.c, Wt, lp, yj, -(long long)B.n, (c - nd) * KCH, lp);   // yj: rows of Z; Wt has the rows of Y
        } else if (vecz) {
            fetch_rows4(C.p, Z, d, xi, 0, c * KCH, d);
            fetch_rows4(C.c, Z, d, yj, 0, c * KCH, d);
        } else {
            fetch_rows(C.p, Z, d, xi, 0, c * KCH, d);
            fetch_rows(C.c, Z, d, yj, 0, c * KCH, d);
        }
    };
    TileAcc acc;
    tile_zero(acc);
    double kv[16];
    // chunk c: its registers go to LDS, the loads of chunk c + DEPTH take their place, chunk c is multiplied
    auto step = [&](Chunk &C, int c) {
        __syncthreads();
        if (c >= nd || vecz) {
            store_rows4(Ps, C.p);
            store_rows4(Cs, C.c);
        } else {
            store_rows(Ps, C.p);
            store_rows(Cs, C.c);
        }
        __syncthreads();
        fetch(C, c + DEPTH);
        tile_mma(acc, Ps, Cs, rows_here, cols_here);
        if (c == nd - 1) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int li = tile_row(e), lj = tile_col(e);
                const long long gi = xi[li], gj = yj[lj];
                double v = 0.0;
                if (gi >= 0 && gj >= 0) {
                    const double cc = cost_from_dot(acc.get(e), cost, xterm[li], yterm[lj]);
                    v = log_values ? -cc * inv_lambda : exp(-cc * inv_lambda);
                }
                kv[e] = v;
            }
            tile_zero(acc);
        }
    };
    Chunk ch[DEPTH] = {};
    __syncthreads();   // xi, yj
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) fetch(ch[j], j);
    for (int c = 0; c < nd + nl; c += DEPTH) {
#pragma unroll
        for (int j = 0; j < DEPTH; ++j)
            if (c + j < nd + nl) step(ch[j], c + j);
    }
    if (U && !bw.lin_u) {
#pragma unroll
        for (int e = 0; e < 16; ++e) kv[e] -= acc.get(e);
    }
    if (bw.lin_u) {
        // derivatives instead of kernel values (Prop. 1): -lambda u_i K^sp_ij v_j and, from the
        // Nystrom value still in `acc`, +lambda u_i K^sp_Nys,ij v_j, into the records of X only
        const double scale = bw.lambda * exp(bw.acc_y[lp] + bw.acc_z[lp]);  // exponents taken out of v and u
        for (int which = 0; which < (U ? 2 : 1); ++which) {
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int li = tile_row(e), lj = tile_col(e);
                const long long gi = xi[li], gj = yj[lj];
                double g = 0.0;
                if (gi >= 0 && gj >= 0) {
                    const double uv = bw.lin_u[gi] * bw.lin_v[gj - B.n] * scale;
                    g = which == 0 ? -uv * kv[e] : uv * acc.get(e);
                }
                vals[li][lj] = (float)g;
            }
            __syncthreads();
            float *dst = which == 0 ? bw.rec_sp : bw.rec_nys;
            const int lane = tid & 63, w = tid >> 6;
            if (dst)
                for (int rr = w; rr < TILE; rr += 4) {
                    const int lj = tj * 64 + lane;
                    if (xdst[rr] >= 0 && lj < ny) dst[xdst[rr] + lj] = vals[rr][lane];
                }
        }
        return;
    }
    // drop pairs an earlier round owns, count the rest
    unsigned mine = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int li = tile_row(e), lj = tile_col(e);
        bool present = xi[li] >= 0 && yj[lj] >= 0;
        bool dup = false;
        for (int q = 0; q < r; ++q) dup |= bx[q][li] == by[q][lj];
        if (!present || dup) kv[e] = log_values ? -INFINITY : 0.0;
        if (present && !dup) ++mine;
        vals[li][lj] = (float)kv[e];
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
                       h.zn, lcn_mode ? h.U : (const float *)nullptr, lcn_mode ? h.Wt : (const float *)nullptr, h.lp,
                       h.log_domain, h.vals_x, h.vals_y, h.counters + 3, BackwardArgs{});
    return hipGetLastError();
}

// Derivatives on the pattern for the lcn mode, in the layout of the row records of X
// (rec_sp, rec_nys: nnz_stored floats each, either may be null).
hipError_t launch_backward_pattern(const Handle &h, float *rec_sp, float *rec_nys, hipStream_t s)
{
    if (h.ntiles <= 0) return hipSuccess;
    BackwardArgs bw;
    bw.lin_u = h.lin_u;
    bw.lin_v = h.lin_v;
    bw.acc_y = h.acc[0];
    bw.acc_z = h.acc[1];
    bw.lambda = h.lambda;
    bw.rec_sp = rec_sp;
    bw.rec_nys = rec_nys;
    hipLaunchKernelGGL(correction_kernel, dim3(h.ntiles), dim3(256), 0, s, h.sort, h.Z, h.d, h.cost, 1.0 / h.lambda,
                       h.zn, h.U, h.Wt, h.lp, 0,
                       (float *)nullptr, (float *)nullptr, (unsigned long long *)nullptr, bw);
    return hipGetLastError();
}

// out[i][k] = -lambda x_i acc_k for i < rows, k < l (Prop. 1: x = u, acc = W v for dU; x = v,
// acc = U^T u for dW^T); x and acc are held with exponents taken out, which `acc_a[lp] + acc_b[lp]` restores
__global__ void outer_kernel(const double *__restrict__ lin, long long rows, const double *__restrict__ acc,
                             const double *__restrict__ acc_a, const double *__restrict__ acc_b, int l, int lp,
                             double lambda, float *__restrict__ out)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows * l) return;
    const long long i = e / l;
    const int k = (int)(e - i * l);
    const double scale = -lambda * exp(acc_a[lp] + acc_b[lp]);
    out[e] = (float)(scale * lin[i] * acc[k]);
}

hipError_t launch_backward_factors(const Handle &h, float *gU, float *gWt, hipStream_t s)
{
    if (gU)
        hipLaunchKernelGGL(outer_kernel, dim3((unsigned)((h.n * h.l + 255) / 256)), dim3(256), 0, s, h.lin_u, h.n,
                           h.acc[0], h.acc[0], h.acc[1], h.l, h.lp, h.lambda, gU);
    if (gWt)
        hipLaunchKernelGGL(outer_kernel, dim3((unsigned)((h.m * h.l + 255) / 256)), dim3(256), 0, s, h.lin_v, h.m,
                           h.acc[1], h.acc[0], h.acc[1], h.l, h.lp, h.lambda, gWt);
    return hipGetLastError();
}

// Nystrom part of the plan for a block of rows: out[i - i0][j] = u_i (U_i . W_:j) v_j, 64 x 64 per workgroup.
__global__ __launch_bounds__(256) void plan_nystrom_kernel(const float *__restrict__ U, const float *__restrict__ Wt,
                                                           int lp, long long i0, long long nrows, long long m,
                                                           const double *__restrict__ lin_u,
                                                           const double *__restrict__ lin_v,
                                                           const double *__restrict__ acc_y,
                                                           const double *__restrict__ acc_z, float *__restrict__ out)
{
    __shared__ __align__(16) float Ps[TILE][LDK];
    __shared__ __align__(16) float Cs[TILE][LDK];
    __shared__ long long xi[TILE], yj[TILE];
    const int tid = threadIdx.x;
    if (tid < TILE) {
        const long long i = (long long)blockIdx.y * TILE + tid;
        xi[tid] = i < nrows ? i0 + i : -1;
    } else if (tid < 2 * TILE) {
        const long long j = (long long)blockIdx.x * TILE + tid - TILE;
        yj[tid - TILE] = j < m ? j : -1;
    }
    TileAcc acc;
    tile_zero(acc);
    for (int k0 = 0; k0 < lp; k0 += KCH) {
        __syncthreads();
        stage_rows(Ps, U, lp, xi, k0, lp);
        stage_rows(Cs, Wt, lp, yj, k0, lp);
        __syncthreads();
        tile_mma(acc, Ps, Cs);
    }
    const double scale = exp(acc_y[lp] + acc_z[lp]);  // exponents taken out of v and u
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const long long gi = xi[tile_row(e)], gj = yj[tile_col(e)];
        if (gi >= 0 && gj >= 0) out[(gi - i0) * m + gj] = (float)(acc.get(e) * lin_u[gi] * lin_v[gj] * scale);
    }
}

hipError_t launch_plan_nystrom(const Handle &h, long long i0, long long nrows, float *out, hipStream_t s)
{
    dim3 grid((unsigned)((h.m + TILE - 1) / TILE), (unsigned)((nrows + TILE - 1) / TILE));
    hipLaunchKernelGGL(plan_nystrom_kernel, grid, dim3(256), 0, s, h.U, h.Wt, h.lp, i0, nrows, h.m, h.lin_u, h.lin_v,
                       h.acc[0], h.acc[1], out);
    return hipGetLastError();
}

// Kernels held as logs (sparse, dense): -lambda exp(log u_i + log K_ij + log v_j) for every stored
// entry, in the layout of the row records of X; one wavefront per row.
__global__ __launch_bounds__(256) void backward_log_kernel(SortBuffers B, const float *__restrict__ vals_x,
                                                           const double *__restrict__ log_u,
                                                           const double *__restrict__ perm_log_v, double lambda,
                                                           float *__restrict__ rec_sp)
{
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= B.n) return;
    const int lane = threadIdx.x & 63;
    const double lu = log_u[i];
    long long at = B.rowbase_x[i];
    for (int r = 0; r < B.R; ++r) {
        const Seg sg = B.seg_x[(long long)r * B.n + i];
        for (int e = lane; e < sg.len; e += 64) {
            const double t = (double)vals_x[at + e] + lu + perm_log_v[sg.vstart + e];
            rec_sp[at + e] = t > -INFINITY ? (float)(-lambda * exp(t)) : 0.f;
        }
        at += sg.len;
    }
}

hipError_t launch_backward_log(const Handle &h, float *rec_sp, hipStream_t s)
{
    hipLaunchKernelGGL(backward_log_kernel, dim3((unsigned)((h.n + 3) / 4)), dim3(256), 0, s, h.sort, h.vals_x, h.lin_u,
                       h.perm_v, h.lambda, rec_sp);
    return hipGetLastError();
}

}  // namespace lcn
