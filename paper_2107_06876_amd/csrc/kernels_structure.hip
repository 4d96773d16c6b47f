// Structure build: input conversion, exact-rule bucket assignment (k-means
// and cross-polytope hashing), the k-means centroid update, the bucket sort
// into blocks, and the CSR export.
//
// This file is compiled with -ffp-contract=off: the bucket of a point is
// decided by fp64 arithmetic evaluated in a fixed order with separate
// multiplies and adds, so that it is a function of the inputs alone.
#include "lcn_internal.h"

#pragma clang fp contract(off)

namespace lcn {

// ------------------------------------------------------------- conversion --

__global__ void convert_kernel(const void *X, long long nx_elems, const void *Y, long long total, int dtype, float *Z,
                               unsigned *range_flag)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long stride = (long long)gridDim.x * blockDim.x;
    bool bad = false;
    for (; i < total; i += stride) {
        const void *src = i < nx_elems ? X : Y;
        long long j = i < nx_elems ? i : i - nx_elems;
        float v;
        if (dtype == LCN_BF16) {
            unsigned bits = ((const unsigned short *)src)[j];
            v = __uint_as_float(bits << 16);
        } else {
            v = ((const float *)src)[j];
        }
        Z[i] = v;
        bad |= !(fabsf(v) < 1024.0f);
    }
    if (bad) atomicOr(range_flag, 1u);
}

hipError_t launch_convert(const void *X, long long n, const void *Y, long long m, int d, int dtype, float *Z,
                          unsigned *range_flag, hipStream_t s)
{
    long long total = (n + m) * d;
    int grid = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(convert_kernel, dim3(grid), dim3(256), 0, s, X, n * d, Y, total, dtype, Z, range_flag);
    return hipGetLastError();
}

// Several small regions cleared by one launch (a clear of its own per region is a launch of its own,
// and a launch costs more than these clears).  Sizes in 4-byte words.
__global__ void clear_regions_kernel(ClearRegions R)
{
    for (int q = 0; q < R.count; ++q)
        for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < R.words[q];
             i += (long long)gridDim.x * blockDim.x)
            R.ptr[q][i] = 0u;
}

hipError_t launch_clear_regions(const ClearRegions &R, hipStream_t s)
{
    long long most = 0;
    for (int q = 0; q < R.count; ++q) most = R.words[q] > most ? R.words[q] : most;
    if (most <= 0) return hipSuccess;
    const long long blocks = (most + 255) / 256;
    hipLaunchKernelGGL(clear_regions_kernel, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0, s, R);
    return hipGetLastError();
}

__global__ void gather_rows_kernel(const float *Z, int d, const long long *idx, int k, float *out)
{
    int c = blockIdx.x;
    const long long src = idx[c];   // negative: no such row, the slot is filled with zeros
    for (int j = threadIdx.x; j < d; j += blockDim.x) out[(long long)c * d + j] = src < 0 ? 0.f : Z[src * d + j];
}

hipError_t launch_gather_rows(const float *Z, int d, const long long *idx, int k, float *out, hipStream_t s)
{
    hipLaunchKernelGGL(gather_rows_kernel, dim3(k), dim3(128), 0, s, Z, d, idx, k, out);
    return hipGetLastError();
}

// ---------------------------------------------------- k-means++ seeding --
//
// Landmarks "sampled via k-means++" (Sec. 4): the first point uniformly, each
// further one with probability proportional to its squared distance w_i to
// the nearest point chosen so far.  The draw is integer work so that it has
// one answer: w_i by the fp64 bucket rule, weight q_i = floor(w_i 2^(38-e))
// where 4 max|z|^2 = f 2^e (1/2 <= f < 1) bounds every distance, pick = lowest
// i with q_0 + .. + q_i > r_t mod (sum q), r_t the t-th splitmix64 output.  A
// chosen point carries w = -1 (weight 0).  If the weights sum to 0 the lowest
// index not chosen yet is taken.
//
// One step = one sweep over the points (distance to the newest landmark,
// minimum, weights, per-workgroup totals) and one single-workgroup pick.

constexpr int PP_POINTS = 64;   // points per workgroup of the sweep: one wavefront, one point per lane
constexpr int PP_MAX_GROUPS = 16384;

__device__ inline int kmeanspp_shift(unsigned long long m2_bits)
{
    // 4 * m2 = f * 2^e with 1/2 <= f < 1: e = biased exponent - 1020 (m2 is 0 or a normal double)
    return 38 - ((int)((m2_bits >> 52) & 0x7FF) - 1020);
}

__device__ inline unsigned long long kmeanspp_weight(double w, int shift)
{
    return w > 0.0 ? (unsigned long long)floor(ldexp(w, shift)) : 0ull;
}

// MODE 0: largest squared norm of a point -> state[0] (bits of a non-negative double order like integers)
// MODE 1: w = D(z, c);  MODE 2: w = min(w, D(z, c));  both: partial[workgroup] = sum of the weights
// The wavefront reads its 64 rows in tiles of 32 dimensions (two rows per load instruction, all 32
// loads of a tile in flight together, the next tile's while this one is summed), turns the tile
// through LDS, and every lane adds up its own point's terms in dimension order.
template <int MODE>
__global__ __launch_bounds__(64) void kmeanspp_sweep_kernel(const float *Z, long long N, int d, const float *c,
                                                            const int *picks, int t, double *w,
                                                            unsigned long long *state, unsigned long long *partial)
{
    __shared__ float tile[64][33];
    __shared__ float csh[32];
    const int lane = threadIdx.x;
    const int half = lane >> 5, col = lane & 31;
    const long long i0 = (long long)blockIdx.x * PP_POINTS;
    // rows past the end repeat the last row (their lanes are dropped at the end)
    long long rowoff[32];
#pragma unroll
    for (int q = 0; q < 32; ++q) {
        const long long row = i0 + 2 * q + half;
        rowoff[q] = (row < N ? row : N - 1) * d;
    }
    float v[32];
    float cv = 0.f;
    auto fetch = [&](int k0) {
        const int kc = k0 + col < d ? k0 + col : d - 1;   // columns past the end repeat the last one (not summed)
#pragma unroll
        for (int q = 0; q < 32; ++q) v[q] = Z[rowoff[q] + kc];
        if (MODE != 0) cv = c[k0 + (lane & 31) < d ? k0 + (lane & 31) : d - 1];
    };
    fetch(0);
    double s = 0.0;
    for (int k0 = 0; k0 < d; k0 += 32) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 32; ++q) tile[2 * q + half][col] = v[q];
        if (lane < 32) csh[lane] = cv;
        __syncthreads();
        if (k0 + 32 < d) fetch(k0 + 32);
        const int kend = d - k0 < 32 ? d - k0 : 32;
        if (kend == 32) {
#pragma unroll
            for (int kk = 0; kk < 32; ++kk) {
                const double df = (double)tile[lane][kk] - (double)csh[kk];
                const double sq = df * df;
                s = s + sq;
            }
        } else {
            for (int kk = 0; kk < kend; ++kk) {
                const double df = (double)tile[lane][kk] - (double)csh[kk];
                const double sq = df * df;
                s = s + sq;
            }
        }
    }
    const long long i = i0 + lane;
    unsigned long long r = 0;
    if (MODE == 0) {
        r = i < N ? (unsigned long long)__double_as_longlong(s) : 0ull;
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long other = __shfl_xor(r, o, 64);
            r = other > r ? other : r;
        }
        if (lane == 0) atomicMax(&state[0], r);
    } else {
        if (i < N) {
            double wn = s;
            if (MODE == 2) wn = fmin(w[i], s);
            if (i == (long long)picks[t]) wn = -1.0;
            w[i] = wn;
            r = kmeanspp_weight(wn, kmeanspp_shift(state[0]));
        }
        for (int o = 32; o > 0; o >>= 1) r += __shfl_xor(r, o, 64);
        if (lane == 0) partial[blockIdx.x] = r;
    }
}

// One workgroup of 1024 threads: the t-th pick from the per-workgroup totals of the sweep, its
// index into picks[t], its row into cent[t].  nb <= 16384 totals, sixteen per thread.
__global__ __launch_bounds__(1024) void kmeanspp_pick_kernel(const float *Z, long long N, int d, const double *w,
                                                             const unsigned long long *state,
                                                             const unsigned long long *partial, int nb,
                                                             const unsigned long long *rnd, int t, int *picks,
                                                             float *cent)
{
    __shared__ unsigned long long scan[1024];
    __shared__ long long found;     // index of the pick
    __shared__ long long blk;       // workgroup of the sweep that holds it
    __shared__ unsigned long long rem_sh;
    const int tid = threadIdx.x;
    if (tid == 0) {
        found = -1;
        blk = -1;
    }
    if (t == 0) {
        __syncthreads();
        if (tid == 0) found = (long long)(rnd[0] % (unsigned long long)N);
        __syncthreads();
    } else {
        unsigned long long v[16], local = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int b = tid * 16 + q;
            v[q] = b < nb ? partial[b] : 0ull;
            local += v[q];
        }
        scan[tid] = local;
        __syncthreads();
        for (int o = 1; o < 1024; o <<= 1) {   // inclusive scan
            const unsigned long long add = tid >= o ? scan[tid - o] : 0ull;
            __syncthreads();
            scan[tid] += add;
            __syncthreads();
        }
        const unsigned long long total = scan[1023];
        if (total == 0) {
            // every point left coincides with a chosen one: lowest index not chosen yet
            long long best = N;
            for (long long i = tid; i < N; i += 1024)
                if (w[i] >= 0.0 && i < best) best = i;
            __syncthreads();
            scan[tid] = (unsigned long long)best;
            __syncthreads();
            for (int o = 512; o > 0; o >>= 1) {
                if (tid < o && scan[tid + o] < scan[tid]) scan[tid] = scan[tid + o];
                __syncthreads();
            }
            if (tid == 0) found = (long long)scan[0];
            __syncthreads();
        } else {
            const unsigned long long target = rnd[t] % total;
            unsigned long long run = scan[tid] - local;   // total of the workgroups before this thread's sixteen
            if (local > 0 && run <= target && target < scan[tid]) {
                bool done = false;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    if (!done && target < run + v[q]) {
                        blk = tid * 16 + q;
                        rem_sh = target - run;
                        done = true;
                    }
                    run += v[q];
                }
            }
            __syncthreads();
            const long long base = blk * PP_POINTS;
            const unsigned long long rem = rem_sh;
            const int shift = kmeanspp_shift(state[0]);
            unsigned long long q = 0;
            if (tid < PP_POINTS && base + tid < N) q = kmeanspp_weight(w[base + tid], shift);
            __syncthreads();
            scan[tid] = q;
            __syncthreads();
            for (int o = 1; o < PP_POINTS; o <<= 1) {
                const unsigned long long add = (tid >= o && tid < PP_POINTS) ? scan[tid - o] : 0ull;
                __syncthreads();
                if (tid < PP_POINTS) scan[tid] += add;
                __syncthreads();
            }
            if (tid < PP_POINTS && q > 0 && scan[tid] - q <= rem && rem < scan[tid]) found = base + tid;
            __syncthreads();
        }
    }
    const long long pick = found;
    if (pick < 0 || pick >= N) return;   // cannot happen; leaves picks[t] untouched rather than reading out of range
    if (tid == 0) picks[t] = (int)pick;
    for (int j = tid; j < d; j += 1024) cent[(long long)t * d + j] = Z[pick * d + j];
}

// k points of Z by k-means++ seeding into cent (k x d); rnd: k splitmix64 outputs (device);
// w: N doubles, partial: ceil(N / 64) totals, picks: k ints, state: one 64-bit word.
hipError_t launch_kmeanspp(const float *Z, long long N, int d, int k, const unsigned long long *rnd, double *w,
                           unsigned long long *partial, int *picks, unsigned long long *state, float *cent,
                           hipStream_t s)
{
    const int nb = (int)((N + PP_POINTS - 1) / PP_POINTS);
    if (nb > PP_MAX_GROUPS || k > N) return hipErrorInvalidValue;
    hipError_t e = hipMemsetAsync(state, 0, sizeof(unsigned long long), s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kmeanspp_sweep_kernel<0>, dim3(nb), dim3(64), 0, s, Z, N, d, (const float *)nullptr,
                       (const int *)nullptr, 0, (double *)nullptr, state, (unsigned long long *)nullptr);
    for (int t = 0; t < k; ++t) {
        hipLaunchKernelGGL(kmeanspp_pick_kernel, dim3(1), dim3(1024), 0, s, Z, N, d, (const double *)w,
                           (const unsigned long long *)state, (const unsigned long long *)partial, nb, rnd, t, picks,
                           cent);
        if (t + 1 == k) break;
        if (t == 0)
            hipLaunchKernelGGL(kmeanspp_sweep_kernel<1>, dim3(nb), dim3(64), 0, s, Z, N, d,
                               (const float *)(cent + (long long)t * d), (const int *)picks, t, w, state, partial);
        else
            hipLaunchKernelGGL(kmeanspp_sweep_kernel<2>, dim3(nb), dim3(64), 0, s, Z, N, d,
                               (const float *)(cent + (long long)t * d), (const int *)picks, t, w, state, partial);
    }
    return hipGetLastError();
}

// ------------------------------------------------- exact-rule assignment --
//
// A block takes 64 points and walks over all candidates (centroids, or
// projection columns) in tiles of 64; each thread keeps a 4 x 4 patch of fp64
// accumulators.  Every accumulator adds its terms in ascending dimension
// order, multiply and add separately, which is the rule the bucket of a point
// is defined by.  KIND 0: squared distance, arg-min (k-means).  KIND 1: dot
// product with the columns of a d x h matrix, arg-max over [g, -g]
// (cross-polytope hashing).

constexpr int TILE = 64;
constexpr int KCH = 32;
constexpr int LDT = TILE + 4;

template <int KIND>
__global__ __launch_bounds__(256) void assign_kernel(const float *__restrict__ Z, long long N, int d,
                                                     const float *__restrict__ C, int k, int32_t *__restrict__ out,
                                                     const int *__restrict__ list, const int *__restrict__ list_count)
{
    __shared__ float Ps[KCH][LDT];
    __shared__ float Cs[KCH][LDT];
    __shared__ double red_v[TILE][17];
    __shared__ int red_i[TILE][17];
    __shared__ long long pidx[TILE];  // the 64 points of this workgroup (-1: none)

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const long long p0 = (long long)blockIdx.x * TILE;
    // with a list, only the listed points are decided (those the MFMA filter could not)
    const long long cnt = list ? (long long)*list_count : N;
    if (p0 >= cnt) return;
    if (tid < TILE) pidx[tid] = p0 + tid < cnt ? (list ? (long long)list[p0 + tid] : p0 + tid) : -1;
    __syncthreads();

    double bestv[4];
    int besti[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bestv[i] = 0.0;
        besti[i] = -1;
    }

    for (int c0 = 0; c0 < k; c0 += TILE) {
        double acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

        for (int k0 = 0; k0 < d; k0 += KCH) {
            __syncthreads();
            // stage 64 points x 32 dims and 64 candidates x 32 dims, zero padded
            {
                const int kk = tid & 31;
                const int r0 = tid >> 5;
#pragma unroll
                for (int pass = 0; pass < 8; ++pass) {
                    int r = r0 + pass * 8;
                    long long p = pidx[r];
                    float v = 0.f;
                    if (p >= 0 && k0 + kk < d) v = Z[p * d + k0 + kk];
                    Ps[kk][r] = v;
                }
                if (KIND == 0) {
#pragma unroll
                    for (int pass = 0; pass < 8; ++pass) {
                        int r = r0 + pass * 8;
                        int c = c0 + r;
                        float v = 0.f;
                        if (c < k && k0 + kk < d) v = C[(long long)c * d + k0 + kk];
                        Cs[kk][r] = v;
                    }
                } else {
                    const int cc = tid & 63;
                    const int kr = tid >> 6;
#pragma unroll
                    for (int pass = 0; pass < 8; ++pass) {
                        int kq = kr + pass * 4;
                        float v = 0.f;
                        if (c0 + cc < k && k0 + kq < d) v = C[(long long)(k0 + kq) * k + c0 + cc];
                        Cs[kq][cc] = v;
                    }
                }
            }
            __syncthreads();
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
                        if (KIND == 0) {
                            double t = pv[i] - cv[j];
                            double t2 = t * t;
                            acc[i][j] = acc[i][j] + t2;
                        } else {
                            double t = pv[i] * cv[j];
                            acc[i][j] = acc[i][j] + t;
                        }
                    }
            }
        }
        // fold this tile's candidates into the running best (lowest index wins ties)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = c0 + tx * 4 + j;
            if (c >= k) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (KIND == 0) {
                    double D = acc[i][j];
                    if (besti[i] < 0 || D < bestv[i] || (D == bestv[i] && c < besti[i])) {
                        bestv[i] = D;
                        besti[i] = c;
                    }
                } else {
                    double g = acc[i][j];
                    // candidate c has value g, candidate k + c has value -g
                    if (besti[i] < 0 || g > bestv[i] || (g == bestv[i] && c < besti[i])) {
                        bestv[i] = g;
                        besti[i] = c;
                    }
                    double ng = -g;
                    if (ng > bestv[i] || (ng == bestv[i] && k + c < besti[i])) {
                        bestv[i] = ng;
                        besti[i] = k + c;
                    }
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        red_v[ty * 4 + i][tx] = bestv[i];
        red_i[ty * 4 + i][tx] = besti[i];
    }
    __syncthreads();
    if (tid < TILE) {
        double bv = 0.0;
        int bi = -1;
        for (int t = 0; t < 16; ++t) {
            double v = red_v[tid][t];
            int ix = red_i[tid][t];
            if (ix < 0) continue;
            bool better;
            if (KIND == 0)
                better = bi < 0 || v < bv || (v == bv && ix < bi);
            else
                better = bi < 0 || v > bv || (v == bv && ix < bi);
            if (better) {
                bv = v;
                bi = ix;
            }
        }
        if (pidx[tid] >= 0) out[pidx[tid]] = bi;
    }
}

// Exact rule for a (short) list of points: one workgroup per listed point, one
// thread per centroid (strided), each adding the dimensions left to right.
__global__ __launch_bounds__(256) void assign_list_kernel(const float *__restrict__ Z, int d,
                                                          const float *__restrict__ C, int k,
                                                          int32_t *__restrict__ out, const int *__restrict__ list,
                                                          const int *__restrict__ list_count)
{
    extern __shared__ float zrow[];  // d floats
    __shared__ double bv_sh[256];
    __shared__ int bi_sh[256];
    const int cnt = *list_count;
    for (int it = blockIdx.x; it < cnt; it += gridDim.x) {
        const long long p = list[it];
        __syncthreads();
        for (int j = threadIdx.x; j < d; j += 256) zrow[j] = Z[p * d + j];
        __syncthreads();
        double bv = 0.0;
        int bi = -1;
        for (int c = threadIdx.x; c < k; c += 256) {
            const float *cr = C + (long long)c * d;
            double s = 0.0;
            int j = 0;
            for (; j + 32 <= d; j += 32) {  // the order of the additions is the rule; 32 loads are requested at once
                float cv[32];
#pragma unroll
                for (int e = 0; e < 32; ++e) cv[e] = cr[j + e];
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    double t = (double)zrow[j + e] - (double)cv[e];
                    double t2 = t * t;
                    s = s + t2;
                }
            }
            for (; j < d; ++j) {
                double t = (double)zrow[j] - (double)cr[j];
                double t2 = t * t;
                s = s + t2;
            }
            if (bi < 0 || s < bv) {  // ascending c: strict < keeps the lowest index
                bv = s;
                bi = c;
            }
        }
        bv_sh[threadIdx.x] = bv;
        bi_sh[threadIdx.x] = bi;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (threadIdx.x < o) {
                const double v2 = bv_sh[threadIdx.x + o];
                const int i2 = bi_sh[threadIdx.x + o];
                const double v1 = bv_sh[threadIdx.x];
                const int i1 = bi_sh[threadIdx.x];
                if (i2 >= 0 && (i1 < 0 || v2 < v1 || (v2 == v1 && i2 < i1))) {
                    bv_sh[threadIdx.x] = v2;
                    bi_sh[threadIdx.x] = i2;
                }
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) out[p] = bi_sh[0];
    }
}

// Exact rule on two candidate centroids: a thread adds the dimensions of one
// (point, centroid) pair left to right; neighbouring threads hold the two
// candidates of a point and the smaller sum wins (the lower index if equal).
__global__ __launch_bounds__(256) void assign_pairs_kernel(const float *__restrict__ Z, int d,
                                                           const float *__restrict__ C, int32_t *__restrict__ out,
                                                           const int *__restrict__ pairs,
                                                           const int *__restrict__ pair_count)
{
    const long long cnt = *pair_count;
    const long long stride = (long long)gridDim.x * blockDim.x;
    // every trip is taken by whole pairs of lanes, so the exchange below always has its partner
    for (long long t0 = (long long)blockIdx.x * blockDim.x; t0 < 2 * cnt; t0 += stride) {
        const long long t = t0 + threadIdx.x;
        const bool live = t < 2 * cnt;
        const long long slot = live ? t >> 1 : 0;
        const long long p = pairs[3 * slot];
        const int c = pairs[3 * slot + 1 + (int)(t & 1)];
        const float *zr = Z + p * d;
        const float *cr = C + (long long)c * d;
        double s = 0.0;
        int j = 0;
        for (; j + 32 <= d; j += 32) {  // the order of the additions is the rule; 64 loads are requested at once
            float zv[32], cv[32];
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                zv[e] = zr[j + e];
                cv[e] = cr[j + e];
            }
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                double u = (double)zv[e] - (double)cv[e];
                double u2 = u * u;
                s = s + u2;
            }
        }
        for (; j < d; ++j) {
            double u = (double)zr[j] - (double)cr[j];
            double u2 = u * u;
            s = s + u2;
        }
        const double so = __shfl_xor(s, 1, 64);
        const int co = __shfl_xor(c, 1, 64);
        if (live && (t & 1) == 0) out[p] = (so < s || (so == s && co < c)) ? co : c;
    }
}

hipError_t launch_assign_pairs(const float *Z, int d, const float *cent, int32_t *out, const int *pairs,
                               const int *pair_count, hipStream_t s)
{
    hipLaunchKernelGGL(assign_pairs_kernel, dim3(512), dim3(256), 0, s, Z, d, cent, out, pairs, pair_count);
    return hipGetLastError();
}

hipError_t launch_assign_kmeans(const float *Z, long long N, int d, const float *cent, int k, int32_t *out,
                                const int *list, const int *list_count, hipStream_t s)
{
    if (list) {
        hipLaunchKernelGGL(assign_list_kernel, dim3(2048), dim3(256), sizeof(float) * (size_t)d, s, Z, d, cent, k, out,
                           list, list_count);
        return hipGetLastError();
    }
    int grid = (int)((N + TILE - 1) / TILE);
    hipLaunchKernelGGL(assign_kernel<0>, dim3(grid), dim3(256), 0, s, Z, N, d, cent, k, out, list, list_count);
    return hipGetLastError();
}

hipError_t launch_assign_crosspolytope(const float *Z, long long N, int d, const float *Rm, int b, int32_t *out,
                                       hipStream_t s)
{
    int grid = (int)((N + TILE - 1) / TILE);
    hipLaunchKernelGGL(assign_kernel<1>, dim3(grid), dim3(256), 0, s, Z, N, d, Rm, b / 2, out, (const int *)nullptr,
                       (const int *)nullptr);
    return hipGetLastError();
}

// ------------------------------------------- hierarchical k-means, AND hash --
//
// Lower levels of hierarchical k-means hashing (App. "Choosing LSH neighbors and
// Nystrom landmarks"): inside every cluster of the level above, a k-means of its
// own.  The points arrive grouped by parent (`order`), cut into chunks of at most
// 64 members of ONE parent: chunk = {parent, first position in order, members}.
// A wavefront takes a chunk, one member per lane, and adds up the squared
// distances to all children of that parent at once (children's centroids in
// LDS, read as broadcasts) -- the bucket rule: fp64, dimensions in order,
// multiply and add separately, lowest index among the minima.  bucket =
// parent * branch + child.
constexpr int HK_MAX_BRANCH = 32;

// Children's centroids as fp64, laid out [parent][dimension][child] with the children padded to
// `brp` (4, 8, 16 or 32): the sweep below reads one dimension of all children of a parent as one
// run of wave-uniform (scalar) loads.  A child that does not exist gets +infinity, which no
// minimum picks.
__global__ void children_layout_kernel(const float *cent, int d, int branch, int brp, const int *nchild,
                                       long long total, double *out)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int j = (int)(e % brp);
    const long long pk = e / brp;
    const int k = (int)(pk % d);
    const long long parent = pk / d;
    out[e] = j < nchild[parent] ? (double)cent[(parent * branch + j) * d + k] : INFINITY;
}

template <int BRP>
__global__ __launch_bounds__(64) void assign_children_kernel(const float *Z, int d, const double *centT, int branch,
                                                             const int *order, const int *chunks, int32_t *out)
{
    __shared__ float tile[64][33];
    __shared__ int mem_sh[64];
    const int lane = threadIdx.x;
    const int half = lane >> 5, col = lane & 31;
    const int parent = __builtin_amdgcn_readfirstlane(chunks[3 * blockIdx.x]);
    const int first = chunks[3 * blockIdx.x + 1], cnt = chunks[3 * blockIdx.x + 2];
    const int me = order[first + (lane < cnt ? lane : cnt - 1)];   // lanes past the end repeat the last member
    mem_sh[lane] = me;
    __syncthreads();
    long long rowoff[32];
#pragma unroll
    for (int q = 0; q < 32; ++q) rowoff[q] = (long long)mem_sh[2 * q + half] * d;
    // wave-uniform address in the constant address space: read through the scalar unit
    typedef const __attribute__((address_space(4))) double *cptr;
    cptr ct = (cptr)(unsigned long long)(centT + (long long)parent * d * BRP);
    double acc[BRP];
#pragma unroll
    for (int j = 0; j < BRP; ++j) acc[j] = 0.0;
    float v[32];
    auto fetch = [&](int k0) {
        const int kc = k0 + col < d ? k0 + col : d - 1;
#pragma unroll
        for (int q = 0; q < 32; ++q) v[q] = Z[rowoff[q] + kc];
    };
    fetch(0);
    for (int k0 = 0; k0 < d; k0 += 32) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 32; ++q) tile[2 * q + half][col] = v[q];
        __syncthreads();
        if (k0 + 32 < d) fetch(k0 + 32);
        const int kend = d - k0 < 32 ? d - k0 : 32;
        for (int kk = 0; kk < kend; ++kk) {
            const double zv = (double)tile[lane][kk];
            cptr crow = ct + (long long)(k0 + kk) * BRP;
#pragma unroll
            for (int j = 0; j < BRP; ++j) {
                const double df = zv - crow[j];
                const double sq = df * df;
                acc[j] = acc[j] + sq;
            }
        }
    }
    int best = 0;
    double bestD = acc[0];
#pragma unroll
    for (int j = 1; j < BRP; ++j) {
        if (acc[j] < bestD) {
            bestD = acc[j];
            best = j;
        }
    }
    if (lane < cnt) out[me] = parent * branch + best;
}

// centT: scratch of parents * d * 32 doubles at most
hipError_t launch_assign_children(const float *Z, int d, const float *cent, long long parents, int branch,
                                  const int *nchild, const int *order, const int *chunks, int nchunks, double *centT,
                                  int32_t *out, hipStream_t s)
{
    if (branch < 1 || branch > HK_MAX_BRANCH) return hipErrorInvalidValue;
    if (nchunks < 1) return hipSuccess;
    const int brp = branch <= 4 ? 4 : branch <= 8 ? 8 : branch <= 16 ? 16 : 32;
    const long long total = parents * d * brp;
    hipLaunchKernelGGL(children_layout_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, cent, d, branch,
                       brp, nchild, total, centT);
#define LCN_CHILDREN(B)                                                                                          \
    hipLaunchKernelGGL(assign_children_kernel<B>, dim3(nchunks), dim3(64), 0, s, Z, d, (const double *)centT, branch, \
                       order, chunks, out)
    if (brp == 4) LCN_CHILDREN(4);
    else if (brp == 8) LCN_CHILDREN(8);
    else if (brp == 16) LCN_CHILDREN(16);
    else LCN_CHILDREN(32);
#undef LCN_CHILDREN
    return hipGetLastError();
}

// AND construction: the bucket of a band of hashes is the tuple of their values,
// numbered acc * b + h, one hash at a time.
__global__ void combine_hash_kernel(int32_t *acc, const int32_t *h, int b, int first, long long N)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) acc[i] = (first ? 0 : acc[i] * b) + h[i];
}

hipError_t launch_combine_hash(int32_t *acc, const int32_t *h, int b, int first, long long N, hipStream_t s)
{
    hipLaunchKernelGGL(combine_hash_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, acc, h, b, first, N);
    return hipGetLastError();
}

// -------------------------------------------------------- k-means update --
//
// Member sums in 2^-32 fixed point: integer addition is associative, so the
// sums are the same in any order (and the counting sort below may place the
// members of a cluster in any order).  Per Lloyd update:
//   count   -- members per cluster (histogram in LDS, one device atomic per
//              workgroup and cluster present);
//   scatter -- point indices grouped by cluster (each workgroup redoes the
//              small scan of the counts, reserves its ranges with one atomic per
//              cluster present and ranks its points in LDS);
//   sum     -- one workgroup per (cluster, slice of 64 dimensions): its 16
//              wavefronts share out the members, every member is one coalesced
//              256-byte read, and the mean is written straight to the centroid.
// The point matrix is read once, by rows; nothing but the centroids is written.
// The count and cursor arrays exist twice and alternate between updates: the sum
// kernel clears the pair the next update will use.

constexpr int KM_POINTS = 2048;  // points per workgroup of count and scatter

__global__ __launch_bounds__(256) void kmeans_count_kernel(const int32_t *__restrict__ assign, long long N, int k,
                                                           int *__restrict__ counts)
{
    extern __shared__ int hist[];  // k
    for (int t = threadIdx.x; t < k; t += 256) hist[t] = 0;
    __syncthreads();
    const long long p0 = (long long)blockIdx.x * KM_POINTS;
    for (int q = threadIdx.x; q < KM_POINTS; q += 256)
        if (p0 + q < N) atomicAdd(&hist[assign[p0 + q]], 1);
    __syncthreads();
    for (int t = threadIdx.x; t < k; t += 256)
        if (hist[t]) atomicAdd(&counts[t], hist[t]);
}

__global__ __launch_bounds__(256) void kmeans_scatter_kernel(const int32_t *__restrict__ assign, long long N, int k,
                                                             const int *__restrict__ counts, int *__restrict__ cursor,
                                                             int *__restrict__ order, int *__restrict__ offs)
{
    extern __shared__ int sh[];  // start[k] (where this workgroup's members of a cluster go), hist[k]
    __shared__ int part[256];
    int *start = sh, *hist = sh + k;
    const int tid = threadIdx.x;
    // exclusive scan of the counts: a contiguous run per thread, then the 256 run totals
    const int seg = (k + 255) / 256;
    const int lo = tid * seg, hi = lo + seg < k ? lo + seg : k;
    int run = 0;
    for (int t = lo; t < hi; ++t) run += counts[t];
    part[tid] = run;
    for (int t = tid; t < k; t += 256) hist[t] = 0;
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int t = 0; t < 256; ++t) {
            const int v = part[t];
            part[t] = acc;
            acc += v;
        }
    }
    __syncthreads();
    run = part[tid];
    for (int t = lo; t < hi; ++t) {
        start[t] = run;
        if (blockIdx.x == 0) offs[t] = run;  // where each cluster's members begin, for the sum kernel
        run += counts[t];
    }
    __syncthreads();
    const long long p0 = (long long)blockIdx.x * KM_POINTS;
    int rank[KM_POINTS / 256], cl[KM_POINTS / 256];
#pragma unroll
    for (int u = 0; u < KM_POINTS / 256; ++u) {
        const long long p = p0 + tid + 256 * u;
        cl[u] = p < N ? assign[p] : -1;
        rank[u] = cl[u] >= 0 ? atomicAdd(&hist[cl[u]], 1) : 0;
    }
    __syncthreads();
    for (int t = tid; t < k; t += 256)
        if (hist[t]) start[t] += atomicAdd(&cursor[t], hist[t]);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < KM_POINTS / 256; ++u)
        if (cl[u] >= 0) order[start[cl[u]] + rank[u]] = (int)(p0 + tid + 256 * u);
}

// grid: (k, ceil(d / SW)); 1024 threads.  SW = 64: a wave-wide load is one member's 64 dimensions.
// SW = 16 (few clusters: more, narrower workgroups): it is 16 dimensions of four members.
template <int SW, int WPB>
__global__ __launch_bounds__(64 * WPB) void kmeans_sum_kernel(const float *__restrict__ Z, int d, int k,
                                                          const int *__restrict__ counts, const int *__restrict__ offs,
                                                          const int *__restrict__ order, float *__restrict__ cent,
                                                          int *__restrict__ counts_next, int *__restrict__ cursor_next,
                                                          unsigned *reset_a, int *reset_b)
{
    constexpr int RPL = 64 / SW;   // members per wave-wide load
    __shared__ long long red[WPB][SW];
    const int c = blockIdx.x, slice = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int sub = lane / SW, jl = lane % SW;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (slice == 0 && threadIdx.x == 0) {  // scratch of the next assignment and update steps starts from zero
        counts_next[c] = 0;
        cursor_next[c] = 0;
        if (c == 0) {
            if (reset_a) *reset_a = 0u;
            if (reset_b) {
                reset_b[0] = 0;
                reset_b[1] = 0;
            }
        }
    }
    const int cnt = counts[c];
    const int *__restrict__ mem = order + offs[c];
    const int j = SW * slice + jl;
    const bool jin = j < d;
    long long sum = 0;
    // the 16 wavefronts share out the members in contiguous runs; a wave reads up to 64 member
    // indices at once (one per lane) and then requests 16 loads before the first is added
    const int per = (cnt + WPB - 1) / WPB;
    const int beg = wave * per;
    const int end = beg + per < cnt ? beg + per : cnt;
    for (int base = beg; base < end; base += 64) {
        const int nloc = end - base < 64 ? end - base : 64;
        const int myidx = lane < nloc ? mem[base + lane] : 0;
        for (int u0 = 0; u0 < nloc; u0 += 16 * RPL) {
            float z[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int uu = u0 + u * RPL + sub;
                long long row;
                if (RPL == 1)
                    row = __builtin_amdgcn_readlane(myidx, uu < 64 ? uu : 63);
                else
                    row = __shfl(myidx, uu < 64 ? uu : 63, 64);
                // an unconditional load (a slot beyond the run reads row 0, a lane beyond the row's end
                // its last entry) keeps all sixteen in flight; what does not count is zeroed afterwards
                const float v = Z[row * d + (jin ? j : d - 1)];
                z[u] = (uu < nloc && jin) ? v : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) sum += __double2ll_rn((double)z[u] * 4294967296.0);
        }
    }
    for (int o = SW; o < 64; o <<= 1) sum += __shfl_xor(sum, o, 64);   // the members a load held side by side
    if (lane < SW) red[wave][lane] = sum;
    __syncthreads();
    if (wave == 0 && lane < SW && jin && cnt > 0) {  // an empty cluster keeps its centroid
        long long tot = 0;
#pragma unroll
        for (int w = 0; w < WPB; ++w) tot += red[w][lane];
        const double mean = ((double)tot * (1.0 / 4294967296.0)) / (double)cnt;
        cent[(long long)c * d + j] = (float)mean;
    }
}

// Rows of up to 512 dimensions: the sums are taken in two steps that do not depend on how the members
// are spread over the clusters.  The member list (grouped by cluster) is cut into chunks of M
// consecutive entries, one wavefront per chunk; the wavefront reads whole rows (lane j holds dimensions
// j, 64 + j, ...: every line of a row is fetched once, eight rows requested before the first is added)
// and, whenever the cluster changes and at its end, writes the sums so far as a partial: chunk g's
// part of cluster c goes to slot g + c, which no other pair shares (chunks and clusters both advance
// along the list).  One workgroup per cluster then adds the partials of the chunks its members lie in
// and writes the mean.  No atomics, every launch as long as the others whatever the cluster sizes.
// The fixed-point value of an entry: z 2^32 + 1.5 2^52 rounds to an integer (to nearest even, as rint
// does) whose low mantissa bits are that integer in two's complement, so the bit patterns are added
// as they are and the constants' share is taken off per member (all modulo 2^64).
int kmeans_sum_chunk(long long N) { return N <= 65536 ? 16 : N <= 131072 ? 32 : N <= 262144 ? 64 : 128; }

size_t kmeans_partial_elems(long long N, int kmax, int d)
{
    if (d > 512) return 1;   // wider rows take the sliced kernel, which needs none
    const int M = kmeans_sum_chunk(N);
    return (size_t)((N + M - 1) / M + kmax) * (size_t)d;
}

constexpr unsigned long long FIX_MAGIC_BITS = 0x4338000000000000ull;   // 1.5 * 2^52

template <int NS>
__global__ __launch_bounds__(256) void kmeans_partial_kernel(const float *__restrict__ Z, long long N, int d, int M,
                                                             const int32_t *__restrict__ assign,
                                                             const int *__restrict__ order,
                                                             unsigned long long *__restrict__ part)
{
    const int lane = threadIdx.x & 63;
    const long long g = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long first = g * M;
    if (first >= N) return;
    const int mine = N - first < M ? (int)(N - first) : M;
    unsigned long long sum[NS];
#pragma unroll
    for (int q = 0; q < NS; ++q) sum[q] = 0ull;
    int cur = -1, held = 0;
    auto flush = [&]() {
        unsigned long long *dst = part + (size_t)(g + cur) * (size_t)d;
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const int j = 64 * q + lane;
            if (j < d) dst[j] = sum[q] - (unsigned long long)held * FIX_MAGIC_BITS;
            sum[q] = 0ull;
        }
        held = 0;
    };
    // Every load below is unconditional: a lane beyond the row's end re-reads the row's last entry and
    // a slot beyond the chunk's end the chunk's last member (what they add is never stored), so the
    // forty loads of eight rows are in flight together.
    int jc[NS];
#pragma unroll
    for (int q = 0; q < NS; ++q) jc[q] = 64 * q + lane < d ? 64 * q + lane : d - 1;
    auto add_row = [&](const float (&zr)[NS]) {
        ++held;
#pragma unroll
        for (int q = 0; q < NS; ++q)
            sum[q] += (unsigned long long)__double_as_longlong(fma((double)zr[q], 4294967296.0, 6755399441055744.0));
    };
    for (int base = 0; base < mine; base += 64) {
        const int nloc = mine - base < 64 ? mine - base : 64;
        const int at = lane < nloc ? lane : nloc - 1;
        const int myidx = order[first + base + at];
        const int mycl = assign[myidx];
        for (int u0 = 0; u0 < nloc; u0 += 8) {
            float z[8][NS];
            int cl[8];
            bool same = u0 + 8 <= nloc;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int uu = u0 + u < nloc ? u0 + u : nloc - 1;
                const float *__restrict__ zrow = Z + (long long)__builtin_amdgcn_readlane(myidx, uu) * d;
                cl[u] = __builtin_amdgcn_readlane(mycl, uu);
                same = same && cl[u] == cur;
#pragma unroll
                for (int q = 0; q < NS; ++q) z[u][q] = zrow[jc[q]];
            }
            if (same) {   // the usual case: eight more members of the current cluster
#pragma unroll
                for (int u = 0; u < 8; ++u) add_row(z[u]);
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (u0 + u < nloc) {   // the same in every lane
                        if (cl[u] != cur) {
                            if (cur >= 0) flush();
                            cur = cl[u];
                        }
                        add_row(z[u]);
                    }
                }
            }
        }
    }
    if (cur >= 0) flush();
}

// One workgroup of eight wavefronts per cluster: the wavefronts share out the chunks the cluster's
// members lie in, four chunks' partials (whole rows, lane j dimensions j, 64 + j, ...) requested
// together; a chunk index beyond the last is clamped and its row not added.
template <int NS>
__global__ __launch_bounds__(512) void kmeans_mean_kernel(const unsigned long long *__restrict__ part, int d, int M,
                                                          const int *__restrict__ counts,
                                                          const int *__restrict__ offs, float *__restrict__ cent,
                                                          int *__restrict__ counts_next,
                                                          int *__restrict__ cursor_next, unsigned *reset_a,
                                                          int *reset_b)
{
    __shared__ unsigned long long red[8][NS][64];
    const int c = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (threadIdx.x == 0) {  // scratch of the next assignment and update steps starts from zero
        counts_next[c] = 0;
        cursor_next[c] = 0;
        if (c == 0) {
            if (reset_a) *reset_a = 0u;
            if (reset_b) {
                reset_b[0] = 0;
                reset_b[1] = 0;
            }
        }
    }
    const int cnt = counts[c];
    if (cnt == 0) return;  // an empty cluster keeps its centroid (the same in every thread)
    const int g0 = offs[c] / M, g1 = (offs[c] + cnt - 1) / M;
    int jc[NS];
    unsigned long long sum[NS];
#pragma unroll
    for (int q = 0; q < NS; ++q) {
        jc[q] = 64 * q + lane < d ? 64 * q + lane : d - 1;
        sum[q] = 0ull;
    }
    for (int g = g0 + wave; g <= g1; g += 32) {
        unsigned long long v[4][NS];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int gg = g + 8 * u <= g1 ? g + 8 * u : g1;
            const unsigned long long *__restrict__ row = part + (size_t)(gg + c) * (size_t)d;
#pragma unroll
            for (int q = 0; q < NS; ++q) v[u][q] = row[jc[q]];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (g + 8 * u <= g1) {   // the same in every lane
#pragma unroll
                for (int q = 0; q < NS; ++q) sum[q] += v[u][q];
            }
    }
#pragma unroll
    for (int q = 0; q < NS; ++q) red[wave][q][lane] = sum[q];
    __syncthreads();
    for (int t = threadIdx.x; t < 64 * NS; t += 512) {
        const int q = t >> 6, jl = t & 63, j = 64 * q + jl;
        if (j < d) {
            unsigned long long tot = 0ull;
#pragma unroll
            for (int w = 0; w < 8; ++w) tot += red[w][q][jl];
            const double mean = ((double)(long long)tot * (1.0 / 4294967296.0)) / (double)cnt;
            cent[(long long)c * d + j] = (float)mean;
        }
    }
}

// counts2 / cursor2: [2][k] each, zero on the first call of a k-means run; offs: [k]; `parity` alternates per call.
// part: kmeans_partial_elems(N, k, d) 64-bit words of scratch (rows of up to 512 dimensions).
// reset_a / reset_b (nullable) are cleared for the next assignment step.
hipError_t launch_kmeans_update(const float *Z, long long N, int d, const int32_t *assign, int k, int *counts2,
                                int *cursor2, int *order, int *offs, long long *part, int parity, float *cent,
                                unsigned *reset_a, int *reset_b, hipStream_t s)
{
    int *counts = counts2 + (size_t)(parity & 1) * k, *counts_next = counts2 + (size_t)((parity + 1) & 1) * k;
    int *cursor = cursor2 + (size_t)(parity & 1) * k, *cursor_next = cursor2 + (size_t)((parity + 1) & 1) * k;
    const unsigned blocks = (unsigned)((N + KM_POINTS - 1) / KM_POINTS);
    hipLaunchKernelGGL(kmeans_count_kernel, dim3(blocks), dim3(256), sizeof(int) * (size_t)k, s, assign, N, k, counts);
    hipLaunchKernelGGL(kmeans_scatter_kernel, dim3(blocks), dim3(256), 2 * sizeof(int) * (size_t)k, s, assign, N, k,
                       counts, cursor, order, offs);
    const int ns = (d + 63) / 64;
    if (ns <= 8) {
        const int M = kmeans_sum_chunk(N);
        const unsigned pblocks = (unsigned)(((N + M - 1) / M + 3) / 4);
#define LCN_SUM_PARTIAL(NS_)                                                                                       \
    hipLaunchKernelGGL((kmeans_partial_kernel<NS_>), dim3(pblocks), dim3(256), 0, s, Z, N, d, M, assign, order,       \
                       (unsigned long long *)part);                                                                    \
    hipLaunchKernelGGL((kmeans_mean_kernel<NS_>), dim3((unsigned)k), dim3(512), 0, s,                                  \
                       (const unsigned long long *)part, d, M, counts, offs, cent, counts_next, cursor_next, reset_a, \
                       reset_b)
        switch (ns) {
            case 1: LCN_SUM_PARTIAL(1); break;
            case 2: LCN_SUM_PARTIAL(2); break;
            case 3: LCN_SUM_PARTIAL(3); break;
            case 4: LCN_SUM_PARTIAL(4); break;
            case 5: LCN_SUM_PARTIAL(5); break;
            case 6: LCN_SUM_PARTIAL(6); break;
            case 7: LCN_SUM_PARTIAL(7); break;
            default: LCN_SUM_PARTIAL(8); break;
        }
#undef LCN_SUM_PARTIAL
    } else if ((long long)k * ((d + 63) / 64) >= 512)
        hipLaunchKernelGGL((kmeans_sum_kernel<64, 16>), dim3((unsigned)k, (unsigned)((d + 63) / 64)), dim3(1024), 0, s, Z,
                           d, k, counts, offs, order, cent, counts_next, cursor_next, reset_a, reset_b);
    else   // few clusters: narrower slices, four times the workgroups
        hipLaunchKernelGGL((kmeans_sum_kernel<16, 16>), dim3((unsigned)k, (unsigned)((d + 15) / 16)), dim3(1024), 0, s, Z,
                           d, k, counts, offs, order, cent, counts_next, cursor_next, reset_a, reset_b);
    return hipGetLastError();
}

// ------------------------------------------------------------ bucket sort --
//
// Stable counting sort of the point indices of each side (X, Y) by bucket,
// per hash round.  Chunks of CH consecutive indices are histogrammed, the
// histograms are prefixed over chunks and buckets, and each chunk is then
// scattered by one wavefront that ranks equal keys in index order.

constexpr int CH = 1024;

__global__ void scan_i64_kernel(long long *data, long long n);

// Exclusive scan of 1024 per-thread values across a workgroup of 1024 threads: returns the sum
// of the values of all lower threads; *total receives the sum of all.  wsum: 16 words of LDS.
__device__ inline long long block_exclusive_scan_1024(long long local, long long *wsum, long long *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    long long incl = local;
    for (int o = 1; o < 64; o <<= 1) {
        const long long up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    __syncthreads();   // wsum may still be read from the previous use
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    long long before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const long long v = wsum[w];
        if (w < wave) before += v;
        all += v;
    }
    *total = all;
    return before + incl - local;
}


int sort_chunks(long long n, long long m)
{
    long long mx = n > m ? n : m;
    return (int)((mx + CH - 1) / CH);
}

__device__ inline long long side_count(const SortBuffers &B, int side) { return side == 0 ? B.n : B.m; }

// grid: (chunks, R, 2)
__global__ __launch_bounds__(256) void sort_hist_kernel(SortBuffers B)
{
    extern __shared__ int hist[];
    const int chunk = blockIdx.x, r = blockIdx.y, side = blockIdx.z;
    const long long cnt = side_count(B, side);
    for (int t = threadIdx.x; t < B.b; t += blockDim.x) hist[t] = 0;
    __syncthreads();
    const long long base = (long long)chunk * CH;
    const int32_t *bk = B.bucket + (long long)r * (B.n + B.m) + (side ? B.n : 0);
    for (int t = threadIdx.x; t < CH; t += blockDim.x) {
        long long i = base + t;
        if (i < cnt) atomicAdd(&hist[bk[i]], 1);
    }
    __syncthreads();
    int *dst = B.hist + (((long long)side * B.R + r) * B.chunks + chunk) * B.b;
    for (int t = threadIdx.x; t < B.b; t += blockDim.x) dst[t] = hist[t];
}

// one thread per (side, round, bucket): exclusive prefix over chunks, bucket totals
__global__ void sort_chunk_prefix_kernel(SortBuffers B)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= 2 * B.R * B.b) return;
    int beta = t % B.b;
    int sr = t / B.b;  // side * R + r
    int *h = B.hist + (long long)sr * B.chunks * B.b + beta;
    int run = 0;
    for (int c = 0; c < B.chunks; ++c) {
        int v = h[(long long)c * B.b];
        h[(long long)c * B.b] = run;
        run += v;
    }
    B.totals[t] = run;
}

// single block: bucket offsets per (side, round), tile offsets over all blocks
__global__ __launch_bounds__(1024) void sort_offsets_kernel(SortBuffers B)
{
    __shared__ long long wsum[16];
    const int tid = threadIdx.x;
    // per (side, round): exclusive scan of totals over buckets; 2R <= 16 sequences
    for (int sr = 0; sr < 2 * B.R; ++sr) {
        const int *tot = B.totals + sr * B.b;
        int *off = B.off + sr * (B.b + 1);
        const int seg = (B.b + 1023) / 1024;
        const int lo = tid * seg, hi = lo + seg < B.b ? lo + seg : B.b;
        long long sum = 0;
        for (int i = lo; i < hi; ++i) sum += tot[i];
        long long all;
        long long run = block_exclusive_scan_1024(sum, wsum, &all);
        if (tid == 0) off[B.b] = (int)all;
        for (int i = lo; i < hi; ++i) {
            off[i] = (int)run;
            run += tot[i];
        }
    }
    // blocks in (round, bucket) order: value offsets (nx * ny) and 64 x 64 build tiles
    const int nb = B.R * B.b;
    const int seg = (nb + 1023) / 1024;
    const int lo = tid * seg, hi = lo + seg < nb ? lo + seg : nb;
    long long sum = 0, sum2 = 0;
    for (int i = lo; i < hi; ++i) {
        const long long nx = B.totals[i];
        const long long ny = B.totals[B.R * B.b + i];
        sum += nx * ny;
        sum2 += ((nx + 63) / 64) * ((ny + 63) / 64);
    }
    long long all, all2;
    (void)block_exclusive_scan_1024(sum, wsum, &all);
    long long run2 = block_exclusive_scan_1024(sum2, wsum, &all2);
    if (tid == 0) {
        B.tile_off[nb] = (int)all2;
        B.totals_out[0] = all;
        B.totals_out[1] = all2;
    }
    for (int i = lo; i < hi; ++i) {
        const long long nx = B.totals[i];
        const long long ny = B.totals[B.R * B.b + i];
        B.tile_off[i] = (int)run2;
        run2 += ((nx + 63) / 64) * ((ny + 63) / 64);
    }
}

// grid: (chunks, R, 2); one workgroup of 16 wavefronts per chunk of 1024 elements, one element
// per thread.  Stable: a wavefront ranks its 64 elements among equal keys by ballots, then the
// wavefronts take their places in the running bucket positions one after the other.
__global__ __launch_bounds__(1024) void sort_scatter_kernel(SortBuffers B)
{
    extern __shared__ int running[];
    const int chunk = blockIdx.x, r = blockIdx.y, side = blockIdx.z;
    const long long cnt = side_count(B, side);
    const long long base = (long long)chunk * CH;
    if (base >= cnt) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sr = side * B.R + r;
    const int *pre = B.hist + ((long long)sr * B.chunks + chunk) * B.b;
    const int *off = B.off + sr * (B.b + 1);
    for (int t = threadIdx.x; t < B.b; t += 1024) running[t] = off[t] + pre[t];
    const int32_t *bk = B.bucket + (long long)r * (B.n + B.m) + (side ? B.n : 0);
    int *perm = B.perm + (side ? (long long)B.R * B.n + (long long)r * B.m : (long long)r * B.n);
    int *pos = B.pos + (side ? (long long)B.R * B.n + (long long)r * B.m : (long long)r * B.n);
    const long long i = base + threadIdx.x;
    const bool valid = i < cnt;
    const int key = valid ? bk[i] : -1;
    int rank = 0, group = 0;
    // rank of this lane among the lanes of its wavefront with the same key (lower lanes first)
    bool pending = valid;
    while (true) {
        const unsigned long long todo = __ballot(pending);
        if (todo == 0ull) break;
        const int leader = __ffsll((long long)todo) - 1;
        const int k0 = __shfl(key, leader, 64);
        const unsigned long long same = __ballot(pending && key == k0);
        if (pending && key == k0) {
            rank = __popcll(same & ((1ull << lane) - 1ull));
            group = __popcll(same);
            pending = false;
        }
    }
    int dst = 0;
    for (int w = 0; w < CH / 64; ++w) {
        __syncthreads();   // running[] as the wavefronts before w left it (w = 0: as initialised)
        if (w == wave && valid) dst = running[key] + rank;
        __syncthreads();   // every lane of wavefront w has read before one lane per key moves the position on
        if (w == wave && valid && rank == group - 1) running[key] += group;
    }
    if (valid) {
        perm[dst] = (int)i;
        pos[i] = dst;
    }
}

// per (round, row): the slice of the other side's bucket-ordered vector the row
// multiplies; per row: the length of its record (written to rowbase, scanned after)
__global__ void seg_kernel(SortBuffers B)
{
    const int side = blockIdx.y;
    const long long cnt = side_count(B, side);
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cnt) return;
    const long long other = side ? B.n : B.m;
    long long total = 0;
    for (int r = 0; r < B.R; ++r) {
        const int32_t *bk = B.bucket + (long long)r * (B.n + B.m) + (side ? B.n : 0);
        const int beta = bk[i];
        const int *off_ot = B.off + ((1 - side) * B.R + r) * (B.b + 1);
        Seg sg;
        sg.len = off_ot[beta + 1] - off_ot[beta];
        sg.vstart = (int)((long long)r * other + off_ot[beta]);
        (side ? B.seg_y : B.seg_x)[(long long)r * cnt + i] = sg;
        total += sg.len;
    }
    (side ? B.rowbase_y : B.rowbase_x)[i] = total;
}

hipError_t launch_bucket_sort(const SortBuffers &B, hipStream_t s)
{
    dim3 grid(B.chunks, B.R, 2);
    size_t lds = sizeof(int) * (size_t)B.b;
    hipLaunchKernelGGL(sort_hist_kernel, grid, dim3(256), lds, s, B);
    int t = 2 * B.R * B.b;
    hipLaunchKernelGGL(sort_chunk_prefix_kernel, dim3((t + 127) / 128), dim3(128), 0, s, B);
    hipLaunchKernelGGL(sort_offsets_kernel, dim3(1), dim3(1024), 0, s, B);
    hipLaunchKernelGGL(sort_scatter_kernel, grid, dim3(1024), lds, s, B);
    long long mx = B.n > B.m ? B.n : B.m;
    hipLaunchKernelGGL(seg_kernel, dim3((unsigned)((mx + 255) / 256), 2), dim3(256), 0, s, B);
    hipLaunchKernelGGL(scan_i64_kernel, dim3(1), dim3(1024), 0, s, B.rowbase_x, B.n);
    hipLaunchKernelGGL(scan_i64_kernel, dim3(1), dim3(1024), 0, s, B.rowbase_y, B.m);
    return hipGetLastError();
}

// Packed per-row metadata read by the sweeps, one record per row:
//   [0:1] start of the row's record of sparse values (int64)
//   [2]   marginal (float)          [4:5] its natural log (double)
//   [6 + 2r], [7 + 2r]  round r: start in the other side's bucket-ordered vector, length
//   [6 + 2R + r]        round r: position of the row in its own side's bucket order
int meta_stride_for(int R) { return (6 + 3 * R + 3) / 4 * 4; }

__global__ void meta_kernel(SortBuffers B, const float *a, const float *b)
{
    const int side = blockIdx.y;
    const long long cnt = side_count(B, side);
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cnt) return;
    int *rec = (side ? B.meta_y : B.meta_x) + i * B.meta_stride;
    const long long base = B.R > 0 ? (side ? B.rowbase_y : B.rowbase_x)[i] : 0;
    const float marg = (side ? b : a)[i];
    const double lm = log((double)marg);
    rec[0] = (int)(unsigned)(base & 0xffffffffll);
    rec[1] = (int)(base >> 32);
    rec[2] = __float_as_int(marg);
    rec[3] = 0;
    rec[4] = __double2loint(lm);
    rec[5] = __double2hiint(lm);
    const int *pos = B.pos + (side ? (long long)B.R * B.n : 0);
    for (int r = 0; r < B.R; ++r) {
        const Seg sg = (side ? B.seg_y : B.seg_x)[(long long)r * cnt + i];
        rec[6 + 2 * r] = sg.vstart;
        rec[7 + 2 * r] = sg.len;
        rec[6 + 2 * B.R + r] = pos[(long long)r * cnt + i];
    }
}

hipError_t launch_build_meta(const SortBuffers &B, const float *a, const float *b, hipStream_t s)
{
    long long mx = B.n > B.m ? B.n : B.m;
    hipLaunchKernelGGL(meta_kernel, dim3((unsigned)((mx + 255) / 256), 2), dim3(256), 0, s, B, a, b);
    return hipGetLastError();
}

// ------------------------------------------------------------- CSR export --
//
// Row i of the pattern is the union over rounds of the Y members of the
// bucket x_i fell into; a pair that an earlier round already holds is
// skipped.  Members of a bucket are in ascending index order (stable sort),
// so the union is an R-way merge of ascending lists.

__device__ inline bool owned_by_earlier_round(const int32_t *bucket, long long N, long long n, int r, long long i,
                                              int j)
{
    for (int q = 0; q < r; ++q)
        if (bucket[(long long)q * N + i] == bucket[(long long)q * N + n + j]) return true;
    return false;
}

// One row by one thread: the R-way merge written out.  Used for rows too long for the
// wavefront version below.
template <bool FILL>
__device__ inline void csr_row_serial(const SortBuffers &B, long long i, const float *vals, const float *vals2,
                                      int log_values, long long *rowcount, const long long *rowptr, int32_t *colidx,
                                      float *val, float *val2)
{
    const long long N = B.n + B.m;
    int head[8], segstart[8];
    int run = 0;
    for (int r = 0; r < B.R; ++r) {
        head[r] = 0;
        segstart[r] = run;
        run += B.seg_x[(long long)r * B.n + i].len;
    }
    const long long base = B.rowbase_x[i];
    long long outp = FILL ? rowptr[i] : 0;
    long long cnt = 0;
    while (true) {
        int bestj = 0x7fffffff, bestr = -1;
        for (int r = 0; r < B.R; ++r) {
            const Seg sg = B.seg_x[(long long)r * B.n + i];
            const int *yperm = B.perm + (long long)B.R * B.n + (long long)r * B.m;
            const int seg0 = sg.vstart - (int)((long long)r * B.m);
            // skip entries an earlier round owns
            while (head[r] < sg.len &&
                   owned_by_earlier_round(B.bucket, N, B.n, r, i, yperm[seg0 + head[r]]))
                ++head[r];
            if (head[r] < sg.len) {
                int j = yperm[seg0 + head[r]];
                if (j < bestj) {
                    bestj = j;
                    bestr = r;
                }
            }
        }
        if (bestr < 0) break;
        if (FILL) {
            if (colidx) colidx[outp] = bestj;
            const long long at = base + segstart[bestr] + head[bestr];
            if (val) val[outp] = log_values ? expf(vals[at]) : vals[at];
            if (val2) val2[outp] = vals2[at];
            ++outp;
        }
        ++cnt;
        ++head[bestr];
    }
    if (!FILL) rowcount[i] = cnt;
}

// One wavefront per row.  The row's stored columns (all rounds, T of them) go into LDS, a dropped
// pair as INT_MAX; the place of a kept pair in the row is the number of kept columns below its own,
// counted by brute force over the T entries (T^2 / 64 LDS reads per lane, T ~ 100).  With one round
// the record already is the CSR row.  FILL = false only counts the kept pairs.
constexpr int CSR_ROW_MAX = 2048;  // entries of a row the wavefront version holds

template <bool FILL>
__global__ __launch_bounds__(256) void csr_kernel(SortBuffers B, const float *vals, const float *vals2,
                                                  int log_values, long long *rowcount, const long long *rowptr,
                                                  int32_t *colidx, float *val, float *val2)
{
    __shared__ int cols_sh[4][CSR_ROW_MAX];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long long i = (long long)blockIdx.x * 4 + w;
    const bool live = i < B.n;
    const long long N = B.n + B.m;
    int T = 0;
    if (live)
        for (int r = 0; r < B.R; ++r) T += B.seg_x[(long long)r * B.n + i].len;
    const long long base = live ? B.rowbase_x[i] : 0;
    const bool serial = live && B.R > 1 && T > CSR_ROW_MAX;
    const bool wide = live && B.R > 1 && !serial;
    int *cols = cols_sh[w];
    if (wide) {
        int off = 0;
        for (int r = 0; r < B.R; ++r) {
            const Seg sg = B.seg_x[(long long)r * B.n + i];
            const int *yperm = B.perm + (long long)B.R * B.n + (long long)r * B.m;
            const int seg0 = sg.vstart - (int)((long long)r * B.m);
            for (int e = lane; e < sg.len; e += 64) {
                const int j = yperm[seg0 + e];
                cols[off + e] = owned_by_earlier_round(B.bucket, N, B.n, r, i, j) ? 0x7fffffff : j;
            }
            off += sg.len;
        }
    }
    __syncthreads();
    if (!live) return;
    if (serial) {
        if (lane == 0) csr_row_serial<FILL>(B, i, vals, vals2, log_values, rowcount, rowptr, colidx, val, val2);
        return;
    }
    const long long outp = FILL ? rowptr[i] : 0;
    long long kept = 0;
    for (int t0 = 0; t0 < T; t0 += 64) {
        const int t = t0 + lane;
        int j = 0x7fffffff;
        if (t < T) j = B.R > 1 ? cols[t] : B.perm[(long long)B.R * B.n + B.seg_x[i].vstart + t];
        const bool keep = j != 0x7fffffff;
        if (!FILL) {
            kept += __popcll(__ballot(keep));
            continue;
        }
        if (!keep) continue;
        int rank = t;  // one round: the record is in column order and nothing is dropped
        if (B.R > 1) {
            rank = 0;
#pragma unroll 8
            for (int q = 0; q < T; ++q) rank += cols[q] < j ? 1 : 0;
        }
        if (colidx) colidx[outp + rank] = j;
        if (val) val[outp + rank] = log_values ? expf(vals[base + t]) : vals[base + t];
        if (val2) val2[outp + rank] = vals2[base + t];
    }
    if (!FILL && lane == 0) rowcount[i] = kept;
}

hipError_t launch_csr_count(const Handle &h, long long *rowcount, hipStream_t s)
{
    hipLaunchKernelGGL(csr_kernel<false>, dim3((unsigned)((h.n + 3) / 4)), dim3(256), 0, s, h.sort, h.vals_x,
                       (const float *)nullptr, h.log_domain, rowcount, (const long long *)nullptr, (int32_t *)nullptr,
                       (float *)nullptr, (float *)nullptr);
    return hipGetLastError();
}

hipError_t launch_csr_fill(const Handle &h, const long long *rowptr, int32_t *colidx, float *val, hipStream_t s)
{
    hipLaunchKernelGGL(csr_kernel<true>, dim3((unsigned)((h.n + 3) / 4)), dim3(256), 0, s, h.sort, h.vals_x,
                       (const float *)nullptr, h.log_domain, (long long *)nullptr, rowptr, colidx, val,
                       (float *)nullptr);
    return hipGetLastError();
}

// Sparse part of the plan for a block of rows, one wavefront per row: every stored pair of the
// row that no earlier round owns adds u_i val_ij v_j to out[i - i0][j] (values held as logs:
// sets exp(log u_i + val_ij + log v_j)).  Each (i, j) is touched by one lane only.
__global__ __launch_bounds__(256) void plan_sparse_kernel(SortBuffers B, const float *__restrict__ vals_x,
                                                          int log_values, long long i0, long long nrows,
                                                          const double *__restrict__ lin_u,
                                                          const double *__restrict__ lin_v,
                                                          const double *__restrict__ acc_y,
                                                          const double *__restrict__ acc_z, int lp,
                                                          float *__restrict__ out)
{
    const long long li = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (li >= nrows) return;
    const long long i = i0 + li;
    const int lane = threadIdx.x & 63;
    const long long N = B.n + B.m;
    const double ui = lin_u[i];
    const double scale = log_values ? 0.0 : exp(acc_y[lp] + acc_z[lp]);
    long long at = B.rowbase_x[i];
    for (int r = 0; r < B.R; ++r) {
        const Seg sg = B.seg_x[(long long)r * B.n + i];
        const int *yperm = B.perm + (long long)B.R * B.n + (long long)r * B.m;
        const int seg0 = sg.vstart - (int)((long long)r * B.m);
        for (int e = lane; e < sg.len; e += 64) {
            const int j = yperm[seg0 + e];
            if (owned_by_earlier_round(B.bucket, N, B.n, r, i, j)) continue;
            const double v = (double)vals_x[at + e];
            float *dst = out + li * B.m + j;
            if (log_values) {
                const double t = v + ui + lin_v[j];
                *dst = t > -INFINITY ? (float)exp(t) : 0.f;
            } else {
                *dst += (float)(v * ui * lin_v[j] * scale);
            }
        }
        at += sg.len;
    }
}

hipError_t launch_plan_sparse(const Handle &h, long long i0, long long nrows, float *out, hipStream_t s)
{
    hipLaunchKernelGGL(plan_sparse_kernel, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, s, h.sort, h.vals_x,
                       h.log_domain, i0, nrows, h.lin_u, h.lin_v, h.acc[0], h.acc[1], h.lp, out);
    return hipGetLastError();
}

// rec / rec2 (nullable): values in the layout of X's row records; val / val2: the same in CSR order
hipError_t launch_csr_values(const Handle &h, const float *rec, const float *rec2, const long long *rowptr, float *val,
                             float *val2, hipStream_t s)
{
    hipLaunchKernelGGL(csr_kernel<true>, dim3((unsigned)((h.n + 3) / 4)), dim3(256), 0, s, h.sort, rec, rec2, 0,
                       (long long *)nullptr, rowptr, (int32_t *)nullptr, val, val2);
    return hipGetLastError();
}

// in-place exclusive scan of n int64 values by one block; data[n] receives the total
// One workgroup; tiles of 4096 elements, four consecutive ones per thread.
__global__ __launch_bounds__(1024) void scan_i64_kernel(long long *data, long long n)
{
    __shared__ long long wsum[16];
    const int tid = threadIdx.x;
    long long carry = 0;
    for (long long t0 = 0; t0 < n; t0 += 4096) {
        const long long i0 = t0 + 4 * tid;
        long long v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = i0 + q < n ? data[i0 + q] : 0;
        long long tile_total;
        long long run = carry + block_exclusive_scan_1024(v[0] + v[1] + v[2] + v[3], wsum, &tile_total);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i0 + q < n) data[i0 + q] = run;
            run += v[q];
        }
        carry += tile_total;
    }
    if (tid == 0) data[n] = carry;
}

hipError_t launch_scan_i64(long long *data, long long n, hipStream_t s)
{
    hipLaunchKernelGGL(scan_i64_kernel, dim3(1), dim3(1024), 0, s, data, n);
    return hipGetLastError();
}

}  // namespace lcn
