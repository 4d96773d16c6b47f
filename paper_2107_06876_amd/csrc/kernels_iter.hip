// The Sinkhorn half-iteration (Sec. 2 eq. 2 on the decomposed kernel of Sec. 4):
// for every row i of one side
//     s_i   = F_i . acc_in  +  sum over hash rounds of  tile_row(i) . perm_in
//     out_i = marg_i / s_i
// and, in the same sweep, acc_out = F^T out for the other side's next sweep.
// For the rows of X: F = U, acc_in = y = W v, acc_out = z = U^T u.
// For the rows of Y: F = W^T, acc_in = z, acc_out = y.
// Each stored value (factor entry or sparse value) is read exactly once per
// sweep.  One wavefront owns a row: consecutive lanes read consecutive
// addresses of the factor row, then of each tile row.
//
// Scalings are kept as fp64 linear values for the arithmetic (range e^+-700,
// which covers what a log-domain float state can express) and reported as
// fp32 natural logs; products are accumulated in fp64.
#include "lcn_internal.h"

namespace lcn {

constexpr int PASS_THREADS = 1024;
constexpr int PASS_WAVES = PASS_THREADS / 64;

__device__ inline double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// natural log of a positive finite double: exponent taken out exactly, the
// mantissa's log in single precision (absolute error about 5e-8)
__device__ inline double fast_log(double x)
{
    int e;
    double mant = frexp(x, &e);
    return (double)logf((float)mant) + (double)e * 0.69314718055994530942;
}

__device__ inline double fast_rcp(double x)
{
    double r = __builtin_amdgcn_rcp(x);
    r = fma(fma(-x, r, 1.0), r, r);
    r = fma(fma(-x, r, 1.0), r, r);
    return r;
}

template <int T, int MODE>
__global__ __launch_bounds__(PASS_THREADS) void pass_kernel(PassSide S, int R, int lp, double *partial,
                                                            double *zero_buf, int use_atomics,
                                                            unsigned long long *counters, int empty_slot,
                                                            double *query_out)
{
    constexpr int TT = T > 0 ? T : 1;
    extern __shared__ double zsh[];  // [PASS_WAVES / 2][lp + 2]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long nwaves = (long long)gridDim.x * PASS_WAVES;
    const long long gw = (long long)blockIdx.x * PASS_WAVES + wave;
    const int stride = lp + 2;

    double yreg[TT], zacc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        yreg[t] = (T > 0 && MODE != PASS_INIT) ? S.acc_in[lane + 64 * t] : 0.0;
        zacc[t] = 0.0;
    }
    double q0 = 0.0, q1 = 0.0;
    unsigned long long nonpos = 0, empty = 0;
    // the accumulator that the launch after this one adds into is cleared here
    if (zero_buf && blockIdx.x == 0)
        for (int k = threadIdx.x; k < lp; k += PASS_THREADS) zero_buf[k] = 0.0;

    for (long long row = gw; row < S.rows; row += nwaves) {
        float f[TT];
        double out;
        if (T > 0) {
#pragma unroll
            for (int t = 0; t < TT; ++t) f[t] = S.F[row * lp + lane + 64 * t];
        }
        if (MODE == PASS_INIT) {
            out = exp((double)S.log_out[row]);
        } else {
            double acc = 0.0;
            if (T > 0) {
#pragma unroll
                for (int t = 0; t < TT; ++t) acc = fma((double)f[t], yreg[t], acc);
            }
            int total_len = 0;
            for (int r = 0; r < R; ++r) {
                const RowInfo ri = S.rinfo[(long long)r * S.rows + row];
                const float *tv = S.tiles + ri.start;
                const double *vv = S.perm_in + ri.vstart;
                for (int e = lane; e < ri.len; e += 64) acc = fma((double)tv[e], vv[e], acc);
                total_len += ri.len;
            }
            const double s = wave_sum(acc);
            const double marg = (double)S.marg[row];
            if (MODE == PASS_UPDATE) {
                float lo;
                if (s > 0.0) {
                    out = marg * fast_rcp(s);
                    lo = (float)(fast_log(marg) - fast_log(s));
                } else if (T == 0 && total_len == 0) {
                    out = 0.0;
                    lo = -INFINITY;
                    ++empty;
                } else {
                    out = NAN;
                    lo = NAN;
                    ++nonpos;
                }
                if (lane == 0) S.log_out[row] = lo;
            } else {  // PASS_QUERY
                out = S.lin_out[row];
                const double ri = out * s;
                if (lane == 0 && S.marg_out) S.marg_out[row] = (float)ri;
                if (out > 0.0) q0 += ri * log(out);
                q1 += fabs(ri - marg);
            }
        }
        if (MODE != PASS_QUERY) {
            if (lane == 0) S.lin_out[row] = out;
            if (lane < R) S.perm_out[(long long)lane * S.rows + S.pos[(long long)lane * S.rows + row]] = out;
            if (T > 0) {
#pragma unroll
                for (int t = 0; t < TT; ++t) zacc[t] = fma((double)f[t], out, zacc[t]);
            }
        }
    }

    // workgroup reduction of the per-wave accumulators (upper half of the waves
    // hands its values to the lower half first), then one partial per workgroup
    constexpr int HALF = PASS_WAVES / 2;
    double *mine = zsh + (wave % HALF) * stride;
    if (wave >= HALF) {
        if (T > 0) {
#pragma unroll
            for (int t = 0; t < TT; ++t) mine[lane + 64 * t] = zacc[t];
        }
        if (lane == 0) {
            mine[lp] = q0;
            mine[lp + 1] = q1;
        }
    }
    __syncthreads();
    if (wave < HALF) {
        if (T > 0) {
#pragma unroll
            for (int t = 0; t < TT; ++t) mine[lane + 64 * t] += zacc[t];
        }
        if (lane == 0) {
            mine[lp] += q0;
            mine[lp + 1] += q1;
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < stride; k += PASS_THREADS) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < HALF; ++w) s += zsh[w * stride + k];
        if (use_atomics) {
            if (k < lp) {
                if (MODE != PASS_QUERY) unsafeAtomicAdd(&S.acc_out[k], s);
            } else if (MODE == PASS_QUERY) {
                unsafeAtomicAdd(&query_out[k - lp], s);
            }
        } else {
            partial[(long long)blockIdx.x * stride + k] = s;
        }
    }
    if (lane == 0 && (nonpos | empty)) {
        if (nonpos) atomicAdd(&counters[0], nonpos);
        if (empty) atomicAdd(&counters[empty_slot], empty);
    }
}

// Adds the per-workgroup partial sums of a sweep in workgroup order (so the
// result does not depend on timing).  One workgroup per 64 entries.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const double *__restrict__ partial, int groups,
                                                              int stride, int lp, double *acc_out, double *query_out,
                                                              int is_query)
{
    __shared__ double sh[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    double s = 0.0;
    if (k < stride) {
#pragma unroll 8
        for (int g = wave; g < groups; g += 4) s += partial[(long long)g * stride + k];
    }
    sh[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && k < stride) {
        s = (sh[0][lane] + sh[1][lane]) + (sh[2][lane] + sh[3][lane]);
        if (k < lp) {
            if (!is_query) acc_out[k] = s;
        } else if (is_query) {
            query_out[k - lp] = s;
        }
    }
}

int pass_grid(const Handle &h)
{
    long long rows = h.n > h.m ? h.n : h.m;
    long long g = (rows + PASS_WAVES - 1) / PASS_WAVES;
    return (int)(g < 512 ? g : 512);
}

template <int T>
static hipError_t launch_pass_t(const PassSide &S, const Handle &h, int side, int mode, double *zero_buf,
                                hipStream_t s)
{
    long long g = (S.rows + PASS_WAVES - 1) / PASS_WAVES;
    int grid = (int)(g < h.grid ? g : h.grid);
    size_t lds = sizeof(double) * (size_t)(PASS_WAVES / 2) * (h.lp + 2);
    double *qout = h.query_out + 2 * side;
    int empty_slot = 1 + side;
    if (mode == PASS_UPDATE)
        hipLaunchKernelGGL((pass_kernel<T, PASS_UPDATE>), dim3(grid), dim3(PASS_THREADS), lds, s, S, h.R, h.lp,
                           h.partial, zero_buf, h.use_atomics, h.counters, empty_slot, qout);
    else if (mode == PASS_QUERY)
        hipLaunchKernelGGL((pass_kernel<T, PASS_QUERY>), dim3(grid), dim3(PASS_THREADS), lds, s, S, h.R, h.lp,
                           h.partial, zero_buf, h.use_atomics, h.counters, empty_slot, qout);
    else
        hipLaunchKernelGGL((pass_kernel<T, PASS_INIT>), dim3(grid), dim3(PASS_THREADS), lds, s, S, h.R, h.lp,
                           h.partial, zero_buf, h.use_atomics, h.counters, empty_slot, qout);
    if (!h.use_atomics) {
        const int stride = h.lp + 2;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((stride + 63) / 64), dim3(256), 0, s, h.partial, grid, stride,
                           h.lp, S.acc_out, qout, mode == PASS_QUERY ? 1 : 0);
    }
    return hipGetLastError();
}

// side 0: rows of X (updates u, consumes y = W v, produces z = U^T u); side 1: rows of Y.
// acc_in / acc_out / acc_zero index the three rotating accumulator buffers (-1: none).
hipError_t launch_pass(const Handle &h, int side, int mode, int acc_in, int acc_out, int acc_zero, float *marg_out,
                       hipStream_t s)
{
    PassSide S;
    if (side == 0) {
        S.rows = h.n;
        S.F = h.U;
        S.tiles = h.tiles;
        S.rinfo = h.sort.rinfo_x;
        S.pos = h.sort.pos;
        S.marg = h.a;
        S.log_out = h.log_u;
        S.lin_out = h.lin_u;
        S.perm_out = h.perm_u;
        S.perm_in = h.perm_v;
    } else {
        S.rows = h.m;
        S.F = h.Wt;
        S.tiles = h.tilesT;
        S.rinfo = h.sort.rinfo_y;
        S.pos = h.sort.pos + (long long)h.R * h.n;
        S.marg = h.b_marg;
        S.log_out = h.log_v;
        S.lin_out = h.lin_v;
        S.perm_out = h.perm_v;
        S.perm_in = h.perm_u;
    }
    S.acc_in = acc_in >= 0 ? h.acc[acc_in] : nullptr;
    S.acc_out = acc_out >= 0 ? h.acc[acc_out] : nullptr;
    S.marg_out = marg_out;
    double *zb = (acc_zero >= 0 && h.use_atomics) ? h.acc[acc_zero] : nullptr;
    switch (h.lp / 64) {
        case 0: return launch_pass_t<0>(S, h, side, mode, zb, s);
        case 1: return launch_pass_t<1>(S, h, side, mode, zb, s);
        case 2: return launch_pass_t<2>(S, h, side, mode, zb, s);
        case 3: return launch_pass_t<3>(S, h, side, mode, zb, s);
        case 4: return launch_pass_t<4>(S, h, side, mode, zb, s);
        case 5: return launch_pass_t<5>(S, h, side, mode, zb, s);
        case 6: return launch_pass_t<6>(S, h, side, mode, zb, s);
        case 7: return launch_pass_t<7>(S, h, side, mode, zb, s);
        case 8: return launch_pass_t<8>(S, h, side, mode, zb, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lcn
