// The Sinkhorn half-iteration (Sec. 2 eq. 2 on the decomposed kernel of Sec. 4):
// for every row i of one side
//     s_i   = F_i . acc_in  +  (row record of sparse values) . (gathered scalings)
//     out_i = marg_i / s_i
// and, in the same sweep, acc_out = F^T out for the other side's next sweep.
// For the rows of X: F = U, acc_in = y = W v, acc_out = z = U^T u.
// For the rows of Y: F = W^T, acc_in = z, acc_out = y.
// Each stored value (factor entry or sparse value) is read exactly once per
// sweep.  One wavefront owns a row: consecutive lanes read consecutive
// addresses of the factor row and of the row's record of sparse values; the
// next row's factor entries and metadata are requested before the current
// row is reduced, so that a wave always has loads in flight.
//
// Log-domain stabilisation (App. "Implementational details"): the state is the
// natural log of each scaling (fp32, what is reported).  Because the Nystrom
// part and the correction have signed entries the kernel cannot itself be held
// as logs, so the largest exponent is taken out per vector instead: the working
// copy of a scaling vector is exp(log x - M) in fp64, with M the largest log of
// that vector one iteration earlier (any reference works; logs move slowly), and
// M travels with every quantity derived from the vector.  Products are
// accumulated in fp64.
#include "lcn_internal.h"

namespace lcn {

constexpr int PASS_THREADS = 1024;
constexpr int PASS_WAVES = PASS_THREADS / 64;
constexpr int MAXR = 8;
#ifndef PASS_MIN_WAVES
#define PASS_MIN_WAVES 1
#endif

// One step of a cross-lane sum of doubles through the DPP data path (no LDS):
// adds to every lane the value of the lane that `CTRL` selects; lanes of rows
// outside ROW_MASK add zero.
template <int CTRL, int ROW_MASK>
__device__ inline double dpp_add(double v)
{
    const int lo = __double2loint(v), hi = __double2hiint(v);
    const int plo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xF, false);
    const int phi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xF, false);
    return v + __hiloint2double(phi, plo);
}

// Sum over the 64 lanes of a wavefront in a fixed order; every lane gets the result.
__device__ inline double wave_sum(double v)
{
    v = dpp_add<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141, 0xF>(v);  // row_half_mirror
    v = dpp_add<0x140, 0xF>(v);  // row_mirror: every lane of a 16-lane row holds the row's sum
    v = dpp_add<0x142, 0xA>(v);  // row_bcast15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);  // row_bcast31 into rows 2 and 3: lane 63 holds the total
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

template <int CTRL, int ROW_MASK>
__device__ inline double dpp_max(double v)
{
    const int lo = __double2loint(v), hi = __double2hiint(v);
    // lanes outside ROW_MASK receive their own value back
    const int plo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, ROW_MASK, 0xF, false);
    const int phi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, ROW_MASK, 0xF, false);
    return fmax(v, __hiloint2double(phi, plo));
}

// Maximum over the 64 lanes of a wavefront; every lane gets the result.
__device__ inline double wave_max(double v)
{
    v = dpp_max<0xB1, 0xF>(v);
    v = dpp_max<0x4E, 0xF>(v);
    v = dpp_max<0x141, 0xF>(v);
    v = dpp_max<0x140, 0xF>(v);
    v = dpp_max<0x142, 0xA>(v);
    v = dpp_max<0x143, 0xC>(v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

// natural log of a positive finite double: exponent taken out exactly, the
// mantissa's log in single precision (absolute error about 5e-8)
__device__ inline double fast_log(double x)
{
    int e;
    double mant = frexp(x, &e);
    return (double)__logf((float)mant) + (double)e * 0.69314718055994530942;
}

__device__ inline double fast_rcp(double x)
{
    double r = __builtin_amdgcn_rcp(x);
    r = fma(fma(-x, r, 1.0), r, r);
    r = fma(fma(-x, r, 1.0), r, r);
    return r;
}

// Factor row held by a wave.  lp = 64 T.  If T is a multiple of 4 a lane holds
// 4 consecutive entries per 256 (one 16-byte load each), else one entry per 64.
template <int T>
struct FRow {
    static constexpr int TT = T > 0 ? T : 1;
    static constexpr bool VEC = (T > 0) && (T % 4 == 0);
    float f[TT];
    __device__ inline void load(const float *__restrict__ F, long long row, int lp, int lane)
    {
        if (T == 0) return;
        if (VEC) {
#pragma unroll
            for (int q = 0; q < T / 4; ++q) {
                const float4 v = *(const float4 *)(F + row * lp + 256 * q + 4 * lane);
                f[4 * q + 0] = v.x;
                f[4 * q + 1] = v.y;
                f[4 * q + 2] = v.z;
                f[4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int t = 0; t < TT; ++t) f[t] = F[row * lp + 64 * t + lane];
        }
    }
    // index into the length-lp vectors of register slot e
    __device__ static inline int kidx(int e, int lane)
    {
        return VEC ? 256 * (e / 4) + 4 * lane + (e % 4) : 64 * e + lane;
    }
};

// Per-row metadata, read from the packed record (see meta_kernel): wave-uniform,
// so it lives in scalar registers.
template <int RR>
struct RowMeta {
    long long base;
    float marg;
    double log_marg;
    int vstart[RR];
    int len[RR];
    int pos;     // lane r < R: position of the row in round r's bucket order
    double lin;  // query mode: the row's current scaling
};

template <int RR, int MODE>
__device__ inline void load_meta(RowMeta<RR> &M, const PassSide &S, int R, long long row, int lane)
{
    const int *__restrict__ rec = S.meta + row * S.meta_stride;
    M.base = ((long long)rec[1] << 32) | (unsigned)rec[0];
    M.marg = __int_as_float(rec[2]);
    M.log_marg = __hiloint2double(rec[5], rec[4]);
#pragma unroll
    for (int r = 0; r < RR; ++r) {
        M.vstart[r] = r < R ? rec[6 + 2 * r] : 0;
        M.len[r] = r < R ? rec[7 + 2 * r] : 0;
    }
    M.pos = (MODE != PASS_QUERY && lane < R) ? rec[6 + 2 * R + lane] : 0;
    M.lin = MODE == PASS_QUERY ? S.lin_out[row] : 0.0;
}

template <int T, int RR, int MODE>
__global__ __launch_bounds__(PASS_THREADS, PASS_MIN_WAVES) void pass_kernel(PassSide S, int R, int lp, double *partial,
                                                            unsigned long long *counters, int empty_slot)
{
    constexpr int TT = T > 0 ? T : 1;
    extern __shared__ double zsh[];  // [PASS_WAVES / 2][lp + 3]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * PASS_WAVES;
    const long long gw = (long long)blockIdx.x * PASS_WAVES + wave;
    const int stride = lp + 3;
    // exponents taken out of this side's vector (m_self) and of the input vectors (m_in)
    // (a query reads the exponent its vector was stored with, kept beside the accumulator it produced)
    const double m_self = MODE == PASS_QUERY ? S.acc_out[lp] : *S.shift_self;
    const double m_in = MODE != PASS_INIT ? S.acc_in[lp] : 0.0;
    const double e_out = MODE == PASS_UPDATE ? exp(-m_in - m_self) : (MODE == PASS_QUERY ? exp(m_in + m_self) : 1.0);
    double maxlog = -INFINITY;

    double yreg[TT], zacc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        yreg[t] = (T > 0 && MODE != PASS_INIT) ? S.acc_in[FRow<T>::kidx(t, lane)] : 0.0;
        zacc[t] = 0.0;
    }
    double q0 = 0.0, q1 = 0.0;
    unsigned long long nonpos = 0, empty = 0;

    // Three-stage software pipeline over the rows a wave owns: metadata is read
    // two rows ahead (scalar loads), the factor row and the first 64 entries of
    // every round's segment one row ahead, and the current row is reduced while
    // those loads are in flight.
    struct RowData {
        FRow<T> f;
        float tv[RR];
        double vv[RR];
    };
    auto issue = [&](RowData &D, const RowMeta<RR> &M, long long r) {
        D.f.load(S.F, r, lp, lane);
        if (MODE != PASS_INIT) {
            const float *__restrict__ vals = S.vals + M.base;
            int off = 0;
#pragma unroll
            for (int q = 0; q < RR; ++q) {
                const bool ok = lane < M.len[q];
                D.tv[q] = ok ? vals[off + lane] : 0.f;
                D.vv[q] = ok ? S.perm_in[M.vstart[q] + lane] : 0.0;
                off += M.len[q];
            }
        }
    };
    RowData cur{}, nxt{};
    RowMeta<RR> mc{}, mn{}, mn2{};
    const int Rm = MODE == PASS_INIT ? 0 : R;
    long long row = gw, next = gw + nwaves, next2 = gw + 2 * nwaves;
    if (row < S.rows) {
        load_meta<RR, MODE>(mc, S, Rm, row, lane);
        if (MODE == PASS_INIT && lane < R) mc.pos = S.meta[row * S.meta_stride + 6 + 2 * R + lane];
        issue(cur, mc, row);
    }
    if (next < S.rows) {
        load_meta<RR, MODE>(mn, S, Rm, next, lane);
        if (MODE == PASS_INIT && lane < R) mn.pos = S.meta[next * S.meta_stride + 6 + 2 * R + lane];
    }
    while (row < S.rows) {
        if (next < S.rows) issue(nxt, mn, next);
        if (next2 < S.rows) {
            load_meta<RR, MODE>(mn2, S, Rm, next2, lane);
            if (MODE == PASS_INIT && lane < R) mn2.pos = S.meta[next2 * S.meta_stride + 6 + 2 * R + lane];
        }
        double out;
        if (MODE == PASS_INIT) {
            const double lo = (double)S.log_out[row];
            out = exp(lo - m_self);
            if (lo > maxlog && lo < INFINITY) maxlog = lo;
        } else {
            double acc = 0.0;
#pragma unroll
            for (int q = 0; q < RR; ++q) acc = fma((double)cur.tv[q], cur.vv[q], acc);
            {   // what is left of segments longer than a wavefront
                const float *__restrict__ vals = S.vals + mc.base;
                int off = 0;
#pragma unroll
                for (int q = 0; q < RR; ++q) {
                    if (mc.len[q] > 64) {
                        const float *tp = vals + off;
                        const double *vp = S.perm_in + mc.vstart[q];
                        for (int e = 64 + lane; e < mc.len[q]; e += 64) acc = fma((double)tp[e], vp[e], acc);
                    }
                    off += mc.len[q];
                }
            }
            if (T > 0) {
#pragma unroll
                for (int t = 0; t < TT; ++t) acc = fma((double)cur.f.f[t], yreg[t], acc);
            }
            const double s = wave_sum(acc);
            const double marg = (double)mc.marg;
            if (MODE == PASS_UPDATE) {
                float lo;
                if (s > 0.0) {
                    out = marg * fast_rcp(s) * e_out;
                    const double lg = mc.log_marg - fast_log(s) - m_in;
                    lo = (float)lg;
                    maxlog = fmax(maxlog, lg);
                } else if (T == 0 && s == 0.0) {  // no kernel entry (or only zero ones): the point carries no mass
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
                out = mc.lin;
                const double ri = out * s * e_out;
                if (lane == 0 && S.marg_out) S.marg_out[row] = (float)ri;
                if (out > 0.0) q0 += ri * (log(out) + m_self);
                q1 += fabs(ri - marg);
            }
        }
        if (MODE != PASS_QUERY) {
            if (lane == 0) S.lin_out[row] = out;
            if (lane < R) S.perm_out[(long long)lane * S.rows + mc.pos] = out;
            if (T > 0) {
#pragma unroll
                for (int t = 0; t < TT; ++t) zacc[t] = fma((double)cur.f.f[t], out, zacc[t]);
            }
        }
        cur = nxt;
        mc = mn;
        mn = mn2;
        row = next;
        next = next2;
        next2 += nwaves;
    }

    // workgroup reduction of the per-wave accumulators (upper half of the waves
    // hands its values to the lower half first), then one partial per workgroup
    constexpr int HALF = PASS_WAVES / 2;
    double *mine = zsh + (wave % HALF) * stride;
    if (wave >= HALF) {
        if (T > 0) {
#pragma unroll
            for (int t = 0; t < TT; ++t) mine[FRow<T>::kidx(t, lane)] = zacc[t];
        }
        if (lane == 0) {
            mine[lp] = q0;
            mine[lp + 1] = q1;
            mine[lp + 2] = maxlog;
        }
    }
    __syncthreads();
    if (wave < HALF) {
        if (T > 0) {
#pragma unroll
            for (int t = 0; t < TT; ++t) mine[FRow<T>::kidx(t, lane)] += zacc[t];
        }
        if (lane == 0) {
            mine[lp] += q0;
            mine[lp + 1] += q1;
            mine[lp + 2] = fmax(mine[lp + 2], maxlog);
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < stride; k += PASS_THREADS) {
        double s = k == lp + 2 ? -INFINITY : 0.0;
#pragma unroll
        for (int w = 0; w < HALF; ++w) s = k == lp + 2 ? fmax(s, zsh[w * stride + k]) : s + zsh[w * stride + k];
        partial[(long long)blockIdx.x * stride + k] = s;
    }
    if (lane == 0 && (nonpos | empty)) {
        if (nonpos) atomicAdd(&counters[0], nonpos);
        if (empty) atomicAdd(&counters[empty_slot], empty);
    }
}

// The half-iteration for kernels without signed parts (sparse K^sp, and the
// dense kernel as its one-bucket case), entirely in logs: the stored values
// are log K_ij = -C_ij / lambda, the vectors are log scalings, and a row's sum
// is a log-sum-exp (App. "Implementational details") with a running maximum per
// lane, so that scalings may drift arbitrarily far (a sparse kernel need not
// have support, App. "Limitations") without over- or underflow.
__device__ inline void lse_step(double t, double &mx, double &sm)
{
    if (t > -INFINITY) {
        const double d = t - mx;
        const double e = (double)__expf(-fabsf((float)d));
        if (d > 0.0) {
            sm = fma(sm, e, 1.0);
            mx = t;
        } else {
            sm += e;
        }
    }
}

template <int RR, int MODE>
__global__ __launch_bounds__(PASS_THREADS) void logpass_kernel(PassSide S, int R, double *partial,
                                                               unsigned long long *counters, int empty_slot)
{
    __shared__ double qsh[PASS_WAVES][2];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * PASS_WAVES;
    double q0 = 0.0, q1 = 0.0;
    unsigned long long empty = 0;

    RowMeta<RR> mc{}, mn{};
    long long row = (long long)blockIdx.x * PASS_WAVES + wave;
    if (row < S.rows) load_meta<RR, MODE>(mc, S, R, row, lane);
    while (row < S.rows) {
        const long long next = row + nwaves;
        double lg;
        if (MODE == PASS_INIT) {
            if (next < S.rows) load_meta<RR, MODE>(mn, S, R, next, lane);
            lg = (double)S.log_out[row];
        } else {
            const float *__restrict__ vals = S.vals + mc.base;
            double mx = -INFINITY, sm = 0.0;
            {
                double t0[RR];
                int segoff[RR];
                int total_len = 0;
#pragma unroll
                for (int r = 0; r < RR; ++r) {
                    segoff[r] = total_len;
                    total_len += mc.len[r];
                    t0[r] = lane < mc.len[r] ? (double)vals[segoff[r] + lane] + S.perm_in[mc.vstart[r] + lane]
                                             : -INFINITY;
                }
                if (next < S.rows) load_meta<RR, MODE>(mn, S, R, next, lane);
#pragma unroll
                for (int r = 0; r < RR; ++r) lse_step(t0[r], mx, sm);
#pragma unroll
                for (int r = 0; r < RR; ++r) {
                    if (mc.len[r] > 64) {
                        const float *tp = vals + segoff[r];
                        const double *vp = S.perm_in + mc.vstart[r];
#pragma unroll 2
                        for (int e = 64 + lane; e < mc.len[r]; e += 64) lse_step((double)tp[e] + vp[e], mx, sm);
                    }
                }
            }
            const double M = wave_max(mx);
            const double part = mx > -INFINITY ? sm * exp(mx - M) : 0.0;
            const double ssum = wave_sum(part);
            const double lse = ssum > 0.0 ? M + log(ssum) : -INFINITY;
            if (MODE == PASS_UPDATE) {
                if (lse > -INFINITY) {
                    lg = mc.log_marg - lse;
                } else {  // no kernel entry reaches this point: it carries no mass
                    lg = -INFINITY;
                    ++empty;
                }
                if (lane == 0) S.log_out[row] = (float)lg;
            } else {  // PASS_QUERY
                lg = mc.lin;
                const double ri = (lg > -INFINITY && lse > -INFINITY) ? exp(lg + lse) : 0.0;
                if (lane == 0 && S.marg_out) S.marg_out[row] = (float)ri;
                if (ri != 0.0) q0 += ri * lg;
                q1 += fabs(ri - (double)mc.marg);
            }
        }
        if (MODE != PASS_QUERY) {
            if (lane == 0) S.lin_out[row] = lg;
            if (lane < R) S.perm_out[(long long)lane * S.rows + mc.pos] = lg;
        }
        mc = mn;
        row = next;
    }
    if (MODE == PASS_QUERY) {
        if (lane == 0) {
            qsh[wave][0] = q0;
            qsh[wave][1] = q1;
        }
        __syncthreads();
        if (threadIdx.x < 3) {
            double s = threadIdx.x == 2 ? -INFINITY : 0.0;
            if (threadIdx.x < 2)
                for (int w = 0; w < PASS_WAVES; ++w) s += qsh[w][threadIdx.x];
            partial[(long long)blockIdx.x * 3 + threadIdx.x] = s;
        }
    }
    if (lane == 0 && empty) atomicAdd(&counters[empty_slot], empty);
}

// Adds the per-workgroup partial sums of a sweep in a fixed order (so the
// result does not depend on timing).  One workgroup per 64 entries; wave w adds
// the partials of workgroups w, w + 16, ..., then the 16 wave sums are added.
// Entry lp + 2 is a maximum (the largest log scaling of the sweep), which
// becomes this side's exponent for the next sweep; entry lp of the output
// accumulator records the exponent that this sweep's vector was stored with.
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const double *__restrict__ partial, int groups,
                                                               int stride, int lp, double *acc_out,
                                                               double *query_out, double *shift_self, int mode)
{
    __shared__ double sh[16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    const bool is_max = k == lp + 2;
    double s = is_max ? -INFINITY : 0.0;
    if (k < stride) {
#pragma unroll 16
        for (int g = wave; g < groups; g += 16) {
            const double v = partial[(long long)g * stride + k];
            s = is_max ? fmax(s, v) : s + v;
        }
    }
    sh[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && k < stride) {
        s = is_max ? -INFINITY : 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) s = is_max ? fmax(s, sh[w][lane]) : s + sh[w][lane];
        if (k < lp) {
            if (mode != PASS_QUERY) acc_out[k] = s;
        } else if (k < lp + 2) {
            if (mode == PASS_QUERY) query_out[k - lp] = s;
        } else if (mode != PASS_QUERY) {
            acc_out[lp] = *shift_self;                              // exponent used by this sweep
            *shift_self = (s > -INFINITY && s < INFINITY) ? s : 0.0;  // exponent for the next one
        }
    }
}

// largest finite entry of a float vector (0 if there is none); one workgroup
__global__ __launch_bounds__(1024) void max_log_kernel(const float *__restrict__ x, long long n, double *out)
{
    __shared__ float sh[1024];
    float m = -INFINITY;
    for (long long i = threadIdx.x; i < n; i += 1024) {
        const float v = x[i];
        if (v > m && v < INFINITY) m = v;
    }
    sh[threadIdx.x] = m;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) sh[threadIdx.x] = fmaxf(sh[threadIdx.x], sh[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = sh[0] > -INFINITY ? (double)sh[0] : 0.0;
}

// Workgroups of a sweep: as many as are resident at once (compute units x
// workgroups per compute unit that the kernel's register use allows), so that
// every row slot is dealt out once and the partial sums stay few.
template <int T, int RR>
static int resident_blocks()
{
    int dev = 0, cus = 256, per_cu = 1;
    if (hipGetDevice(&dev) == hipSuccess) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
    }
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pass_kernel<T, RR, PASS_UPDATE>, PASS_THREADS,
                                                     sizeof(double) * (PASS_WAVES / 2) * (64 * T + 3)) != hipSuccess ||
        per_cu < 1)
        per_cu = 1;
    (void)hipGetLastError();
    return cus * per_cu;
}

int pass_grid(const Handle &h)
{
    long long rows = h.n > h.m ? h.n : h.m;
    long long g = (rows + PASS_WAVES - 1) / PASS_WAVES;
    long long cap = h.grid_cap;
    if (cap <= 0) {
        if (h.log_domain) {
            cap = 512;
        } else {
            const bool r8 = h.R > 4;
            switch (h.lp / 64) {
                case 0: cap = r8 ? resident_blocks<0, 8>() : resident_blocks<0, 4>(); break;
                case 1: cap = r8 ? resident_blocks<1, 8>() : resident_blocks<1, 4>(); break;
                case 2: cap = r8 ? resident_blocks<2, 8>() : resident_blocks<2, 4>(); break;
                case 3: cap = r8 ? resident_blocks<3, 8>() : resident_blocks<3, 4>(); break;
                case 4: cap = r8 ? resident_blocks<4, 8>() : resident_blocks<4, 4>(); break;
                case 5: cap = r8 ? resident_blocks<5, 8>() : resident_blocks<5, 4>(); break;
                case 6: cap = r8 ? resident_blocks<6, 8>() : resident_blocks<6, 4>(); break;
                case 7: cap = r8 ? resident_blocks<7, 8>() : resident_blocks<7, 4>(); break;
                default: cap = r8 ? resident_blocks<8, 8>() : resident_blocks<8, 4>(); break;
            }
        }
    }
    return (int)(g < cap ? g : cap);
}

template <int T, int RR>
static hipError_t launch_pass_tr(const PassSide &S, const Handle &h, int side, int mode, hipStream_t s)
{
    long long g = (S.rows + PASS_WAVES - 1) / PASS_WAVES;
    int grid = (int)(g < h.grid ? g : h.grid);
    const int stride = h.lp + 3;
    size_t lds = sizeof(double) * (size_t)(PASS_WAVES / 2) * stride;
    double *qout = h.query_out + 2 * side;
    int empty_slot = 1 + side;
    if (mode == PASS_INIT)
        hipLaunchKernelGGL(max_log_kernel, dim3(1), dim3(1024), 0, s, S.log_out, S.rows, S.shift_self);
    if (mode == PASS_UPDATE)
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_UPDATE>), dim3(grid), dim3(PASS_THREADS), lds, s, S, h.R, h.lp,
                           h.partial, h.counters, empty_slot);
    else if (mode == PASS_QUERY)
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_QUERY>), dim3(grid), dim3(PASS_THREADS), lds, s, S, h.R, h.lp,
                           h.partial, h.counters, empty_slot);
    else
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_INIT>), dim3(grid), dim3(PASS_THREADS), lds, s, S, h.R, h.lp,
                           h.partial, h.counters, empty_slot);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((stride + 63) / 64), dim3(1024), 0, s, h.partial, grid, stride,
                       h.lp, S.acc_out, qout, S.shift_self, mode);
    return hipGetLastError();
}

template <int T>
static hipError_t launch_pass_t(const PassSide &S, const Handle &h, int side, int mode, hipStream_t s)
{
    if (h.R <= 4) return launch_pass_tr<T, 4>(S, h, side, mode, s);
    return launch_pass_tr<T, 8>(S, h, side, mode, s);
}

// side 0: rows of X (updates u, consumes y = W v, produces z = U^T u); side 1: rows of Y.
// acc_in / acc_out index the accumulator buffers (-1: none).
hipError_t launch_pass(const Handle &h, int side, int mode, int acc_in, int acc_out, float *marg_out, hipStream_t s)
{
    PassSide S;
    if (side == 0) {
        S.rows = h.n;
        S.F = h.U;
        S.vals = h.vals_x;
        S.meta = h.sort.meta_x;
        S.log_out = h.log_u;
        S.lin_out = h.lin_u;
        S.perm_out = h.perm_u;
        S.perm_in = h.perm_v;
    } else {
        S.rows = h.m;
        S.F = h.Wt;
        S.vals = h.vals_y;
        S.meta = h.sort.meta_y;
        S.log_out = h.log_v;
        S.lin_out = h.lin_v;
        S.perm_out = h.perm_v;
        S.perm_in = h.perm_u;
    }
    S.acc_in = acc_in >= 0 ? h.acc[acc_in] : nullptr;
    S.acc_out = acc_out >= 0 ? h.acc[acc_out] : nullptr;
    S.marg_out = marg_out;
    S.meta_stride = h.sort.meta_stride;
    S.shift_self = h.shift + side;
    if (h.log_domain) {
        long long g = (S.rows + PASS_WAVES - 1) / PASS_WAVES;
        const int grid = (int)(g < h.grid ? g : h.grid);
        const int empty_slot = 1 + side;
        if (h.R <= 4) {
            if (mode == PASS_UPDATE)
                hipLaunchKernelGGL((logpass_kernel<4, PASS_UPDATE>), dim3(grid), dim3(PASS_THREADS), 0, s, S, h.R,
                                   h.partial, h.counters, empty_slot);
            else if (mode == PASS_QUERY)
                hipLaunchKernelGGL((logpass_kernel<4, PASS_QUERY>), dim3(grid), dim3(PASS_THREADS), 0, s, S, h.R,
                                   h.partial, h.counters, empty_slot);
            else
                hipLaunchKernelGGL((logpass_kernel<4, PASS_INIT>), dim3(grid), dim3(PASS_THREADS), 0, s, S, h.R,
                                   h.partial, h.counters, empty_slot);
        } else {
            if (mode == PASS_UPDATE)
                hipLaunchKernelGGL((logpass_kernel<8, PASS_UPDATE>), dim3(grid), dim3(PASS_THREADS), 0, s, S, h.R,
                                   h.partial, h.counters, empty_slot);
            else if (mode == PASS_QUERY)
                hipLaunchKernelGGL((logpass_kernel<8, PASS_QUERY>), dim3(grid), dim3(PASS_THREADS), 0, s, S, h.R,
                                   h.partial, h.counters, empty_slot);
            else
                hipLaunchKernelGGL((logpass_kernel<8, PASS_INIT>), dim3(grid), dim3(PASS_THREADS), 0, s, S, h.R,
                                   h.partial, h.counters, empty_slot);
        }
        if (mode == PASS_QUERY)
            hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(1024), 0, s, h.partial, grid, 3, 0, S.acc_out,
                               h.query_out + 2 * side, S.shift_self, mode);
        return hipGetLastError();
    }
    switch (h.lp / 64) {
        case 0: return launch_pass_t<0>(S, h, side, mode, s);
        case 1: return launch_pass_t<1>(S, h, side, mode, s);
        case 2: return launch_pass_t<2>(S, h, side, mode, s);
        case 3: return launch_pass_t<3>(S, h, side, mode, s);
        case 4: return launch_pass_t<4>(S, h, side, mode, s);
        case 5: return launch_pass_t<5>(S, h, side, mode, s);
        case 6: return launch_pass_t<6>(S, h, side, mode, s);
        case 7: return launch_pass_t<7>(S, h, side, mode, s);
        case 8: return launch_pass_t<8>(S, h, side, mode, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lcn
