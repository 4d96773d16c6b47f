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
#include "iter_common.h"

namespace lcn {

// FUSED (update sweeps after the first of a run): the previous sweep's partial
// sums have not been added up yet.  The first ceil((lp + 3) / 64) workgroups of
// this launch do that before their own rows and publish the totals; every
// workgroup requests its first rows, then waits for the totals (bounded wait;
// the reducing workgroups have the lowest indices, are dispatched first and
// wait for nothing, so the wait ends).  This saves a dependent kernel launch
// per sweep without any device-wide fence.
template <int T, int RR, int MODE, bool FUSED>
__global__ __launch_bounds__(PASS_THREADS, PASS_MIN_WAVES) void pass_kernel(PassSide S, int R, int lp, double *partial,
                                                            unsigned long long *counters, int empty_slot,
                                                            FuseArgs Fz)
{
    constexpr int TT = T > 0 ? T : 1;
    extern __shared__ double zsh[];  // [PASS_WAVES / 2][lp + 3], then [lp + 2] and [16][64] if FUSED
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * PASS_WAVES;
    // Rows are dealt out from the last workgroup down: the reducing workgroups of a fused
    // sweep (the first few) start late, so they get the row slots that may hold one row less.
    // The dealing is the same with and without fusion, so both give the same bits.
    const long long gw = (long long)(gridDim.x - 1 - blockIdx.x) * PASS_WAVES + wave;
    const int stride = lp + 3;
    // exponents taken out of this side's vector (m_self) and of the input vectors (m_in)
    // (a query reads the exponent its vector was stored with, kept beside the accumulator it produced)
    if (MODE == PASS_UPDATE) mark_pending(Fz, lp);
    if (FUSED && (int)blockIdx.x < (stride + 63) / 64)
        reduce_publish(Fz, blockIdx.x, lp, zsh + (size_t)(PASS_WAVES / 2) * stride + lp + 2);
    const double m_self = MODE == PASS_QUERY ? S.acc_out[lp] : *S.shift_self;
    double m_in = 0.0, e_out = 1.0;
    double maxlog = -INFINITY;

    double yreg[TT], zacc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        yreg[t] = 0.0;
        zacc[t] = 0.0;
    }
    if (!FUSED) {
        m_in = MODE != PASS_INIT ? S.acc_in[lp] : 0.0;
        e_out = MODE == PASS_UPDATE ? exp(-m_in - m_self) : (MODE == PASS_QUERY ? exp(m_in + m_self) : 1.0);
#pragma unroll
        for (int t = 0; t < TT; ++t)
            yreg[t] = (T > 0 && MODE != PASS_INIT) ? S.acc_in[FRow<T>::kidx(t, lane)] : 0.0;
    }
    double q0 = 0.0, q1 = 0.0;
    unsigned long long nonpos = 0, empty = 0, range = 0;

    // Three-stage software pipeline over the rows a wave owns: metadata is read
    // two rows ahead (scalar loads), the factor row and the first 64 entries of
    // every round's segment one row ahead, and the current row is reduced while
    // those loads are in flight.
    struct RowData {
        FRow<T> f;
        float tv[RR];
        float vv[RR];
    };
    // The bucket-ordered copies of the scalings are single precision in this kernel (the buffers are
    // sized for doubles; the logarithmic kernels keep doubles there): they are gathered once per
    // stored value, and at half the size they stay in the per-die cache beside the streamed rows.
    // The exponent taken out keeps the largest entry near one, and the copies are stored times
    // PERM_SCALE = 2^64 (exact): single precision then holds entries from 2^-190 (e^-131) below the
    // vector's largest up to 2^63 (e^43) above it.  A sum's sparse part is scaled back before the
    // factor part is added.  An entry that grows past that within one iteration overflows its copy:
    // counted, and the run is reported as failed (LCN_ERR_RANGE).
    const float *__restrict__ perm_in = reinterpret_cast<const float *>(S.perm_in);
    float *__restrict__ perm_out = reinterpret_cast<float *>(S.perm_out);
    // Loads are issued for whole wavefront-wide chunks without predication: lanes
    // beyond a segment's length read the next stored values (masked when used; the
    // arrays end with 64 entries of slack) and the zero slot behind the gathered vector.
    const unsigned zero_slot = (unsigned)((R > 0 ? R : 1) * S.rows_in);
    auto issue = [&](RowData &D, const RowMeta<RR> &M, long long r) {
        D.f.load(S.F, r, lp, lane);
        if (MODE != PASS_INIT) {
            const float *__restrict__ vals = S.vals + M.base;
            unsigned off = lane;
#pragma unroll
            for (int q = 0; q < RR; ++q) {
                D.tv[q] = vals[off];
                D.vv[q] = perm_in[lane < M.len[q] ? (unsigned)M.vstart[q] + lane : zero_slot];
                off += (unsigned)M.len[q];
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
    if (FUSED) {
        double *ysh = zsh + (size_t)(PASS_WAVES / 2) * stride;
        if (wave == 0) fused_fetch(Fz, S.acc_in, lp, ysh);
        __syncthreads();
        m_in = ysh[lp];
        e_out = ysh[lp + 1];
        if (T > 0) {
#pragma unroll
            for (int t = 0; t < TT; ++t) yreg[t] = ysh[FRow<T>::kidx(t, lane)];
        }
    }
    // one row: `C` holds the row's data, `N` receives the next row's
    auto step = [&](RowData &C, RowData &N) {
        if (next < S.rows) issue(N, mn, next);
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
            for (int q = 0; q < RR; ++q) acc = fma((double)(lane < mc.len[q] ? C.tv[q] : 0.f), (double)C.vv[q], acc);
            {   // what is left of segments longer than a wavefront
                const float *__restrict__ vals = S.vals + mc.base;
                int off = 0;
#pragma unroll
                for (int q = 0; q < RR; ++q) {
                    if (mc.len[q] > 64) {
                        // 256 entries per trip, all eight loads requested before the first is used
                        const float *tp = vals + off;
                        const float *vp = perm_in + mc.vstart[q];
                        for (int e0 = 64; e0 < mc.len[q]; e0 += 256) {
                            float tt[4];
                            float pv[4];
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const int e = e0 + 64 * k + lane;
                                const bool ok = e < mc.len[q];
                                tt[k] = tp[ok ? e : 0];
                                pv[k] = vp[ok ? e : 0];
                                if (!ok) tt[k] = 0.f;
                            }
#pragma unroll
                            for (int k = 0; k < 4; ++k) acc = fma((double)tt[k], (double)pv[k], acc);
                        }
                    }
                    off += mc.len[q];
                }
            }
            acc *= PERM_UNSCALE;
            if (T > 0) {
#pragma unroll
                for (int t = 0; t < TT; ++t) acc = fma((double)C.f.f[t], yreg[t], acc);
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
            const float outf = (float)(out * PERM_SCALE);
            if (R > 0 && outf == INFINITY) ++range;   // without hash rounds nothing reads the copies
            if (lane < R) perm_out[(long long)lane * S.rows + mc.pos] = outf;
            if (T > 0) {
#pragma unroll
                for (int t = 0; t < TT; ++t) zacc[t] = fma((double)C.f.f[t], out, zacc[t]);
            }
        }
        mc = mn;
        mn = mn2;
        row = next;
        next = next2;
        next2 += nwaves;
    };
    if (T < 6) {
        // the two data buffers swap roles from row to row (no register copies)
        while (row < S.rows) {
            step(cur, nxt);
            if (row >= S.rows) break;
            step(nxt, cur);
        }
    } else {
        // long factor rows: one copy of the loop body keeps the kernel within its registers
        while (row < S.rows) {
            step(cur, nxt);
            cur = nxt;
        }
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
    if (lane == 0 && (nonpos | empty | range)) {
        if (nonpos) atomicAdd(&counters[0], nonpos);
        if (empty) atomicAdd(&counters[empty_slot], empty);
        if (range) atomicAdd(&counters[6], range);
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
            // f(log kernel value, log scaling) for every stored entry of the row; a lane past the end
            // of a piece passes a scaling of -infinity
            auto walk = [&](auto &&f) {
                float k0[RR];
                double p0[RR];
                int segoff[RR];
                int total_len = 0;
#pragma unroll
                for (int r = 0; r < RR; ++r) {
                    segoff[r] = total_len;
                    total_len += mc.len[r];
                    const bool in = lane < mc.len[r];
                    k0[r] = in ? vals[segoff[r] + lane] : 0.f;
                    p0[r] = in ? S.perm_in[mc.vstart[r] + lane] : -INFINITY;
                }
#pragma unroll
                for (int r = 0; r < RR; ++r) f(k0[r], p0[r]);
#pragma unroll
                for (int r = 0; r < RR; ++r) {
                    if (mc.len[r] > 64) {
                        const float *tp = vals + segoff[r];
                        const double *vp = S.perm_in + mc.vstart[r];
                        // four wavefront-wide pieces per trip, all eight loads requested before the first use
                        for (int e0 = 64 + lane; e0 < mc.len[r]; e0 += 256) {
                            float kv[4];
                            double pv[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const int e = e0 + 64 * q;
                                const bool in = e < mc.len[r];
                                kv[q] = in ? tp[e] : 0.f;
                                pv[q] = in ? vp[e] : -INFINITY;
                            }
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (e0 - lane + 64 * q < mc.len[r])   // the same in every lane: whole pieces are skipped
                                    f(kv[q], pv[q]);
                        }
                    }
                }
            };
            // The row's log-sum-exp.  First with the row's previous value as the shift (what its current
            // scaling was computed from: near the answer, so the terms are of order one): one subtraction,
            // one single-precision exp and one addition per entry.  If that shift is unusable (no previous
            // value, or the sum leaves single precision's range) the row is walked again with a running
            // maximum per lane, which cannot over- or underflow.
            const double prev = MODE == PASS_QUERY ? mc.lin : S.lin_out[row];
            const double shift = mc.log_marg - prev;
            if (next < S.rows) load_meta<RR, MODE>(mn, S, R, next, lane);
            double lse;
            bool done = false;
            if (shift > -INFINITY && shift < INFINITY) {
                float accf = 0.f;
                walk([&](float k, double pl) { accf += __expf(k + (float)(pl - shift)); });
                const double tot = wave_sum((double)accf);
                if (tot > 1e-30 && tot < 1e30) {
                    lse = shift + fast_log(tot);
                    done = true;
                }
            }
            if (!done) {   // the same in every lane
                double mx = -INFINITY, sm = 0.0;
                walk([&](float k, double pl) { lse_step((double)k + pl, mx, sm); });
                const double M = wave_max(mx);
                const double part = mx > -INFINITY ? sm * exp(mx - M) : 0.0;
                const double ssum = wave_sum(part);
                lse = ssum > 0.0 ? M + log(ssum) : -INFINITY;
            }
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

// The dense kernel (one bucket, one round): every row multiplies the same vector, so a workgroup
// takes DENSE_ROWS consecutive rows and reads each piece of the vector once for all of them
// (one row per wavefront reads it once per row: twice the bytes of the kernel matrix itself,
// from cache).  Its DENSE_WAVES wavefronts share out the columns in pieces of 128 and merge their
// running (maximum, scaled sum) pairs through LDS.  Otherwise as logpass_kernel; PASS_INIT stays
// with logpass_kernel.
constexpr int DENSE_ROWS = 8;
constexpr int DENSE_WAVES = 4;

template <int MODE>
__global__ __launch_bounds__(64 * DENSE_WAVES) void logpass_dense_kernel(PassSide S, double *partial,
                                                                         unsigned long long *counters, int empty_slot)
{
    __shared__ double msh[DENSE_WAVES][DENSE_ROWS][2];
    __shared__ int flag;   // some row of the group needs the second pass
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    double q0 = 0.0, q1 = 0.0;
    unsigned long long empty = 0;
    for (long long r0 = (long long)blockIdx.x * DENSE_ROWS; r0 < S.rows; r0 += (long long)gridDim.x * DENSE_ROWS) {
        RowMeta<1> mt[DENSE_ROWS];
#pragma unroll
        for (int i = 0; i < DENSE_ROWS; ++i)   // rows past the end repeat the last row and are dropped below
            load_meta<1, MODE>(mt[i], S, 1, r0 + i < S.rows ? r0 + i : S.rows - 1, lane);
        const int len = mt[0].len[0];
        const double *__restrict__ vp = S.perm_in + mt[0].vstart[0];
        // two wavefront-wide pieces per trip; the next trip's loads are requested before this trip's
        // values are used
        auto fetch = [&](int e0, double (&p)[2], float (&k)[DENSE_ROWS][2]) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int e = e0 + 64 * q;
                const bool in = e < len;
                p[q] = in ? vp[e] : -INFINITY;
#pragma unroll
                for (int i = 0; i < DENSE_ROWS; ++i) k[i][q] = in ? S.vals[mt[i].base + e] : 0.f;
            }
        };
        // f(row of the group, log kernel value, log scaling, piece) for this wavefront's share of the columns
        auto walk = [&](auto &&f) {
            double pv[2], pvn[2];
            float kv[DENSE_ROWS][2], kvn[DENSE_ROWS][2];
            fetch(128 * wave + lane, pv, kv);
            for (int e0 = 128 * wave + lane; e0 < len; e0 += 128 * DENSE_WAVES) {
                fetch(e0 + 128 * DENSE_WAVES, pvn, kvn);   // beyond the row: nothing is read
                f(kv, pv);
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    pv[q] = pvn[q];
#pragma unroll
                    for (int i = 0; i < DENSE_ROWS; ++i) kv[i][q] = kvn[i][q];
                }
            }
        };
        // First pass: every row's previous log-sum-exp as its shift (see logpass_kernel), sums in single
        // precision; shifts as one common fp64 base plus a small per-row offset.
        double shift[DENSE_ROWS];
        bool usable = true;
#pragma unroll
        for (int i = 0; i < DENSE_ROWS; ++i) {
            const long long row = r0 + i < S.rows ? r0 + i : S.rows - 1;
            shift[i] = mt[i].log_marg - (MODE == PASS_QUERY ? mt[i].lin : S.lin_out[row]);
            usable = usable && shift[i] > -INFINITY && shift[i] < INFINITY;
        }
        __syncthreads();   // the previous group's merge has read msh and flag
        if (usable) {   // the same in every thread
            float off[DENSE_ROWS], accf[DENSE_ROWS];
#pragma unroll
            for (int i = 0; i < DENSE_ROWS; ++i) {
                off[i] = (float)(shift[i] - shift[0]);
                accf[i] = 0.f;
            }
            walk([&](const float (&kv)[DENSE_ROWS][2], const double (&pv)[2]) {
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const float pf = (float)(pv[q] - shift[0]);
#pragma unroll
                    for (int i = 0; i < DENSE_ROWS; ++i) accf[i] += __expf(kv[i][q] + (pf - off[i]));
                }
            });
#pragma unroll
            for (int i = 0; i < DENSE_ROWS; ++i) {
                const double tot = wave_sum((double)accf[i]);
                if (lane == 0) msh[wave][i][0] = tot;
            }
        }
        if (threadIdx.x == 0) flag = usable ? 0 : 1;
        __syncthreads();
        double lse = 0.0;   // wavefront 0, lane i: row r0 + i
        if (usable && wave == 0 && lane < DENSE_ROWS) {
            double tot = 0.0;
#pragma unroll
            for (int w = 0; w < DENSE_WAVES; ++w) tot += msh[w][lane][0];
            double sh_l = shift[0];
#pragma unroll
            for (int i = 1; i < DENSE_ROWS; ++i) sh_l = lane == i ? shift[i] : sh_l;
            if (tot > 1e-30 && tot < 1e30)
                lse = sh_l + fast_log(tot);
            else if (r0 + lane < S.rows)
                flag = 1;   // benign race: every writer stores 1
        }
        __syncthreads();
        if (flag) {   // the same in every thread: some sum left single precision's range, walk again with running maxima
            double mx[DENSE_ROWS], sm[DENSE_ROWS];
#pragma unroll
            for (int i = 0; i < DENSE_ROWS; ++i) {
                mx[i] = -INFINITY;
                sm[i] = 0.0;
            }
            walk([&](const float (&kv)[DENSE_ROWS][2], const double (&pv)[2]) {
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int i = 0; i < DENSE_ROWS; ++i) lse_step((double)kv[i][q] + pv[q], mx[i], sm[i]);
            });
#pragma unroll
            for (int i = 0; i < DENSE_ROWS; ++i) {
                const double M = wave_max(mx[i]);
                const double part = mx[i] > -INFINITY ? sm[i] * exp(mx[i] - M) : 0.0;
                const double ssum = wave_sum(part);
                if (lane == 0) {
                    msh[wave][i][0] = M;
                    msh[wave][i][1] = ssum;
                }
            }
            __syncthreads();
            if (wave == 0 && lane < DENSE_ROWS) {
                double M = -INFINITY;
#pragma unroll
                for (int w = 0; w < DENSE_WAVES; ++w) M = fmax(M, msh[w][lane][0]);
                double ssum = 0.0;
#pragma unroll
                for (int w = 0; w < DENSE_WAVES; ++w)
                    if (msh[w][lane][0] > -INFINITY) ssum += msh[w][lane][1] * exp(msh[w][lane][0] - M);
                lse = ssum > 0.0 ? M + log(ssum) : -INFINITY;
            }
        }
        // wavefront 0, lane i finishes row r0 + i
        if (wave == 0 && lane < DENSE_ROWS && r0 + lane < S.rows) {
            const long long row = r0 + lane;
            // this lane's row record (the registers hold it per row index, which is a lane here)
            const int *rec = S.meta + row * S.meta_stride;
            if (MODE == PASS_UPDATE) {
                const double log_marg = __hiloint2double(rec[5], rec[4]);
                double lg;
                if (lse > -INFINITY) {
                    lg = log_marg - lse;
                } else {  // no kernel entry reaches this point: it carries no mass
                    lg = -INFINITY;
                    ++empty;
                }
                S.log_out[row] = (float)lg;
                S.lin_out[row] = lg;
                S.perm_out[rec[6 + 2 * 1]] = lg;   // one round: the row's position in the bucket order
            } else {  // PASS_QUERY
                const double lg = S.lin_out[row];
                const double ri = (lg > -INFINITY && lse > -INFINITY) ? exp(lg + lse) : 0.0;
                if (S.marg_out) S.marg_out[row] = (float)ri;
                if (ri != 0.0) q0 += ri * lg;
                q1 += fabs(ri - (double)__int_as_float(rec[2]));
            }
        }
    }
    if (MODE == PASS_QUERY) {
        // only wavefront 0 holds terms, one row per lane
        q0 = wave_sum(q0);
        q1 = wave_sum(q1);
        if (threadIdx.x == 0) {
            partial[(long long)blockIdx.x * 3 + 0] = q0;
            partial[(long long)blockIdx.x * 3 + 1] = q1;
            partial[(long long)blockIdx.x * 3 + 2] = -INFINITY;
        }
    }
    empty = (unsigned long long)wave_sum((double)empty);
    if (threadIdx.x == 0 && empty) atomicAdd(&counters[empty_slot], empty);
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

static size_t pass_lds_bytes(int lp, bool fused)
{
    size_t doubles = (size_t)(PASS_WAVES / 2) * (lp + 3);
    if (fused) doubles += (size_t)lp + 2 + 16 * 64;
    return sizeof(double) * doubles;
}

// Workgroups of a sweep: as many as are resident at once (compute units x
// workgroups per compute unit that the kernel's register use allows), so that
// every row slot is dealt out once and the partial sums stay few.
int device_compute_units()
{
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
    }
    (void)hipGetLastError();
    return cus;
}

template <int T, int RR>
static int resident_blocks()
{
    int cus = device_compute_units(), per_cu = 1;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pass_kernel<T, RR, PASS_UPDATE, true>, PASS_THREADS,
                                                     pass_lds_bytes(64 * T, true)) != hipSuccess ||
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
static hipError_t launch_pass_tr(const PassSide &S, const Handle &h, int side, int mode, const FuseArgs *fuse,
                                 bool fused_in, bool reduce_after, double *partial, unsigned long long *cnt,
                                 hipStream_t s)
{
    long long g = (S.rows + PASS_WAVES - 1) / PASS_WAVES;
    int grid = (int)(g < h.grid ? g : h.grid);
    const int stride = h.lp + 3;
    double *qout = h.query_out + 2 * side;
    int empty_slot = 1 + side;
    FuseArgs none{};
    if (mode == PASS_INIT)
        hipLaunchKernelGGL(max_log_kernel, dim3(1), dim3(1024), 0, s, S.log_out, S.rows, S.shift_self);
    if (mode == PASS_UPDATE && fused_in)
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_UPDATE, true>), dim3(grid), dim3(PASS_THREADS),
                           pass_lds_bytes(h.lp, true), s, S, h.R, h.lp, partial, cnt, empty_slot, *fuse);
    else if (mode == PASS_UPDATE)
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_UPDATE, false>), dim3(grid), dim3(PASS_THREADS),
                           pass_lds_bytes(h.lp, false), s, S, h.R, h.lp, partial, cnt, empty_slot,
                           fuse ? *fuse : none);
    else if (mode == PASS_QUERY)
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_QUERY, false>), dim3(grid), dim3(PASS_THREADS),
                           pass_lds_bytes(h.lp, false), s, S, h.R, h.lp, partial, cnt, empty_slot, none);
    else
        hipLaunchKernelGGL((pass_kernel<T, RR, PASS_INIT, false>), dim3(grid), dim3(PASS_THREADS),
                           pass_lds_bytes(h.lp, false), s, S, h.R, h.lp, partial, cnt, empty_slot, none);
    if (reduce_after)
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((stride + 63) / 64), dim3(1024), 0, s, partial, grid, stride,
                           h.lp, S.acc_out, qout, S.shift_self, mode);
    return hipGetLastError();
}

template <int T>
static hipError_t launch_pass_t(const PassSide &S, const Handle &h, int side, int mode, const FuseArgs *fuse,
                                bool fused_in, bool reduce_after, double *partial, unsigned long long *cnt,
                                hipStream_t s)
{
    if (h.R <= 4) return launch_pass_tr<T, 4>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
    return launch_pass_tr<T, 8>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
}

// side 0: rows of X (updates u, consumes y = W v, produces z = U^T u); side 1: rows of Y.
// acc_in / acc_out index the accumulator buffers (-1: none).
static PassSide make_side(const Handle &h, int side, int acc_in, int acc_out, float *marg_out)
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
        S.rows_in = h.m;
    } else {
        S.rows = h.m;
        S.F = h.Wt;
        S.vals = h.vals_y;
        S.meta = h.sort.meta_y;
        S.log_out = h.log_v;
        S.lin_out = h.lin_v;
        S.perm_out = h.perm_v;
        S.perm_in = h.perm_u;
        S.rows_in = h.n;
    }
    S.acc_in = acc_in >= 0 ? h.acc[acc_in] : nullptr;
    S.acc_out = acc_out >= 0 ? h.acc[acc_out] : nullptr;
    S.marg_out = marg_out;
    S.meta_stride = h.sort.meta_stride;
    S.shift_self = h.shift + side;
    return S;
}

static hipError_t launch_logpass(const PassSide &S, const Handle &h, int side, int mode, hipStream_t s)
{
    long long g = (S.rows + PASS_WAVES - 1) / PASS_WAVES;
    const int grid = (int)(g < h.grid ? g : h.grid);
    const int empty_slot = 1 + side;
    if (h.mode == LCN_MODE_DENSE && mode != PASS_INIT) {
        const long long gd = (S.rows + DENSE_ROWS - 1) / DENSE_ROWS;
        // a query leaves 3 partial sums per workgroup and there is room for h.grid of them; an update
        // leaves none and may fill every compute unit with eight of these small workgroups
        const long long cap = mode == PASS_QUERY ? (long long)h.grid : 8ll * (h.cus > 0 ? h.cus : 256);
        const int dgrid = (int)(gd < cap ? gd : cap);
        if (mode == PASS_UPDATE)
            hipLaunchKernelGGL(logpass_dense_kernel<PASS_UPDATE>, dim3(dgrid), dim3(64 * DENSE_WAVES), 0, s, S, h.partial,
                               h.counters, empty_slot);
        else
            hipLaunchKernelGGL(logpass_dense_kernel<PASS_QUERY>, dim3(dgrid), dim3(64 * DENSE_WAVES), 0, s, S, h.partial,
                               h.counters, empty_slot);
        if (mode == PASS_QUERY)
            hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(1024), 0, s, h.partial, dgrid, 3, 0, S.acc_out,
                               h.query_out + 2 * side, S.shift_self, mode);
        return hipGetLastError();
    }
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

// workgroups of a sweep over `rows` rows (= partial sums it leaves)
static int sweep_groups(const Handle &h, long long rows)
{
    const long long g = (rows + PASS_WAVES - 1) / PASS_WAVES;
    return (int)(g < h.grid ? g : h.grid);
}

static hipError_t dispatch_pass(const PassSide &S, const Handle &h, int side, int mode, const FuseArgs *fuse,
                                bool fused_in, bool reduce_after, double *partial, hipStream_t s,
                                unsigned long long *cnt = nullptr)
{
    if (!cnt) cnt = h.counters;
    switch (h.lp / 64) {
        case 0: return launch_pass_t<0>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 1: return launch_pass_t<1>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 2: return launch_pass_t<2>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 3: return launch_pass_t<3>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 4: return launch_pass_t<4>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 5: return launch_pass_t<5>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 6: return launch_pass_t<6>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 7: return launch_pass_t<7>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        case 8: return launch_pass_t<8>(S, h, side, mode, fuse, fused_in, reduce_after, partial, cnt, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_pass(const Handle &h, int side, int mode, int acc_in, int acc_out, float *marg_out, hipStream_t s)
{
    const PassSide S = make_side(h, side, acc_in, acc_out, marg_out);
    if (h.log_domain) return launch_logpass(S, h, side, mode, s);
    return dispatch_pass(S, h, side, mode, nullptr, false, true, h.partial, s);
}

// `iters` iterations = 2 iters update sweeps (rows of X, then rows of Y).  With
// fused reduction every sweep but the first adds up its predecessor's partial
// sums itself (two partial buffers alternate) and one reduction launch at the end
// completes the state; otherwise every sweep is followed by its reduction launch.
//
// A state that has not been iterated yet (after the build or after new scalings
// were set) has exponents that say nothing about the vectors the first sweeps
// produce: from u = v = 1 the first u is of the order of 1 / (K 1), possibly
// e^(+-hundreds).  For such a state each side's first sweep is run twice: once
// only to learn the largest log of its result (everything else it writes is
// overwritten, its fault counts go to slots nobody reads), then for real with
// that exponent.  From then on a vector's exponent is its largest log one
// iteration earlier, and logs move little per iteration.
hipError_t launch_update_sweeps(Handle &h, int iters, hipStream_t s)
{
    // a sweep's first ceil((lp + 3) / 64) workgroups add up its predecessor's partial sums: a side with
    // fewer workgroups than that (a handful of rows) cannot, and every sweep gets its reduction launch
    const int reducers = (h.lp + 3 + 63) / 64;
    const bool fused = h.fused_reduce && !h.log_domain && sweep_groups(h, h.n) >= reducers &&
                       sweep_groups(h, h.m) >= reducers;
    int first = 0;
    if (h.fresh && h.double_first && !h.log_domain && iters > 0) {
        unsigned long long *discard = h.counters + 8;
        const PassSide SX = make_side(h, 0, 0, 1, nullptr), SY = make_side(h, 1, 1, 0, nullptr);
        hipError_t e = dispatch_pass(SX, h, 0, PASS_UPDATE, nullptr, false, true, h.partial, s, discard);
        if (e == hipSuccess) e = dispatch_pass(SX, h, 0, PASS_UPDATE, nullptr, false, true, h.partial, s);
        if (e == hipSuccess) e = dispatch_pass(SY, h, 1, PASS_UPDATE, nullptr, false, true, h.partial, s, discard);
        if (e != hipSuccess) return e;
        first = 1;   // the loop below starts with the sweep over Y, now with its exponent known
    }
    h.last_launches = 2 * iters + (first ? 2 : 0);   // half-iteration launches of this run, the repeated ones included
    if (iters > 0) h.fresh = 0;
    for (int t = first; t < 2 * iters; ++t) {
        const int side = t & 1;
        const PassSide S = make_side(h, side, side == 0 ? 0 : 1, side == 0 ? 1 : 0, nullptr);
        hipError_t e;
        if (h.log_domain) {
            e = launch_logpass(S, h, side, PASS_UPDATE, s);
        } else if (!fused) {
            e = dispatch_pass(S, h, side, PASS_UPDATE, nullptr, false, true, h.partial, s);
        } else {
            double *mine = (t & 1) ? h.partial2 : h.partial;
            const bool last = t == 2 * iters - 1;
            if (t == first) {
                // not fused itself, but its successor reduces into this sweep's output accumulator
                FuseArgs F{};
                F.mark_pending = last ? nullptr : h.acc[side == 0 ? 1 : 0];
                e = dispatch_pass(S, h, side, PASS_UPDATE, &F, false, last, mine, s);
            } else {
                const long long rows_prev = side == 0 ? h.m : h.n;
                FuseArgs F;
                F.prev_partial = (t & 1) ? h.partial : h.partial2;
                F.prev_groups = sweep_groups(h, rows_prev);
                F.acc = h.acc[side == 0 ? 0 : 1];
                F.shift_other = h.shift + (1 - side);
                F.shift_self = h.shift + side;
                F.mark_pending = last ? nullptr : h.acc[side == 0 ? 1 : 0];
                F.timeouts = h.counters + 5;
                F.wait_ticks = h.wait_ticks;
                e = dispatch_pass(S, h, side, PASS_UPDATE, &F, true, last, mine, s);
            }
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lcn
