// Device helpers shared by the two half-iteration kernels (one row per
// wavefront, and four rows per wavefront): cross-lane sums, the short log and
// reciprocal used by the scaling update, the factor-row register layout and the
// in-kernel completion of the previous sweep's reduction.
#pragma once

#include "lcn_internal.h"

namespace lcn {

constexpr int PASS_THREADS = 1024;
constexpr int PASS_WAVES = PASS_THREADS / 64;
constexpr int MAXR = 8;
// what the single-precision bucket-ordered copies of a scaling vector are stored times, and its inverse
constexpr double PERM_SCALE = 18446744073709551616.0;          // 2^64
constexpr double PERM_UNSCALE = 1.0 / 18446744073709551616.0;  // 2^-64
#ifndef PASS_MIN_WAVES
#define PASS_MIN_WAVES 1
#endif

// One step of a cross-lane sum of doubles through the DPP data path (no LDS):
// adds to every lane the value of the lane that `CTRL` selects; lanes of rows
// outside ROW_MASK add zero.  With a full row mask every lane receives a value,
// so the destination needs no initial value.
template <int CTRL, int ROW_MASK>
__device__ inline double dpp_add(double v)
{
    const int lo = __double2loint(v), hi = __double2hiint(v);
    int plo, phi;
    if (ROW_MASK == 0xF) {
        plo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xF, 0xF, false);
        phi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xF, 0xF, false);
    } else {
        plo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xF, false);
        phi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xF, false);
    }
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
        F += row * lp;
        if (VEC) {
#pragma unroll
            for (int q = 0; q < T / 4; ++q) {
                const float4 v = *(const float4 *)(F + (unsigned)(256 * q + 4 * lane));
                f[4 * q + 0] = v.x;
                f[4 * q + 1] = v.y;
                f[4 * q + 2] = v.z;
                f[4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int t = 0; t < TT; ++t) f[t] = F[(unsigned)(64 * t + lane)];
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
    // the records are written once at build time: reading them through the constant
    // address space lets the compiler use scalar loads although the kernel also stores
    typedef const __attribute__((address_space(4))) int *const_int_ptr;
    const_int_ptr rec = (const_int_ptr)(S.meta + row * S.meta_stride);
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

// A sweep that finishes the previous sweep's reduction itself passes the totals
// from the reducing workgroups to all others through the accumulator itself:
// the sweep before filled the accumulator with ACC_PENDING (a NaN bit pattern no
// arithmetic produces), the reducing workgroups overwrite it with device-scope
// stores, and a reader simply re-reads (device scope) until no entry is pending.
// No flag and no fence is involved, so a hand-over costs one store and one load
// through memory.
constexpr unsigned long long ACC_PENDING = 0x7FF8A5A55A5AC3C3ull;

struct FuseArgs {
    const double *prev_partial;  // [prev_groups][lp + 3] partial sums the previous sweep left
    int prev_groups;
    double *acc;                 // where the totals go: this sweep's input accumulator (lp + 2 entries)
    double *shift_other;         // exponent of the other side's vector (the previous sweep's own)
    const double *shift_self;    // exponent of this side's vector
    double *mark_pending;        // accumulator the NEXT sweep reduces into (nullable): filled with ACC_PENDING
    unsigned long long *timeouts;
    unsigned long long wait_ticks;  // how long a workgroup re-reads pending totals before it gives up (100 MHz clock)
};

// Marks the accumulator that the next sweep will fill as pending (one wavefront of
// one workgroup; ordinary stores, visible to the next launch).
__device__ inline void mark_pending(const FuseArgs &Fz, int lp)
{
    if (Fz.mark_pending && blockIdx.x == gridDim.x - 1 && threadIdx.x < 64)
        for (int k = threadIdx.x; k <= lp + 1; k += 64) ((unsigned long long *)Fz.mark_pending)[k] = ACC_PENDING;
}

// The sum of the per-workgroup partials in the fixed order of
// reduce_partials_kernel (bitwise the same result), by workgroup `b` for its 64
// entries, published with device-scope stores.  Nothing here waits, so a
// reducing workgroup always gets through.
__device__ inline void reduce_publish(const FuseArgs &Fz, int b, int lp, double *red)
{
    double *acc = Fz.acc;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int stride = lp + 3;
    const int k = b * 64 + lane;
    const bool is_max = k == lp + 2;
    // 16 running sums as in reduce_partials_kernel (sum a takes partials a, a + 16, ...),
    // shared out among the wavefronts this workgroup has
    for (int a = wave; a < 16; a += nw) {
        double s = is_max ? -INFINITY : 0.0;
        if (k < stride) {
#pragma unroll 16
            for (int g = a; g < Fz.prev_groups; g += 16) {
                const double v = Fz.prev_partial[(long long)g * stride + k];
                s = is_max ? fmax(s, v) : s + v;
            }
        }
        red[a * 64 + lane] = s;
    }
    __syncthreads();
    if (wave == 0 && k < stride) {
        double s = is_max ? -INFINITY : 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) s = is_max ? fmax(s, red[w * 64 + lane]) : s + red[w * 64 + lane];
        if (k < lp) {
            __hip_atomic_store(acc + k, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else if (is_max) {
            // the exponent the previous sweep's vector was stored with, and the factor
            // exp(-m_in - m_self) this sweep applies to its results
            const double m_in = *Fz.shift_other;
            __hip_atomic_store(acc + lp, m_in, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(acc + lp + 1, exp(-m_in - *Fz.shift_self), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            *Fz.shift_other = (s > -INFINITY && s < INFINITY) ? s : 0.0;
        }
    }
}

// Reads the totals (lp + 2 doubles) into `ysh`, re-reading until the reducing
// workgroups of this launch have replaced every pending entry (bounded wait).
// Called by one wavefront of every workgroup; the caller synchronises the
// workgroup afterwards.
__device__ inline void fused_fetch(const FuseArgs &Fz, const double *acc, int lp, double *ysh)
{
    const int lane = threadIdx.x & 63;
    const unsigned long long *src = (const unsigned long long *)acc;
    // once a wait has timed out no later wait is attempted (the run is reported as failed)
    bool give_up = __hip_atomic_load(Fz.timeouts, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull;
    const unsigned long long t0 = wall_clock64();
    for (;;) {
        bool pending = false;
        for (int k = lane; k <= lp + 1; k += 64) {
            const unsigned long long v = __hip_atomic_load(src + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            pending |= v == ACC_PENDING;
            ((unsigned long long *)ysh)[k] = v;
        }
        if (!__any(pending) || give_up) break;
        if (wall_clock64() - t0 > Fz.wait_ticks) {
            if (lane == 0) atomicAdd(Fz.timeouts, 1ull);
            give_up = true;
        }
    }
}

}  // namespace lcn
