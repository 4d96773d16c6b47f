// k-means assignment as an MFMA distance GEMM used as a *filter*.
//
// The bucket of a point is defined by an exact fp64 rule (see
// kernels_structure.hip).  Evaluating that rule for every (point, centroid)
// pair is ALU bound; here the scores  ||c||^2 - 2 z.c  are computed on the
// matrix cores, which ranks the centroids of a point up to a rounding bound
// delta.  If the two best scores of a point are further apart than 2 delta,
// the best one is also the exact rule's answer; otherwise the point is put on a
// list and decided by the exact rule.
//
// Arithmetic: every fp32 value is split into bf16 planes, x = x1 + x2 + r with
// x1 = bf16(x), x2 = bf16(x - x1), |r| <= 2^-16 |x|, and the dot product is
// taken as  z1.c1 + z1.c2 + z2.c1  with v_mfma_f32_32x32x16_bf16 (products of
// bf16 values are exact in the fp32 accumulators): three bf16 instructions do
// the work of eight fp32 ones (v_mfma_f32_32x32x2f32) at sixteen times their
// rate.  Inputs that were given as bf16 have z2 = 0 and need two products.
//
// Layout: the planes are stored in the order the instruction wants its
// operands.  For a group of 32 rows (points or centroids) and a step of 16
// dimensions, lane l holds row l % 32, dimensions 8 (l / 32) .. + 7: one
// 16-byte piece per lane, 1 KB per (group, step), so an operand is ONE fully
// coalesced 16-byte load per lane, from global memory (points: private to a
// wavefront, read once per pass over the centroids) or from LDS (centroids:
// shared by the four wavefronts of a workgroup, staged two steps at a time
// through two buffers).
//
// Tiling for 64-wide wavefronts: a workgroup of 4 waves takes 128 points and
// walks over the centroids 128 at a time; each wave owns 32 points (the N side
// of the instruction) and 4 x 32 centroids (the M side), i.e. four 32x32
// accumulator tiles.  With centroids on M a lane holds 16 centroids of ONE
// point per tile, so the running arg-min needs no cross-lane work until the two
// half-waves are merged at the end.
#include <mutex>

#include "lcn_internal.h"

namespace lcn {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

// bf16 of a finite float, round to nearest even: |x - bf16(x)| <= 2^-8 |x|
__device__ inline unsigned bf16_bits(float x)
{
    const unsigned u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

constexpr int FP = 128;  // points per workgroup
constexpr int FC = 128;  // centroids per pass

static inline int steps_of(int d) { return (d + 15) / 16; }

// With more than 256 centroids a thread of the exact list kernel walks several chains of d
// dependent additions; then it pays to separate the points that have just two candidates.
bool filter_uses_pairs(int k) { return k > 256; }

size_t split_plane_bytes(long long rows, int d)
{
    return (size_t)((rows + 31) / 32) * (size_t)steps_of(d) * 1024;
}

// Splits the rows of `src` (rows x d, fp32) into `planes` bf16 planes in operand
// order: out[plane][group][step][lane] (16 bytes each); rows and dimensions
// beyond the matrix are zero.  One workgroup per group of 32 rows.
// NORMS (the centroids): also the squared norm of every row as fp32 into cn, and the
// largest of them into cmax_bits (the bit pattern of a non-negative float orders like an
// unsigned integer; cmax_bits is zero on entry).
template <bool NORMS>
__global__ __launch_bounds__(256) void split_planes_kernel(const float *__restrict__ src, long long rows, int d, int S,
                                                           int planes, bf16x8 *__restrict__ out, long long plane_stride,
                                                           float *__restrict__ cn, unsigned *cmax_bits)
{
    __shared__ double red[4][32];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long long group = blockIdx.x;
    const long long row = group * 32 + (lane & 31);
    double sq = 0.0;
    for (int s = w; s < S; s += 4) {
        const int k0 = 16 * s + 8 * (lane >> 5);
        u16x8 p1, p2;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x = (row < rows && k0 + e < d) ? src[row * d + k0 + e] : 0.f;
            if (NORMS) sq = fma((double)x, (double)x, sq);
            const unsigned h = bf16_bits(x);
            p1[e] = (unsigned short)h;
            p2[e] = (unsigned short)bf16_bits(x - __uint_as_float(h << 16));  // the difference is exact in fp32
        }
        const long long at = (group * S + s) * 64 + lane;
        out[at] = __builtin_bit_cast(bf16x8, p1);
        if (planes > 1) out[plane_stride + at] = __builtin_bit_cast(bf16x8, p2);
    }
    if (NORMS) {
        sq += __shfl_xor(sq, 32, 64);   // the two halves of a row's 16 dimensions per step
        if (lane < 32) red[w][lane] = sq;
        __syncthreads();
        if (w == 0 && lane < 32 && row < rows) {
            const float f = (float)(red[0][lane] + red[1][lane] + red[2][lane] + red[3][lane]);
            cn[row] = f;
            atomicMax(cmax_bits, __float_as_uint(f * 1.0000002f));
        }
    }
}

hipError_t launch_split_planes(const float *src, long long rows, int d, int planes, void *out, hipStream_t s)
{
    const long long groups = (rows + 31) / 32;
    const int S = steps_of(d);
    hipLaunchKernelGGL(split_planes_kernel<false>, dim3((unsigned)groups), dim3(256), 0, s, src, rows, d, S, planes,
                       (bf16x8 *)out, (long long)(split_plane_bytes(rows, d) / 16), (float *)nullptr,
                       (unsigned *)nullptr);
    return hipGetLastError();
}

// What the filter makes of a point's three smallest scores.
// |score - exact score| <= delta = err_coef (||z||^2 + max ||c||^2), see launch_assign_filter.
// The exact rule's winner scores at most best + 2 delta, so:
//   second beyond that      -> bidx is the winner;
//   only third beyond that  -> the winner is bidx or sidx (decided by the exact rule on those two);
//   otherwise               -> the exact rule over all centroids.
template <bool TOP3>
__device__ inline void filter_decide(long long p, float best, float second, float third, int bidx, int sidx,
                                     const double *__restrict__ zn, const unsigned *__restrict__ cmax_bits,
                                     float err_coef, int32_t *__restrict__ out, int *__restrict__ flagged,
                                     int *__restrict__ pairs, int *nflagged)
{
    out[p] = bidx;
    const float cmax = __uint_as_float(*cmax_bits);
    const float delta = err_coef * ((float)zn[p] * 1.0000002f + cmax);
    if (!(second - best > 2.f * delta)) {
        if (TOP3 && third - best > 2.f * delta) {
            const int slot = atomicAdd(nflagged + 1, 1);
            pairs[3 * (long long)slot] = (int)p;
            pairs[3 * (long long)slot + 1] = bidx;
            pairs[3 * (long long)slot + 2] = sidx;
        } else {
            const int slot = atomicAdd(nflagged, 1);
            flagged[slot] = (int)p;
        }
    }
}

// ZP: planes of the points (2: fp32 input, 1: input exactly representable in bf16).
// TOP3: also track the third smallest score and the second's centroid, so that a point
// with exactly two candidates goes to the exact rule on those two; pays off when the
// exact rule over all centroids is long (many centroids).
template <int ZP, bool TOP3>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void assign_filter_kernel(const bf16x8 *__restrict__ Zt, long long zplane, long long N,
                                                            int S, const bf16x8 *__restrict__ Ct, long long cplane,
                                                            int k, const float *__restrict__ cn,
                                                            const double *__restrict__ zn,
                                                            const unsigned *__restrict__ cmax_bits, float err_coef,
                                                            int32_t *__restrict__ out, int *__restrict__ flagged,
                                                            int *__restrict__ pairs, int *nflagged)
{
    // [buffer][step of the stage][centroid group][plane][lane]: 32 KB
    __shared__ bf16x8 Cs[2][2][4][2][64];
    __shared__ float cn_s[FC];  // squared norms of the pass's centroids (+inf beyond the last one)
    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const long long ngroups = (N + 31) / 32;
    long long P = (long long)blockIdx.x * (FP / 32) + w;  // the wave's group of 32 points
    const bool active = P < ngroups;
    if (!active) P = ngroups - 1;  // idle waves of the last workgroup repeat a group and write nothing
    const bf16x8 *__restrict__ zsrc = Zt + P * S * 64 + lane;
    const int cgroups = (k + 31) / 32;
    const int nstage = (S + 1) / 2;
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = (__bf16)0.f;

    // the three smallest scores of the lane's point so far, with the centroids of the first two
    float best = INFINITY, second = INFINITY, third = INFINITY;
    int bidx = 0, sidx = 0;
    // (kept sorted: the new smallest is the median of (-inf, best, s), the new second that of
    // (best, second, s), the new third that of (second, third, s); plain selects, no branch)
    auto offer = [&](float s, int c) {
        const bool lt1 = s < best;
        if (TOP3) {
            const bool lt2 = s < second;
            const int keep = lt2 ? c : sidx;
            third = __builtin_amdgcn_fmed3f(second, third, s);
            sidx = lt1 ? bidx : keep;
        }
        second = __builtin_amdgcn_fmed3f(best, second, s);
        bidx = lt1 ? c : bidx;
        best = __builtin_amdgcn_fmed3f(-INFINITY, best, s);
    };

    for (int c0 = 0; c0 < k; c0 += FC) {
        floatx16 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

        // A stage is 16 pieces of 1 KB: (step ks, centroid group t, plane pl); thread tid
        // fetches lane tid % 64 of pieces tid / 64 + 4 j.
        bf16x8 creg[4];
        auto fetch_c = [&](int stage) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int piece = w + 4 * j;
                const int ks = piece >> 3, t = (piece >> 1) & 3, pl = piece & 1;
                // unconditional: a step past the last repeats the last (the points' operand is zero there),
                // a group past the last repeats the last (its scores are masked by a norm of +inf)
                const int s = 2 * stage + ks < S ? 2 * stage + ks : S - 1;
                const int cg = c0 / 32 + t < cgroups ? c0 / 32 + t : cgroups - 1;
                creg[j] = Ct[pl * cplane + ((long long)cg * S + s) * 64 + lane];
            }
        };
        auto store_c = [&](int buf) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int piece = w + 4 * j;
                Cs[buf][piece >> 3][(piece >> 1) & 3][piece & 1][lane] = creg[j];
            }
        };
        bf16x8 zcur[2][ZP], znext[2][ZP];
        auto fetch_z = [&](int stage, bf16x8 (&dst)[2][ZP]) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int s = 2 * stage + ks;
#pragma unroll
                for (int pl = 0; pl < ZP; ++pl) {
                    const bf16x8 v = zsrc[pl * zplane + (long long)(s < S ? s : S - 1) * 64];   // unconditional
                    dst[ks][pl] = s < S ? v : zero;
                }
            }
        };
        __syncthreads();  // the previous pass has finished reading the buffers
        if (tid < FC) cn_s[tid] = c0 + tid < k ? cn[c0 + tid] : INFINITY;
        fetch_c(0);
        fetch_z(0, zcur);
        store_c(0);
        __syncthreads();
        for (int i = 0; i < nstage; ++i) {
            const int buf = i & 1;
            if (i + 1 < nstage) {
                fetch_c(i + 1);
                fetch_z(i + 1, znext);
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bf16x8 c1 = Cs[buf][ks][t][0][lane];
                    const bf16x8 c2 = Cs[buf][ks][t][1][lane];
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c1, zcur[ks][0], acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c2, zcur[ks][0], acc[t], 0, 0, 0);
                    if (ZP > 1) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c1, zcur[ks][ZP - 1], acc[t], 0, 0, 0);
                }
            }
            if (i + 1 < nstage) {
                store_c(buf ^ 1);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int pl = 0; pl < ZP; ++pl) zcur[ks][pl] = znext[ks][pl];
            }
            __syncthreads();
        }
        // scores of this pass's centroids for the lane's point; element v of tile t is
        // centroid row (v / 4) * 8 + half * 4 + v % 4 of the tile (a centroid beyond the
        // last one scores +inf and never wins)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int cl = t * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                offer(fmaf(-2.f, acc[t][v], cn_s[cl]), c0 + cl);
            }
    }
    // merge the two half-waves that share a point: the other half's three smallest are offered in turn
    {
        const float ob = __shfl_xor(best, 32, 64), os = __shfl_xor(second, 32, 64), ot = __shfl_xor(third, 32, 64);
        const int oi = __shfl_xor(bidx, 32, 64), osi = __shfl_xor(sidx, 32, 64);
        offer(ob, oi);
        offer(os, osi);
        offer(ot, 0);  // cannot rank above third: two scores of the other half are not larger
    }
    const long long p = P * 32 + col;
    if (active && half == 0 && p < N)
        filter_decide<TOP3>(p, best, second, third, bidx, sidx, zn, cmax_bits, err_coef, out, flagged, pairs, nflagged);
}

// The filter for points given as bf16 (one plane) against many centroids: the 128 points of a
// workgroup stay in LDS for the whole launch (4 S KB, read from memory once instead of once per 128
// centroids), and the roles of the four wavefronts are turned round: a wavefront takes ALL 128
// points (four accumulator tiles, one per group of 32 points) against ONE group of 32 centroids per
// pass, whose operands it reads from memory (the cache: every workgroup streams the same 2 k S KB)
// straight into registers, a few steps ahead in a ring of registers.  Per step a wavefront reads
// four operands from LDS and two from memory for eight matrix instructions -- half the LDS traffic
// of the kernel above, and nothing in the loop waits for the workgroup.  Every load is
// unconditional (indices beyond the end are clamped; what they fetch is not used), so the waits
// count exactly the loads that must have landed.  A lane tracks the smallest scores of four
// points, over the centroids its wavefront saw; half-wavefronts and wavefronts are merged at the end.
constexpr int FR_MERGE_BYTES = 4 * FP * 5 * 4;

template <bool TOP3>
__global__ __launch_bounds__(256, 2) void assign_filter_resident_kernel(
    const bf16x8 *__restrict__ Zt, long long N, int S, const bf16x8 *__restrict__ Ct, long long cplane, int k,
    const float *__restrict__ cn, const double *__restrict__ zn, const unsigned *__restrict__ cmax_bits, float err_coef,
    int32_t *__restrict__ out, int *__restrict__ flagged, int *__restrict__ pairs, int *nflagged)
{
    extern __shared__ __align__(16) unsigned char fr_lds[];
    bf16x8 *Zs = reinterpret_cast<bf16x8 *>(fr_lds);   // [4 point groups][S][64]
    const int tid = threadIdx.x;
    const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const long long ngroups = (N + 31) / 32;
    const long long G0 = (long long)blockIdx.x * 4;
    {   // wavefront w brings in point group G0 + w (the last workgroup repeats the last group)
        const long long gl = G0 + w < ngroups ? G0 + w : ngroups - 1;
        const bf16x8 *__restrict__ src = Zt + gl * S * 64 + lane;
        bf16x8 *dst = Zs + (size_t)w * S * 64 + lane;
        for (int s0 = 0; s0 < S; s0 += 8) {
            bf16x8 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = src[(long long)(s0 + u < S ? s0 + u : S - 1) * 64];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < S) dst[(s0 + u) * 64] = t[u];
        }
    }
    __syncthreads();

    const int cgroups = (k + 31) / 32, npass = (k + FC - 1) / FC;
    // Steps a centroid operand is requested ahead.  Two is enough and best: what bounds the stream is not
    // its latency but the first-level cache, which holds fewer lines than eight wavefronts can ask for
    // (a ring of 4, 6, 8 steps measured 2 %, 11 %, 7 % slower; a pass is padded to whole turns).
    constexpr int RING = 2;
    const int SP = (S + RING - 1) / RING * RING;  // a pass in whole turns of the ring; steps S .. SP - 1 multiply nothing
    // where the next request of the ring goes: pass lp (its centroid group's first operand at lbase), step ls
    // Workgroups take the passes in rotated order (workgroup b starts with pass b mod npass): all of
    // them stream the same operands at the same pace, and in the same order they would all ask the
    // same few cache channels at once.
    const int rot = (int)(blockIdx.x % (unsigned)npass);
    auto pass_of = [&](int i) {
        i = i < npass ? i : npass - 1;   // past the last pass: its operands once more, unused
        i += rot;
        return i < npass ? i : i - npass;
    };
    auto group_base = [&](int i) {
        const int pass = pass_of(i);
        int cg = 4 * pass + w;
        cg = cg < cgroups ? cg : cgroups - 1;
        return Ct + (long long)cg * S * 64 + lane;
    };
    int lp = 0, ls = 0;
    const bf16x8 *__restrict__ lbase = group_base(0);
    auto request = [&](bf16x8 &d1, bf16x8 &d2) {
        const bf16x8 *cp = lbase + (ls < S ? ls : S - 1) * 64;
        d1 = cp[0];
        d2 = cp[cplane];
        if (++ls == SP) {   // the same in every lane; nothing is loaded inside
            ls = 0;
            lbase = group_base(++lp);
        }
    };
    float best[4], second[4], third[4];
    int bidx[4], sidx[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        best[g] = second[g] = third[g] = INFINITY;
        bidx[g] = sidx[g] = 0;
    }
    bf16x8 r1[RING], r2[RING];   // the ring: the centroid group's two planes for the next RING steps
#pragma unroll
    for (int u = 0; u < RING; ++u) request(r1[u], r2[u]);
    // the points' operands of a step are read from LDS one step ahead, into two sets of registers in turn
    bf16x8 za[4], zb[4];
    auto zread = [&](bf16x8 (&z)[4], int step) {
        const int sz = step < S ? step : S - 1;
#pragma unroll
        for (int g = 0; g < 4; ++g) z[g] = Zs[((size_t)g * S + sz) * 64 + lane];
    };
    zread(za, 0);
    for (int pi = 0; pi < npass; ++pi) {
        const int pass = pass_of(pi);
        // squared norms of the lane's sixteen centroids of this pass (+inf beyond the last centroid:
        // such a row repeats the last group's operands and never wins)
        float cnv[16];
        const int cbase = FC * pass + 32 * w + 4 * half;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ci = cbase + 8 * q + j;
                const float v = cn[ci < k ? ci : k - 1];
                cnv[4 * q + j] = ci < k ? v : INFINITY;
            }
        floatx16 acc[4];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[g][v] = 0.f;
        for (int s0 = 0; s0 < SP; s0 += RING) {
#pragma unroll
            for (int u = 0; u < RING; ++u) {
                const int st = s0 + u;
                bf16x8(&zc)[4] = (u & 1) ? zb : za;
                bf16x8(&zn)[4] = (u & 1) ? za : zb;
                zread(zn, st + 1 < SP ? st + 1 : 0);   // after a pass's last step comes the next pass's first
                const bf16x8 a1 = r1[u], a2 = r2[u];
                if (st < S) {   // the same in every lane; no load inside
#pragma unroll
                    for (int g = 0; g < 4; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, zc[g], acc[g], 0, 0, 0);
#pragma unroll
                    for (int g = 0; g < 4; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, zc[g], acc[g], 0, 0, 0);
                }
                request(r1[u], r2[u]);
            }
        }
        // element v of tile g: centroid row (v / 4) * 8 + half * 4 + v % 4 of the wavefront's group, for
        // point column `col` of point group g.  The three smallest stay sorted: the new smallest is the
        // median of (-inf, best, score), the new second that of (best, second, score), the new third
        // that of (second, third, score).  A centroid is remembered as 16 pass + v (a scalar) and
        // turned into its index at the end.
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float b = best[g], s2 = second[g], t3 = third[g];
            int bi = bidx[g], si = sidx[g];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float sc = fmaf(-2.f, acc[g][v], cnv[v]);
                const int code = 16 * pass + v;
                const bool lt1 = sc < b;
                if (TOP3) {
                    const bool lt2 = sc < s2;
                    const int keep = lt2 ? code : si;
                    t3 = __builtin_amdgcn_fmed3f(s2, t3, sc);
                    si = lt1 ? bi : keep;
                }
                s2 = __builtin_amdgcn_fmed3f(b, s2, sc);
                bi = lt1 ? code : bi;
                b = __builtin_amdgcn_fmed3f(-INFINITY, b, sc);
            }
            best[g] = b, second[g] = s2, third[g] = t3;
            bidx[g] = bi, sidx[g] = si;
        }
    }
    // from 16 pass + v to the centroid's index
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        bidx[g] = FC * (bidx[g] >> 4) + 32 * w + 4 * half + ((bidx[g] >> 2) & 3) * 8 + (bidx[g] & 3);
        sidx[g] = FC * (sidx[g] >> 4) + 32 * w + 4 * half + ((sidx[g] >> 2) & 3) * 8 + (sidx[g] & 3);
    }
    // merge: the other half-wavefront's three smallest are offered in turn (the third cannot rank
    // above third: two scores of its own set are not larger), then the four wavefronts' through LDS
    auto offer = [&](float &b, float &s2, float &t3, int &bi, int &si, float sc, int c) {
        const bool lt1 = sc < b, lt2 = sc < s2;
        if (TOP3) {
            t3 = fminf(t3, fmaxf(sc, s2));
            si = lt1 ? bi : (lt2 ? c : si);
        }
        s2 = fminf(s2, fmaxf(sc, b));
        bi = lt1 ? c : bi;
        b = fminf(b, sc);
    };
    __syncthreads();   // every wavefront has finished reading the points
    float *mf = reinterpret_cast<float *>(fr_lds);             // [3][4 wavefronts][128 points]
    int *mi = reinterpret_cast<int *>(fr_lds) + 3 * 4 * FP;     // [2][4][128]
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const float ob = __shfl_xor(best[g], 32, 64), os = __shfl_xor(second[g], 32, 64),
                    ot = __shfl_xor(third[g], 32, 64);
        const int oi = __shfl_xor(bidx[g], 32, 64), osi = __shfl_xor(sidx[g], 32, 64);
        offer(best[g], second[g], third[g], bidx[g], sidx[g], ob, oi);
        offer(best[g], second[g], third[g], bidx[g], sidx[g], os, osi);
        offer(best[g], second[g], third[g], bidx[g], sidx[g], ot, 0);
        if (half == 0) {
            const int pt = 32 * g + col;
            mf[(0 * 4 + w) * FP + pt] = best[g];
            mf[(1 * 4 + w) * FP + pt] = second[g];
            mf[(2 * 4 + w) * FP + pt] = third[g];
            mi[(0 * 4 + w) * FP + pt] = bidx[g];
            mi[(1 * 4 + w) * FP + pt] = sidx[g];
        }
    }
    __syncthreads();
    if (tid < FP) {
        const long long p = G0 * 32 + tid;
        if (p < N) {
            float b = INFINITY, s2 = INFINITY, t3 = INFINITY;
            int bi = 0, si = 0;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                offer(b, s2, t3, bi, si, mf[(0 * 4 + ww) * FP + tid], mi[(0 * 4 + ww) * FP + tid]);
                offer(b, s2, t3, bi, si, mf[(1 * 4 + ww) * FP + tid], mi[(1 * 4 + ww) * FP + tid]);
                offer(b, s2, t3, bi, si, mf[(2 * 4 + ww) * FP + tid], 0);
            }
            filter_decide<TOP3>(p, b, s2, t3, bi, si, zn, cmax_bits, err_coef, out, flagged, pairs, nflagged);
        }
    }
}

// More than 64 KB of dynamic LDS has to be allowed per kernel and device before the first such launch.
// Done once per device and kernel (and again only for a larger size), under a lock: the k-means runs
// of a build launch from several host threads.
static hipError_t allow_dynamic_lds(const void *kernel, int which, size_t bytes)
{
    static std::mutex mu;
    static size_t allowed[64][2] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    std::lock_guard<std::mutex> lock(mu);
    if (allowed[dev][which] >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) allowed[dev][which] = bytes;
    return e;
}

// Zt: the points' planes (launch_split_planes, `zplanes` of them); Ct: room for two planes of k centroids.
// flagged: points for the exact rule over all centroids (count nflagged[0]); pairs: (point, centroid, centroid)
// triples for the exact rule on two centroids (count nflagged[1]).
hipError_t launch_assign_filter(const void *Zt, int zplanes, long long N, int d, const float *cent, int k, void *Ct,
                                const double *zn, float *cn, unsigned *cmax_bits, int32_t *out, int *flagged,
                                int *pairs, int *nflagged, hipStream_t s)
{
    // cmax_bits and nflagged[0..1] are zero on entry: cleared by the caller before the first
    // call and by the centroid update after every call
    const int S = steps_of(d);
    // the centroids' two bf16 planes, their squared norms and the largest norm in one launch
    hipLaunchKernelGGL(split_planes_kernel<true>, dim3((unsigned)((k + 31) / 32)), dim3(256), 0, s, cent, (long long)k, d,
                       S, 2, (bf16x8 *)Ct, (long long)(split_plane_bytes(k, d) / 16), cn, cmax_bits);
    // Bound on |computed score - exact score| / (||z||^2 + max ||c||^2):
    //  * dropped products: z.c - (z1.c1 + z1.c2 + z2.c1) = z2.c2 + r_z.c + z.r_c - ..., each at most
    //    2^-16 sum |z_k||c_k| (plus terms of order 2^-24), and sum |z_k||c_k| <= (||z||^2 + ||c||^2) / 2;
    //    with z2 = r_z = 0 only z.r_c remains;
    //  * accumulation: every matrix instruction adds 16 exact products to an fp32 accumulator; charged
    //    with 16 units in the last place of the largest partial sum, 16 * 2^-24 sum |z_k||c_k| each;
    //  * ||c||^2 rounded to fp32 and the final subtraction: below 2^-21 (||z||^2 + ||c||^2).
    // The score doubles the dot product's error, which cancels the 1/2 above.
    const int products = zplanes > 1 ? 3 : 2;
    const float err_coef = (zplanes > 1 ? 3.05f : 1.05f) * 1.52587890625e-5f +
                           (float)(products * S) * 9.5367431640625e-7f + 4.76837158203125e-7f;
    const float err_safe = 1.02f * err_coef;  // |z1| and |c1| may exceed |z| and |c| by a factor 1 + 2^-8
    const long long zplane = (long long)(split_plane_bytes(N, d) / 16);
    const long long cplane = (long long)(split_plane_bytes(k, d) / 16);
    const unsigned grid = (unsigned)((N + FP - 1) / FP);
    const bool top3 = filter_uses_pairs(k);
    // points given as bf16, several passes over the centroids, and two workgroups' points fit the LDS
    // of a compute unit: the kernel that keeps the points on chip
    if (zplanes == 1 && k > FC && S <= 19) {
        const size_t lds = (size_t)4 * S * 1024 > (size_t)FR_MERGE_BYTES ? (size_t)4 * S * 1024 : (size_t)FR_MERGE_BYTES;
        const unsigned rgrid = (unsigned)(((N + 31) / 32 + 3) / 4);
#define LCN_RESIDENT_LAUNCH(T3_)                                                                                       \
    do {                                                                                                               \
        hipError_t e_ = allow_dynamic_lds(reinterpret_cast<const void *>(&assign_filter_resident_kernel<T3_>),         \
                                          T3_ ? 1 : 0, lds);                                                           \
        if (e_ != hipSuccess) return e_;                                                                               \
        hipLaunchKernelGGL((assign_filter_resident_kernel<T3_>), dim3(rgrid), dim3(256), lds, s, (const bf16x8 *)Zt,   \
                           N, S, (const bf16x8 *)Ct, cplane, k, cn, zn, cmax_bits, err_safe, out, flagged, pairs,      \
                           nflagged);                                                                                  \
    } while (0)
        if (top3)
            LCN_RESIDENT_LAUNCH(true);
        else
            LCN_RESIDENT_LAUNCH(false);
#undef LCN_RESIDENT_LAUNCH
        return hipGetLastError();
    }
#define LCN_FILTER_LAUNCH(ZP_, T3_)                                                                                   \
    hipLaunchKernelGGL((assign_filter_kernel<ZP_, T3_>), dim3(grid), dim3(256), 0, s, (const bf16x8 *)Zt, zplane, N,  \
                       S, (const bf16x8 *)Ct, cplane, k, cn, zn, cmax_bits, err_safe, out, flagged, pairs, nflagged)
    if (zplanes > 1) {
        if (top3)
            LCN_FILTER_LAUNCH(2, true);
        else
            LCN_FILTER_LAUNCH(2, false);
    } else {
        if (top3)
            LCN_FILTER_LAUNCH(1, true);
        else
            LCN_FILTER_LAUNCH(1, false);
    }
#undef LCN_FILTER_LAUNCH
    return hipGetLastError();
}

}  // namespace lcn
