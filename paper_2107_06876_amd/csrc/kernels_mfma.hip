// k-means assignment as an MFMA distance GEMM used as a *filter*.
//
// The bucket of a point is defined by an exact fp64 rule (see
// kernels_structure.hip).  Evaluating that rule for every (point, centroid)
// pair is ALU bound; here the scores  ||c||^2 - 2 z.c  are computed with fp32
// matrix instructions (v_mfma_f32_32x32x2f32), which ranks the centroids of a
// point up to a rigorous rounding bound delta.  If the two best scores of a
// point are further apart than 2 delta, the best one is also the exact rule's
// answer; otherwise the point is put on a list and decided by the exact rule.
//
// Tiling for 64-wide wavefronts: a workgroup of 4 waves takes 128 points and
// walks over the centroids 128 at a time; each wave owns 32 points (the N side
// of the instruction) and 4 x 32 centroids (the M side), i.e. four 32x32
// accumulator tiles.  With centroids on M a lane holds 16 centroids of ONE
// point per tile, so the running arg-min needs no cross-lane work until the two
// half-waves are merged at the end.
#include "lcn_internal.h"

namespace lcn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int FP = 128;  // points per workgroup
constexpr int FC = 128;  // centroids per pass
constexpr int FK = 32;   // dimensions per staged chunk
constexpr int FLD = FK + 1;

// squared norms of the centroids as fp32 plus their maximum (bit pattern of a
// non-negative float orders like an unsigned integer)
__global__ void centroid_norms_kernel(const float *__restrict__ C, int k, int d, float *__restrict__ cn,
                                      unsigned *cmax_bits)
{
    const int c = blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
    if (c >= k) return;
    const int lane = threadIdx.x & 63;
    double s = 0.0;
    for (int j = lane; j < d; j += 64) {
        const double v = (double)C[(long long)c * d + j];
        s = fma(v, v, s);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) {
        const float f = (float)s;
        cn[c] = f;
        atomicMax(cmax_bits, __float_as_uint(f * 1.0000002f));
    }
}

__global__ __launch_bounds__(256) void assign_filter_kernel(const float *__restrict__ Z, long long N, int d,
                                                            const float *__restrict__ C, int k,
                                                            const float *__restrict__ cn,
                                                            const double *__restrict__ zn,
                                                            const unsigned *__restrict__ cmax_bits,
                                                            int32_t *__restrict__ out, int *__restrict__ flagged,
                                                            int *nflagged)
{
    __shared__ float Zs[FP][FLD];
    __shared__ float Cs[FC][FLD];
    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const long long p0 = (long long)blockIdx.x * FP;

    float best = INFINITY, second = INFINITY;
    int bidx = 0;

    for (int c0 = 0; c0 < k; c0 += FC) {
        floatx16 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

        // the next chunk of dimensions is fetched into registers while the matrix
        // instructions work on the current one
        const int skk = tid & 31;
        const int sr0 = tid >> 5;
        float zreg[FP / 8], creg[FC / 8];
        auto fetch = [&](int k0) {
            const bool kin = k0 + skk < d;
#pragma unroll
            for (int pass = 0; pass < FP / 8; ++pass) {
                const long long p = p0 + sr0 + pass * 8;
                zreg[pass] = (kin && p < N) ? Z[p * d + k0 + skk] : 0.f;
            }
#pragma unroll
            for (int pass = 0; pass < FC / 8; ++pass) {
                const int c = c0 + sr0 + pass * 8;
                creg[pass] = (kin && c < k) ? C[(long long)c * d + k0 + skk] : 0.f;
            }
        };
        fetch(0);
        for (int k0 = 0; k0 < d; k0 += FK) {
            __syncthreads();
#pragma unroll
            for (int pass = 0; pass < FP / 8; ++pass) Zs[sr0 + pass * 8][skk] = zreg[pass];
#pragma unroll
            for (int pass = 0; pass < FC / 8; ++pass) Cs[sr0 + pass * 8][skk] = creg[pass];
            __syncthreads();
            if (k0 + FK < d) fetch(k0 + FK);
#pragma unroll
            for (int kk = 0; kk < FK; kk += 2) {
                const float b = Zs[w * 32 + col][kk + half];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float a = Cs[t * 32 + col][kk + half];
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[t], 0, 0, 0);
                }
            }
        }
        // scores of this pass's centroids for the lane's point; element v of tile t is
        // centroid row (v / 4) * 8 + half * 4 + v % 4 of the tile
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = c0 + t * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                if (c < k) {
                    const float s = cn[c] - 2.f * acc[t][v];
                    if (s < best) {
                        second = best;
                        best = s;
                        bidx = c;
                    } else if (s < second) {
                        second = s;
                    }
                }
            }
    }
    // merge the two half-waves that share a point
    const float ob = __shfl_xor(best, 32, 64);
    const float os = __shfl_xor(second, 32, 64);
    const int oi = __shfl_xor(bidx, 32, 64);
    const float hi = fmaxf(best, ob);
    second = fminf(hi, fminf(second, os));
    if (ob < best || (ob == best && oi < bidx)) {
        best = ob;
        bidx = oi;
    }
    const long long p = p0 + w * 32 + col;
    if (half == 0 && p < N) {
        out[p] = bidx;
        // rounding bound of a score: (d + 4) u (||z||^2 + ||c||^2) with u = 2^-24, doubled for safety
        const float cmax = __uint_as_float(*cmax_bits);
        const float delta = 2.5f * (float)(d + 4) * 5.9604645e-8f * ((float)zn[p] * 1.0000002f + cmax);
        if (!(second - best > 2.f * delta)) {
            const int slot = atomicAdd(nflagged, 1);
            flagged[slot] = (int)p;
        }
    }
}

hipError_t launch_assign_filter(const float *Z, long long N, int d, const float *cent, int k, const double *zn,
                                float *cn, unsigned *cmax_bits, int32_t *out, int *flagged, int *nflagged,
                                hipStream_t s)
{
    // cmax_bits and nflagged are zero on entry: cleared by the caller before the first
    // call and by the centroid update after every call
    hipLaunchKernelGGL(centroid_norms_kernel, dim3((k + 3) / 4), dim3(256), 0, s, cent, k, d, cn, cmax_bits);
    hipLaunchKernelGGL(assign_filter_kernel, dim3((unsigned)((N + FP - 1) / FP)), dim3(256), 0, s, Z, N, d, cent, k, cn,
                       zn, cmax_bits, out, flagged, nflagged);
    return hipGetLastError();
}

}  // namespace lcn
