// Host side of the C ABI declared in include/lcn.h: argument checks, the
// workspace layout, and the order in which the build and iteration kernels are
// enqueued.  No arithmetic of the method happens on the host except the choice
// of the k-means start indices (integer only).
#include <cstdlib>
#include <mutex>
#include <new>
#include <thread>
#include <unordered_map>
#include <vector>

#include "lcn_internal.h"

using namespace lcn;

namespace {

// ---------------------------------------------------------------- helpers --

struct Bump {
    char *base;
    size_t cap, used;
    bool dry;
    template <class T>
    T *take(size_t count)
    {
        size_t bytes = (count * sizeof(T) + 255) & ~(size_t)255;
        size_t at = used;
        used += bytes;
        if (dry || used > cap) return nullptr;
        return (T *)(base + at);
    }
};

uint64_t splitmix64(uint64_t &state)
{
    uint64_t z = (state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

// The first k slots of a Fisher-Yates shuffle of 0..N-1 driven by splitmix64,
// step t swapping slot t with slot t + next() mod (N - t); only touched slots
// are stored.
std::vector<long long> seeded_indices(uint64_t seed, long long N, int k)
{
    std::unordered_map<long long, long long> moved;
    auto at = [&](long long i) {
        auto it = moved.find(i);
        return it == moved.end() ? i : it->second;
    };
    std::vector<long long> idx((size_t)k);
    uint64_t s = seed;
    for (int t = 0; t < k; ++t) {
        long long j = t + (long long)(splitmix64(s) % (uint64_t)(N - t));
        long long vt = at(t), vj = at(j);
        moved[t] = vj;
        moved[j] = vt;
        idx[(size_t)t] = vj;
    }
    return idx;
}

bool uses_landmarks(int mode) { return mode == LCN_MODE_NYSTROM || mode == LCN_MODE_LCN; }
bool uses_lsh(int mode) { return mode == LCN_MODE_SPARSE || mode == LCN_MODE_LCN; }

constexpr int KM_LANES = 4;   // k-means runs of a build that may be in flight together

struct KmScratch {  // what one k-means run needs for itself
    long long *idx;
    float *cent;
    int *counts2, *cursor2, *order, *offs;  // k-means update: [2][kmax], [2][kmax], [N], [kmax]
    long long *part;                        // ... and its partial sums
    int32_t *assign;
    float *cn;
    unsigned *cmax_bits;
    int *flagged, *nflagged, *pairs;
    unsigned long long *pp_state;  // k-means++: bits of the largest squared norm
    int *horder, *hchunks, *nchild;  // hierarchical k-means: points grouped by parent, chunk list, children per parent
    double *hcent;                   // ... and the children's centroids as fp64, [parent][dimension][child padded]
    char *ct;                        // bf16 planes of the centroids (assignment filter)
};

struct Scratch {  // build-only buffers
    long long *starts;  // seeded start indices of every k-means run of the build: landmarks, then one set per round
    double *Vt64, *A64, *Lt, *Li, *Ainv, *ln, *Dinv, *Tm;
    int *fail_flag;
    long long *totals;
    char *zt;  // bf16 planes of the points (assignment filter)
    int zplanes;
    KmScratch km[KM_LANES];
};

// Lays out everything except the sparse values.  With bump.dry only sizes are
// computed.
void layout(Handle &h, Bump &bump, Scratch &sc)
{
    const long long N = h.n + h.m;
    const int kmax = h.l > h.b ? h.l : h.b;
    h.Z = bump.take<float>((size_t)N * h.d);
    h.zn = bump.take<double>((size_t)N);
    h.a = bump.take<float>((size_t)h.n);
    h.b_marg = bump.take<float>((size_t)h.m);
    h.counters = bump.take<unsigned long long>(16);
    h.query_out = bump.take<double>(4);
    sc.fail_flag = bump.take<int>(4);
    sc.totals = bump.take<long long>(4);
    h.L = bump.take<float>((size_t)(h.l > 0 ? h.l : 1) * h.d);
    sc.starts = bump.take<long long>((size_t)(h.l > 0 ? h.l : 1) + (size_t)(h.R > 0 ? h.R : 1) * (size_t)h.b);
    // bf16 planes for the assignment filter: points (one plane if the input was bf16), centroids
    sc.zplanes = h.in_dtype == LCN_BF16 ? 1 : 2;
    sc.zt = bump.take<char>((size_t)sc.zplanes * split_plane_bytes(N, h.d));
    for (int q = 0; q < KM_LANES; ++q) {
        KmScratch &km = sc.km[q];
        km.idx = bump.take<long long>((size_t)kmax);
        km.cent = bump.take<float>((size_t)kmax * h.d);
        // counts2 .. nflagged are cleared together at the start of a k-means run
        km.counts2 = bump.take<int>(2 * (size_t)kmax);
        km.cursor2 = bump.take<int>(2 * (size_t)kmax);
        km.cmax_bits = bump.take<unsigned>(4);
        km.nflagged = bump.take<int>(4);
        km.order = bump.take<int>((size_t)N);
        km.offs = bump.take<int>((size_t)kmax);
        km.part = bump.take<long long>(kmeans_partial_elems(N, kmax, h.d));
        km.assign = bump.take<int32_t>((size_t)N);
        km.cn = bump.take<float>((size_t)kmax);
        km.ct = bump.take<char>(2 * split_plane_bytes(kmax, h.d));
        km.pp_state = bump.take<unsigned long long>(4);
        if (h.hier_levels > 1) {
            km.horder = bump.take<int>((size_t)N);
            km.hchunks = bump.take<int>(3 * ((size_t)N / 64 + (size_t)kmax + 1));
            km.nchild = bump.take<int>((size_t)kmax);
            // parents * padded children <= 8 * buckets (a level of fewer than 4 children is padded to 4)
            km.hcent = bump.take<double>(8 * (size_t)h.b * h.d);
        }
        km.flagged = bump.take<int>((size_t)N + 8);  // also the k-means++ sweep's 64-bit totals, one per 64 points
        km.pairs = bump.take<int>(3 * (size_t)N);
    }
    h.bucket = bump.take<int32_t>((size_t)(h.R > 0 ? h.R : 1) * N);

    SortBuffers &B = h.sort;
    B.R = h.R;
    B.b = h.b;
    B.n = h.n;
    B.m = h.m;
    B.bucket = h.bucket;
    B.chunks = sort_chunks(h.n, h.m);
    const size_t Rb = (size_t)(h.R > 0 ? h.R : 1) * h.b;
    B.hist = bump.take<int>(2 * Rb * B.chunks);
    B.totals = bump.take<int>(2 * Rb);
    B.off = bump.take<int>(2 * (size_t)(h.R > 0 ? h.R : 1) * (h.b + 1));
    B.perm = bump.take<int>((size_t)(h.R > 0 ? h.R : 1) * N);
    B.pos = bump.take<int>((size_t)(h.R > 0 ? h.R : 1) * N);
    B.tile_off = bump.take<int>(Rb + 1);
    B.totals_out = sc.totals;
    B.seg_x = bump.take<Seg>((size_t)(h.R > 0 ? h.R : 1) * h.n);
    B.seg_y = bump.take<Seg>((size_t)(h.R > 0 ? h.R : 1) * h.m);
    B.rowbase_x = bump.take<long long>((size_t)h.n + 1);
    B.rowbase_y = bump.take<long long>((size_t)h.m + 1);
    B.meta_stride = meta_stride_for(h.R);
    B.meta_x = bump.take<int>((size_t)h.n * B.meta_stride);
    B.meta_y = bump.take<int>((size_t)h.m * B.meta_stride);

    const size_t lp1 = h.lp > 0 ? h.lp : 1;
    h.U = bump.take<float>((size_t)h.n * lp1);
    h.Wt = bump.take<float>((size_t)h.m * lp1);
    const size_t l1 = h.l > 0 ? h.l : 1;
    sc.Vt64 = bump.take<double>((size_t)h.m * l1);
    sc.A64 = bump.take<double>(l1 * l1);
    sc.Lt = bump.take<double>(l1 * l1);
    sc.Li = bump.take<double>(l1 * l1);
    sc.Ainv = bump.take<double>(l1 * l1);
    sc.ln = bump.take<double>(l1);
    sc.Dinv = bump.take<double>((l1 + 63) / 64 * 64 * 64);
    sc.Tm = bump.take<double>(64 * l1);

    h.log_u = bump.take<float>((size_t)h.n);
    h.log_v = bump.take<float>((size_t)h.m);
    h.lin_u = bump.take<double>((size_t)h.n);
    h.lin_v = bump.take<double>((size_t)h.m);
    // each is followed by a slot that stays zero (what masked-out lanes of a sweep read)
    h.perm_u = bump.take<double>((size_t)(h.R > 0 ? h.R : 1) * h.n + 8);
    h.perm_v = bump.take<double>((size_t)(h.R > 0 ? h.R : 1) * h.m + 8);
    for (int i = 0; i < 2; ++i) h.acc[i] = bump.take<double>(lp1 + 2);
    h.shift = bump.take<double>(2);
    h.grid = bump.dry ? 1024 : pass_grid(h);
    h.partial = bump.take<double>((size_t)(bump.dry ? 1024 : h.grid) * (h.lp + 3));
    h.partial2 = bump.take<double>((size_t)(bump.dry ? 1024 : h.grid) * (h.lp + 3));
}

lcn_status check_params(long long n, long long m, int d, int dtype, float lambda, int cost, int mode,
                        const lcn_landmark_params *lm, const lcn_lsh_params *lsh)
{
    if (n < 1 || m < 1 || d < 1) return LCN_ERR_INVALID_ARG;
    if (n > (1ll << 30) || m > (1ll << 30) || d > 8192) return LCN_ERR_INVALID_ARG;  // a row of d floats must fit LDS
    if (dtype != LCN_F32 && dtype != LCN_BF16) return LCN_ERR_INVALID_ARG;
    if (!(lambda > 0.f) || !(lambda < INFINITY)) return LCN_ERR_INVALID_ARG;
    if (cost < LCN_COST_SQEUCLID || cost > LCN_COST_COSINE) return LCN_ERR_INVALID_ARG;
    if (mode < LCN_MODE_DENSE || mode > LCN_MODE_LCN) return LCN_ERR_INVALID_ARG;
    bool kmeans = false;
    if (uses_landmarks(mode)) {
        if (!lm) return LCN_ERR_INVALID_ARG;
        if (lm->num_landmarks < 1 || lm->num_landmarks > 512 || lm->num_landmarks > n + m) return LCN_ERR_INVALID_ARG;
        if (lm->kmeans_iters < 0) return LCN_ERR_INVALID_ARG;
        if (!(lm->ridge >= 0.0)) return LCN_ERR_INVALID_ARG;
        if (lm->init < LCN_INIT_SAMPLE || lm->init > LCN_INIT_GIVEN) return LCN_ERR_INVALID_ARG;
        if ((lm->init == LCN_INIT_GIVEN) != (lm->init_centroids != nullptr)) return LCN_ERR_INVALID_ARG;
        kmeans = true;
    }
    if (uses_lsh(mode)) {
        if (!lsh) return LCN_ERR_INVALID_ARG;
        if (lsh->num_buckets < 1 || lsh->num_buckets > 4096) return LCN_ERR_INVALID_ARG;
        if (lsh->num_rounds < 1 || lsh->num_rounds > 8) return LCN_ERR_INVALID_ARG;
        if (lsh->and_width < 0 || lsh->and_width > 12) return LCN_ERR_INVALID_ARG;
        if (lsh->hash == LCN_HASH_KMEANS) {
            if (lsh->kmeans_iters < 1 || lsh->and_width > 1) return LCN_ERR_INVALID_ARG;
            if (lsh->branching[0] > 0) {   // hierarchical: the factors must multiply to num_buckets
                long long prod = 1;
                for (int j = 0; j < 3 && lsh->branching[j] > 0; ++j) {
                    if (j > 0 && lsh->branching[j] > 32) return LCN_ERR_INVALID_ARG;
                    prod *= lsh->branching[j];
                    if (prod > 4096) return LCN_ERR_INVALID_ARG;
                }
                for (int j = 0; j < 3; ++j) {
                    if (lsh->branching[j] < 0) return LCN_ERR_INVALID_ARG;
                    if (j > 0 && lsh->branching[j] > 0 && lsh->branching[j - 1] == 0) return LCN_ERR_INVALID_ARG;
                }
                if (prod != lsh->num_buckets || lsh->branching[0] > n + m) return LCN_ERR_INVALID_ARG;
            } else if (lsh->num_buckets > n + m) {
                return LCN_ERR_INVALID_ARG;
            }
            kmeans = true;
        } else if (lsh->hash == LCN_HASH_CROSSPOLYTOPE) {
            if ((lsh->num_buckets & 1) || !lsh->projections) return LCN_ERR_INVALID_ARG;
            if (lsh->branching[0] != 0) return LCN_ERR_INVALID_ARG;
            long long prod = 1;
            for (int j = 0; j < (lsh->and_width > 1 ? lsh->and_width : 1); ++j) {
                prod *= lsh->num_buckets;
                if (prod > 4096) return LCN_ERR_INVALID_ARG;   // buckets of a band: num_buckets ^ and_width
            }
        } else {
            return LCN_ERR_INVALID_ARG;
        }
    }
    if (kmeans && n + m > (1ll << 20)) return LCN_ERR_INVALID_ARG;
    return LCN_OK;
}

void fill_shape(Handle &h, long long n, long long m, int d, int mode, const lcn_landmark_params *lm,
                const lcn_lsh_params *lsh)
{
    h.n = n;
    h.m = m;
    h.d = d;
    h.mode = mode;
    h.log_domain = (mode == LCN_MODE_SPARSE || mode == LCN_MODE_DENSE) ? 1 : 0;
    h.l = uses_landmarks(mode) ? lm->num_landmarks : 0;
    h.lp = (h.l + 63) / 64 * 64;
    h.hier_levels = 0;
    h.and_width = 1;
    if (uses_lsh(mode)) {
        h.R = lsh->num_rounds;
        h.b = lsh->num_buckets;
        h.hash = lsh->hash;
        if (lsh->hash == LCN_HASH_KMEANS) {
            while (h.hier_levels < 3 && lsh->branching[h.hier_levels] > 0) ++h.hier_levels;
        } else if (lsh->and_width > 1) {   // a band's bucket is a tuple of and_width hash values
            h.and_width = lsh->and_width;
            for (int j = 1; j < h.and_width; ++j) h.b *= lsh->num_buckets;
        }
    } else if (mode == LCN_MODE_DENSE) {  // the dense kernel is the single-bucket sparse kernel
        h.R = 1;
        h.b = 1;
        h.hash = -1;
    } else {
        h.R = 0;
        h.b = 1;
        h.hash = -1;
    }
}

#define HIPCHK(expr)                         \
    do {                                     \
        hipError_t e_ = (expr);              \
        if (e_ != hipSuccess) {              \
            (void)hipGetLastError();         \
            return LCN_ERR_DEVICE;           \
        }                                    \
    } while (0)

// T Lloyd iterations on Z from the start `init` names (LCN_INIT_*): centroids into cent, the last
// iteration's assignment into assign (untouched if T == 0).
// start_dev (nullable): the k seeded start indices, already on the device (LCN_INIT_SAMPLE only).
// km: the run's own scratch; s: the stream it is ordered on.
lcn_status run_kmeans(Handle &h, Scratch &sc, KmScratch &km, hipStream_t s, int k, int T, uint64_t seed, float *cent,
                      int32_t *assign, const long long *start_dev = nullptr, int init = LCN_INIT_SAMPLE,
                      const float *given = nullptr)
{
    const long long N = h.n + h.m;
    if (init == LCN_INIT_GIVEN) {
        HIPCHK(hipMemcpyAsync(cent, given, sizeof(float) * (size_t)k * h.d, hipMemcpyDeviceToDevice, s));
    } else if (init == LCN_INIT_KMEANSPP) {
        std::vector<unsigned long long> rnd((size_t)k);
        uint64_t st = seed;
        for (int t = 0; t < k; ++t) rnd[(size_t)t] = splitmix64(st);
        HIPCHK(hipMemcpyAsync(km.idx, rnd.data(), sizeof(unsigned long long) * (size_t)k, hipMemcpyHostToDevice,
                              s));
        HIPCHK(hipStreamSynchronize(s));  // rnd is a local host vector
        // the assignment's buffers are free until the first Lloyd iteration
        HIPCHK(launch_kmeanspp(h.Z, N, h.d, k, (const unsigned long long *)km.idx, (double *)km.pairs,
                               (unsigned long long *)km.flagged, km.order, km.pp_state, cent, s));
    } else if (start_dev) {
        HIPCHK(launch_gather_rows(h.Z, h.d, start_dev, k, cent, s));
    } else {
        std::vector<long long> idx = seeded_indices(seed, N, k);
        HIPCHK(hipMemcpyAsync(km.idx, idx.data(), sizeof(long long) * (size_t)k, hipMemcpyHostToDevice, s));
        HIPCHK(hipStreamSynchronize(s));  // idx is a local host vector
        HIPCHK(launch_gather_rows(h.Z, h.d, km.idx, k, cent, s));
    }
    // member counts and cursors of the update, the filter's largest centroid norm and its two
    // counters lie side by side: one clear
    HIPCHK(hipMemsetAsync(km.counts2, 0, (size_t)((char *)(km.nflagged + 4) - (char *)km.counts2), s));
    for (int it = 0; it < T; ++it) {
        if (h.exact_assign_only) {
            HIPCHK(launch_assign_kmeans(h.Z, N, h.d, cent, k, assign, nullptr, nullptr, s));
        } else {
            HIPCHK(launch_assign_filter(sc.zt, sc.zplanes, N, h.d, cent, k, km.ct, h.zn, km.cn, km.cmax_bits, assign,
                                        km.flagged, km.pairs, km.nflagged, s));
            if (filter_uses_pairs(k))
                HIPCHK(launch_assign_pairs(h.Z, h.d, cent, assign, km.pairs, km.nflagged + 1, s));
            HIPCHK(launch_assign_kmeans(h.Z, N, h.d, cent, k, assign, km.flagged, km.nflagged, s));
        }
        // the last iteration leaves the count of undecided points in place for lcn_get_info
        HIPCHK(launch_kmeans_update(h.Z, N, h.d, assign, k, km.counts2, km.cursor2, km.order, km.offs, km.part, it, cent,
                                    km.cmax_bits, it + 1 < T ? km.nflagged : nullptr, s));
    }
    return LCN_OK;
}

// Hierarchical k-means hashing: level 0 is a k-means on all points; level j >= 1 runs, inside every
// cluster of level j-1, a k-means with branching[j] clusters on that cluster's members (in index
// order; fewer members than that: one cluster per member), seeded with seed + j * 2^32 + parent.
// bucket = parent * branching[j] + child.  The grouping by parent and the seeded starts are made on
// the host from a copy of the level above (one synchronisation per level).
lcn_status run_hier_kmeans(Handle &h, Scratch &sc, KmScratch &km, hipStream_t s, const int32_t *branching, int levels,
                           int T, uint64_t seed, int32_t *dst)
{
    const long long N = h.n + h.m;
    lcn_status st = run_kmeans(h, sc, km, s, branching[0], T, seed, km.cent, dst);
    if (st != LCN_OK) return st;
    long long parents = branching[0];
    std::vector<int32_t> ids((size_t)N);
    std::vector<int> order((size_t)N), offs, nchild, chunks;
    std::vector<long long> start;
    for (int lev = 1; lev < levels; ++lev) {
        const int bl = branching[lev];
        const long long k = parents * bl;
        HIPCHK(hipMemcpyAsync(ids.data(), dst, sizeof(int32_t) * (size_t)N, hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        offs.assign((size_t)parents + 1, 0);
        for (long long i = 0; i < N; ++i) offs[(size_t)ids[(size_t)i] + 1] += 1;
        for (long long c = 0; c < parents; ++c) offs[(size_t)c + 1] += offs[(size_t)c];
        {
            std::vector<int> cur(offs.begin(), offs.end() - 1);
            for (long long i = 0; i < N; ++i) order[(size_t)cur[(size_t)ids[(size_t)i]]++] = (int)i;   // stable
        }
        start.assign((size_t)k, -1);
        nchild.assign((size_t)parents, 0);
        chunks.clear();
        for (long long c = 0; c < parents; ++c) {
            const int nc = offs[(size_t)c + 1] - offs[(size_t)c];
            if (nc == 0) continue;
            const int kc = bl < nc ? bl : nc;
            nchild[(size_t)c] = kc;
            std::vector<long long> pick = seeded_indices(seed + ((uint64_t)lev << 32) + (uint64_t)c, nc, kc);
            for (int j = 0; j < kc; ++j)
                start[(size_t)(c * bl + j)] = order[(size_t)offs[(size_t)c] + (size_t)pick[(size_t)j]];
            for (int s0 = 0; s0 < nc; s0 += 64) {
                chunks.push_back((int)c);
                chunks.push_back(offs[(size_t)c] + s0);
                chunks.push_back(nc - s0 < 64 ? nc - s0 : 64);
            }
        }
        const int nchunks = (int)(chunks.size() / 3);
        HIPCHK(hipMemcpyAsync(km.idx, start.data(), sizeof(long long) * (size_t)k, hipMemcpyHostToDevice, s));
        HIPCHK(hipMemcpyAsync(km.nchild, nchild.data(), sizeof(int) * (size_t)parents, hipMemcpyHostToDevice,
                              s));
        HIPCHK(hipMemcpyAsync(km.horder, order.data(), sizeof(int) * (size_t)N, hipMemcpyHostToDevice, s));
        HIPCHK(hipMemcpyAsync(km.hchunks, chunks.data(), sizeof(int) * chunks.size(), hipMemcpyHostToDevice,
                              s));
        HIPCHK(hipStreamSynchronize(s));  // the host vectors are reused by the next level
        HIPCHK(launch_gather_rows(h.Z, h.d, km.idx, (int)k, km.cent, s));
        HIPCHK(hipMemsetAsync(km.counts2, 0, 2 * sizeof(int) * (size_t)k, s));
        HIPCHK(hipMemsetAsync(km.cursor2, 0, 2 * sizeof(int) * (size_t)k, s));
        for (int it = 0; it < T; ++it) {
            HIPCHK(launch_assign_children(h.Z, h.d, km.cent, parents, bl, km.nchild, km.horder, km.hchunks, nchunks,
                                          km.hcent, dst, s));
            HIPCHK(launch_kmeans_update(h.Z, N, h.d, dst, (int)k, km.counts2, km.cursor2, km.order, km.offs, km.part,
                                        it, km.cent, nullptr, nullptr, s));
        }
        parents = k;
    }
    return LCN_OK;
}

lcn_status status_from_counters(Handle &h)
{
    unsigned long long c[7];
    HIPCHK(hipMemcpyAsync(c, h.counters, sizeof(c), hipMemcpyDeviceToHost, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    if (c[5]) return LCN_ERR_DEVICE;  // a sweep gave up waiting for its totals
    // a scaling that outgrew the single-precision copy the sparse part reads turns later sums into
    // NaN, which count as non-positive too: the overflow is the cause and is reported
    if (c[6]) return LCN_ERR_RANGE;
    if (c[0]) return LCN_ERR_NONPOSITIVE;
    if (c[1] | c[2]) return LCN_WARN_NO_SUPPORT;
    return LCN_OK;
}

// From the stored log scalings: working copies, bucket-ordered copies, and the
// accumulators z = U^T u (buffer 1) and y = W v (buffer 0).
lcn_status init_state(Handle &h, bool clear_logs = false)
{
    const size_t R1 = (size_t)(h.R > 0 ? h.R : 1);
    // the slot behind the bucket-ordered copies that stays zero: entry R n (R m) of an array of doubles
    // (logarithmic sweeps) or of floats (linear sweeps)
    ClearRegions cl{};
    cl.add(h.perm_u + R1 * h.n, 8 * sizeof(double));
    cl.add(h.perm_v + R1 * h.m, 8 * sizeof(double));
    if (!h.log_domain) {
        cl.add(reinterpret_cast<float *>(h.perm_u) + R1 * h.n, 8 * sizeof(float));
        cl.add(reinterpret_cast<float *>(h.perm_v) + R1 * h.m, 8 * sizeof(float));
    }
    if (clear_logs) {   // scalings at their start, v = 1 (and u, until the first sweep replaces it)
        cl.add(h.log_u, sizeof(float) * (size_t)h.n);
        cl.add(h.log_v, sizeof(float) * (size_t)h.m);
    }
    HIPCHK(launch_clear_regions(cl, h.stream));
    HIPCHK(launch_pass(h, 0, PASS_INIT, -1, 1, nullptr, h.stream));
    HIPCHK(launch_pass(h, 1, PASS_INIT, -1, 0, nullptr, h.stream));
    h.fresh = 1;
    return LCN_OK;
}

// KM_LANES - 1 streams per device for the process (default priority, not synchronising with the null
// stream), created on first use and never destroyed; the last lane is the caller's stream, which
// would otherwise idle while the lanes work (a process has four hardware queues by default, and a
// fifth stream would share one of them with another lane and run in turn with it).  False if they
// cannot be had.
bool lane_streams(hipStream_t (&out)[KM_LANES])
{
    static std::mutex mu;
    static hipStream_t streams[64][KM_LANES] = {};
    static bool ready[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (!ready[dev]) {
        for (int q = 0; q < KM_LANES - 1; ++q) {
            if (!streams[dev][q] && hipStreamCreateWithFlags(&streams[dev][q], hipStreamNonBlocking) != hipSuccess) {
                (void)hipGetLastError();
                streams[dev][q] = nullptr;
                return false;
            }
        }
        ready[dev] = true;
    }
    for (int q = 0; q < KM_LANES - 1; ++q) out[q] = streams[dev][q];
    return true;
}

// One lcn_build call: what it holds while it runs, and its stages as member functions, called in
// order by build_one.  Whichever way the build ends, the destructor first joins the host threads,
// then drains every stream (the caller's inputs and the host vector `starts` are read by work
// that may still be in flight), then lets the members go.
//
// The k-means runs of a build (landmarks, one per hash round) and the factors are independent
// chains of short launches, and the host needs about as long to enqueue such a launch as the
// device to execute it.  Each run therefore gets scratch of its own and one of KM_LANES streams of
// the library's own ("lanes": forked from and joined into the caller's stream by events), and the
// hash rounds of a lane are enqueued by a host thread of their own while the calling thread
// enqueues the landmarks and the factors.
struct Builder {
    Handle &h;
    Bump bump;
    const lcn_landmark_params *lm;
    const lcn_lsh_params *lsh;
    const long long n, m, N;
    const int d, cost, mode;
    Scratch sc{};
    std::vector<long long> starts;   // seeded starts of all flat k-means runs (host copy of sc.starts)
    const long long *starts_landmarks = nullptr, *starts_rounds = nullptr;
    hipStream_t lane[KM_LANES] = {};
    bool forked = false;             // the lanes are streams of their own (else all are the caller's stream)
    bool lane_used[KM_LANES] = {};
    hipEvent_t join[KM_LANES] = {}, extra[2] = {};
    std::thread threads[KM_LANES];
    lcn_status thread_status[KM_LANES];
    const int *last_nflagged = nullptr;   // the undecided counts of the build's last k-means run
    int device_id = 0;

    Builder(Handle &handle, const lcn_landmark_params *lm_, const lcn_lsh_params *lsh_, int cost_, int mode_)
        : h(handle), bump{handle.ws, handle.ws_bytes, 0, false}, lm(lm_), lsh(lsh_), n(handle.n), m(handle.m),
          N(handle.n + handle.m), d(handle.d), cost(cost_), mode(mode_)
    {
        for (int q = 0; q < KM_LANES; ++q) {
            lane[q] = h.stream;
            thread_status[q] = LCN_OK;
        }
    }
    Builder(const Builder &) = delete;
    Builder &operator=(const Builder &) = delete;
    ~Builder()
    {
        join_threads();
        for (int q = 0; q < KM_LANES; ++q) {
            if (forked) (void)hipStreamSynchronize(lane[q]);
            if (join[q]) (void)hipEventDestroy(join[q]);
        }
        for (int q = 0; q < 2; ++q)
            if (extra[q]) (void)hipEventDestroy(extra[q]);
        (void)hipStreamSynchronize(h.stream);
    }
    void join_threads()
    {
        for (int q = 0; q < KM_LANES; ++q)
            if (threads[q].joinable()) threads[q].join();
    }
    bool kmeans_hashing() const { return uses_lsh(mode) && h.hash == LCN_HASH_KMEANS; }
    // the landmarks and the factors keep lane 0 to themselves
    int lane_of_round(int r) const { return h.l > 0 ? 1 + r % (KM_LANES - 1) : r % KM_LANES; }

    // Inputs into the workspace (fp32 points, norms, bf16 planes, marginals), seeded starts to the
    // device in one copy, lanes forked.
    lcn_status prepare(const void *X, const void *Y, const float *a, const float *b, int dtype, bool overlap)
    {
        (void)hipGetDevice(&device_id);
        forked = overlap && lane_streams(lane);
        lane[KM_LANES - 1] = h.stream;
        if (!forked)
            for (int q = 0; q < KM_LANES; ++q) lane[q] = h.stream;
        HIPCHK(hipEventCreate(&h.ev0));
        HIPCHK(hipEventCreate(&h.ev1));
        ClearRegions cl{};
        cl.add(h.counters, 16 * sizeof(unsigned long long));
        cl.add(sc.fail_flag, 4 * sizeof(int));
        cl.add(sc.totals, 4 * sizeof(long long));
        HIPCHK(launch_clear_regions(cl, h.stream));
        HIPCHK(hipMemcpyAsync(h.a, a, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, h.stream));
        HIPCHK(hipMemcpyAsync(h.b_marg, b, sizeof(float) * (size_t)m, hipMemcpyDeviceToDevice, h.stream));
        HIPCHK(launch_convert(X, n, Y, m, d, dtype, h.Z, (unsigned *)(h.counters + 4), h.stream));
        HIPCHK(launch_sqnorms(h.Z, N, d, h.zn, h.stream));
        // bf16 planes of the points for the assignment filter of every k-means run
        if (!h.exact_assign_only && (h.l > 0 || kmeans_hashing()))
            HIPCHK(launch_split_planes(h.Z, N, d, sc.zplanes, sc.zt, h.stream));

        const bool lm_sample = h.l > 0 && lm->init == LCN_INIT_SAMPLE;
        const bool flat_rounds = kmeans_hashing() && h.hier_levels <= 1;
        if (lm_sample) {
            std::vector<long long> idx = seeded_indices(lm->seed, N, h.l);
            starts.insert(starts.end(), idx.begin(), idx.end());
        }
        const size_t rounds_at = starts.size();
        if (flat_rounds)
            for (int r = 0; r < h.R; ++r) {
                std::vector<long long> idx = seeded_indices(lsh->seed + (uint64_t)r, N, h.b);
                starts.insert(starts.end(), idx.begin(), idx.end());
            }
        if (!starts.empty()) {
            HIPCHK(hipMemcpyAsync(sc.starts, starts.data(), sizeof(long long) * starts.size(), hipMemcpyHostToDevice,
                                  h.stream));
            if (lm_sample) starts_landmarks = sc.starts;
            if (flat_rounds) starts_rounds = sc.starts + rounds_at;
        }
        if (forked) {
            HIPCHK(hipEventRecord(h.ev1, h.stream));
            for (int q = 0; q < KM_LANES; ++q) {
                HIPCHK(hipEventCreateWithFlags(&join[q], hipEventDisableTiming));
                HIPCHK(hipStreamWaitEvent(lane[q], h.ev1, 0));
            }
            for (int q = 0; q < 2; ++q) HIPCHK(hipEventCreateWithFlags(&extra[q], hipEventDisableTiming));
        }
        return LCN_OK;
    }

    // All hash rounds (Sec. 3) that lane q carries, in order.
    lcn_status rounds_of_lane(int q)
    {
        for (int r = 0; r < h.R; ++r) {
            if (lane_of_round(r) != q) continue;
            int32_t *dst = h.bucket + (long long)r * N;
            KmScratch &km = sc.km[q];
            hipStream_t ls = lane[q];
            if (h.hash == LCN_HASH_KMEANS) {
                lcn_status rs;
                if (h.hier_levels > 1)
                    rs = run_hier_kmeans(h, sc, km, ls, lsh->branching, h.hier_levels, lsh->kmeans_iters,
                                         lsh->seed + (uint64_t)r, dst);
                else
                    rs = run_kmeans(h, sc, km, ls, h.b, lsh->kmeans_iters, lsh->seed + (uint64_t)r, km.cent, dst,
                                    starts_rounds + (long long)r * h.b);
                if (rs != LCN_OK) return rs;
            } else if (h.and_width > 1) {
                const int b1 = lsh->num_buckets;   // buckets of one hash; the band has b1 ^ and_width
                for (int j = 0; j < h.and_width; ++j) {
                    const float *Rm = lsh->projections + ((long long)r * h.and_width + j) * d * (b1 / 2);
                    HIPCHK(launch_assign_crosspolytope(h.Z, N, d, Rm, b1, km.assign, ls));
                    HIPCHK(launch_combine_hash(dst, km.assign, b1, j == 0, N, ls));
                }
            } else {
                const float *Rm = lsh->projections + (long long)r * d * (h.b / 2);
                HIPCHK(launch_assign_crosspolytope(h.Z, N, d, Rm, h.b, dst, ls));
            }
        }
        return LCN_OK;
    }

    // Starts the hash rounds: with lanes and k-means hashing one host thread per lane enqueues them
    // (so that they overlap with what the calling thread enqueues next), otherwise they are enqueued
    // here and now.
    lcn_status start_hash_rounds()
    {
        if (mode == LCN_MODE_DENSE) {
            HIPCHK(hipMemsetAsync(h.bucket, 0, sizeof(int32_t) * (size_t)N, h.stream));
            return LCN_OK;
        }
        if (!uses_lsh(mode)) return LCN_OK;
        for (int r = 0; r < h.R; ++r) lane_used[lane_of_round(r)] = true;
        if (kmeans_hashing() && h.R > 0) last_nflagged = sc.km[lane_of_round(h.R - 1)].nflagged;
        const bool threaded = forked && kmeans_hashing();
        for (int q = 0; q < KM_LANES; ++q) {
            bool has_round = false;
            for (int r = 0; r < h.R; ++r) has_round = has_round || lane_of_round(r) == q;
            if (!has_round) continue;
            bool started = false;
            if (threaded) {
                try {
                    threads[q] = std::thread([this, q]() {
                        (void)hipSetDevice(device_id);
                        try {
                            thread_status[q] = rounds_of_lane(q);
                        } catch (...) {   // out of host memory in a container
                            thread_status[q] = LCN_ERR_ALLOC;
                        }
                    });
                    started = true;
                } catch (...) {   // no thread to be had: this thread does it
                }
            }
            if (!started) {
                const lcn_status st = rounds_of_lane(q);
                if (st != LCN_OK) return st;
            }
        }
        return LCN_OK;
    }

    // landmarks: centroids of k-means on X u Y, or sampled points (Sec. 4); lane 0
    lcn_status landmarks()
    {
        if (h.l == 0) return LCN_OK;
        const lcn_status st = run_kmeans(h, sc, sc.km[0], lane[0], h.l, lm->kmeans_iters, lm->seed, h.L, sc.km[0].assign,
                                         starts_landmarks, lm->init, lm->init_centroids);
        if (st != LCN_OK) return st;
        lane_used[0] = true;
        if (!last_nflagged) last_nflagged = sc.km[0].nflagged;
        return LCN_OK;
    }

    // Nystrom factors (Sec. 4; App. "Implementational details").  They need the landmarks only and run
    // beside the hash rounds: A and its inverse follow the landmarks on lane 0, U and V go to lanes 1
    // and 2 (behind the hash rounds queued there), W = A^{-1} V waits for both.
    lcn_status factors()
    {
        if (h.l == 0) return LCN_OK;
        hipStream_t fs = lane[0], us = lane[0], vs = lane[0];
        if (forked) {
            us = lane[1];
            vs = lane[2];
            HIPCHK(hipEventRecord(extra[0], lane[0]));   // landmarks done
            HIPCHK(hipStreamWaitEvent(us, extra[0], 0));
            HIPCHK(hipStreamWaitEvent(vs, extra[0], 0));
            lane_used[1] = lane_used[2] = true;
        }
        const float *Xz = h.Z, *Yz = h.Z + (long long)n * d;
        HIPCHK(launch_sqnorms(h.L, h.l, d, sc.ln, fs));   // every cost is formed from dot products and norms
        if (forked) {   // the landmarks' norms are an input of U and V as well
            HIPCHK(hipEventRecord(extra[0], fs));
            HIPCHK(hipStreamWaitEvent(us, extra[0], 0));
            HIPCHK(hipStreamWaitEvent(vs, extra[0], 0));
        }
        // A and its inverse first: a chain of small launches that the two big ones would otherwise
        // keep waiting for compute units; U and V are enqueued behind it and run beside its second half
        HIPCHK(hipMemsetAsync(h.Wt, 0, sizeof(float) * (size_t)m * h.lp, fs));
        HIPCHK(launch_kernel_matrix(h.L, h.l, h.L, h.l, d, cost, h.lambda, sc.ln, sc.ln,
                                    nullptr, sc.A64, h.l, fs));
        HIPCHK(launch_spd_inverse(sc.A64, h.l, h.ridge, sc.Lt, sc.Li, sc.Ainv, sc.Dinv, sc.Tm, sc.fail_flag, fs));
        HIPCHK(hipMemsetAsync(h.U, 0, sizeof(float) * (size_t)n * h.lp, us));
        HIPCHK(launch_kernel_matrix(Xz, n, h.L, h.l, d, cost, h.lambda, h.zn, sc.ln,
                                    h.U, nullptr, h.lp, us));
        HIPCHK(launch_kernel_matrix(Yz, m, h.L, h.l, d, cost, h.lambda, h.zn + n, sc.ln,
                                    nullptr, sc.Vt64, h.l, vs));
        if (forked) {
            HIPCHK(hipEventRecord(extra[1], vs));   // V done
            HIPCHK(hipStreamWaitEvent(fs, extra[1], 0));
        }
        // W^T = V^T A^{-1} (A^{-1} is symmetric)
        HIPCHK(launch_gemm_f64(sc.Vt64, sc.Ainv, m, h.l, h.l, h.Wt, h.lp, fs));
        return LCN_OK;
    }

    // lane 0 holds the landmarks and the factors only
    bool factors_apart() const { return forked && h.l > 0; }

    // Buckets -> blocks (bucket sort, per-row metadata); the host learns the pair count, the
    // undecided-point count and the input-range flag (the build's one wait for the device) and lays
    // out the sparse values.
    lcn_status structure(size_t *bytes_needed)
    {
        join_threads();
        for (int q = 0; q < KM_LANES; ++q)
            if (thread_status[q] != LCN_OK) return thread_status[q];
        if (forked) {   // the buckets are needed from here on, the factors only by the sparse values
            for (int q = factors_apart() ? 1 : 0; q < KM_LANES; ++q) {
                if (!lane_used[q]) continue;
                HIPCHK(hipEventRecord(join[q], lane[q]));
                HIPCHK(hipStreamWaitEvent(h.stream, join[q], 0));
            }
        }
        long long totals[2] = {0, 0};
        unsigned long long range_flag = 0;
        if (h.R > 0) {
            HIPCHK(launch_bucket_sort(h.sort, h.stream));
            HIPCHK(hipMemcpyAsync(totals, sc.totals, sizeof(totals), hipMemcpyDeviceToHost, h.stream));
        }
        HIPCHK(launch_build_meta(h.sort, h.a, h.b_marg, h.stream));
        int undecided2[2] = {0, 0};  // points sent to the exact rule over all centroids, and over two
        if (last_nflagged)
            HIPCHK(hipMemcpyAsync(undecided2, last_nflagged, 2 * sizeof(int), hipMemcpyDeviceToHost, h.stream));
        HIPCHK(hipMemcpyAsync(&range_flag, h.counters + 4, sizeof(range_flag), hipMemcpyDeviceToHost, h.stream));
        HIPCHK(hipEventRecord(h.ev0, h.stream));
        HIPCHK(hipEventSynchronize(h.ev0));
        if (range_flag && (h.l > 0 || h.hash == LCN_HASH_KMEANS)) return LCN_ERR_INVALID_ARG;  // |x| >= 2^10 or not finite
        h.nnz_stored = totals[0];
        h.undecided_last = (long long)undecided2[0] + undecided2[1];
        h.ntiles = (int)totals[1];

        // 64 entries of slack: a sweep reads whole wavefront-wide chunks and masks the excess
        h.vals_x = bump.take<float>((size_t)h.nnz_stored + 64);
        h.vals_y = bump.take<float>((size_t)h.nnz_stored + 64);
        h.ws_used = bump.used;
        if (bytes_needed) *bytes_needed = bump.used + 256;
        if (bump.used > h.ws_bytes) return LCN_ERR_ALLOC;
        return LCN_OK;
    }

    // Sparse values per bucket block (Sec. 3 / Sec. 4), scalings at their start v = 1 (eq. 2), the
    // state derived from them; the build's final synchronisation.
    lcn_status values_and_state()
    {
        if (factors_apart()) {
            HIPCHK(hipEventRecord(join[0], lane[0]));
            HIPCHK(hipStreamWaitEvent(h.stream, join[0], 0));
        }
        if (h.R > 0) HIPCHK(launch_correction(h, h.ntiles, h.stream));
        const lcn_status st = init_state(h, true);
        if (st != LCN_OK) return st;
        int fail = 0;
        unsigned long long uniq = 0;
        HIPCHK(hipMemcpyAsync(&fail, sc.fail_flag, sizeof(int), hipMemcpyDeviceToHost, h.stream));
        HIPCHK(hipMemcpyAsync(&uniq, h.counters + 3, sizeof(uniq), hipMemcpyDeviceToHost, h.stream));
        HIPCHK(hipStreamSynchronize(h.stream));
        if (fail) return LCN_ERR_SINGULAR;
        h.nnz_unique = (long long)uniq;
        return LCN_OK;
    }
};

bool valid(lcn_handle hh) { return hh && ((Handle *)hh)->magic == HANDLE_MAGIC; }

// Scratch of lcn_backward_static: one array per device in the library's own device image, there from
// the moment the image is loaded until the process ends.  Host code never uses the array's name as an
// address: the device address is looked up once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[LCN_STATIC_SCRATCH_BYTES];

lcn_status static_scratch(void **out)
{
    static std::mutex mu;
    static void *ptr_of_device[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return LCN_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return LCN_ERR_DEVICE;
        }
        ptr_of_device[dev] = ptr;
    }
    *out = ptr_of_device[dev];
    return LCN_OK;
}

}  // namespace

extern "C" {

lcn_status lcn_workspace_bytes(int64_t n, int64_t m, int32_t d, int32_t mode, const lcn_landmark_params *lm,
                               const lcn_lsh_params *lsh, int64_t nnz_guess, size_t *bytes)
{
    if (!bytes) return LCN_ERR_INVALID_ARG;
    lcn_status st = check_params(n, m, d, LCN_F32, 1.f, LCN_COST_SQEUCLID, mode, lm, lsh);
    if (st != LCN_OK) return st;
    Handle h{};
    fill_shape(h, n, m, d, mode, lm, lsh);
    Bump bump{nullptr, 0, 0, true};
    Scratch sc{};
    layout(h, bump, sc);
    long long nnz = nnz_guess;
    if (nnz <= 0) {
        if (mode == LCN_MODE_DENSE)
            nnz = n * m;
        else if (h.R > 0)
            nnz = (long long)(1.5 * (double)h.R * (double)n * (double)m / (double)h.b) + 4096;
        else
            nnz = 0;
    }
    bump.take<float>((size_t)nnz + 64);
    bump.take<float>((size_t)nnz + 64);
    *bytes = bump.used + 256;
    return LCN_OK;
}

static lcn_status build_one(const void *X, int64_t n, const void *Y, int64_t m, int32_t d, int32_t dtype, const float *a,
                            const float *b, float lambda, int32_t cost, int32_t mode, const lcn_landmark_params *lm,
                            const lcn_lsh_params *lsh, void *workspace, size_t workspace_bytes, void *hip_stream,
                            size_t *bytes_needed, lcn_handle *out);

lcn_status lcn_build(const void *X, int64_t n, const void *Y, int64_t m, int32_t d, int32_t dtype, const float *a,
                     const float *b, float lambda, int32_t cost, int32_t mode, const lcn_landmark_params *lm,
                     const lcn_lsh_params *lsh, void *workspace, size_t workspace_bytes, void *hip_stream,
                     size_t *bytes_needed, lcn_handle *out)
{
    if (!out) return LCN_ERR_INVALID_ARG;
    *out = nullptr;
    try {   // host containers are the only things in there that can throw: out of host memory
        return build_one(X, n, Y, m, d, dtype, a, b, lambda, cost, mode, lm, lsh, workspace, workspace_bytes, hip_stream,
                         bytes_needed, out);
    } catch (...) {
        *out = nullptr;
        return LCN_ERR_ALLOC;
    }
}

static lcn_status build_one(const void *X, int64_t n, const void *Y, int64_t m, int32_t d, int32_t dtype, const float *a,
                            const float *b, float lambda, int32_t cost, int32_t mode, const lcn_landmark_params *lm,
                            const lcn_lsh_params *lsh, void *workspace, size_t workspace_bytes, void *hip_stream,
                            size_t *bytes_needed, lcn_handle *out)
{
    *out = nullptr;
    if (!X || !Y || !a || !b || !workspace || ((uintptr_t)workspace & 255)) return LCN_ERR_INVALID_ARG;
    lcn_status st = check_params(n, m, d, dtype, lambda, cost, mode, lm, lsh);
    if (st != LCN_OK) return st;

    Handle *hp = new (std::nothrow) Handle{};
    if (!hp) return LCN_ERR_ALLOC;
    Handle &h = *hp;
    struct Guard {
        Handle *p;
        ~Guard()
        {
            if (p) {
                if (p->ev0) (void)hipEventDestroy(p->ev0);
                if (p->ev1) (void)hipEventDestroy(p->ev1);
                delete p;
            }
        }
    } guard{hp};

    fill_shape(h, n, m, d, mode, lm, lsh);
    h.in_dtype = dtype;
    h.cost = cost;
    h.lambda = (double)lambda;
    h.ridge = uses_landmarks(mode) ? lm->ridge : 0.0;
    h.stream = (hipStream_t)hip_stream;
    h.ws = (char *)workspace;
    h.ws_bytes = workspace_bytes;
    bool build_overlap = true;
    {
        const char *env = getenv("LCN_PASS_GRID");
        h.grid_cap = env ? atoi(env) : 0;
        env = getenv("LCN_EXACT_ASSIGN_ONLY");
        h.exact_assign_only = env ? atoi(env) : 0;
        env = getenv("LCN_FUSED_REDUCE");
        h.fused_reduce = env ? atoi(env) : 1;
        env = getenv("LCN_WAIT_TICKS");
        h.wait_ticks = env ? strtoull(env, nullptr, 10) : 20000000ull;
        env = getenv("LCN_DOUBLE_FIRST_SWEEP");
        h.double_first = env ? atoi(env) : 1;
        env = getenv("LCN_BUILD_OVERLAP");
        build_overlap = env ? atoi(env) != 0 : true;
        h.cus = device_compute_units();
    }
    Builder B(h, lm, lsh, cost, mode);   // after the handle's guard: it is torn down first
    layout(h, B.bump, B.sc);
    if (B.bump.used > workspace_bytes) {
        if (bytes_needed) lcn_workspace_bytes(n, m, d, mode, lm, lsh, 0, bytes_needed);
        return LCN_ERR_ALLOC;
    }
    // hash rounds first: their threads enqueue while this one goes on with the landmarks and factors
    if ((st = B.prepare(X, Y, a, b, dtype, build_overlap)) != LCN_OK) return st;
    if ((st = B.start_hash_rounds()) != LCN_OK) return st;
    if ((st = B.landmarks()) != LCN_OK) return st;
    if ((st = B.factors()) != LCN_OK) return st;
    if ((st = B.structure(bytes_needed)) != LCN_OK) return st;
    if ((st = B.values_and_state()) != LCN_OK) return st;

    h.magic = HANDLE_MAGIC;
    guard.p = nullptr;
    *out = (lcn_handle)hp;
    return LCN_OK;
}

lcn_status sinkhorn_run(lcn_handle hh, int32_t iters)
{
    if (iters < 0) return LCN_ERR_INVALID_ARG;
    if (is_batched_handle(hh)) return batched_run(hh, iters);
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    HIPCHK(hipEventRecord(h.ev0, h.stream));
    // per iteration: u from y = W v (produces z = U^T u), then v from z (produces y)
    HIPCHK(launch_update_sweeps(h, iters, h.stream));
    HIPCHK(hipEventRecord(h.ev1, h.stream));
    lcn_status st = status_from_counters(h);
    if (st == LCN_ERR_DEVICE) return st;
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, h.ev0, h.ev1));
    h.last_ms = ms;   // h.last_launches: set by launch_update_sweeps
    return st;
}

static lcn_status query(Handle &h, float *row_dev, float *col_dev, double q[4])
{
    HIPCHK(launch_pass(h, 0, PASS_QUERY, 0, 1, row_dev, h.stream));  // acc_out is only read (its exponent slot)
    HIPCHK(launch_pass(h, 1, PASS_QUERY, 1, 0, col_dev, h.stream));
    HIPCHK(hipMemcpyAsync(q, h.query_out, 4 * sizeof(double), hipMemcpyDeviceToHost, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status transport_cost(lcn_handle hh, double *d_host)
{
    if (!d_host) return LCN_ERR_INVALID_ARG;
    if (is_batched_handle(hh)) return batched_query(hh, d_host, nullptr, nullptr, nullptr);
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    double q[4];
    lcn_status st = query(h, nullptr, nullptr, q);
    if (st != LCN_OK) return st;
    *d_host = h.lambda * (q[0] + q[2]);
    return LCN_OK;
}

lcn_status plan_marginals(lcn_handle hh, float *row_dev, float *col_dev, double *l1_residual_host)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    double q[4];
    lcn_status st = query(h, row_dev, col_dev, q);
    if (st != LCN_OK) return st;
    if (l1_residual_host) *l1_residual_host = q[1] + q[3];
    return LCN_OK;
}

lcn_status lcn_get_scalings(lcn_handle hh, float *log_u_dev, float *log_v_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (log_u_dev)
        HIPCHK(hipMemcpyAsync(log_u_dev, h.log_u, sizeof(float) * (size_t)h.n, hipMemcpyDeviceToDevice, h.stream));
    if (log_v_dev)
        HIPCHK(hipMemcpyAsync(log_v_dev, h.log_v, sizeof(float) * (size_t)h.m, hipMemcpyDeviceToDevice, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_set_scalings(lcn_handle hh, const float *log_u_dev, const float *log_v_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    if (!log_u_dev || !log_v_dev) return LCN_ERR_INVALID_ARG;
    Handle &h = *(Handle *)hh;
    HIPCHK(hipMemcpyAsync(h.log_u, log_u_dev, sizeof(float) * (size_t)h.n, hipMemcpyDeviceToDevice, h.stream));
    HIPCHK(hipMemcpyAsync(h.log_v, log_v_dev, sizeof(float) * (size_t)h.m, hipMemcpyDeviceToDevice, h.stream));
    lcn_status st = init_state(h);
    if (st != LCN_OK) return st;
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_get_landmarks(lcn_handle hh, float *L_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (h.l == 0) return LCN_ERR_STATE;
    if (!L_dev) return LCN_ERR_INVALID_ARG;
    HIPCHK(hipMemcpyAsync(L_dev, h.L, sizeof(float) * (size_t)h.l * h.d, hipMemcpyDeviceToDevice, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_get_buckets(lcn_handle hh, int32_t *bucket_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (h.R == 0) return LCN_ERR_STATE;
    if (!bucket_dev) return LCN_ERR_INVALID_ARG;
    HIPCHK(hipMemcpyAsync(bucket_dev, h.bucket, sizeof(int32_t) * (size_t)h.R * (h.n + h.m), hipMemcpyDeviceToDevice,
                          h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_get_csr(lcn_handle hh, int64_t *nnz_host, int64_t *rowptr_dev, int32_t *colidx_dev, float *val_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (h.R == 0) return LCN_ERR_STATE;
    if (!rowptr_dev) return LCN_ERR_INVALID_ARG;
    HIPCHK(launch_csr_count(h, (long long *)rowptr_dev, h.stream));
    HIPCHK(launch_scan_i64((long long *)rowptr_dev, h.n, h.stream));
    long long total = 0;
    HIPCHK(hipMemcpyAsync(&total, rowptr_dev + h.n, sizeof(long long), hipMemcpyDeviceToHost, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    if (nnz_host) *nnz_host = total;
    if (colidx_dev) {
        HIPCHK(launch_csr_fill(h, (const long long *)rowptr_dev, colidx_dev, val_dev, h.stream));
        HIPCHK(hipStreamSynchronize(h.stream));
    }
    return LCN_OK;
}

lcn_status lcn_get_factors(lcn_handle hh, float *U_dev, float *Wt_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (h.l == 0) return LCN_ERR_STATE;
    const size_t w = sizeof(float) * (size_t)h.l, pitch = sizeof(float) * (size_t)h.lp;
    if (U_dev) HIPCHK(hipMemcpy2DAsync(U_dev, w, h.U, pitch, w, (size_t)h.n, hipMemcpyDeviceToDevice, h.stream));
    if (Wt_dev) HIPCHK(hipMemcpy2DAsync(Wt_dev, w, h.Wt, pitch, w, (size_t)h.m, hipMemcpyDeviceToDevice, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

static size_t backward_scratch(const Handle &h)
{
    const size_t rowptr = ((sizeof(long long) * (size_t)(h.n + 1)) + 255) / 256 * 256;
    const size_t rec = ((sizeof(float) * (size_t)(h.nnz_stored + 64)) + 255) / 256 * 256;
    return rowptr + 2 * rec;
}

lcn_status lcn_backward_scratch_bytes(lcn_handle hh, size_t *bytes)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    if (!bytes) return LCN_ERR_INVALID_ARG;
    const Handle &h = *(Handle *)hh;
    *bytes = h.R > 0 ? backward_scratch(h) : 0;
    return LCN_OK;
}

lcn_status lcn_backward(lcn_handle hh, float *gU_dev, float *gWt_dev, float *gsp_dev, float *gnys_dev,
                        void *scratch_dev, size_t scratch_bytes)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if ((gU_dev || gWt_dev) && h.l == 0) return LCN_ERR_STATE;
    if (gsp_dev && h.R == 0) return LCN_ERR_STATE;
    if (gnys_dev && (h.R == 0 || h.l == 0)) return LCN_ERR_STATE;
    if (gsp_dev || gnys_dev) {   // checked before anything is launched: an error leaves every output untouched
        if (!scratch_dev || ((uintptr_t)scratch_dev & 255)) return LCN_ERR_INVALID_ARG;
        if (scratch_bytes < backward_scratch(h)) return LCN_ERR_ALLOC;
    }
    if (gU_dev || gWt_dev) HIPCHK(launch_backward_factors(h, gU_dev, gWt_dev, h.stream));
    if (gsp_dev || gnys_dev) {
        const size_t rowptr_bytes = ((sizeof(long long) * (size_t)(h.n + 1)) + 255) / 256 * 256;
        const size_t rec_bytes = ((sizeof(float) * (size_t)(h.nnz_stored + 64)) + 255) / 256 * 256;
        long long *rowptr = (long long *)scratch_dev;
        float *rec_sp = (float *)((char *)scratch_dev + rowptr_bytes);
        float *rec_nys = (float *)((char *)scratch_dev + rowptr_bytes + rec_bytes);
        HIPCHK(launch_csr_count(h, rowptr, h.stream));
        HIPCHK(launch_scan_i64(rowptr, h.n, h.stream));
        if (h.log_domain)
            HIPCHK(launch_backward_log(h, rec_sp, h.stream));
        else
            HIPCHK(launch_backward_pattern(h, gsp_dev ? rec_sp : nullptr, gnys_dev ? rec_nys : nullptr, h.stream));
        HIPCHK(launch_csr_values(h, gsp_dev ? rec_sp : nullptr, gnys_dev ? rec_nys : nullptr, rowptr, gsp_dev, gnys_dev,
                                 h.stream));
    }
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_backward_static(lcn_handle hh, float *gU_dev, float *gWt_dev, float *gsp_dev, float *gnys_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    const Handle &h = *(Handle *)hh;
    void *ptr = nullptr;
    if ((gsp_dev || gnys_dev) && h.R > 0) {
        if (backward_scratch(h) > (size_t)LCN_STATIC_SCRATCH_BYTES) return LCN_ERR_ALLOC;
        const lcn_status st = static_scratch(&ptr);
        if (st != LCN_OK) return st;
    }
    // every word of the scratch that is read is written first by the same call (row pointers by the
    // count and scan, the two record arrays by the pattern kernels): nothing has to start at zero
    return lcn_backward(hh, gU_dev, gWt_dev, gsp_dev, gnys_dev, ptr, ptr ? (size_t)LCN_STATIC_SCRATCH_BYTES : 0);
}

lcn_status lcn_plan_rows(lcn_handle hh, int64_t i0, int64_t nrows, float *out_dev)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (!out_dev || i0 < 0 || nrows < 0 || i0 + nrows > h.n) return LCN_ERR_INVALID_ARG;
    if (nrows == 0) return LCN_OK;
    if (h.l > 0)
        HIPCHK(launch_plan_nystrom(h, i0, nrows, out_dev, h.stream));
    else
        HIPCHK(hipMemsetAsync(out_dev, 0, sizeof(float) * (size_t)nrows * (size_t)h.m, h.stream));
    if (h.R > 0) HIPCHK(launch_plan_sparse(h, i0, nrows, out_dev, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    return LCN_OK;
}

lcn_status lcn_get_info(lcn_handle hh, lcn_info *info)
{
    if (!valid(hh)) return LCN_ERR_STATE;
    if (!info) return LCN_ERR_INVALID_ARG;
    Handle &h = *(Handle *)hh;
    unsigned long long c[6];
    HIPCHK(hipMemcpyAsync(c, h.counters, sizeof(c), hipMemcpyDeviceToHost, h.stream));
    HIPCHK(hipStreamSynchronize(h.stream));
    if (c[5]) return LCN_ERR_DEVICE;  // a sweep gave up waiting for its totals
    info->n = h.n;
    info->m = h.m;
    info->d = h.d;
    info->l = h.l;
    info->rounds = h.R;
    info->buckets = h.b;
    info->nnz_stored = h.nnz_stored;
    info->nnz_unique = h.nnz_unique;
    info->nonpositive = (int64_t)c[0];
    info->empty_rows = (int64_t)c[1];
    info->empty_cols = (int64_t)c[2];
    info->workspace_used = h.ws_used;
    info->undecided_last = h.undecided_last;
    return LCN_OK;
}

lcn_status lcn_last_error_counts(lcn_handle hh, int64_t *nonpositive, int64_t *empty_rows, int64_t *empty_cols)
{
    unsigned long long c[6] = {0, 0, 0, 0, 0, 0};
    if (is_batched_handle(hh)) {
        const lcn_status st = batched_counts(hh, c);
        if (st != LCN_OK) return st;
    } else {
        if (!valid(hh)) return LCN_ERR_STATE;
        Handle &h = *(Handle *)hh;
        HIPCHK(hipMemcpyAsync(c, h.counters, sizeof(c), hipMemcpyDeviceToHost, h.stream));
        HIPCHK(hipStreamSynchronize(h.stream));
    }
    if (nonpositive) *nonpositive = (int64_t)c[0];
    if (empty_rows) *empty_rows = (int64_t)c[1];
    if (empty_cols) *empty_cols = (int64_t)c[2];
    return c[5] ? LCN_ERR_DEVICE : LCN_OK;   // a sweep gave up waiting for its totals
}

lcn_status lcn_last_run_timing(lcn_handle hh, float *ms_host, int32_t *launches_host)
{
    if (is_batched_handle(hh)) return batched_timing(hh, ms_host, launches_host);
    if (!valid(hh)) return LCN_ERR_STATE;
    Handle &h = *(Handle *)hh;
    if (ms_host) *ms_host = h.last_ms;
    if (launches_host) *launches_host = h.last_launches;
    return LCN_OK;
}

void lcn_destroy(lcn_handle hh)
{
    if (is_batched_handle(hh)) {
        batched_destroy(hh);
        return;
    }
    if (!valid(hh)) return;
    Handle *h = (Handle *)hh;
    (void)hipStreamSynchronize(h->stream);
    (void)hipEventDestroy(h->ev0);
    (void)hipEventDestroy(h->ev1);
    h->magic = 0;
    delete h;
}

const char *lcn_status_string(int32_t status)
{
    switch (status) {
        case LCN_OK: return "ok";
        case LCN_ERR_INVALID_ARG: return "invalid argument";
        case LCN_ERR_ALLOC: return "workspace too small";
        case LCN_ERR_DEVICE: return "HIP error";
        case LCN_ERR_STATE: return "bad handle or call not available in this mode";
        case LCN_ERR_SINGULAR: return "landmark kernel matrix is not positive definite";
        case LCN_ERR_NONPOSITIVE: return "non-positive kernel-vector product";
        case LCN_WARN_NO_SUPPORT: return "sparse kernel has rows or columns without entries";
        case LCN_ERR_RANGE: return "a scaling grew by more than e^43 within one iteration";
        default: return "unknown status";
    }
}

}  // extern "C"
