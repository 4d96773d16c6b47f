// Internal declarations shared by the HIP translation units of the LCN-Sinkhorn
// library.  Nothing here is part of the public ABI (see include/lcn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcn.h"

namespace lcn {

// One row (or column) of the sparse part in one hash round: `len` values that
// multiply `len` consecutive entries of the other side's bucket-ordered
// scaling vector starting at `vstart`.  A row's values of all rounds are stored
// back to back (round 0 first) starting at its row base.
struct Seg {
    int vstart;
    int len;
};

// Everything the half-iteration kernel needs for one side (rows of U with the
// row-major tiles, or rows of W^T with the transposed tiles).
struct PassSide {
    long long rows;         // n or m
    const float *F;         // rows x lp factor (U or W^T), zero padded to lp
    const float *vals;      // sparse values, one contiguous record per row of this side
    const int *meta;        // packed per-row metadata, meta_stride ints per row (see meta_kernel)
    int meta_stride;
    float *log_out;         // log u or log v (fp32 state that is reported)
    double *lin_out;        // u or v, linear, by original index
    double *perm_out;       // [R][rows] u or v in bucket order of each round
    const double *perm_in;  // [R][other] the other side's scaling in bucket order, then a slot that stays zero
    long long rows_in;      // rows of the other side
    const double *acc_in;   // lp + 1: y = W v (for rows of U) or z = U^T u (for rows of W^T), then its exponent
    double *acc_out;        // lp + 1: accumulated F^T out, then the exponent taken out of `out`
    double *shift_self;     // exponent taken out of this side's scaling vector (updated every sweep)
    float *marg_out;        // query mode: plan marginal of each row (nullable)
};

enum PassMode { PASS_UPDATE = 0, PASS_QUERY = 1, PASS_INIT = 2 };

// What the tile kernel of the sparse values needs to produce derivatives instead (lin_u == nullptr: values).
struct BackwardArgs {
    const double *lin_u = nullptr, *lin_v = nullptr;  // scalings with their exponents taken out
    const double *acc_y = nullptr, *acc_z = nullptr;  // accumulators; entry lp holds the exponent of v resp. u
    double lambda = 0.0;
    float *rec_sp = nullptr, *rec_nys = nullptr;      // outputs, layout of the row records of X
};

struct Handle;

// ---- structure build (kernels_structure.hip) -------------------------------
hipError_t launch_convert(const void *X, long long n, const void *Y, long long m, int d, int dtype, float *Z,
                          unsigned *range_flag, hipStream_t s);
hipError_t launch_gather_rows(const float *Z, int d, const long long *idx, int k, float *out, hipStream_t s);
// up to eight regions of 4-byte words set to zero by one launch
struct ClearRegions {
    unsigned *ptr[8];
    long long words[8];
    int count;
    void add(void *p, size_t bytes)
    {
        ptr[count] = (unsigned *)p;
        words[count++] = (long long)(bytes / 4);
    }
};
hipError_t launch_clear_regions(const ClearRegions &R, hipStream_t s);
hipError_t launch_assign_children(const float *Z, int d, const float *cent, long long parents, int branch,
                                  const int *nchild, const int *order, const int *chunks, int nchunks, double *centT,
                                  int32_t *out, hipStream_t s);
hipError_t launch_combine_hash(int32_t *acc, const int32_t *h, int b, int first, long long N, hipStream_t s);
hipError_t launch_kmeanspp(const float *Z, long long N, int d, int k, const unsigned long long *rnd, double *w,
                           unsigned long long *partial, int *picks, unsigned long long *state, float *cent,
                           hipStream_t s);
// exact rule for all points (list == nullptr) or for the listed ones
hipError_t launch_assign_kmeans(const float *Z, long long N, int d, const float *cent, int k, int32_t *out,
                                const int *list, const int *list_count, hipStream_t s);
// bf16 planes of a row-major fp32 matrix in matrix-instruction operand order (kernels_mfma.hip)
size_t split_plane_bytes(long long rows, int d);
hipError_t launch_split_planes(const float *src, long long rows, int d, int planes, void *out, hipStream_t s);
// MFMA filter: writes the assignment of every point and lists those it could not decide.
// Zt: planes of the points (zplanes of them); Ct: room for two planes of k centroids.
hipError_t launch_assign_filter(const void *Zt, int zplanes, long long N, int d, const float *cent, int k, void *Ct,
                                const double *zn, float *cn, unsigned *cmax_bits, int32_t *out, int *flagged,
                                int *pairs, int *nflagged, hipStream_t s);
bool filter_uses_pairs(int k);
// exact rule on two candidate centroids per listed point: pairs = (point, c1, c2) triples
hipError_t launch_assign_pairs(const float *Z, int d, const float *cent, int32_t *out, const int *pairs,
                               const int *pair_count, hipStream_t s);
hipError_t launch_assign_crosspolytope(const float *Z, long long N, int d, const float *Rm, int b, int32_t *out,
                                       hipStream_t s);
// counts2 / cursor2: [2][k] ints each, zero before the first update of a k-means run; order: [N], offs: [k] ints;
// part: kmeans_partial_elems(N, largest k, d) 64-bit words of scratch for the partial sums;
// `parity` alternates from update to update.  reset_a / reset_b (nullable) are cleared for the next
// assignment step.
hipError_t launch_kmeans_update(const float *Z, long long N, int d, const int32_t *assign, int k, int *counts2,
                                int *cursor2, int *order, int *offs, long long *part, int parity, float *cent,
                                unsigned *reset_a, int *reset_b, hipStream_t s);
size_t kmeans_partial_elems(long long N, int kmax, int d);

struct SortBuffers {
    int R, b;
    long long n, m;
    const int32_t *bucket;  // [R][n+m]
    int *hist;              // scratch [2][R][chunks][b]
    int chunks;             // max over sides
    int *totals;            // [2][R][b]
    int *off;               // [2][R][b+1]  (x side then y side)
    int *perm;              // x: [R][n] then y: [R][m]
    int *pos;               // x: [R][n] then y: [R][m]
    int *tile_off;          // [R*b + 1] start of each block in the list of 64x64 build tiles
    long long *totals_out;  // [2]: nnz_stored, build tiles
    Seg *seg_x;             // [R][n]
    Seg *seg_y;             // [R][m]
    long long *rowbase_x;   // [n + 1]
    long long *rowbase_y;   // [m + 1]
    int *meta_x;            // [n][meta_stride] packed per-row metadata for the sweeps
    int *meta_y;            // [m][meta_stride]
    int meta_stride;        // ints per record: 6 + 3 R rounded up to a multiple of 4
};
hipError_t launch_bucket_sort(const SortBuffers &B, hipStream_t s);
hipError_t launch_build_meta(const SortBuffers &B, const float *a, const float *b, hipStream_t s);
int meta_stride_for(int R);
int sort_chunks(long long n, long long m);

hipError_t launch_csr_count(const Handle &h, long long *rowcount, hipStream_t s);
hipError_t launch_scan_i64(long long *data, long long n, hipStream_t s);  // in-place exclusive scan, data[n] = total
hipError_t launch_csr_fill(const Handle &h, const long long *rowptr, int32_t *colidx, float *val, hipStream_t s);

// ---- factor build (kernels_factors.hip) ------------------------------------
hipError_t launch_sqnorms(const float *P, long long rows, int d, double *out, hipStream_t s);
// out[i][k] = exp(-c(P_i, Q_k) / lambda); P: rows x d, Q: cols x d.  Writes fp32 (ld = ldo) and/or fp64.
hipError_t launch_kernel_matrix(const float *P, long long rows, const float *Q, int cols, int d, int cost,
                                double lambda, const double *pn, const double *qn, float *out32, double *out64,
                                int ldo, hipStream_t s);
hipError_t launch_spd_inverse(double *A, int l, double ridge, double *Lm, double *Xm, double *Ainv, double *Dinv,
                              double *Tm, int *fail_flag, hipStream_t s);
// C (M x N, fp32, ld ldc) = A (M x K, fp64) * B (K x N, fp64)
hipError_t launch_gemm_f64(const double *A, const double *B, long long M, int N, int K, float *C32, int ldc,
                           hipStream_t s);
hipError_t launch_correction(const Handle &h, int ntiles, hipStream_t s);
// derivatives of the distance (Prop. 1): factor parts, and pattern parts in the layout of X's row records
hipError_t launch_backward_factors(const Handle &h, float *gU, float *gWt, hipStream_t s);
hipError_t launch_backward_pattern(const Handle &h, float *rec_sp, float *rec_nys, hipStream_t s);
hipError_t launch_backward_log(const Handle &h, float *rec_sp, hipStream_t s);
// rows of the plan as a dense block: Nystrom part (sets), then sparse part (adds; sets for kernels held as logs)
hipError_t launch_plan_nystrom(const Handle &h, long long i0, long long nrows, float *out, hipStream_t s);
hipError_t launch_plan_sparse(const Handle &h, long long i0, long long nrows, float *out, hipStream_t s);
// row records of X -> canonical CSR order (rowptr from launch_csr_count + launch_scan_i64)
hipError_t launch_csr_values(const Handle &h, const float *rec, const float *rec2, const long long *rowptr, float *val,
                             float *val2, hipStream_t s);

// ---- iteration (kernels_iter.hip) ------------------------------------------
hipError_t launch_pass(const Handle &h, int side, int mode, int acc_in, int acc_out, float *marg_out, hipStream_t s);
hipError_t launch_update_sweeps(Handle &h, int iters, hipStream_t s);
int device_compute_units();
int pass_grid(const Handle &h);

// ---- batched small problems (kernels_batched.hip) ---------------------------
bool is_batched_handle(const void *h);
lcn_status batched_run(void *h, int iters);
lcn_status batched_query(void *h, double *dist_host, double *resid_host, float *row_dev, float *col_dev);
lcn_status batched_timing(void *h, float *ms, int *launches);
lcn_status batched_counts(void *h, unsigned long long c[3]);
void batched_destroy(void *h);

struct Handle {
    uint32_t magic;
    long long n, m;
    int d, l, lp, R, b;
    int mode, cost, hash;
    int in_dtype;              // storage type X and Y were given in
    int hier_levels;           // levels of hierarchical k-means hashing (0 or 1: flat)
    int and_width;             // hashes per band of cross-polytope hashing (AND construction)
    int log_domain;            // kernel without signed parts (sparse, dense): values and vectors are logs
    double lambda, ridge;
    hipStream_t stream;
    char *ws;
    size_t ws_bytes, ws_used;

    // inputs (copies)
    float *Z;          // (n+m) x d fp32
    double *zn;        // squared norms of the rows of Z (cosine cost)
    float *a, *b_marg; // marginals
    // structure
    float *L;          // l x d landmarks
    int32_t *bucket;   // [R][n+m]
    SortBuffers sort;
    long long nnz_stored, nnz_unique;
    long long undecided_last;
    int ntiles;
    // factors
    float *U;          // n x lp
    float *Wt;         // m x lp
    float *vals_x;     // sparse values, one record per row of X
    float *vals_y;     // the same values, one record per row of Y
    // state
    float *log_u, *log_v;
    double *lin_u, *lin_v;
    double *perm_u, *perm_v;   // [R][n], [R][m]
    double *acc[2];            // lp + 2 each (last slot: scratch of the fused reduction): [0] y = W v, [1] z = U^T u, each followed by its exponent
    double *shift;             // [2]: exponent taken out of u and of v
    double *partial;           // [grid][lp + 3] per-workgroup partial sums of a sweep
    double *partial2;          // second buffer: consecutive sweeps alternate when the reduction is fused
    int fused_reduce;          // sweeps add up their predecessor's partial sums themselves
    int fresh;                 // the scalings have not been iterated since they were set: their exponents are stale
    unsigned long long wait_ticks;  // bound of a sweep's wait for its totals, in ticks of the 100 MHz clock (default 0.2 s)
    int double_first;          // run the first sweeps of a fresh state twice (on unless switched off for tests)
    int cus;                   // compute units of the device
    double *query_out;         // [2 sides][2]: sum r log u, sum |r - a|
    // [0] non-positive sums, [1] empty rows, [2] empty columns, [3] unique pairs, [4] input range flag,
    // [5] expired waits, [6] overflowed single-precision scaling copies, [8..15] counts of sweeps whose
    // results are discarded
    unsigned long long *counters;
    int grid;
    int grid_cap;              // upper bound on the workgroups of a sweep (0 = default)
    int exact_assign_only;     // skip the MFMA filter and decide every bucket by the exact rule

    hipEvent_t ev0, ev1;
    float last_ms;
    int last_launches;
};

constexpr uint32_t HANDLE_MAGIC = 0x4C434E31u;  // "LCN1"

}  // namespace lcn
