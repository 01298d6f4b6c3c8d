// Internal declarations shared by the HIP translation units of libadacons.
// Nothing here is visible across the C ABI (include/adacons.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adacons.h"

namespace adacons {

constexpr int kNMax = ADACONS_N_MAX;
constexpr int kBlock = 256;  // threads per workgroup (4 wavefronts of 64) in every kernel
constexpr int kWave = 64;

// Device-resident part of a coefficient stream (one per adacons_state).
struct DevState {
    // EMA of the order statistics, sorted order (Eq. 11): two copies, m[parity] is the current one.
    // Launches in which one workgroup updates the state while others still read it (the short path:
    // stage A2 inside stage A3) read m[parity ^ 1] and write m[parity] after stage A1 flipped `parity`;
    // every other update rewrites m[parity] in place.
    double m[2][kNMax];
    double gamma[kNMax];     // weights applied by the last aggregation (Eq. 12-13)
    double a_raw[kNMax];     // first-order coefficients a_i (Eq. 7)
    double a_smooth[kNMax];  // after the sorted EMA, redistributed to the workers (Eq. 11)
    float gamma32[kNMax];    // gamma rounded for the weighted-sum kernel
    unsigned long long step; // number of coefficient updates so far
    unsigned numeric_flags;  // ADACONS_NUM_* of the last update
    unsigned parity;         // which copy of m is current (0 or 1)
};
__device__ inline double *current_m(DevState *ds) { return ds->m[ds->parity & 1u]; }
__device__ inline const double *current_m(const DevState *ds) { return ds->m[ds->parity & 1u]; }
static_assert(sizeof(DevState) % sizeof(unsigned) == 0, "DevState is cleared word by word");

struct CoeffParams {
    int N;
    double beta;
    unsigned flags;
};

// Where stage A1 leaves its results and what stage A2 works on.
struct GramWork {
    double *partials;  // [rows][N(N+1)/2], one row per workgroup
    double *K;         // [N][N]
    DevState *ds;
    CoeffParams cp;
};

__host__ __device__ inline int num_pairs(int N) { return N * (N + 1) / 2; }
constexpr int kFinishMaxN = 44;   // largest N whose packed Gram row, N (N + 1) / 2 sums, one workgroup of 1024 threads reduces
// Position of (i, j), i <= j, in the row-major packed upper triangle.
__host__ __device__ inline int pair_index(int i, int j, int N) { return i * N - (i * (i - 1)) / 2 + (j - i); }

struct LaunchShape {
    int num_cu;
    int blocks_per_cu;  // <= 0: let the launcher decide
    int max_rows;       // capacity of the partials workspace in rows
    int cached_head_mb; // stage A1: MiB at the head of G read with cache-allocating loads; < 0: all
    int gram_products;  // stage A1, 8 < N <= 64, fp32: value of ADACONS_TUNE_GRAM_PRODUCTS
    int wsum_park_kb;   // stage A3: value of ADACONS_TUNE_WSUM_PARK_KB (LDS for parked output tiles; 0: store tile by tile)
    int wsum_row_slices; // stage A3: value of ADACONS_TUNE_WSUM_ROW_SLICES
    bool short_path;    // two launches: stage A1 flips the state's parity and leaves the partial rows to stage A3
};

// gram.hip
hipError_t launch_gram(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                       const LaunchShape &shape, const GramWork &want, bool with_coeffs, hipStream_t stream,
                       hipEvent_t between = nullptr,  // `between`: recorded after the main Gram kernel
                       int *rows_out = nullptr);      // short path (shape.short_path): the number of partial rows written
hipError_t launch_coeffs(const CoeffParams &cp, double *K, DevState *ds, hipStream_t stream);
int gram_rows_needed(int N, int num_cu);
hipError_t launch_clear_state(DevState *ds, double *K, int nn, hipStream_t stream);  // K may be NULL
hipError_t launch_state_load(DevState *ds, int N, const double *m_in, hipStream_t stream);
hipError_t launch_state_store(const DevState *ds, int N, double *m_out, double *coeffs, unsigned *numeric_flags,
                              hipStream_t stream);  // coeffs (3 N doubles) and numeric_flags may be NULL

// stats.hip: A1 reduced to diag K and its row sums, then A2 (N > 8)
hipError_t launch_stats(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok, const LaunchShape &shape,
                        double *partials, DevState *ds, const CoeffParams &cp, hipStream_t stream,
                        hipEvent_t between = nullptr,
                        int *rows_out = nullptr);   // short path (shape.short_path): the number of partial rows written

// api.hip: record the thread-local text adacons_last_error() returns; gives back `s`
adacons_status set_error(adacons_status s, const char *fmt, ...);

// worker.hip
hipError_t launch_pair_stats(const void *x, const void *y, int64_t d, adacons_dtype dtype, int num_cu,
                             int max_rows, double *partials, double *stats, hipStream_t s);
hipError_t launch_coeffs_from_stats(const double *q, const double *r, DevState *ds, const CoeffParams &cp,
                                    hipStream_t s);
hipError_t launch_scale(void *g, int64_t d, adacons_dtype dtype, int num_cu, const float *gamma, hipStream_t s);

// wsum.hip
hipError_t launch_wsum(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                       const LaunchShape &shape, const float *gamma, float *out, hipStream_t stream,
                       bool apply = false, float lr = 0.f);  // apply: out -= lr * sum
// Whether launch_wsum takes the row-slice kernel for N rows of ngroups 128-bit column groups.
bool row_slices_pay(int N, int64_t ngroups, const LaunchShape &shape);
// Short path (16-byte aligned rows): stage A3 whose every workgroup first adds the nrows partial rows of
// stage A1 and runs stage A2 for itself; workgroup 0 writes K and the state.  N <= 8: wsum_short_kernel.
// N > 8: the row-slice kernel; stats_rows: the rows are those of the statistics-only pass (2 N doubles, any
// N); otherwise packed Gram rows (N <= 44).
hipError_t launch_wsum_short(const void *G, int N, int64_t d, adacons_dtype dtype, const LaunchShape &shape,
                             const GramWork &work, int nrows, bool stats_rows, float *out, hipStream_t stream,
                             bool apply = false, float lr = 0.f);

}  // namespace adacons
