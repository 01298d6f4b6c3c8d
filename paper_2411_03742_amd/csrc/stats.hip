// Stage A1 reduced to what the coefficients consume: q_i = ||g_i||^2 and r_i = <g_i, sum_j g_j>
// (the norm and the dot product with the all-reduced gradient that steps 1-2 of Algorithm 1
// compute per worker; Eq. 7 needs nothing else of K = G G^T).  O(N) arithmetic per column
// instead of the Gram matrix' N (N + 1) / 2 products, so the pass stays bound by memory for every
// N.  Selected by ADACONS_TUNE_STATS_ONLY for N > 8; K is then not produced.
//
// A wavefront takes a chunk of 16 * VECW columns of all N rows with 128-bit loads that cover four
// rows by 256 contiguous bytes each (lane l: row 4 j + l / 16 in load j, column group l % 16), so
// the chunk lives in the registers of the wavefront and is read from memory once (N > 64: eight rows
// by 128 bytes per load and chunks of 8 * VECW columns, which keeps the register count of N <= 64):
//   s   = column sums over the rows: in-lane over the loads, then across the lane groups;
//   q_i += <v_i, v_i>, r_i += <v_i, s> per lane for each of its rows, all in fp64.
// The next chunk is in flight while the current one is summed.  At the end the sixteen lanes of a
// group are added in a fixed butterfly order, the four wavefronts in index order: one partial row
// [q_0 .. q_{N-1}, r_0 .. r_{N-1}] per workgroup, reduced by stats_finish_kernel, which then runs
// the coefficient update (stage A2).  No atomics; results do not depend on scheduling.
#include "adacons_internal.h"
#include "coeff_device.h"
#include "device_util.h"

#include <type_traits>

namespace adacons {

namespace {

// NT = ceil(N / 16): the kernel is compiled for 16, 32, ..., 128 rows.  One load instruction covers
// kRowsPerLoad rows (4 up to 64 rows, 8 above), so a chunk takes kLoads = 16 NT / kRowsPerLoad loads.
// A wavefront takes kSuper consecutive chunks at a time so that about sixteen loads are in flight
// per buffer for every NT.
// (bf16 needs twice the arithmetic per byte and is bound by the fp64 units: fewer chunks in flight
// keep its register count at two wavefronts per SIMD).
template <int NT, typename T> struct StatsShape {
    static constexpr int kRowsPerLoad = (NT > 4) ? 8 : 4;
    static constexpr int kLanesPerRow = kWave / kRowsPerLoad;   // lanes (column groups) side by side in one row
    static constexpr int kLoads = 16 * NT / kRowsPerLoad;
    static constexpr int kSuper = (sizeof(T) == 4) ? (kLoads <= 4 ? 4 : (kLoads <= 8 ? 2 : 1)) : (kLoads <= 4 ? 2 : 1);
};

template <int NT, typename T>
__global__ void __launch_bounds__(kBlock, (StatsShape<NT, T>::kLoads * VecWidth<T>::value > 48) ? 1 : 2)
stats_wave_kernel(const T *__restrict__ G, int N, int64_t d, int64_t dcols, int64_t nchunks, int64_t cached_chunks,
                  double *__restrict__ partials, DevState *flip) {
    // flip (or NULL): the short path's stage A3 reads the state copy this launch retires (see gram_vec_kernel)
    if (flip && blockIdx.x == 0 && threadIdx.x == 0) flip->parity ^= 1u;
    constexpr int VECW = VecWidth<T>::value;
    constexpr int kLoads = StatsShape<NT, T>::kLoads;
    constexpr int kSuper = StatsShape<NT, T>::kSuper;
    constexpr int RPL = StatsShape<NT, T>::kRowsPerLoad, LPR = StatsShape<NT, T>::kLanesPerRow;
    constexpr int64_t kChunk = LPR * VECW;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, cl = lane % LPR;   // load j: row RPL j + grp, column group cl of the chunk

    double qacc[kLoads], racc[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) qacc[j] = racc[j] = 0.0;

    // branch-free loads: rows >= N and columns >= dcols (a multiple of VECW; rows are d elements apart)
    // read a clamped address and are zeroed
    auto load_chunk = [&](u32x4 (&dst)[kSuper][kLoads], int64_t ch, auto stream) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kSuper; ++u)
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                const int row = RPL * j + grp;
                const int64_t col = (ch * kSuper + u) * kChunk + (int64_t)cl * VECW;
                const bool live = row < N && col < dcols;
                const int rowc = row < N ? row : N - 1;
                const int64_t colc = col < dcols ? col : dcols - VECW;
                const gu32x4 *src = reinterpret_cast<const gu32x4 *>(G + (int64_t)rowc * d + colc);
                u32x4 x;
                if constexpr (decltype(stream)::value) x = __builtin_nontemporal_load(src);
                else x = *src;
                dst[u][j] = live ? x : u32x4{0u, 0u, 0u, 0u};
            }
    };
    // fp64 throughout (exact products, sums rounded at 2^-53): for fp32 inputs the pass stays bound
    // by memory; for bf16 inputs (twice the columns per byte) the fp64 units become the limit
    auto consume_one = [&](const u32x4 (&src)[kLoads]) __attribute__((always_inline)) {
        double s[VECW];
#pragma unroll
        for (int c = 0; c < VECW; ++c) s[c] = 0.0;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            float v[VECW];
            widen_bits<T>(src[j], v);
#pragma unroll
            for (int c = 0; c < VECW; ++c) s[c] += (double)v[c];
        }
#pragma unroll
        for (int c = 0; c < VECW; ++c) {
#pragma unroll
            for (int off = LPR; off < kWave; off <<= 1) s[c] += __shfl_xor(s[c], off, 64);
        }
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            float v[VECW];
            widen_bits<T>(src[j], v);
#pragma unroll
            for (int c = 0; c < VECW; ++c) {
                const double x = (double)v[c];
                qacc[j] = fma(x, x, qacc[j]);
                racc[j] = fma(x, s[c], racc[j]);
            }
        }
    };

    auto consume = [&](const u32x4 (&src)[kSuper][kLoads]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kSuper; ++u) consume_one(src[u]);
    };

    const int64_t wstride = (int64_t)gridDim.x * (kBlock / kWave);
    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t ch = (int64_t)slot * (kBlock / kWave) + wave;
    u32x4 bufA[kSuper][kLoads], bufB[kSuper][kLoads];
    // two chunks: while one buffer is summed the other one is being filled; past the end the last
    // chunk is loaded again and never used
    auto two_steps = [&](auto stream) __attribute__((always_inline)) {
        int64_t chn = ch + wstride;
        load_chunk(bufB, chn < nchunks ? chn : nchunks - 1, stream);
        consume(bufA);
        ch = chn;
        if (ch >= nchunks) return;
        chn = ch + wstride;
        load_chunk(bufA, chn < nchunks ? chn : nchunks - 1, stream);
        consume(bufB);
        ch = chn;
    };
    // Chunks below cached_chunks are fetched with ordinary loads (the head of G stays in the
    // memory-side cache for the second pass), the rest with non-temporal ones.  Two loops, not a
    // branch per chunk: loads that differ only in that hint would be merged into one kind.
    if (ch < nchunks) load_chunk(bufA, ch, std::false_type{});
    while (ch < nchunks && ch + 2 * wstride < cached_chunks) two_steps(std::false_type{});
    while (ch < nchunks) two_steps(std::true_type{});

    // lanes of one group (same rows, different columns): fixed butterfly; then wavefronts in order
    __shared__ double lds[kBlock / kWave][2 * kNMax];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        double q = qacc[j], r = racc[j];
#pragma unroll
        for (int off = LPR / 2; off >= 1; off >>= 1) {
            q += __shfl_xor(q, off, 64);
            r += __shfl_xor(r, off, 64);
        }
        if (cl == 0) {
            lds[wave][RPL * j + grp] = q;
            lds[wave][kNMax + RPL * j + grp] = r;
        }
    }
    __syncthreads();
    const int tid = threadIdx.x;
    if (tid < 2 * N) {
        const int e = tid < N ? tid : kNMax + (tid - N);
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) tot += lds[w][e];
        partials[(size_t)blockIdx.x * (2 * N) + tid] = tot;
    }
}

// One workgroup: adds the partial rows in a fixed order (interleaved sub-sums, then slices in
// order) and runs the coefficient update on the 2 N totals.
constexpr int kStatsFinishBlock = 1024;
__global__ void __launch_bounds__(kStatsFinishBlock)
stats_finish_kernel(const double *partials, int nrows, DevState *ds, CoeffParams cp) {
    __shared__ double lds[kStatsFinishBlock];
    const int N = cp.N, tid = threadIdx.x;
    const double m_old = (tid < N) ? current_m(ds)[tid] : 0.0;
    double q, r;
    reduce_stat_rows<kStatsFinishBlock>(partials, nrows, N, lds, q, r);
    update_coefficients_from_stats(q, r, ds, cp, lds, m_old);
}

// The last d - col0 < 8 columns, which no whole 128-bit group covers: one more partial row.
template <typename T>
__global__ void __launch_bounds__(kNMax)
stats_edge_kernel(const T *__restrict__ G, int N, int64_t d, int64_t col0, double *__restrict__ row_out) {
    const int i = threadIdx.x;
    if (i >= N) return;
    const int ncols = (int)(d - col0);
    double q = 0.0, r = 0.0;
    for (int c = 0; c < ncols; ++c) {
        double s = 0.0;
        for (int j = 0; j < N; ++j) {
            float v[1];
            load_vec<T, 1, false>(G + (int64_t)j * d + col0 + c, v);
            s += (double)v[0];
        }
        float x[1];
        load_vec<T, 1, false>(G + (int64_t)i * d + col0 + c, x);
        q = fma((double)x[0], (double)x[0], q);
        r = fma((double)x[0], s, r);
    }
    row_out[i] = q;
    row_out[N + i] = r;
}

template <int NT, typename T>
hipError_t run_stats(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape, double *partials,
                     DevState *ds, hipStream_t s, int *grid_out) {
    static const int occ = [] {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, stats_wave_kernel<NT, T>, kBlock, 0) != hipSuccess || nb < 1)
            nb = 1;
        return nb;
    }();
    const int64_t chunk = StatsShape<NT, T>::kLanesPerRow * VecWidth<T>::value * StatsShape<NT, T>::kSuper;   // columns a wavefront takes at a time
    const int64_t nchunks = (dcols + chunk - 1) / chunk;
    const int waves = kBlock / kWave;
    int per_cu = shape.blocks_per_cu > 0 ? shape.blocks_per_cu : 2;
    if (per_cu > occ) per_cu = occ;
    int64_t grid = (int64_t)shape.num_cu * per_cu;
    const int64_t work = (nchunks + waves - 1) / waves;
    if (grid > work) grid = work;
    if (grid > shape.max_rows) grid = shape.max_rows;
    if (grid < 1) grid = 1;
    *grid_out = (int)grid;
    // Non-temporal loads past the cached head only when every row starts on a 128-byte line: with
    // rows shifted against the lines the 256-byte pieces share lines with their neighbours, and
    // lines that are not kept in L2 are fetched twice (measured slower).  cached_head_mb < 0:
    // ordinary loads only.
    const bool rows_on_lines = reinterpret_cast<uintptr_t>(G) % 128 == 0 && (d * (int64_t)sizeof(T)) % 128 == 0;
    int64_t cached_chunks = nchunks + 2 * grid * waves;   // beyond every prefetch
    if (shape.cached_head_mb >= 0 && rows_on_lines)
        cached_chunks = ((int64_t)shape.cached_head_mb << 20) / ((int64_t)N * chunk * (int64_t)sizeof(T));
    hipLaunchKernelGGL((stats_wave_kernel<NT, T>), dim3((unsigned)grid), dim3(kBlock), 0, s, static_cast<const T *>(G),
                       N, d, dcols, nchunks, cached_chunks, partials, shape.short_path ? ds : nullptr);
    return hipGetLastError();
}

template <typename T>
hipError_t dispatch_stats(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape, double *partials,
                          DevState *ds, hipStream_t s, int *grid_out) {
    switch ((N + 15) / 16) {
        case 1: return run_stats<1, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 2: return run_stats<2, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 3: return run_stats<3, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 4: return run_stats<4, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 5: return run_stats<5, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 6: return run_stats<6, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 7: return run_stats<7, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 8: return run_stats<8, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// The partial rows need 2 N doubles per workgroup (never more than the N (N + 1) / 2 of a Gram row for
// N >= 3).  Without 16-byte aligned rows (vec_ok false) the kernel covers the whole 128-bit groups of
// every row from element-aligned addresses and stats_edge_kernel adds a row for the columns left over.
// shape.short_path: stage A1 only (it flips the state's parity); *rows_out receives the number of partial
// rows, which stage A3 adds itself.
hipError_t launch_stats(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok, const LaunchShape &shape_in,
                        double *partials, DevState *ds, const CoeffParams &cp, hipStream_t stream, hipEvent_t between,
                        int *rows_out) {
    if (shape_in.short_path && (!vec_ok || !rows_out)) return hipErrorInvalidValue;
    const int64_t vec = (dtype == ADACONS_F32) ? 4 : 8;
    const int64_t dcols = vec_ok ? d : d / vec * vec;
    LaunchShape shape = shape_in;
    if (!vec_ok) {
        if (shape.max_rows < 2) return hipErrorInvalidValue;
        shape.max_rows -= 1;   // room for the edge row
    }
    int grid = 0;
    hipError_t e = (dtype == ADACONS_F32) ? dispatch_stats<float>(G, N, d, dcols, shape, partials, ds, stream, &grid)
                                          : dispatch_stats<bf16_bits>(G, N, d, dcols, shape, partials, ds, stream, &grid);
    if (e == hipSuccess && dcols < d) {
        double *row = partials + (size_t)grid * (2 * N);
        if (dtype == ADACONS_F32)
            hipLaunchKernelGGL(stats_edge_kernel<float>, dim3(1), dim3(kNMax), 0, stream, static_cast<const float *>(G),
                               N, d, dcols, row);
        else
            hipLaunchKernelGGL(stats_edge_kernel<bf16_bits>, dim3(1), dim3(kNMax), 0, stream,
                               static_cast<const bf16_bits *>(G), N, d, dcols, row);
        e = hipGetLastError();
        grid += 1;
    }
    if (e == hipSuccess && between) e = hipEventRecord(between, stream);
    if (e != hipSuccess) return e;
    if (shape.short_path) {
        *rows_out = grid;
        return hipSuccess;
    }
    hipLaunchKernelGGL(stats_finish_kernel, dim3(1), dim3(kStatsFinishBlock), 0, stream, partials, grid, ds, cp);
    return hipGetLastError();
}

}  // namespace adacons
