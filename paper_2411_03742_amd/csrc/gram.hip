// Stage A1 (K = G G^T) and stage A2 (coefficients, sorted momentum, normalisation).
//
// A1 computes every inner product <g_i, g_j> of Eq. 7 (third line) / the double sum of Eq. 8
// in one pass over G.  Two kernels:
//   gram_vec_kernel   N <= 8: one thread owns VEC consecutive columns of all N rows
//                     (N 128-bit loads in flight) and keeps the N(N+1)/2 sums in fp64 registers.
//   gram_mfma_kernel  8 < N <= 64: rows grouped in tiles of 16; one wavefront feeds
//                     v_mfma_f32_16x16x4_f32 with the same registers as A and B operand
//                     (K is G times its own transpose), fp32 tile accumulators flushed into
//                     fp64 every kFlush steps.
// Both are persistent grids; every workgroup writes one row of partial sums, there are no
// floating-point atomics, and the rows are added in a fixed order, so results are
// bit-identical from run to run for a given launch shape.
//
// A2 is a single workgroup (the last one of A1 to finish, or a launch of its own).
#include "adacons_internal.h"
#include "coeff_device.h"
#include "device_util.h"

#include <type_traits>

namespace adacons {

// ------------------------------------------------------------------------------------------
// Reduction of the partial rows and the coefficient update
// ------------------------------------------------------------------------------------------

// Unpack p (position in the packed upper triangle) into (i, j), i <= j.
__device__ __forceinline__ void unpack_pair(int p, int N, int &i, int &j) {
    int row = 0, left = p;
    while (left >= N - row) {
        left -= N - row;
        ++row;
    }
    i = row;
    j = row + left;
}

// K[i][j] = K[j][i] = sum over rows of partials[.][p]: min(blockDim.x / np, 32) interleaved sub-sums per
// pair, added in slice order.  One workgroup, N(N+1)/2 <= blockDim.x; lds >= blockDim.x doubles.
// When K_lds is given, K is also left there (N x N) for the coefficient update that follows.
__device__ void reduce_partial_rows(const double *partials, int nrows, int N, double *K, double *lds,
                                    double *K_lds = nullptr) {
    const int np = num_pairs(N);
    const int tid = threadIdx.x;
    // at most 32 slices: the slice sums are added one after the other by a single thread per pair
    const int slices = ((int)blockDim.x / np < 32) ? (int)blockDim.x / np : 32;
    const int s = tid / np, p = tid - s * np;
    if (s < slices) lds[s * np + p] = sum_rows(partials, np, p, s, slices, nrows);
    __syncthreads();
    if (tid < np) {
        double tot = 0.0;
        for (int q = 0; q < slices; ++q) tot += lds[q * np + tid];
        int i, j;
        unpack_pair(tid, N, i, j);
        K[(size_t)i * N + j] = tot;
        K[(size_t)j * N + i] = tot;
        if (K_lds) {
            K_lds[i * N + j] = tot;
            K_lds[j * N + i] = tot;
        }
    }
    __syncthreads();
}

// Called by every workgroup of a Gram kernel after its partial row is stored.  The workgroup
// that takes the last ticket reduces all rows (and runs A2 when asked).  No workgroup waits for
// another: every wave reaches the end of the kernel.
__device__ void gram_tail(const GramTail &tail, double *lds) {
    if (tail.mode == kGramPartialsOnly) return;
    __shared__ unsigned s_ticket;
    __threadfence();  // release: this workgroup's partial row is visible device-wide
    __syncthreads();
    if (threadIdx.x == 0) s_ticket = atomicAdd(&tail.ds->blocks_done, 1u);
    __syncthreads();
    if (s_ticket != gridDim.x - 1) return;
    __threadfence();  // acquire: see every other workgroup's row
    const double m_old = ((int)threadIdx.x < tail.cp.N) ? tail.ds->m[threadIdx.x] : 0.0;
    reduce_partial_rows(tail.partials, (int)gridDim.x, tail.cp.N, tail.K, lds);
    if (tail.mode == kGramFinishCoeffs) update_coefficients(tail.K, tail.ds, tail.cp, lds, m_old);
    if (threadIdx.x == 0) tail.ds->blocks_done = 0;  // ready for the next launch on this stream
}

// Reduction of the partial rows as a launch of its own (large N: more pairs than one workgroup
// has threads).  Workgroup c owns pairs [64 c, 64 c + 64); four interleaved sub-sums per pair.
__global__ void __launch_bounds__(kBlock) reduce_kernel(const double *partials, int nrows, int N, double *K) {
    __shared__ double lds[kBlock];
    const int np = num_pairs(N);
    const int pl = threadIdx.x & 63, s = threadIdx.x >> 6;
    const int p = blockIdx.x * 64 + pl;
    lds[s * 64 + pl] = (p < np) ? sum_rows(partials, np, p, s, 4, nrows) : 0.0;
    __syncthreads();
    if (s == 0 && p < np) {
        const double tot = ((lds[pl] + lds[64 + pl]) + lds[128 + pl]) + lds[192 + pl];
        int i, j;
        unpack_pair(p, N, i, j);
        K[(size_t)i * N + j] = tot;
        K[(size_t)j * N + i] = tot;
    }
}

// Reduction of the partial rows and (optionally) the coefficient update in one workgroup of
// kFinishBlock threads, for N(N+1)/2 <= kFinishBlock: the launch between the two streaming passes.
constexpr int kFinishBlock = 1024;
constexpr int kFinishMaxN = 44;  // largest N with N(N+1)/2 <= kFinishBlock
__global__ void __launch_bounds__(kFinishBlock)
finish_kernel(const double *partials, int nrows, double *K, DevState *ds, CoeffParams cp, int with_coeffs) {
    __shared__ double lds[kFinishBlock];
    __shared__ double K_lds[kFinishMaxN * kFinishMaxN];
    const double m_old = ((int)threadIdx.x < cp.N) ? ds->m[threadIdx.x] : 0.0;
    reduce_partial_rows(partials, nrows, cp.N, K, lds, K_lds);
    if (with_coeffs) update_coefficients(K_lds, ds, cp, lds, m_old);
}

// The coefficient update as a launch of its own (N > 44, after reduce_kernel).  Four threads share a
// row of K: each adds a quarter of it (elements j = quarter, quarter + 4, ...: neighbouring threads
// read neighbouring addresses, the loads of one thread are independent), the quarters are added in
// order; a single thread walking its row of N dependent-latency loads took 12 us at N = 64.
__global__ void __launch_bounds__(kBlock) coeff_kernel(const double *K, DevState *ds, CoeffParams cp) {
    __shared__ double lds[3 * kNMax];
    __shared__ double part[4][ADACONS_GRAM_N_MAX];
    static_assert(4 * ADACONS_GRAM_N_MAX <= kBlock, "four threads per row");
    const int N = cp.N, tid = threadIdx.x;
    const double m_old = (tid < N) ? ds->m[tid] : 0.0;
    const int row = tid >> 2, quarter = tid & 3;
    if (row < N) {
        double acc = 0.0;
#pragma unroll 4
        for (int j = quarter; j < N; j += 4) acc += K[(size_t)row * N + j];
        part[quarter][row] = acc;
    }
    __syncthreads();
    double q = 0.0, r = 0.0;
    if (tid < N) {
        q = K[(size_t)tid * N + tid];
        r = ((part[0][tid] + part[1][tid]) + part[2][tid]) + part[3][tid];
    }
    update_coefficients_from_stats(q, r, ds, cp, lds, m_old);
}

// ------------------------------------------------------------------------------------------
// A1, N <= 8: fp64 register tile per thread
// ------------------------------------------------------------------------------------------
// One column group: N 128-bit loads, then N(N+1)/2 fp64 FMAs per column.
template <int N, typename T, int VEC, bool NT>
__device__ __forceinline__ void gram_vec_step(const T *__restrict__ G, int64_t d, int64_t g,
                                              double (&acc)[N * (N + 1) / 2]) {
    float v[N][VEC];
#pragma unroll
    for (int i = 0; i < N; ++i) load_vec<T, VEC, NT>(G + (int64_t)i * d + g * VEC, v[i]);
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        double x[N];
#pragma unroll
        for (int i = 0; i < N; ++i) x[i] = (double)v[i][c];
        int p = 0;
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int j = i; j < N; ++j) {
                acc[p] = fma(x[i], x[j], acc[p]);
                ++p;
            }
    }
}

template <int N, typename T, int VEC>
__global__ void __launch_bounds__(kBlock, 2)
gram_vec_kernel(const T *__restrict__ G, int64_t d, int64_t ngroups, int64_t cached_groups, GramTail tail) {
    constexpr int NP = N * (N + 1) / 2;
    __shared__ double lds[(4 * NP > kBlock) ? 4 * NP : kBlock];
    double acc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = 0.0;

    // The head of G is read with ordinary loads, so that it stays in the memory-side cache for
    // the second pass (which starts there); the rest streams through with non-temporal loads.
    // Two loops, so that the two kinds of load are not merged into one.
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t g = (int64_t)slot * kBlock + threadIdx.x;
    const int64_t head_end = cached_groups < ngroups ? cached_groups : ngroups;
    for (; g < head_end; g += stride) gram_vec_step<N, T, VEC, false>(G, d, g, acc);
    for (; g < ngroups; g += stride) gram_vec_step<N, T, VEC, true>(G, d, g, acc);

    // workgroup sum: recursive halving inside each wavefront, then the four wavefronts in order
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    {
        const double tot = wave_reduce_scatter<NP>(acc, lane);
        const int p = wave_scatter_index(lane);
        if (p < NP) lds[wave * NP + p] = tot;
    }
    __syncthreads();
    if (threadIdx.x < NP) {
        const int p = threadIdx.x;
        tail.partials[(size_t)blockIdx.x * NP + p] = ((lds[p] + lds[NP + p]) + lds[2 * NP + p]) + lds[3 * NP + p];
    }
    __syncthreads();
    gram_tail(tail, lds);
}

// ------------------------------------------------------------------------------------------
// A1, 8 < N <= 64: 16x16 tiles on the matrix cores
// ------------------------------------------------------------------------------------------
// v_mfma_f32_16x16x4_f32 operand layout (64 lanes):
//   A (16x4):  lane l holds A[l % 16][l / 16]        B (4x16): lane l holds B[l / 16][l % 16]
//   D (16x16): lane l, register r holds D[4 * (l / 16) + r][l % 16]
// For a Gram tile pair (I, J): A[i][k] = G[16 I + i][col k], B[k][j] = G[16 J + j][col k], so
// lane l supplies G[16 T + l % 16][col(l / 16)] for both operands.  A lane loads four consecutive
// columns (one 128-bit load): its component c belongs to column  base + 4 (l / 16) + c,  and one
// MFMA per component contracts four columns that sit 4 apart -- any pairing is valid as long as
// A and B use the same one.
// 16-column steps between flushes of the fp32 tile sums into fp64.  The matrix cores' fp32
// accumulation rounds with a small systematic bias (measured ~2e-7 relative on a sum of squares
// after 128 products, ~4e-7 after 256), so the fp32 chains are kept to 8 steps = 128 products.
constexpr int kFlush = 8;
constexpr int kUnits = 4;   // 16-column steps a wavefront loads back to back (one chunk)

// Block-level end of an MFMA Gram kernel: add the four wavefronts' tile sums in order through LDS
// (lds[(p * 4 + r) * 64 + lane], NT(NT+1)/2 * 256 doubles) and scatter them into this workgroup's
// packed-upper-triangle row.  Lane l, register r of tile pair (I, J) holds
// K[16 I + 4 (l / 16) + r][16 J + l % 16].
template <int NT>
__device__ __forceinline__ void mfma_store_partial_row(const double (&acc64)[NT * (NT + 1) / 2][4], double *lds, int N,
                                                       double *row_out) {
    constexpr int NPT = NT * (NT + 1) / 2;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int w = 0; w < kBlock / kWave; ++w) {
        if (wave == w) {
#pragma unroll
            for (int p = 0; p < NPT; ++p)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int e = (p * 4 + r) * kWave + lane;
                    lds[e] = (w == 0) ? acc64[p][r] : lds[e] + acc64[p][r];
                }
        }
        __syncthreads();
    }
    for (int e = threadIdx.x; e < NPT * 256; e += kBlock) {
        const int l = e & (kWave - 1), r = (e >> 6) & 3, p = e >> 8;
        int I = 0, left = p;
        while (left >= NT - I) {
            left -= NT - I;
            ++I;
        }
        const int J = I + left;
        const int i = I * 16 + 4 * (l >> 4) + r;
        const int j = J * 16 + (l & 15);
        if (i < N && j < N && i <= j) row_out[pair_index(i, j, N)] = lds[e];
    }
}

// Load one chunk (kUnits * 16 columns of all NT row tiles) in operand layout.  Rows >= N and
// columns >= d count as zero: the load itself goes to a clamped (valid) address and the value is
// replaced afterwards, so that the loads stay free of branches and the waits on them exact.
// STREAM: non-temporal loads.
template <int NT, typename T, bool STREAM>
__device__ __forceinline__ void mfma_load_chunk(const T *__restrict__ G, int N, int64_t d, int64_t ch, int r16,
                                                int kq, float (&v)[kUnits][NT][4]) {
#pragma unroll
    for (int u = 0; u < kUnits; ++u) {
        const int64_t col = (ch * kUnits + u) * 16 + kq * 4;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int row = t * 16 + r16;
            const int rowc = row < N ? row : N - 1;
            // d is a multiple of the vector width here (>= 4 for fp32, >= 8 for bf16)
            const bool live = row < N && col < d;
            const int64_t colc = col < d ? col : d - 4;
            const T *p = G + (int64_t)rowc * d + colc;
            float w[4];
            if constexpr (sizeof(T) == 4) {
                load_vec<float, 4, STREAM>(reinterpret_cast<const float *>(p), w);
            } else {
                // 4 bf16 = one 64-bit load
                typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 *q = reinterpret_cast<const u32x2 *>(p);
                u32x2 x;
                if constexpr (STREAM) x = __builtin_nontemporal_load(q); else x = *q;
                w[0] = __uint_as_float(x.x << 16);
                w[1] = __uint_as_float(x.x & 0xffff0000u);
                w[2] = __uint_as_float(x.y << 16);
                w[3] = __uint_as_float(x.y & 0xffff0000u);
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) v[u][t][c] = live ? w[c] : 0.f;
        }
    }
}

// STREAM selects non-temporal loads (kept for measurement; the launcher uses ordinary loads).
// The next chunk's loads are issued before the current chunk's MFMAs, so that the matrix
// cores and the memory pipeline work at the same time even with one wavefront per SIMD.
template <int NT, typename T, bool STREAM>
__global__ void __launch_bounds__(kBlock, (NT >= 3) ? 1 : 2)
gram_mfma_kernel(const T *__restrict__ G, int N, int64_t d, int64_t nchunks, GramTail tail) {
    constexpr int NPT = NT * (NT + 1) / 2;
    __shared__ double lds[(NPT * 256 > kBlock) ? NPT * 256 : kBlock];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r16 = lane & 15, kq = lane >> 4;

    f32x4 acc32[NPT];
    double acc64[NPT][4];
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] = 0.0;
    }

    // a chunk = kUnits * 16 consecutive columns, taken by one wavefront
    const int64_t wstride = (int64_t)gridDim.x * (kBlock / kWave);
    int since_flush = 0;
    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t ch = (int64_t)slot * (kBlock / kWave) + wave;
    float cur[kUnits][NT][4], nxt[kUnits][NT][4];
    if (ch < nchunks) mfma_load_chunk<NT, T, STREAM>(G, N, d, ch, r16, kq, cur);
    while (ch < nchunks) {
        const int64_t chn = ch + wstride;
        // past the end the last chunk is simply loaded again (in bounds, never used)
        mfma_load_chunk<NT, T, STREAM>(G, N, d, chn < nchunks ? chn : nchunks - 1, r16, kq, nxt);
#pragma unroll
        for (int u = 0; u < kUnits; ++u) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                int p = 0;
#pragma unroll
                for (int I = 0; I < NT; ++I)
#pragma unroll
                    for (int J = I; J < NT; ++J) {
                        acc32[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(cur[u][I][c], cur[u][J][c], acc32[p], 0, 0, 0);
                        ++p;
                    }
            }
        }
        since_flush += kUnits;
        if (since_flush >= kFlush) {
            since_flush = 0;
#pragma unroll
            for (int p = 0; p < NPT; ++p) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
                acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int u = 0; u < kUnits; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int c = 0; c < 4; ++c) cur[u][t][c] = nxt[u][t][c];
        ch = chn;
    }
#pragma unroll
    for (int p = 0; p < NPT; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];

    mfma_store_partial_row<NT>(acc64, lds, N, tail.partials + (size_t)blockIdx.x * num_pairs(N));
    __syncthreads();
    gram_tail(tail, lds);
}


// ------------------------------------------------------------------------------------------
// A1, 8 < N <= 64, 128-bit path: tiles staged through LDS
// ------------------------------------------------------------------------------------------
// The direct kernel above touches 16 rows with every load instruction and cycles through all
// 16 NT rows sixteen times per 64 columns; with rows ~100 MB apart that thrashes the per-CU
// address-translation cache (measured at N = 64: one miss per four requests).  Here the
// workgroup stages a tile of 16 NT rows x kSegs KB per row in LDS: every load instruction reads
// 1 KB of ONE row, fully coalesced, and each row is visited once per tile.  Then each wavefront
// takes a quarter of the tile's columns and feeds the matrix cores from LDS (ds_read in operand
// layout).  The 16-byte chunks of a tile row are XOR-swizzled with the row number so that the
// column-wise operand reads hit distinct banks.  The next tile's global loads are in flight
// while the current tile is multiplied.
template <int NT> struct LdsTileShape {
    static constexpr int kRows = 16 * NT;
    static constexpr int kSegs = (NT == 1) ? 4 : (NT == 2) ? 2 : 1;   // 1 KB segments per tile row
    static constexpr int kLoads = kRows * kSegs / (kBlock / kWave);   // load instructions per wavefront
    static constexpr int kRowBytes = kSegs * 1024;
    static constexpr int kTileBytes = kRows * kRowBytes;              // <= 64 KB
};

template <int NT, typename T>
__global__ void __launch_bounds__(kBlock, (NT >= 4) ? 1 : 2)
gram_mfma_lds_kernel(const T *__restrict__ G, int N, int64_t d, int64_t ntiles, double *__restrict__ partials) {
    typedef LdsTileShape<NT> S;
    constexpr int NPT = NT * (NT + 1) / 2;
    constexpr int kVec = 16 / (int)sizeof(T);                 // elements per 16-byte chunk
    constexpr int kTileCols = S::kRowBytes / (int)sizeof(T);  // columns per tile
    constexpr int kUnitsPerWave = kTileCols / 64;             // 16-column MFMA steps per wavefront and tile
    static_assert(NPT * 256 * 8 <= S::kTileBytes, "the final reduction reuses the tile buffer");
    __shared__ __attribute__((aligned(16))) unsigned char tile[S::kTileBytes];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r16 = lane & 15, kq = lane >> 4;

    f32x4 acc32[NPT];
    double acc64[NPT][4];
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] = 0.0;
    }

    // stage registers: load j of this wavefront covers tile row (wave * kLoads + j) / kSegs,
    // segment (wave * kLoads + j) % kSegs, bytes [16 lane, 16 lane + 16) of that segment
    u32x4 stage[S::kLoads];
    auto load_tile = [&](int64_t t) {
#pragma unroll
        for (int j = 0; j < S::kLoads; ++j) {
            const int idx = wave * S::kLoads + j;
            const int row = idx / S::kSegs, seg = idx % S::kSegs;
            const int64_t col = t * kTileCols + (int64_t)seg * (1024 / (int)sizeof(T)) + lane * kVec;
            const bool live = row < N && col < d;   // d is a multiple of kVec on this path
            const int rowc = row < N ? row : N - 1;
            const int64_t colc = col < d ? col : d - kVec;
            const u32x4 x = *reinterpret_cast<const u32x4 *>(G + (int64_t)rowc * d + colc);
            stage[j] = live ? x : u32x4{0u, 0u, 0u, 0u};
        }
    };

    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t t = slot;
    int since_flush = 0;
    if (t < ntiles) load_tile(t);
    while (t < ntiles) {   // t is uniform over the workgroup: every thread takes the same trips
#pragma unroll
        for (int j = 0; j < S::kLoads; ++j) {
            const int idx = wave * S::kLoads + j;
            const int row = idx / S::kSegs, seg = idx % S::kSegs;
            const int chunk = (seg * 64 + lane) ^ (row & 15);
            *reinterpret_cast<u32x4 *>(tile + row * S::kRowBytes + chunk * 16) = stage[j];
        }
        __syncthreads();
        const int64_t tn = t + gridDim.x;
        load_tile(tn < ntiles ? tn : ntiles - 1);   // past the end: the last tile again, never used

#pragma unroll
        for (int u = 0; u < kUnitsPerWave; ++u) {
            float v[NT][4];
            const int col = wave * (kTileCols / 4) + u * 16 + kq * 4;   // first of this lane's 4 columns
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const int row = tt * 16 + r16;
                const int byte = col * (int)sizeof(T);
                const int chunk = (byte >> 4) ^ (row & 15);
                const unsigned char *src = tile + row * S::kRowBytes + chunk * 16 + (byte & 15);
                if constexpr (sizeof(T) == 4) {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(src);
                    v[tt][0] = x.x; v[tt][1] = x.y; v[tt][2] = x.z; v[tt][3] = x.w;
                } else {
                    const uint2 x = *reinterpret_cast<const uint2 *>(src);
                    v[tt][0] = __uint_as_float(x.x << 16);
                    v[tt][1] = __uint_as_float(x.x & 0xffff0000u);
                    v[tt][2] = __uint_as_float(x.y << 16);
                    v[tt][3] = __uint_as_float(x.y & 0xffff0000u);
                }
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                int p = 0;
#pragma unroll
                for (int I = 0; I < NT; ++I)
#pragma unroll
                    for (int J = I; J < NT; ++J) {
                        acc32[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(v[I][c], v[J][c], acc32[p], 0, 0, 0);
                        ++p;
                    }
            }
            if (++since_flush == kFlush) {
                since_flush = 0;
#pragma unroll
                for (int p = 0; p < NPT; ++p) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
                    acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
        __syncthreads();   // all operand reads done before the tile buffer is overwritten
        t = tn;
    }
#pragma unroll
    for (int p = 0; p < NPT; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
    mfma_store_partial_row<NT>(acc64, reinterpret_cast<double *>(tile), N,
                               partials + (size_t)blockIdx.x * num_pairs(N));
}


// ------------------------------------------------------------------------------------------
// A1, 8 < N <= 64, fp32, 128-bit path: coalesced loads, per-wavefront transpose through LDS
// ------------------------------------------------------------------------------------------
// Measured at N = 64: the operand-layout loads of gram_mfma_kernel alone (no MFMA) take longer
// than its MFMAs alone (1.33 ms vs 0.92 ms for 6.5 GB): 64-byte pieces of 16 rows per
// instruction reach only 4.9 TB/s, 256-byte pieces of 4 rows 6.1 TB/s.  Here a wavefront loads
// its 64-column chunk with coalesced instructions (4 rows x 256 B each), parks it in its OWN
// 16 NT x 256 B slice of LDS (16-byte pieces XOR-swizzled with the row number: conflict-free in
// both directions) and reads it back in operand layout.  Nothing is shared between wavefronts,
// so there is no workgroup barrier in the loop; the next chunk's loads are in flight while the
// current chunk is multiplied.
// bf16 inputs take the same kernel: a 16-byte piece then holds eight columns (chunks of 128 columns),
// and the operands go to v_mfma_f32_16x16x32_bf16 as they are -- bf16 products are exact in the fp32
// accumulator, at sixteen times the rate of the fp32 instruction.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

template <int NT, typename T>
__global__ void __launch_bounds__(kBlock, (NT >= 4) ? 1 : 2)
gram_mfma_wave_kernel(const T *__restrict__ G, int N, int64_t d, int64_t dcols, int64_t nchunks,
                      int64_t cached_chunks, double *__restrict__ partials) {
    constexpr int NPT = NT * (NT + 1) / 2;
    constexpr int kRows = 16 * NT, kLoads = 4 * NT;          // 4 rows per load instruction
    constexpr int VECW = VecWidth<T>::value;                  // columns per 16-byte piece
    constexpr int kCols = 16 * VECW;                          // columns per chunk: 256 bytes of every row
    constexpr int kSliceBytes = kRows * 256;                  // one wavefront's chunk
    static_assert(NPT * 256 * 8 <= 4 * kSliceBytes, "the final reduction reuses the slices");
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[4 * kSliceBytes];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r16 = lane & 15, kq = lane >> 4;
    unsigned char *slice = lds_raw + wave * kSliceBytes;

    f32x4 acc32[NPT];
    double acc64[NPT][4];
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] = 0.0;
    }

    // load j of a chunk: row 4 j + lane / 16, columns chunk * kCols + VECW (lane % 16) .. + VECW - 1
    f32x4 stage[kLoads];
    // interior: every row exists (N = 16 NT) and the chunk lies inside d, so no clamp and no zero-fill
    // (the address selects and zero masks cost more vector instructions than the loads themselves)
    auto load_chunk_as = [&](int64_t ch, auto stream, auto interior) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int row = 4 * j + (lane >> 4);
            const int64_t col = ch * kCols + (lane & 15) * VECW;
            if constexpr (decltype(interior)::value) {
                const gf32x4 *src = reinterpret_cast<const gf32x4 *>(G + (int64_t)row * d + col);
                if constexpr (decltype(stream)::value) stage[j] = __builtin_nontemporal_load(src);
                else stage[j] = *src;
            } else {
                const bool live = row < N && col < dcols;   // dcols is a multiple of VECW
                const int rowc = row < N ? row : N - 1;
                const int64_t colc = col < dcols ? col : dcols - VECW;
                const gf32x4 *src = reinterpret_cast<const gf32x4 *>(G + (int64_t)rowc * d + colc);
                f32x4 x;
                if constexpr (decltype(stream)::value) x = __builtin_nontemporal_load(src);
                else x = *src;
                stage[j] = live ? x : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    };
    const int64_t full_chunks = (N == kRows) ? dcols / kCols : 0;   // chunks below this index are interior
    auto load_chunk = [&](int64_t ch, auto stream) __attribute__((always_inline)) {
        if (ch < full_chunks) load_chunk_as(ch, stream, std::true_type{});
        else load_chunk_as(ch, stream, std::false_type{});
    };

    const int64_t wstride = (int64_t)gridDim.x * (kBlock / kWave);
    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t ch = (int64_t)slot * (kBlock / kWave) + wave;
    int since_flush = 0;
    // one chunk: park the staged registers in the slice, start the next chunk's loads, multiply
    auto step = [&](auto stream) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int row = 4 * j + (lane >> 4);
            const int piece = (lane & 15) ^ (row & 15);
            *reinterpret_cast<f32x4 *>(slice + row * 256 + piece * 16) = stage[j];
        }
        const int64_t chn = ch + wstride;
        load_chunk(chn < nchunks ? chn : nchunks - 1, stream);   // past the end: the last chunk again, never used
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            f32x4 v[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int row = t * 16 + r16;
                const int piece = (u * 4 + kq) ^ (row & 15);
                v[t] = *reinterpret_cast<const f32x4 *>(slice + row * 256 + piece * 16);
            }
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    int p = 0;
#pragma unroll
                    for (int I = 0; I < NT; ++I)
#pragma unroll
                        for (int J = I; J < NT; ++J) {
                            acc32[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(v[I][c], v[J][c], acc32[p], 0, 0, 0);
                            ++p;
                        }
                }
            } else {
                // lane l: row l % 16, columns 32 u + 8 (l / 16) .. + 7 of the chunk
                int p = 0;
#pragma unroll
                for (int I = 0; I < NT; ++I)
#pragma unroll
                    for (int J = I; J < NT; ++J) {
                        acc32[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v[I]),
                                                                           __builtin_bit_cast(bf16x8, v[J]), acc32[p], 0, 0, 0);
                        ++p;
                    }
            }
        }
        since_flush += kCols / 16;
        if (since_flush >= kFlush) {
            since_flush = 0;
#pragma unroll
            for (int p = 0; p < NPT; ++p) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
                acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        ch = chn;
    };
    // Chunks below cached_chunks are fetched with ordinary loads (the head of G stays in the
    // memory-side cache for the second pass), the rest with non-temporal ones.  Two loops, not a
    // branch per chunk: loads that differ only in that hint would be merged into one kind.
    if (ch < nchunks) load_chunk(ch, std::false_type{});
    while (ch < nchunks && ch + wstride < cached_chunks) step(std::false_type{});
    while (ch < nchunks) step(std::true_type{});
#pragma unroll
    for (int p = 0; p < NPT; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
    __syncthreads();   // every wavefront is done with its slice before the buffer is reused
    mfma_store_partial_row<NT>(acc64, reinterpret_cast<double *>(lds_raw), N,
                               partials + (size_t)blockIdx.x * num_pairs(N));
}

// ------------------------------------------------------------------------------------------
// A1, 8 < N <= 64, fp32, 128-bit path: products on the bf16 matrix-core path, fp32-exact by splitting
// ------------------------------------------------------------------------------------------
// The fp32 matrix-core instruction multiplies 32 element pairs per cycle and SIMD; the bf16 one
// sixteen times as many.  An fp32 value is the exact sum of three bf16 values, x = h + m + l
// (8 significant bits each, by truncation: h = top half of x's bits, m = top half of x - h,
// l = x - h - m), so x y = hh + (hm + mh) + (hl + lh + mm) + terms below 2^-24 |x y|: six bf16
// products, each exact, replace one fp32 product at 2.7 times the rate.  The wavefront loads its
// 64-column chunk as in gram_mfma_wave_kernel, splits it in registers and parks the three planes
// in its own LDS slice (rows of 64 bf16 = 128 B, 16-byte pieces XOR-swizzled with the row number);
// operands for v_mfma_f32_16x16x32_bf16 (lane l: row l % 16, columns 8 (l / 16) .. + 7 of a 32-column
// half) are read back with one 128-bit LDS load each.  Sums stay in fp32 inside the instruction;
// the tile sums are flushed into fp64 registers every two chunks, as in the fp32 kernels.

template <int NT>
__global__ void __launch_bounds__(kBlock, (NT >= 3) ? 1 : 2)
gram_mfma_split_kernel(const float *__restrict__ G, int N, int64_t d, int64_t dcols, int64_t nchunks,
                       int64_t cached_chunks, double *__restrict__ partials) {
    constexpr int NPT = NT * (NT + 1) / 2;
    constexpr int kRows = 16 * NT, kLoads = 4 * NT;          // 4 rows per load instruction
    constexpr int kPlaneBytes = kRows * 128;                  // kRows x 64 bf16
    constexpr int kSliceBytes = 3 * kPlaneBytes;              // h, m, l of one wavefront's chunk
    static_assert(NPT * 256 * 8 <= 4 * kSliceBytes, "the final reduction reuses the slices");
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[4 * kSliceBytes];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r16 = lane & 15, kq = lane >> 4;
    unsigned char *slice = lds_raw + wave * kSliceBytes;

    f32x4 acc32[NPT];
    double acc64[NPT][4];
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] = 0.0;
    }

    // load j of a chunk: row 4 j + lane / 16, columns chunk * 64 + 4 (lane % 16) .. + 3
    f32x4 stage[kLoads];
    // interior: every row exists (N = 16 NT) and the chunk lies inside d, so no clamp and no zero-fill
    auto load_chunk_as = [&](int64_t ch, auto stream, auto interior) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int row = 4 * j + (lane >> 4);
            const int64_t col = ch * 64 + (lane & 15) * 4;
            if constexpr (decltype(interior)::value) {
                const gf32x4 *src = reinterpret_cast<const gf32x4 *>(G + (int64_t)row * d + col);
                if constexpr (decltype(stream)::value) stage[j] = __builtin_nontemporal_load(src);
                else stage[j] = *src;
            } else {
                const bool live = row < N && col < dcols;   // dcols is a multiple of 4
                const int rowc = row < N ? row : N - 1;
                const int64_t colc = col < dcols ? col : dcols - 4;
                const gf32x4 *src = reinterpret_cast<const gf32x4 *>(G + (int64_t)rowc * d + colc);
                f32x4 x;
                if constexpr (decltype(stream)::value) x = __builtin_nontemporal_load(src);
                else x = *src;
                stage[j] = live ? x : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    };
    const int64_t full_chunks = (N == kRows) ? dcols / 64 : 0;   // chunks below this index are interior
    auto load_chunk = [&](int64_t ch, auto stream) __attribute__((always_inline)) {
        if (ch < full_chunks) load_chunk_as(ch, stream, std::true_type{});
        else load_chunk_as(ch, stream, std::false_type{});
    };

    const int64_t wstride = (int64_t)gridDim.x * (kBlock / kWave);
    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t ch = (int64_t)slot * (kBlock / kWave) + wave;
    int since_flush = 0;
    auto step = [&](auto stream) __attribute__((always_inline)) {
        // split into three bf16 planes and park them
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int row = 4 * j + (lane >> 4), cl = lane & 15;
            unsigned hb[4], mb[4], lb[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float x = stage[j][c];
                hb[c] = __float_as_uint(x) & 0xffff0000u;
                const float r1 = x - __uint_as_float(hb[c]);          // exact
                mb[c] = __float_as_uint(r1) & 0xffff0000u;
                const float r2 = r1 - __uint_as_float(mb[c]);         // exact, at most 8 significant bits
                lb[c] = __float_as_uint(r2);
            }
            // two bf16 (the upper halves) per dword: the lower column in the lower half
            const int off = row * 128 + ((((cl >> 1) ^ (row & 7))) << 4) + ((cl & 1) << 3);
            const u32x2 ph = {__builtin_amdgcn_perm(hb[1], hb[0], 0x07060302u), __builtin_amdgcn_perm(hb[3], hb[2], 0x07060302u)};
            const u32x2 pm = {__builtin_amdgcn_perm(mb[1], mb[0], 0x07060302u), __builtin_amdgcn_perm(mb[3], mb[2], 0x07060302u)};
            const u32x2 pl = {__builtin_amdgcn_perm(lb[1], lb[0], 0x07060302u), __builtin_amdgcn_perm(lb[3], lb[2], 0x07060302u)};
            *reinterpret_cast<u32x2 *>(slice + off) = ph;
            *reinterpret_cast<u32x2 *>(slice + kPlaneBytes + off) = pm;
            *reinterpret_cast<u32x2 *>(slice + 2 * kPlaneBytes + off) = pl;
        }
        const int64_t chn = ch + wstride;
        load_chunk(chn < nchunks ? chn : nchunks - 1, stream);   // past the end: the last chunk again, never used
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            bf16x8 op[3][NT];
#pragma unroll
            for (int P = 0; P < 3; ++P)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int row = t * 16 + r16;
                    const int piece = (u * 4 + kq) ^ (row & 7);
                    op[P][t] = *reinterpret_cast<const bf16x8 *>(slice + P * kPlaneBytes + row * 128 + piece * 16);
                }
            int p = 0;
#pragma unroll
            for (int I = 0; I < NT; ++I)
#pragma unroll
                for (int J = I; J < NT; ++J) {
                    f32x4 a = acc32[p];
                    // smallest terms first
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[1][I], op[1][J], a, 0, 0, 0);
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][I], op[2][J], a, 0, 0, 0);
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[2][I], op[0][J], a, 0, 0, 0);
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][I], op[1][J], a, 0, 0, 0);
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[1][I], op[0][J], a, 0, 0, 0);
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][I], op[0][J], a, 0, 0, 0);
                    acc32[p] = a;
                    ++p;
                }
        }
        since_flush += 4;
        if (since_flush >= kFlush) {
            since_flush = 0;
#pragma unroll
            for (int p = 0; p < NPT; ++p) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
                acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        ch = chn;
    };
    if (ch < nchunks) load_chunk(ch, std::false_type{});
    while (ch < nchunks && ch + wstride < cached_chunks) step(std::false_type{});
    while (ch < nchunks) step(std::true_type{});
#pragma unroll
    for (int p = 0; p < NPT; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
    __syncthreads();   // every wavefront is done with its slice before the buffer is reused
    mfma_store_partial_row<NT>(acc64, reinterpret_cast<double *>(lds_raw), N,
                               partials + (size_t)blockIdx.x * num_pairs(N));
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
template <typename Kern>
static int occupancy(Kern k) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k, kBlock, 0) != hipSuccess || nb < 1) nb = 1;
    return nb;
}

// blocks_per_cu <= 0 picks `dflt` workgroups per CU (never more than the occupancy allows).
static int grid_for(int64_t work_blocks, const LaunchShape &shape, int occ, int dflt) {
    int per_cu = shape.blocks_per_cu > 0 ? shape.blocks_per_cu : dflt;
    if (per_cu > occ) per_cu = occ;
    int64_t grid = (int64_t)shape.num_cu * per_cu;
    if (grid > work_blocks) grid = work_blocks;
    if (grid > shape.max_rows) grid = shape.max_rows;
    if (grid < 1) grid = 1;
    return (int)grid;
}

int gram_rows_needed(int N, int num_cu) {
    (void)N;
    return num_cu * 8;  // upper bound on workgroups per CU for any Gram kernel
}

// dcols: the columns this launch covers, a multiple of VEC (rows are d elements apart).
template <int N, typename T, int VEC>
static hipError_t run_vec(const void *G, int64_t d, int64_t dcols, const LaunchShape &shape, const GramTail &tail,
                          hipStream_t s, int *grid_out) {
    static const int occ = occupancy(gram_vec_kernel<N, T, VEC>);
    const int64_t ngroups = dcols / VEC;
    // measured best: one workgroup per CU for fp32, two for bf16 (twice the FMAs per byte)
    const int grid = grid_for((ngroups + kBlock - 1) / kBlock, shape, occ, sizeof(T) == 2 ? 2 : 1);
    *grid_out = grid;
    // shape.cached_head_mb < 0: everything with ordinary loads
    int64_t cached_groups = ngroups;
    if (shape.cached_head_mb >= 0)
        cached_groups = ((int64_t)shape.cached_head_mb << 20) / ((int64_t)N * VEC * (int64_t)sizeof(T));
    hipLaunchKernelGGL((gram_vec_kernel<N, T, VEC>), dim3(grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(G), d, ngroups, cached_groups, tail);
    return hipGetLastError();
}

template <typename T, int VEC>
static hipError_t dispatch_vec(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                               const GramTail &tail, hipStream_t s, int *grid_out) {
    switch (N) {
        case 1: return run_vec<1, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 2: return run_vec<2, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 3: return run_vec<3, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 4: return run_vec<4, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 5: return run_vec<5, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 6: return run_vec<6, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 7: return run_vec<7, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        case 8: return run_vec<8, T, VEC>(G, d, dcols, shape, tail, s, grid_out);
        default: return hipErrorInvalidValue;
    }
}

template <int NT, typename T, bool STREAM>
static hipError_t run_mfma_as(const void *G, int N, int64_t d, const LaunchShape &shape, const GramTail &tail,
                              hipStream_t s, int *grid_out) {
    static const int occ = occupancy(gram_mfma_kernel<NT, T, STREAM>);
    const int64_t cols_per_chunk = 16 * kUnits;
    const int64_t nchunks = (d + cols_per_chunk - 1) / cols_per_chunk;
    const int waves = kBlock / kWave;
    const int grid = grid_for((nchunks + waves - 1) / waves, shape, occ, NT >= 3 ? 1 : 2);
    *grid_out = grid;
    hipLaunchKernelGGL((gram_mfma_kernel<NT, T, STREAM>), dim3(grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(G), N, d, nchunks, tail);
    return hipGetLastError();
}

template <int NT, typename T>
static hipError_t run_mfma_lds(const void *G, int N, int64_t d, const LaunchShape &shape, const GramTail &tail,
                               hipStream_t s, int *grid_out) {
    const int64_t tile_cols = LdsTileShape<NT>::kRowBytes / (int64_t)sizeof(T);
    const int64_t ntiles = (d + tile_cols - 1) / tile_cols;
    const int grid = grid_for(ntiles, shape, NT >= 4 ? 1 : 2, NT >= 4 ? 1 : 2);   // 64 KB of LDS per workgroup
    *grid_out = grid;
    hipLaunchKernelGGL((gram_mfma_lds_kernel<NT, T>), dim3(grid), dim3(kBlock), 0, s, static_cast<const T *>(G), N,
                       d, ntiles, tail.partials);
    return hipGetLastError();
}

// SPLIT (fp32 only): products on the bf16 matrix-core path (gram_mfma_split_kernel) instead of the fp32 one.
// dcols: the columns this launch covers, a multiple of the 128-bit vector width (rows are d elements apart).
template <int NT, typename T, bool SPLIT>
static hipError_t run_mfma_wave(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                                const GramTail &tail, hipStream_t s, int *grid_out) {
    auto kern = [] {
        if constexpr (SPLIT && sizeof(T) == 4) return gram_mfma_split_kernel<NT>;
        else return gram_mfma_wave_kernel<NT, T>;
    }();
    static const int occ = occupancy(kern);
    const int64_t cols = 16 * VecWidth<T>::value;   // columns per chunk
    const int64_t nchunks = (dcols + cols - 1) / cols;
    const int waves = kBlock / kWave;
    const int dflt = SPLIT ? (NT >= 3 ? 1 : 2) : (NT >= 4 ? 1 : 2);
    const int grid = grid_for((nchunks + waves - 1) / waves, shape, occ, dflt);
    *grid_out = grid;
    // Non-temporal loads past the cached head pay off only when every row starts on a 128-byte line
    // (measured at N = 16: 6.8 against 6.3 TB/s); with rows shifted against the lines a 256-byte
    // piece shares its first and last line with its neighbours, and lines that are not kept in L2
    // are then fetched twice (6.1 against 6.3 TB/s).  shape.cached_head_mb < 0: ordinary loads only.
    const bool rows_on_lines = reinterpret_cast<uintptr_t>(G) % 128 == 0 && (d * (int64_t)sizeof(T)) % 128 == 0;
    int64_t cached_chunks = nchunks + (int64_t)grid * waves;   // beyond every prefetch
    if (shape.cached_head_mb >= 0 && rows_on_lines)
        cached_chunks = ((int64_t)shape.cached_head_mb << 20) / ((int64_t)N * 256);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, static_cast<const T *>(G), N, d, dcols, nchunks,
                       cached_chunks, tail.partials);
    return hipGetLastError();
}

// The wavefront-transpose kernels (variants 2 and 3) take any element-aligned G and any dcols that is a
// multiple of the vector width; the direct and LDS-tile kernels (variants 1 and 0) and the fused tail
// need 16-byte aligned rows and dcols = d, which the caller guarantees before selecting them.
template <int NT, typename T>
static hipError_t run_mfma(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                           const GramTail &tail, hipStream_t s, int *grid_out) {
    // 4 = automatic: measured at d = 25.6 M, the split-bf16 products win at N = 64 (1.10 against
    // 1.29 ms) and N = 48 (0.80 against 0.88 ms) and are even at N <= 32 (where the whole step
    // measured 2 % slower with them).  bf16 inputs need no split (3 = 2).
    const int variant = shape.mfma_direct == 4 ? ((NT >= 3 && sizeof(T) == 4) ? 3 : 2) : shape.mfma_direct;
    if (tail.mode == kGramPartialsOnly && variant == 2)
        return run_mfma_wave<NT, T, false>(G, N, d, dcols, shape, tail, s, grid_out);
    if (tail.mode == kGramPartialsOnly && variant == 3)
        return run_mfma_wave<NT, T, true>(G, N, d, dcols, shape, tail, s, grid_out);
    if (dcols != d) return hipErrorInvalidValue;
    // the LDS-staged kernel leaves the reduction to a later launch
    if (tail.mode == kGramPartialsOnly && shape.mfma_direct == 0)
        return run_mfma_lds<NT, T>(G, N, d, shape, tail, s, grid_out);
    // Ordinary loads only: one load instruction takes 64 contiguous bytes of each of 16 rows, so
    // the other half of every 128-byte line is needed by the next instruction; non-temporal loads
    // do not keep the line and measured 20 % slower here.
    return run_mfma_as<NT, T, false>(G, N, d, shape, tail, s, grid_out);
}

template <typename T>
static hipError_t dispatch_mfma(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                                const GramTail &tail, hipStream_t s, int *grid_out) {
    switch ((N + 15) / 16) {
        case 1: return run_mfma<1, T>(G, N, d, dcols, shape, tail, s, grid_out);
        case 2: return run_mfma<2, T>(G, N, d, dcols, shape, tail, s, grid_out);
        case 3: return run_mfma<3, T>(G, N, d, dcols, shape, tail, s, grid_out);
        case 4: return run_mfma<4, T>(G, N, d, dcols, shape, tail, s, grid_out);
        default: return hipErrorInvalidValue;
    }
}

// The last d - col0 < 8 columns of every row, which no whole 128-bit group covers: their products go
// into one more partial row (packed upper triangle), added with the others by the reduction.
template <typename T>
__global__ void __launch_bounds__(kBlock)
gram_edge_kernel(const T *__restrict__ G, int N, int64_t d, int64_t col0, double *__restrict__ row_out) {
    const int np = num_pairs(N);
    const int ncols = (int)(d - col0);
    for (int p = threadIdx.x; p < np; p += kBlock) {
        int i, j;
        unpack_pair(p, N, i, j);
        double tot = 0.0;
        for (int c = 0; c < ncols; ++c) {
            float a[1], b[1];
            load_vec<T, 1, false>(G + (int64_t)i * d + col0 + c, a);
            load_vec<T, 1, false>(G + (int64_t)j * d + col0 + c, b);
            tot = fma((double)a[0], (double)b[0], tot);
        }
        row_out[p] = tot;
    }
}

// tail.mode names the state wanted at the end (K reduced, or K and the coefficient update).
// With `fuse` and N(N+1)/2 <= kBlock the Gram kernel's last workgroup does it; otherwise one
// finish_kernel launch does (N <= 44), or a multi-workgroup reduction followed by coeff_kernel.
hipError_t launch_gram(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                       const LaunchShape &shape_in, const GramTail &want, bool fuse, hipStream_t stream,
                       hipEvent_t between) {
    // Without 16-byte aligned rows (vec_ok false) the same 128-bit kernels run from element-aligned
    // addresses over the whole groups of every row, the columns left over (fewer than one group) go
    // through gram_edge_kernel into one more partial row, and nothing is fused into the Gram kernel.
    const int64_t vec = (dtype == ADACONS_F32) ? 4 : 8;
    const int64_t dcols = vec_ok ? d : d / vec * vec;
    LaunchShape shape = shape_in;
    if (!vec_ok) {
        if (shape.max_rows < 2) return hipErrorInvalidValue;
        shape.max_rows -= 1;   // room for the edge row
        if (shape.mfma_direct != 2 && shape.mfma_direct != 3) shape.mfma_direct = 4;
    }
    GramTail tail = want;
    const bool fused = fuse && vec_ok && num_pairs(N) <= kBlock;
    if (!fused) tail.mode = kGramPartialsOnly;
    int grid = 0;
    hipError_t e;
    if (N <= 8) {
        e = (dtype == ADACONS_F32) ? dispatch_vec<float, 4>(G, N, d, dcols, shape, tail, stream, &grid)
                                   : dispatch_vec<bf16_bits, 8>(G, N, d, dcols, shape, tail, stream, &grid);
    } else {
        e = (dtype == ADACONS_F32) ? dispatch_mfma<float>(G, N, d, dcols, shape, tail, stream, &grid)
                                   : dispatch_mfma<bf16_bits>(G, N, d, dcols, shape, tail, stream, &grid);
    }
    if (e == hipSuccess && dcols < d) {
        double *row = want.partials + (size_t)grid * num_pairs(N);
        if (dtype == ADACONS_F32)
            hipLaunchKernelGGL(gram_edge_kernel<float>, dim3(1), dim3(kBlock), 0, stream,
                               static_cast<const float *>(G), N, d, dcols, row);
        else
            hipLaunchKernelGGL(gram_edge_kernel<bf16_bits>, dim3(1), dim3(kBlock), 0, stream,
                               static_cast<const bf16_bits *>(G), N, d, dcols, row);
        e = hipGetLastError();
        grid += 1;
    }
    if (e == hipSuccess && between) e = hipEventRecord(between, stream);
    if (e != hipSuccess || fused) return e;
    if (N <= kFinishMaxN) {
        hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(kFinishBlock), 0, stream, want.partials, grid, want.K,
                           want.ds, want.cp, want.mode == kGramFinishCoeffs ? 1 : 0);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(reduce_kernel, dim3((num_pairs(N) + 63) / 64), dim3(kBlock), 0, stream,
                       want.partials, grid, N, want.K);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (want.mode == kGramFinishCoeffs) return launch_coeffs(want.cp, want.K, want.ds, stream);
    return hipSuccess;
}

// Zero the device state with a kernel (a fill kernel, unlike a memset node, is safe for a caller
// that captures the stream into a HIP graph).
__global__ void __launch_bounds__(kBlock) clear_state_kernel(DevState *ds, double *K, int nn) {
    unsigned *w = reinterpret_cast<unsigned *>(ds);
    for (unsigned i = threadIdx.x; i < sizeof(DevState) / sizeof(unsigned); i += kBlock) w[i] = 0u;
    if (K)
        for (int i = threadIdx.x; i < nn; i += kBlock) K[i] = 0.0;
}

hipError_t launch_clear_state(DevState *ds, double *K, int nn, hipStream_t stream) {
    hipLaunchKernelGGL(clear_state_kernel, dim3(1), dim3(kBlock), 0, stream, ds, K, nn);
    return hipGetLastError();
}

// The carried state of Eq. 11 moved between a caller's array and a state block (the entry point that
// works in the library's file-scope scratch array keeps no state of its own between calls).
__global__ void __launch_bounds__(kNMax) state_load_kernel(DevState *ds, int N, const double *__restrict__ m_in) {
    const int i = threadIdx.x;
    ds->m[i] = (i < N) ? m_in[i] : 0.0;
    if (i == 0) {
        ds->numeric_flags = 0u;
        ds->blocks_done = 0u;
    }
}

__global__ void __launch_bounds__(kNMax)
state_store_kernel(const DevState *ds, int N, double *__restrict__ m_out, double *__restrict__ coeffs,
                   unsigned *__restrict__ numeric_flags) {
    const int i = threadIdx.x;
    if (i < N) {
        m_out[i] = ds->m[i];
        if (coeffs) {
            coeffs[i] = ds->gamma[i];
            coeffs[N + i] = ds->a_raw[i];
            coeffs[2 * N + i] = ds->a_smooth[i];
        }
    }
    if (i == 0 && numeric_flags) *numeric_flags = ds->numeric_flags;
}

hipError_t launch_state_load(DevState *ds, int N, const double *m_in, hipStream_t stream) {
    hipLaunchKernelGGL(state_load_kernel, dim3(1), dim3(kNMax), 0, stream, ds, N, m_in);
    return hipGetLastError();
}

hipError_t launch_state_store(const DevState *ds, int N, double *m_out, double *coeffs, unsigned *numeric_flags,
                              hipStream_t stream) {
    hipLaunchKernelGGL(state_store_kernel, dim3(1), dim3(kNMax), 0, stream, ds, N, m_out, coeffs, numeric_flags);
    return hipGetLastError();
}

hipError_t launch_coeffs(const CoeffParams &cp, double *K, DevState *ds, hipStream_t stream) {
    hipLaunchKernelGGL(coeff_kernel, dim3(1), dim3(kBlock), 0, stream, K, ds, cp);
    return hipGetLastError();
}

}  // namespace adacons
