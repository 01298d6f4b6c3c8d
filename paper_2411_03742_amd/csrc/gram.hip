// Stage A1 (K = G G^T) and stage A2 (coefficients, sorted momentum, normalisation).
//
// A1 computes every inner product <g_i, g_j> of Eq. 7 (third line) / the double sum of Eq. 8
// in one pass over G:
//   gram_vec_kernel         N <= 8: one thread owns VEC consecutive columns of all N rows
//                           (N 128-bit loads in flight) and keeps the N(N+1)/2 sums in fp64 registers.
//   gram_mfma_wave_kernel   8 < N <= 64: rows grouped in tiles of 16; a wavefront loads a chunk of all
//                           rows with coalesced instructions, transposes it through its own LDS slice
//                           and feeds the matrix cores with the same registers as A and B operand
//                           (K is G times its own transpose); fp32 tile sums flushed into fp64.
//   gram_mfma_split_coop_kernel  fp32 inputs with every product formed from six exact bf16 products,
//                           two wavefronts sharing a chunk (default for N > 32).
// All are persistent grids; every workgroup writes one row of partial sums, there are no
// floating-point atomics, and the rows are added in a fixed order, so results are
// bit-identical from run to run for a given launch shape.
//
// A2 is a single workgroup launched between the two streaming passes.
#include "adacons_internal.h"
#include "coeff_device.h"
#include "device_util.h"

#include <type_traits>

namespace adacons {

// ------------------------------------------------------------------------------------------
// Reduction of the partial rows and the coefficient update
// ------------------------------------------------------------------------------------------

// Reduction of the partial rows as a launch of its own (large N: more pairs than one workgroup
// has threads).  Workgroup c owns pairs [16 c, 16 c + 16); sixteen interleaved sub-sums per pair
// (rows s, s + 16, ...), added in slice order.
constexpr int kReducePairs = 16, kReduceSlices = kBlock / kReducePairs;
__global__ void __launch_bounds__(kBlock) reduce_kernel(const double *partials, int nrows, int N, double *K) {
    __shared__ double lds[kBlock];
    const int np = num_pairs(N);
    const int pl = threadIdx.x % kReducePairs, s = threadIdx.x / kReducePairs;
    const int p = blockIdx.x * kReducePairs + pl;
    lds[s * kReducePairs + pl] = (p < np) ? sum_rows(partials, np, p, s, kReduceSlices, nrows) : 0.0;
    __syncthreads();
    if (s == 0 && p < np) {
        double tot = 0.0;
        for (int q = 0; q < kReduceSlices; ++q) tot += lds[q * kReducePairs + pl];
        int i, j;
        unpack_pair(p, N, i, j);
        K[(size_t)i * N + j] = tot;
        K[(size_t)j * N + i] = tot;
    }
}

// Reduction of the partial rows and (optionally) the coefficient update in one workgroup of
// kFinishBlock threads, for N(N+1)/2 <= kFinishBlock: the launch between the two streaming passes.
constexpr int kFinishBlock = 1024;
static_assert(kFinishMaxN * (kFinishMaxN + 1) / 2 <= kFinishBlock, "one thread per pair");
__global__ void __launch_bounds__(kFinishBlock)
finish_kernel(const double *partials, int nrows, double *K, DevState *ds, CoeffParams cp, int with_coeffs) {
    __shared__ double lds[kFinishBlock];
    __shared__ double K_lds[kFinishMaxN * kFinishMaxN];
    const double m_old = ((int)threadIdx.x < cp.N) ? current_m(ds)[threadIdx.x] : 0.0;
    reduce_partial_rows<kFinishBlock>(partials, nrows, cp.N, K, lds, K_lds);
    if (with_coeffs) update_coefficients(K_lds, ds, cp, lds, m_old);
}

// The coefficient update as a launch of its own (after reduce_kernel).  Four threads share a
// row of K: each adds a quarter of it (elements j = quarter, quarter + 4, ...: neighbouring threads
// read neighbouring addresses, the loads of one thread are independent), the quarters are added in
// order; a single thread walking its row of N dependent-latency loads took 12 us at N = 64.
__global__ void __launch_bounds__(kBlock) coeff_kernel(const double *K, DevState *ds, CoeffParams cp) {
    __shared__ double lds[3 * kNMax];
    __shared__ double part[4][ADACONS_GRAM_N_MAX];
    static_assert(4 * ADACONS_GRAM_N_MAX <= kBlock, "four threads per row");
    const int N = cp.N, tid = threadIdx.x;
    const double m_old = (tid < N) ? current_m(ds)[tid] : 0.0;
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

// U column groups per thread at a time: the N U loads are issued together, then the products of the
// groups in ascending order -- the same sums in the same order as U single steps.
template <int N, typename T, int VEC, bool NT, int U>
__device__ __forceinline__ void gram_vec_steps(const T *__restrict__ G, int64_t d, int64_t g, int64_t stride,
                                               double (&acc)[N * (N + 1) / 2]) {
    float v[U][N][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < N; ++i) load_vec<T, VEC, NT>(G + (int64_t)i * d + (g + u * stride) * VEC, v[u][i]);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            double x[N];
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = (double)v[u][i][c];
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

// U > 1 (the short path: G of a few megabytes, a handful of sweeps per thread): the loads of U sweeps
// are in flight together, so a thread waits for memory once or twice instead of once per sweep.
// flip (or NULL): the state block whose parity word workgroup 0 flips -- the short path's stage A3
// then reads the old copy of the momentum state and writes the other one.
template <int N, typename T, int VEC, int U>
__global__ void __launch_bounds__(kBlock, 2)
gram_vec_kernel(const T *__restrict__ G, int64_t d, int64_t ngroups, int64_t cached_groups,
                double *__restrict__ partials, DevState *flip) {
    constexpr int NP = N * (N + 1) / 2;
    __shared__ double lds[(4 * NP > kBlock) ? 4 * NP : kBlock];
    double acc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = 0.0;
    if (flip && blockIdx.x == 0 && threadIdx.x == 0) flip->parity ^= 1u;

    // The head of G is read with ordinary loads, so that it stays in the memory-side cache for
    // the second pass (which starts there); the rest streams through with non-temporal loads.
    // Two loops, so that the two kinds of load are not merged into one.
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int slot = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);
    int64_t g = (int64_t)slot * kBlock + threadIdx.x;
    const int64_t head_end = cached_groups < ngroups ? cached_groups : ngroups;
    if constexpr (U > 1)
        for (; g + (U - 1) * stride < head_end; g += U * stride) gram_vec_steps<N, T, VEC, false, U>(G, d, g, stride, acc);
    for (; g < head_end; g += stride) gram_vec_step<N, T, VEC, false>(G, d, g, acc);
    if constexpr (U > 1)
        for (; g + (U - 1) * stride < ngroups; g += U * stride) gram_vec_steps<N, T, VEC, true, U>(G, d, g, stride, acc);
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
        partials[(size_t)blockIdx.x * NP + p] = ((lds[p] + lds[NP + p]) + lds[2 * NP + p]) + lds[3 * NP + p];
    }
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
                      int64_t cached_chunks, double *__restrict__ partials, DevState *flip) {
    if (flip && blockIdx.x == 0 && threadIdx.x == 0) flip->parity ^= 1u;   // as in gram_vec_kernel
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
    // interior 1: every row exists (N = 16 NT) and the chunk lies inside d, so no clamp and no zero-fill
    // (the address selects and zero masks cost more vector instructions than the loads themselves).
    // interior 2: the chunk lies inside d but N < 16 NT: a load instruction whose four rows all exist goes
    // out as it is, one whose rows all lie past N is not issued at all (N is uniform, so these are scalar
    // branches), and in the instruction that straddles N the lanes of absent rows are switched off.  Measured
    // at d = 25.6 M fp32 with every instruction clamped and masked: N = 12 0.340 ms (N = 16: 0.265), N = 24
    // 0.599 ms (N = 32: 0.534).
    auto load_chunk_as = [&](int64_t ch, auto stream, auto interior) __attribute__((always_inline)) {
        constexpr int kInterior = decltype(interior)::value;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int row = 4 * j + (lane >> 4);
            const int64_t col = ch * kCols + (lane & 15) * VECW;
            if (kInterior == 1 || (kInterior == 2 && 4 * j + 4 <= N)) {
                const gf32x4 *src = reinterpret_cast<const gf32x4 *>(G + (int64_t)row * d + col);
                if constexpr (decltype(stream)::value) stage[j] = __builtin_nontemporal_load(src);
                else stage[j] = *src;
            } else if (kInterior == 2 && 4 * j >= N) {
                stage[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            } else if (kInterior == 2) {
                // the instruction that straddles N: lanes of absent rows sit it out
                stage[j] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (row < N) {
                    const gf32x4 *src = reinterpret_cast<const gf32x4 *>(G + (int64_t)row * d + col);
                    if constexpr (decltype(stream)::value) stage[j] = __builtin_nontemporal_load(src);
                    else stage[j] = *src;
                }
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
    const int64_t full_chunks = dcols / kCols;   // chunks below this index lie inside d
    auto load_chunk = [&](int64_t ch, auto stream) __attribute__((always_inline)) {
        if (ch >= full_chunks) load_chunk_as(ch, stream, std::integral_constant<int, 0>{});
        else if (N == kRows) load_chunk_as(ch, stream, std::integral_constant<int, 1>{});
        else load_chunk_as(ch, stream, std::integral_constant<int, 2>{});
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
// A1, 8 < N <= 64, fp32: products on the bf16 matrix-core path, fp32-exact by splitting
// ------------------------------------------------------------------------------------------
// The fp32 matrix-core instruction multiplies 32 element pairs per cycle and SIMD; the bf16 one
// sixteen times as many.  An fp32 value is the exact sum of three bf16 values, x = h + m + l
// (8 significant bits each, by truncation: h = top half of x's bits, m = top half of x - h,
// l = x - h - m), so x y = hh + (hm + mh) + (hl + lh + mm) + terms below 2^-24 |x y|: six bf16
// products, each exact, replace one fp32 product at 2.7 times the rate.  A chunk of 64 columns of all
// rows is loaded as in gram_mfma_wave_kernel (4 rows x 256 B per instruction), split in registers, and
// its three planes are parked in LDS (rows of 64 bf16 = 128 B, 16-byte pieces XOR-swizzled with the row
// number); operands for v_mfma_f32_16x16x32_bf16 (lane l: row l % 16, columns 8 (l / 16) .. + 7 of a
// 32-column half) are read back with one 128-bit LDS load each.  Sums stay in fp32 inside the
// instruction; the tile sums are flushed into fp64 registers every two chunks, as in the fp32 kernel.
//
// A workgroup of W = 2 wavefronts shares one chunk: each loads, splits and parks half of the rows, and
// each owns half of the tile pairs -- half of the accumulators and operands (176 registers at N = 64
// where one wavefront with all ten tile pairs needs about 300), so two wavefronts fit a SIMD, four
// workgroups a CU, and one wavefront's vector work (the split) overlaps another's matrix-core work.
// Two workgroup barriers per chunk (planes complete / planes free again).  The tile pairs of the
// wavefronts are disjoint, so each scatters its own sums into the workgroup's partial row without a
// reduction between them.  Measured on N = 64, d = 25,557,032: 1.06 ms against 1.12 ms for one
// wavefront per chunk; four wavefronts per chunk (110 registers, sixteen wavefronts per CU) 1.18 ms, six
// workgroups of two per CU 1.15 ms; workgroups that walk runs of 2 / 4 / 8 consecutive chunks (so that a
// line two chunks share is asked for twice by the same workgroup) 1.07 / 1.08 / 1.08 ms.

// Which of the two wavefronts owns tile pair p (pairs in row-major upper-triangle order): the first
// half of the pairs, which share the first row tiles, and the second half.
__host__ __device__ constexpr int coop_role(int NT, int W, int p) { return p < (NT * (NT + 1) / 2 + W - 1) / W ? 0 : 1; }
__host__ __device__ constexpr int coop_local(int NT, int W, int p) {   // index of pair p among its owner's pairs
    int n = 0;
    for (int q = 0; q < p; ++q) n += coop_role(NT, W, q) == coop_role(NT, W, p) ? 1 : 0;
    return n;
}
__host__ __device__ constexpr int coop_max_pairs(int NT, int W) {
    int best = 0;
    for (int p = 0; p < NT * (NT + 1) / 2; ++p) best = coop_local(NT, W, p) + 1 > best ? coop_local(NT, W, p) + 1 : best;
    return best;
}

template <int NT, int W>
__global__ void __launch_bounds__(W * kWave, 2)
gram_mfma_split_coop_kernel(const float *__restrict__ G, int N, int64_t d, int64_t dcols, int64_t nchunks,
                            int64_t cached_chunks, double *__restrict__ partials, DevState *flip) {
    if (flip && blockIdx.x == 0 && threadIdx.x == 0) flip->parity ^= 1u;   // as in gram_vec_kernel
    constexpr int NPW = coop_max_pairs(NT, W);                // tile pairs per wavefront at most
    constexpr int kRows = 16 * NT;
    constexpr int kLoads = 4 * NT;                            // load instructions per chunk (4 rows each) ...
    constexpr int kLoadsW = kLoads / W;                       // ... per wavefront
    static_assert(W == 2 && kLoads % W == 0, "two wavefronts, the rows split evenly over them");
    constexpr int kPlaneBytes = kRows * 128;                  // kRows x 64 bf16
    __shared__ __attribute__((aligned(16))) unsigned char planes[3 * kPlaneBytes];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r16 = lane & 15, kq = lane >> 4;

    f32x4 acc32[NPW];
    double acc64[NPW][4];
#pragma unroll
    for (int p = 0; p < NPW; ++p) {
        acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] = 0.0;
    }

    // load j of this wavefront: row 4 (wave kLoadsW + j) + lane / 16, columns chunk * 64 + 4 (lane % 16) .. + 3
    f32x4 stage[kLoadsW];
    // interior: every row exists (N = 16 NT) and the chunk lies inside d, so no clamp and no zero-fill
    auto load_chunk = [&](int64_t ch, auto stream, auto interior) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLoadsW; ++j) {
            const int row = 4 * (wave * kLoadsW + j) + (lane >> 4);
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

    const int64_t stride = (int64_t)gridDim.x;
    int64_t ch = xcd_contiguous_slot((int)blockIdx.x, (int)gridDim.x);   // uniform over the workgroup
    int since_flush = 0;
    // the products of the tile pairs wavefront ROLE owns for one 32-column half; operand tiles that none of
    // its pairs touch are not read
    auto multiply = [&](auto role, int u) __attribute__((always_inline)) {
        constexpr int ROLE = decltype(role)::value;
        bf16x8 op[3][NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            bool used = false;
            int p = 0;
#pragma unroll
            for (int I = 0; I < NT; ++I)
#pragma unroll
                for (int J = I; J < NT; ++J) {
                    if (coop_role(NT, W, p) == ROLE && (I == t || J == t)) used = true;
                    ++p;
                }
            if (used) {
                const int row = t * 16 + r16;
                const int piece = (u * 4 + kq) ^ (row & 7);
#pragma unroll
                for (int P = 0; P < 3; ++P)
                    op[P][t] = *reinterpret_cast<const bf16x8 *>(planes + P * kPlaneBytes + row * 128 + piece * 16);
            }
        }
        // term by term across the pairs, so that consecutive instructions write different accumulators;
        // per pair the smallest terms first
        auto term = [&](auto a, auto b) __attribute__((always_inline)) {
            int p = 0;
#pragma unroll
            for (int I = 0; I < NT; ++I)
#pragma unroll
                for (int J = I; J < NT; ++J) {
                    if (coop_role(NT, W, p) == ROLE) {
                        const int q = coop_local(NT, W, p);
                        acc32[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[decltype(a)::value][I], op[decltype(b)::value][J],
                                                                           acc32[q], 0, 0, 0);
                    }
                    ++p;
                }
        };
        using P_h = std::integral_constant<int, 0>;
        using P_m = std::integral_constant<int, 1>;
        using P_l = std::integral_constant<int, 2>;
        term(P_m{}, P_m{});
        term(P_h{}, P_l{});
        term(P_l{}, P_h{});
        term(P_h{}, P_m{});
        term(P_m{}, P_h{});
        term(P_h{}, P_h{});
    };
    auto step = [&](auto stream, auto interior_next) __attribute__((always_inline)) {
        // split this wavefront's rows into three bf16 planes and park them
#pragma unroll
        for (int j = 0; j < kLoadsW; ++j) {
            const int row = 4 * (wave * kLoadsW + j) + (lane >> 4), cl = lane & 15;
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
            *reinterpret_cast<u32x2 *>(planes + off) = ph;
            *reinterpret_cast<u32x2 *>(planes + kPlaneBytes + off) = pm;
            *reinterpret_cast<u32x2 *>(planes + 2 * kPlaneBytes + off) = pl;
        }
        __syncthreads();   // every wavefront's share of the planes is in place
        const int64_t chn = ch + stride;
        load_chunk(chn < nchunks ? chn : nchunks - 1, stream, interior_next);   // past the end: the last chunk again, never used
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (wave == 0) multiply(std::integral_constant<int, 0>{}, u);
            else multiply(std::integral_constant<int, 1>{}, u);
        }
        since_flush += 4;
        if (since_flush >= kFlush) {
            since_flush = 0;
#pragma unroll
            for (int p = 0; p < NPW; ++p) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];
                acc32[p] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        __syncthreads();   // every wavefront has read its operands: the planes may be overwritten
        ch = chn;
    };
    if (ch < nchunks) load_chunk(ch, std::false_type{}, std::false_type{});
    // Four loops in a row rather than one loop with branches: chunks whose successor is interior first
    // (the head of G with ordinary loads, then the streamed part), then whatever is left -- the ragged
    // end of the rows, or everything when N is not a multiple of 16 -- with clamped addresses and
    // zero-fill.  Kept apart so that the address arithmetic of the general path, which the compiler
    // computes ahead of its loop, does not occupy registers during the fast loops.
    const int64_t fast_end = full_chunks < cached_chunks ? full_chunks : cached_chunks;
    while (ch < nchunks && ch + stride < fast_end) step(std::false_type{}, std::true_type{});
    while (ch < nchunks && ch + stride < full_chunks) step(std::true_type{}, std::true_type{});
    while (ch < nchunks && ch + stride < cached_chunks) step(std::false_type{}, std::false_type{});
    while (ch < nchunks) step(std::true_type{}, std::false_type{});
#pragma unroll
    for (int p = 0; p < NPW; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[p][r] += (double)acc32[p][r];

    // lane l, register r of tile pair (I, J) holds K[16 I + 4 (l / 16) + r][16 J + l % 16]
    double *row_out = partials + (size_t)blockIdx.x * num_pairs(N);
    auto scatter = [&](auto role) __attribute__((always_inline)) {
        constexpr int ROLE = decltype(role)::value;
        int p = 0;
#pragma unroll
        for (int I = 0; I < NT; ++I)
#pragma unroll
            for (int J = I; J < NT; ++J) {
                if (coop_role(NT, W, p) == ROLE) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = I * 16 + 4 * kq + r, j = J * 16 + r16;
                        if (i < N && j < N && i <= j) row_out[pair_index(i, j, N)] = acc64[coop_local(NT, W, p)][r];
                    }
                }
                ++p;
            }
    };
    if (wave == 0) scatter(std::integral_constant<int, 0>{});
    else scatter(std::integral_constant<int, 1>{});
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
static hipError_t run_vec(const void *G, int64_t d, int64_t dcols, const LaunchShape &shape, double *partials,
                          DevState *ds, hipStream_t s, int *grid_out) {
    static const int occ = occupancy(gram_vec_kernel<N, T, VEC, 1>);
    const int64_t ngroups = dcols / VEC;
    // measured best: one workgroup per CU for fp32, two for bf16 (twice the FMAs per byte)
    const int grid = grid_for((ngroups + kBlock - 1) / kBlock, shape, occ, sizeof(T) == 2 ? 2 : 1);
    *grid_out = grid;
    // Streams: few rows put few loads in flight (N per thread and sweep), so U sweeps are requested together until
    // a thread has about eight outstanding.  Measured, A1 at d = 25.6 M fp32, U = 1 -> U below: N = 1 50 -> 22 us,
    // N = 2 61 -> 36, N = 3 69 -> 51, N = 4 78 -> 67 us; bf16 (two workgroups per CU): N = 1 19 -> 13, N = 2
    // 23 -> 21 us, N >= 3 no gain.  Same sums in the same order for any U.
    constexpr int U_stream = (sizeof(T) == 4) ? (N <= 2 ? 4 : (N <= 4 ? 2 : 1)) : (N == 1 ? 4 : (N == 2 ? 2 : 1));
    if (shape.short_path) {
        // same grid, same columns per thread, same order of the sums as the kernel below: K comes out bit for
        // bit the same; everything with ordinary loads (stage A3 finds G in the caches)
        // sixteen 128-bit loads in flight per thread where the widened values fit the registers
        constexpr int U = (N * VEC <= 16) ? 4 : (N * VEC <= 32 ? 2 : 1);
        // forced on a stream too long for the caches: the cached-head policy of the long path
        int64_t head = ngroups;
        if ((int64_t)N * dcols * (int64_t)sizeof(T) > ((int64_t)32 << 20) && shape.cached_head_mb >= 0)
            head = ((int64_t)shape.cached_head_mb << 20) / ((int64_t)N * VEC * (int64_t)sizeof(T));
        if (head < ngroups) {
            hipLaunchKernelGGL((gram_vec_kernel<N, T, VEC, U_stream>), dim3(grid), dim3(kBlock), 0, s,
                               static_cast<const T *>(G), d, ngroups, head, partials, ds);
            return hipGetLastError();
        }
        hipLaunchKernelGGL((gram_vec_kernel<N, T, VEC, U>), dim3(grid), dim3(kBlock), 0, s,
                           static_cast<const T *>(G), d, ngroups, ngroups, partials, ds);
        return hipGetLastError();
    }
    // shape.cached_head_mb < 0: everything with ordinary loads
    int64_t cached_groups = ngroups;
    if (shape.cached_head_mb >= 0)
        cached_groups = ((int64_t)shape.cached_head_mb << 20) / ((int64_t)N * VEC * (int64_t)sizeof(T));
    hipLaunchKernelGGL((gram_vec_kernel<N, T, VEC, U_stream>), dim3(grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(G), d, ngroups, cached_groups, partials, static_cast<DevState *>(nullptr));
    return hipGetLastError();
}

template <typename T, int VEC>
static hipError_t dispatch_vec(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                               double *partials, DevState *ds, hipStream_t s, int *grid_out) {
    switch (N) {
        case 1: return run_vec<1, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 2: return run_vec<2, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 3: return run_vec<3, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 4: return run_vec<4, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 5: return run_vec<5, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 6: return run_vec<6, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 7: return run_vec<7, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        case 8: return run_vec<8, T, VEC>(G, d, dcols, shape, partials, ds, s, grid_out);
        default: return hipErrorInvalidValue;
    }
}

// dcols: the columns this launch covers, a multiple of the 128-bit vector width (rows are d elements apart).
template <int NT, typename T>
static hipError_t run_mfma_wave(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                                double *partials, DevState *ds, hipStream_t s, int *grid_out) {
    auto kern = gram_mfma_wave_kernel<NT, T>;
    static const int occ = occupancy(kern);
    const int64_t cols = 16 * VecWidth<T>::value;   // columns per chunk
    const int64_t nchunks = (dcols + cols - 1) / cols;
    const int waves = kBlock / kWave;
    const int dflt = NT >= 4 ? 1 : 2;
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
                       cached_chunks, partials, shape.short_path ? ds : nullptr);
    return hipGetLastError();
}

// The split-bf16 products with W wavefronts per chunk: one chunk and one partial row per workgroup.
template <int NT, int W>
static hipError_t run_mfma_coop(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                                double *partials, DevState *ds, hipStream_t s, int *grid_out) {
    static const int occ = [] {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, gram_mfma_split_coop_kernel<NT, W>, W * kWave, 0) != hipSuccess || nb < 1) nb = 1;
        return nb;
    }();
    const int64_t nchunks = (dcols + 63) / 64;
    const int grid = grid_for(nchunks, shape, occ, 4);   // four workgroups per CU measured best (three: +8 %, six: +9 %)
    *grid_out = grid;
    const bool rows_on_lines = reinterpret_cast<uintptr_t>(G) % 128 == 0 && (d * 4) % 128 == 0;
    int64_t cached_chunks = nchunks + (int64_t)grid;   // beyond every prefetch
    if (shape.cached_head_mb >= 0 && rows_on_lines)
        cached_chunks = ((int64_t)shape.cached_head_mb << 20) / ((int64_t)N * 256);
    hipLaunchKernelGGL((gram_mfma_split_coop_kernel<NT, W>), dim3(grid), dim3(W * kWave), 0, s, static_cast<const float *>(G), N,
                       d, dcols, nchunks, cached_chunks, partials, shape.short_path ? ds : nullptr);
    return hipGetLastError();
}

// shape.gram_products: 0 = the fp32 matrix-core instruction, 1 = split-bf16 products, 2 = by N.
// Measured at d = 25.6 M, fp32: the split-bf16 products win at N = 64 (1.06 against 1.29 ms) and N = 48
// (0.80 against 0.88 ms) and are even at N <= 32 (where the whole step measured 2 % slower with them).
// bf16 inputs need no split: their products are exact on the bf16 instruction as they are.
template <int NT, typename T>
static hipError_t run_mfma(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                           double *partials, DevState *ds, hipStream_t s, int *grid_out) {
    if constexpr (sizeof(T) == 4) {
        if (shape.gram_products == 1 || (shape.gram_products == 2 && NT >= 3))
            return run_mfma_coop<NT, 2>(G, N, d, dcols, shape, partials, ds, s, grid_out);
    }
    return run_mfma_wave<NT, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
}

template <typename T>
static hipError_t dispatch_mfma(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                                double *partials, DevState *ds, hipStream_t s, int *grid_out) {
    switch ((N + 15) / 16) {
        case 1: return run_mfma<1, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 2: return run_mfma<2, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 3: return run_mfma<3, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
        case 4: return run_mfma<4, T>(G, N, d, dcols, shape, partials, ds, s, grid_out);
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

// Stage A1, then the reduction of the partial rows into K and (with_coeffs) stage A2: one finish_kernel
// launch for small N or few rows, a multi-workgroup reduction followed by coeff_kernel otherwise.
hipError_t launch_gram(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                       const LaunchShape &shape_in, const GramWork &want, bool with_coeffs, hipStream_t stream,
                       hipEvent_t between, int *rows_out) {
    if (shape_in.short_path && (N > kFinishMaxN || !vec_ok || !rows_out)) return hipErrorInvalidValue;
    // Without 16-byte aligned rows (vec_ok false) the same 128-bit kernels run from element-aligned
    // addresses over the whole groups of every row, and the columns left over (fewer than one group) go
    // through gram_edge_kernel into one more partial row.
    const int64_t vec = (dtype == ADACONS_F32) ? 4 : 8;
    const int64_t dcols = vec_ok ? d : d / vec * vec;
    LaunchShape shape = shape_in;
    if (!vec_ok) {
        if (shape.max_rows < 2) return hipErrorInvalidValue;
        shape.max_rows -= 1;   // room for the edge row
    }
    int grid = 0;
    hipError_t e;
    if (N <= 8) {
        e = (dtype == ADACONS_F32) ? dispatch_vec<float, 4>(G, N, d, dcols, shape, want.partials, want.ds, stream, &grid)
                                   : dispatch_vec<bf16_bits, 8>(G, N, d, dcols, shape, want.partials, want.ds, stream, &grid);
    } else {
        e = (dtype == ADACONS_F32) ? dispatch_mfma<float>(G, N, d, dcols, shape, want.partials, want.ds, stream, &grid)
                                   : dispatch_mfma<bf16_bits>(G, N, d, dcols, shape, want.partials, want.ds, stream, &grid);
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
    if (e != hipSuccess) return e;
    if (shape.short_path) {   // stage A3 adds the rows and runs stage A2 itself
        *rows_out = grid;
        return hipSuccess;
    }
    // One workgroup adds the rows and runs the update where that is a short job: its threads share a sum
    // min(1024 / pairs, 32) ways, and a thread should not walk more than 32 rows.  Measured (time of stage A2
    // between events): N = 44, 512 rows 129 us in one workgroup, 16 us as the two launches below; N = 32, 512
    // rows 42 against 12 us; N = 16, 512 rows 17 against 12 us, 32 rows 8.7 us in one workgroup.
    const int np = num_pairs(N);
    const int shares = kFinishBlock / np < 32 ? kFinishBlock / np : 32;
    const bool one_workgroup = N <= kFinishMaxN && grid <= 32 * shares;
    if (one_workgroup) {
        hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(kFinishBlock), 0, stream, want.partials, grid, want.K,
                           want.ds, want.cp, with_coeffs ? 1 : 0);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(reduce_kernel, dim3((num_pairs(N) + kReducePairs - 1) / kReducePairs), dim3(kBlock), 0, stream,
                       want.partials, grid, N, want.K);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (with_coeffs) return launch_coeffs(want.cp, want.K, want.ds, stream);
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
    ds->m[0][i] = (i < N) ? m_in[i] : 0.0;
    ds->m[1][i] = 0.0;
    if (i == 0) {
        ds->numeric_flags = 0u;
        ds->parity = 0u;
    }
}

__global__ void __launch_bounds__(kNMax)
state_store_kernel(const DevState *ds, int N, double *__restrict__ m_out, double *__restrict__ coeffs,
                   unsigned *__restrict__ numeric_flags) {
    const int i = threadIdx.x;
    if (i < N) {
        m_out[i] = current_m(ds)[i];
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
