// Layer-wise AdaCons aggregation (the variant Sec. 4 of the paper mentions beside the model-wise one):
// steps A1-A3 run independently on every contiguous column segment of G, with one coefficient set
// and one Eq. 11 momentum state per layer -- in three launches for all layers.
//
// Every layer is cut into runs of at most run_groups column groups (one group = one 128-bit load per
// row); a run never crosses a layer boundary.  Layer boundaries need not be multiples of the group
// width: the group that straddles two layers belongs to a run of each, and the columns that
// belong to the other layer are masked (zeroed in A1, not stored in A3).  Nor need d be one: the
// last group of a row then holds fewer than VEC columns of it, and is read VEC columns back from
// the end of the row instead (the columns it shares with the group before are masked).  All
// 128-bit accesses are issued from element-aligned addresses.
//   A1  workgroup b takes the runs order[b], order[b + grid], ... -- full-length runs in column order (so
//       that at any time all workgroups read one compact window of every row), then the short ones,
//       longest first; a run's descriptor comes through scalar loads, the next one's is in flight
//       while the current run streams.
//       Inside a run the N(N+1)/2 fp64 sums stay in registers; one partial row is written per
//       run, indexed by the run, so the result does not depend on which workgroup took which run.
//       Runs are numbered in column order, so the runs of one layer are consecutive.  No
//       workgroup ever waits for another.
//   A2  one workgroup per layer adds that layer's partial rows in a fixed order and runs the
//       coefficient update on the layer's own state.
//   A3  grid-stride over the runs; the run's layer selects the weights.
// N <= 8 keeps the whole Gram matrix of a column group in one thread's registers.  For N > 8 stage
// A1 computes per layer what Eq. 7 consumes -- q_i = ||g_i||^2 and r_i = <g_i, sum_j g_j> over the
// layer's columns -- with the wavefront-cooperative scheme of the statistics-only pass: a chunk
// of 16 column groups of all N rows lives in the registers of one wavefront.
#include <algorithm>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "adacons_internal.h"
#include "coeff_device.h"
#include "device_util.h"

namespace adacons {

struct LayerRun {
    int64_t g0;      // first column group (group = VEC columns)
    int64_t cb, ce;  // the layer's column range [cb, ce)
    int n;           // groups in this run, 1..run_groups
    int layer;
};

constexpr int kLayersMaxN = 8;           // largest N with the Gram matrix per thread; above: statistics
// Column groups per run.  Workgroup b of stage A1 takes the runs order[b], order[b + grid], ... (the
// full-length runs in column order, then the shorter ones, longest first), so the pass lasts as long as
// the workgroup with the most column groups.  The length is chosen per layout: every multiple of 512
// groups (an eighth of a run must be a whole piece of stage A3) from 1024 to 16384 is laid out, the
// assignment above is played through, and the length with the smallest largest share wins; a run's
// fixed cost (descriptor, final reduction, barriers) is counted as kRunOverhead groups.  A fixed
// length of 4608 left 363 of 512 workgroups with three runs and the others with two on one 25.6 M
// column layer: 11 % more time than the bytes need.
constexpr int kRunOverhead = 512;
static int choose_run_groups(const int64_t *offsets, int L, int vec, int grid) {
    int best_len = 4 * kBlock;
    if (L > (1 << 16)) return best_len;   // a great many small layers: every run is short whatever the length
    int64_t best_cost = -1;
    std::vector<int64_t> load((size_t)grid);
    std::vector<int> rest;
    for (int len = 4 * kBlock; len <= 64 * kBlock; len += 512) {
        std::fill(load.begin(), load.end(), (int64_t)0);
        rest.clear();
        int64_t slot = 0;   // position in the order: full-length runs first, as they come
        for (int l = 0; l < L; ++l) {
            const int64_t groups = (offsets[l + 1] + vec - 1) / vec - offsets[l] / vec;
            const int64_t full = groups / len;
            for (int64_t r = 0; r < full; ++r) load[(size_t)(slot++ % grid)] += len + kRunOverhead;
            if (groups % len) rest.push_back((int)(groups % len));
        }
        std::sort(rest.begin(), rest.end(), [](int a, int b) { return a > b; });
        for (int n : rest) load[(size_t)(slot++ % grid)] += n + kRunOverhead;
        const int64_t cost = *std::max_element(load.begin(), load.end());
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best_len = len;
        }
    }
    return best_len;
}

// ------------------------------------------------------------------------------------------
// A1
// ------------------------------------------------------------------------------------------
// N 128-bit loads of column group g and the N(N+1)/2 fp64 FMAs per column; columns outside
// [cb, ce) (the other layer's part of a straddling group) count as zero.
template <int N, typename T, int VEC, bool EDGE, bool STREAM>
__device__ __forceinline__ void gram_layers_step(const T *__restrict__ G, int64_t d, int64_t g, int64_t cb, int64_t ce,
                                                 double (&acc)[N * (N + 1) / 2]) {
    const int64_t c0 = g * VEC;
    // a group that reaches past the end of the row (d not a multiple of VEC) is read from d - VEC
    const int64_t lb = (EDGE && c0 + VEC > d) ? d - VEC : c0;
    float v[N][VEC];
#pragma unroll
    for (int i = 0; i < N; ++i) load_vec<T, VEC, STREAM>(G + (int64_t)i * d + lb, v[i]);
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        const bool live = !EDGE || (lb + c >= c0 && lb + c >= cb && lb + c < ce);
        double x[N];
#pragma unroll
        for (int i = 0; i < N; ++i) x[i] = live ? (double)v[i][c] : 0.0;
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
gram_layers_kernel(const T *__restrict__ G, int64_t d, const LayerRun *__restrict__ runs, int nruns,
                   const int *__restrict__ order, double *__restrict__ partials, int64_t cached_groups) {
    constexpr int NP = N * (N + 1) / 2;
    __shared__ double lds[4 * NP];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    // Workgroup b takes the runs order[b], order[b + grid], ...: the index is uniform, so a run's
    // descriptor comes through scalar loads, and the next run's is requested while this run streams.
    int k = (int)blockIdx.x;
    int r = 0;
    LayerRun run = {};
    if (k < nruns) {
        r = order[k];
        run = runs[r];
    }
    while (k < nruns) {
        const int kn = k + (int)gridDim.x;
        int rn = 0;
        LayerRun run_next = run;
        if (kn < nruns) {
            rn = order[kn];
            run_next = runs[rn];
        }
        __syncthreads();             // the previous run's sums have been read out of LDS
        double acc[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) acc[p] = 0.0;
        const int64_t g_end = run.g0 + run.n;
        // Only the first and the last group of a run can straddle a layer boundary.  Runs in the
        // head of G (below cached_groups) use ordinary loads, so that the head stays in the
        // memory-side cache for stage A3; the others stream past the caches.  Two loops: loads
        // that differ only in that hint would otherwise be merged into one kind.
        if (run.g0 < cached_groups) {
            for (int64_t g = run.g0 + threadIdx.x; g < g_end; g += kBlock) {
                if (g == run.g0 || g == g_end - 1)
                    gram_layers_step<N, T, VEC, true, false>(G, d, g, run.cb, run.ce, acc);
                else
                    gram_layers_step<N, T, VEC, false, false>(G, d, g, run.cb, run.ce, acc);
            }
        } else {
            for (int64_t g = run.g0 + threadIdx.x; g < g_end; g += kBlock) {
                if (g == run.g0 || g == g_end - 1)
                    gram_layers_step<N, T, VEC, true, true>(G, d, g, run.cb, run.ce, acc);
                else
                    gram_layers_step<N, T, VEC, false, true>(G, d, g, run.cb, run.ce, acc);
            }
        }
        // workgroup sum in a fixed order into this run's partial row
        {
            const double tot = wave_reduce_scatter<NP>(acc, lane);
            const int p = wave_scatter_index(lane);
            if (p < NP) lds[wave * NP + p] = tot;
        }
        __syncthreads();
        if (threadIdx.x < NP) {
            const int p = threadIdx.x;
            partials[(size_t)r * NP + p] = ((lds[p] + lds[NP + p]) + lds[2 * NP + p]) + lds[3 * NP + p];
        }
        k = kn;
        r = rn;
        run = run_next;
    }
}

// A1 for N > 8.  Same run bookkeeping as above; inside a run wavefront w takes the chunks
// w, w + 4, ... of LPR column groups.  Load j of a chunk: row RPL j + lane / LPR, group lane % LPR
// (four rows by 256 contiguous bytes per instruction up to 64 rows; eight rows by 128 bytes above,
// which keeps the registers of the 64-row instantiation).  Column sums s over the rows (in-lane, then
// across the lane groups), then q_i += <v_i, v_i>, r_i += <v_i, s> in fp64.  Groups past the
// end of the run and columns of a straddling group that belong to the neighbouring layer are
// zeroed.  One partial row [q_0 .. q_{N-1}, r_0 .. r_{N-1}] per run.
template <int NT, typename T>
__global__ void __launch_bounds__(kBlock, (((NT > 4) ? 2 * NT : 4 * NT) * VecWidth<T>::value >= 48) ? 1 : 2)
stats_layers_kernel(const T *__restrict__ G, int N, int64_t d, const LayerRun *__restrict__ runs, int nruns,
                    const int *__restrict__ order, double *__restrict__ partials) {
    constexpr int VECW = VecWidth<T>::value;
    constexpr int RPL = (NT > 4) ? 8 : 4;          // rows per load instruction
    constexpr int LPR = kWave / RPL;               // lanes (column groups) side by side in one row
    constexpr int kLoads = 16 * NT / RPL;
    __shared__ double lds[kBlock / kWave][2 * kNMax];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int grp = lane / LPR, cl = lane % LPR;
    // runs order[b], order[b + grid], ... of workgroup b; the next run's descriptor is requested early
    int k = (int)blockIdx.x;
    int r = 0;
    LayerRun run = {};
    if (k < nruns) {
        r = order[k];
        run = runs[r];
    }
    while (k < nruns) {
        const int kn = k + (int)gridDim.x;
        int rn = 0;
        LayerRun run_next = run;
        if (kn < nruns) {
            rn = order[kn];
            run_next = runs[rn];
        }
        __syncthreads();             // the previous run's sums have been read out of LDS
        double qacc[kLoads], racc[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) qacc[j] = racc[j] = 0.0;
        const int64_t g_end = run.g0 + run.n;
        const int nchunks = (run.n + LPR - 1) / LPR;
        // interior chunk: all of its groups belong to the run, none of their columns to a neighbouring
        // layer, and every row exists -- no clamps, no masks (they cost more than the arithmetic)
        auto chunk = [&](int c, auto interior) __attribute__((always_inline)) {
            constexpr bool kInterior = decltype(interior)::value;
            const int64_t g = run.g0 + LPR * (int64_t)c + cl;
            const bool in_run = kInterior || g < g_end;
            const int64_t gc = in_run ? g : g_end - 1;          // clamped: always a group of this run
            const int64_t c0 = gc * VECW;
            // a group that reaches past the end of the row (d not a multiple of VECW) is read from d - VECW
            const int64_t lb = (!kInterior && c0 + VECW > d) ? d - VECW : c0;
            u32x4 x[kLoads];
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                const int row = RPL * j + grp;
                const int rowc = (kInterior || row < N) ? row : N - 1;
                x[j] = *reinterpret_cast<const gu32x4 *>(G + (int64_t)rowc * d + lb);
            }
            bool live[VECW];
#pragma unroll
            for (int k = 0; k < VECW; ++k)
                live[k] = kInterior || (in_run && lb + k >= c0 && lb + k >= run.cb && lb + k < run.ce);
            double ssum[VECW];
#pragma unroll
            for (int k = 0; k < VECW; ++k) ssum[k] = 0.0;
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                float v[VECW];
                widen_bits<T>(x[j], v);
                const bool row_ok = kInterior || RPL * j + grp < N;
#pragma unroll
                for (int k = 0; k < VECW; ++k) ssum[k] += (row_ok && live[k]) ? (double)v[k] : 0.0;
            }
#pragma unroll
            for (int k = 0; k < VECW; ++k) {
#pragma unroll
                for (int off = LPR; off < kWave; off <<= 1) ssum[k] += __shfl_xor(ssum[k], off, kWave);
            }
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                float v[VECW];
                widen_bits<T>(x[j], v);
                const bool row_ok = kInterior || RPL * j + grp < N;
#pragma unroll
                for (int k = 0; k < VECW; ++k) {
                    const double y = (row_ok && live[k]) ? (double)v[k] : 0.0;
                    qacc[j] = fma(y, y, qacc[j]);
                    racc[j] = fma(y, ssum[k], racc[j]);
                }
            }
        };
        for (int c = wave; c < nchunks; c += kBlock / kWave) {
            const int64_t first = (run.g0 + LPR * (int64_t)c) * VECW;      // the chunk's columns [first, first + LPR VECW)
            const bool interior = N == 16 * NT && LPR * c + LPR <= run.n && first >= run.cb && first + LPR * VECW <= run.ce;
            if (interior) chunk(c, std::true_type{});
            else chunk(c, std::false_type{});
        }
        // the lanes of a group in a fixed butterfly order, then the wavefronts in index order
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            double q = qacc[j], rr = racc[j];
#pragma unroll
            for (int off = LPR / 2; off >= 1; off >>= 1) {
                q += __shfl_xor(q, off, kWave);
                rr += __shfl_xor(rr, off, kWave);
            }
            if (cl == 0) {
                lds[wave][RPL * j + grp] = q;
                lds[wave][kNMax + RPL * j + grp] = rr;
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < 2 * N) {
            const int t = threadIdx.x;
            const int e = t < N ? t : kNMax + (t - N);
            partials[(size_t)r * (2 * N) + t] = ((lds[0][e] + lds[1][e]) + lds[2][e]) + lds[3][e];
        }
        k = kn;
        r = rn;
        run = run_next;
    }
}

// ------------------------------------------------------------------------------------------
// A2: one workgroup per layer
// ------------------------------------------------------------------------------------------
constexpr int kLayerFinishBlock = 1024;
__global__ void __launch_bounds__(kLayerFinishBlock)
finish_layers_kernel(const double *__restrict__ partials, const int *__restrict__ layer_entry0, double *K_all,
                     DevState *ds_all, CoeffParams cp) {
    __shared__ double lds[4 * kNMax];
    __shared__ double K_lds[kLayersMaxN * kLayersMaxN];
    const bool stats = cp.N > kLayersMaxN;                   // rows hold [q, r] instead of the packed K
    const int l = blockIdx.x, N = cp.N, np = stats ? 2 * N : num_pairs(N);
    DevState *ds = ds_all + l;
    const double m_old = ((int)threadIdx.x < N) ? current_m(ds)[threadIdx.x] : 0.0;
    const int e0 = layer_entry0[l], e1 = layer_entry0[l + 1];
    // interleaved sub-sums over this layer's entries (entry order inside a slice), then the slices in order
    __shared__ double slice_sum[kLayerFinishBlock];
    const int slices = kLayerFinishBlock / np, sl = (int)threadIdx.x / np, pp = (int)threadIdx.x - sl * np;
    if (sl < slices) {
        double acc = 0.0;
        for (int e = e0 + sl; e < e1; e += slices) acc += partials[(size_t)e * np + pp];
        slice_sum[sl * np + pp] = acc;
    }
    __syncthreads();
    if (stats) {
        double q = 0.0, r = 0.0;
        if ((int)threadIdx.x < N) {
            for (int k = 0; k < slices; ++k) {
                q += slice_sum[k * np + threadIdx.x];
                r += slice_sum[k * np + N + threadIdx.x];
            }
        }
        update_coefficients_from_stats(q, r, ds, cp, lds, m_old);
        return;
    }
    if ((int)threadIdx.x < np) {
        const int p = threadIdx.x;
        double tot = 0.0;
        for (int q = 0; q < slices; ++q) tot += slice_sum[q * np + p];
        int i = 0, left = p;
        while (left >= N - i) {
            left -= N - i;
            ++i;
        }
        const int j = i + left;
        double *K = K_all + (size_t)l * N * N;
        K[i * N + j] = tot;
        K[j * N + i] = tot;
        K_lds[i * N + j] = tot;
        K_lds[j * N + i] = tot;
    }
    __syncthreads();
    update_coefficients(K_lds, ds, cp, lds, m_old);
}

// ------------------------------------------------------------------------------------------
// A3
// ------------------------------------------------------------------------------------------
// A run is cut into pieces of kWsumPiece column groups (run_groups is a multiple of it); a workgroup
// sweeps the pieces grid-stride.  A piece that lies inside its run and its layer is a full tile: two
// groups per thread, all 2 N loads issued before the first use, no predicates (as in the model-wise
// stage A3); the pieces at the end of a run or on a layer boundary go group by group with masks.
constexpr int kWsumPiece = 2 * kBlock;

template <int N, typename T, int VEC>
__global__ void __launch_bounds__(kBlock)
wsum_layers_kernel(const T *__restrict__ G, int64_t d, const LayerRun *__restrict__ runs, int nruns,
                   const int64_t *__restrict__ offsets, const DevState *__restrict__ ds_all, float *__restrict__ out,
                   int run_groups) {
    const int split = run_groups / kWsumPiece;
    const int grid = (int)gridDim.x, b = (int)blockIdx.x;
    const int slot = (grid % 8) ? b : (b % 8) * (grid / 8) + b / 8;   // XCD-contiguous pieces
    const int64_t npieces = (int64_t)nruns * split;
    for (int64_t pc = slot; pc < npieces; pc += grid) {
        const LayerRun run = runs[pc / split];
        const int first = (int)(pc % split) * kWsumPiece;
        if (first >= run.n) continue;
        const int last = (first + kWsumPiece < run.n) ? first + kWsumPiece : run.n;
        const float *gam = ds_all[run.layer].gamma32;
        float w[N];
#pragma unroll
        for (int i = 0; i < N; ++i) w[i] = gam[i];
        const int64_t cb = run.cb, ce = run.ce;
        const int64_t p0 = (run.g0 + first) * VEC;                     // first column of the piece
        if (first + kWsumPiece <= run.n && p0 >= cb && p0 + (int64_t)kWsumPiece * VEC <= ce) {
            float v[2][N][VEC];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < N; ++i)
                    load_vec<T, VEC, true>(G + (int64_t)i * d + p0 + ((int64_t)u * kBlock + threadIdx.x) * VEC, v[u][i]);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float acc[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
#pragma unroll
                for (int i = 0; i < N; ++i)
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc[c] = fmaf(w[i], v[u][i][c], acc[c]);
                float *dst = out + p0 + ((int64_t)u * kBlock + threadIdx.x) * VEC;
#pragma unroll
                for (int c = 0; c < VEC; c += 4) {
                    const f32x4 x = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
                    __builtin_nontemporal_store(x, reinterpret_cast<gf32x4 *>(dst + c));
                }
            }
            continue;
        }
        for (int k = first + (int)threadIdx.x; k < last; k += kBlock) {
            const int64_t c0 = (run.g0 + k) * VEC;
            const int64_t lb = (c0 + VEC > d) ? d - VEC : c0;   // the group at the ragged end of a row
            float v[N][VEC];
#pragma unroll
            for (int i = 0; i < N; ++i) load_vec<T, VEC, true>(G + (int64_t)i * d + lb, v[i]);
            float acc[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
#pragma unroll
            for (int i = 0; i < N; ++i)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = fmaf(w[i], v[i][c], acc[c]);
            if (c0 >= cb && c0 + VEC <= ce) {
#pragma unroll
                for (int c = 0; c < VEC; c += 4) {
                    const f32x4 x = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
                    __builtin_nontemporal_store(x, reinterpret_cast<gf32x4 *>(out + c0 + c));
                }
            } else {
                // group shared with a neighbouring layer, or at the ragged end of a row: store only
                // this group's columns of this layer
#pragma unroll
                for (int c = 0; c < VEC; ++c)
                    if (lb + c >= c0 && lb + c >= cb && lb + c < ce) out[lb + c] = acc[c];
            }
        }
    }
}

// One column group of stage A3 for a run-time number of rows: rows eight at a time, weights through
// uniform loads; a group shared with a neighbouring layer or at the ragged end of a row stores only
// this group's columns of this layer [cb, ce).
template <typename T, int VEC>
__device__ __forceinline__ void wsum_layers_rt_group(const T *__restrict__ G, int N, int64_t d, const float *gam,
                                                     int64_t c0, int64_t cb, int64_t ce, float *__restrict__ out) {
    const int64_t lb = (c0 + VEC > d) ? d - VEC : c0;   // a group that reaches past the row is read from d - VEC
    float acc[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
    for (int i0 = 0; i0 < N; i0 += 8) {
        float v[8][VEC];
#pragma unroll
        for (int ii = 0; ii < 8; ++ii)
            if (i0 + ii < N) load_vec<T, VEC, true>(G + (int64_t)(i0 + ii) * d + lb, v[ii]);
#pragma unroll
        for (int ii = 0; ii < 8; ++ii)
            if (i0 + ii < N) {
                const float w = gam[i0 + ii];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = fmaf(w, v[ii][c], acc[c]);
            }
    }
    if (c0 >= cb && c0 + VEC <= ce) {
#pragma unroll
        for (int c = 0; c < VEC; c += 4) {
            const f32x4 x = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
            __builtin_nontemporal_store(x, reinterpret_cast<gf32x4 *>(out + c0 + c));
        }
    } else {
#pragma unroll
        for (int c = 0; c < VEC; ++c)
            if (lb + c >= c0 && lb + c >= cb && lb + c < ce) out[lb + c] = acc[c];
    }
}

// A3 for N > 8: the number of rows is a run-time value, rows are walked eight at a time, the
// weights are read through uniform (scalar) loads of the run's layer.
template <typename T, int VEC>
__global__ void __launch_bounds__(kBlock)
wsum_layers_rt_kernel(const T *__restrict__ G, int N, int64_t d, const LayerRun *__restrict__ runs, int nruns,
                      const DevState *__restrict__ ds_all, float *__restrict__ out, int run_groups) {
    const int kWsumSplit = run_groups / kWsumPiece;
    constexpr int kPiece = kWsumPiece;
    const int grid = (int)gridDim.x, b = (int)blockIdx.x;
    const int slot = (grid % 8) ? b : (b % 8) * (grid / 8) + b / 8;   // XCD-contiguous pieces
    const int64_t npieces = (int64_t)nruns * kWsumSplit;
    for (int64_t pc = slot; pc < npieces; pc += grid) {
        const LayerRun run = runs[pc / kWsumSplit];
        const int first = (int)(pc % kWsumSplit) * kPiece;
        if (first >= run.n) continue;
        const int last = (first + kPiece < run.n) ? first + kPiece : run.n;
        const float *gam = ds_all[run.layer].gamma32;
        const int64_t cb = run.cb, ce = run.ce;
        for (int k = first + (int)threadIdx.x; k < last; k += kBlock) {
            wsum_layers_rt_group<T, VEC>(G, N, d, gam, (run.g0 + k) * VEC, cb, ce, out);
        }
    }
}

// The same with the output parked in LDS and written in bursts (long fp32 streams of many rows: a
// steady trickle of stores among the loads costs such a pass about a tenth of its time).  One
// workgroup per CU; a piece that lies inside its run and its layer leaves an image of its
// kWsumPiece * VEC output columns in LDS, and `cap` images are written back to back; the other
// pieces go group by group with masks as above.  Same sums in the same order as the kernel above.
template <typename T, int VEC>
__global__ void __launch_bounds__(kBlock)
wsum_layers_rt_parked_kernel(const T *__restrict__ G, int N, int64_t d, const LayerRun *__restrict__ runs, int nruns,
                             const DevState *__restrict__ ds_all, float *__restrict__ out, int run_groups, int cap) {
    constexpr int kPiece = kWsumPiece;
    constexpr int kPieceCols = kPiece * VEC;
    extern __shared__ __attribute__((aligned(16))) float park[];            // cap images of kPieceCols floats ...
    int64_t *dest = reinterpret_cast<int64_t *>(park + (size_t)cap * kPieceCols);   // ... and their first columns
    const int split = run_groups / kPiece;
    const int grid = (int)gridDim.x, b = (int)blockIdx.x;
    const int slot = (grid % 8) ? b : (b % 8) * (grid / 8) + b / 8;   // XCD-contiguous pieces
    const int64_t npieces = (int64_t)nruns * split;
    int parked = 0;
    auto flush = [&]() __attribute__((always_inline)) {
        __syncthreads();   // images and destinations are complete
        for (int k = 0; k < parked; ++k) {
            float *dst = out + dest[k];
            const float *src = park + (size_t)k * kPieceCols;
#pragma unroll
            for (int q = 0; q < kPieceCols / 4 / kBlock; ++q) {
                const int e = (q * kBlock + (int)threadIdx.x) * 4;   // 1 KB per wavefront and instruction
                __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(src + e), reinterpret_cast<gf32x4 *>(dst + e));
            }
        }
        __syncthreads();   // the images may be overwritten
        parked = 0;
    };
    for (int64_t pc = slot; pc < npieces; pc += grid) {   // uniform over the workgroup
        const LayerRun run = runs[pc / split];
        const int first = (int)(pc % split) * kPiece;
        if (first >= run.n) continue;
        const int last = (first + kPiece < run.n) ? first + kPiece : run.n;
        const float *gam = ds_all[run.layer].gamma32;
        const int64_t cb = run.cb, ce = run.ce;
        const int64_t p0 = (run.g0 + first) * VEC;   // first column of the piece
        if (first + kPiece <= run.n && p0 >= cb && p0 + (int64_t)kPieceCols <= ce) {
            constexpr int U = kPiece / kBlock;   // groups per thread
            float acc[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[u][c] = 0.f;
            for (int i0 = 0; i0 < N; i0 += 8) {
                float v[U][8][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int ii = 0; ii < 8; ++ii)
                        if (i0 + ii < N)
                            load_vec<T, VEC, true>(G + (int64_t)(i0 + ii) * d + p0 + ((int64_t)u * kBlock + threadIdx.x) * VEC, v[u][ii]);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int ii = 0; ii < 8; ++ii)
                        if (i0 + ii < N) {
                            const float w = gam[i0 + ii];
#pragma unroll
                            for (int c = 0; c < VEC; ++c) acc[u][c] = fmaf(w, v[u][ii][c], acc[u][c]);
                        }
            }
            float *img = park + (size_t)parked * kPieceCols;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < VEC; c += 4) {
                    const f32x4 x = {acc[u][c], acc[u][c + 1], acc[u][c + 2], acc[u][c + 3]};
                    *reinterpret_cast<f32x4 *>(img + ((size_t)u * kBlock + threadIdx.x) * VEC + c) = x;
                }
            if (threadIdx.x == 0) dest[parked] = p0;
            if (++parked == cap) flush();
            continue;
        }
        for (int k = first + (int)threadIdx.x; k < last; k += kBlock) {
            wsum_layers_rt_group<T, VEC>(G, N, d, gam, (run.g0 + k) * VEC, cb, ce, out);
        }
    }
    if (parked > 0) flush();
}

// Launch of stage A3 for N > 8: parked output where it measured faster model-wise (fp32, N >= 12,
// d >= 2^24), else the plain kernel.
template <typename T, int VEC>
static hipError_t launch_wsum_layers_rt(const void *G, int N, int64_t d, const LayerRun *runs, int nruns, int run_groups,
                                        int wsum_grid, const DevState *ds_all, float *out, hipStream_t s) {
    if (sizeof(T) == 4 && N >= 12 && d >= ((int64_t)1 << 24)) {
        constexpr int kImageBytes = kWsumPiece * VEC * 4;
        constexpr int cap = 128 * 1024 / kImageBytes;
        constexpr int lds_bytes = cap * kImageBytes + cap * 8;
        static bool allowed[64] = {};   // more than 64 KB of dynamic LDS: allowed once per kernel and device
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64 || !allowed[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(wsum_layers_rt_parked_kernel<T, VEC>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            if (e != hipSuccess) return e;
            if (dev >= 0 && dev < 64) allowed[dev] = true;
        }
        hipLaunchKernelGGL((wsum_layers_rt_parked_kernel<T, VEC>), dim3(wsum_grid / 8), dim3(kBlock), lds_bytes, s,
                           static_cast<const T *>(G), N, d, runs, nruns, ds_all, out, run_groups, cap);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((wsum_layers_rt_kernel<T, VEC>), dim3(wsum_grid), dim3(kBlock), 0, s, static_cast<const T *>(G),
                       N, d, runs, nruns, ds_all, out, run_groups);
    return hipGetLastError();
}

template <int NT, typename T, int VEC>
static hipError_t run_layers_stats(const void *G, int N, int64_t d, const LayerRun *runs, int nruns, int run_groups, const int *order,
                                   int gram_grid, int wsum_grid, const int *layer_entry0, int L, double *partials,
                                   double *K_all, DevState *ds_all, CoeffParams cp, float *out,
                                   hipStream_t s) {
    hipLaunchKernelGGL((stats_layers_kernel<NT, T>), dim3(gram_grid), dim3(kBlock), 0, s, static_cast<const T *>(G), N,
                       d, runs, nruns, order, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(finish_layers_kernel, dim3(L), dim3(kLayerFinishBlock), 0, s, partials, layer_entry0, K_all,
                       ds_all, cp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    return launch_wsum_layers_rt<T, VEC>(G, N, d, runs, nruns, run_groups, wsum_grid, ds_all, out, s);
}

template <typename T, int VEC, typename... A>
static hipError_t dispatch_layers_stats(int N, const void *G, A... a) {
    switch ((N + 15) / 16) {
        case 1: return run_layers_stats<1, T, VEC>(G, N, a...);
        case 2: return run_layers_stats<2, T, VEC>(G, N, a...);
        case 3: return run_layers_stats<3, T, VEC>(G, N, a...);
        case 4: return run_layers_stats<4, T, VEC>(G, N, a...);
        case 5: return run_layers_stats<5, T, VEC>(G, N, a...);
        case 6: return run_layers_stats<6, T, VEC>(G, N, a...);
        case 7: return run_layers_stats<7, T, VEC>(G, N, a...);
        case 8: return run_layers_stats<8, T, VEC>(G, N, a...);
        default: return hipErrorInvalidValue;
    }
}

template <int N, typename T, int VEC>
static hipError_t run_layers(const void *G, int64_t d, const LayerRun *runs, int nruns, int run_groups, const int *order, int gram_grid, int wsum_grid,
                             const int64_t *offsets, const int *layer_entry0, int L, double *partials, double *K_all,
                             DevState *ds_all, CoeffParams cp, float *out, hipStream_t s) {
    // the first 320 MiB of G with cache-allocating loads (same policy as the model-wise stage A1)
    const int64_t cached_groups = ((int64_t)320 << 20) / ((int64_t)N * VEC * (int64_t)sizeof(T));
    hipLaunchKernelGGL((gram_layers_kernel<N, T, VEC>), dim3(gram_grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(G), d, runs, nruns, order, partials, cached_groups);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(finish_layers_kernel, dim3(L), dim3(kLayerFinishBlock), 0, s, partials, layer_entry0, K_all,
                       ds_all, cp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL((wsum_layers_kernel<N, T, VEC>), dim3(wsum_grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(G), d, runs, nruns, offsets, ds_all, out, run_groups);
    return hipGetLastError();
}

template <typename T, int VEC, typename... A>
static hipError_t dispatch_layers(int N, A... a) {
    switch (N) {
        case 1: return run_layers<1, T, VEC>(a...);
        case 2: return run_layers<2, T, VEC>(a...);
        case 3: return run_layers<3, T, VEC>(a...);
        case 4: return run_layers<4, T, VEC>(a...);
        case 5: return run_layers<5, T, VEC>(a...);
        case 6: return run_layers<6, T, VEC>(a...);
        case 7: return run_layers<7, T, VEC>(a...);
        case 8: return run_layers<8, T, VEC>(a...);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace adacons

using namespace adacons;

struct adacons_layers {
    int N, L, device;
    int64_t d;
    adacons_dtype dtype;
    double beta;
    unsigned flags;
    int nruns, run_groups, gram_grid, wsum_grid;
    LayerRun *runs;       // device, nruns
    int64_t *offsets;     // device, L + 1
    int *layer_entry0;    // device, L + 1
    double *partials;     // device, nruns x N(N+1)/2
    double *K;            // device, L x N x N
    DevState *ds;         // device, L
    int *order;           // device, nruns: the order stage A1 takes the runs in (full-length runs in column order, then the
                          // shorter ones, longest first, so that the sweep ends on small pieces)
};

namespace {
adacons_status lfail(adacons_status s, const char *msg) { return set_error(s, "%s", msg); }
}  // namespace

extern "C" {

adacons_status adacons_destroy_layers(adacons_layers *ls) {
    if (!ls) return ADACONS_OK;
    void *bufs[] = {ls->runs, ls->offsets, ls->layer_entry0, ls->partials, ls->K, ls->ds, ls->order};
    for (void *p : bufs)
        if (p) (void)hipFree(p);
    delete ls;
    return ADACONS_OK;
}

adacons_status adacons_init_layers(adacons_layers **out_ls, int N, int L, const int64_t *offsets_host,
                                   adacons_dtype dtype, double beta, unsigned flags, void *hip_stream) {
    if (!out_ls) return lfail(ADACONS_EINVAL, "ls is NULL");
    *out_ls = nullptr;
    if (!offsets_host) return lfail(ADACONS_EINVAL, "offsets_host is NULL");
    if (N < 1 || L < 1) return lfail(ADACONS_EINVAL, "N < 1 or L < 1");
    if (N > ADACONS_N_MAX) return lfail(ADACONS_EUNSUPPORTED, "N > ADACONS_N_MAX");
    if (dtype != ADACONS_F32 && dtype != ADACONS_BF16) return lfail(ADACONS_EUNSUPPORTED, "unknown dtype");
    if (!(beta >= 0.0 && beta < 1.0)) return lfail(ADACONS_EINVAL, "beta outside [0, 1)");
    if (flags & ~ADACONS_FLAG_ALL_) return lfail(ADACONS_EINVAL, "unknown flag bits");
    if (offsets_host[0] != 0) return lfail(ADACONS_EINVAL, "offsets[0] must be 0");
    for (int l = 0; l < L; ++l)
        if (offsets_host[l + 1] <= offsets_host[l]) return lfail(ADACONS_EINVAL, "offsets must ascend strictly");
    if (L > (1 << 20)) return lfail(ADACONS_EINVAL, "too many layers");
    if (offsets_host[L] < (dtype == ADACONS_BF16 ? 8 : 4))
        return lfail(ADACONS_EINVAL, "layer-wise aggregation needs d >= one 128-bit group (4 fp32 / 8 bf16 elements)");

    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
        return lfail(ADACONS_EHIP, "no HIP device");
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return lfail(ADACONS_EUNSUPPORTED, "built for gfx950 only");

    const int vec = dtype == ADACONS_BF16 ? 8 : 4;
    // measured (ResNet-50 layout, N = 8): 144 us at two workgroups per CU, 152 at one, 155 at three; with few
    // rows a thread has few loads in flight (N per column group), and more workgroups make up for it
    const int per_cu = N <= 2 ? 8 : (N <= 4 ? 4 : 2);
    const int grid_target = prop.multiProcessorCount * per_cu;
    const int run_groups = choose_run_groups(offsets_host, L, vec, grid_target);
    // runs: per layer, the groups that contain any of its columns, cut into pieces of run_groups
    std::vector<LayerRun> runs;
    std::vector<int> layer_entry0(L + 1);
    for (int l = 0; l < L; ++l) {
        layer_entry0[l] = (int)runs.size();
        const int64_t g_first = offsets_host[l] / vec, g_last = (offsets_host[l + 1] + vec - 1) / vec;
        for (int64_t g = g_first; g < g_last; g += run_groups) {
            LayerRun r;
            r.g0 = g;
            r.cb = offsets_host[l];
            r.ce = offsets_host[l + 1];
            r.n = (int)((g_last - g < run_groups) ? g_last - g : run_groups);
            r.layer = l;
            runs.push_back(r);
        }
        if (runs.size() > (size_t)0x0fffffff) return lfail(ADACONS_EINVAL, "too many runs");
    }
    const int nruns = (int)runs.size();
    layer_entry0[L] = nruns;
    std::vector<int> order;
    order.reserve(nruns);
    for (int r = 0; r < nruns; ++r)
        if (runs[r].n == run_groups) order.push_back(r);
    {
        std::vector<int> rest;
        for (int r = 0; r < nruns; ++r)
            if (runs[r].n != run_groups) rest.push_back(r);
        std::stable_sort(rest.begin(), rest.end(), [&](int a, int b) { return runs[a].n > runs[b].n; });
        order.insert(order.end(), rest.begin(), rest.end());
    }
    int gram_grid = grid_target;
    if (gram_grid > nruns) gram_grid = nruns;

    adacons_layers *ls = new (std::nothrow) adacons_layers();
    if (!ls) return lfail(ADACONS_ENOMEM, "host allocation failed");
    memset(ls, 0, sizeof *ls);
    ls->N = N; ls->L = L; ls->device = dev; ls->d = offsets_host[L]; ls->dtype = dtype; ls->beta = beta; ls->flags = flags;
    ls->nruns = nruns; ls->run_groups = run_groups; ls->gram_grid = gram_grid;
    ls->wsum_grid = prop.multiProcessorCount * 8;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int np = N > kLayersMaxN ? 2 * N : num_pairs(N);   // doubles per partial row
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&ls->runs), sizeof(LayerRun) * (size_t)nruns);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ls->offsets), sizeof(int64_t) * (size_t)(L + 1));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ls->layer_entry0), sizeof(int) * (size_t)(L + 1));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ls->partials), sizeof(double) * (size_t)nruns * np);
    // K per layer exists only where stage A1 forms it (N <= kLayersMaxN); the statistics pass never touches it
    const size_t k_doubles = N > kLayersMaxN ? 1 : (size_t)L * N * N;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ls->K), sizeof(double) * k_doubles);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ls->ds), sizeof(DevState) * (size_t)L);
    if (e == hipSuccess) e = hipMemcpyAsync(ls->runs, runs.data(), sizeof(LayerRun) * (size_t)nruns, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(ls->offsets, offsets_host, sizeof(int64_t) * (size_t)(L + 1), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(ls->layer_entry0, layer_entry0.data(), sizeof(int) * (size_t)(L + 1), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ls->order), sizeof(int) * (size_t)nruns);
    if (e == hipSuccess) e = hipMemcpyAsync(ls->order, order.data(), sizeof(int) * (size_t)nruns, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemsetAsync(ls->ds, 0, sizeof(DevState) * (size_t)L, s);
    if (e == hipSuccess) e = hipMemsetAsync(ls->K, 0, sizeof(double) * k_doubles, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);   // the host vectors above go out of scope
    if (e != hipSuccess) {
        adacons_destroy_layers(ls);
        return lfail(e == hipErrorOutOfMemory ? ADACONS_ENOMEM : ADACONS_EHIP, hipGetErrorString(e));
    }
    *out_ls = ls;
    return ADACONS_OK;
}

adacons_status adacons_aggregate_layers(const void *G, int N, int64_t d, adacons_dtype dtype, adacons_layers *ls,
                                        float *out, void *hip_stream) {
    if (!ls || !G || !out) return lfail(ADACONS_EINVAL, "NULL argument");
    if (N != ls->N || d != ls->d || dtype != ls->dtype) return lfail(ADACONS_EINVAL, "N, d or dtype differ from init");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ls->device) return lfail(ADACONS_EINVAL, "the layer state lives on another device");
    const size_t es = dtype == ADACONS_BF16 ? 2 : 4;
    const uintptr_t g0 = reinterpret_cast<uintptr_t>(G), o0 = reinterpret_cast<uintptr_t>(out);
    if (g0 % es || o0 % 4) return lfail(ADACONS_EALIGN, "G or out not aligned to its element size");
    const uintptr_t g1 = g0 + (uint64_t)N * (uint64_t)d * es, o1 = o0 + (uint64_t)d * 4;
    if (o0 < g1 && g0 < o1) return lfail(ADACONS_EINVAL, "out overlaps G");
    CoeffParams cp;
    cp.N = N; cp.beta = ls->beta; cp.flags = ls->flags;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (N > kLayersMaxN) {
        if (dtype == ADACONS_F32)
            e = dispatch_layers_stats<float, 4>(N, G, d, (const LayerRun *)ls->runs, ls->nruns, ls->run_groups, (const int *)ls->order,
                                                ls->gram_grid, ls->wsum_grid, (const int *)ls->layer_entry0, ls->L,
                                                ls->partials, ls->K, ls->ds, cp, out, s);
        else
            e = dispatch_layers_stats<bf16_bits, 8>(N, G, d, (const LayerRun *)ls->runs, ls->nruns, ls->run_groups, (const int *)ls->order,
                                                    ls->gram_grid, ls->wsum_grid, (const int *)ls->layer_entry0, ls->L,
                                                    ls->partials, ls->K, ls->ds, cp, out, s);
    } else if (dtype == ADACONS_F32)
        e = dispatch_layers<float, 4>(N, G, d, (const LayerRun *)ls->runs, ls->nruns, ls->run_groups, (const int *)ls->order, ls->gram_grid, ls->wsum_grid,
                                      (const int64_t *)ls->offsets, (const int *)ls->layer_entry0, ls->L, ls->partials,
                                      ls->K, ls->ds, cp, out, s);
    else
        e = dispatch_layers<bf16_bits, 8>(N, G, d, (const LayerRun *)ls->runs, ls->nruns, ls->run_groups, (const int *)ls->order, ls->gram_grid, ls->wsum_grid,
                                          (const int64_t *)ls->offsets, (const int *)ls->layer_entry0, ls->L,
                                          ls->partials, ls->K, ls->ds, cp, out, s);
    if (e != hipSuccess) return lfail(ADACONS_EHIP, hipGetErrorString(e));
    return ADACONS_OK;
}

adacons_status adacons_layer_coeffs(const adacons_layers *ls, double *gamma_host, double *raw_host,
                                    double *smoothed_host, uint32_t *numeric_flags, void *hip_stream) {
    if (!ls || !gamma_host) return lfail(ADACONS_EINVAL, "NULL argument");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    std::vector<DevState> host((size_t)ls->L);
    hipError_t e = hipMemcpyAsync(host.data(), ls->ds, sizeof(DevState) * (size_t)ls->L, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return lfail(ADACONS_EHIP, hipGetErrorString(e));
    for (int l = 0; l < ls->L; ++l) {
        for (int i = 0; i < ls->N; ++i) {
            gamma_host[(size_t)l * ls->N + i] = host[l].gamma[i];
            if (raw_host) raw_host[(size_t)l * ls->N + i] = host[l].a_raw[i];
            if (smoothed_host) smoothed_host[(size_t)l * ls->N + i] = host[l].a_smooth[i];
        }
        if (numeric_flags) numeric_flags[l] = host[l].numeric_flags;
    }
    return ADACONS_OK;
}

}  // extern "C"
