// Stage A3: out[k] = sum_i gamma_i G[i][k]  (Eq. 12), fp32 accumulate, fp32 out.
//
// A streaming kernel: one thread owns VEC consecutive columns, loads them from all N rows
// (128-bit loads, eight rows in flight at a time), applies the weights in worker order
// i = 0..N-1 with fused multiply-adds, and writes VEC floats.  G is read for the last time
// here and `out` is not read back by this library, so both use non-temporal accesses.  The tiles are
// walked forwards: the pass starts on the head of G, which stage A1 left in the memory-side cache.
#include "adacons_internal.h"
#include "coeff_device.h"
#include "device_util.h"

namespace adacons {

constexpr int kRowsInFlight = 8;
constexpr int kParkBlock = kBlock;   // workgroup size of wsum_parked_kernel (512 measured 3-8 % slower)

// APPLY = false: out[col..] = acc (non-temporal).  APPLY = true: the descent step of Eq. 4 in
// place, out[col..] = out[col..] - lr * acc (out is then the parameter vector w).  w streams past the
// caches like everything else here: read and written with ordinary accesses it pushed the head of G, which
// stage A1 left for this pass, out of the memory-side cache, and the fused step cost 52-95 us on top of the
// plain aggregation at d = 25.6 M (N = 16, 64) where the extra 102 MB read is worth 16; streamed, 14 us.
// wv: the VEC values of w, requested by the caller together with the rows of G (APPLY only; read at the
// time of the store they would add a memory latency to every tile).
template <int VEC, bool APPLY>
__device__ __forceinline__ void store_out(float *__restrict__ out, int64_t col, const float (&acc)[VEC], float lr,
                                          const float (&wv)[VEC]) {
#pragma unroll
    for (int c = 0; c < VEC; c += 4) {
        gf32x4 *dst = reinterpret_cast<gf32x4 *>(out + col + c);
        if constexpr (APPLY) {
            const f32x4 x = {fmaf(-lr, acc[c], wv[c]), fmaf(-lr, acc[c + 1], wv[c + 1]), fmaf(-lr, acc[c + 2], wv[c + 2]),
                             fmaf(-lr, acc[c + 3], wv[c + 3])};
            __builtin_nontemporal_store(x, dst);
        } else {
            const f32x4 x = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
            __builtin_nontemporal_store(x, dst);
        }
    }
}

// The updated parameters on the short path (a few megabytes: they stay in the caches for the next step): ordinary stores.
template <int VEC>
__device__ __forceinline__ void store_params(float *__restrict__ w, int64_t col, const float (&x)[VEC]) {
#pragma unroll
    for (int c = 0; c < VEC; c += 4) {
        const f32x4 y = {x[c], x[c + 1], x[c + 2], x[c + 3]};
        *reinterpret_cast<gf32x4 *>(w + col + c) = y;
    }
}

// Eight columns per lane (bf16 inputs): a lane's two 16-byte stores would each fill every other
// 16 bytes of the wavefront's 2 KB of output, i.e. half of every 32-byte sector per instruction.
// Exchanged across the wavefront first, each store instruction writes 1 KB without gaps: lane l
// takes columns 4 l .. 4 l + 3 of the first half from lane l / 2 and of the second half from
// lane 32 + l / 2.  All 64 lanes must be active.  `wave_col` is the first column of the wavefront.
__device__ __forceinline__ void store_out_wave8(float *__restrict__ out, int64_t wave_col, const float (&acc)[8]) {
    const int lane = threadIdx.x & (kWave - 1);
    const int odd = lane & 1;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int src = h * 32 + (lane >> 1);
        float v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float lo = __shfl(acc[c], src, kWave), hi = __shfl(acc[4 + c], src, kWave);
            v[c] = odd ? hi : lo;
        }
        const f32x4 x = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(x, reinterpret_cast<gf32x4 *>(out + wave_col + h * 256 + lane * 4));
    }
}

// One tile = BLK * UNR column groups (BLK = workgroup size): thread t owns groups base + u * BLK, u < UNR.
// FULL: every group of the tile exists, so the loads carry no predicate and are all issued
// before the first use.  PARK (FULL tiles only): the sums go to `park`, an image of the tile's
// BLK * UNR * VEC output columns in LDS, instead of to memory.
template <int NCT, typename T, int VEC, int UNR, bool FULL, bool APPLY, bool PARK = false, int BLK = kBlock>
__device__ __forceinline__ void wsum_tile(const T *__restrict__ G, const int N, const int64_t d, const int64_t ngroups,
                                          const int64_t base, const float *gam, float *__restrict__ out, float lr,
                                          float *park = nullptr) {
    float acc[UNR][VEC];
    float wv[UNR][VEC];   // APPLY, stored directly: the parameters this tile updates, requested ahead of the rows
    bool live[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        live[u] = FULL || (base + (int64_t)u * BLK < ngroups);
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[u][c] = 0.f;
        if constexpr (APPLY && !PARK) {
            if (live[u]) {
#pragma unroll
                for (int c = 0; c < VEC; c += 4) {
                    const f32x4 w4 = __builtin_nontemporal_load(reinterpret_cast<const gf32x4 *>(out + (base + (int64_t)u * BLK) * VEC + c));
                    wv[u][c] = w4.x, wv[u][c + 1] = w4.y, wv[u][c + 2] = w4.z, wv[u][c + 3] = w4.w;
                }
            }
        }
    }
#pragma clang loop unroll_count(NCT > 0 ? (NCT + kRowsInFlight - 1) / kRowsInFlight : 1)
    for (int i0 = 0; i0 < N; i0 += kRowsInFlight) {
        float v[UNR][kRowsInFlight][VEC];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int ii = 0; ii < kRowsInFlight; ++ii)
                if ((NCT > 0 || i0 + ii < N) && (NCT == 0 || i0 + ii < NCT) && live[u])
                    load_vec<T, VEC, true>(G + (int64_t)(i0 + ii) * d + (base + (int64_t)u * BLK) * VEC, v[u][ii]);
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int ii = 0; ii < kRowsInFlight; ++ii)
                if ((NCT > 0 || i0 + ii < N) && (NCT == 0 || i0 + ii < NCT) && live[u]) {
                    const float w = gam[i0 + ii];
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc[u][c] = fmaf(w, v[u][ii][c], acc[u][c]);
                }
    }
    if constexpr (PARK) {
        static_assert(FULL, "only whole tiles are parked");
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int c = 0; c < VEC; c += 4) {
                const f32x4 x = {acc[u][c], acc[u][c + 1], acc[u][c + 2], acc[u][c + 3]};
                *reinterpret_cast<f32x4 *>(park + ((size_t)u * BLK + threadIdx.x) * VEC + c) = x;
            }
    } else if constexpr (FULL && !APPLY && VEC == 8) {
        const int64_t wave_base = base - (threadIdx.x & (kWave - 1));   // group of lane 0
#pragma unroll
        for (int u = 0; u < UNR; ++u) store_out_wave8(out, (wave_base + (int64_t)u * BLK) * VEC, acc[u]);
    } else {
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (live[u]) store_out<VEC, APPLY>(out, (base + (int64_t)u * BLK) * VEC, acc[u], lr, wv[u]);
    }
}

// NCT > 0: N known at compile time (rows fully unrolled, weights in registers, N <= 16);
// NCT == 0: N taken from n_rt, rows walked eight at a time, weights in LDS.
// Eight wavefronts per SIMD (at most 64 vector registers) where the tile fits them: fp32 rows known at
// compile time, sixteen 128-bit loads per thread.  The launcher asks for eight workgroups per CU; at 72
// registers only seven are resident, and the pass measured 7 % slower (N = 8, d = 25.6 M: 148 against 138 us).
template <int NCT, typename T, int UNR, bool APPLY>
constexpr int wsum_min_waves() { return (sizeof(T) == 4 && NCT > 0 && NCT * UNR <= 16) ? (APPLY ? 5 : 8) : 1; }

template <int NCT, typename T, int VEC, int UNR, bool APPLY>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(wsum_min_waves<NCT, T, UNR, APPLY>(), 8)))
wsum_kernel(const T *__restrict__ G, int n_rt, int64_t d, int64_t ngroups, const float *__restrict__ gamma,
            float *__restrict__ out, float lr) {
    const int N = (NCT > 0) ? NCT : n_rt;
    __shared__ float gam_lds[kNMax];
    float gam_reg[NCT > 0 ? NCT : 1];
    const float *gam;
    if constexpr (NCT > 0) {
#pragma unroll
        for (int i = 0; i < NCT; ++i) gam_reg[i] = gamma[i];
        gam = gam_reg;
    } else {
        if (threadIdx.x < N) gam_lds[threadIdx.x] = gamma[threadIdx.x];
        __syncthreads();
        gam = gam_lds;
    }
    constexpr int64_t kTile = (int64_t)kBlock * UNR;
    const int64_t ntiles = (ngroups + kTile - 1) / kTile;
    // each XCD (workgroup index % 8) takes a contiguous run of tiles inside one sweep of the grid,
    // so that the 128-byte lines shared by neighbouring tiles are shared inside one L2
    const int grid = (int)gridDim.x, b = (int)blockIdx.x;
    const int slot = (grid % 8) ? b : (b % 8) * (grid / 8) + b / 8;
    for (int64_t t = slot; t < ntiles; t += gridDim.x) {
        const int64_t tt = t;
        const int64_t base = tt * kTile + threadIdx.x;
        if ((tt + 1) * kTile <= ngroups)
            wsum_tile<NCT, T, VEC, UNR, true, APPLY>(G, N, d, ngroups, base, gam, out, lr);
        else
            wsum_tile<NCT, T, VEC, UNR, false, APPLY>(G, N, d, ngroups, base, gam, out, lr);
    }
}

// The same sums with the output parked in LDS and written in bursts.  Measured on long streams
// (N = 64, d = 25.6 M: 6.5 GB read per 102 MB written): stores issued tile by tile, a steady trickle
// among the reads, cost 170 us on top of the 950 us the reads take; one workgroup per CU that parks
// `cap` whole tiles of output (128 KB) and then writes them back to back costs 20 us.  Every
// workgroup takes the same tiles as in wsum_kernel; a partial last tile is stored directly.
template <int NCT, typename T, int VEC, int UNR, bool APPLY, int BLK>
__global__ void __launch_bounds__(BLK)
wsum_parked_kernel(const T *__restrict__ G, int n_rt, int64_t d, int64_t ngroups, const float *__restrict__ gamma,
                   float *__restrict__ out, float lr, int cap) {
    extern __shared__ __attribute__((aligned(16))) float park[];   // cap tiles of kTileCols floats
    const int N = (NCT > 0) ? NCT : n_rt;
    __shared__ float gam_lds[kNMax];
    float gam_reg[NCT > 0 ? NCT : 1];
    const float *gam;
    if constexpr (NCT > 0) {
#pragma unroll
        for (int i = 0; i < NCT; ++i) gam_reg[i] = gamma[i];
        gam = gam_reg;
    } else {
        if (threadIdx.x < N) gam_lds[threadIdx.x] = gamma[threadIdx.x];
        __syncthreads();
        gam = gam_lds;
    }
    constexpr int64_t kTile = (int64_t)BLK * UNR;
    constexpr int kTileCols = BLK * UNR * VEC;
    const int64_t ntiles = (ngroups + kTile - 1) / kTile;
    const int grid = (int)gridDim.x, b = (int)blockIdx.x;
    const int slot = (grid % 8) ? b : (b % 8) * (grid / 8) + b / 8;
    // the q-th tile of this workgroup: one per sweep of the grid, as in wsum_kernel (runs of neighbouring
    // tiles per workgroup measured 10-20 % slower for N >= 12 at d = 25.6 M)
    auto tile_of = [&](int64_t q) __attribute__((always_inline)) -> int64_t { return (int64_t)slot + q * grid; };
    // parked tiles are the q_first-th, ... of this workgroup: written out when `cap` of them are waiting
    auto flush = [&](int64_t q_first, int n) __attribute__((always_inline)) {
        __syncthreads();   // the images are complete
        constexpr int kPieces = kTileCols / 4 / BLK;   // 128-bit pieces per thread and tile
        if constexpr (APPLY) {
            // the parameters of four tiles are requested together, then updated and written: one memory latency
            // per four tiles, not one per tile
            constexpr int kAhead = 4;
            for (int k0 = 0; k0 < n; k0 += kAhead) {
                f32x4 w[kAhead][kPieces];
#pragma unroll
                for (int a = 0; a < kAhead; ++a)
                    if (k0 + a < n) {
                        const float *dst = out + tile_of(q_first + k0 + a) * kTileCols;
#pragma unroll
                        for (int q = 0; q < kPieces; ++q)
                            w[a][q] = __builtin_nontemporal_load(reinterpret_cast<const gf32x4 *>(dst + (q * BLK + (int)threadIdx.x) * 4));
                    }
#pragma unroll
                for (int a = 0; a < kAhead; ++a)
                    if (k0 + a < n) {
                        float *dst = out + tile_of(q_first + k0 + a) * kTileCols;
                        const float *src = park + (size_t)(k0 + a) * kTileCols;
#pragma unroll
                        for (int q = 0; q < kPieces; ++q) {
                            const int e = (q * BLK + (int)threadIdx.x) * 4;
                            const f32x4 x = *reinterpret_cast<const f32x4 *>(src + e);
                            const f32x4 y = {fmaf(-lr, x.x, w[a][q].x), fmaf(-lr, x.y, w[a][q].y), fmaf(-lr, x.z, w[a][q].z),
                                             fmaf(-lr, x.w, w[a][q].w)};
                            __builtin_nontemporal_store(y, reinterpret_cast<gf32x4 *>(dst + e));
                        }
                    }
            }
        } else {
            for (int k = 0; k < n; ++k) {
                float *dst = out + tile_of(q_first + k) * kTileCols;
                const float *src = park + (size_t)k * kTileCols;
#pragma unroll
                for (int q = 0; q < kPieces; ++q) {
                    const int e = (q * BLK + (int)threadIdx.x) * 4;   // 1 KB per wavefront and instruction
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(src + e);
                    __builtin_nontemporal_store(x, reinterpret_cast<gf32x4 *>(dst + e));
                }
            }
        }
        __syncthreads();   // the images may be overwritten
    };
    int parked = 0;
    int64_t q_first = 0;
    for (int64_t q = 0;; ++q) {   // uniform over the workgroup
        const int64_t t = tile_of(q);
        if (t >= ntiles) break;   // tile_of ascends
        const int64_t tt = t;
        const int64_t base = tt * kTile + threadIdx.x;
        if ((tt + 1) * kTile <= ngroups) {
            if (parked == 0) q_first = q;
            wsum_tile<NCT, T, VEC, UNR, true, APPLY, true, BLK>(G, N, d, ngroups, base, gam, out, lr,
                                                           park + (size_t)parked * kTileCols);
            if (++parked == cap) {
                flush(q_first, parked);
                parked = 0;
            }
        } else {
            if (parked > 0) {   // keeps the parked tiles consecutive in this workgroup's sequence
                flush(q_first, parked);
                parked = 0;
            }
            wsum_tile<NCT, T, VEC, UNR, false, APPLY, false, BLK>(G, N, d, ngroups, base, gam, out, lr);
        }
    }
    if (parked > 0) flush(q_first, parked);
}

// Many workers with few parameters each (N > 8, a gradient of a few thousand columns): too few columns
// to fill the chip with one thread per column group, and that thread would walk its N rows eight at a
// time, N / 8 memory latencies in a row.  Here a workgroup of sixteen wavefronts takes 64 column groups
// and shares out the rows: wavefront w adds rows [w R, (w + 1) R), R = ceil(N / 16) <= 8, all requested at
// once; the sixteen partial sums are added in wavefront order through LDS.  Every element still passes
// through at most N + 1 roundings (R + 16 <= N + 1 for N >= 16; below, the slices without rows add +0.0,
// which is exact).
constexpr int kRowsBlock = 1024, kRowSlices = kRowsBlock / kWave;
static_assert(kRowsBlock == kReduceThreads, "the short variant reduces the partial rows with one share per thread");

// gamma: N weights, in global memory or LDS.  part: kRowSlices x (kWave * VEC) floats of LDS.
// between(): run by the whole workgroup once the loads are requested (the short variant produces the
// weights there, while the loads are in flight).
template <typename T, int VEC, bool APPLY, typename Between>
__device__ __forceinline__ void wsum_rows_tile(const T *__restrict__ G, int N, int64_t d, int64_t ngroups,
                                               const float *gamma, float *__restrict__ out, float lr,
                                               float (*part)[kWave * VEC], Between between) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int R = (N + kRowSlices - 1) / kRowSlices;
    const int i0 = wave * R;
    const int64_t grp = (int64_t)blockIdx.x * kWave + lane;
    const int64_t gc = grp < ngroups ? grp : ngroups - 1;   // clamped: in bounds, the sums are not stored
    float v[kRowsInFlight][VEC];
#pragma unroll
    for (int ii = 0; ii < kRowsInFlight; ++ii)
        if (ii < R && i0 + ii < N) load_vec<T, VEC, true>(G + (int64_t)(i0 + ii) * d + gc * VEC, v[ii]);
    between();
    float acc[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
#pragma unroll
    for (int ii = 0; ii < kRowsInFlight; ++ii)
        if (ii < R && i0 + ii < N) {
            const float w = gamma[i0 + ii];
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = fmaf(w, v[ii][c], acc[c]);
        }
#pragma unroll
    for (int c = 0; c < VEC; c += 4) {
        const f32x4 x = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
        *reinterpret_cast<f32x4 *>(&part[wave][lane * VEC + c]) = x;
    }
    __syncthreads();
    // one output column per thread: consecutive threads read consecutive words of every slice
    if ((int)threadIdx.x < kWave * VEC) {
        const int64_t col = (int64_t)blockIdx.x * (kWave * VEC) + threadIdx.x;
        if (col < ngroups * VEC) {
            float tot = part[0][threadIdx.x];
#pragma unroll
            for (int s = 1; s < kRowSlices; ++s) tot += part[s][threadIdx.x];
            out[col] = APPLY ? fmaf(-lr, tot, out[col]) : tot;
        }
    }
}

template <typename T, int VEC, bool APPLY>
__global__ void __launch_bounds__(kRowsBlock)
wsum_rows_kernel(const T *__restrict__ G, int N, int64_t d, int64_t ngroups, const float *__restrict__ gamma,
                 float *__restrict__ out, float lr) {
    __shared__ __attribute__((aligned(16))) float part[kRowSlices][kWave * VEC];
    wsum_rows_tile<T, VEC, APPLY>(G, N, d, ngroups, gamma, out, lr, part, [] {});
}

// The short path of this regime (see wsum_short_kernel): the aggregation is launch latencies and little
// else, so stage A2 runs here, in every workgroup, on the few partial rows stage A1 left (the launcher caps
// them at 8192 sums), summed as finish_kernel / stats_finish_kernel sum them; workgroup 0 writes K and the
// state.  stats_rows: the rows hold q and r (statistics-only pass); otherwise packed Gram rows (N <= 44).
template <typename T, int VEC, bool APPLY>
__global__ void __launch_bounds__(kRowsBlock)
wsum_rows_short_kernel(const T *__restrict__ G, int N, int64_t d, int64_t ngroups, const double *__restrict__ partials,
                       int nrows, int stats_rows, double *__restrict__ K, DevState *ds, CoeffParams cp,
                       float *__restrict__ out, float lr) {
    __shared__ __attribute__((aligned(16))) float part[kRowSlices][kWave * VEC];
    __shared__ double lds[kReduceThreads];
    __shared__ double K_lds[kFinishMaxN * kFinishMaxN];
    __shared__ float gam_lds[kNMax];
    auto stage_a2 = [&]() __attribute__((always_inline)) {
        const int tid = threadIdx.x;
        const bool writer = blockIdx.x == 0;
        const unsigned parity = ds->parity;            // flipped by stage A1 of this call
        const double m0 = (tid < N) ? ds->m[0][tid] : 0.0, m1 = (tid < N) ? ds->m[1][tid] : 0.0;
        double q = 0.0, r = 0.0;
        if (stats_rows) {
            reduce_stat_rows<kRowsBlock>(partials, nrows, N, lds, q, r);
        } else {
            reduce_partial_rows<kRowsBlock>(partials, nrows, N, writer ? K : nullptr, lds, K_lds);
            if (tid < N) {
                q = K_lds[tid * N + tid];
                for (int j = 0; j < N; ++j) r += K_lds[tid * N + j];   // as update_coefficients adds them
            }
        }
        const unsigned cur = parity & 1u;
        double *m_cur = ds->m[cur];
        const double m_old = cur ? m0 : m1;            // the copy stage A1 retired
        if (writer && tid < N) m_cur[tid] = m_old;     // entries the update leaves alone carry over
        update_coefficients_from_stats(q, r, ds, cp, lds, m_old, m_cur, gam_lds, writer);
        __syncthreads();
    };
    wsum_rows_tile<T, VEC, APPLY>(G, N, d, ngroups, gam_lds, out, lr, part, stage_a2);
}

// Measured, whole step, columns -> row slices: N = 128, d = 1000 fp32 37.8 -> 18.6 us, d = 65536 56.7 -> 35.8 us;
// N = 32, d = 8192 22.0 -> 16.0 us; bf16 N = 128, d = 8192 72.6 -> 21.2 us, N = 64, d = 262144 82.1 -> 35.1 us.
// Even at N = 16 (two batches of rows either way).  The gain ends where the column kernel fills the chip by
// itself: beyond 256 column groups per CU (fp32 d = 262144: 73.1 -> 68.9 us at N = 128; d = 524288: 68.6 ->
// 80.3 us at N = 64, 38.7 -> 45.0 us at N = 32).
// 8 < N <= 16 with at most 1 MiB of gradients (16 bytes a group and row): no faster by itself, but it is the
// second pass the two-launch short path is built on.
bool row_slices_pay(int N, int64_t ngroups, const LaunchShape &shape) {
    if (N <= 8 || shape.wsum_row_slices == 0) return false;
    if (shape.wsum_row_slices == 2) return true;
    if (N <= 16) return (int64_t)N * ngroups * 16 <= ((int64_t)1 << 20);
    return ngroups <= (int64_t)256 * shape.num_cu;
}

template <typename T, int VEC>
static hipError_t run_rows(const void *G, int N, int64_t d, int64_t dcols, const float *gamma, float *out, bool apply,
                           float lr, hipStream_t s) {
    const int64_t ngroups = dcols / VEC;
    const int64_t grid = (ngroups + kWave - 1) / kWave;
    if (grid < 1 || grid > 0x7fffffff) return hipErrorInvalidValue;
    if (apply)
        hipLaunchKernelGGL((wsum_rows_kernel<T, VEC, true>), dim3((unsigned)grid), dim3(kRowsBlock), 0, s,
                           static_cast<const T *>(G), N, d, ngroups, gamma, out, lr);
    else
        hipLaunchKernelGGL((wsum_rows_kernel<T, VEC, false>), dim3((unsigned)grid), dim3(kRowsBlock), 0, s,
                           static_cast<const T *>(G), N, d, ngroups, gamma, out, 0.f);
    return hipGetLastError();
}

template <typename T, int VEC>
static hipError_t run_rows_short(const void *G, int N, int64_t d, const GramWork &work, int nrows, bool stats_rows,
                                 float *out, bool apply, float lr, hipStream_t s) {
    const int64_t ngroups = d / VEC;
    const int64_t grid = (ngroups + kWave - 1) / kWave;
    if (grid < 1 || grid > 0x7fffffff) return hipErrorInvalidValue;
    CoeffParams cp = work.cp;
    cp.N = N;
    if (apply)
        hipLaunchKernelGGL((wsum_rows_short_kernel<T, VEC, true>), dim3((unsigned)grid), dim3(kRowsBlock), 0, s,
                           static_cast<const T *>(G), N, d, ngroups, work.partials, nrows, stats_rows ? 1 : 0, work.K,
                           work.ds, cp, out, lr);
    else
        hipLaunchKernelGGL((wsum_rows_short_kernel<T, VEC, false>), dim3((unsigned)grid), dim3(kRowsBlock), 0, s,
                           static_cast<const T *>(G), N, d, ngroups, work.partials, nrows, stats_rows ? 1 : 0, work.K,
                           work.ds, cp, out, 0.f);
    return hipGetLastError();
}

template <typename Kern>
static int occupancy(Kern k) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k, kBlock, 0) != hipSuccess || nb < 1) nb = 1;
    return nb;
}

// dcols: the columns this launch covers, a multiple of VEC (rows are d elements apart).
template <int NCT, typename T, int VEC, int UNR, bool APPLY>
static hipError_t run_as(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape, const float *gamma,
                         float *out, float lr, hipStream_t s) {
    static const int occ = occupancy(wsum_kernel<NCT, T, VEC, UNR, APPLY>);
    const int64_t ngroups = dcols / VEC;
    const int64_t work = (ngroups + (int64_t)kBlock * UNR - 1) / ((int64_t)kBlock * UNR);
    // Measured: eight workgroups per CU while G is small enough for the memory-side cache to matter
    // (N = 8, 0.8 GB: 138 us against 150 us at one per CU); one per CU for long streams of few rows
    // (N <= 8, 1.6 GB and up: 2-7 % faster); N >= 16 shows no preference beyond noise.
    const bool long_stream = N <= 8 && (int64_t)N * d * (int64_t)sizeof(T) >= (int64_t)5 << 28;   // 1.25 GiB
    // Parked output (wsum_parked_kernel).  Measured, plain -> parked: N = 64, d = 25.6 M 1.16 -> 1.02 ms;
    // N = 32 0.60 -> 0.52 ms; N = 16 0.295 -> 0.263 ms, and 1.51 -> 1.40 ms at d = 124 M; N = 12 0.220 -> 0.207 ms;
    // even (+-4 %) at d = 4 M .. 16.7 M, 3-5 % slower for N <= 9 at d = 25.6 M, 10-25 % slower at d = 1 M; bf16
    // inputs lose (N >= 32: twice the time; but see long_bf16 below).  Streams of 1.25 GiB and more through the run-time-N kernel
    // (N other than 4, 8, 16) gain too: N = 1, 2, 3, 5 4-8 %, N = 9, 10, 11 7-12 %, N = 6, 7 even; the
    // kernels compiled for N = 4 and N = 8 stay 4-6 % ahead of it at any length.  Value 1 leaves the
    // choice to these tables.
    const bool long_generic = NCT == 0 && (int64_t)N * d * (int64_t)sizeof(T) >= (int64_t)5 << 28;
    const bool park_pays = sizeof(T) == 4 && d >= ((int64_t)1 << 24) && (N >= 12 || long_generic);
    // bf16 rows known at compile time (N = 4, 8) in streams of 2.5 GiB and more, where a fifth to a third of the
    // traffic is output: two or three parked tiles (32-48 KB) measured 4-6 % faster (N = 8, d = 335 M: 1.179 ->
    // 1.109-1.119 ms, d = 200 M 0.685 -> 0.651 ms; N = 4, d = 335 M: 0.688 -> 0.657 ms), 64 KB 4 %, 128 KB 2 %;
    // even at 1.6 GB, slower below; N = 2 and N = 16 lose at any length.
    const bool long_bf16 = sizeof(T) == 2 && NCT > 0 && NCT <= 8 && (int64_t)N * d * (int64_t)sizeof(T) >= (int64_t)5 << 29;
    const int park_kb = shape.wsum_park_kb == 1 ? (park_pays ? 128 : (long_bf16 ? 48 : 0)) : shape.wsum_park_kb;
    if (park_kb >= 8) {
        // output tiles parked in LDS: one workgroup of kParkBlock threads per CU (or as many as asked for,
        // sharing the LDS)
        constexpr int kTileBytes = kParkBlock * UNR * VEC * 4;
        constexpr int kMaxParkBytes = 144 * 1024;
        // more than 64 KB of dynamic LDS has to be allowed once per kernel and device (setting it again is harmless)
        static bool allowed[64] = {};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64 || !allowed[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(wsum_parked_kernel<NCT, T, VEC, UNR, APPLY, kParkBlock>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxParkBytes);
            if (e != hipSuccess) return e;
            if (dev >= 0 && dev < 64) allowed[dev] = true;
        }
        const int per_cu_p = shape.blocks_per_cu > 0 ? shape.blocks_per_cu : 1;
        int64_t bytes = (int64_t)park_kb * 1024;
        if (bytes > kMaxParkBytes) bytes = kMaxParkBytes;
        int cap = (int)(bytes / per_cu_p / kTileBytes);
        if (cap < 1) cap = 1;
        const int64_t work_p = (ngroups + (int64_t)kParkBlock * UNR - 1) / ((int64_t)kParkBlock * UNR);
        int64_t grid_p = (int64_t)shape.num_cu * per_cu_p;
        if (grid_p > work_p) grid_p = work_p;
        if (grid_p < 1) grid_p = 1;
        hipLaunchKernelGGL((wsum_parked_kernel<NCT, T, VEC, UNR, APPLY, kParkBlock>), dim3((unsigned)grid_p),
                           dim3(kParkBlock), (size_t)cap * kTileBytes, s, static_cast<const T *>(G), N, d, ngroups, gamma,
                           out, lr, cap);
        return hipGetLastError();
    }
    int per_cu = shape.blocks_per_cu > 0 ? shape.blocks_per_cu : (long_stream ? 1 : 8);
    if (per_cu > occ) per_cu = occ;
    int64_t grid = (int64_t)shape.num_cu * per_cu;
    if (grid > work) grid = work;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL((wsum_kernel<NCT, T, VEC, UNR, APPLY>), dim3((unsigned)grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(G), N, d, ngroups, gamma, out, lr);
    return hipGetLastError();
}

// apply = false: out = sum_i gamma_i g_i.  apply = true: out -= lr * sum_i gamma_i g_i (Eq. 4 fused).
struct WsumMode {
    bool apply;
    float lr;
};

template <int NCT, typename T, int VEC, int UNR>
static hipError_t run(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape, const float *gamma,
                      float *out, const WsumMode &m, hipStream_t s) {
    return m.apply ? run_as<NCT, T, VEC, UNR, true>(G, N, d, dcols, shape, gamma, out, m.lr, s)
                   : run_as<NCT, T, VEC, UNR, false>(G, N, d, dcols, shape, gamma, out, 0.f, s);
}

template <typename T, int VEC, int UNR>
static hipError_t dispatch(const void *G, int N, int64_t d, int64_t dcols, const LaunchShape &shape,
                           const float *gamma, float *out, const WsumMode &m, hipStream_t s) {
    switch (N) {
        case 4: return run<4, T, VEC, UNR>(G, N, d, dcols, shape, gamma, out, m, s);
        case 8: return run<8, T, VEC, UNR>(G, N, d, dcols, shape, gamma, out, m, s);
        case 16: return run<16, T, VEC, 1>(G, N, d, dcols, shape, gamma, out, m, s);  // 16 loads in flight already
        default:
            // rows walked eight at a time: a second tile per thread doubles the staged values, which for bf16 inputs
            // (eight widened columns per load) are 128 registers and leave two wavefronts per SIMD.  Measured at
            // d = 25.6 M, bf16, two tiles -> one: N = 64 0.92 -> 0.60 ms, N = 32 0.46 -> 0.30, N = 12 0.172 -> 0.116,
            // N = 6 0.093 -> 0.068 ms; fp32 inputs keep two (N = 6 0.111 against 0.119 ms with one).
            return run<0, T, VEC, (sizeof(T) == 2) ? 1 : UNR>(G, N, d, dcols, shape, gamma, out, m, s);
    }
}

// ------------------------------------------------------------------------------------------
// Short path: stage A2 inside stage A3
// ------------------------------------------------------------------------------------------
// For gradients of a few megabytes the three launches of an aggregation cost more than the bytes
// (measured at N = 4, d = 2^20: 13 us a step, of which the launch of stage A2 alone is 2-3 us, against
// 6 us for the traffic).  Here stage A3 does stage A2's work itself: every workgroup requests its first
// tile of G, then -- while those loads are in flight -- adds the partial rows stage A1 left (the same
// sums in the same order as finish_kernel, so K is the same bit for bit) and runs the coefficient
// update; all workgroups arrive at the same weights, workgroup 0 alone writes K and the state.  The
// momentum state is read from the copy stage A1 retired (parity flipped there) and written to the
// other one, so no workgroup reads what workgroup 0 writes in this launch.
template <int N, typename T, int VEC, int UNR, bool APPLY>
__global__ void __launch_bounds__(kBlock)
wsum_short_kernel(const T *__restrict__ G, int64_t d, int64_t ngroups, const double *__restrict__ partials, int nrows,
                  double *__restrict__ K, DevState *ds, CoeffParams cp, float *__restrict__ out, float lr) {
    __shared__ double lds[kReduceThreads];
    __shared__ double K_lds[8 * 8];
    __shared__ float gam_lds[8];
    static_assert(N <= 8, "the short path serves N <= 8");
    constexpr int64_t kTile = (int64_t)kBlock * UNR;
    const int64_t ntiles = (ngroups + kTile - 1) / kTile;
    const int grid = (int)gridDim.x, b = (int)blockIdx.x;
    const int slot = (grid % 8) ? b : (b % 8) * (grid / 8) + b / 8;   // XCD-contiguous tiles, as in wsum_kernel

    float v[UNR][N][VEC];
    float wv[UNR][VEC];   // APPLY: the parameters the tile updates, requested with its rows
    bool live[UNR];
    auto load_tile = [&](int64_t t) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t grp = t * kTile + (int64_t)u * kBlock + threadIdx.x;
            live[u] = grp < ngroups;
            const int64_t gc = live[u] ? grp : ngroups - 1;   // clamped: in bounds, the sums are not stored
#pragma unroll
            for (int i = 0; i < N; ++i) load_vec<T, VEC, true>(G + (int64_t)i * d + gc * VEC, v[u][i]);
            if constexpr (APPLY) {
#pragma unroll
                for (int c = 0; c < VEC; c += 4) {
                    const f32x4 w4 = *reinterpret_cast<const gf32x4 *>(out + gc * VEC + c);
                    wv[u][c] = w4.x, wv[u][c + 1] = w4.y, wv[u][c + 2] = w4.z, wv[u][c + 3] = w4.w;
                }
            }
        }
    };
    int64_t t = slot;
    if (t < ntiles) load_tile(t);

    // stage A2 (the loads above are in flight meanwhile)
    const int tid = threadIdx.x;
    const bool writer = blockIdx.x == 0;
    // both copies of the state are requested before the parity word is known, and the partial rows with
    // them: one memory latency for the whole of stage A2's input, not three in a row
    const unsigned parity = ds->parity;            // flipped by stage A1 of this call
    const double m0 = (tid < N) ? ds->m[0][tid] : 0.0, m1 = (tid < N) ? ds->m[1][tid] : 0.0;
    reduce_partial_rows<kBlock>(partials, nrows, N, writer ? K : nullptr, lds, K_lds);
    const unsigned cur = parity & 1u;
    double *m_cur = ds->m[cur];
    const double m_old = cur ? m0 : m1;            // the copy stage A1 retired
    // entries the update leaves alone (momentum off, a non-finite statistic) carry over to the new copy
    if (writer && tid < N) m_cur[tid] = m_old;
    CoeffParams cpn = cp;
    cpn.N = N;
    update_coefficients(K_lds, ds, cpn, lds, m_old, m_cur, gam_lds, writer);
    __syncthreads();
    float w[N];
#pragma unroll
    for (int i = 0; i < N; ++i) w[i] = gam_lds[i];

    while (t < ntiles) {
        float acc[UNR][VEC];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[u][c] = 0.f;
#pragma unroll
            for (int i = 0; i < N; ++i)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[u][c] = fmaf(w[i], v[u][i][c], acc[u][c]);
        }
        if constexpr (APPLY) {   // the step itself, before the next tile's loads reuse wv
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[u][c] = fmaf(-lr, acc[u][c], wv[u][c]);
        }
        const int64_t base = t * kTile + threadIdx.x;
        bool was_live[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) was_live[u] = live[u];
        t += grid;
        if (t < ntiles) load_tile(t);   // the next tile's loads before this tile's stores
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (was_live[u]) {
                if constexpr (APPLY) store_params<VEC>(out, (base + (int64_t)u * kBlock) * VEC, acc[u]);
                else store_out<VEC, false>(out, (base + (int64_t)u * kBlock) * VEC, acc[u], lr, acc[u]);
            }
    }
}

template <int N, typename T, int VEC>
static hipError_t run_short(const void *G, int64_t d, const LaunchShape &shape, const GramWork &work, int nrows,
                            float *out, bool apply, float lr, hipStream_t s) {
    constexpr int UNR = (N * VEC <= 32) ? 2 : 1;   // at most sixteen 128-bit loads in flight per thread
    const int64_t ngroups = d / VEC;
    const int64_t ntiles = (ngroups + (int64_t)kBlock * UNR - 1) / ((int64_t)kBlock * UNR);
    const int per_cu = shape.blocks_per_cu > 0 ? shape.blocks_per_cu : 8;
    int64_t grid = (int64_t)shape.num_cu * per_cu;
    if (grid > ntiles) grid = ntiles;
    if (grid < 1) grid = 1;
    if (apply)
        hipLaunchKernelGGL((wsum_short_kernel<N, T, VEC, UNR, true>), dim3((unsigned)grid), dim3(kBlock), 0, s,
                           static_cast<const T *>(G), d, ngroups, work.partials, nrows, work.K, work.ds, work.cp, out, lr);
    else
        hipLaunchKernelGGL((wsum_short_kernel<N, T, VEC, UNR, false>), dim3((unsigned)grid), dim3(kBlock), 0, s,
                           static_cast<const T *>(G), d, ngroups, work.partials, nrows, work.K, work.ds, work.cp, out, 0.f);
    return hipGetLastError();
}

template <typename T, int VEC>
static hipError_t dispatch_short(const void *G, int N, int64_t d, const LaunchShape &shape, const GramWork &work,
                                 int nrows, float *out, bool apply, float lr, hipStream_t s) {
    switch (N) {
        case 1: return run_short<1, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 2: return run_short<2, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 3: return run_short<3, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 4: return run_short<4, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 5: return run_short<5, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 6: return run_short<6, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 7: return run_short<7, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        case 8: return run_short<8, T, VEC>(G, d, shape, work, nrows, out, apply, lr, s);
        default: return hipErrorInvalidValue;
    }
}

// Rows and output 16-byte aligned, d a multiple of the vector width (the caller checks).
hipError_t launch_wsum_short(const void *G, int N, int64_t d, adacons_dtype dtype, const LaunchShape &shape,
                             const GramWork &work, int nrows, bool stats_rows, float *out, hipStream_t stream,
                             bool apply, float lr) {
    if (N > 8 || stats_rows) {
        if (!stats_rows && N > kFinishMaxN) return hipErrorInvalidValue;
        return (dtype == ADACONS_F32)
                   ? run_rows_short<float, 4>(G, N, d, work, nrows, stats_rows, out, apply, lr, stream)
                   : run_rows_short<bf16_bits, 8>(G, N, d, work, nrows, stats_rows, out, apply, lr, stream);
    }
    return (dtype == ADACONS_F32) ? dispatch_short<float, 4>(G, N, d, shape, work, nrows, out, apply, lr, stream)
                                  : dispatch_short<bf16_bits, 8>(G, N, d, shape, work, nrows, out, apply, lr, stream);
}

// The last d - col0 < 8 columns, which no whole 128-bit group covers: one thread per column.
template <typename T>
__global__ void __launch_bounds__(kWave)
wsum_edge_kernel(const T *__restrict__ G, int N, int64_t d, int64_t col0, const float *__restrict__ gamma,
                 float *__restrict__ out, int apply, float lr) {
    const int64_t col = col0 + threadIdx.x;
    if (col >= d) return;
    float acc = 0.f;
    for (int i = 0; i < N; ++i) {
        float v[1];
        load_vec<T, 1, false>(G + (int64_t)i * d + col, v);
        acc = fmaf(gamma[i], v[0], acc);
    }
    out[col] = apply ? fmaf(-lr, acc, out[col]) : acc;
}

// Without 16-byte aligned rows and output (vec_ok false) the same kernels run from element-aligned
// addresses over the whole 128-bit groups of every row; wsum_edge_kernel takes the columns left over.
hipError_t launch_wsum(const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                       const LaunchShape &shape, const float *gamma, float *out, hipStream_t stream,
                       bool apply, float lr) {
    const WsumMode m = {apply, lr};
    const int64_t vec = (dtype == ADACONS_F32) ? 4 : 8;
    const int64_t dcols = vec_ok ? d : d / vec * vec;
    hipError_t e;
    if (dcols >= vec && row_slices_pay(N, dcols / vec, shape))
        e = (dtype == ADACONS_F32) ? run_rows<float, 4>(G, N, d, dcols, gamma, out, apply, lr, stream)
                                   : run_rows<bf16_bits, 8>(G, N, d, dcols, gamma, out, apply, lr, stream);
    else
        e = (dtype == ADACONS_F32) ? dispatch<float, 4, 2>(G, N, d, dcols, shape, gamma, out, m, stream)
                                   : dispatch<bf16_bits, 8, 2>(G, N, d, dcols, shape, gamma, out, m, stream);
    if (e != hipSuccess || dcols == d) return e;
    if (dtype == ADACONS_F32)
        hipLaunchKernelGGL(wsum_edge_kernel<float>, dim3(1), dim3(kWave), 0, stream, static_cast<const float *>(G), N, d,
                           dcols, gamma, out, apply ? 1 : 0, lr);
    else
        hipLaunchKernelGGL(wsum_edge_kernel<bf16_bits>, dim3(1), dim3(kWave), 0, stream,
                           static_cast<const bf16_bits *>(G), N, d, dcols, gamma, out, apply ? 1 : 0, lr);
    return hipGetLastError();
}

}  // namespace adacons
