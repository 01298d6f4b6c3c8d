// One worker's share of Algorithm 1 -- the arithmetic on either side of its collectives:
//   step 1-2  after the all-reduce of the gradients a worker holds its own g and the sum gsum,
//             and needs <g, gsum> and ||g||: pair_stats_kernel streams the two vectors once and
//             accumulates their 2 x 2 Gram matrix (||g||^2, <g, gsum>, ||gsum||^2) in fp64.
//   step 3    with the N pairs gathered, coeff_stats_kernel runs the coefficient update (stage A2).
//   step 4    scale_kernel rescales the local gradient in place, g <- gamma_i g, ready for the
//             final all-reduce.
// The collectives themselves are not part of this library.
#include "adacons_internal.h"
#include "coeff_device.h"
#include "device_util.h"

namespace adacons {

constexpr int kPairUnroll = 4;   // column groups per thread and sweep: 8 loads in flight

template <typename T, int VEC>
__global__ void __launch_bounds__(kBlock)
pair_stats_kernel(const T *__restrict__ x, const T *__restrict__ y, int64_t d, double *__restrict__ partials) {
    __shared__ double lds[4 * 3];
    double acc[3] = {0.0, 0.0, 0.0};   // sum x^2, sum x y, sum y^2
    // whole 128-bit groups (element-aligned addresses are enough); the d mod VEC elements left over
    // are taken one each by the first threads of workgroup 0
    const int64_t ngroups = d / VEC;
    if (blockIdx.x == 0 && ngroups * VEC + threadIdx.x < d) {
        float a[1], b[1];
        load_vec<T, 1, false>(x + ngroups * VEC + threadIdx.x, a);
        load_vec<T, 1, false>(y + ngroups * VEC + threadIdx.x, b);
        const double xa = (double)a[0], yb = (double)b[0];
        acc[0] = xa * xa;
        acc[1] = xa * yb;
        acc[2] = yb * yb;
    }
    const int64_t stride = (int64_t)gridDim.x * kBlock * kPairUnroll;
    for (int64_t g0 = (int64_t)blockIdx.x * kBlock * kPairUnroll + threadIdx.x; g0 < ngroups; g0 += stride) {
        float a[kPairUnroll][VEC], b[kPairUnroll][VEC];
        const bool full = g0 + (int64_t)(kPairUnroll - 1) * kBlock < ngroups;
        if (full) {
#pragma unroll
            for (int u = 0; u < kPairUnroll; ++u) {
                load_vec<T, VEC, true>(x + (g0 + (int64_t)u * kBlock) * VEC, a[u]);
                load_vec<T, VEC, true>(y + (g0 + (int64_t)u * kBlock) * VEC, b[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kPairUnroll; ++u) {
                const int64_t g = g0 + (int64_t)u * kBlock;
                if (g < ngroups) {
                    load_vec<T, VEC, true>(x + g * VEC, a[u]);
                    load_vec<T, VEC, true>(y + g * VEC, b[u]);
                } else {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) a[u][c] = b[u][c] = 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kPairUnroll; ++u)
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const double xa = (double)a[u][c], yb = (double)b[u][c];
                acc[0] = fma(xa, xa, acc[0]);
                acc[1] = fma(xa, yb, acc[1]);
                acc[2] = fma(yb, yb, acc[2]);
            }
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    {
        const double tot = wave_reduce_scatter<3>(acc, lane);
        const int p = wave_scatter_index(lane);
        if (p < 3) lds[wave * 3 + p] = tot;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int p = threadIdx.x;
        partials[(size_t)blockIdx.x * 3 + p] = ((lds[p] + lds[3 + p]) + lds[6 + p]) + lds[9 + p];
    }
}

// stats[0..2] = sum over the partial rows, row order inside 64 interleaved slices, slices in order
__global__ void __launch_bounds__(kBlock) pair_finish_kernel(const double *__restrict__ partials, int nrows,
                                                             double *__restrict__ stats) {
    __shared__ double lds[kBlock];
    const int sl = threadIdx.x / 3, p = threadIdx.x - 3 * sl;
    constexpr int slices = kBlock / 3;
    double acc = 0.0;
    if (sl < slices)
        for (int b = sl; b < nrows; b += slices) acc += partials[(size_t)b * 3 + p];
    lds[threadIdx.x] = (sl < slices) ? acc : 0.0;
    __syncthreads();
    if (threadIdx.x < 3) {
        double tot = 0.0;
        for (int q = 0; q < slices; ++q) tot += lds[q * 3 + threadIdx.x];
        stats[threadIdx.x] = tot;
    }
}

__global__ void __launch_bounds__(kBlock) coeff_stats_kernel(const double *__restrict__ q, const double *__restrict__ r,
                                                             DevState *ds, CoeffParams cp) {
    __shared__ double lds[3 * kNMax];
    const int tid = threadIdx.x;
    const double m_old = (tid < cp.N) ? current_m(ds)[tid] : 0.0;
    update_coefficients_from_stats(tid < cp.N ? q[tid] : 0.0, tid < cp.N ? r[tid] : 0.0, ds, cp, lds, m_old);
}

__device__ __forceinline__ unsigned bf16_round_bits(float f) {   // round to nearest even
    const unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <typename T, int VEC>
__global__ void __launch_bounds__(kBlock) scale_kernel(T *__restrict__ g, int64_t d, const float *__restrict__ gamma) {
    const float w = gamma[0];
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    // whole 128-bit groups from element-aligned addresses; the first threads of workgroup 0 take the
    // d mod VEC elements left over
    const int64_t ngroups = d / VEC;
    if (blockIdx.x == 0 && ngroups * VEC + threadIdx.x < d) {
        T *p = g + ngroups * VEC + threadIdx.x;
        float v[1];
        load_vec<T, 1, false>(p, v);
        if constexpr (sizeof(T) == 4) *p = v[0] * w;
        else *p = (bf16_bits)bf16_round_bits(v[0] * w);
    }
    for (int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x; k < ngroups; k += stride) {
        float v[VEC];
        load_vec<T, VEC, false>(g + k * VEC, v);
#pragma unroll
        for (int c = 0; c < VEC; ++c) v[c] *= w;
        if constexpr (sizeof(T) == 4) {
            const f32x4 x = {v[0], v[1], v[2], v[3]};
            *reinterpret_cast<gf32x4 *>(g + k * VEC) = x;
        } else {
            u32x4 x;
            x.x = bf16_round_bits(v[0]) | (bf16_round_bits(v[1]) << 16);
            x.y = bf16_round_bits(v[2]) | (bf16_round_bits(v[3]) << 16);
            x.z = bf16_round_bits(v[4]) | (bf16_round_bits(v[5]) << 16);
            x.w = bf16_round_bits(v[6]) | (bf16_round_bits(v[7]) << 16);
            *reinterpret_cast<gu32x4 *>(g + k * VEC) = x;
        }
    }
}

template <typename T, int VEC>
static hipError_t run_pair(const void *x, const void *y, int64_t d, int num_cu, int max_rows, double *partials,
                           double *stats, hipStream_t s) {
    const int64_t ngroups = d / VEC;
    int64_t grid = (ngroups + (int64_t)kBlock * kPairUnroll - 1) / ((int64_t)kBlock * kPairUnroll);
    if (grid > (int64_t)num_cu * 4) grid = (int64_t)num_cu * 4;
    if (grid > max_rows) grid = max_rows;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL((pair_stats_kernel<T, VEC>), dim3((unsigned)grid), dim3(kBlock), 0, s,
                       static_cast<const T *>(x), static_cast<const T *>(y), d, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(pair_finish_kernel, dim3(1), dim3(kBlock), 0, s, partials, (int)grid, stats);
    return hipGetLastError();
}

hipError_t launch_pair_stats(const void *x, const void *y, int64_t d, adacons_dtype dtype, int num_cu,
                             int max_rows, double *partials, double *stats, hipStream_t s) {
    if (dtype == ADACONS_F32) return run_pair<float, 4>(x, y, d, num_cu, max_rows, partials, stats, s);
    return run_pair<bf16_bits, 8>(x, y, d, num_cu, max_rows, partials, stats, s);
}

hipError_t launch_coeffs_from_stats(const double *q, const double *r, DevState *ds, const CoeffParams &cp,
                                    hipStream_t s) {
    hipLaunchKernelGGL(coeff_stats_kernel, dim3(1), dim3(kBlock), 0, s, q, r, ds, cp);
    return hipGetLastError();
}

template <typename T, int VEC>
static hipError_t run_scale(void *g, int64_t d, int num_cu, const float *gamma, hipStream_t s) {
    int64_t grid = (d / VEC + kBlock - 1) / kBlock;
    if (grid > (int64_t)num_cu * 8) grid = (int64_t)num_cu * 8;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL((scale_kernel<T, VEC>), dim3((unsigned)grid), dim3(kBlock), 0, s, static_cast<T *>(g), d,
                       gamma);
    return hipGetLastError();
}

hipError_t launch_scale(void *g, int64_t d, adacons_dtype dtype, int num_cu, const float *gamma, hipStream_t s) {
    if (dtype == ADACONS_F32) return run_scale<float, 4>(g, d, num_cu, gamma, s);
    return run_scale<bf16_bits, 8>(g, d, num_cu, gamma, s);
}

}  // namespace adacons
