// Device-side helpers: 128-bit loads of fp32 / bf16 gradient elements, wavefront sums.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adacons {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// 128 bits of global memory that are only aligned to the element (fp32: 4 bytes, bf16: 2 bytes).
// The device runs with unaligned access enabled, so these still compile to one 128-bit load or
// store; rows of G that do not start on a 16-byte boundary cost extra cache-line visits, not a fault.
typedef float gf32x4 __attribute__((ext_vector_type(4), aligned(4)));
typedef unsigned gu32x4 __attribute__((ext_vector_type(4), aligned(2)));

typedef uint16_t bf16_bits;  // a bfloat16 as stored: the upper half of an IEEE binary32

__device__ __forceinline__ float bf16_widen(unsigned bits16) { return __uint_as_float(bits16 << 16); }

// Elements per 128-bit load.
template <typename T> struct VecWidth;
template <> struct VecWidth<float> { static constexpr int value = 4; };
template <> struct VecWidth<bf16_bits> { static constexpr int value = 8; };

// Load VEC consecutive elements at p (p aligned to VEC*sizeof(T)) and widen them to fp32.
// NT selects a non-temporal load (data not needed in cache again).
template <typename T, int VEC, bool NT = false>
__device__ __forceinline__ void load_vec(const T *__restrict__ p, float (&v)[VEC]);

template <>
__device__ __forceinline__ void load_vec<float, 4, false>(const float *__restrict__ p, float (&v)[4]) {
    const f32x4 x = *reinterpret_cast<const gf32x4 *>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
}
template <>
__device__ __forceinline__ void load_vec<float, 4, true>(const float *__restrict__ p, float (&v)[4]) {
    const f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const gf32x4 *>(p));
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
}
template <>
__device__ __forceinline__ void load_vec<float, 1, false>(const float *__restrict__ p, float (&v)[1]) { v[0] = p[0]; }
template <>
__device__ __forceinline__ void load_vec<float, 1, true>(const float *__restrict__ p, float (&v)[1]) {
    v[0] = __builtin_nontemporal_load(p);
}

__device__ __forceinline__ void unpack_bf16x8(const u32x4 x, float (&v)[8]) {
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xffff0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xffff0000u);
}
template <>
__device__ __forceinline__ void load_vec<bf16_bits, 8, false>(const bf16_bits *__restrict__ p, float (&v)[8]) {
    unpack_bf16x8(*reinterpret_cast<const gu32x4 *>(p), v);
}
template <>
__device__ __forceinline__ void load_vec<bf16_bits, 8, true>(const bf16_bits *__restrict__ p, float (&v)[8]) {
    unpack_bf16x8(__builtin_nontemporal_load(reinterpret_cast<const gu32x4 *>(p)), v);
}
template <>
__device__ __forceinline__ void load_vec<bf16_bits, 1, false>(const bf16_bits *__restrict__ p, float (&v)[1]) {
    v[0] = bf16_widen(p[0]);
}
template <>
__device__ __forceinline__ void load_vec<bf16_bits, 1, true>(const bf16_bits *__restrict__ p, float (&v)[1]) {
    v[0] = bf16_widen(__builtin_nontemporal_load(p));
}

// The 16 bytes of one 128-bit load as VecWidth<T> fp32 values (fp32: reinterpreted, bf16: widened).
template <typename T> __device__ __forceinline__ void widen_bits(const u32x4 x, float (&v)[VecWidth<T>::value]);
template <> __device__ __forceinline__ void widen_bits<float>(const u32x4 x, float (&v)[4]) {
    v[0] = __uint_as_float(x.x); v[1] = __uint_as_float(x.y); v[2] = __uint_as_float(x.z); v[3] = __uint_as_float(x.w);
}
template <> __device__ __forceinline__ void widen_bits<bf16_bits>(const u32x4 x, float (&v)[8]) { unpack_bf16x8(x, v); }

// Sum over the 64 lanes of a wavefront in a fixed butterfly order; every lane gets the total.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sums NP per-lane values over the 64 lanes of a wavefront by recursive halving: in the step with
// lane distance 32, 16, ..., 1 a lane keeps the values whose index has the same parity as its
// lane bit and sends the others to its partner, so the number of values halves each step
// (NP/2 + NP/4 + ... exchanges instead of 6 NP).  Afterwards lane l holds the total of value
// index bitrev6(l) -- wave_scatter_index(l) -- when that is < NP, and 0 otherwise.  The order of
// the additions is fixed, so results are reproducible.
__device__ __forceinline__ int wave_scatter_index(int lane) {
    return ((lane >> 5) & 1) | (((lane >> 4) & 1) << 1) | (((lane >> 3) & 1) << 2) | (((lane >> 2) & 1) << 3) |
           (((lane >> 1) & 1) << 4) | ((lane & 1) << 5);
}

template <int M, int DIST>
__device__ __forceinline__ double wave_reduce_scatter_step(const double (&in)[M], int lane) {
    constexpr int H = (M + 1) / 2;
    const bool odd = (lane & DIST) != 0;
    double out[H];
#pragma unroll
    for (int k = 0; k < H; ++k) {
        const double lo = in[2 * k];
        const double hi = (2 * k + 1 < M) ? in[2 * k + 1] : 0.0;
        const double keep = odd ? hi : lo;
        const double send = odd ? lo : hi;
        out[k] = keep + __shfl_xor(send, DIST, 64);
    }
    if constexpr (DIST == 1) {
        static_assert(H == 1, "at most 64 values per wavefront");
        return out[0];
    } else {
        return wave_reduce_scatter_step<H, DIST / 2>(out, lane);
    }
}

template <int NP>
__device__ __forceinline__ double wave_reduce_scatter(const double (&v)[NP], int lane) {
    static_assert(NP <= 64, "one value per lane at the end");
    return wave_reduce_scatter_step<NP, 32>(v, lane);
}

// sum over rows b = first, first + step, ... (< nrows) of partials[b][p], b ascending; the loads
// of up to sixteen rows are issued together (rows past the end read as +0.0, which leaves a sum
// unchanged), the additions keep the row order
__device__ __forceinline__ double sum_rows(const double *partials, int np, int p, int first, int step, int nrows) {
    double acc = 0.0;
    for (int b = first; b < nrows; b += 16 * step) {
        double t[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int row = b + k * step;
            t[k] = (row < nrows) ? partials[(size_t)row * np + p] : 0.0;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) acc += t[k];
    }
    return acc;
}

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b % 8) and every XCD
// has its own L2.  Rows of G are in general not aligned to a 128-byte line relative to each
// other, so the line at the boundary of two neighbouring column segments is needed by two
// workgroups; giving each XCD a contiguous run of segments makes those two share an L2.
// Returns the segment (0 .. grid-1) workgroup b takes inside one sweep of the grid.
__device__ __forceinline__ int xcd_contiguous_slot(int b, int grid) {
    constexpr int kXcds = 8;
    if (grid % kXcds) return b;
    return (b % kXcds) * (grid / kXcds) + b / kXcds;
}

}  // namespace adacons
