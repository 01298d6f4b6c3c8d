// Stage A2 as a device function shared by every kernel that ends in a coefficient update.
#pragma once

#include <hip/hip_runtime.h>

#include "adacons_internal.h"
#include "device_util.h"

namespace adacons {

// Stage A2.  One workgroup (at least max(N, 16) threads, lds of 3 N doubles); thread i < N is worker i.  fp64 throughout.
//   q_i = K_ii, r_i = sum_j K_ij                      (||g_i||^2 and N <g_i, gbar>)
//   a_i = r_i / (N sqrt(q_i))                          Eq. 7, positive for a descent direction
//   rank_i = #{j : a_j < a_i or (a_j = a_i and j < i)} ascending, ties to the lower index
//   m[rank_i] <- beta m[rank_i] + (1 - beta) a_i ; a~_i = m[rank_i]      Eq. 11
//   c_i = a~_i / sqrt(q_i)                             column normalisation, Eq. 8
//   gamma_i = c_i / sum_k c_k                          Eq. 12-13 (weights sum to one)
// Variants: ADACONS_FLAG_INDEX_EMA uses rank_i = i (Eq. 10); ADACONS_FLAG_LAMBDA_EQ13 divides by
// sum_k a~_k instead (lambda as Eq. 13 prints it).
// Degenerate inputs: q_i = 0 gives a_i = c_i = 0; NaN/Inf in q or r, or |sum c| <= 1e-12 sum|c|,
// gives gamma_i = 1/N; the EMA state is not touched when a statistic is non-finite.
// m_old: the state entry m[tid] loaded by the caller ahead of time (thread tid < N), so that the
// global-memory latency of the state overlaps the reduction; it is exchanged through LDS.
// Core: thread tid < N passes its own q = ||g_tid||^2 and r = <g_tid, sum_j g_j>.
// m_new: where the updated state goes (NULL: the current copy, in place).  gam_lds (or NULL): receives the
// weights as fp32, N floats in LDS, for a caller that goes on to apply them.  write = false: compute only,
// leave the state block alone (workgroups that run the update redundantly beside the one that owns it).
__device__ inline void update_coefficients_from_stats(double q, double r, DevState *ds, const CoeffParams cp,
                                                      double *lds, double m_old, double *m_new = nullptr,
                                                      float *gam_lds = nullptr, bool write = true) {
    if (!m_new) m_new = current_m(ds);
    const int N = cp.N;
    const int tid = threadIdx.x;
    double *m_sh = lds + 2 * N;  // [N]
    if (tid < N) m_sh[tid] = m_old;
    double *a_sh = lds;          // [N]
    double *c_sh = lds + N;      // [N]
    __shared__ int s_bad, s_zero;
    __shared__ double s_sum, s_abs;
    if (tid == 0) {
        s_bad = 0;
        s_zero = 0;
    }
    __syncthreads();

    double a = 0.0;
    if (tid < N) {
        if (!isfinite(q) || !isfinite(r)) atomicOr(&s_bad, 1);
    }
    __syncthreads();
    const bool finite = (s_bad == 0);
    if (tid < N) {
        if (q > 0.0) {
            a = r / ((double)N * sqrt(q));
        } else {
            a = 0.0;
            if (finite) atomicOr(&s_zero, 1);
        }
        a_sh[tid] = a;
    }
    __syncthreads();

    unsigned nf = 0;
    if (!finite) {
        nf = ADACONS_NUM_NONFINITE | ADACONS_NUM_UNIFORM_FALLBACK;
        if (tid < N) {
            const double g = 1.0 / (double)N;
            if (gam_lds) gam_lds[tid] = (float)g;
            if (write) {
                ds->gamma[tid] = g;
                ds->gamma32[tid] = (float)g;
                ds->a_raw[tid] = a;
                ds->a_smooth[tid] = a;
            }
        }
    } else {
        if (s_zero) nf |= ADACONS_NUM_ZERO_NORM;
        double as = a;
        if ((cp.flags & ADACONS_FLAG_MOMENTUM) && tid < N) {
            int rank = tid;   // ADACONS_FLAG_INDEX_EMA: state entry i belongs to worker i (Eq. 10)
            if (!(cp.flags & ADACONS_FLAG_INDEX_EMA)) {
                rank = 0;
                for (int j = 0; j < N; ++j) {
                    const double aj = a_sh[j];
                    rank += (aj < a || (aj == a && j < tid)) ? 1 : 0;
                }
            }
            // ranks are a permutation of 0..N-1: every state entry has exactly one writer
            const double mk = cp.beta * m_sh[rank] + (1.0 - cp.beta) * a;
            if (write) m_new[rank] = mk;
            as = mk;
        }
        double c = 0.0;
        if (tid < N) {
            c = (q > 0.0) ? as / sqrt(q) : 0.0;
            // what is made to sum to one: the weights c, or (ADACONS_FLAG_LAMBDA_EQ13) the coefficients a~
            c_sh[tid] = (cp.flags & ADACONS_FLAG_LAMBDA_EQ13) ? as : c;
        }
        __syncthreads();
        // sum c and sum |c| in a fixed order: sixteen interleaved sub-sums (elements t, t + 16, ...), then the
        // sub-sums in order -- for N <= 16 that is the plain index order; a single thread walking 128 entries
        // took about a microsecond of every launch that ends in this update
        __shared__ double s_part[2][16];
        if (tid < 16) {
            double s = 0.0, sabs = 0.0;
            for (int i = tid; i < N; i += 16) {
                s += c_sh[i];
                sabs += fabs(c_sh[i]);
            }
            s_part[0][tid] = s;
            s_part[1][tid] = sabs;
        }
        __syncthreads();
        if (tid == 0) {
            double s = 0.0, sabs = 0.0;
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                s += s_part[0][t];
                sabs += s_part[1][t];
            }
            s_sum = s;
            s_abs = sabs;
        }
        __syncthreads();
        double g = c;
        if (cp.flags & ADACONS_FLAG_NORMALIZE) {
            const double s = s_sum, sabs = s_abs;
            if (!isfinite(s) || sabs == 0.0 || fabs(s) <= 1e-12 * sabs) {
                nf |= ADACONS_NUM_UNIFORM_FALLBACK;
                g = 1.0 / (double)N;
            } else {
                g = c / s;
            }
        }
        if (tid < N) {
            if (gam_lds) gam_lds[tid] = (float)g;
            if (write) {
                ds->gamma[tid] = g;
                ds->gamma32[tid] = (float)g;
                ds->a_raw[tid] = a;
                ds->a_smooth[tid] = as;
            }
        }
    }
    if (tid == 0 && write) {
        ds->numeric_flags = nf;
        ds->step += 1ull;
    }
}

// From the Gram matrix: q_i is its diagonal, r_i its row sum (j ascending).
__device__ inline void update_coefficients(const double *K, DevState *ds, const CoeffParams cp, double *lds,
                                           double m_old, double *m_new = nullptr, float *gam_lds = nullptr,
                                           bool write = true) {
    const int N = cp.N, tid = threadIdx.x;
    double q = 0.0, r = 0.0;
    if (tid < N) {
        q = K[(size_t)tid * N + tid];
        for (int j = 0; j < N; ++j) r += K[(size_t)tid * N + j];
    }
    update_coefficients_from_stats(q, r, ds, cp, lds, m_old, m_new, gam_lds, write);
}

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

// K[i][j] = K[j][i] = sum over rows of partials[.][p]: min(kReduceThreads / np, 32) interleaved sub-sums per
// pair, added in slice order.  One workgroup of any size, N(N+1)/2 <= kReduceThreads: the work is laid out
// for kReduceThreads threads and a smaller workgroup takes several of those shares per thread, so that the
// sums, and with them every bit of K, do not depend on the size of the workgroup that forms them.
// lds >= kReduceThreads doubles.  K (global, or NULL) and K_lds (or NULL) receive the N x N matrix.
// BD: the workgroup's size (a divisor of kReduceThreads).
constexpr int kReduceThreads = 1024;
static_assert(kFinishMaxN * (kFinishMaxN + 1) / 2 <= kReduceThreads, "one workgroup reduces a whole Gram row");
template <int BD>
__device__ inline void reduce_partial_rows(const double *partials, int nrows, int N, double *K, double *lds,
                                           double *K_lds = nullptr) {
    static_assert(kReduceThreads % BD == 0, "whole shares per thread");
    const int np = num_pairs(N);
    // at most 32 slices: the slice sums are added one after the other by a single thread per pair
    const int slices = (kReduceThreads / np < 32) ? kReduceThreads / np : 32;
    // the shares of one thread are independent of each other: unrolled, their loads go out together
    double sub[kReduceThreads / BD];
#pragma unroll
    for (int k = 0; k < kReduceThreads / BD; ++k) {
        const int vt = k * BD + (int)threadIdx.x;
        const int s = vt / np, p = vt - s * np;
        sub[k] = (vt < slices * np) ? sum_rows(partials, np, p, s, slices, nrows) : 0.0;
    }
#pragma unroll
    for (int k = 0; k < kReduceThreads / BD; ++k) {
        const int vt = k * BD + (int)threadIdx.x;
        if (vt < slices * np) lds[vt] = sub[k];   // vt = s * np + p
    }
    __syncthreads();
    for (int p = threadIdx.x; p < np; p += blockDim.x) {
        double tot = 0.0;
        for (int q = 0; q < slices; ++q) tot += lds[q * np + p];
        int i, j;
        unpack_pair(p, N, i, j);
        if (K) {
            K[(size_t)i * N + j] = tot;
            K[(size_t)j * N + i] = tot;
        }
        if (K_lds) {
            K_lds[i * N + j] = tot;
            K_lds[j * N + i] = tot;
        }
    }
    __syncthreads();
}

// The statistics-only pass: rows of [q_0 .. q_{N-1}, r_0 .. r_{N-1}].  Thread tid < N receives the totals
// of worker tid: kReduceThreads / (2 N) interleaved sub-sums per entry, added in slice order.  The same
// virtual layout as above, so the totals do not depend on the size of the workgroup.  lds >= kReduceThreads
// doubles, free again on return.
template <int BD>
__device__ inline void reduce_stat_rows(const double *partials, int nrows, int N, double *lds, double &q, double &r) {
    static_assert(kReduceThreads % BD == 0, "whole shares per thread");
    const int np = 2 * N;
    const int slices = kReduceThreads / np;
    double sub[kReduceThreads / BD];
#pragma unroll
    for (int k = 0; k < kReduceThreads / BD; ++k) {
        const int vt = k * BD + (int)threadIdx.x;
        const int s = vt / np, p = vt - s * np;
        sub[k] = (s < slices) ? sum_rows(partials, np, p, s, slices, nrows) : 0.0;
    }
#pragma unroll
    for (int k = 0; k < kReduceThreads / BD; ++k) {
        const int vt = k * BD + (int)threadIdx.x;
        if (vt < slices * np) lds[vt] = sub[k];   // vt = s * np + p
    }
    __syncthreads();
    q = 0.0;
    r = 0.0;
    if ((int)threadIdx.x < N) {
        for (int k = 0; k < slices; ++k) {
            q += lds[k * np + threadIdx.x];
            r += lds[k * np + N + threadIdx.x];
        }
    }
    __syncthreads();   // the totals are in registers before the caller reuses the buffer
}

}  // namespace adacons
