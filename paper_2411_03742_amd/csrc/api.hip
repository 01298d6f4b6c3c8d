// C ABI of libadacons (declared in include/adacons.h): argument checks, state ownership,
// stream-ordered launches of the three stages.  No kernel code here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "adacons_internal.h"

using namespace adacons;

// ---- what adacons_aggregate_noalloc() works in --------------------------------------------------
// Everything adacons_init_state() would allocate for one call -- the device state block, K and the
// partial-sum workspace of stage A1 -- laid out in one file-scope device array.  Every GPU the
// library runs on holds its own copy at its own address until the process ends; in host code the
// array's name is only a handle for hipGetSymbolAddress(), never an address to pass on.
constexpr size_t kScratchBytes = (size_t)20 << 20;   // 20 MiB per GPU: room for the 1024 partial rows of the N = 64 Gram pass
constexpr size_t kScratchStateOff = 0;
constexpr size_t kScratchKOff = (sizeof(DevState) + 255) / 256 * 256;
constexpr size_t kScratchKBytes = ((size_t)ADACONS_N_MAX * ADACONS_N_MAX + 2 * (size_t)ADACONS_N_MAX) * sizeof(double);
constexpr size_t kScratchPartialsOff = (kScratchKOff + kScratchKBytes + 255) / 256 * 256;
constexpr size_t kScratchPartialsBytes = kScratchBytes - kScratchPartialsOff;
static_assert(kScratchPartialsOff < kScratchBytes, "scratch too small");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct adacons_state {
    int N;
    int64_t d_max;
    double beta;
    unsigned flags;
    int device;
    int num_cu;
    DevState *ds;      // device
    double *partials;  // device, [max_rows][N(N+1)/2]
    double *K;         // device, [N][N]
    int max_rows;
    bool k_valid;      // K holds the Gram matrix of the last call (false after a statistics-only A1)
    int tune[ADACONS_TUNE_COUNT_];
    // per-kernel timing (adacons_profile_begin/end)
    std::vector<hipEvent_t> events;  // 4 per call: before A1, after the Gram kernel, after A2, after A3
    std::vector<unsigned char> prof_short;  // per recorded call: it took the short path (no launch of its own for A2)
    int prof_capacity;
    int prof_calls;
};

namespace {

thread_local char g_err[512] = "";

adacons_status fail(adacons_status s, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

adacons_status hip_fail(hipError_t e, const char *what) {
    return fail(ADACONS_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(call)                                    \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) return hip_fail(e_, #call); \
    } while (0)

const int kTuneDefault[ADACONS_TUNE_COUNT_] = {0 /* kernel's own default */, 0 /* same */, 320, 2, 0, 1, 1, 1};

size_t elem_size(adacons_dtype t) { return t == ADACONS_BF16 ? 2 : 4; }

// Doubles in one partial row of stage A1: N (N + 1) / 2 sums of products, or q and r per worker (2 N)
// where K is not formed; at least the 3 sums of the one-worker statistics.
size_t partial_row_doubles(int N) {
    return N > ADACONS_GRAM_N_MAX ? 2 * (size_t)N : (size_t)(num_pairs(N) < 3 ? 3 : num_pairs(N));
}

// Checks shared by the three compute entry points.  out may be NULL (stage A1 alone).
adacons_status check_call(const void *G, int N, int64_t d, adacons_dtype dtype, const adacons_state *st,
                          const float *out, bool need_out, bool *vec_ok) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    if (!G) return fail(ADACONS_EINVAL, "G is NULL");
    if (need_out && !out) return fail(ADACONS_EINVAL, "out is NULL");
    if (dtype != ADACONS_F32 && dtype != ADACONS_BF16) return fail(ADACONS_EUNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (N != st->N) return fail(ADACONS_EINVAL, "N=%d does not match the state's N=%d", N, st->N);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != st->device)
        return fail(ADACONS_EINVAL, "the state lives on device %d, the current device is %d", st->device, dev);
    if (d < 1 || d > st->d_max)
        return fail(ADACONS_EINVAL, "d=%lld outside [1, d_max=%lld]", (long long)d, (long long)st->d_max);
    const size_t es = elem_size(dtype);
    const uintptr_t g0 = reinterpret_cast<uintptr_t>(G);
    if (g0 % es) return fail(ADACONS_EALIGN, "G not aligned to its element size");
    bool ok = (g0 % 16 == 0) && ((uint64_t)d * es % 16 == 0);
    if (need_out) {
        const uintptr_t o0 = reinterpret_cast<uintptr_t>(out);
        if (o0 % 4) return fail(ADACONS_EALIGN, "out not 4-byte aligned");
        const uintptr_t g1 = g0 + (uint64_t)N * (uint64_t)d * es, o1 = o0 + (uint64_t)d * 4;
        if (o0 < g1 && g0 < o1) return fail(ADACONS_EINVAL, "out overlaps G");
        ok = ok && (o0 % 16 == 0);
    }
    *vec_ok = ok;
    return ADACONS_OK;
}

LaunchShape shape_of(const adacons_state *st, adacons_tune_key key) {
    LaunchShape s;
    s.num_cu = st->num_cu;
    s.blocks_per_cu = st->tune[key];
    s.max_rows = st->max_rows;
    const int head = st->tune[ADACONS_TUNE_CACHED_HEAD_MB];
    s.cached_head_mb = head >= (1 << 20) ? -1 : head;  // a huge value means all of G
    s.gram_products = st->tune[ADACONS_TUNE_GRAM_PRODUCTS];
    s.wsum_park_kb = st->tune[ADACONS_TUNE_WSUM_PARK_KB];
    s.wsum_row_slices = st->tune[ADACONS_TUNE_WSUM_ROW_SLICES];
    s.short_path = false;
    return s;
}

GramWork work_of(adacons_state *st) {
    GramWork t;
    t.partials = st->partials;
    t.K = st->K;
    t.ds = st->ds;
    t.cp.N = st->N;
    t.cp.beta = st->beta;
    t.cp.flags = st->flags;
    return t;
}

bool uses_stats_pass(const adacons_state *st, int N) {
    return (st->tune[ADACONS_TUNE_STATS_ONLY] != 0 && N > 8) || N > ADACONS_GRAM_N_MAX;
}

// Many workers with few parameters each (N > 8, at most 1 MiB of gradients, second pass by row slices): a
// step is launch latencies and little else, and takes the short path below, where every workgroup of stage
// A3 adds the partial rows itself.  Stage A1 then writes at most 8192 sums (16 rows at N = 32, 32 rows of
// statistics at N = 128; such gradients give it that many workgroups at most anyway) -- on the long path too,
// so that both form the coefficients from the same rows.
constexpr int64_t kShortPathBytes = (int64_t)32 << 20;      // N <= 8
constexpr int64_t kShortPathBytesWide = (int64_t)1 << 20;   // N > 8
constexpr int kShortPathSums = 8192;
bool many_workers_short_gradients(const adacons_state *st, int N, int64_t d, adacons_dtype dtype) {
    if (N <= 8 || (int64_t)N * d * (int64_t)elem_size(dtype) > kShortPathBytesWide) return false;
    if (!uses_stats_pass(st, N) && N > kFinishMaxN) return false;   // K takes more than one workgroup to reduce
    const int64_t vec = 16 / (int64_t)elem_size(dtype);
    return row_slices_pay(N, d / vec, shape_of(st, ADACONS_TUNE_WSUM_BLOCKS_PER_CU));
}
LaunchShape first_pass_shape(const adacons_state *st, int N, int64_t d, adacons_dtype dtype) {
    LaunchShape shape = shape_of(st, ADACONS_TUNE_GRAM_BLOCKS_PER_CU);
    if (many_workers_short_gradients(st, N, d, dtype)) {
        const int row = uses_stats_pass(st, N) ? 2 * N : num_pairs(N);
        const int cap = kShortPathSums / row;   // >= 8 (N <= 44 Gram: 990 sums; N <= 128 statistics: 256)
        if (shape.max_rows > cap) shape.max_rows = cap;
    }
    return shape;
}

// Stages A1 + A2 of an aggregation: the Gram kernels, or the statistics-only pass when selected.
hipError_t launch_first_pass(adacons_state *st, const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                             hipStream_t s, hipEvent_t between) {
    const LaunchShape shape = first_pass_shape(st, N, d, dtype);
    if (uses_stats_pass(st, N)) {
        st->k_valid = false;
        return launch_stats(G, N, d, dtype, vec_ok, shape, st->partials, st->ds, work_of(st).cp, s, between);
    }
    st->k_valid = true;
    return launch_gram(G, N, d, dtype, vec_ok, shape, work_of(st), true, s, between);
}

// Gradients small enough to sit in the caches between the two passes take the short path: two launches,
// stage A2 inside stage A3 (see wsum_short_kernel and, for N > 8, wsum_rows_short_kernel).
bool takes_short_path(const adacons_state *st, int N, int64_t d, adacons_dtype dtype, bool vec_ok) {
    const int mode = st->tune[ADACONS_TUNE_SHORT_PATH];
    if (mode == 0 || !vec_ok) return false;
    if (N <= 8) {
        // Measured crossovers (two launches against three, whole step): fp32 wins up to 32 MiB for every N <= 8
        // (N = 8: -7 % at 32 MiB, +7 % at 64; N = 2 still -8 % at 128 MiB); bf16 rows hold twice the columns per
        // byte and stage A3 keeps them widened in registers, so its limit is lower: N <= 2 32 MiB (-5 %, +9 % at
        // 64), N <= 6 16 MiB (N = 4: -14 % at 16, +6 % at 32), N = 7, 8 8 MiB (N = 8: -6 % at 8, +10 % at 16,
        // +31 % at 32).
        int64_t limit = kShortPathBytes;
        if (dtype == ADACONS_BF16 && N > 2) limit = (N <= 6) ? kShortPathBytes / 2 : kShortPathBytes / 4;
        return mode == 2 || (int64_t)N * d * (int64_t)elem_size(dtype) <= limit;
    }
    return many_workers_short_gradients(st, N, d, dtype);
}

// All three stages of one aggregation on stream s: out = sum, or (apply) out -= lr * sum.
// ev (or NULL): four events, recorded before A1, after the Gram kernel, after A2, after A3.
hipError_t enqueue_aggregate(adacons_state *st, const void *G, int N, int64_t d, adacons_dtype dtype, bool vec_ok,
                             float *out, bool apply, float lr, hipStream_t s, hipEvent_t *ev, bool *took_short = nullptr) {
    hipError_t e = hipSuccess;
    if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return e;
    const bool short_path = takes_short_path(st, N, d, dtype, vec_ok);
    if (took_short) *took_short = short_path;
    if (short_path) {
        LaunchShape shape = first_pass_shape(st, N, d, dtype);
        shape.short_path = true;
        int rows = 0;
        const bool stats_rows = uses_stats_pass(st, N);
        st->k_valid = !stats_rows;
        e = stats_rows ? launch_stats(G, N, d, dtype, vec_ok, shape, st->partials, st->ds, work_of(st).cp, s,
                                      ev ? ev[1] : nullptr, &rows)
                       : launch_gram(G, N, d, dtype, vec_ok, shape, work_of(st), true, s, ev ? ev[1] : nullptr, &rows);
        if (e != hipSuccess) return e;
        e = launch_wsum_short(G, N, d, dtype, shape_of(st, ADACONS_TUNE_WSUM_BLOCKS_PER_CU), work_of(st), rows, stats_rows,
                              out, s, apply, lr);
    } else {
        if ((e = launch_first_pass(st, G, N, d, dtype, vec_ok, s, ev ? ev[1] : nullptr)) != hipSuccess) return e;
        if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
        e = launch_wsum(G, N, d, dtype, vec_ok, shape_of(st, ADACONS_TUNE_WSUM_BLOCKS_PER_CU), st->ds->gamma32, out, s, apply, lr);
    }
    if (e == hipSuccess && ev) e = hipEventRecord(ev[3], s);
    return e;
}

// Per device: the address of that device's copy of `scratch`, resolved once with the device current.
struct DeviceScratch {
    void *ptr;
    int num_cu;
    bool resolved;
};
constexpr int kMaxDevices = 64;
DeviceScratch g_scratch[kMaxDevices] = {};
std::mutex g_scratch_mu;

adacons_status scratch_of(int dev, DeviceScratch *out) {
    if (dev < 0 || dev >= kMaxDevices) return fail(ADACONS_EUNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    DeviceScratch &e = g_scratch[dev];
    if (!e.resolved) {
        hipDeviceProp_t prop;
        HIP_TRY(hipGetDeviceProperties(&prop, dev));
        if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return fail(ADACONS_EUNSUPPORTED, "built for gfx950 only, device is %s", prop.gcnArchName);
        void *p = nullptr;
        hipError_t rc = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy
        if (rc != hipSuccess) return hip_fail(rc, "hipGetSymbolAddress(scratch)");
        if (!p) return fail(ADACONS_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        e.ptr = p;
        e.num_cu = prop.multiProcessorCount;
        e.resolved = true;
    }
    *out = e;
    return ADACONS_OK;
}

}  // namespace

adacons_status adacons::set_error(adacons_status s, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

extern "C" {

const char *adacons_status_string(adacons_status s) {
    switch (s) {
        case ADACONS_OK: return "ok";
        case ADACONS_EINVAL: return "invalid argument";
        case ADACONS_EUNSUPPORTED: return "unsupported";
        case ADACONS_EALIGN: return "misaligned pointer";
        case ADACONS_EHIP: return "HIP runtime error";
        case ADACONS_ENOMEM: return "out of memory";
    }
    return "unknown status";
}

const char *adacons_last_error(void) { return g_err; }

adacons_status adacons_init_state(adacons_state **out_st, int N, int64_t d_max, double beta, unsigned flags,
                                  void *hip_stream) {
    if (!out_st) return fail(ADACONS_EINVAL, "st is NULL");
    *out_st = nullptr;
    if (N < 1) return fail(ADACONS_EINVAL, "N=%d < 1", N);
    if (N > ADACONS_N_MAX) return fail(ADACONS_EUNSUPPORTED, "N=%d > ADACONS_N_MAX=%d", N, ADACONS_N_MAX);
    if (d_max < 1) return fail(ADACONS_EINVAL, "d_max < 1");
    if (!(beta >= 0.0 && beta < 1.0)) return fail(ADACONS_EINVAL, "beta=%g outside [0, 1)", beta);
    if (flags & ~ADACONS_FLAG_ALL_) return fail(ADACONS_EINVAL, "unknown flag bits 0x%x", flags);

    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(ADACONS_EUNSUPPORTED, "built for gfx950 only, device is %s", prop.gcnArchName);

    adacons_state *st = new (std::nothrow) adacons_state();
    if (!st) return fail(ADACONS_ENOMEM, "host allocation failed");
    st->N = N;
    st->d_max = d_max;
    st->beta = beta;
    st->flags = flags;
    st->device = dev;
    st->num_cu = prop.multiProcessorCount;
    st->ds = nullptr;
    st->partials = nullptr;
    st->K = nullptr;
    st->max_rows = gram_rows_needed(N, st->num_cu);
    for (int k = 0; k < ADACONS_TUNE_COUNT_; ++k) st->tune[k] = kTuneDefault[k];
    st->prof_capacity = 0;
    st->k_valid = N <= ADACONS_GRAM_N_MAX;   // zeroed at creation; never produced for larger N
    st->prof_calls = 0;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&st->ds), sizeof(DevState));
    const size_t row_doubles = partial_row_doubles(N);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&st->partials), (size_t)st->max_rows * row_doubles * sizeof(double));
    // K, then q and r of adacons_update_from_stats (2 N doubles), then the caller's weights of
    // adacons_weighted_sum as fp32 (N floats)
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&st->K), ((size_t)N * N + 3 * (size_t)N) * sizeof(double));
    if (e == hipSuccess) e = launch_clear_state(st->ds, st->K, N * N, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        adacons_status rc = (e == hipErrorOutOfMemory) ? fail(ADACONS_ENOMEM, "device allocation failed")
                                                       : hip_fail(e, "adacons_init_state");
        adacons_destroy_state(st);
        return rc;
    }
    *out_st = st;
    return ADACONS_OK;
}

adacons_status adacons_destroy_state(adacons_state *st) {
    if (!st) return ADACONS_OK;
    for (hipEvent_t ev : st->events) (void)hipEventDestroy(ev);
    if (st->ds) (void)hipFree(st->ds);
    if (st->partials) (void)hipFree(st->partials);
    if (st->K) (void)hipFree(st->K);
    delete st;
    return ADACONS_OK;
}

adacons_status adacons_reset_state(adacons_state *st, void *hip_stream) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    HIP_TRY(launch_clear_state(st->ds, nullptr, 0, static_cast<hipStream_t>(hip_stream)));
    return ADACONS_OK;
}

adacons_status adacons_aggregate(const void *G, int N, int64_t d, adacons_dtype dtype, adacons_state *st,
                                 float *out, void *hip_stream) {
    bool vec_ok = false;
    adacons_status rc = check_call(G, N, d, dtype, st, out, true, &vec_ok);
    if (rc != ADACONS_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool prof = st->prof_capacity > 0 && st->prof_calls < st->prof_capacity;
    hipEvent_t *ev = prof ? &st->events[(size_t)st->prof_calls * 4] : nullptr;

    bool took_short = false;
    HIP_TRY(enqueue_aggregate(st, G, N, d, dtype, vec_ok, out, false, 0.f, s, ev, &took_short));
    if (prof) {
        st->prof_short[(size_t)st->prof_calls] = took_short ? 1 : 0;
        st->prof_calls += 1;
    }
    return ADACONS_OK;
}

adacons_status adacons_aggregate_apply(const void *G, int N, int64_t d, adacons_dtype dtype, adacons_state *st,
                                       float *w, float lr, void *hip_stream) {
    bool vec_ok = false;
    adacons_status rc = check_call(G, N, d, dtype, st, w, true, &vec_ok);
    if (rc != ADACONS_OK) return rc;
    if (!std::isfinite(lr)) return fail(ADACONS_EINVAL, "lr is not finite");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(enqueue_aggregate(st, G, N, d, dtype, vec_ok, w, true, lr, s, nullptr));
    return ADACONS_OK;
}

adacons_status adacons_worker_stats(const void *g, const void *gsum, int64_t d, adacons_dtype dtype,
                                    adacons_state *st, double *stats_dev, void *hip_stream) {
    if (!st || !g || !gsum || !stats_dev) return fail(ADACONS_EINVAL, "NULL argument");
    if (dtype != ADACONS_F32 && dtype != ADACONS_BF16) return fail(ADACONS_EUNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (d < 1 || d > st->d_max) return fail(ADACONS_EINVAL, "d outside [1, d_max]");
    const size_t es = elem_size(dtype);
    const uintptr_t a = reinterpret_cast<uintptr_t>(g), b = reinterpret_cast<uintptr_t>(gsum);
    if (a % es || b % es || reinterpret_cast<uintptr_t>(stats_dev) % 8) return fail(ADACONS_EALIGN, "misaligned pointer");
    HIP_TRY(launch_pair_stats(g, gsum, d, dtype, st->num_cu, st->max_rows, st->partials, stats_dev,
                              static_cast<hipStream_t>(hip_stream)));
    return ADACONS_OK;
}

adacons_status adacons_update_from_stats(adacons_state *st, const double *sq_host, const double *dot_host,
                                         void *hip_stream) {
    if (!st || !sq_host || !dot_host) return fail(ADACONS_EINVAL, "NULL argument");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    double *q = st->K + (size_t)st->N * st->N, *r = q + st->N;
    HIP_TRY(hipMemcpyAsync(q, sq_host, (size_t)st->N * sizeof(double), hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(r, dot_host, (size_t)st->N * sizeof(double), hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));   // the host arrays are the caller's
    CoeffParams cp;
    cp.N = st->N; cp.beta = st->beta; cp.flags = st->flags;
    HIP_TRY(launch_coeffs_from_stats(q, r, st->ds, cp, s));
    return ADACONS_OK;
}

adacons_status adacons_worker_scale(void *g, int64_t d, adacons_dtype dtype, const adacons_state *st, int worker,
                                    void *hip_stream) {
    if (!st || !g) return fail(ADACONS_EINVAL, "NULL argument");
    if (dtype != ADACONS_F32 && dtype != ADACONS_BF16) return fail(ADACONS_EUNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (worker < 0 || worker >= st->N) return fail(ADACONS_EINVAL, "worker %d outside [0, N)", worker);
    if (d < 1) return fail(ADACONS_EINVAL, "d < 1");
    const size_t es = elem_size(dtype);
    const uintptr_t a = reinterpret_cast<uintptr_t>(g);
    if (a % es) return fail(ADACONS_EALIGN, "g not aligned to its element size");
    HIP_TRY(launch_scale(g, d, dtype, st->num_cu, st->ds->gamma32 + worker, static_cast<hipStream_t>(hip_stream)));
    return ADACONS_OK;
}

adacons_status adacons_coeffs(const adacons_state *st, double *gamma_host, double *raw_host, double *smoothed_host,
                              uint32_t *numeric_flags, void *hip_stream) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    if (!gamma_host) return fail(ADACONS_EINVAL, "gamma_host is NULL");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const size_t nb = (size_t)st->N * sizeof(double);
    HIP_TRY(hipMemcpyAsync(gamma_host, st->ds->gamma, nb, hipMemcpyDeviceToHost, s));
    if (raw_host) HIP_TRY(hipMemcpyAsync(raw_host, st->ds->a_raw, nb, hipMemcpyDeviceToHost, s));
    if (smoothed_host) HIP_TRY(hipMemcpyAsync(smoothed_host, st->ds->a_smooth, nb, hipMemcpyDeviceToHost, s));
    unsigned nf = 0;
    if (numeric_flags) HIP_TRY(hipMemcpyAsync(&nf, &st->ds->numeric_flags, sizeof nf, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (numeric_flags) *numeric_flags = nf;
    return ADACONS_OK;
}

adacons_status adacons_gram(const void *G, int N, int64_t d, adacons_dtype dtype, adacons_state *st,
                            void *hip_stream) {
    bool vec_ok = false;
    adacons_status rc = check_call(G, N, d, dtype, st, nullptr, false, &vec_ok);
    if (rc != ADACONS_OK) return rc;
    if (N > ADACONS_GRAM_N_MAX)
        return fail(ADACONS_EUNSUPPORTED, "K is formed for N <= %d only (N=%d)", ADACONS_GRAM_N_MAX, N);
    st->k_valid = true;
    HIP_TRY(launch_gram(G, N, d, dtype, vec_ok, shape_of(st, ADACONS_TUNE_GRAM_BLOCKS_PER_CU), work_of(st), false,
                        static_cast<hipStream_t>(hip_stream)));
    return ADACONS_OK;
}

adacons_status adacons_read_gram(const adacons_state *st, double *K_host, void *hip_stream) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    if (!K_host) return fail(ADACONS_EINVAL, "K_host is NULL");
    if (!st->k_valid) return fail(ADACONS_EINVAL, "the last call computed the statistics only (ADACONS_TUNE_STATS_ONLY or N > ADACONS_GRAM_N_MAX): no K");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(hipMemcpyAsync(K_host, st->K, (size_t)st->N * st->N * sizeof(double), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return ADACONS_OK;
}

adacons_status adacons_weighted_sum(const void *G, int N, int64_t d, adacons_dtype dtype, const double *gamma_host,
                                    adacons_state *st, float *out, void *hip_stream) {
    bool vec_ok = false;
    adacons_status rc = check_call(G, N, d, dtype, st, out, true, &vec_ok);
    if (rc != ADACONS_OK) return rc;
    if (!gamma_host) return fail(ADACONS_EINVAL, "gamma_host is NULL");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    float g32[kNMax];
    for (int i = 0; i < N; ++i) g32[i] = (float)gamma_host[i];
    // the caller's weights get a buffer of their own: what adacons_coeffs() reports stays the last aggregation's
    float *user_gamma = reinterpret_cast<float *>(st->K + (size_t)N * N + 2 * (size_t)N);
    HIP_TRY(hipMemcpyAsync(user_gamma, g32, (size_t)N * sizeof(float), hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));  // g32 lives on this frame
    HIP_TRY(launch_wsum(G, N, d, dtype, vec_ok, shape_of(st, ADACONS_TUNE_WSUM_BLOCKS_PER_CU), user_gamma, out, s));
    return ADACONS_OK;
}

adacons_status adacons_state_export(const adacons_state *st, double *m_host, int64_t *step, void *hip_stream) {
    if (!st || !m_host || !step) return fail(ADACONS_EINVAL, "NULL argument");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned long long t = 0;
    unsigned parity = 0;
    HIP_TRY(hipMemcpyAsync(&parity, &st->ds->parity, sizeof parity, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(&t, &st->ds->step, sizeof t, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));   // which of the two copies of m is the current one
    HIP_TRY(hipMemcpyAsync(m_host, st->ds->m[parity & 1u], (size_t)st->N * sizeof(double), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *step = (int64_t)t;
    return ADACONS_OK;
}

adacons_status adacons_state_import(adacons_state *st, const double *m_host, int64_t step, void *hip_stream) {
    if (!st || !m_host) return fail(ADACONS_EINVAL, "NULL argument");
    if (step < 0) return fail(ADACONS_EINVAL, "step < 0");
    for (int i = 0; i < st->N; ++i)
        if (!std::isfinite(m_host[i])) return fail(ADACONS_EINVAL, "m[%d] is not finite", i);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const unsigned long long t = (unsigned long long)step;
    // both copies: whichever is current holds the imported state
    HIP_TRY(hipMemcpyAsync(st->ds->m[0], m_host, (size_t)st->N * sizeof(double), hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(st->ds->m[1], m_host, (size_t)st->N * sizeof(double), hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(&st->ds->step, &t, sizeof t, hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    return ADACONS_OK;
}

adacons_status adacons_tune(adacons_state *st, adacons_tune_key key, int value) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    if ((int)key < 0 || key >= ADACONS_TUNE_COUNT_) return fail(ADACONS_EINVAL, "unknown tuning key %d", (int)key);
    if (value < 0) value = kTuneDefault[key];
    if ((key == ADACONS_TUNE_GRAM_BLOCKS_PER_CU || key == ADACONS_TUNE_WSUM_BLOCKS_PER_CU) && value > 8)
        return fail(ADACONS_EINVAL, "at most 8 workgroups per CU");
    if (key == ADACONS_TUNE_GRAM_PRODUCTS && value > 2) return fail(ADACONS_EINVAL, "ADACONS_TUNE_GRAM_PRODUCTS takes 0, 1 or 2");
    if (key == ADACONS_TUNE_SHORT_PATH && value > 2) return fail(ADACONS_EINVAL, "ADACONS_TUNE_SHORT_PATH takes 0, 1 or 2");
    if (key == ADACONS_TUNE_WSUM_ROW_SLICES && value > 2) return fail(ADACONS_EINVAL, "ADACONS_TUNE_WSUM_ROW_SLICES takes 0, 1 or 2");
    if (key == ADACONS_TUNE_WSUM_PARK_KB && value != 0 && value != 1 && (value < 8 || value > 144))
        return fail(ADACONS_EINVAL, "ADACONS_TUNE_WSUM_PARK_KB takes 0, 1 or 8..144");
    st->tune[key] = value;
    return ADACONS_OK;
}

adacons_status adacons_profile_begin(adacons_state *st, int max_calls) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    if (max_calls < 1 || max_calls > 4096) return fail(ADACONS_EINVAL, "max_calls outside [1, 4096]");
    while ((int)st->events.size() < 4 * max_calls) {
        hipEvent_t ev;
        HIP_TRY(hipEventCreate(&ev));
        st->events.push_back(ev);
    }
    st->prof_short.assign((size_t)max_calls, 0);
    st->prof_capacity = max_calls;
    st->prof_calls = 0;
    return ADACONS_OK;
}

adacons_status adacons_profile_end(adacons_state *st, double *gram_ms, double *coeff_ms, double *wsum_ms,
                                   int *calls, void *hip_stream) {
    if (!st) return fail(ADACONS_EINVAL, "state is NULL");
    HIP_TRY(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
    double a = 0.0, b = 0.0, w = 0.0;
    for (int c = 0; c < st->prof_calls; ++c) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, st->events[4 * c], st->events[4 * c + 1]));
        a += ms;
        if (st->prof_short[(size_t)c]) {   // stage A2 ran inside stage A3: no time of its own
            HIP_TRY(hipEventElapsedTime(&ms, st->events[4 * c + 1], st->events[4 * c + 3]));
            w += ms;
            continue;
        }
        HIP_TRY(hipEventElapsedTime(&ms, st->events[4 * c + 1], st->events[4 * c + 2]));
        b += ms;
        HIP_TRY(hipEventElapsedTime(&ms, st->events[4 * c + 2], st->events[4 * c + 3]));
        w += ms;
    }
    const int n = st->prof_calls;
    if (gram_ms) *gram_ms = n ? a / n : 0.0;
    if (coeff_ms) *coeff_ms = n ? b / n : 0.0;
    if (wsum_ms) *wsum_ms = n ? w / n : 0.0;
    if (calls) *calls = n;
    st->prof_capacity = 0;
    st->prof_calls = 0;
    return ADACONS_OK;
}

adacons_status adacons_aggregate_noalloc(const void *G, int N, int64_t d, adacons_dtype dtype, double beta,
                                         unsigned flags, double *m_dev, double *coeffs_dev,
                                         uint32_t *numeric_flags_dev, float *out, void *hip_stream) {
    if (N < 1) return fail(ADACONS_EINVAL, "N=%d < 1", N);
    if (N > ADACONS_N_MAX)
        return fail(ADACONS_EUNSUPPORTED, "N=%d beyond the maximum of %d workers this entry point's scratch array holds", N,
                    ADACONS_N_MAX);
    if (!(beta >= 0.0 && beta < 1.0)) return fail(ADACONS_EINVAL, "beta=%g outside [0, 1)", beta);
    if (flags & ~ADACONS_FLAG_ALL_) return fail(ADACONS_EINVAL, "unknown flag bits 0x%x", flags);
    if (!m_dev) return fail(ADACONS_EINVAL, "m_dev is NULL");
    if (reinterpret_cast<uintptr_t>(m_dev) % 8 || reinterpret_cast<uintptr_t>(coeffs_dev) % 8 ||
        reinterpret_cast<uintptr_t>(numeric_flags_dev) % 4)
        return fail(ADACONS_EALIGN, "m_dev / coeffs_dev / numeric_flags_dev not aligned to their element size");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    DeviceScratch sc;
    adacons_status rc = scratch_of(dev, &sc);
    if (rc != ADACONS_OK) return rc;
    unsigned char *base = static_cast<unsigned char *>(sc.ptr);

    // a state on this frame whose device pointers lie in the scratch array: default launch shapes
    adacons_state tmp;
    tmp.N = N;
    tmp.d_max = d;
    tmp.beta = beta;
    tmp.flags = flags;
    tmp.device = dev;
    tmp.num_cu = sc.num_cu;
    tmp.ds = reinterpret_cast<DevState *>(base + kScratchStateOff);
    tmp.K = reinterpret_cast<double *>(base + kScratchKOff);
    tmp.partials = reinterpret_cast<double *>(base + kScratchPartialsOff);
    const size_t row_doubles = partial_row_doubles(N);
    size_t rows = kScratchPartialsBytes / (row_doubles * sizeof(double));
    const size_t want_rows = (size_t)gram_rows_needed(N, sc.num_cu);
    if (rows > want_rows) rows = want_rows;
    if (rows < 2) return fail(ADACONS_EUNSUPPORTED, "scratch array too small for N=%d", N);
    tmp.max_rows = (int)rows;   // the first pass never launches more workgroups than it has rows for
    tmp.k_valid = false;
    for (int k = 0; k < ADACONS_TUNE_COUNT_; ++k) tmp.tune[k] = kTuneDefault[k];
    tmp.prof_capacity = 0;
    tmp.prof_calls = 0;

    bool vec_ok = false;
    rc = check_call(G, N, d, dtype, &tmp, out, true, &vec_ok);
    if (rc != ADACONS_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(launch_state_load(tmp.ds, N, m_dev, s));
    HIP_TRY(enqueue_aggregate(&tmp, G, N, d, dtype, vec_ok, out, false, 0.f, s, nullptr));
    HIP_TRY(launch_state_store(tmp.ds, N, m_dev, coeffs_dev, numeric_flags_dev, s));
    return ADACONS_OK;
}

}  // extern "C"
