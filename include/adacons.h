/*
 * adacons.h -- C ABI of the MI355X (gfx950) AdaCons gradient-aggregation library.
 *
 * AdaCons (arXiv 2411.03742) replaces the plain average of N workers' gradients
 * by a weighted sum  psi = sum_i gamma_i g_i  (Eq. 4, Eq. 12) whose weights come
 * from a first-order step on the N-dimensional subspace objective (Eq. 5-7),
 * smoothed by a momentum on the *sorted* coefficients (Eq. 11) and normalised
 * to sum to one (Sec. 3.4, Eq. 12-13).
 *
 * This library is the single-GPU hot path of that aggregator.  The N gradients
 * are the rows of one N x d matrix G resident in device memory; one call
 * computes, in three stream-ordered stages,
 *
 *   A1  K = G G^T                      (Eq. 7 third line: every <g_i, g_j>; its diagonal
 *                                       gives ||g_i||^2, its row sums N <g_i, gbar>)
 *   A2  a_i = <g_i, gbar>/||g_i||      (Eq. 7)  ->  sorted EMA (Eq. 11)  ->  c_i = a~_i/||g_i||
 *       (second normalisation of the column-normalised subspace matrix, Eq. 8)
 *       ->  gamma = c / sum c          (Eq. 12-13)
 *   A3  out = sum_i gamma_i g_i        (Eq. 12)
 *
 * Conventions common to every call
 *   - No torch or C++ types cross this boundary: plain pointers and sizes.
 *   - "device pointer" = memory of the current HIP device (hipMalloc or a
 *     framework's allocator); "host pointer" = ordinary host memory.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - Every function returns an adacons_status; nothing throws or aborts.
 *     adacons_last_error() gives a thread-local text for the last failure.
 *   - Numeric degeneracy (a zero gradient, NaN/Inf, weights that cancel) is not
 *     an error: it raises bits in a device-side status word that
 *     adacons_coeffs() returns (ADACONS_NUM_*).
 *   - One state is one coefficient stream: calls that use the same state must be
 *     ordered on one stream (or otherwise serialised by the caller).
 */
#ifndef ADACONS_H
#define ADACONS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADACONS_N_MAX 128     /* largest supported worker count (the largest N in the paper: Appendix A, linear regression) */
#define ADACONS_GRAM_N_MAX 64 /* largest N for which stage A1 forms the whole matrix K; above it stage A1
                                 computes what Eq. 7 consumes, diag K and the row sums of K (the norm and the
                                 dot product with the summed gradient of Alg. 1), and K is not available */

typedef struct adacons_state adacons_state; /* opaque, library-owned */

typedef enum {
    ADACONS_F32 = 0, /* G holds IEEE binary32 */
    ADACONS_BF16 = 1 /* G holds bfloat16 (upper half of binary32); accumulation and out stay fp32 */
} adacons_dtype;

typedef enum {
    ADACONS_OK = 0,
    ADACONS_EINVAL = 1,       /* null pointer, bad size, N mismatch, beta outside [0,1), aliasing */
    ADACONS_EUNSUPPORTED = 2, /* N > ADACONS_N_MAX, unknown dtype, wrong GPU architecture */
    ADACONS_EALIGN = 3,       /* G or out not aligned to its element size */
    ADACONS_EHIP = 4,         /* a HIP runtime call failed (see adacons_last_error) */
    ADACONS_ENOMEM = 5        /* device or host allocation failed */
} adacons_status;

/* Variant flags (the ablation columns of Table 2).  Default = both. */
enum {
    ADACONS_FLAG_MOMENTUM = 1u,  /* sorted EMA of Eq. 11; off: a~ = a */
    ADACONS_FLAG_NORMALIZE = 2u, /* sum-to-one weights of Eq. 12-13; off: gamma_i = c_i (lambda = 1, Eq. 8) */
    ADACONS_FLAG_DEFAULT = 3u,
    /* Two variants the paper discusses, off by default: */
    ADACONS_FLAG_INDEX_EMA = 4u,   /* with MOMENTUM: m_i <- beta m_i + (1-beta) a_i per worker index (Eq. 10),
                                      the momentum Sec. 3.3 replaces by the sorted one of Eq. 11 */
    ADACONS_FLAG_LAMBDA_EQ13 = 8u, /* with NORMALIZE: lambda = 1 / sum_k a~_k exactly as Eq. 13 prints it: the
                                      coefficients on the column-normalised subspace matrix, gamma_i ||g_i||,
                                      sum to one instead of the weights on the raw gradients */
    ADACONS_FLAG_ALL_ = 15u
};

/* Bits of the numeric status word returned by adacons_coeffs(). */
enum {
    ADACONS_NUM_ZERO_NORM = 1u,       /* some ||g_i|| = 0: that worker gets a_i = c_i = 0 */
    ADACONS_NUM_NONFINITE = 2u,       /* NaN/Inf reached K: EMA state left untouched */
    ADACONS_NUM_UNIFORM_FALLBACK = 4u /* gamma_i = 1/N used (non-finite, or |sum c| <= 1e-12 sum|c|) */
};

/*
 * Create the carried state of one coefficient stream: the EMA vector m of
 * Eq. 11 (N doubles kept in sorted order, zero-initialised), the call counter,
 * the coefficient buffers and the partial-sum workspace of stage A1, all on the
 * current HIP device.  This is the only call that allocates device memory.  Later calls
 * with this state must be made with the same device current (else ADACONS_EINVAL).
 *   st       out: receives the handle (host pointer to a host pointer)
 *   N        number of workers, 1 <= N <= ADACONS_N_MAX
 *   d_max    largest gradient length later calls may pass, >= 1
 *   beta     EMA factor of Eq. 11, 0 <= beta < 1 (the paper uses 0.99, Table 2)
 *   flags    ADACONS_FLAG_* bits
 * Errors: EINVAL, EUNSUPPORTED, ENOMEM, EHIP.  Synchronises `hip_stream` once.
 */
adacons_status adacons_init_state(adacons_state **st, int N, int64_t d_max, double beta,
                                  unsigned flags, void *hip_stream);

/* Free everything the state owns.  The caller must have drained all work using it. */
adacons_status adacons_destroy_state(adacons_state *st);

/* m := 0, call counter := 0 (asynchronous on the stream). */
adacons_status adacons_reset_state(adacons_state *st, void *hip_stream);

/*
 * One aggregation psi_t({g_i}) (Eq. 4 with Eq. 12): stages A1, A2, A3 enqueued on
 * `hip_stream`.  Asynchronous; allocates nothing; never synchronises.
 *   G      device pointer, N x d row-major contiguous (row i = g_i, row stride d elements),
 *          element type `dtype`; read twice; must stay valid until the stream reaches the
 *          end of this call's work; must be aligned to its element size.  Every shape runs on
 *          the same 128-bit kernels: when G or out is not 16-byte aligned, or d*sizeof(elem) is not
 *          a multiple of 16 (rows then start off the 16-byte grid), the accesses are issued from
 *          element-aligned addresses and the d mod 4 (fp32) or d mod 8 (bf16) columns that no whole
 *          group covers are added by a small extra launch per stage; measured 6.1 against 6.25 TB/s
 *          at N = 8, d = 25.6 M + 1.  A caller that flattens gradients itself gains 2-5 % by padding
 *          d to a multiple of 128 bytes (rows on cache lines).
 *   N, d   must satisfy N == state's N, 1 <= d <= d_max
 *   out    device pointer to d floats (fp32 for both dtypes), caller-owned, written once,
 *          4-byte aligned, must not overlap G
 * State mutated: m (Eq. 11), call counter, gamma / raw / smoothed coefficient buffers, K,
 * numeric status word.
 * Errors: EINVAL, EUNSUPPORTED, EALIGN, EHIP (launch failure).
 */
adacons_status adacons_aggregate(const void *G, int N, int64_t d, adacons_dtype dtype,
                                 adacons_state *st, float *out, void *hip_stream);

/*
 * The aggregation fused with the descent step it feeds (Eq. 4 with Eq. 12):
 *     w[k] <- w[k] - lr * sum_i gamma_i G[i][k]
 * Stages A1 and A2 as in adacons_aggregate; stage A3 reads and rewrites the fp32 parameter
 * vector w (device pointer, d floats, caller-owned, must not overlap G) instead of writing `out`,
 * which saves the d-sized write and re-read between aggregator and optimiser.  lr is the step
 * size eta_t (finite).  Same argument rules, state changes and errors as adacons_aggregate.
 */
adacons_status adacons_aggregate_apply(const void *G, int N, int64_t d, adacons_dtype dtype,
                                       adacons_state *st, float *w, float lr, void *hip_stream);

/*
 * adacons_aggregate() for callers that cannot allocate device memory and therefore cannot call
 * adacons_init_state(): code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It calls no hipMalloc, hipFree or other allocating routine.  Stages A1, A2, A3 run with
 * the same kernels and default launch shapes as adacons_aggregate() (results are bit-identical to it);
 * what that call keeps in its state -- the partial sums of stage A1, K, the coefficient block -- lives in
 * a 20 MiB array in the library's device image (one copy per GPU, held until the process ends), and the
 * carried state of the momentum is the caller's:
 *   beta, flags       as in adacons_init_state
 *   m_dev             device pointer, N doubles, 8-byte aligned, read and rewritten: the EMA vector m (sorted
 *                     order); zeros before the first step
 *   coeffs_dev        device pointer, 3 N doubles (gamma, then the first-order, then the smoothed
 *                     coefficients), written; or NULL
 *   numeric_flags_dev device pointer, one 32-bit word (ADACONS_NUM_* of this call), written; or NULL
 *   G, N, d, dtype, out, hip_stream   as in adacons_aggregate
 * Limits: N <= ADACONS_N_MAX (ADACONS_EUNSUPPORTED beyond, with a message naming the limit); any d >= 1.
 * Asynchronous; never synchronises.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on one GPU (two streams, two threads) race; calls ordered on one stream do not.  The first call on
 * a device looks the array's address up (hipGetSymbolAddress, once per device): make it outside a graph
 * capture.  Errors: EINVAL, EUNSUPPORTED, EALIGN, EHIP.
 */
adacons_status adacons_aggregate_noalloc(const void *G, int N, int64_t d, adacons_dtype dtype, double beta,
                                         unsigned flags, double *m_dev, double *coeffs_dev,
                                         uint32_t *numeric_flags_dev, float *out, void *hip_stream);

/*
 * Read back the coefficients of the most recent adacons_aggregate() on this state
 * (the three stages of Fig. 7: first-order, after momentum, after normalisation).
 * Copies on `hip_stream` and waits for it: the only synchronising call of the hot API.
 *   gamma_host     host pointer, N doubles: the weights gamma_i actually applied
 *   raw_host       host pointer, N doubles, or NULL: a_i of Eq. 7
 *   smoothed_host  host pointer, N doubles, or NULL: a~_i after Eq. 11
 *   numeric_flags  host pointer or NULL: ADACONS_NUM_* bits of that call
 */
adacons_status adacons_coeffs(const adacons_state *st, double *gamma_host, double *raw_host,
                              double *smoothed_host, uint32_t *numeric_flags, void *hip_stream);

/*
 * Stage A1 alone: K = G G^T (Eq. 7 third line / the double sum of Eq. 8) into the state's
 * K buffer, without touching the coefficient state.  Same argument rules as
 * adacons_aggregate.  Asynchronous.  ADACONS_EUNSUPPORTED for N > ADACONS_GRAM_N_MAX.
 */
adacons_status adacons_gram(const void *G, int N, int64_t d, adacons_dtype dtype,
                            adacons_state *st, void *hip_stream);

/* Copy the state's K (N x N doubles, row-major, symmetric) to the host; synchronises the stream.
 * ADACONS_EINVAL when the last call on this state did not produce K (ADACONS_TUNE_STATS_ONLY, or
 * N > ADACONS_GRAM_N_MAX). */
adacons_status adacons_read_gram(const adacons_state *st, double *K_host, void *hip_stream);

/*
 * Stage A3 alone: out = sum_i gamma_i g_i (Eq. 12) with caller-supplied weights.
 *   gamma_host  host pointer, N doubles (rounded to fp32 for the kernel); copied to a buffer of the
 *               state on the stream; what adacons_coeffs() reports is not touched
 * Other arguments as in adacons_aggregate.  Synchronises the stream once (host weights).
 */
adacons_status adacons_weighted_sum(const void *G, int N, int64_t d, adacons_dtype dtype,
                                    const double *gamma_host, adacons_state *st, float *out,
                                    void *hip_stream);

/*
 * Checkpoint / resume of the carried state of Eq. 11: m (N doubles, sorted order) and the call
 * counter.  Both synchronise the stream.  Import requires the same N.
 */
adacons_status adacons_state_export(const adacons_state *st, double *m_host, int64_t *step,
                                    void *hip_stream);
adacons_status adacons_state_import(adacons_state *st, const double *m_host, int64_t step,
                                    void *hip_stream);

/*
 * Tuning knobs (launch shape and choice of kernel; results stay within the documented tolerances, and are
 * bit-identical between runs for a fixed setting).  value < 0 restores the default.
 */
typedef enum {
    ADACONS_TUNE_GRAM_BLOCKS_PER_CU = 0, /* persistent workgroups per CU in stage A1 (at most 8) */
    ADACONS_TUNE_WSUM_BLOCKS_PER_CU = 1, /* persistent workgroups per CU in stage A3 (at most 8) */
    ADACONS_TUNE_CACHED_HEAD_MB = 2,     /* A1 reads the first `value` MiB of G with cache-allocating loads and
                                            streams the rest past the caches, so that A3 finds the head in the
                                            memory-side cache.  Default 320; >= 2^20 means all of G */
    ADACONS_TUNE_GRAM_PRODUCTS = 3,      /* A1, 8 < N <= 64, fp32 inputs: 0 = products on the fp32 matrix-core
                                            instruction; 1 = every product formed from six exact bf16 products on
                                            the bf16 matrix-core instruction (an fp32 value is the exact sum of
                                            three bf16 values; dropped terms < 2^-24 of the product); 2 (default)
                                            = 1 for N > 32, else 0.  bf16 inputs always take the bf16 instruction */
    ADACONS_TUNE_STATS_ONLY = 4,         /* 1: for N > 8 stage A1 computes only what Eq. 7 consumes, the diagonal
                                            of K and its row sums (||g_i||^2 and <g_i, sum_j g_j>: Alg. 1 steps
                                            1-2), in O(N) operations per column; K is then not produced and
                                            adacons_read_gram() reports ADACONS_EINVAL.  0 (default): full K
                                            (N > ADACONS_GRAM_N_MAX takes this pass whatever the value) */
    ADACONS_TUNE_WSUM_PARK_KB = 5,       /* A3 keeps whole tiles of output in LDS and writes them in bursts instead of
                                            tile by tile among the loads.  0: never; 1 (default): where it measured
                                            faster (long fp32 streams of many rows); 8 .. 144: always, with that
                                            many KB of LDS */
    ADACONS_TUNE_SHORT_PATH = 6,         /* two launches instead of three (16-byte aligned rows): stage A3 adds stage
                                            A1's partial sums and runs stage A2 itself (same results, bit for bit).
                                            0: never; 1 (default): N <= 8 with at most 32 MiB of gradients (bf16: 16 MiB
                                            for 2 < N <= 6, 8 MiB for N = 7, 8), which
                                            stay in the caches between the passes and are bound by launches, not
                                            bytes, and N > 8 with at most 1 MiB where stage A3 runs by row slices
                                            (not for 44 < N <= 64 with the full matrix K); 2: also N <= 8 at any
                                            size */
    ADACONS_TUNE_WSUM_ROW_SLICES = 7,    /* A3 for many workers with few parameters each (N > 8): the rows are
                                            shared out over the sixteen wavefronts of a workgroup, which adds their
                                            partial sums in wavefront order, instead of one thread walking all N
                                            rows of its columns.  0: never; 1 (default): where it measured faster;
                                            2: whenever N > 8 */
    ADACONS_TUNE_COUNT_
} adacons_tune_key;
adacons_status adacons_tune(adacons_state *st, adacons_tune_key key, int value);

/*
 * Per-kernel timing with HIP events on the caller's stream, for roofline reporting.
 * adacons_profile_begin() creates event pairs for up to max_calls aggregations (this
 * allocates; call it outside any timed region); later adacons_aggregate() calls record an
 * event before stage A1, after the Gram kernel, after A2 and after A3.  adacons_profile_end()
 * waits for the stream, returns the mean duration in milliseconds of the Gram kernel (gram_ms), of
 * the partial-sum reduction + coefficient update (coeff_ms; 0 for calls on the short path, where
 * stage A3 does that work) and of A3 (wsum_ms) over the recorded calls and their count, and
 * stops recording.  Any output pointer may be NULL.
 */
adacons_status adacons_profile_begin(adacons_state *st, int max_calls);
adacons_status adacons_profile_end(adacons_state *st, double *gram_ms, double *coeff_ms, double *wsum_ms,
                                   int *calls, void *hip_stream);

/*
 * ---- One worker's share of Algorithm 1 ---------------------------------------------------
 * The arithmetic on either side of the paper's collectives, for a caller that keeps the
 * gradients distributed (one worker per GPU) and runs the collectives itself:
 *   after all-reducing the gradients (Alg. 1 step 1) a worker holds its own g and their sum;
 *   adacons_worker_stats gives <g, gsum> and ||g||^2 in one pass over the two vectors;
 *   with the N pairs gathered (step 2), adacons_update_from_stats runs the coefficient update
 *   (Eq. 7, Eq. 11, Eq. 12-13; step 3) on the state; adacons_worker_scale rescales the local
 *   gradient in place by its weight (step 4), ready for the final all-reduce.
 */

/*
 *   g, gsum    device pointers, d elements of `dtype` each (may be the same pointer), aligned to the
 *              element size; any d
 *   st         supplies the partial-sum workspace; d <= its d_max
 *   stats_dev  device pointer, 3 doubles, 8-byte aligned: ||g||^2, <g, gsum>, ||gsum||^2
 * Asynchronous, allocates nothing.  Errors: EINVAL, EUNSUPPORTED, EALIGN, EHIP.
 */
adacons_status adacons_worker_stats(const void *g, const void *gsum, int64_t d, adacons_dtype dtype,
                                    adacons_state *st, double *stats_dev, void *hip_stream);

/*
 * Stage A2 from gathered statistics instead of a Gram matrix:
 *   sq_host[i] = ||g_i||^2, dot_host[i] = <g_i, sum_j g_j>   (host pointers, N doubles each)
 * Updates the state exactly as adacons_aggregate's coefficient step does (readable through
 * adacons_coeffs).  Copies from the host arrays and waits for the copy once.
 */
adacons_status adacons_update_from_stats(adacons_state *st, const double *sq_host, const double *dot_host,
                                         void *hip_stream);

/*
 * g <- gamma[worker] * g in place (device pointer, d elements; bf16 is rounded to nearest even),
 * with the weight the state currently holds for `worker` (0 <= worker < N).  Asynchronous.
 */
adacons_status adacons_worker_scale(void *g, int64_t d, adacons_dtype dtype, const adacons_state *st,
                                    int worker, void *hip_stream);

/*
 * ---- Layer-wise aggregation --------------------------------------------------------------
 * Sec. 4 of the paper computes the aggregation model-wise and mentions the layer-wise variant beside it.
 * Here the d columns are split into L contiguous segments ("layers"); every
 * layer gets its own Gram matrix, its own coefficients and its own Eq. 11 momentum state, i.e. the
 * steps A1-A3 above run independently on G[:, offsets[l] : offsets[l+1]) for every l, in three
 * launches for all layers together.  For N <= 8 stage A1 forms every layer's
 * Gram matrix; for N > 8 it forms what Eq. 7 consumes of it, ||g_i||^2 and <g_i, sum_j g_j> over the
 * layer's columns (Alg. 1 steps 1-2 per layer).
 */
typedef struct adacons_layers adacons_layers; /* opaque, library-owned */

/*
 * Build the per-layer state (L zero-initialised momentum vectors, tile tables, workspaces) on the
 * current device.  Allocates; synchronises `hip_stream` once.
 *   ls            out: receives the handle
 *   N             workers, 1 <= N <= ADACONS_N_MAX
 *   L             number of layers, >= 1
 *   offsets_host  host pointer, L + 1 ascending column offsets, offsets[0] = 0, offsets[L] = d;
 *                 empty layers (equal consecutive offsets) are not allowed; d must be at least one
 *                 128-bit group (4 fp32 / 8 bf16 elements)
 *   dtype         element type later calls will pass (fixes the tile geometry)
 *   beta, flags   as in adacons_init_state
 * Errors: EINVAL, EUNSUPPORTED (N > ADACONS_N_MAX, unknown dtype), ENOMEM, EHIP.
 */
adacons_status adacons_init_layers(adacons_layers **ls, int N, int L, const int64_t *offsets_host,
                                   adacons_dtype dtype, double beta, unsigned flags, void *hip_stream);
adacons_status adacons_destroy_layers(adacons_layers *ls);

/*
 * One layer-wise aggregation: out[k] = sum_i gamma[layer(k)][i] G[i][k].  Asynchronous, allocates
 * nothing.  G, N, d, dtype, out as in adacons_aggregate, with d == offsets[L] and dtype as given at
 * init; G and out aligned to their element size (else EALIGN): as there, any d and any such alignment
 * run on the 128-bit kernels.
 */
adacons_status adacons_aggregate_layers(const void *G, int N, int64_t d, adacons_dtype dtype,
                                        adacons_layers *ls, float *out, void *hip_stream);

/*
 * Coefficients of the most recent adacons_aggregate_layers(): L x N doubles each, row l = layer l.
 * raw_host, smoothed_host, numeric_flags (L words) may be NULL.  Synchronises the stream.
 */
adacons_status adacons_layer_coeffs(const adacons_layers *ls, double *gamma_host, double *raw_host,
                                    double *smoothed_host, uint32_t *numeric_flags, void *hip_stream);

const char *adacons_status_string(adacons_status s);
const char *adacons_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ADACONS_H */
