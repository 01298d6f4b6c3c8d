/*
 * The library used from plain C: HIP runtime for memory, nothing else.  Checks two cases whose
 * results have closed forms (no reference implementation involved):
 *   1. identical worker gradients reduce to plain averaging (Sec. 3.2): gamma_i = 1/N, out = g;
 *   2. worker i holds (i + 1) g: a_i = <g_i, gbar> / ||g_i|| is the same for every worker, so
 *      gamma_i is proportional to 1 / (i + 1) (Eq. 8, Eq. 12-13) and out = N / H_N * g, H_N the
 *      N-th harmonic number.
 * Values are small integers, so the inputs are exact in fp32.  Exit code 0 on success.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "adacons.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 10; } } while (0)
#define CHECK_ADA(x) do { adacons_status s_ = (x); if (s_ != ADACONS_OK) { fprintf(stderr, "%s: %s (%s)\n", #x, adacons_status_string(s_), adacons_last_error()); return 11; } } while (0)

static int run_case(int N, long long d, int scaled)
{
    float *hG = (float *)malloc(sizeof(float) * (size_t)N * (size_t)d);
    float *hout = (float *)malloc(sizeof(float) * (size_t)d);
    if (!hG || !hout) return 12;
    for (int i = 0; i < N; ++i)
        for (long long k = 0; k < d; ++k)
            hG[(size_t)i * d + k] = (float)((scaled ? i + 1 : 1) * (int)(k % 17 - 8));
    float *dG = NULL, *dout = NULL;
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HIP(hipMalloc((void **)&dG, sizeof(float) * (size_t)N * (size_t)d));
    CHECK_HIP(hipMalloc((void **)&dout, sizeof(float) * (size_t)d));
    CHECK_HIP(hipMemcpy(dG, hG, sizeof(float) * (size_t)N * (size_t)d, hipMemcpyHostToDevice));

    adacons_state *st = NULL;
    CHECK_ADA(adacons_init_state(&st, N, d, 0.99, ADACONS_FLAG_DEFAULT, stream));
    CHECK_ADA(adacons_aggregate(dG, N, d, ADACONS_F32, st, dout, stream));
    double gamma[ADACONS_N_MAX];
    uint32_t flags = 99;
    CHECK_ADA(adacons_coeffs(st, gamma, NULL, NULL, &flags, stream));
    CHECK_HIP(hipMemcpy(hout, dout, sizeof(float) * (size_t)d, hipMemcpyDeviceToHost));

    double harmonic = 0.0;
    for (int i = 0; i < N; ++i) harmonic += 1.0 / (i + 1);
    int bad = (flags != 0);
    for (int i = 0; i < N; ++i) {
        const double want = scaled ? (1.0 / (i + 1)) / harmonic : 1.0 / N;
        if (fabs(gamma[i] - want) > 1e-9 * want) { fprintf(stderr, "gamma[%d] = %.15g, expected %.15g\n", i, gamma[i], want); bad = 1; }
    }
    const double scale = scaled ? (double)N / harmonic : 1.0;
    for (long long k = 0; k < d; ++k) {
        const double want = scale * (double)(int)(k % 17 - 8);
        if (fabs(hout[k] - want) > 1e-5 * (fabs(want) + 1.0)) { fprintf(stderr, "out[%lld] = %g, expected %g\n", k, hout[k], want); bad = 1; break; }
    }
    /* an error must come back as a status, with a message, and leave the state usable */
    if (adacons_aggregate(dG, N + 1, d, ADACONS_F32, st, dout, stream) != ADACONS_EINVAL || adacons_last_error()[0] == 0) bad = 1;
    CHECK_ADA(adacons_aggregate(dG, N, d, ADACONS_F32, st, dout, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_ADA(adacons_destroy_state(st));
    CHECK_HIP(hipFree(dG));
    CHECK_HIP(hipFree(dout));
    CHECK_HIP(hipStreamDestroy(stream));
    free(hG);
    free(hout);
    printf("N=%d d=%lld %s: %s\n", N, d, scaled ? "scaled copies" : "identical gradients", bad ? "FAILED" : "ok");
    return bad;
}

int main(void)
{
    int rc = 0;
    rc |= run_case(4, 100003, 0);
    rc |= run_case(8, 1000000, 1);
    rc |= run_case(32, 65540, 1);
    rc |= run_case(64, 20000, 0);
    return rc;
}
