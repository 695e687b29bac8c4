/*
 * A consumer of libqn's C ABI written in plain C, with no Python and no torch:
 * device memory comes from hipMalloc, inputs from a counter-based generator on
 * the host, and every result is compared with the CPU oracle (linked in here as
 * the checker, never by the library).  Built by tests/host/build_consumer.py,
 * run on the GPU by tests/test_gpu_c_consumer.py.
 *
 * For each problem it runs the whole step three ways -- qn_update (library-owned
 * scratch), qn_update_ws (caller-owned scratch) and qn_update_noalloc (static
 * scratch) -- checks that the three agree bit for bit, and compares with the
 * oracle's literal evaluation of eq. (2)-(4): same j, theta_new within 1e-5 in
 * relative L2 norm and 2e-5 of max|theta_new| element by element.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "qn.h"
#include "qn_oracle.h"

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                             \
        }                                                                         \
    } while (0)

/* splitmix64: a published counter-based generator; uniform in (0, 1) */
static double u01(uint64_t seed, uint64_t i)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ULL * (i + 1);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return ((double)(z >> 11) + 0.5) / 9007199254740992.0;
}
static double gauss(uint64_t seed, uint64_t i)
{
    return sqrt(-2.0 * log(u01(seed, 2 * i))) * cos(6.283185307179586 * u01(seed, 2 * i + 1));
}

static int run_case(int64_t n, int m, float tau, float lambda, uint64_t seed)
{
    const size_t elems = (size_t)n * m;
    float *th = (float *)malloc(elems * 4), *gr = (float *)malloc(elems * 4);
    float *got[3];
    double *want = (double *)malloc((size_t)n * 8);
    if (!th || !gr || !want)
        return 2;
    /* diagonal quadratic: grad_k = a * theta_k - b + noise, theta_k = theta0 + spread */
    for (int64_t i = 0; i < n; ++i) {
        const double a = exp(log(1e-3) + (log(1e2) - log(1e-3)) * u01(seed, i));
        const double b = gauss(seed + 1, i), t0 = gauss(seed + 2, i);
        for (int k = 0; k < m; ++k) {
            const float t = (float)(t0 + 1e-2 * gauss(seed + 3, (uint64_t)k * n + i));
            th[(size_t)k * n + i] = t;
            gr[(size_t)k * n + i] = (float)(a * t - b + 1e-3 * gauss(seed + 4, (uint64_t)k * n + i));
        }
    }
    int j_want = -7;
    if (qno_update_literal(th, gr, QNO_F32, n, m, n, tau, lambda, want, &j_want, NULL, NULL,
                           NULL, NULL) != 0) {
        printf("oracle failed\n");
        return 2;
    }

    float *d_th, *d_gr, *d_out;
    int *d_j;
    void *d_ws;
    const size_t ws_bytes = qn_workspace_bytes(n, m, QN_F32);
    CK(hipMalloc((void **)&d_th, elems * 4));
    CK(hipMalloc((void **)&d_gr, elems * 4));
    CK(hipMalloc((void **)&d_out, (size_t)n * 4));
    CK(hipMalloc((void **)&d_j, sizeof(int)));
    CK(hipMalloc(&d_ws, ws_bytes));
    CK(hipMemcpy(d_th, th, elems * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_gr, gr, elems * 4, hipMemcpyHostToDevice));
    hipStream_t stream;
    CK(hipStreamCreate(&stream));

    int bad = 0, j_got[3];
    for (int way = 0; way < 3; ++way) {
        got[way] = (float *)malloc((size_t)n * 4);
        CK(hipMemsetAsync(d_out, 0xff, (size_t)n * 4, stream));
        int rc;
        if (way == 0)
            rc = qn_update(d_th, d_gr, n, m, tau, lambda, d_out, d_j, stream);
        else if (way == 1)
            rc = qn_update_ws(d_th, d_gr, QN_F32, n, m, n, tau, lambda, d_out, d_j, d_ws, ws_bytes,
                              stream);
        else
            rc = qn_update_noalloc(d_th, d_gr, QN_F32, n, m, n, tau, lambda, d_out, d_j, stream);
        if (rc != QN_OK) {
            printf("way %d: %s\n", way, qn_status_string(rc));
            return 2;
        }
        CK(hipStreamSynchronize(stream));
        CK(hipMemcpy(got[way], d_out, (size_t)n * 4, hipMemcpyDeviceToHost));
        CK(hipMemcpy(&j_got[way], d_j, sizeof(int), hipMemcpyDeviceToHost));
    }
    double d2 = 0.0, w2 = 0.0, dmax = 0.0, wmax = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double d = (double)got[0][i] - want[i];
        d2 += d * d;
        w2 += want[i] * want[i];
        dmax = fabs(d) > dmax ? fabs(d) : dmax;
        wmax = fabs(want[i]) > wmax ? fabs(want[i]) : wmax;
    }
    const double rel = sqrt(d2 / w2);
    const int same = memcmp(got[0], got[1], (size_t)n * 4) == 0 &&
                     memcmp(got[0], got[2], (size_t)n * 4) == 0 && j_got[0] == j_got[1] &&
                     j_got[0] == j_got[2];
    bad = !(same && j_got[0] == j_want && rel <= 1e-5 && dmax <= 2e-5 * wmax);
    printf("n=%lld m=%d lambda=%g: j %d (oracle %d), rel L2 %.3e, max|d|/max|want| %.3e, "
           "three entry points %s -> %s\n",
           (long long)n, m, (double)lambda, j_got[0], j_want, rel, dmax / wmax,
           same ? "bit-identical" : "DIFFER", bad ? "FAIL" : "ok");

    /* a workspace one byte short is refused before anything runs */
    if (qn_update_ws(d_th, d_gr, QN_F32, n, m, n, tau, lambda, d_out, d_j, d_ws, ws_bytes - 1,
                     stream) != QN_EWORKSPACE) {
        printf("short workspace was not refused\n");
        bad = 1;
    }
    CK(hipStreamDestroy(stream));
    CK(hipFree(d_th)); CK(hipFree(d_gr)); CK(hipFree(d_out)); CK(hipFree(d_j)); CK(hipFree(d_ws));
    free(th); free(gr); free(want);
    for (int way = 0; way < 3; ++way)
        free(got[way]);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= run_case(4096, 4, 1.0f, 0.01f, 11);        /* fp64 Gram kernel */
    bad |= run_case(100003, 8, 0.5f, 0.05f, 12);      /* streaming pass, columns not 16-byte aligned */
    bad |= run_case(65536, 32, 1.0f, 0.01f, 13);
    bad |= run_case(20, 33, 1.0f, 0.3f, 14);          /* n < m */
    if (qn_shutdown() != QN_OK)
        bad = 1;
    printf(bad ? "C consumer: FAILED\n" : "C consumer: all ok\n");
    return bad ? 1 : 0;
}
