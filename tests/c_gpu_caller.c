/* The hot path from plain C, with no Python and no PyTorch in the process: device memory and the
 * stream come from the HIP runtime, the attention from libelsa.so, the expected values from the C
 * oracle (FP64).  Built by tests/build_c_gpu_caller.py; run by tests/test_gpu_c_caller.py.
 * Cases: FP32, B = 2, H = 3, n = 300 (ragged tail), d = 64, without and with the causal mask, on
 * the default stream and on a stream of its own; then the same rows through
 * elsa_attn_fwd_split_kv + elsa_combine.  Error metric: |delta| / (|ref| + rms of the row). */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "elsa.h"

int elsa_oracle_attn_rows(const float *q, const float *k, const float *v, int B, int H, int n, int d, double scale,
                          int causal, const int32_t *kv_len, const int64_t *rows, int64_t nrows, double *out);

#define HIP_OK(call)                                                        \
    do {                                                                    \
        hipError_t e_ = (call);                                             \
        if (e_ != hipSuccess) {                                             \
            printf("FAILED %s -> %s\n", #call, hipGetErrorString(e_));      \
            return 2;                                                       \
        }                                                                   \
    } while (0)

static uint32_t lcg_state = 12345u;
static float lcg_uniform(void) { /* (-1, 1) */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((float)(lcg_state >> 8) + 0.5f) / 8388608.0f - 1.0f;
}

static double worst_error(const float *got, const double *ref, int rows, int d) {
    double worst = 0.0;
    for (int r = 0; r < rows; ++r) {
        double ss = 0.0;
        for (int t = 0; t < d; ++t) ss += ref[(size_t)r * d + t] * ref[(size_t)r * d + t];
        const double rms = sqrt(ss / d);
        for (int t = 0; t < d; ++t) {
            const double x = ref[(size_t)r * d + t];
            const double e = fabs((double)got[(size_t)r * d + t] - x) / (fabs(x) + rms);
            if (!(e <= worst)) worst = e; /* a NaN in the output becomes the worst error */
        }
    }
    return worst;
}

int main(void) {
    enum { B = 2, H = 3, N = 300, D = 64, C = 3 };
    const size_t elems = (size_t)B * H * N * D, rows = (size_t)B * H * N;
    const float scale = 0.125f;
    const double tol = 2e-5;
    int fails = 0;
    float *q = malloc(elems * 4), *k = malloc(elems * 4), *v = malloc(elems * 4), *got = malloc(elems * 4);
    double *ref = malloc(elems * 8);
    int64_t *all_rows = malloc(rows * 8);
    if (!q || !k || !v || !got || !ref || !all_rows) return 2;
    for (size_t i = 0; i < elems; ++i) { q[i] = 2.0f * lcg_uniform(); k[i] = 2.0f * lcg_uniform(); v[i] = lcg_uniform(); }
    for (size_t r = 0; r < rows; ++r) all_rows[r] = (int64_t)r;

    int ndev = 0;
    HIP_OK(hipGetDeviceCount(&ndev));
    if (ndev < 1) { printf("FAILED no GPU\n"); return 2; }
    HIP_OK(hipSetDevice(0));
    void *dq, *dk, *dv, *dout, *dm, *dS, *dW;
    hipStream_t stream;
    HIP_OK(hipMalloc(&dq, elems * 4));
    HIP_OK(hipMalloc(&dk, elems * 4));
    HIP_OK(hipMalloc(&dv, elems * 4));
    HIP_OK(hipMalloc(&dout, elems * 4));
    HIP_OK(hipMalloc(&dm, rows * C * 4));
    HIP_OK(hipMalloc(&dS, rows * C * 4));
    HIP_OK(hipMalloc(&dW, elems * C * 4));
    HIP_OK(hipStreamCreate(&stream));
    HIP_OK(hipMemcpy(dq, q, elems * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dk, k, elems * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dv, v, elems * 4, hipMemcpyHostToDevice));

    for (int causal = 0; causal < 2; ++causal) {
        if (elsa_oracle_attn_rows(q, k, v, B, H, N, D, (double)scale, causal, NULL, all_rows, (int64_t)rows, ref) != 0) return 2;
        for (int own_stream = 0; own_stream < 2; ++own_stream) {
            HIP_OK(hipMemset(dout, 0xff, elems * 4)); /* NaN pattern: every element must be written */
            const int rc = elsa_attn_fwd(dq, dk, dv, dout, B, H, N, D, scale, causal, ELSA_F32, own_stream ? (void *)stream : NULL);
            if (rc != ELSA_OK) { printf("FAILED elsa_attn_fwd: %s\n", elsa_status_string(rc)); return 1; }
            HIP_OK(hipStreamSynchronize(own_stream ? stream : NULL));
            HIP_OK(hipMemcpy(got, dout, elems * 4, hipMemcpyDeviceToHost));
            const double e = worst_error(got, ref, (int)rows, D);
            printf("elsa_attn_fwd causal=%d stream=%s kernel=%s worst error %.3g (tolerance %.0e)\n", causal,
                   own_stream ? "own" : "default", elsa_last_kernel(), e, tol);
            if (!(e <= tol)) ++fails;
        }
    }

    /* key chunks kept as states (m, S, W), then merged: Eq. 3 / Eq. 4 through the boundary */
    if (elsa_oracle_attn_rows(q, k, v, B, H, N, D, (double)scale, 0, NULL, all_rows, (int64_t)rows, ref) != 0) return 2;
    HIP_OK(hipMemset(dout, 0xff, elems * 4));
    int rc = elsa_attn_fwd_split_kv(dq, dk, dv, (float *)dm, (float *)dS, (float *)dW, B, H, N, D, scale, 0, NULL, C, ELSA_F32, stream);
    if (rc == ELSA_OK) rc = elsa_combine((const float *)dm, (const float *)dS, (const float *)dW, dout, B, H, N, D, C, ELSA_F32, stream);
    if (rc != ELSA_OK) { printf("FAILED split_kv/combine: %s\n", elsa_status_string(rc)); return 1; }
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(got, dout, elems * 4, hipMemcpyDeviceToHost));
    {
        const double e = worst_error(got, ref, (int)rows, D);
        printf("elsa_attn_fwd_split_kv x%d + elsa_combine worst error %.3g (tolerance %.0e)\n", C, e, tol);
        if (!(e <= tol)) ++fails;
    }

    HIP_OK(hipStreamDestroy(stream));
    HIP_OK(hipFree(dq)); HIP_OK(hipFree(dk)); HIP_OK(hipFree(dv)); HIP_OK(hipFree(dout));
    HIP_OK(hipFree(dm)); HIP_OK(hipFree(dS)); HIP_OK(hipFree(dW));
    free(q); free(k); free(v); free(got); free(ref); free(all_rows);
    printf("%s\n", fails ? "c gpu caller: FAILED" : "c gpu caller: ok");
    return fails ? 1 : 0;
}
