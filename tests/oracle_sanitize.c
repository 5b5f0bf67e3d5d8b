/* The oracle's C source under AddressSanitizer and UBSan: this driver is compiled together with
 * oracle/elsa_oracle.c (-fsanitize=address,undefined) and runs a condensed battery of the pins with
 * awkward sizes (n = 1, ragged chunks, more chunks than keys, empty rows, n_q != n_k, d_v != d), so
 * that any out-of-bounds index, overflow or misaligned access in the checker itself stops the run.
 * Exit status 0 = every check held and no sanitizer report. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int elsa_oracle_attn_rows(const float *, const float *, const float *, int, int, int, int, double, int, const int32_t *,
                          const int64_t *, int64_t, double *);
int elsa_oracle_fold_rows(const float *, const float *, const float *, int, int, int, int, double, int, const int32_t *,
                          const int64_t *, int64_t, double *);
int elsa_oracle_lse_rows(const float *, const float *, int, int, int, int, double, int, const int32_t *, const int64_t *,
                         int64_t, double *);
int elsa_oracle_partials_rows(const float *, const float *, const float *, int, int, int, int, double, int,
                              const int32_t *, int, const int64_t *, int64_t, double *, double *, double *);
void elsa_oracle_merge_case(double, double, const double *, double, double, const double *, int, double *, double *, double *);
void elsa_oracle_merge_unsum(double, double, const double *, double, double, const double *, int, double *, double *, double *);
int elsa_oracle_combine_rows(const double *, const double *, const double *, int64_t, int, int, double *);
int elsa_oracle_cross_rows(const float *, const float *, const float *, int, int, int, int, int, double, int,
                           const int32_t *, const int64_t *, int64_t, double *, double *);
int elsa_oracle_dv_rows(const float *, const float *, const float *, int, int, int, int, int, int, double, int,
                        const int32_t *, const int64_t *, int64_t, double *, double *);
int elsa_ladder_f32_fold_rows(const float *, const float *, const float *, int, int, int, int, float, int,
                              const int32_t *, const int64_t *, int64_t, float *);

static int fails = 0;
#define CHECK(cond)                                                     \
    do {                                                                \
        if (!(cond)) {                                                  \
            printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #cond);     \
            ++fails;                                                    \
        }                                                               \
    } while (0)

/* small deterministic numbers in (-1, 1) */
static uint64_t rng = 0x2545F4914F6CDD1DULL;
static float draw(void)
{
    rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
    return (float)((double)(rng >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *fill(size_t count)
{
    float *p = (float *)malloc(sizeof(float) * (count ? count : 1));
    for (size_t i = 0; i < count; ++i) p[i] = draw();
    return p;
}
static int close_to(double a, double b) { return fabs(a - b) <= 1e-11 * (1.0 + fabs(b)); }

static void square_case(int B, int H, int n, int d, int causal, const int32_t *kv_len, int C)
{
    size_t cnt = (size_t)B * H * n * d;
    int64_t R = (int64_t)B * H * n;
    float *q = fill(cnt), *k = fill(cnt), *v = fill(cnt);
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)R);
    for (int64_t r = 0; r < R; ++r) rows[r] = R - 1 - r;          /* any order */
    double *a = (double *)malloc(sizeof(double) * (size_t)R * d), *f = (double *)malloc(sizeof(double) * (size_t)R * d);
    double *c = (double *)malloc(sizeof(double) * (size_t)R * d), *lse = (double *)malloc(sizeof(double) * (size_t)R);
    float *lad = (float *)malloc(sizeof(float) * (size_t)R * d);
    double *pm = (double *)malloc(sizeof(double) * (size_t)R * C), *pS = (double *)malloc(sizeof(double) * (size_t)R * C);
    double *pW = (double *)malloc(sizeof(double) * (size_t)R * C * d);
    CHECK(elsa_oracle_attn_rows(q, k, v, B, H, n, d, 0.37, causal, kv_len, rows, R, a) == 0);
    CHECK(elsa_oracle_fold_rows(q, k, v, B, H, n, d, 0.37, causal, kv_len, rows, R, f) == 0);
    CHECK(elsa_oracle_lse_rows(q, k, B, H, n, d, 0.37, causal, kv_len, rows, R, lse) == 0);
    CHECK(elsa_oracle_partials_rows(q, k, v, B, H, n, d, 0.37, causal, kv_len, C, rows, R, pm, pS, pW) == 0);
    CHECK(elsa_oracle_combine_rows(pm, pS, pW, R, C, d, c) == 0);
    CHECK(elsa_ladder_f32_fold_rows(q, k, v, B, H, n, d, 0.37f, causal, kv_len, rows, R, lad) == 0);
    for (int64_t i = 0; i < R * d; ++i) {
        CHECK(close_to(f[i], a[i]));                               /* Alg. 1 = Eq. 1 */
        CHECK(close_to(c[i], a[i]));                               /* Prop. 1 */
        CHECK(fabs((double)lad[i] - a[i]) <= 1e-4);
    }
    for (int64_t r = 0; r < R; ++r) {                              /* lse = merged m + ln S of the chunk states */
        double m = -INFINITY, S = 0.0;
        for (int cc = 0; cc < C; ++cc) if (pm[r * C + cc] > m) m = pm[r * C + cc];
        for (int cc = 0; cc < C; ++cc) if (pS[r * C + cc] > 0.0) S += pS[r * C + cc] * exp(pm[r * C + cc] - m);
        if (S > 0.0) CHECK(close_to(m + log(S), lse[r])); else CHECK(lse[r] == -INFINITY);
    }
    free(q); free(k); free(v); free(rows); free(a); free(f); free(c); free(lse); free(lad); free(pm); free(pS); free(pW);
}

static void rect_case(int B, int H, int nq, int nk, int d, int dv, int causal, const int32_t *kv_len)
{
    float *q = fill((size_t)B * H * nq * d), *k = fill((size_t)B * H * nk * d);
    float *v = fill((size_t)B * H * nk * d), *vw = fill((size_t)B * H * nk * dv);
    int64_t R = (int64_t)B * H * nq;
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)R);
    for (int64_t r = 0; r < R; ++r) rows[r] = r;
    double *o = (double *)malloc(sizeof(double) * (size_t)R * d), *l = (double *)malloc(sizeof(double) * (size_t)R);
    double *ow = (double *)malloc(sizeof(double) * (size_t)R * dv), *lw = (double *)malloc(sizeof(double) * (size_t)R);
    CHECK(elsa_oracle_cross_rows(q, k, v, B, H, nq, nk, d, 0.41, causal, kv_len, rows, R, o, l) == 0);
    CHECK(elsa_oracle_cross_rows(q, k, v, B, H, nq, nk, d, 0.41, causal, kv_len, rows, R, o, NULL) == 0);
    CHECK(elsa_oracle_dv_rows(q, k, vw, B, H, nq, nk, d, dv, 0.41, causal, kv_len, rows, R, ow, lw) == 0);
    for (int64_t r = 0; r < R; ++r) CHECK((l[r] == lw[r]) || close_to(l[r], lw[r]));   /* same scores, same normaliser */
    if (nq == nk) {                                                /* square: the rectangular routine is the square one */
        double *a = (double *)malloc(sizeof(double) * (size_t)R * d);
        CHECK(elsa_oracle_attn_rows(q, k, v, B, H, nq, d, 0.41, causal, kv_len, rows, R, a) == 0);
        for (int64_t i = 0; i < R * d; ++i) CHECK(close_to(o[i], a[i]));
        free(a);
    }
    free(q); free(k); free(v); free(vw); free(rows); free(o); free(l); free(ow); free(lw);
}

int main(void)
{
    /* closed forms: one key -> its value row; q = 0 -> column mean */
    {
        float q[2] = {0.3f, -0.7f}, k[2] = {1.5f, 2.5f}, v[2] = {4.0f, -9.0f};
        int64_t row = 0;
        double o[2];
        CHECK(elsa_oracle_attn_rows(q, k, v, 1, 1, 1, 2, 0.5, 0, NULL, &row, 1, o) == 0);
        CHECK(o[0] == 4.0 && o[1] == -9.0);
        CHECK(elsa_oracle_fold_rows(q, k, v, 1, 1, 1, 2, 0.5, 1, NULL, &row, 1, o) == 0);
        CHECK(o[0] == 4.0 && o[1] == -9.0);
    }
    {
        float q[3] = {0, 0, 0}, k[9] = {1, 2, 3, 4, 5, 6, 7, 8, 9}, v[9] = {3, 0, 0, 6, 3, 0, 9, 3, 3};
        int64_t rows[3] = {0, 1, 2};
        float qq[9] = {0};
        double o[9];
        (void)q;
        CHECK(elsa_oracle_attn_rows(qq, k, v, 1, 1, 3, 3, 1.0, 0, NULL, rows, 3, o) == 0);
        CHECK(close_to(o[0], 6.0) && close_to(o[1], 2.0) && close_to(o[2], 1.0));
        CHECK(elsa_oracle_attn_rows(qq, k, v, 1, 1, 3, 3, 1.0, 1, NULL, rows, 3, o) == 0);   /* causal: running mean */
        CHECK(close_to(o[0], 3.0) && close_to(o[3], 4.5) && close_to(o[6], 6.0));
    }
    /* merge laws incl. identities */
    {
        double Wa[2] = {2.0, -1.0}, Wb[2] = {0.5, 4.0}, We[2] = {0.0, 0.0}, Wo[2], Wu[2], mo, So, mu, Su;
        elsa_oracle_merge_case(0.3, 1.5, Wa, -INFINITY, 0.0, We, 2, &mo, &So, Wo);
        CHECK(mo == 0.3 && So == 1.5 && Wo[0] == 2.0 && Wo[1] == -1.0);
        elsa_oracle_merge_case(-INFINITY, 0.0, We, -INFINITY, 0.0, We, 2, &mo, &So, Wo);
        CHECK(mo == -INFINITY && So == 0.0 && Wo[0] == 0.0);
        elsa_oracle_merge_case(0.3, 1.5, Wa, 1.1, 2.0, Wb, 2, &mo, &So, Wo);
        elsa_oracle_merge_unsum(0.3, 1.5, Wa, 1.1, 2.0, Wb, 2, &mu, &Su, Wu);
        CHECK(mo == mu && close_to(So, Su) && close_to(Wo[0], Wu[0]) && close_to(Wo[1], Wu[1]));
        CHECK(close_to(So, 2.0 + 1.5 * exp(0.3 - 1.1)));
    }
    {
        int32_t len5[5] = {40, 1, 0, 17, 99};      /* incl. an empty entry and one beyond n (clamped) */
        int32_t len2[2] = {3, 9};
        square_case(1, 1, 1, 4, 0, NULL, 1);
        square_case(2, 3, 33, 8, 0, NULL, 3);
        square_case(2, 3, 33, 8, 1, NULL, 7);
        square_case(5, 1, 40, 4, 0, len5, 3);
        square_case(5, 2, 40, 4, 1, len5, 40);     /* one key per chunk */
        square_case(1, 2, 5, 16, 1, NULL, 9);      /* more chunks than keys: trailing chunks are identities */
        rect_case(2, 2, 5, 23, 8, 3, 0, NULL);
        rect_case(2, 2, 5, 23, 8, 3, 1, len2);
        rect_case(2, 2, 23, 5, 4, 16, 1, NULL);    /* first queries see no key */
        rect_case(1, 3, 11, 11, 8, 8, 1, NULL);
        rect_case(2, 1, 1, 64, 8, 32, 1, len2);
    }
    printf("%s\n", fails ? "oracle under sanitizers: FAILED" : "oracle under sanitizers: ok");
    return fails ? 1 : 0;
}
