/*
 * ELSA oracle -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, single-threaded IEEE FP64 CPU implementation of what the ELSA
 * hot path computes.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP library.
 *
 * Layout everywhere: contiguous row-major [B][H][n][d], d_v == d.  Inputs are
 * float arrays (FP16 experiments pass FP16-representable floats), widened
 * exactly to double before any arithmetic.  A "row" is the flat query index
 * r = (b*H + h)*n + i.
 *
 * Parity pins (tests/test_oracle_*.py): hand-computed closed forms (n = 1,
 * n = 2 sigmoid mixture, q = 0 column mean), a library float64 softmax used as
 * a black box, agreement of the definition with the sequential fold and with
 * arbitrary merge trees, the monoid laws, shift invariance, one-hot dominance,
 * causal-prefix equivalence, key-permutation invariance; the rectangular (n_q != n_k) routine
 * against the library softmax with a rectangular mask, against the square routine on the tail
 * rows of a longer problem, and a hand-computed single-query case.  The paper prints no
 * worked softmax example, so exact output values beyond those closed forms are
 * pinned by these independent formulations only.
 *
 * Readings where the paper is silent:
 *   - a masked key is the identity element (skipped); causal means key j is
 *     visible to query i iff j <= i; key padding means j < kv_len[b];
 *   - a row with no visible key outputs zeros (state stays at the identity,
 *     0/0 := 0);
 *   - a merge whose two maxima are both -inf returns the identity (the case
 *     form of the merge would otherwise evaluate exp(-inf - -inf)).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* number of keys visible to query i of batch b */
static int64_t visible_keys(int64_t i, int64_t n, int causal, const int32_t *kv_len, int64_t b)
{
    int64_t lim = kv_len ? (int64_t)kv_len[b] : n;
    if (lim > n) lim = n;
    if (lim < 0) lim = 0;
    if (causal && i + 1 < lim) lim = i + 1;
    return lim;
}

/* s_j = scale * <q_i, k_j>   (Sec. 3, score definition above Eq. 1) */
static double score(const float *qi, const float *kj, int d, double scale)
{
    double acc = 0.0;
    for (int t = 0; t < d; ++t) acc += (double)qi[t] * (double)kj[t];
    return scale * acc;
}

/*
 * Definition: y_i = sum_j e^{s_ij} v_j / sum_j e^{s_ij}  (Eq. 1), evaluated in
 * the max-subtracted form of the vectorized reference (Eq. 12): m = max_j s,
 * E = exp(s - m), y = (E V) / sum(E).
 * out: [nrows][d] doubles.  Returns 0, or -1 on allocation failure.
 */
int elsa_oracle_attn_rows(const float *q, const float *k, const float *v,
                          int B, int H, int n, int d, double scale, int causal,
                          const int32_t *kv_len,
                          const int64_t *rows, int64_t nrows, double *out)
{
    (void)B;
    double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    if (!s) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % n, bh = row / n, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *kb = k + (size_t)bh * n * d;
        const float *vb = v + (size_t)bh * n * d;
        double *o = out + (size_t)r * d;
        int64_t L = visible_keys(i, n, causal, kv_len, b);
        for (int t = 0; t < d; ++t) o[t] = 0.0;
        if (L <= 0) continue;
        double m = -INFINITY;
        for (int64_t j = 0; j < L; ++j) {
            s[j] = score(qi, kb + (size_t)j * d, d, scale);
            if (s[j] > m) m = s[j];
        }
        double S = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            double e = exp(s[j] - m);
            S += e;
            const float *vj = vb + (size_t)j * d;
            for (int t = 0; t < d; ++t) o[t] += e * (double)vj[t];
        }
        for (int t = 0; t < d; ++t) o[t] /= S;
    }
    free(s);
    return 0;
}

/*
 * Log-normaliser of every sampled row: lse_i = ln sum_j e^{s_ij} = m + ln sum_j e^{s_ij - m}
 * (the row sum s of Eq. 12 with its maximum put back); -inf for a row with no visible key.
 * The attention probabilities of the drift metrics are P_ij = e^{s_ij - lse_i}.
 */
int elsa_oracle_lse_rows(const float *q, const float *k,
                         int B, int H, int n, int d, double scale, int causal,
                         const int32_t *kv_len,
                         const int64_t *rows, int64_t nrows, double *lse)
{
    (void)B;
    double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    if (!s) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % n, bh = row / n, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *kb = k + (size_t)bh * n * d;
        int64_t L = visible_keys(i, n, causal, kv_len, b);
        double m = -INFINITY, S = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            s[j] = score(qi, kb + (size_t)j * d, d, scale);
            if (s[j] > m) m = s[j];
        }
        for (int64_t j = 0; j < L; ++j) S += exp(s[j] - m);
        lse[r] = (L > 0) ? m + log(S) : -INFINITY;
    }
    free(s);
    return 0;
}

/* Eq. 3, declared here for the fold below; defined with the other merge forms further down. */
void elsa_oracle_merge_case(double ma, double Sa, const double *Wa,
                            double mb, double Sb, const double *Wb, int d,
                            double *mo, double *So, double *Wo);

/*
 * Per-query sequential evaluation (Alg. 1) as what it is in the monoid's terms: the running
 * state starts at the identity e = (-inf, 0, 0) and absorbs the keys one at a time,
 *     u <- u (+) (s_j, 1, v_j),
 * each key lifted to its one-element state (Sec. 3.2) and merged with the operator of Eq. 3;
 * the output is W / S of the final state (zeros for a row that saw no key).
 */
int elsa_oracle_fold_rows(const float *q, const float *k, const float *v,
                          int B, int H, int n, int d, double scale, int causal,
                          const int32_t *kv_len,
                          const int64_t *rows, int64_t nrows, double *out)
{
    (void)B;
    size_t dd = (size_t)(d > 0 ? d : 1);
    double *buf = (double *)malloc(sizeof(double) * dd * 3);
    if (!buf) return -1;
    double *Wrun = buf, *Wkey = buf + dd, *Wnext = buf + 2 * dd;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % n, bh = row / n, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *keys = k + (size_t)bh * n * d;
        const float *vals = v + (size_t)bh * n * d;
        int64_t L = visible_keys(i, n, causal, kv_len, b);
        double m_run = -INFINITY, S_run = 0.0;                 /* u = e */
        for (int t = 0; t < d; ++t) Wrun[t] = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            double m_next, S_next;
            for (int t = 0; t < d; ++t) Wkey[t] = (double)vals[(size_t)j * d + t];
            elsa_oracle_merge_case(m_run, S_run, Wrun,
                                   score(qi, keys + (size_t)j * d, d, scale), 1.0, Wkey, d,
                                   &m_next, &S_next, Wnext);
            m_run = m_next; S_run = S_next;
            memcpy(Wrun, Wnext, sizeof(double) * (size_t)d);
        }
        for (int t = 0; t < d; ++t) out[(size_t)r * d + t] = (S_run > 0.0) ? Wrun[t] / S_run : 0.0;
    }
    free(buf);
    return 0;
}

/*
 * Block states for Prop. 1 / the split-KV contract.  Chunk c of C covers keys
 * [c*ceil(n/C), min(n, (c+1)*ceil(n/C))).  For each sampled row and chunk the
 * state over the *visible* keys of that chunk is
 *   m_c = max s_j,  S_c = sum e^{s_j - m_c},  W_c = sum e^{s_j - m_c} v_j
 * (the normalized state of Sec. 3.2), or the identity (-inf, 0, 0) when no key
 * of the chunk is visible.
 * part_m, part_S: [nrows][C]; part_W: [nrows][C][d].
 */
int elsa_oracle_partials_rows(const float *q, const float *k, const float *v,
                              int B, int H, int n, int d, double scale, int causal,
                              const int32_t *kv_len, int num_splits,
                              const int64_t *rows, int64_t nrows,
                              double *part_m, double *part_S, double *part_W)
{
    (void)B;
    int C = num_splits;
    int64_t chunk = ((int64_t)n + C - 1) / C;
    double *s = (double *)malloc(sizeof(double) * (size_t)(chunk > 0 ? chunk : 1));
    if (!s) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % n, bh = row / n, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *kb = k + (size_t)bh * n * d;
        const float *vb = v + (size_t)bh * n * d;
        int64_t L = visible_keys(i, n, causal, kv_len, b);
        for (int c = 0; c < C; ++c) {
            int64_t lo = (int64_t)c * chunk, hi = lo + chunk;
            if (hi > L) hi = L;
            double *Wc = part_W + ((size_t)r * C + c) * d;
            double m = -INFINITY, S = 0.0;
            for (int t = 0; t < d; ++t) Wc[t] = 0.0;
            for (int64_t j = lo; j < hi; ++j) {
                s[j - lo] = score(qi, kb + (size_t)j * d, d, scale);
                if (s[j - lo] > m) m = s[j - lo];
            }
            for (int64_t j = lo; j < hi; ++j) {
                double e = exp(s[j - lo] - m);
                S += e;
                const float *vj = vb + (size_t)j * d;
                for (int t = 0; t < d; ++t) Wc[t] += e * (double)vj[t];
            }
            part_m[(size_t)r * C + c] = m;
            part_S[(size_t)r * C + c] = S;
        }
    }
    free(s);
    return 0;
}

/*
 * Merge operator, case form (Eq. 3): keep the larger maximum, scale the other
 * operand by exp(m_small - m_large) <= 1.  Both maxima -inf -> identity.
 * Wa, Wb, Wo: d doubles.  Wo may alias neither input.
 */
void elsa_oracle_merge_case(double ma, double Sa, const double *Wa,
                            double mb, double Sb, const double *Wb, int d,
                            double *mo, double *So, double *Wo)
{
    if (ma == -INFINITY && mb == -INFINITY) {
        *mo = -INFINITY; *So = 0.0;
        for (int t = 0; t < d; ++t) Wo[t] = 0.0;
        return;
    }
    if (ma >= mb) {
        double f = exp(mb - ma);
        *mo = ma; *So = Sa + Sb * f;
        for (int t = 0; t < d; ++t) Wo[t] = Wa[t] + Wb[t] * f;
    } else {
        double f = exp(ma - mb);
        *mo = mb; *So = Sb + Sa * f;
        for (int t = 0; t < d; ++t) Wo[t] = Wb[t] + Wa[t] * f;
    }
}

/*
 * Merge operator, compact form (Eq. 4): renorm(max(ma, mb), un(a) + un(b)) with
 * un(m,S,W) = (S e^m, W e^m) and renorm(m,S~,W~) = (m, S~ e^-m, W~ e^-m).
 * Literal: overflows for |m| beyond ~700, so tests keep m moderate.
 */
void elsa_oracle_merge_unsum(double ma, double Sa, const double *Wa,
                             double mb, double Sb, const double *Wb, int d,
                             double *mo, double *So, double *Wo)
{
    double m = ma > mb ? ma : mb;
    if (m == -INFINITY) {
        *mo = m; *So = 0.0;
        for (int t = 0; t < d; ++t) Wo[t] = 0.0;
        return;
    }
    double ea = exp(ma), eb = exp(mb), em = exp(-m);
    *mo = m;
    *So = (Sa * ea + Sb * eb) * em;
    for (int t = 0; t < d; ++t) Wo[t] = (Wa[t] * ea + Wb[t] * eb) * em;
}

/*
 * Combine (Prop. 1): left-to-right merge of C chunk states per row with the
 * case-form operator, then y = W / S; all-identity rows give zeros.
 * part_m, part_S: [nrows][C]; part_W: [nrows][C][d]; out: [nrows][d].
 */
int elsa_oracle_combine_rows(const double *part_m, const double *part_S, const double *part_W,
                             int64_t nrows, int C, int d, double *out)
{
    double *Wa = (double *)malloc(sizeof(double) * (size_t)(d > 0 ? d : 1) * 2);
    if (!Wa) return -1;
    double *Wt = Wa + d;
    for (int64_t r = 0; r < nrows; ++r) {
        double m = -INFINITY, S = 0.0;
        for (int t = 0; t < d; ++t) Wa[t] = 0.0;
        for (int c = 0; c < C; ++c) {
            double mo, So;
            elsa_oracle_merge_case(m, S, Wa, part_m[(size_t)r * C + c], part_S[(size_t)r * C + c],
                                   part_W + ((size_t)r * C + c) * d, d, &mo, &So, Wt);
            m = mo; S = So;
            memcpy(Wa, Wt, sizeof(double) * (size_t)d);
        }
        for (int t = 0; t < d; ++t) out[(size_t)r * d + t] = (S > 0.0) ? Wa[t] / S : 0.0;
    }
    free(Wa);
    return 0;
}

/*
 * Rectangular attention: n_q queries against n_k keys per (batch, head) -- cross-attention,
 * chunked prefill, and single-query decoding against a cache.  Eq. 1 does not tie the number of
 * queries to the number of keys; the row formula is the same.  q, out: [B][H][n_q][d];
 * k, v: [B][H][n_k][d]; a row is r = (b*H + h)*n_q + i.
 * Reading for the causal mask (the paper states it for n_q = n_k only): the LAST query is
 * aligned with the LAST key, i.e. key j is visible to query i iff j <= i + (n_k - n_q); queries
 * with no visible key (possible when n_k < n_q) output zeros and lse = -inf.
 * out: [nrows][d]; lse: [nrows] or NULL.
 */
int elsa_oracle_cross_rows(const float *q, const float *k, const float *v,
                           int B, int H, int nq, int nk, int d, double scale, int causal,
                           const int32_t *kv_len,
                           const int64_t *rows, int64_t nrows, double *out, double *lse)
{
    (void)B;
    double *s = (double *)malloc(sizeof(double) * (size_t)(nk > 0 ? nk : 1));
    if (!s) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % nq, bh = row / nq, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *kb = k + (size_t)bh * nk * d;
        const float *vb = v + (size_t)bh * nk * d;
        double *o = out + (size_t)r * d;
        int64_t L = kv_len ? (int64_t)kv_len[b] : nk;
        if (L > nk) L = nk;
        if (causal) {
            int64_t last = i + ((int64_t)nk - (int64_t)nq);     /* last visible key */
            if (last + 1 < L) L = last + 1;
        }
        if (L < 0) L = 0;
        for (int t = 0; t < d; ++t) o[t] = 0.0;
        if (lse) lse[r] = -INFINITY;
        if (L == 0) continue;
        double m = -INFINITY;
        for (int64_t j = 0; j < L; ++j) {
            s[j] = score(qi, kb + (size_t)j * d, d, scale);
            if (s[j] > m) m = s[j];
        }
        double S = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            double e = exp(s[j] - m);
            S += e;
            const float *vj = vb + (size_t)j * d;
            for (int t = 0; t < d; ++t) o[t] += e * (double)vj[t];
        }
        for (int t = 0; t < d; ++t) o[t] /= S;
        if (lse) lse[r] = m + log(S);
    }
    free(s);
    return 0;
}

/*
 * Attention with value rows of their own width d_v (the paper's setting V in R^{n x d_v},
 * Sec. "Problem setup"; the state's W lives in R^{d_v}): scores use the d columns of q and k,
 * the weighted sum runs over the d_v columns of v.  Written out as the definition, one row at a
 * time:  y_i = sum_j softmax_j(scale q_i.k_j) v_j  over the visible keys.
 * q: [B][H][n_q][d]; k: [B][H][n_k][d]; v: [B][H][n_k][d_v]; masks as for the rectangular routine
 * above (causal: key j visible to query i iff j <= i + (n_k - n_q); kv_len per batch entry).
 * out: [nrows][d_v]; lse: [nrows] or NULL.
 */
int elsa_oracle_dv_rows(const float *q, const float *k, const float *v,
                        int B, int H, int nq, int nk, int d, int dv, double scale, int causal,
                        const int32_t *kv_len,
                        const int64_t *rows, int64_t nrows, double *out, double *lse)
{
    (void)B;
    double *w = (double *)malloc(sizeof(double) * (size_t)(nk > 0 ? nk : 1));
    if (!w) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % nq, bh = row / nq, b = bh / H;
        const float *qrow = q + (size_t)row * d;
        const float *keys = k + (size_t)bh * nk * d;
        const float *vals = v + (size_t)bh * nk * dv;
        double *y = out + (size_t)r * dv;
        int64_t vis = kv_len ? (int64_t)kv_len[b] : nk;          /* number of visible keys */
        if (vis > nk) vis = nk;
        if (causal) {
            int64_t diag = i + ((int64_t)nk - (int64_t)nq) + 1;  /* keys 0 .. diag-1 */
            if (diag < vis) vis = diag;
        }
        if (vis < 0) vis = 0;
        for (int c = 0; c < dv; ++c) y[c] = 0.0;
        if (lse) lse[r] = -INFINITY;
        if (vis == 0) continue;
        double top = -INFINITY;
        for (int64_t j = 0; j < vis; ++j) {
            w[j] = score(qrow, keys + (size_t)j * d, d, scale);
            if (w[j] > top) top = w[j];
        }
        double Z = 0.0;
        for (int64_t j = 0; j < vis; ++j) {
            w[j] = exp(w[j] - top);
            Z += w[j];
        }
        for (int c = 0; c < dv; ++c) {
            double acc = 0.0;
            for (int64_t j = 0; j < vis; ++j) acc += w[j] * (double)vals[(size_t)j * dv + c];
            y[c] = acc / Z;
        }
        if (lse) lse[r] = top + log(Z);
    }
    free(w);
    return 0;
}

/*
 * FP32 ladder (diagnostic only): the same key-by-key absorption u <- u (+) (s_j, 1, v_j) of
 * Alg. 1 with every product, sum and exponential in IEEE single precision.  It shows what error
 * any FP32-accumulating evaluation carries on a given input, so that a tolerance violation can be
 * attributed to the conditioning of the metric rather than to a kernel defect.
 * out: [nrows][d] floats.
 */
static float f32_mul(float a, float b) { volatile float p = a * b; return p; }   /* volatile: one rounding, no contraction */
static float f32_add(float a, float b) { volatile float p = a + b; return p; }

/* Eq. 3 in single precision, in place on the running state (m, S, W); the other operand is (mk, Sk, Wk). */
static void merge_case_f32(float *m, float *S, float *W, float mk, float Sk, const float *Wk, int d)
{
    if (*m == -INFINITY && mk == -INFINITY) return;            /* e (+) e = e */
    if (*m >= mk) {
        float f = expf(mk - *m);
        *S = f32_add(*S, f32_mul(Sk, f));
        for (int t = 0; t < d; ++t) W[t] = f32_add(W[t], f32_mul(Wk[t], f));
    } else {
        float f = expf(*m - mk);
        *S = f32_add(Sk, f32_mul(*S, f));
        for (int t = 0; t < d; ++t) W[t] = f32_add(Wk[t], f32_mul(W[t], f));
        *m = mk;
    }
}

int elsa_ladder_f32_fold_rows(const float *q, const float *k, const float *v,
                              int B, int H, int n, int d, float scale, int causal,
                              const int32_t *kv_len,
                              const int64_t *rows, int64_t nrows, float *out)
{
    (void)B;
    float *W = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    if (!W) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % n, bh = row / n, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *keys = k + (size_t)bh * n * d;
        const float *vals = v + (size_t)bh * n * d;
        int64_t L = visible_keys(i, n, causal, kv_len, b);
        float m = -INFINITY, S = 0.0f;
        for (int t = 0; t < d; ++t) W[t] = 0.0f;
        for (int64_t j = 0; j < L; ++j) {
            float dot = 0.0f;
            for (int t = 0; t < d; ++t) dot = f32_add(dot, f32_mul(qi[t], keys[(size_t)j * d + t]));
            merge_case_f32(&m, &S, W, f32_mul(scale, dot), 1.0f, vals + (size_t)j * d, d);
        }
        for (int t = 0; t < d; ++t) out[(size_t)r * d + t] = (L > 0) ? W[t] / S : 0.0f;
    }
    free(W);
    return 0;
}

/*
 * Round a double to the nearest IEEE binary16 value, ties to even (11 significant bits, exponents
 * 2^-14 .. 2^15, gradual underflow with spacing 2^-24, overflow to infinity), returned as a double.
 */
double elsa_oracle_round_f16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(fabs(x), &e);                 /* |x| = f * 2^e, f in [0.5, 1)  ->  |x| in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - 10;               /* spacing of halves in that binade */
    if (ulp_exp < -24) ulp_exp = -24;         /* below 2^-14: fixed spacing 2^-24 */
    double r = ldexp(nearbyint(ldexp(x, -ulp_exp)), ulp_exp);   /* nearbyint: ties to even in the default mode */
    if (fabs(r) > 65504.0) return x > 0 ? INFINITY : -INFINITY;
    return r;
}

/*
 * FP16-operand ladder (diagnostic only): what the FP16 variant must incur by its own definition.
 * The definition (Eq. 1, max-subtracted) in FP64, except that -- as in the FP16 I/O variant with FP32
 * state -- every weight e^{s_j - m} is rounded to binary16 where it multiplies v_j (the normaliser sums
 * the unrounded weights) and the output is rounded to binary16.  Used to tell which violations of an
 * elementwise tolerance belong to the FP16 operand format rather than to a kernel.
 * out: [nrows][d] doubles holding binary16 values.
 */
int elsa_ladder_f16_rows(const float *q, const float *k, const float *v,
                         int B, int H, int n, int d, double scale, int causal,
                         const int32_t *kv_len,
                         const int64_t *rows, int64_t nrows, double *out)
{
    (void)B;
    double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    if (!s) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t row = rows[r];
        int64_t i = row % n, bh = row / n, b = bh / H;
        const float *qi = q + (size_t)row * d;
        const float *keys = k + (size_t)bh * n * d;
        const float *vals = v + (size_t)bh * n * d;
        double *y = out + (size_t)r * d;
        int64_t L = visible_keys(i, n, causal, kv_len, b);
        for (int t = 0; t < d; ++t) y[t] = 0.0;
        if (L <= 0) continue;
        double top = -INFINITY, Z = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            s[j] = score(qi, keys + (size_t)j * d, d, scale);
            if (s[j] > top) top = s[j];
        }
        for (int64_t j = 0; j < L; ++j) {
            double w = exp(s[j] - top);
            double wh = elsa_oracle_round_f16(w);
            Z += w;
            for (int t = 0; t < d; ++t) y[t] += wh * (double)vals[(size_t)j * d + t];
        }
        for (int t = 0; t < d; ++t) y[t] = elsa_oracle_round_f16(y[t] / Z);
    }
    free(s);
    return 0;
}
