/*
 * CPU oracle for LOOKAT (product-quantised key cache + ADC attention decode).
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and
 * the benchmark's cpu-baseline leg may load this file.  It shares no code with the
 * HIP library: every routine below is a plain loop that follows the paper's
 * definition of the step, in the paper's order, with fp64 arithmetic.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 *        (-ffp-contract=off matters: the encoder's distance is defined with a
 *        separately rounded subtract, multiply and add for every coordinate).
 *
 * Notation (paper, Sec. 3.4 / 3.5 / Algorithm 1):
 *   d_k   head dimension            m      number of subspaces
 *   d_sub = d_k / m                 K      centroids per subspace (paper: 256)
 *   C_i   codebook of subspace i,   C_i[c] is a d_sub vector
 *   k~_l  the m codes of cached key l,  LUT_i[c] = q^(i) . C_i[c]
 *
 * Array layouts (row-major, last index fastest):
 *   keys      [B,H,N,d_k]      fp32, or fp16 passed as raw uint16 bit patterns
 *   codebooks [H,m,K,d_sub]    fp32   (one set per head)
 *   codes     [B,H,N,m]        uint8
 *   q         [B,H,T,d_k]      fp32 or fp16 bits
 *   lut       [B,H,T,m,K]      fp32
 *   values    [B,H,L,d_k]      fp16 bits
 *   out       [B,H,d_k]        fp32
 *
 * Pinned by tests/test_oracle_pins.py (ADC identity, zero-distortion case equal to
 * dense attention, brute-force argmin, forced ties, softmax row sums, convex hull,
 * closed-form hand examples, Lloyd monotonicity).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F16 1
#define ORACLE_F32 2

/* IEEE binary16 bit pattern -> double, exactly. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* zero and subnormals */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac + 1024), expo - 25);
    }
    return sign ? -v : v;
}

static double load_as_double(const void *p, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F16)
        return half_bits_to_double(((const uint16_t *)p)[idx]);
    return (double)((const float *)p)[idx];
}

/* Squared distance of the encoder (Sec. 3.4, "Encoding"): coordinates taken in
 * ascending order, each subtract / multiply / add rounded once in fp64. */
static double sq_dist(const double *x, const float *y, int d_sub)
{
    double acc = 0.0;
    for (int j = 0; j < d_sub; ++j) {
        double diff = x[j] - (double)y[j];
        double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

/* Nearest centroid with a strict '<' scan over c ascending: among equal
 * distances the lowest index wins; a NaN distance never wins. */
static int nearest_centroid(const double *x, const float *cb, int K, int d_sub, double *best_d)
{
    int best = 0;
    double bd = sq_dist(x, cb, d_sub);
    for (int c = 1; c < K; ++c) {
        double d = sq_dist(x, cb + (int64_t)c * d_sub, d_sub);
        if (d < bd) {
            bd = d;
            best = c;
        }
    }
    if (best_d)
        *best_d = bd;
    return best;
}

/* Sec. 3.4 "Encoding": codes[b,h,n,i] = argmin_c || k^(i) - C_i[c] ||^2 . */
int oracle_encode_keys(int B, int H, int64_t N, int d_k, int m, int K,
                       const void *keys, int key_dtype,
                       const float *codebooks, uint8_t *codes)
{
    if (m <= 0 || d_k % m || K <= 0 || K > 256)
        return -2;
    int d_sub = d_k / m;
    int64_t BH = (int64_t)B * H;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        int h = (int)(bh % H);
        double *x = (double *)malloc(sizeof(double) * (size_t)d_sub);
        for (int64_t n = 0; n < N; ++n) {
            for (int i = 0; i < m; ++i) {
                int64_t base = (bh * N + n) * d_k + (int64_t)i * d_sub;
                for (int j = 0; j < d_sub; ++j)
                    x[j] = load_as_double(keys, key_dtype, base + j);
                const float *cb = codebooks + ((int64_t)h * m + i) * K * d_sub;
                codes[(bh * N + n) * m + i] = (uint8_t)nearest_centroid(x, cb, K, d_sub, NULL);
            }
        }
        free(x);
    }
    return 0;
}

/* Sec. 3.5 "Precomputation Lookup Tables" / Algorithm 1, first loop:
 * LUT_i[c] = sum_j q[i*d_sub + j] * C_i[c][j], fp64 sum in ascending j,
 * rounded once to fp32 (the table is an interface value). */
int oracle_build_lut(int B, int H, int T, int d_k, int m, int K,
                     const void *q, int q_dtype,
                     const float *codebooks, float *lut)
{
    if (m <= 0 || d_k % m || K <= 0)
        return -2;
    int d_sub = d_k / m;
    int64_t BH = (int64_t)B * H;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        int h = (int)(bh % H);
        for (int t = 0; t < T; ++t) {
            int64_t qbase = (bh * T + t) * d_k;
            for (int i = 0; i < m; ++i) {
                const float *cb = codebooks + ((int64_t)h * m + i) * K * d_sub;
                for (int c = 0; c < K; ++c) {
                    double acc = 0.0;
                    for (int j = 0; j < d_sub; ++j) {
                        double qv = load_as_double(q, q_dtype, qbase + (int64_t)i * d_sub + j);
                        acc = acc + qv * (double)cb[(int64_t)c * d_sub + j];
                    }
                    lut[(((bh * T + t) * m) + i) * K + c] = (float)acc;
                }
            }
        }
    }
    return 0;
}

/* Sec. 3.5 "Lookup and Sum" / Algorithm 1, second loop:
 * s_l = sum_i LUT_i[ k~_l[i] ], i ascending, fp64 sum of the fp32 table entries. */
static double adc_score(const float *lut, const uint8_t *code, int m, int K)
{
    double s = 0.0;
    for (int i = 0; i < m; ++i)
        s = s + (double)lut[(int64_t)i * K + code[i]];
    return s;
}

/* Scores only: scores[b,h,l] (fp32, unscaled). lut is [B,H,m,K] (T = 1). */
int oracle_adc_scores(int B, int H, int64_t L, int m, int K,
                      const float *lut, const uint8_t *codes, float *scores)
{
    int64_t BH = (int64_t)B * H;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        const float *t = lut + bh * m * K;
        for (int64_t l = 0; l < L; ++l)
            scores[bh * L + l] = (float)adc_score(t, codes + (bh * L + l) * m, m, K);
    }
    return 0;
}

/* Algorithm 1, "standard attention continuation":
 *   alpha = softmax(scale * s)   (the algorithm's scale is 1/sqrt(d_k)),
 *   o     = sum_l alpha_l v_l.
 * Optional outputs (may be NULL): scores [B,H,L] fp32 unscaled, alpha [B,H,L] fp64. */
int oracle_attend_decode(int B, int H, int64_t L, int d_k, int m, int K,
                         const float *lut, const uint8_t *codes,
                         const uint16_t *values, double scale,
                         float *out, float *scores_out, double *alpha_out)
{
    if (L <= 0)
        return -2;
    int64_t BH = (int64_t)B * H;
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        const float *t = lut + bh * m * K;
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *o = (double *)malloc(sizeof(double) * (size_t)d_k);
        if (!s || !o) {
            rc = -8;
            free(s);
            free(o);
            continue;
        }
        for (int64_t l = 0; l < L; ++l) {
            double raw = adc_score(t, codes + (bh * L + l) * m, m, K);
            if (scores_out)
                scores_out[bh * L + l] = (float)raw;
            s[l] = scale * raw;
        }
        double mx = s[0];
        for (int64_t l = 1; l < L; ++l)
            if (s[l] > mx)
                mx = s[l];
        double z = 0.0;
        for (int64_t l = 0; l < L; ++l) {
            s[l] = exp(s[l] - mx);
            z = z + s[l];
        }
        for (int j = 0; j < d_k; ++j)
            o[j] = 0.0;
        for (int64_t l = 0; l < L; ++l) {
            double a = s[l] / z;
            if (alpha_out)
                alpha_out[bh * L + l] = a;
            const uint16_t *v = values + (bh * L + l) * d_k;
            for (int j = 0; j < d_k; ++j)
                o[j] = o[j] + a * half_bits_to_double(v[j]);
        }
        for (int j = 0; j < d_k; ++j)
            out[bh * d_k + j] = (float)o[j];
        free(s);
        free(o);
    }
    return rc;
}

/* Grouped queries (the paper's "Future Work": LOOKAT combined with grouped-query attention;
 * key/value sharing across heads: "Structural Approaches").  `group` consecutive query heads share
 * one key/value head; per query head hq the computation is Algorithm 1 unchanged, with the codes
 * and values of key/value head hq / group:
 *   lut [B, H*group, m, K], codes [B, H, L, m], values [B, H, L, d_k]  ->  out [B, H*group, d_k],
 *   scores_out [B, H*group, L] (may be NULL). */
int oracle_attend_decode_gqa(int B, int H, int group, int64_t L, int d_k, int m, int K,
                             const float *lut, const uint8_t *codes,
                             const uint16_t *values, double scale,
                             float *out, float *scores_out)
{
    if (L <= 0 || group <= 0)
        return -2;
    int HQ = H * group;
    int64_t BHQ = (int64_t)B * HQ;
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int64_t bq = 0; bq < BHQ; ++bq) {
        int64_t b = bq / HQ;
        int hq = (int)(bq % HQ);
        int64_t kv = b * H + hq / group;            /* the key/value head this query head reads */
        const float *t = lut + bq * m * K;
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *o = (double *)malloc(sizeof(double) * (size_t)d_k);
        if (!s || !o) {
            rc = -8;
            free(s);
            free(o);
            continue;
        }
        for (int64_t l = 0; l < L; ++l) {
            double raw = adc_score(t, codes + (kv * L + l) * m, m, K);
            if (scores_out)
                scores_out[bq * L + l] = (float)raw;
            s[l] = scale * raw;
        }
        double mx = s[0];
        for (int64_t l = 1; l < L; ++l)
            if (s[l] > mx)
                mx = s[l];
        double z = 0.0;
        for (int64_t l = 0; l < L; ++l) {
            s[l] = exp(s[l] - mx);
            z = z + s[l];
        }
        for (int j = 0; j < d_k; ++j)
            o[j] = 0.0;
        for (int64_t l = 0; l < L; ++l) {
            double a = s[l] / z;
            const uint16_t *v = values + (kv * L + l) * d_k;
            for (int j = 0; j < d_k; ++j)
                o[j] = o[j] + a * half_bits_to_double(v[j]);
        }
        for (int j = 0; j < d_k; ++j)
            out[bq * d_k + j] = (float)o[j];
        free(s);
        free(o);
    }
    return rc;
}


/* Prefill form of the lookup-and-sum: the T queries of a block are the last T positions
 * of a cache of L >= T keys, so query t sits at position t + (L - T) and scores the keys
 * l <= t + (L - T) (causal, self included; for L == T: l <= t).  Entries it may not see are
 * written as -inf.  lut is [B,H,T,m,K]; scores [B,H,T,L] fp32 unscaled. */
int oracle_score_prefill(int B, int H, int T, int64_t L, int m, int K,
                         const float *lut, const uint8_t *codes, float *scores)
{
    int64_t BH = (int64_t)B * H;
    if (L < T)
        return -2;
    const int64_t off = L - T;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        for (int t = 0; t < T; ++t) {
            const float *tab = lut + (bh * T + t) * m * K;
            for (int64_t l = 0; l < L; ++l) {
                float v;
                if (l <= t + off)
                    v = (float)adc_score(tab, codes + (bh * L + l) * m, m, K);
                else
                    v = -INFINITY;
                scores[(bh * T + t) * L + l] = v;
            }
        }
    }
    return 0;
}

/* ---- helpers used only to pin the routines above ------------------------- */

/* k^_l = [ C_1[c_1], ..., C_m[c_m] ]  (the vector the codes stand for). */
int oracle_decode_codes(int B, int H, int64_t N, int d_k, int m, int K,
                        const uint8_t *codes, const float *codebooks, float *keys_hat)
{
    int d_sub = d_k / m;
    int64_t BH = (int64_t)B * H;
    for (int64_t bh = 0; bh < BH; ++bh) {
        int h = (int)(bh % H);
        for (int64_t n = 0; n < N; ++n)
            for (int i = 0; i < m; ++i) {
                int c = codes[(bh * N + n) * m + i];
                const float *cb = codebooks + (((int64_t)h * m + i) * K + c) * d_sub;
                memcpy(keys_hat + (bh * N + n) * d_k + (int64_t)i * d_sub, cb, sizeof(float) * (size_t)d_sub);
            }
    }
    return 0;
}

/* Dense attention of Sec. 3.1 for one query per (b,h):
 * softmax(scale * q K^T) V with fp32 keys, fp16 values, all in fp64. */
int oracle_dense_attention(int B, int H, int64_t L, int d_k,
                           const void *q, int q_dtype, const float *keys,
                           const uint16_t *values, double scale, float *out)
{
    int64_t BH = (int64_t)B * H;
    for (int64_t bh = 0; bh < BH; ++bh) {
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double mx = -INFINITY;
        for (int64_t l = 0; l < L; ++l) {
            double acc = 0.0;
            for (int j = 0; j < d_k; ++j)
                acc += load_as_double(q, q_dtype, bh * d_k + j) * (double)keys[(bh * L + l) * d_k + j];
            s[l] = scale * acc;
            if (s[l] > mx)
                mx = s[l];
        }
        double z = 0.0;
        for (int64_t l = 0; l < L; ++l) {
            s[l] = exp(s[l] - mx);
            z += s[l];
        }
        for (int j = 0; j < d_k; ++j) {
            double o = 0.0;
            for (int64_t l = 0; l < L; ++l)
                o += s[l] / z * half_bits_to_double(values[(bh * L + l) * d_k + j]);
            out[bh * d_k + j] = (float)o;
        }
        free(s);
    }
    return 0;
}

/* One Lloyd iteration of Sec. 3.4 "Prototype Learning" on calibration keys
 * calib [H,Nc,d_k] fp32: assign every sub-vector to its nearest centroid (same
 * rule as the encoder), then move each centroid to the fp64 mean of its members
 * (summed in ascending key order, rounded to fp32); a centroid without members
 * stays where it was.  objective[h*m+i] receives the sum of squared distances of
 * the assignment step, i.e. the k-means objective of the INPUT codebooks. */
int oracle_kmeans_step(int H, int64_t Nc, int d_k, int m, int K,
                       const float *calib, const float *cb_in, float *cb_out,
                       double *objective)
{
    if (m <= 0 || d_k % m || K <= 0 || K > 256)
        return -2;
    int d_sub = d_k / m;
    int64_t HM = (int64_t)H * m;
#pragma omp parallel for schedule(dynamic)
    for (int64_t hm = 0; hm < HM; ++hm) {
        int h = (int)(hm / m), i = (int)(hm % m);
        const float *cb = cb_in + hm * K * d_sub;
        double *sum = (double *)calloc((size_t)K * d_sub, sizeof(double));
        int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
        double *x = (double *)malloc(sizeof(double) * (size_t)d_sub);
        double obj = 0.0;
        for (int64_t n = 0; n < Nc; ++n) {
            const float *kv = calib + ((int64_t)h * Nc + n) * d_k + (int64_t)i * d_sub;
            for (int j = 0; j < d_sub; ++j)
                x[j] = (double)kv[j];
            double bd;
            int c = nearest_centroid(x, cb, K, d_sub, &bd);
            obj += bd;
            cnt[c] += 1;
            for (int j = 0; j < d_sub; ++j)
                sum[(int64_t)c * d_sub + j] += x[j];
        }
        for (int c = 0; c < K; ++c)
            for (int j = 0; j < d_sub; ++j) {
                int64_t o = hm * K * d_sub + (int64_t)c * d_sub + j;
                cb_out[o] = cnt[c] ? (float)(sum[(int64_t)c * d_sub + j] / (double)cnt[c]) : cb[(int64_t)c * d_sub + j];
            }
        if (objective)
            objective[hm] = obj;
        free(sum);
        free(cnt);
        free(x);
    }
    return 0;
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
