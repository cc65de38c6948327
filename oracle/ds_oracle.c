/*
 * ds_oracle.c -- plain CPU oracle for Double Sparsity decode attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the decode step computes, written from the paper (Algorithm 1, the
 * dense formula of Sec. 2.1, the label cache of Sec. 4.2 and the calibration of
 * Sec. 4.1).  Only the tests, the smoke check and the bench's cpu_baseline leg
 * may load it.  It shares no code, header, table or helper with the HIP path.
 *
 * Conventions
 *   - fp16 inputs arrive as raw uint16 bit patterns and are widened exactly to
 *     double; every sum is a plain left-to-right double loop.  No blocking, no
 *     fusion, no reordering beyond what each formula states.
 *   - One "unit" is one (batch b, KV head h).  q head hq uses KV head hq / G,
 *     G = Hq / Hkv.
 *   - Layouts (row-major, element counts):
 *       q        [B, Hq, d]            fp16
 *       K, V     [B, Hkv, L_max, d]    fp16   (tokens 0..L-1 valid)
 *       label    [B, Hkv, L_max, r]    fp16   (4-bit variant: codes [B, Hkv, L_max, ceil(r/8)] uint32
 *                                      and amax [B, Hkv, r] float)
 *       channels [Hkv, r]              int32  (shared across batch)
 *       scores   [B, Hkv, L]           double
 *       idx      [B, Hkv, k]           int32  (first k_eff ascending, rest -1)
 *       out      [B, Hq, d]            double
 *   - OpenMP is used over units only.
 *
 * Pins: every function here is pinned by the CPU tests (brute-force sort,
 * numpy float64 dense attention, closed forms, a hand-derived fixture); none
 * is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- fp16 bit pattern -> double, exact (IEEE binary16) ------------------- */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)mant, -24);               /* zero and subnormals   */
    else if (expo == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant + 1024), expo - 25); /* (1+m/1024)*2^(e-15)  */
    return sign ? -v : v;
}

void ds_oracle_half_to_double(const uint16_t *src, double *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = half_to_double(src[i]);
}

/* ---- Sec. 4.2: label cache = the r calibrated channels of every key ------ */
/* label[b,h,t,j] = K[b,h,t,channels[h,j]] for t in [t0, t0+n).  A build is
 * t0=0, n=L; a decode-step append is the new tokens only.                    */
void ds_oracle_label_write(const uint16_t *K, const int32_t *channels,
                           uint16_t *label, int B, int Hkv, int L_max, int d,
                           int r, int t0, int n)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int t = t0; t < t0 + n; ++t)
                for (int j = 0; j < r; ++j) {
                    int64_t row = ((int64_t)b * Hkv + h) * L_max + t;
                    label[row * r + j] = K[row * d + channels[h * r + j]];
                }
}

/* ---- Alg. 1 steps 1-2: label query and approximate scores ---------------- */
/* s_hat[t] = sum_{g in group} sum_j q_g[C[j]] * label[t,j]; no 1/sqrt(d), no
 * softmax.  precision = 64: the definition, in double.
 * precision = 32: the same sum taken in binary32 in the order a streaming
 * kernel would use: qsum[j] = sum_g (float)q_g[C[j]] (g ascending), then
 * acc = fma(qsum[j], label[t,j], acc) for j ascending from acc = 0.  That mode
 * exists so that an integer decision (the top-k set) can be compared between
 * two implementations that both take it in binary32.                         */
void ds_oracle_scores(const uint16_t *q, const uint16_t *label,
                      const int32_t *channels, double *scores, int B, int Hq,
                      int Hkv, int d, int L, int L_max, int r, int precision)
{
    int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            const uint16_t *lab = label + ((int64_t)b * Hkv + h) * L_max * r;
            double *out = scores + ((int64_t)b * Hkv + h) * L;
            if (precision == 32) {
                float *qs = (float *)malloc(sizeof(float) * r);
                for (int j = 0; j < r; ++j) {
                    float a = 0.0f;
                    for (int g = 0; g < G; ++g) {
                        const uint16_t *qg = q + ((int64_t)b * Hq + h * G + g) * d;
                        a = a + (float)half_to_double(qg[channels[h * r + j]]);
                    }
                    qs[j] = a;
                }
                for (int t = 0; t < L; ++t) {
                    float acc = 0.0f;
                    for (int j = 0; j < r; ++j)
                        acc = fmaf(qs[j], (float)half_to_double(lab[(int64_t)t * r + j]), acc);
                    out[t] = (double)acc;
                }
                free(qs);
            } else {
                for (int t = 0; t < L; ++t) {
                    double acc = 0.0;
                    for (int g = 0; g < G; ++g) {
                        const uint16_t *qg = q + ((int64_t)b * Hq + h * G + g) * d;
                        for (int j = 0; j < r; ++j)
                            acc += half_to_double(qg[channels[h * r + j]]) *
                                   half_to_double(lab[(int64_t)t * r + j]);
                    }
                    out[t] = acc;
                }
            }
        }
}

/* ---- Sec. 4.2, label cache kept in 4 bits ---------------------------------- */
/* The paper states only that the label cache can be stored in 4-bit; the
 * quantiser below is this build's reading (symmetric, one step size per batch
 * entry, KV head and label channel, fixed when the cache is built):
 *   amax[b,h,j] = max over t < L of |K[b,h,t,C[h,j]]|          (exact)
 *   inv  = 7 / amax, step = amax / 7      (binary32 divisions; both 0 if amax = 0)
 *   code[t,j] = clamp(rint((float)K[t,C[j]] * inv), -8, 7)      (binary32 product,
 *               round half to even); the label value is code * step.
 * Eight codes share a 32-bit word: channel j of a token sits in bits
 * [4 (j mod 8), 4 (j mod 8) + 4) of the token's word j / 8 as a two's-complement
 * nibble; nibbles past r are zero.  codes [B, Hkv, L_max, W], W = ceil(r / 8).
 * Tokens appended later are coded with the amax of the build (they saturate
 * at -8 / 7 if they exceed it).                                              */
void ds_oracle_label_q4_amax(const uint16_t *K, const int32_t *channels, float *amax,
                             int B, int Hkv, int L, int L_max, int d, int r)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int j = 0; j < r; ++j) {
                double m = 0.0;
                for (int t = 0; t < L; ++t) {
                    int64_t row = ((int64_t)b * Hkv + h) * L_max + t;
                    double x = fabs(half_to_double(K[row * d + channels[h * r + j]]));
                    if (x > m) m = x;
                }
                amax[((int64_t)b * Hkv + h) * r + j] = (float)m; /* exact: an fp16 value */
            }
}

void ds_oracle_label_q4_write(const uint16_t *K, const int32_t *channels, const float *amax,
                              uint32_t *codes, int B, int Hkv, int L_max, int d, int r,
                              int t0, int n)
{
    int W = (r + 7) / 8;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int t = t0; t < t0 + n; ++t) {
                int64_t row = ((int64_t)b * Hkv + h) * L_max + t;
                for (int w = 0; w < W; ++w) codes[row * W + w] = 0u;
                for (int j = 0; j < r; ++j) {
                    float a = amax[((int64_t)b * Hkv + h) * r + j];
                    float inv = a > 0.0f ? 7.0f / a : 0.0f;
                    float x = (float)half_to_double(K[row * d + channels[h * r + j]]);
                    float y = rintf(x * inv);
                    int c = y < -8.0f ? -8 : (y > 7.0f ? 7 : (int)y);
                    codes[row * W + j / 8] |= ((uint32_t)c & 0xfu) << (4 * (j % 8));
                }
            }
}

static int q4_code(const uint32_t *codes_row, int j)
{
    int nib = (int)((codes_row[j / 8] >> (4 * (j % 8))) & 0xfu);
    return nib >= 8 ? nib - 16 : nib;
}

/* Approximate scores from the 4-bit label cache:
 *   s_hat[t] = sum_{g in group} sum_j q_g[C[j]] * (code[t,j] * step[j]).
 * precision = 64: that sum in double (step is the stored binary32 value).
 * precision = 32: binary32 in streaming order: w[j] = (sum_g (float)q_g[C[j]],
 * g ascending) * step[j], then acc = fma(w[j], (float)code[t,j], acc), j ascending. */
void ds_oracle_scores_q4(const uint16_t *q, const uint32_t *codes, const float *amax,
                         const int32_t *channels, double *scores, int B, int Hq, int Hkv,
                         int d, int L, int L_max, int r, int precision)
{
    int G = Hq / Hkv, W = (r + 7) / 8;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            const uint32_t *cu = codes + ((int64_t)b * Hkv + h) * L_max * W;
            const float *au = amax + ((int64_t)b * Hkv + h) * r;
            double *out = scores + ((int64_t)b * Hkv + h) * L;
            float *step = (float *)malloc(sizeof(float) * r);
            float *wq = (float *)malloc(sizeof(float) * r);
            for (int j = 0; j < r; ++j) {
                step[j] = au[j] / 7.0f;
                float a = 0.0f;
                for (int g = 0; g < G; ++g) {
                    const uint16_t *qg = q + ((int64_t)b * Hq + h * G + g) * d;
                    a = a + (float)half_to_double(qg[channels[h * r + j]]);
                }
                wq[j] = a * step[j];
            }
            for (int t = 0; t < L; ++t) {
                const uint32_t *row = cu + (int64_t)t * W;
                if (precision == 32) {
                    float acc = 0.0f;
                    for (int j = 0; j < r; ++j) acc = fmaf(wq[j], (float)q4_code(row, j), acc);
                    out[t] = (double)acc;
                } else {
                    double acc = 0.0;
                    for (int g = 0; g < G; ++g) {
                        const uint16_t *qg = q + ((int64_t)b * Hq + h * G + g) * d;
                        for (int j = 0; j < r; ++j)
                            acc += half_to_double(qg[channels[h * r + j]]) *
                                   ((double)q4_code(row, j) * (double)step[j]);
                    }
                    out[t] = acc;
                }
            }
            free(step);
            free(wq);
        }
}

/* ---- Alg. 1 step 3: argtopk ---------------------------------------------- */
typedef struct { double s; int32_t t; } scored_t;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;          /* larger score first               */
    if (x->s < y->s) return 1;
    return (x->t > y->t) - (x->t < y->t); /* equal (incl. -0 == +0): lower t  */
}

static int by_int(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Full sort of all L tokens by (score descending, index ascending); the first
 * k_eff = min(k, L) are the selection.  idx[0..k_eff) is returned in ascending
 * token order, idx[k_eff..k) = -1.  If sorted_scores != NULL it receives all L
 * scores in sorted (descending) order, so a caller can read the k-th and
 * (k+1)-th values.                                                           */
void ds_oracle_topk(const double *scores, int L, int k, int32_t *idx,
                    double *sorted_scores)
{
    scored_t *a = (scored_t *)malloc(sizeof(scored_t) * (size_t)L);
    for (int t = 0; t < L; ++t) { a[t].s = scores[t]; a[t].t = t; }
    qsort(a, (size_t)L, sizeof(scored_t), by_score_desc_then_index);
    int k_eff = k < L ? k : L;
    for (int i = 0; i < k_eff; ++i) idx[i] = a[i].t;
    qsort(idx, (size_t)k_eff, sizeof(int32_t), by_int);
    for (int i = k_eff; i < k; ++i) idx[i] = -1;
    if (sorted_scores)
        for (int t = 0; t < L; ++t) sorted_scores[t] = a[t].s;
    free(a);
}

/* ---- Alg. 1 steps 4-5 / Sec. 2.1: softmax attention over a token list ---- */
/* y = softmax(q . K[I,:]^T / sqrt(d)) . V[I,:] for one query row and one
 * unit's K, V (pointers to that unit's [L_max, d] block).                    */
static void attend_list(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                        const int32_t *I, int n, int d, double *y)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    for (int i = 0; i < n; ++i) {
        const uint16_t *krow = K + (int64_t)I[i] * d;
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
            acc += half_to_double(q[c]) * half_to_double(krow[c]);
        s[i] = acc / sqrt((double)d);
        if (s[i] > m) m = s[i];
    }
    double Z = 0.0;
    for (int i = 0; i < n; ++i) { s[i] = exp(s[i] - m); Z += s[i]; }
    for (int c = 0; c < d; ++c) y[c] = 0.0;
    for (int i = 0; i < n; ++i) {
        const uint16_t *vrow = V + (int64_t)I[i] * d;
        double p = s[i] / Z;
        for (int c = 0; c < d; ++c) y[c] += p * half_to_double(vrow[c]);
    }
    free(s);
}

/* Attention of every q head over a GIVEN per-unit index list idx[B,Hkv,k]
 * (entries < 0 are skipped).  Used for steps 4-5 after the oracle's own
 * selection, and to evaluate the output on another implementation's legal
 * choice inside a near-tie band.                                             */
void ds_oracle_attend_idx(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                          const int32_t *idx, double *out, int B, int Hq, int Hkv,
                          int d, int L_max, int k)
{
    int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t u = (int64_t)b * Hkv + h;
            const int32_t *I = idx + u * k;
            int32_t *list = (int32_t *)malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
            int n = 0;
            for (int i = 0; i < k; ++i) if (I[i] >= 0) list[n++] = I[i];
            for (int g = 0; g < G; ++g) {
                int64_t hq = (int64_t)b * Hq + h * G + g;
                attend_list(q + hq * d, K + u * L_max * d, V + u * L_max * d,
                            list, n, d, out + hq * d);
            }
            free(list);
        }
}

/* ---- Sec. 2.1: dense decode attention over all L tokens ------------------ */
void ds_oracle_dense_decode(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                            double *out, int B, int Hq, int Hkv, int d, int L,
                            int L_max)
{
    int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t u = (int64_t)b * Hkv + h;
            int32_t *all = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
            for (int t = 0; t < L; ++t) all[t] = t;
            for (int g = 0; g < G; ++g) {
                int64_t hq = (int64_t)b * Hq + h * G + g;
                attend_list(q + hq * d, K + u * L_max * d, V + u * L_max * d,
                            all, L, d, out + hq * d);
            }
            free(all);
        }
}

/* ---- Algorithm 1, whole: scores -> argtopk -> attention over the k rows --- */
/* label must already hold the label cache (ds_oracle_label_write).  scores_out
 * ([B,Hkv,L] double) and sorted_out ([B,Hkv,L] double, descending) may be NULL. */
void ds_oracle_sparse_decode(const uint16_t *q, const uint16_t *label,
                             const uint16_t *K, const uint16_t *V,
                             const int32_t *channels, double *out, int32_t *idx,
                             double *scores_out, double *sorted_out, int B, int Hq,
                             int Hkv, int d, int L, int L_max, int r, int k,
                             int precision)
{
    int64_t units = (int64_t)B * Hkv;
    double *scores = scores_out ? scores_out
                                : (double *)malloc(sizeof(double) * (size_t)(units * L));
    ds_oracle_scores(q, label, channels, scores, B, Hq, Hkv, d, L, L_max, r, precision);
#pragma omp parallel for schedule(dynamic)
    for (int64_t u = 0; u < units; ++u)
        ds_oracle_topk(scores + u * L, L, k, idx + u * k,
                       sorted_out ? sorted_out + u * L : NULL);
    ds_oracle_attend_idx(q, K, V, idx, out, B, Hq, Hkv, d, L_max, k);
    if (!scores_out) free(scores);
}

/* Algorithm 1 with the scores taken from the 4-bit label cache. */
void ds_oracle_sparse_decode_q4(const uint16_t *q, const uint32_t *codes, const float *amax,
                                const uint16_t *K, const uint16_t *V, const int32_t *channels,
                                double *out, int32_t *idx, double *scores_out,
                                double *sorted_out, int B, int Hq, int Hkv, int d, int L,
                                int L_max, int r, int k, int precision)
{
    int64_t units = (int64_t)B * Hkv;
    double *scores = scores_out ? scores_out
                                : (double *)malloc(sizeof(double) * (size_t)(units * L));
    ds_oracle_scores_q4(q, codes, amax, channels, scores, B, Hq, Hkv, d, L, L_max, r, precision);
#pragma omp parallel for schedule(dynamic)
    for (int64_t u = 0; u < units; ++u)
        ds_oracle_topk(scores + u * L, L, k, idx + u * k,
                       sorted_out ? sorted_out + u * L : NULL);
    ds_oracle_attend_idx(q, K, V, idx, out, B, Hq, Hkv, d, L_max, k);
    if (!scores_out) free(scores);
}

/* ---- Sec. 4.1: offline calibration of the outlier channels --------------- */
/* A = q.K^T = sum_c S_c with S_c = q_c * k_c; the channels with the largest
 * |S_c| over a calibration set are kept.  Averaged over every (query sample,
 * key sample) pair, mean |q_c k_c| factorises into mean|q_c| * mean|k_c|.
 * mode 0 (q outlier): importance = mean_{n,g} |q[n, h*G+g, c]|
 * mode 1 (k outlier): importance = mean_n   |k[n, h, c]|
 * mode 2 (qk outlier): the product of the two.
 * The r most important channels of each KV head are returned in ascending
 * channel order; equal importance keeps the lower channel.                   */
typedef struct { double w; int32_t c; } weighted_t;

static int by_weight_desc_then_channel(const void *a, const void *b)
{
    const weighted_t *x = (const weighted_t *)a, *y = (const weighted_t *)b;
    if (x->w > y->w) return -1;
    if (x->w < y->w) return 1;
    return (x->c > y->c) - (x->c < y->c);
}

void ds_oracle_calibrate(const uint16_t *q_calib, const uint16_t *k_calib, int N,
                         int Hq, int Hkv, int d, int r, int mode,
                         int32_t *channels_out, double *importance_out)
{
    int G = Hq / Hkv;
    for (int h = 0; h < Hkv; ++h) {
        weighted_t *w = (weighted_t *)malloc(sizeof(weighted_t) * (size_t)d);
        for (int c = 0; c < d; ++c) {
            double mq = 0.0, mk = 0.0;
            for (int n = 0; n < N; ++n) {
                for (int g = 0; g < G; ++g)
                    mq += fabs(half_to_double(q_calib[((int64_t)n * Hq + h * G + g) * d + c]));
                mk += fabs(half_to_double(k_calib[((int64_t)n * Hkv + h) * d + c]));
            }
            mq /= (double)N * G;
            mk /= (double)N;
            w[c].w = mode == 0 ? mq : mode == 1 ? mk : mq * mk;
            w[c].c = c;
            if (importance_out) importance_out[(int64_t)h * d + c] = w[c].w;
        }
        qsort(w, (size_t)d, sizeof(weighted_t), by_weight_desc_then_channel);
        for (int j = 0; j < r; ++j) channels_out[h * r + j] = w[j].c;
        qsort(channels_out + h * r, (size_t)r, sizeof(int32_t), by_int);
        free(w);
    }
}
