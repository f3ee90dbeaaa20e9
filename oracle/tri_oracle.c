/*
 * tri_oracle.c -- CPU oracle for the TriAttention KV-cache compression step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal, double-precision
 * evaluation of the paper's formulas that the HIP path is checked against.
 * It shares no code, header, table or helper with the HIP library, and only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * The product path never routes through it.
 *
 * Every function follows one passage of the paper (cited at the function) and
 * evaluates it as printed: an explicit loop over the future offsets, atan2 for
 * the phases, hypot for the magnitudes, cos for the series.  Nothing is folded,
 * blocked or reordered.
 *
 * Pins (tests/test_oracle_*.py): brute-force RoPE rotation with the 2x2
 * matrices of Section 2.1 Eq. 1; invariance under a common position shift;
 * single-band closed form; zero-distance dot product; the (a_f, b_f) form of
 * Appendix B.3; the two printed forms of S_norm; z-score moments; O(N^2) rank
 * counting for top-B; byte-wise gather.  The paper prints no worked numerical
 * example, so beyond those pins numerical parity is unpinned.
 *
 * Conventions
 *   d          head dimension, F = d/2 frequency bands
 *   stats      per query head: [F][3] float = (Re E[q_f], Im E[q_f], E||q_f||)
 *   pairs      0: band f = (x[2f], x[2f+1])  (Section 2.1 Eq. 1)
 *              1: band f = (x[f],  x[f+d/2]) (half-split checkpoints)
 *   dtype      0: float32, 1: bfloat16 (stored as uint16, widened exactly)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1
#define ORACLE_F64 2 /* keys this file has un-rotated itself (post-RoPE caches) */
#define ORACLE_PAIR_INTERLEAVED 0
#define ORACLE_PAIR_HALF 1

/* exact widening of one stored element to double */
static double load_elem(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == ORACLE_F64) return ((const double *)base)[idx];
    return (double)((const float *)base)[idx];
}

/* the complex number a d-vector holds in frequency band f (Section 2.1) */
static void load_band(const void *vec, int dtype, int64_t first, int d, int pairs, int f,
                      double *re, double *im)
{
    if (pairs == ORACLE_PAIR_HALF) {
        *re = load_elem(vec, dtype, first + f);
        *im = load_elem(vec, dtype, first + f + d / 2);
    } else {
        *re = load_elem(vec, dtype, first + 2 * (int64_t)f);
        *im = load_elem(vec, dtype, first + 2 * (int64_t)f + 1);
    }
}

/* Section 2.1: omega_f = theta^(-2f/d) */
double tri_oracle_omega(double theta, int d, int f)
{
    return pow(theta, -2.0 * (double)f / (double)d);
}

/*
 * Offline calibration (Section 4.1, text after the S_trig and S_norm^(0)
 * equations; Appendix B.5): per (layer, query head, band) the complex mean of
 * the pre-RoPE query samples and the mean of their moduli.
 *   q    [T][L][Hq][d]
 *   out  [L][Hq][F][3] float = (Re E[q_f], Im E[q_f], E||q_f||), rounded once
 */
int tri_oracle_centers(const void *q, int dtype, int64_t T, int L, int Hq, int d, int pairs,
                       float *out)
{
    if (T <= 0 || d <= 0 || (d & 1)) return -1;
    int F = d / 2;
    for (int l = 0; l < L; ++l)
        for (int h = 0; h < Hq; ++h)
            for (int f = 0; f < F; ++f) {
                double sre = 0.0, sim = 0.0, sabs = 0.0;
                for (int64_t t = 0; t < T; ++t) {
                    int64_t first = ((t * L + l) * Hq + h) * (int64_t)d;
                    double re, im;
                    load_band(q, dtype, first, d, pairs, f, &re, &im);
                    sre += re;
                    sim += im;
                    sabs += hypot(re, im);
                }
                float *o = out + (((int64_t)l * Hq + h) * F + f) * 3;
                o[0] = (float)(sre / (double)T);
                o[1] = (float)(sim / (double)T);
                o[2] = (float)(sabs / (double)T);
            }
    return 0;
}

/*
 * Appendix B.5, Mean Resultant Length per frequency band:
 *   R_f = ||E[q_f]|| / E||q_f||
 * (a band whose samples are all zero has R_f = 0 by convention).
 *   stats [n][F][3] as written by tri_oracle_centers, out [n][F] double
 */
int tri_oracle_mrl(const float *stats, int64_t n, int F, double *out)
{
    for (int64_t i = 0; i < n * F; ++i) {
        double re = (double)stats[3 * i + 0], im = (double)stats[3 * i + 1], ab = (double)stats[3 * i + 2];
        out[i] = ab > 0.0 ? hypot(re, im) / ab : 0.0;
    }
    return 0;
}

/*
 * Appendix B.7, expected contribution of band f to the attention logit and the dominant bands:
 *   C_f = E||q_f|| * E||k_f||,   bands ranked by C_f, the top K kept
 * (equal contributions: the lower band first).  Query head h of the L x Hq heads is paired with KV
 * head h / G of the same layer.
 *   qstats [L][Hq][F][3], kstats [L][Hkv][F][3], contrib [L][Hq][F] double, top [L][Hq][K] int32
 */
int tri_oracle_band_contrib(const float *qstats, const float *kstats, int L, int Hq, int Hkv, int F, int K,
                            double *contrib, int32_t *top)
{
    if (Hkv <= 0 || Hq % Hkv || K < 0 || K > F) return -1;
    int G = Hq / Hkv;
    for (int l = 0; l < L; ++l)
        for (int h = 0; h < Hq; ++h) {
            const float *q = qstats + ((int64_t)l * Hq + h) * F * 3;
            const float *k = kstats + ((int64_t)l * Hkv + h / G) * F * 3;
            double *c = contrib + ((int64_t)l * Hq + h) * F;
            for (int f = 0; f < F; ++f) c[f] = (double)q[3 * f + 2] * (double)k[3 * f + 2];
            /* selection sort of the K largest: plain and obviously stable */
            int32_t *t = top + ((int64_t)l * Hq + h) * K;
            for (int r = 0; r < K; ++r) {
                int best = -1;
                for (int f = 0; f < F; ++f) {
                    int taken = 0;
                    for (int p = 0; p < r; ++p) taken |= t[p] == f;
                    if (taken) continue;
                    if (best < 0 || c[f] > c[best]) best = f;
                }
                t[r] = best;
            }
        }
    return 0;
}

/*
 * Section 4.1, trigonometric series score:
 *   S_trig(k, x) = sum_f ||E[q_f]|| * ||k_f|| * cos(omega_f * x + phi_f),
 *   phi_f = arg E[q_f] - arg k_f,
 * x being the query-key distance at which the series is evaluated.
 */
double tri_oracle_s_trig(const float *stats, const void *key, int dtype, int64_t first, int d,
                         int pairs, double theta, int64_t dist)
{
    int F = d / 2;
    double s = 0.0;
    for (int f = 0; f < F; ++f) {
        double qre = (double)stats[3 * f + 0], qim = (double)stats[3 * f + 1];
        double kre, kim;
        load_band(key, dtype, first, d, pairs, f, &kre, &kim);
        double A = hypot(qre, qim);
        double m = hypot(kre, kim);
        double phi = atan2(qim, qre) - atan2(kim, kre);
        s += A * m * cos(tri_oracle_omega(theta, d, f) * (double)dist + phi);
    }
    return s;
}

/*
 * Section 4.2, concentration-weighted norm score, second printed form:
 *   S_norm(k) = sum_f (E||q_f|| - ||E[q_f]||) * ||k_f||
 */
double tri_oracle_s_norm(const float *stats, const void *key, int dtype, int64_t first, int d,
                         int pairs)
{
    int F = d / 2;
    double s = 0.0;
    for (int f = 0; f < F; ++f) {
        double qre = (double)stats[3 * f + 0], qim = (double)stats[3 * f + 1];
        double qabs = (double)stats[3 * f + 2];
        double kre, kim;
        load_band(key, dtype, first, d, pairs, f, &kre, &kim);
        s += (qabs - hypot(qre, qim)) * hypot(kre, kim);
    }
    return s;
}

/*
 * Section 4.2, first printed form of the same score, through the Mean
 * Resultant Length R_f = ||E[q_f]|| / E||q_f||:
 *   S_norm(k) = sum_f (1 - R_f) * E||q_f|| * ||k_f||
 * Kept separate so a test can hold the two forms against each other.
 */
double tri_oracle_s_norm_mrl(const float *stats, const void *key, int dtype, int64_t first, int d,
                             int pairs)
{
    int F = d / 2;
    double s = 0.0;
    for (int f = 0; f < F; ++f) {
        double qre = (double)stats[3 * f + 0], qim = (double)stats[3 * f + 1];
        double qabs = (double)stats[3 * f + 2];
        double kre, kim;
        load_band(key, dtype, first, d, pairs, f, &kre, &kim);
        double R = qabs > 0.0 ? hypot(qre, qim) / qabs : 1.0;
        s += (1.0 - R) * qabs * hypot(kre, kim);
    }
    return s;
}

/*
 * Section 4.2, combined score averaged over the future offsets:
 *   S(k, x)  = S_trig(k, x) + S_norm(k)
 *   S~(k)    = (1/|D|) sum_{delta in D} S(k, Delta + delta),  Delta = p_q - p_k
 */
double tri_oracle_score_avg(const float *stats, const void *key, int dtype, int64_t first, int d,
                            int pairs, double theta, int64_t p_q, int64_t p_k,
                            const int64_t *offsets, int n_off)
{
    int64_t Delta = p_q - p_k;
    double acc = 0.0;
    for (int j = 0; j < n_off; ++j) {
        double S = tri_oracle_s_trig(stats, key, dtype, first, d, pairs, theta, Delta + offsets[j]) +
                   tri_oracle_s_norm(stats, key, dtype, first, d, pairs);
        acc += S;
    }
    return acc / (double)n_off;
}

/*
 * All raw scores of one head-instance (one sequence, layer and KV head): the
 * averaged score of every cached key under each of the G query heads of the
 * group (Section 4.3: one score per query head of the group for every key).
 *   stats  [G][F][3]     K  N rows of d elements, row n at element n*row_stride
 *   pos    [N] int32     raw [G][N] double
 */
int tri_oracle_raw_scores(const float *stats, int G, const void *K, int dtype, int64_t row_stride,
                          const int32_t *pos, int64_t N, int64_t cur_pos, int d, int pairs,
                          double theta, const int64_t *offsets, int n_off, double *raw)
{
    if (d <= 0 || (d & 1) || n_off <= 0 || G <= 0) return -1;
    int F = d / 2;
    for (int g = 0; g < G; ++g)
        for (int64_t n = 0; n < N; ++n)
            raw[(int64_t)g * N + n] =
                tri_oracle_score_avg(stats + (int64_t)g * F * 3, K, dtype, n * row_stride, d, pairs,
                                     theta, cur_pos, (int64_t)pos[n], offsets, n_off);
    return 0;
}

/*
 * Section 4.1, the norm score before the concentration weighting ("w/o R" in the
 * ablation of Section 5):
 *   S_norm^(0)(k) = sum_f E||q_f|| * ||k_f||
 */
double tri_oracle_s_norm0(const float *stats, const void *key, int dtype, int64_t first, int d,
                          int pairs)
{
    int F = d / 2;
    double s = 0.0;
    for (int f = 0; f < F; ++f) {
        double qabs = (double)stats[3 * f + 2];
        double kre, kim;
        load_band(key, dtype, first, d, pairs, f, &kre, &kim);
        s += qabs * hypot(kre, kim);
    }
    return s;
}

/*
 * The scoring variants the ablation study removes a component from (Section 5,
 * ablations of the scoring components and of the adaptive weighting):
 *   0  S_trig + S_norm          the method
 *   1  S_trig                   "w/o S_norm"
 *   2  S_norm                   "w/o S_trig"
 *   3  S_trig + S_norm^(0)      "w/o R"
 * each averaged over the future offsets exactly as in tri_oracle_score_avg.
 */
double tri_oracle_score_avg_variant(const float *stats, const void *key, int dtype, int64_t first,
                                    int d, int pairs, double theta, int64_t p_q, int64_t p_k,
                                    const int64_t *offsets, int n_off, int variant)
{
    int64_t Delta = p_q - p_k;
    double acc = 0.0;
    for (int j = 0; j < n_off; ++j) {
        double S = 0.0;
        if (variant != 2) S += tri_oracle_s_trig(stats, key, dtype, first, d, pairs, theta, Delta + offsets[j]);
        if (variant == 0 || variant == 2) S += tri_oracle_s_norm(stats, key, dtype, first, d, pairs);
        if (variant == 3) S += tri_oracle_s_norm0(stats, key, dtype, first, d, pairs);
        acc += S;
    }
    return acc / (double)n_off;
}

/*
 * A key read from a post-RoPE cache: the stored vector is R(p_k) k, every band
 * rotated by omega_f * p_k with the 2x2 matrix of Section 2.1 Eq. 1.  The inverse
 * of that matrix (its transpose) gives back the pre-RoPE key the scores are
 * defined on.  out: d doubles, laid out like the stored vector.
 */
void tri_oracle_unrotate_key(const void *key, int dtype, int64_t first, int d, int pairs,
                             double theta, int64_t p_k, double *out)
{
    int F = d / 2;
    for (int f = 0; f < F; ++f) {
        double xr, xi;
        load_band(key, dtype, first, d, pairs, f, &xr, &xi);
        double ang = tri_oracle_omega(theta, d, f) * (double)p_k;
        double c = cos(ang), s = sin(ang);
        double kr = c * xr + s * xi;  /* transpose of [[c, -s], [s, c]] */
        double ki = -s * xr + c * xi;
        if (pairs == ORACLE_PAIR_HALF) {
            out[f] = kr;
            out[f + F] = ki;
        } else {
            out[2 * f] = kr;
            out[2 * f + 1] = ki;
        }
    }
}

/*
 * tri_oracle_raw_scores with a scoring variant (see tri_oracle_score_avg_variant) and,
 * with rotated != 0, for a cache that stores post-RoPE keys.
 */
int tri_oracle_raw_scores_ex(const float *stats, int G, const void *K, int dtype, int64_t row_stride,
                             const int32_t *pos, int64_t N, int64_t cur_pos, int d, int pairs,
                             double theta, const int64_t *offsets, int n_off, int variant, int rotated,
                             double *raw)
{
    if (d <= 0 || (d & 1) || n_off <= 0 || G <= 0 || variant < 0 || variant > 3) return -1;
    int F = d / 2;
    double *tmp = (double *)malloc(sizeof(double) * (size_t)d);
    if (!tmp) return -2;
    for (int64_t n = 0; n < N; ++n) {
        const void *key = K;
        int kd = dtype;
        int64_t first = n * row_stride;
        if (rotated) {
            tri_oracle_unrotate_key(K, dtype, first, d, pairs, theta, (int64_t)pos[n], tmp);
            key = tmp;
            kd = ORACLE_F64;
            first = 0;
        }
        for (int g = 0; g < G; ++g)
            raw[(int64_t)g * N + n] =
                tri_oracle_score_avg_variant(stats + (int64_t)g * F * 3, key, kd, first, d, pairs, theta,
                                             cur_pos, (int64_t)pos[n], offsets, n_off, variant);
    }
    free(tmp);
    return 0;
}

/*
 * Section 4.3, normalise-then-aggregate:
 *   S^(g)(k) = (S~(g)(k) - mu_g) / sigma_g, mu_g and sigma_g over all N keys
 *   S_final(k) = max_g S^(g)(k)
 * sigma is the population standard deviation (divide by N); a head whose
 * scores are all equal (sigma = 0) contributes 0 for every key.
 *   raw [G][N]   mu, sigma [G]   final [N]
 */
int tri_oracle_gqa_final(const double *raw, int G, int64_t N, double *mu, double *sigma,
                         double *final)
{
    if (G <= 0 || N <= 0) return -1;
    for (int g = 0; g < G; ++g) {
        const double *s = raw + (int64_t)g * N;
        double sum = 0.0;
        for (int64_t n = 0; n < N; ++n) sum += s[n];
        double m = sum / (double)N;
        double ss = 0.0;
        for (int64_t n = 0; n < N; ++n) ss += (s[n] - m) * (s[n] - m);
        /* all scores equal: sigma is 0, whatever the rounding of sum / N left in s[n] - m */
        double lo = s[0], hi = s[0];
        for (int64_t n = 1; n < N; ++n) {
            if (s[n] < lo) lo = s[n];
            if (s[n] > hi) hi = s[n];
        }
        if (lo == hi) ss = 0.0;
        mu[g] = m;
        sigma[g] = sqrt(ss / (double)N);
    }
    for (int64_t n = 0; n < N; ++n) {
        double best = 0.0;
        for (int g = 0; g < G; ++g) {
            double z = sigma[g] > 0.0 ? (raw[(int64_t)g * N + n] - mu[g]) / sigma[g] : 0.0;
            if (g == 0 || z > best) best = z;
        }
        final[n] = best;
    }
    return 0;
}

/* ---- top-B: a full stable sort (Section 4.3: the B keys with the largest final score stay) ---- */

typedef struct {
    double score;
    int32_t index;
} ranked;

/* merge sort: descending score, equal scores keep ascending index */
static void merge_sort_ranked(ranked *a, ranked *tmp, int64_t n)
{
    if (n < 2) return;
    int64_t h = n / 2;
    merge_sort_ranked(a, tmp, h);
    merge_sort_ranked(a + h, tmp, n - h);
    int64_t i = 0, j = h, o = 0;
    while (i < h && j < n) {
        /* take from the right half only when it is strictly larger */
        if (a[j].score > a[i].score) tmp[o++] = a[j++];
        else tmp[o++] = a[i++];
    }
    while (i < h) tmp[o++] = a[i++];
    while (j < n) tmp[o++] = a[j++];
    memcpy(a, tmp, (size_t)n * sizeof *a);
}

static int cmp_i32(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    return (a > b) - (a < b);
}

/*
 * Keep the min(N, B) largest scores; of equal scores the lower index wins;
 * the kept indices are returned in ascending order.  -0.0 equals +0.0.
 */
int tri_oracle_topk(const double *final, int64_t N, int64_t B, int32_t *idx, int32_t *cnt)
{
    if (N < 0 || B < 0) return -1;
    int64_t keep = N < B ? N : B;
    *cnt = (int32_t)keep;
    if (keep == 0) return 0;
    ranked *a = (ranked *)malloc((size_t)N * sizeof *a);
    ranked *t = (ranked *)malloc((size_t)N * sizeof *t);
    if (!a || !t) {
        free(a);
        free(t);
        return -2;
    }
    for (int64_t n = 0; n < N; ++n) {
        a[n].score = final[n];
        a[n].index = (int32_t)n;
    }
    merge_sort_ranked(a, t, N);
    for (int64_t j = 0; j < keep; ++j) idx[j] = a[j].index;
    qsort(idx, (size_t)keep, sizeof *idx, cmp_i32);
    free(a);
    free(t);
    return 0;
}

/*
 * Eviction as a compaction (Section 4.3: every other key leaves the cache): row j of the
 * result is row idx[j] of the source.  idx ascending, so idx[j] >= j and the
 * ascending loop is also correct when dst and src are the same buffer.
 */
int tri_oracle_compact_rows(const void *src, int64_t src_stride_bytes, int64_t row_bytes,
                            const int32_t *idx, int32_t cnt, void *dst, int64_t dst_stride_bytes)
{
    for (int32_t j = 0; j < cnt; ++j)
        memmove((char *)dst + (int64_t)j * dst_stride_bytes,
                (const char *)src + (int64_t)idx[j] * src_stride_bytes, (size_t)row_bytes);
    return 0;
}

/*
 * Eviction that moves as few slots as possible (same passage; the paper fixes no slot order): the kept
 * keys that already sit in slots [0, cnt) stay; the i-th free slot below cnt (ascending) receives the
 * i-th kept key stored at or beyond cnt (ascending).  rows: K or V or positions, row n at byte n*stride.
 */
int tri_oracle_compact_fill(void *rows, int64_t stride_bytes, int64_t row_bytes, const int32_t *idx, int32_t cnt)
{
    char *kept = (char *)calloc((size_t)(cnt > 0 ? cnt : 1), 1);
    if (!kept) return -2;
    int32_t first_tail = cnt;   /* first entry of idx that lies at or beyond cnt */
    for (int32_t j = 0; j < cnt; ++j) {
        if (idx[j] < cnt) kept[idx[j]] = 1;
        else if (first_tail == cnt) first_tail = j;
    }
    int32_t t = first_tail;
    for (int32_t hole = 0; hole < cnt && t < cnt; ++hole) {
        if (kept[hole]) continue;
        memcpy((char *)rows + (int64_t)hole * stride_bytes, (const char *)rows + (int64_t)idx[t] * stride_bytes,
               (size_t)row_bytes);
        ++t;
    }
    free(kept);
    return 0;
}

/* ---- paged layout (block table; not in the paper, a storage choice) ---- */

/* element offset of slot n of (layer, sequence, head) in a paged pool */
static int64_t paged_offset(const int32_t *block_table, int32_t max_blocks, int32_t block_size,
                            int64_t stride_layer, int64_t stride_block, int64_t stride_head,
                            int64_t stride_slot, int layer, int seq, int head, int64_t n)
{
    int64_t blk = block_table[(int64_t)seq * max_blocks + n / block_size];
    return layer * stride_layer + blk * stride_block + head * stride_head +
           (n % block_size) * stride_slot;
}

/* copy the N rows of one head-instance out of a paged pool, in slot order */
int tri_oracle_paged_gather(const void *pool, int64_t elem_bytes, int64_t row_elems,
                            const int32_t *block_table, int32_t max_blocks, int32_t block_size,
                            int64_t stride_layer, int64_t stride_block, int64_t stride_head,
                            int64_t stride_slot, int layer, int seq, int head, int64_t N, void *out)
{
    for (int64_t n = 0; n < N; ++n) {
        int64_t off = paged_offset(block_table, max_blocks, block_size, stride_layer, stride_block,
                                   stride_head, stride_slot, layer, seq, head, n);
        memcpy((char *)out + n * row_elems * elem_bytes, (const char *)pool + off * elem_bytes,
               (size_t)(row_elems * elem_bytes));
    }
    return 0;
}

/* in-place compaction of one head-instance inside a paged pool: slot j <- slot idx[j] */
int tri_oracle_paged_compact(void *pool, int64_t elem_bytes, int64_t row_elems,
                             const int32_t *block_table, int32_t max_blocks, int32_t block_size,
                             int64_t stride_layer, int64_t stride_block, int64_t stride_head,
                             int64_t stride_slot, int layer, int seq, int head, const int32_t *idx,
                             int32_t cnt)
{
    for (int32_t j = 0; j < cnt; ++j) {
        int64_t so = paged_offset(block_table, max_blocks, block_size, stride_layer, stride_block,
                                  stride_head, stride_slot, layer, seq, head, idx[j]);
        int64_t dof = paged_offset(block_table, max_blocks, block_size, stride_layer, stride_block,
                                   stride_head, stride_slot, layer, seq, head, j);
        memmove((char *)pool + dof * elem_bytes, (const char *)pool + so * elem_bytes,
                (size_t)(row_elems * elem_bytes));
    }
    return 0;
}
