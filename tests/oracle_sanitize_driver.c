/*
 * Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of oracle/tri_oracle.c (test infrastructure).
 * Every exported function of the oracle runs on heap buffers of exactly the size its contract names, so that a read
 * or write past an operand is a sanitizer report, and a handful of results are checked against values that follow
 * from the definitions by hand (single band, shift invariance, rank counting, byte-wise gathers).  Exit status 0 =
 * no report and every check passed.  Built and run by tests/test_oracle_sanitizers.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double tri_oracle_omega(double theta, int d, int f);
int tri_oracle_centers(const void *q, int dtype, int64_t T, int L, int Hq, int d, int pairs, float *out);
int tri_oracle_mrl(const float *stats, int64_t n, int F, double *out);
int tri_oracle_band_contrib(const float *qstats, const float *kstats, int L, int Hq, int Hkv, int F, int K,
                            double *contrib, int32_t *top);
double tri_oracle_s_trig(const float *stats, const void *key, int dtype, int64_t first, int d, int pairs,
                         double theta, int64_t dist);
double tri_oracle_s_norm(const float *stats, const void *key, int dtype, int64_t first, int d, int pairs);
double tri_oracle_s_norm_mrl(const float *stats, const void *key, int dtype, int64_t first, int d, int pairs);
double tri_oracle_score_avg(const float *stats, const void *key, int dtype, int64_t first, int d, int pairs,
                            double theta, int64_t p_q, int64_t p_k, const int64_t *offsets, int n_off);
int tri_oracle_raw_scores(const float *stats, int G, const void *K, int dtype, int64_t row_stride,
                          const int32_t *pos, int64_t N, int64_t cur_pos, int d, int pairs, double theta,
                          const int64_t *offsets, int n_off, double *raw);
double tri_oracle_score_avg_variant(const float *stats, const void *key, int dtype, int64_t first, int d, int pairs,
                                    double theta, int64_t p_q, int64_t p_k, const int64_t *offsets, int n_off,
                                    int variant);
void tri_oracle_unrotate_key(const void *key, int dtype, int64_t first, int d, int pairs, double theta, int64_t p_k,
                             double *out);
int tri_oracle_raw_scores_ex(const float *stats, int G, const void *K, int dtype, int64_t row_stride,
                             const int32_t *pos, int64_t N, int64_t cur_pos, int d, int pairs, double theta,
                             const int64_t *offsets, int n_off, int variant, int rotated, double *raw);
int tri_oracle_gqa_final(const double *raw, int G, int64_t N, double *mu, double *sigma, double *final);
int tri_oracle_topk(const double *final, int64_t N, int64_t B, int32_t *idx, int32_t *cnt);
int tri_oracle_compact_rows(const void *src, int64_t src_stride_bytes, int64_t row_bytes, const int32_t *idx,
                            int32_t cnt, void *dst, int64_t dst_stride_bytes);
int tri_oracle_compact_fill(void *rows, int64_t stride_bytes, int64_t row_bytes, const int32_t *idx, int32_t cnt);
int tri_oracle_paged_gather(const void *pool, int64_t elem_bytes, int64_t row_elems, const int32_t *block_table,
                            int32_t max_blocks, int32_t block_size, int64_t stride_layer, int64_t stride_block,
                            int64_t stride_head, int64_t stride_slot, int layer, int seq, int head, int64_t N,
                            void *out);
int tri_oracle_paged_compact(void *pool, int64_t elem_bytes, int64_t row_elems, const int32_t *block_table,
                             int32_t max_blocks, int32_t block_size, int64_t stride_layer, int64_t stride_block,
                             int64_t stride_head, int64_t stride_slot, int layer, int seq, int head,
                             const int32_t *idx, int32_t cnt);

static int failures = 0;
#define CHECK(cond)                                                         \
    do {                                                                    \
        if (!(cond)) {                                                      \
            fprintf(stderr, "line %d: check failed: %s\n", __LINE__, #cond); \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

/* counter-based pseudo-random numbers: the same stream every run */
static uint64_t mix(uint64_t x)
{
    x += 0x9e3779b97f4a7c15ull;
    x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
    x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
    return x ^ (x >> 31);
}
static double unif(uint64_t *ctr) { return (double)(mix((*ctr)++) >> 11) * (1.0 / 9007199254740992.0) * 2.0 - 1.0; }
static uint16_t to_bf16(double v)
{
    float f = (float)v;
    uint32_t b;
    memcpy(&b, &f, 4);
    return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}

enum { D = 16, F = D / 2, G = 2, N = 37, L = 2, HQ = 4, HKV = 2, T = 5 };

int main(void)
{
    uint64_t ctr = 1;
    const double theta = 1e4;
    const int64_t offsets_src[3] = {1, 2, 4};
    int64_t *offsets = malloc(sizeof offsets_src);
    memcpy(offsets, offsets_src, sizeof offsets_src);

    /* ---- calibration, MRL, band contributions ---- */
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int pairs = 0; pairs < 2; ++pairs) {
            size_t n = (size_t)T * L * HQ * D;
            void *q = malloc(n * (dtype ? 2 : 4));
            for (size_t i = 0; i < n; ++i) {
                double v = unif(&ctr);
                if (dtype) ((uint16_t *)q)[i] = to_bf16(v);
                else ((float *)q)[i] = (float)v;
            }
            float *st = malloc((size_t)L * HQ * F * 3 * sizeof(float));
            CHECK(tri_oracle_centers(q, dtype, T, L, HQ, D, pairs, st) == 0);
            CHECK(tri_oracle_centers(q, dtype, 0, L, HQ, D, pairs, st) == -1);
            double *mrl = malloc((size_t)L * HQ * F * sizeof(double));
            CHECK(tri_oracle_mrl(st, (int64_t)L * HQ, F, mrl) == 0);
            for (int i = 0; i < L * HQ * F; ++i) CHECK(mrl[i] >= 0.0 && mrl[i] <= 1.0 + 1e-6);
            float *kst = malloc((size_t)L * HKV * F * 3 * sizeof(float));
            for (int i = 0; i < L * HKV * F * 3; ++i) kst[i] = (float)fabs(unif(&ctr));
            double *contrib = malloc((size_t)L * HQ * F * sizeof(double));
            int32_t *top = malloc((size_t)L * HQ * 3 * sizeof(int32_t));
            CHECK(tri_oracle_band_contrib(st, kst, L, HQ, HKV, F, 3, contrib, top) == 0);
            for (int i = 0; i < L * HQ * 3; ++i) CHECK(top[i] >= 0 && top[i] < F);
            CHECK(tri_oracle_band_contrib(st, kst, L, HQ, HKV, F, F + 1, contrib, top) == -1);
            free(top); free(contrib); free(kst); free(mrl); free(st); free(q);
        }

    /* ---- scores: one head-instance of N keys, both layouts and both element types ---- */
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int pairs = 0; pairs < 2; ++pairs) {
            float *stats = malloc((size_t)G * F * 3 * sizeof(float));
            for (int i = 0; i < G * F; ++i) {
                stats[3 * i] = (float)unif(&ctr);
                stats[3 * i + 1] = (float)unif(&ctr);
                stats[3 * i + 2] = (float)(1.5 + 0.5 * unif(&ctr));
            }
            void *K = malloc((size_t)N * D * (dtype ? 2 : 4));
            for (int i = 0; i < N * D; ++i) {
                double v = unif(&ctr);
                if (dtype) ((uint16_t *)K)[i] = to_bf16(v);
                else ((float *)K)[i] = (float)v;
            }
            int32_t *pos = malloc(N * sizeof(int32_t));
            for (int n = 0; n < N; ++n) pos[n] = 3 * n + (n & 1);
            const int64_t cur = 200;
            double *raw = malloc((size_t)G * N * sizeof(double));
            CHECK(tri_oracle_raw_scores(stats, G, K, dtype, D, pos, N, cur, D, pairs, theta, offsets, 3, raw) == 0);
            /* the per-key entry point gives the same number, and a common shift of both positions changes nothing */
            for (int g = 0; g < G; ++g)
                for (int n = 0; n < N; n += 9) {
                    double a = tri_oracle_score_avg(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs, theta,
                                                    cur, pos[n], offsets, 3);
                    double b = tri_oracle_score_avg(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs, theta,
                                                    cur + 1000, pos[n] + 1000, offsets, 3);
                    CHECK(fabs(a - raw[(size_t)g * N + n]) <= 1e-12 * (1.0 + fabs(a)));
                    CHECK(fabs(a - b) <= 1e-9 * (1.0 + fabs(a)));
                    double tr = tri_oracle_s_trig(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs, theta, 7);
                    double nm = tri_oracle_s_norm(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs);
                    double nr = tri_oracle_s_norm_mrl(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs);
                    CHECK(isfinite(tr) && isfinite(nm) && fabs(nm - nr) <= 1e-9 * (1.0 + fabs(nm)));
                    /* variants 1 and 2 split variant 0 into its two terms */
                    double v0 = tri_oracle_score_avg_variant(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs,
                                                             theta, cur, pos[n], offsets, 3, 0);
                    double v1 = tri_oracle_score_avg_variant(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs,
                                                             theta, cur, pos[n], offsets, 3, 1);
                    double v2 = tri_oracle_score_avg_variant(stats + (size_t)g * F * 3, K, dtype, (int64_t)n * D, D, pairs,
                                                             theta, cur, pos[n], offsets, 3, 2);
                    CHECK(fabs(v0 - a) <= 1e-12 * (1.0 + fabs(a)) && fabs(v1 + v2 - v0) <= 1e-9 * (1.0 + fabs(v0)));
                }
            /* post-RoPE storage: un-rotating a key that sits at position 0 returns it */
            double *un = malloc(D * sizeof(double));
            tri_oracle_unrotate_key(K, dtype, 0, D, pairs, theta, 0, un);
            for (int f = 0; f < F; ++f) {
                int i_re = pairs ? f : 2 * f;
                double want = dtype ? 0.0 : (double)((float *)K)[i_re];
                if (!dtype) CHECK(fabs(un[pairs ? f : 2 * f] - want) <= 1e-12);
            }
            free(un);
            double *raw2 = malloc((size_t)G * N * sizeof(double));
            CHECK(tri_oracle_raw_scores_ex(stats, G, K, dtype, D, pos, N, cur, D, pairs, theta, offsets, 3, 0, 0, raw2) == 0);
            for (int i = 0; i < G * N; ++i) CHECK(raw2[i] == raw[i]);
            CHECK(tri_oracle_raw_scores_ex(stats, G, K, dtype, D, pos, N, cur, D, pairs, theta, offsets, 3, 0, 1, raw2) == 0);
            CHECK(tri_oracle_raw_scores_ex(stats, G, K, dtype, D, pos, N, cur, D, pairs, theta, offsets, 3, 4, 0, raw2) == -1);
            CHECK(tri_oracle_raw_scores(stats, G, K, dtype, D, pos, 0, cur, D, pairs, theta, offsets, 3, raw2) == 0);

            /* ---- z-score, max over the group, top-B with ties ---- */
            double *mu = malloc(G * sizeof(double)), *sg = malloc(G * sizeof(double)), *fin = malloc(N * sizeof(double));
            CHECK(tri_oracle_gqa_final(raw, G, N, mu, sg, fin) == 0);
            for (int g = 0; g < G; ++g) {
                double m = 0.0;
                for (int n = 0; n < N; ++n) m += raw[(size_t)g * N + n];
                CHECK(fabs(m / N - mu[g]) <= 1e-12 * (1.0 + fabs(mu[g])) && sg[g] > 0.0);
            }
            fin[5] = fin[11];   /* a tie */
            for (int B = 0; B <= N + 2; B += 3) {
                int32_t *idx = malloc((size_t)(B > 0 ? B : 1) * sizeof(int32_t)), cnt = -1;
                CHECK(tri_oracle_topk(fin, N, B, idx, &cnt) == 0 && cnt == (B < N ? B : N));
                for (int j = 0; j < cnt; ++j) {   /* ascending slots, each ranked by counting */
                    CHECK(j == 0 || idx[j] > idx[j - 1]);
                    int better = 0;
                    for (int n = 0; n < N; ++n)
                        better += fin[n] > fin[idx[j]] || (fin[n] == fin[idx[j]] && n < idx[j]);
                    CHECK(better < cnt);
                }
                free(idx);
            }
            CHECK(tri_oracle_gqa_final(raw, G, 0, mu, sg, fin) == -1);
            free(fin); free(sg); free(mu); free(raw2); free(raw); free(pos); free(K); free(stats);
        }

    /* ---- compaction: rows, in-place fill, paged pools ---- */
    {
        enum { ROWS = 23, RB = 12, KEEP = 7 };
        unsigned char *src = malloc(ROWS * RB), *dst = malloc(KEEP * RB);
        for (int i = 0; i < ROWS * RB; ++i) src[i] = (unsigned char)mix(ctr++);
        int32_t idx[KEEP] = {0, 3, 4, 9, 15, 21, 22};
        int32_t *ih = malloc(sizeof idx);
        memcpy(ih, idx, sizeof idx);
        CHECK(tri_oracle_compact_rows(src, RB, RB, ih, KEEP, dst, RB) == 0);
        for (int j = 0; j < KEEP; ++j) CHECK(memcmp(dst + j * RB, src + idx[j] * RB, RB) == 0);
        unsigned char *fill = malloc(ROWS * RB);
        memcpy(fill, src, ROWS * RB);
        CHECK(tri_oracle_compact_fill(fill, RB, RB, ih, KEEP) == 0);
        for (int j = 0; j < KEEP; ++j) {   /* the first KEEP rows hold exactly the kept rows, in some order */
            int found = 0;
            for (int r = 0; r < KEEP; ++r) found += memcmp(fill + r * RB, src + idx[j] * RB, RB) == 0;
            CHECK(found >= 1);
        }
        CHECK(tri_oracle_compact_rows(src, RB, RB, ih, KEEP, src, RB) == 0);   /* in place */
        for (int j = 0; j < KEEP; ++j) CHECK(memcmp(src + j * RB, dst + j * RB, RB) == 0);
        free(fill); free(ih); free(dst); free(src);

        enum { BS = 4, NB = 6, ROW = 3, NS = 2, NH = 2, NL = 2, LEN = 10 };   /* pool [NL][NB*NS][NH][BS][ROW] floats */
        const int64_t s_slot = ROW, s_head = (int64_t)BS * ROW, s_blk = (int64_t)NH * BS * ROW, s_layer = (int64_t)NB * NS * s_blk;
        float *pool = malloc((size_t)NL * s_layer * sizeof(float));
        for (int64_t i = 0; i < NL * s_layer; ++i) pool[i] = (float)i;
        int32_t *bt = malloc(NS * NB * sizeof(int32_t));
        for (int s = 0; s < NS; ++s)
            for (int b = 0; b < NB; ++b) bt[s * NB + b] = (b * 5 + 3 * s + 1) % (NB * NS);   /* a permutation per s */
        float *out = malloc(LEN * ROW * sizeof(float));
        CHECK(tri_oracle_paged_gather(pool, 4, ROW, bt, NB, BS, s_layer, s_blk, s_head, s_slot, 1, 1, 1, LEN, out) == 0);
        for (int n = 0; n < LEN; ++n) {
            int64_t off = 1 * s_layer + bt[1 * NB + n / BS] * s_blk + 1 * s_head + (n % BS) * s_slot;
            CHECK(out[n * ROW] == (float)off && out[n * ROW + ROW - 1] == (float)(off + ROW - 1));
        }
        int32_t pidx[4] = {1, 2, 6, 9};
        int32_t *pih = malloc(sizeof pidx);
        memcpy(pih, pidx, sizeof pidx);
        CHECK(tri_oracle_paged_compact(pool, 4, ROW, bt, NB, BS, s_layer, s_blk, s_head, s_slot, 1, 1, 1, pih, 4) == 0);
        float *out2 = malloc(4 * ROW * sizeof(float));
        CHECK(tri_oracle_paged_gather(pool, 4, ROW, bt, NB, BS, s_layer, s_blk, s_head, s_slot, 1, 1, 1, 4, out2) == 0);
        for (int j = 0; j < 4; ++j) CHECK(memcmp(out2 + j * ROW, out + pidx[j] * ROW, ROW * sizeof(float)) == 0);
        free(out2); free(pih); free(out); free(bt); free(pool);
    }
    CHECK(tri_oracle_omega(theta, D, 0) == 1.0 && fabs(tri_oracle_omega(theta, D, F) - 1.0 / theta) <= 1e-18);
    free(offsets);
    if (failures) {
        fprintf(stderr, "%d checks failed\n", failures);
        return 1;
    }
    puts("oracle sanitizer driver: all checks passed");
    return 0;
}
