/* Runs every entry point of the CPU oracle on small seeded inputs, edge cases included, in a build with
 * -fsanitize=address,undefined: out-of-bounds accesses, leaks and undefined arithmetic end the run.
 * Test infrastructure (tests/test_sanitizers.py builds and runs it); prints "oracle sanitizer run ok". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double ico_widen_bf16(uint16_t h);
double ico_widen_e4m3(uint8_t b);
int ico_indexer_scores(int dtype, const void *q, const void *k, const float *w, const float *q_scale, const float *k_scale,
                       int B, int Tq, int Lk, int H, int d, long q_pos0, const int *rows, int n_rows, double *out);
int ico_topk_row(const double *scores, int nv, int k_sel, int32_t *idx, double *sel, double *kth, double *next, double *mean_abs);
int ico_indexer_topk(int dtype, const void *q, const void *k, const float *w, const float *q_scale, const float *k_scale,
                     int B, int Tq, int Lk, int H, int d, long q_pos0, int k_sel, const int *rows, int n_rows, int32_t *idx,
                     double *sel, double *kth, double *next, double *mean_abs);
int ico_sparse_attn(const uint16_t *Q, const uint16_t *KV, const int32_t *idx, int B, int Tq, int Lk, int Hq, int d_qk, int d_v,
                    int v_off, int row_elems, int k_sel, double sm_scale, const int *rows, int n_rows, int idx_rows_are_subset,
                    double *O, double *lse);
int ico_dense_causal_attn(const uint16_t *Q, const uint16_t *KV, int B, int Tq, int Lk, int Hq, int d_qk, int d_v, int v_off,
                          int row_elems, double sm_scale, long q_pos0, double *O);
int ico_topk_overlap(const int32_t *const *idx, int n_layers, long nq, int k_sel, int Lk, uint64_t *inter, uint64_t *sizes);
int ico_cosine_rows(const uint16_t *A, const uint16_t *B, long n_rows, long row_len, double *per_row, double *mean);
int ico_num_threads(void);

static uint32_t rng = 2603122010u;
static uint32_t next_u32(void) { rng = rng * 1664525u + 1013904223u; return rng; }
static uint16_t rand_bf16(void)
{   /* sign, exponent near 1.0, random mantissa: finite values of order one */
    return (uint16_t)(((next_u32() >> 31) << 15) | ((124u + (next_u32() >> 30)) << 7) | (next_u32() >> 25));
}
#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed line %d: %s\n", __LINE__, #x); return 1; } } while (0)

int main(void)
{
    for (int b = 0; b < 65536; b += 97) (void)ico_widen_bf16((uint16_t)b);
    for (int b = 0; b < 256; ++b) (void)ico_widen_e4m3((uint8_t)b);
    CHECK(ico_num_threads() >= 1);

    enum { B = 2, Tq = 9, Lk = 23, H = 3, d = 16, KS = 5 };
    uint16_t *q = malloc(sizeof(uint16_t) * B * Tq * H * d), *k = malloc(sizeof(uint16_t) * B * Lk * d);
    uint8_t *q8 = malloc(B * Tq * H * d), *k8 = malloc(B * Lk * d);
    float *w = malloc(sizeof(float) * B * Tq * H), *qs = malloc(sizeof(float) * B * Tq), *ks = malloc(sizeof(float) * B * Lk);
    for (int i = 0; i < B * Tq * H * d; ++i) { q[i] = rand_bf16(); q8[i] = (uint8_t)(next_u32() >> 25); }
    for (int i = 0; i < B * Lk * d; ++i) { k[i] = rand_bf16(); k8[i] = (uint8_t)(next_u32() >> 25); }
    for (int i = 0; i < B * Tq * H; ++i) w[i] = (float)(next_u32() >> 8) / 16777216.0f - 0.25f;
    for (int i = 0; i < B * Tq; ++i) qs[i] = 0.5f;
    for (int i = 0; i < B * Lk; ++i) ks[i] = 2.0f;
    double *sc = malloc(sizeof(double) * B * Tq * Lk);
    long p0s[] = {0, Lk - Tq, Lk + 4, -3};
    for (int c = 0; c < 4; ++c) {
        CHECK(ico_indexer_scores(0, q, k, w, NULL, NULL, B, Tq, Lk, H, d, p0s[c], NULL, 0, sc) == 0);
        CHECK(ico_indexer_scores(1, q8, k8, w, qs, ks, B, Tq, Lk, H, d, p0s[c], NULL, 0, sc) == 0);
    }
    int rows[3] = {0, 4, Tq - 1};
    CHECK(ico_indexer_scores(0, q, k, w, NULL, NULL, B, Tq, Lk, H, d, Lk - Tq, rows, 3, sc) == 0);
    CHECK(ico_indexer_scores(0, NULL, k, w, NULL, NULL, B, Tq, Lk, H, d, 0, NULL, 0, sc) != 0);

    int32_t *idx = malloc(sizeof(int32_t) * B * Tq * KS);
    double *sel = malloc(sizeof(double) * B * Tq * KS), *kth = malloc(sizeof(double) * B * Tq), *nxt = malloc(sizeof(double) * B * Tq),
           *mab = malloc(sizeof(double) * B * Tq);
    CHECK(ico_indexer_topk(0, q, k, w, NULL, NULL, B, Tq, Lk, H, d, Lk - Tq, KS, NULL, 0, idx, sel, kth, nxt, mab) == 0);
    CHECK(ico_indexer_topk(0, q, k, w, NULL, NULL, B, Tq, Lk, H, d, 0, KS, NULL, 0, idx, NULL, NULL, NULL, NULL) == 0);   /* rows shorter than k */
    CHECK(ico_indexer_topk(1, q8, k8, w, qs, ks, B, Tq, Lk, H, d, 0, KS, rows, 3, idx, sel, kth, nxt, mab) == 0);
    double row[7] = {1.0, 1.0, -2.0, 1.0, 0.0, 3.0, 1.0};
    int32_t ri[4]; double rs[4], a, b2, c2;
    CHECK(ico_topk_row(row, 7, 4, ri, rs, &a, &b2, &c2) == 0 && ri[0] == 5 && ri[1] == 0 && ri[2] == 1 && ri[3] == 3);   /* ties: lower position */
    CHECK(ico_topk_row(row, 2, 4, ri, rs, &a, &b2, &c2) == 0 && ri[2] == -1);
    CHECK(ico_topk_row(row, 0, 4, ri, rs, &a, &b2, &c2) == 0 && ri[0] == -1);

    enum { Hq = 2, dqk = 16, dv = 8, voff = 16, rowe = 24 };
    uint16_t *Q = malloc(sizeof(uint16_t) * B * Tq * Hq * dqk), *KV = malloc(sizeof(uint16_t) * B * Lk * rowe);
    for (int i = 0; i < B * Tq * Hq * dqk; ++i) Q[i] = rand_bf16();
    for (int i = 0; i < B * Lk * rowe; ++i) KV[i] = rand_bf16();
    CHECK(ico_indexer_topk(0, q, k, w, NULL, NULL, B, Tq, Lk, H, d, Lk - Tq, KS, NULL, 0, idx, NULL, NULL, NULL, NULL) == 0);
    idx[1] = -1;                                            /* a hole */
    for (int j = 0; j < KS; ++j) idx[(Tq + 2) * KS + j] = -1;   /* an empty row */
    double *O = malloc(sizeof(double) * B * Tq * Hq * dv), *lse = malloc(sizeof(double) * B * Tq * Hq);
    CHECK(ico_sparse_attn(Q, KV, idx, B, Tq, Lk, Hq, dqk, dv, voff, rowe, KS, 0.25, NULL, 0, 0, O, lse) == 0);
    CHECK(isinf(lse[(Tq + 2) * Hq]) && O[(Tq + 2) * Hq * dv] == 0.0);
    CHECK(ico_sparse_attn(Q, KV, idx, B, Tq, Lk, Hq, dqk, dv, voff, rowe, KS, 0.25, NULL, 0, 0, O, NULL) == 0);
    CHECK(ico_dense_causal_attn(Q, KV, B, Tq, Lk, Hq, dqk, dv, voff, rowe, 0.25, Lk - Tq, O) == 0);
    CHECK(ico_dense_causal_attn(Q, KV, B, Tq, Lk, Hq, dqk, dv, voff, rowe, 0.25, 0, O) == 0);

    int32_t *idx2 = malloc(sizeof(int32_t) * B * Tq * KS);
    memcpy(idx2, idx, sizeof(int32_t) * B * Tq * KS);
    idx2[0] = (idx2[0] + 1) % Lk;
    const int32_t *layers[2] = {idx, idx2};
    uint64_t inter[4], sizes[2];
    CHECK(ico_topk_overlap(layers, 2, (long)B * Tq, KS, Lk, inter, sizes) == 0 && inter[0] == sizes[0] && inter[1] <= sizes[0]);
    double per[B * Tq], mean;
    CHECK(ico_cosine_rows(Q, Q, B * Tq, Hq * dqk, per, &mean) == 0 && fabs(mean - 1.0) < 1e-12);
    CHECK(ico_cosine_rows(Q, Q + 1, B * Tq - 1, Hq * dqk, NULL, &mean) == 0);

    free(q); free(k); free(q8); free(k8); free(w); free(qs); free(ks); free(sc); free(idx); free(idx2); free(sel); free(kth);
    free(nxt); free(mab); free(Q); free(KV); free(O); free(lse);
    puts("oracle sanitizer run ok");
    return 0;
}
