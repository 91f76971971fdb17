/*
 * CPU oracle for the IndexCache / DeepSeek-Sparse-Attention hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU library computes.  It shares no code, header, table or helper with
 * the HIP path and must never be linked into, imported by or called from it.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Everything is widened exactly to fp64 and accumulated in fp64, in the order
 * the definitions below state; no blocking, fusion or reordering.
 *
 * What is defined here and where it comes from:
 *   - indexer score  I[t,s] = sum_j w[t,j] * ReLU( q[t,j,:] . k[s,:] )
 *       the indexer of Sec. 2.1: every indexer head takes the dot product of
 *       the query with each earlier key, a ReLU gates it, the heads are summed
 *       with per-head weights (score vector I_t in R^L of Sec. 3 Notation).  The explicit formula, one key vector per position
 *       shared by all indexer heads and w outside the ReLU, is the reading
 *       this build takes for the cited DSA indexer.
 *   - T_t = Top-k(I_t) (Sec. 3 Notation), ties broken towards the lower
 *       position, fewer than k visible keys => all of them, -1 padded.
 *   - sparse core attention over exactly the selected rows (Sec. 2.1: the core
 *       attention sees nothing but the selected subset), MQA/MLA form
 *       with one shared KV row per position.
 *   - dense causal attention (textbook) used only to pin the sparse one.
 *   - pairwise cross-layer overlap of the index sets (App. A).
 *   - cosine similarity of two attention outputs (App. C); the exhaustive pattern search over
 *     a similarity matrix that pins the dynamic program lives in oracle.py.
 * The Full/Shared layer loop of Fig. 2(b) lives in oracle.py on top of these.
 *
 * Causality: key s is visible to query row i of a sequence iff
 *   s <= q_pos0 + i  and  s < Lk   (inclusive causal mask).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ICO_BF16 = 0, ICO_FP8_E4M3 = 1 };

/* ---- O1: exact widening ------------------------------------------------- */

/* bfloat16 is the upper half of an IEEE binary32. */
static double widen_bf16(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3 ("fn": finite + NaN, no infinity):
 * 1 sign, 4 exponent (bias 7), 3 mantissa; exponent 0 => subnormal m/8*2^-6;
 * S.1111.111 is NaN; S.1111.110 = 448 is the largest finite value. */
static double widen_e4m3(uint8_t b)
{
    int sign = b >> 7;
    int e = (b >> 3) & 0xF;
    int m = b & 0x7;
    double v;
    if (e == 0xF && m == 0x7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

double ico_widen_bf16(uint16_t h) { return widen_bf16(h); }
double ico_widen_e4m3(uint8_t b) { return widen_e4m3(b); }

static double elem(int dtype, const void *p, size_t i)
{
    if (dtype == ICO_BF16)
        return widen_bf16(((const uint16_t *)p)[i]);
    return widen_e4m3(((const uint8_t *)p)[i]);
}

/* ---- O2: indexer score of one (query row, key) pair ---------------------- */

static double score_pair(int dtype, const void *q, const void *k, const float *w,
                         const float *q_scale, const float *k_scale,
                         size_t qrow /* flat (b,i) */, size_t krow /* flat (b,s) */,
                         int H, int d)
{
    double total = 0.0;
    double sc = 1.0;
    if (dtype == ICO_FP8_E4M3)
        sc = (double)q_scale[qrow] * (double)k_scale[krow];
    for (int j = 0; j < H; ++j) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
            dot += elem(dtype, q, (qrow * H + j) * (size_t)d + c) *
                   elem(dtype, k, krow * (size_t)d + c);
        dot *= sc;
        if (dot < 0.0)
            dot = 0.0;
        total += (double)w[qrow * H + j] * dot;
    }
    return total;
}

static int n_visible(long q_pos0, int i, int Lk)
{
    long p = q_pos0 + i;
    if (p < 0)
        return 0;
    return (int)((p + 1 < (long)Lk) ? p + 1 : Lk);
}

/*
 * Scores for chosen query rows.  rows == NULL means all Tq rows (n_rows = Tq).
 * out is [B, n_rows, Lk] fp64; keys that the causal mask hides get -inf.
 */
int ico_indexer_scores(int dtype, const void *q, const void *k, const float *w,
                       const float *q_scale, const float *k_scale,
                       int B, int Tq, int Lk, int H, int d, long q_pos0,
                       const int *rows, int n_rows, double *out)
{
    if (!q || !k || !w || !out)
        return 1;
    if (dtype == ICO_FP8_E4M3 && (!q_scale || !k_scale))
        return 1;
    if (!rows)
        n_rows = Tq;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int r = 0; r < n_rows; ++r) {
            int i = rows ? rows[r] : r;
            int nv = n_visible(q_pos0, i, Lk);
            double *o = out + ((size_t)b * n_rows + r) * (size_t)Lk;
            for (int s = 0; s < Lk; ++s) {
                if (s < nv)
                    o[s] = score_pair(dtype, q, k, w, q_scale, k_scale,
                                      (size_t)b * Tq + i, (size_t)b * Lk + s, H, d);
                else
                    o[s] = -INFINITY;
            }
        }
    }
    return 0;
}

/* ---- O3: top-k with the fixed tie-break ---------------------------------- */

typedef struct {
    double score;
    int pos;
} cand_t;

/* Order: higher score first; equal scores => lower position first. */
static int cand_before(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->score > y->score)
        return -1;
    if (x->score < y->score)
        return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

/*
 * Select from one already-scored row: the first n = min(nv, k_sel) candidates in
 * the order above go to idx (in that order), the tail is -1.  Optional outputs:
 * sel (their scores, tail NaN), kth = score of the last selected, next = score
 * of the best unselected (-inf if there is none), mean_abs = mean |score| over
 * the visible keys.
 */
int ico_topk_row(const double *scores, int nv, int k_sel, int32_t *idx, double *sel,
                 double *kth, double *next, double *mean_abs)
{
    if (!scores || !idx || nv < 0 || k_sel <= 0)
        return 1;
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)(nv > 0 ? nv : 1));
    if (!c)
        return 2;
    double sum_abs = 0.0;
    for (int s = 0; s < nv; ++s) {
        c[s].score = scores[s];
        c[s].pos = s;
        sum_abs += fabs(scores[s]);
    }
    qsort(c, (size_t)nv, sizeof(cand_t), cand_before);
    int n = nv < k_sel ? nv : k_sel;
    for (int m = 0; m < k_sel; ++m) {
        idx[m] = m < n ? c[m].pos : -1;
        if (sel)
            sel[m] = m < n ? c[m].score : NAN;
    }
    if (kth)
        *kth = n > 0 ? c[n - 1].score : NAN;
    if (next)
        *next = nv > n ? c[n].score : -INFINITY;
    if (mean_abs)
        *mean_abs = nv > 0 ? sum_abs / nv : 0.0;
    free(c);
    return 0;
}

/*
 * Indexer + top-k for chosen rows (rows == NULL: all).  idx [B,n_rows,k_sel];
 * sel [B,n_rows,k_sel] (nullable); kth/next/mean_abs [B,n_rows] (nullable).
 */
int ico_indexer_topk(int dtype, const void *q, const void *k, const float *w,
                     const float *q_scale, const float *k_scale,
                     int B, int Tq, int Lk, int H, int d, long q_pos0, int k_sel,
                     const int *rows, int n_rows, int32_t *idx, double *sel,
                     double *kth, double *next, double *mean_abs)
{
    if (!q || !k || !w || !idx || k_sel <= 0)
        return 1;
    if (dtype == ICO_FP8_E4M3 && (!q_scale || !k_scale))
        return 1;
    if (!rows)
        n_rows = Tq;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int r = 0; r < n_rows; ++r) {
            int i = rows ? rows[r] : r;
            int nv = n_visible(q_pos0, i, Lk);
            double *sc = (double *)malloc(sizeof(double) * (size_t)(nv > 0 ? nv : 1));
            if (!sc) {
                bad = 1;
                continue;
            }
            for (int s = 0; s < nv; ++s)
                sc[s] = score_pair(dtype, q, k, w, q_scale, k_scale,
                                   (size_t)b * Tq + i, (size_t)b * Lk + s, H, d);
            size_t o = (size_t)b * n_rows + r;
            if (ico_topk_row(sc, nv, k_sel, idx + o * k_sel, sel ? sel + o * k_sel : NULL,
                             kth ? kth + o : NULL, next ? next + o : NULL,
                             mean_abs ? mean_abs + o : NULL))
                bad = 1;
            free(sc);
        }
    }
    return bad ? 2 : 0;
}

/* ---- O4: sparse MQA attention over the selected rows ---------------------- */

/*
 * Q [B,Tq,Hq,d_qk] bf16, KV [B,Lk,row_elems] bf16 (one shared KV head),
 * idx [B,Tq,k_sel] (entries < 0 are skipped).  For each chosen row and head:
 *   z_m = sm_scale * <Q[i,h,:], KV[idx_m, 0:d_qk]>
 *   p   = softmax(z) over the valid m
 *   O[i,h,e] = sum_m p_m * KV[idx_m, v_off + e],  e < d_v
 * out O [B,n_rows,Hq,d_v] fp64, lse [B,n_rows,Hq] fp64 (nullable; natural log of
 * sum exp z).  A row with no valid entry gives O = 0 and lse = -inf.
 * idx_rows_are_subset: 0 => idx has Tq rows and is indexed by the real row
 * number; 1 => idx has n_rows rows, aligned with `rows`.
 */
int ico_sparse_attn(const uint16_t *Q, const uint16_t *KV, const int32_t *idx,
                    int B, int Tq, int Lk, int Hq, int d_qk, int d_v, int v_off,
                    int row_elems, int k_sel, double sm_scale,
                    const int *rows, int n_rows, int idx_rows_are_subset,
                    double *O, double *lse)
{
    if (!Q || !KV || !idx || !O)
        return 1;
    if (d_qk > row_elems || v_off + d_v > row_elems)
        return 1;
    if (!rows)
        n_rows = Tq;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int r = 0; r < n_rows; ++r) {
            int i = rows ? rows[r] : r;
            const int32_t *id = idx + ((size_t)b * (idx_rows_are_subset ? n_rows : Tq) +
                                       (idx_rows_are_subset ? r : i)) * (size_t)k_sel;
            double *z = (double *)malloc(sizeof(double) * (size_t)k_sel);
            if (!z) {
                bad = 1;
                continue;
            }
            for (int h = 0; h < Hq; ++h) {
                const uint16_t *qv = Q + (((size_t)b * Tq + i) * Hq + h) * (size_t)d_qk;
                double zmax = -INFINITY;
                int any = 0;
                for (int m = 0; m < k_sel; ++m) {
                    if (id[m] < 0 || id[m] >= Lk) {
                        if (id[m] >= Lk)
                            bad = 1;
                        continue;
                    }
                    const uint16_t *kv = KV + ((size_t)b * Lk + id[m]) * (size_t)row_elems;
                    double dot = 0.0;
                    for (int c = 0; c < d_qk; ++c)
                        dot += widen_bf16(qv[c]) * widen_bf16(kv[c]);
                    z[m] = sm_scale * dot;
                    if (z[m] > zmax)
                        zmax = z[m];
                    any = 1;
                }
                double *o = O + (((size_t)b * n_rows + r) * Hq + h) * (size_t)d_v;
                for (int e = 0; e < d_v; ++e)
                    o[e] = 0.0;
                double denom = 0.0;
                if (any) {
                    for (int m = 0; m < k_sel; ++m)
                        if (id[m] >= 0 && id[m] < Lk)
                            denom += exp(z[m] - zmax);
                    for (int m = 0; m < k_sel; ++m) {
                        if (id[m] < 0 || id[m] >= Lk)
                            continue;
                        double p = exp(z[m] - zmax) / denom;
                        const uint16_t *kv = KV + ((size_t)b * Lk + id[m]) * (size_t)row_elems;
                        for (int e = 0; e < d_v; ++e)
                            o[e] += p * widen_bf16(kv[v_off + e]);
                    }
                }
                if (lse)
                    lse[((size_t)b * n_rows + r) * Hq + h] = any ? zmax + log(denom) : -INFINITY;
            }
            free(z);
        }
    }
    return bad ? 2 : 0;
}

/* ---- O6: dense causal attention (textbook), the pin for O4 ---------------- */

/* Same layouts; attends to every key s <= q_pos0 + i, s < Lk. O [B,Tq,Hq,d_v]. */
int ico_dense_causal_attn(const uint16_t *Q, const uint16_t *KV,
                          int B, int Tq, int Lk, int Hq, int d_qk, int d_v, int v_off,
                          int row_elems, double sm_scale, long q_pos0, double *O)
{
    if (!Q || !KV || !O)
        return 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < Tq; ++i) {
            int nv = n_visible(q_pos0, i, Lk);
            double *z = (double *)malloc(sizeof(double) * (size_t)(nv > 0 ? nv : 1));
            for (int h = 0; h < Hq; ++h) {
                const uint16_t *qv = Q + (((size_t)b * Tq + i) * Hq + h) * (size_t)d_qk;
                double zmax = -INFINITY;
                for (int s = 0; s < nv; ++s) {
                    const uint16_t *kv = KV + ((size_t)b * Lk + s) * (size_t)row_elems;
                    double dot = 0.0;
                    for (int c = 0; c < d_qk; ++c)
                        dot += widen_bf16(qv[c]) * widen_bf16(kv[c]);
                    z[s] = sm_scale * dot;
                    if (z[s] > zmax)
                        zmax = z[s];
                }
                double denom = 0.0;
                for (int s = 0; s < nv; ++s)
                    denom += exp(z[s] - zmax);
                double *o = O + (((size_t)b * Tq + i) * Hq + h) * (size_t)d_v;
                for (int e = 0; e < d_v; ++e)
                    o[e] = 0.0;
                for (int s = 0; s < nv; ++s) {
                    double p = exp(z[s] - zmax) / denom;
                    const uint16_t *kv = KV + ((size_t)b * Lk + s) * (size_t)row_elems;
                    for (int e = 0; e < d_v; ++e)
                        o[e] += p * widen_bf16(kv[v_off + e]);
                }
            }
            free(z);
        }
    }
    return 0;
}

/* ---- cross-layer top-k overlap (App. A) ---------------------------------
 * For every ordered pair of layers (i, j): how many of layer j's selected
 * positions layer i selected too, summed over the query rows, and the size of
 * layer i's sets, summed likewise.  The appendix reports |T(i) ^ T(j)| / k
 * averaged over rows that all hold k entries; with rows that hold fewer
 * (positions < k) the ratio of the two sums below is this build's reading:
 *   overlap(i, j) = sum_t |T_t(i) ^ T_t(j)| / sum_t |T_t(i)|.
 * idx: n_layers tensors [nq, k_sel], entries < 0 or >= Lk are not members;
 * the members of one row are distinct.  inter: [n_layers * n_layers],
 * sizes: [n_layers].  Plain marking of layer i's row, then counting j's. */
int ico_topk_overlap(const int32_t *const *idx, int n_layers, long nq, int k_sel, int Lk,
                     uint64_t *inter, uint64_t *sizes)
{
    if (!idx || !inter || !sizes || n_layers <= 0 || nq < 0 || k_sel <= 0 || Lk <= 0) return 1;
    unsigned char *mark = (unsigned char *)calloc((size_t)Lk, 1);
    if (!mark) return 2;
    memset(inter, 0, sizeof(uint64_t) * (size_t)n_layers * n_layers);
    memset(sizes, 0, sizeof(uint64_t) * (size_t)n_layers);
    for (long t = 0; t < nq; ++t) {
        for (int i = 0; i < n_layers; ++i) {
            const int32_t *ri = idx[i] + t * k_sel;
            for (int m = 0; m < k_sel; ++m)
                if (ri[m] >= 0 && ri[m] < Lk) {
                    mark[ri[m]] = 1;
                    sizes[i] += 1;
                }
            for (int j = 0; j < n_layers; ++j) {
                const int32_t *rj = idx[j] + t * k_sel;
                uint64_t c = 0;
                for (int m = 0; m < k_sel; ++m)
                    if (rj[m] >= 0 && rj[m] < Lk && mark[rj[m]]) c += 1;
                inter[(size_t)i * n_layers + j] += c;
            }
            for (int m = 0; m < k_sel; ++m)
                if (ri[m] >= 0 && ri[m] < Lk) mark[ri[m]] = 0;
        }
    }
    free(mark);
    return 0;
}

/* ---- similarity of two attention outputs (App. C) -------------------------
 * Cosine similarity of corresponding rows of two bf16 tensors [n_rows, row_len]
 * (one row = one query token's output over all heads), and its mean over the
 * rows: the appendix's "how well does layer j's index serve layer i" number is
 * this mean between the output under the layer's own indices and the output
 * under the reused ones.  Reading where the paper is silent: the cosine is
 * taken per token and averaged; a pair of all-zero rows counts as 1, a zero
 * row against a non-zero one as 0.  per_row may be NULL. */
int ico_cosine_rows(const uint16_t *A, const uint16_t *B, long n_rows, long row_len, double *per_row, double *mean)
{
    if (!A || !B || !mean || n_rows <= 0 || row_len <= 0) return 1;
    double acc = 0.0;
    for (long r = 0; r < n_rows; ++r) {
        double ab = 0.0, aa = 0.0, bb = 0.0;
        for (long c = 0; c < row_len; ++c) {
            const double x = widen_bf16(A[r * row_len + c]), y = widen_bf16(B[r * row_len + c]);
            ab += x * y;
            aa += x * x;
            bb += y * y;
        }
        double cs;
        if (aa == 0.0 && bb == 0.0) cs = 1.0;
        else if (aa == 0.0 || bb == 0.0) cs = 0.0;
        else cs = ab / (sqrt(aa) * sqrt(bb));
        if (per_row) per_row[r] = cs;
        acc += cs;
    }
    *mean = acc / (double)n_rows;
    return 0;
}

#ifdef _OPENMP
#include <omp.h>
int ico_num_threads(void) { return omp_get_max_threads(); }
#else
int ico_num_threads(void) { return 1; }
#endif
