/*
 * SALS decode-step attention: reference oracle (TEST INFRASTRUCTURE ONLY).
 *
 * A plain, slow, fp64 CPU implementation of "Sparse Attention in Latent
 * Space" (arXiv 2510.24273), Algorithm 1, one function per step, written
 * from the paper's definitions.  It shares no code with the HIP library and
 * must never be called from the product path: only the test-suite, the
 * smoke check and the bench's cpu_baseline leg may use it.
 *
 * Conventions (all arrays dense, row-major, double):
 *   U    [D_kv x r]  joint projector U_r of Sec. 4.2 (column-orthonormal in
 *                    the paper; nothing here assumes it).  D_kv = H_kv * d.
 *   Kc   [S x r]     latent key cache  K~ = K U_r      (Eq. 1, Sec. 4.2)
 *   Vc   [S x r]     latent value cache (same construction with U_v; the
 *                    paper's traffic model of Sec. 4.5 counts low-rank key
 *                    and value caches of k*r elements each)
 *   q    [H x d]     pre-RoPE query heads; query head h reads KV head
 *                    g(h) = h / (H / H_kv)
 * Token t of the cache sits at RoPE position t; the query position is given.
 *
 * Every pin of these functions lives in tests/test_oracle_pins.py.
 * Parity status: every function below is pinned there, except closeness of
 * the sparse output to *dense* attention on real model activations, which is
 * the paper's accuracy claim and stays "parity unpinned".
 *
 * OpenMP is used only over independent output rows.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int sals_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sum the query heads that share a KV head (identity when H == H_kv).
 * The paper projects "the query" with a D_kv-wide projector and is silent on
 * grouped-query models; summing per group makes the latent score equal
 * sum_h q_h . k_{g(h)} exactly when U U^T = I (Eq. 2). */
void sals_oracle_group_sum(const double *q, int H, int H_kv, int d, double *q_sum)
{
    int G = H / H_kv;
    for (int g = 0; g < H_kv; ++g)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int m = 0; m < G; ++m)
                acc += q[(size_t)(g * G + m) * d + c];
            q_sum[(size_t)g * d + c] = acc;
        }
}

/* Latent projection  x~ = U_r^T x  (Sec. 4.3; Algorithm 1, projection step).
 * x [D], U [D x r]  ->  xt [r]. */
void sals_oracle_project(const double *x, const double *U, int D, int r, double *xt)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < r; ++i) {
        double acc = 0.0;
        for (int c = 0; c < D; ++c)
            acc += U[(size_t)c * r + i] * x[c];
        xt[i] = acc;
    }
}

/* Latent score  s_j = q~_{:r*} . k~_{j,:r*}  (Sec. 4.3; Algorithm 1, score
 * step).  Raw dot products: no 1/sqrt(d), no softmax, no RoPE. */
void sals_oracle_scores(const double *qt, const double *Kc, int S, int r, int r_score,
                        double *s)
{
#pragma omp parallel for schedule(static)
    for (int j = 0; j < S; ++j) {
        double acc = 0.0;
        for (int i = 0; i < r_score; ++i)
            acc += qt[i] * Kc[(size_t)j * r + i];
        s[j] = acc;
    }
}

typedef struct { double s; int32_t j; } scored_t;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

/* Critical-token selection  C = TopK(s, k)  (Algorithm 1, selection step),
 * composed with always-kept sink and recent tokens as in Sec. 5.2 (x sink,
 * y critical, z recent).  Sinks [0,n_sink) and the recent window
 * [S-n_recent,S) are kept unconditionally and are not candidates; the
 * top_k largest of the remaining scores are added (ties: smaller index
 * first).  If the cache has no more than top_k+n_sink+n_recent tokens,
 * every token is selected.
 * idx receives: sinks ascending, critical tokens by decreasing score, recent
 * ascending.  Returns |C|. */
int sals_oracle_topk(const double *s, int S, int top_k, int n_sink, int n_recent,
                     int32_t *idx)
{
    int n = 0;
    if (S <= top_k + n_sink + n_recent) {
        for (int j = 0; j < S; ++j) idx[n++] = j;
        return n;
    }
    int lo = n_sink, hi = S - n_recent, n_cand = hi - lo;
    scored_t *cand = (scored_t *)malloc((size_t)(n_cand > 0 ? n_cand : 1) * sizeof(scored_t));
    for (int j = lo; j < hi; ++j) { cand[j - lo].s = s[j]; cand[j - lo].j = j; }
    qsort(cand, (size_t)n_cand, sizeof(scored_t), by_score_desc_then_index);
    for (int j = 0; j < n_sink; ++j) idx[n++] = j;
    for (int m = 0; m < top_k; ++m) idx[n++] = cand[m].j;
    for (int j = hi; j < S; ++j) idx[n++] = j;
    free(cand);
    return n;
}

/* Selective reconstruction  X_C = X~_C U_r^T  (Algorithm 1, reconstruction
 * step; Sec. 4.4): all r latent coordinates, only the selected rows.
 * Xc [S x r], idx [n], U [D x r]  ->  X [n x D]. */
void sals_oracle_reconstruct(const double *Xc, const int32_t *idx, int n, const double *U,
                             int D, int r, double *X)
{
#pragma omp parallel for schedule(static)
    for (int j = 0; j < n; ++j) {
        const double *row = Xc + (size_t)idx[j] * r;
        for (int c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int i = 0; i < r; ++i)
                acc += row[i] * U[(size_t)c * r + i];
            X[(size_t)j * D + c] = acc;
        }
    }
}

/* Rotary position embedding of n_vec vectors of width d, vector v at integer
 * position pos[v / vec_per_pos] (Algorithm 1, RoPE step; the paper cites the
 * standard RoPE and fixes neither pairing nor frequency rescaling).
 * Frequency of pair i is theta^(-2i/d).  style 0: pair (i, i+d/2);
 * style 1: pair (2i, 2i+1).  In place. */
void sals_oracle_rope(double *x, int n_vec, int d, const int32_t *pos, int vec_per_pos,
                      double theta, int style)
{
    int half = d / 2;
#pragma omp parallel for schedule(static)
    for (int v = 0; v < n_vec; ++v) {
        double p = (double)pos[v / vec_per_pos];
        double *xv = x + (size_t)v * d;
        for (int i = 0; i < half; ++i) {
            double phi = p * pow(theta, -2.0 * (double)i / (double)d);
            double c = cos(phi), sn = sin(phi);
            int a = style == 0 ? i : 2 * i;
            int b = style == 0 ? i + half : 2 * i + 1;
            double xa = xv[a], xb = xv[b];
            xv[a] = xa * c - xb * sn;
            xv[b] = xb * c + xa * sn;
        }
    }
}

/* Sparse softmax attention over the selected set (Eq. 5; Algorithm 1,
 * softmax and output steps): per query head h with KV head g(h),
 *   l_j = qR[h] . KR[j,g] / sqrt(d),  p = softmax_j(l),  y[h] = sum_j p_j V[j,g].
 * qR [H x d], KR and V [n x H_kv x d]  ->  y [H x d]; if p_out is not NULL it
 * receives the probabilities [H x n]. */
void sals_oracle_attend(const double *qR, const double *KR, const double *V, int n, int H,
                        int H_kv, int d, double *y, double *p_out)
{
    int G = H / H_kv;
    size_t D = (size_t)H_kv * d;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        int g = h / G;
        double *l = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
        double m = -INFINITY;
        for (int j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c)
                acc += qR[(size_t)h * d + c] * KR[(size_t)j * D + (size_t)g * d + c];
            l[j] = acc / sqrt((double)d);
            if (l[j] > m) m = l[j];
        }
        double z = 0.0;
        for (int j = 0; j < n; ++j) { l[j] = exp(l[j] - m); z += l[j]; }
        for (int c = 0; c < d; ++c) y[(size_t)h * d + c] = 0.0;
        for (int j = 0; j < n; ++j) {
            double p = l[j] / z;
            if (p_out) p_out[(size_t)h * n + j] = p;
            for (int c = 0; c < d; ++c)
                y[(size_t)h * d + c] += p * V[(size_t)j * D + (size_t)g * d + c];
        }
        free(l);
    }
}

/* Steps 4-9 of Algorithm 1 for one sequence, given the selected set:
 * reconstruct K_C and V_C, rotate q and K_C, attend.  y [H x d]. */
void sals_oracle_sparse_attend(const double *q, int q_pos, const double *Kc, const double *Vc,
                               const double *Uk, const double *Uv, const int32_t *idx, int n,
                               int H, int H_kv, int d, int r, double theta, int rope_style,
                               double *y)
{
    int D = H_kv * d;
    size_t nn = (size_t)(n > 0 ? n : 1);
    double *KC = (double *)malloc(nn * D * sizeof(double));
    double *VC = (double *)malloc(nn * D * sizeof(double));
    double *qR = (double *)malloc((size_t)H * d * sizeof(double));
    sals_oracle_reconstruct(Kc, idx, n, Uk, D, r, KC);
    sals_oracle_reconstruct(Vc, idx, n, Uv, D, r, VC);
    memcpy(qR, q, (size_t)H * d * sizeof(double));
    int32_t qp = q_pos;
    sals_oracle_rope(qR, H, d, &qp, H, theta, rope_style);
    sals_oracle_rope(KC, n * H_kv, d, idx, H_kv, theta, rope_style);
    sals_oracle_attend(qR, KC, VC, n, H, H_kv, d, y, NULL);
    free(KC); free(VC); free(qR);
}

/* Whole decode step of Algorithm 1 for one sequence whose new token has
 * already been appended (or with an explicit query position): project,
 * score, select, reconstruct, rotate, attend.  Optional outputs (may be
 * NULL): qt_out [r], s_out [S], idx_out [top_k+n_sink+n_recent], n_sel_out. */
void sals_oracle_decode_step(const double *q, int q_pos, const double *Kc, const double *Vc,
                             const double *Uk, const double *Uv, int S, int H, int H_kv,
                             int d, int r, int r_score, int top_k, int n_sink, int n_recent,
                             double theta, int rope_style, double *y, double *qt_out,
                             double *s_out, int32_t *idx_out, int32_t *n_sel_out)
{
    int D = H_kv * d;
    int k_tot = top_k + n_sink + n_recent;
    double *q_sum = (double *)malloc((size_t)D * sizeof(double));
    double *qt = (double *)malloc((size_t)r * sizeof(double));
    double *s = (double *)malloc((size_t)(S > 0 ? S : 1) * sizeof(double));
    int32_t *idx = (int32_t *)malloc((size_t)(k_tot > 0 ? k_tot : 1) * sizeof(int32_t));
    sals_oracle_group_sum(q, H, H_kv, d, q_sum);
    sals_oracle_project(q_sum, Uk, D, r, qt);
    sals_oracle_scores(qt, Kc, S, r, r_score, s);
    int n = sals_oracle_topk(s, S, top_k, n_sink, n_recent, idx);
    sals_oracle_sparse_attend(q, q_pos, Kc, Vc, Uk, Uv, idx, n, H, H_kv, d, r, theta,
                              rope_style, y);
    if (qt_out) memcpy(qt_out, qt, (size_t)r * sizeof(double));
    if (s_out) memcpy(s_out, s, (size_t)S * sizeof(double));
    if (idx_out) memcpy(idx_out, idx, (size_t)n * sizeof(int32_t));
    if (n_sel_out) *n_sel_out = n;
    free(q_sum); free(qt); free(s); free(idx);
}
