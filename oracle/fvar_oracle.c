/*
 * CPU oracle for the late-scale block of a next-scale-prediction (VAR) model
 * run with FasterVAR's training-free reduction.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, loop-by-loop statement of
 * what the path computes, kept deliberately free of blocking, fusion or
 * reordering so it can be checked against the paper by eye.  Only the tests,
 * the smoke check and the benchmark's CPU-baseline leg may call it; the GPU
 * library shares no code with it and must never route through it.
 *
 * Arithmetic: every tensor is stored in fp32.  Every reduction (dot products,
 * row energies, LayerNorm statistics, softmax sums) is accumulated in double,
 * left to right, and rounded to fp32 once when stored, so each stored value is
 * the correctly rounded fp32 value of its defining sum to within double
 * rounding.  In particular a token score is fl32(sum_j x_ij^2) with the sum in
 * double: products of fp32 (or bf16) values are exact in double, so the stored
 * score does not depend on summation order except in vanishingly rare
 * double-rounding cases.
 *
 * Layouts: row-major.  Linear weights follow the "out,in" convention:
 * W[out][in], y = x W^T + b.  The KV cache of one sample is [L][H][Dh].
 *
 * Pins (tests, CPU only): closed forms for scores; brute-force ordering for
 * top-k including ties; softmax rows summing to one and special caches
 * (single key, all-equal keys); an fp64 framework cross-check of the dense
 * block; keep ratio 1.0 reproducing the dense block exactly; incremental cache
 * == block-causal mask; split-KV merge; lossless fill on exactly rank-r data;
 * normal equations and the Eckart-Young bound for the factors.
 * Parity unpinned: how close the pruned+filled output is to the true dense
 * output (the paper reports only image-level metrics for that).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- Representative-token scoring: Sec. "Representative Token Restoration",
 * the row energy ||F~_{k-1}^{(i)}||^2 in the sampling probability P_i. ---- */
void fvo_scores(const float *x, int M, int d, float *s)
{
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double acc = 0.0;
        for (int j = 0; j < d; ++j) {
            double v = (double)x[(size_t)i * d + j];
            acc += v * v;
        }
        s[i] = (float)acc;
    }
}

/* P_i = ||row_i||^2 / ||F||_F^2 (same section). */
void fvo_importance(const float *s, int M, float *P)
{
    double tot = 0.0;
    for (int i = 0; i < M; ++i) tot += (double)s[i];
    for (int i = 0; i < M; ++i) P[i] = (float)((double)s[i] / tot);
}

/* ---- The index set I: the k most important rows, deterministic reading:
 * order tokens by (score descending, index ascending), take the first k,
 * return them ascending; the complement ascending in `drop`. ---- */
typedef struct { float s; int32_t i; } fvo_pair;

static int fvo_pair_cmp(const void *pa, const void *pb)
{
    const fvo_pair *a = (const fvo_pair *)pa, *b = (const fvo_pair *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->i > b->i) - (a->i < b->i);   /* total order => qsort is safe */
}

void fvo_topk(const float *s, int M, int k, int32_t *keep, int32_t *drop)
{
    fvo_pair *p = (fvo_pair *)malloc(sizeof(fvo_pair) * (size_t)(M > 0 ? M : 1));
    uint8_t *kept = (uint8_t *)calloc((size_t)(M > 0 ? M : 1), 1);
    for (int i = 0; i < M; ++i) { p[i].s = s[i]; p[i].i = i; }
    qsort(p, (size_t)M, sizeof(fvo_pair), fvo_pair_cmp);
    for (int j = 0; j < k; ++j) kept[p[j].i] = 1;
    int a = 0, b = 0;
    for (int i = 0; i < M; ++i) {
        if (kept[i]) { if (keep) keep[a] = i; ++a; }
        else         { if (drop) drop[b] = i; ++b; }
    }
    free(p); free(kept);
}

/* ---- (M,d) -> (k,d): the reduced feature is the kept rows themselves. ---- */
void fvo_gather_rows(const float *x, const int32_t *idx, int k, int d, float *out)
{
    for (int j = 0; j < k; ++j)
        memcpy(out + (size_t)j * d, x + (size_t)idx[j] * d, sizeof(float) * (size_t)d);
}

/* ---- Pieces of the block phi.  The paper never opens phi; a plain
 * pre-LayerNorm transformer block (LN, QKV, softmax attention, output
 * projection, residual, LN, tanh-GELU MLP, residual) is assumed. ---- */
void fvo_layernorm(const float *x, int rows, int d, const float *gamma, const float *beta,
                   float eps, float *out)
{
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < rows; ++i) {
        const float *xr = x + (size_t)i * d;
        double mu = 0.0;
        for (int j = 0; j < d; ++j) mu += (double)xr[j];
        mu /= d;
        double var = 0.0;
        for (int j = 0; j < d; ++j) { double c = (double)xr[j] - mu; var += c * c; }
        var /= d;                                   /* biased variance */
        double rstd = 1.0 / sqrt(var + (double)eps);
        for (int j = 0; j < d; ++j) {
            double v = ((double)xr[j] - mu) * rstd;
            if (gamma) v *= (double)gamma[j];
            if (beta)  v += (double)beta[j];
            out[(size_t)i * d + j] = (float)v;
        }
    }
}

/* y[rows,out] = x[rows,in] * W[out,in]^T + bias */
void fvo_linear(const float *x, int rows, int in, const float *W, const float *bias, int out,
                float *y)
{
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < rows; ++i) {
        const float *xr = x + (size_t)i * in;
        for (int o = 0; o < out; ++o) {
            const float *wr = W + (size_t)o * in;
            double acc = bias ? (double)bias[o] : 0.0;
            for (int j = 0; j < in; ++j) acc += (double)xr[j] * (double)wr[j];
            y[(size_t)i * out + o] = (float)acc;
        }
    }
}

/* tanh-form GELU, in place */
void fvo_gelu_tanh(float *x, size_t n)
{
    const double c = 0.7978845608028654;           /* sqrt(2/pi) */
    #pragma omp parallel for schedule(static)
    for (long long i = 0; i < (long long)n; ++i) {
        double v = (double)x[i];
        x[i] = (float)(0.5 * v * (1.0 + tanh(c * (v + 0.044715 * v * v * v))));
    }
}

/* Softmax attention of n queries over L cached rows.
 * q:[n][H][Dh], K,V:[L][H][Dh], o:[n][H][Dh].
 * mask (optional): [n][L] bytes, nonzero = visible.  lse/psum (optional): [n][H],
 * log-sum-exp of the scaled logits and the sum of the stored fp32 probabilities. */
void fvo_attention(const float *q, const float *K, const float *V, int n, int L, int H, int Dh,
                   float scale, const uint8_t *mask, float *o, float *lse, float *psum)
{
    #pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        float  *prob  = (float  *)malloc(sizeof(float)  * (size_t)(L > 0 ? L : 1));
        #pragma omp for collapse(2) schedule(static)
        for (int i = 0; i < n; ++i) {
            for (int h = 0; h < H; ++h) {
                const float *qv = q + ((size_t)i * H + h) * Dh;
                double mx = -INFINITY;
                for (int t = 0; t < L; ++t) {
                    if (mask && !mask[(size_t)i * L + t]) { logit[t] = -INFINITY; continue; }
                    const float *kv = K + ((size_t)t * H + h) * Dh;
                    double acc = 0.0;
                    for (int c = 0; c < Dh; ++c) acc += (double)qv[c] * (double)kv[c];
                    logit[t] = acc * (double)scale;
                    if (logit[t] > mx) mx = logit[t];
                }
                double den = 0.0;
                for (int t = 0; t < L; ++t) den += exp(logit[t] - mx);
                double ps = 0.0;
                for (int t = 0; t < L; ++t) {
                    prob[t] = (float)(exp(logit[t] - mx) / den);
                    ps += (double)prob[t];
                }
                float *ov = o + ((size_t)i * H + h) * Dh;
                for (int c = 0; c < Dh; ++c) {
                    double acc = 0.0;
                    for (int t = 0; t < L; ++t)
                        acc += (double)prob[t] * (double)V[((size_t)t * H + h) * Dh + c];
                    ov[c] = (float)acc;
                }
                if (lse)  lse[(size_t)i * H + h]  = (float)(mx + log(den));
                if (psum) psum[(size_t)i * H + h] = (float)ps;
            }
        }
        free(logit); free(prob);
    }
}

/* Weights of one block; any bias / affine pointer may be NULL. */
typedef struct {
    const float *ln1_g, *ln1_b;
    const float *w_qkv, *b_qkv;   /* [3d][d], [3d]; output columns ordered q | k | v */
    const float *w_o,   *b_o;     /* [d][d] */
    const float *ln2_g, *ln2_b;
    const float *w_fc1, *b_fc1;   /* [F][d] */
    const float *w_fc2, *b_fc2;   /* [d][F] */
} fvo_weights;

/* The block phi on n rows of one sample (Alg. "FasterVAR": F^o = phi(.)).
 * x:[n][d].  Kc,Vc:[Lcap][H][Dh] with rows [0,len) valid on entry; the n new
 * key/value rows are appended at [len,len+n) in row order, and every query
 * attends to all len+n rows (all cached scales are <= the current one). */
void fvo_block_forward(const float *x, int n, int d, int H, int Dh, int F, const fvo_weights *w,
                       float eps, float scale, float *Kc, float *Vc, int len, float *y)
{
    size_t nd = (size_t)n * d;
    float *u   = (float *)malloc(sizeof(float) * nd);
    float *qkv = (float *)malloc(sizeof(float) * nd * 3);
    float *qq  = (float *)malloc(sizeof(float) * nd);
    float *att = (float *)malloc(sizeof(float) * nd);
    float *h1  = (float *)malloc(sizeof(float) * nd);
    float *hid = (float *)malloc(sizeof(float) * (size_t)n * F);

    fvo_layernorm(x, n, d, w->ln1_g, w->ln1_b, eps, u);
    fvo_linear(u, n, d, w->w_qkv, w->b_qkv, 3 * d, qkv);
    for (int i = 0; i < n; ++i) {
        memcpy(qq + (size_t)i * d,           qkv + (size_t)i * 3 * d,         sizeof(float) * (size_t)d);
        memcpy(Kc + ((size_t)len + i) * d,   qkv + (size_t)i * 3 * d + d,     sizeof(float) * (size_t)d);
        memcpy(Vc + ((size_t)len + i) * d,   qkv + (size_t)i * 3 * d + 2 * d, sizeof(float) * (size_t)d);
    }
    fvo_attention(qq, Kc, Vc, n, len + n, H, Dh, scale, NULL, att, NULL, NULL);
    fvo_linear(att, n, d, w->w_o, w->b_o, d, h1);
    for (size_t i = 0; i < nd; ++i) h1[i] = x[i] + h1[i];
    fvo_layernorm(h1, n, d, w->ln2_g, w->ln2_b, eps, u);
    fvo_linear(u, n, d, w->w_fc1, w->b_fc1, F, hid);
    fvo_gelu_tanh(hid, (size_t)n * F);
    fvo_linear(hid, n, F, w->w_fc2, w->b_fc2, d, y);
    for (size_t i = 0; i < nd; ++i) y[i] = h1[i] + y[i];

    free(u); free(qkv); free(qq); free(att); free(h1); free(hid);
}

/* Restoration of the full token map (Eq. "redefine" with each cached row
 * replaced by its rank-r restoration W_r F_r):
 *   Y^(i) = y_keep[pos(i)]                 for i in I,
 *   Y^(i) = sum_t W_c[i][t] * G_c[t][:]    otherwise.
 * y_keep:[k][d], Wc:[M][r], Gc:[r][d], Y:[M][d]. */
void fvo_lowrank_fill(const float *y_keep, const int32_t *keep, const int32_t *drop, int M, int k,
                      int d, int r, const float *Wc, const float *Gc, float *Y)
{
    for (int j = 0; j < k; ++j)
        memcpy(Y + (size_t)keep[j] * d, y_keep + (size_t)j * d, sizeof(float) * (size_t)d);
    #pragma omp parallel for schedule(static)
    for (int j = 0; j < M - k; ++j) {
        int i = drop[j];
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int t = 0; t < r; ++t)
                acc += (double)Wc[(size_t)i * r + t] * (double)Gc[(size_t)t * d + c];
            Y[(size_t)i * d + c] = (float)acc;
        }
    }
}

/* One pruned late-scale block step for one sample: score -> select -> gather
 * -> phi on the kept rows -> fill + scatter.  Outputs every intermediate the
 * GPU path is compared on. */
void fvo_pruned_step(const float *x, int M, int k, int d, int H, int Dh, int F, const fvo_weights *w,
                     float eps, float scale, float *Kc, float *Vc, int len, int r, const float *Wc,
                     const float *Gc, float *scores, int32_t *keep, int32_t *drop, float *y_keep,
                     float *Y)
{
    float *xk = (float *)malloc(sizeof(float) * (size_t)k * d);
    fvo_scores(x, M, d, scores);
    fvo_topk(scores, M, k, keep, drop);
    fvo_gather_rows(x, keep, k, d, xk);
    fvo_block_forward(xk, k, d, H, Dh, F, w, eps, scale, Kc, Vc, len, y_keep);
    fvo_lowrank_fill(y_keep, keep, drop, M, k, d, r, Wc, Gc, Y);
    free(xk);
}

/* Number of OpenMP threads the loops above use (reported next to oracle timings). */
#ifdef _OPENMP
#include <omp.h>
int fvo_num_threads(void) { return omp_get_max_threads(); }
#else
int fvo_num_threads(void) { return 1; }
#endif
