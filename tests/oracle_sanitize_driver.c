/*
 * Driver that runs every function of oracle/fvar_oracle.c once on small ragged shapes with
 * every buffer allocated at exactly the size the function's contract states, so that an
 * AddressSanitizer / UndefinedBehaviorSanitizer build (see test_oracle_pins.py) reports any
 * access past an end, any misaligned or overflowing arithmetic and any leak.  It checks no
 * values (the pins do that); it prints a checksum so that nothing is optimised away.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    const float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o, *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} fvo_weights;

void fvo_scores(const float *x, int M, int d, float *s);
void fvo_importance(const float *s, int M, float *P);
void fvo_topk(const float *s, int M, int k, int32_t *keep, int32_t *drop);
void fvo_gather_rows(const float *x, const int32_t *idx, int k, int d, float *out);
void fvo_layernorm(const float *x, int rows, int d, const float *gamma, const float *beta, float eps,
                   float *y);
void fvo_linear(const float *x, int rows, int in, const float *W, const float *bias, int out, float *y);
void fvo_gelu_tanh(float *x, size_t n);
void fvo_attention(const float *q, const float *K, const float *V, int n, int L, int H, int Dh,
                   float scale, const uint8_t *mask, float *o, float *lse, float *psum);
void fvo_block_forward(const float *x, int n, int d, int H, int Dh, int F, const fvo_weights *w,
                       float eps, float scale, float *Kc, float *Vc, int len, float *y);
void fvo_lowrank_fill(const float *y_keep, const int32_t *keep, const int32_t *drop, int M, int k,
                      int d, int r, const float *Wc, const float *Gc, float *Y);
void fvo_pruned_step(const float *x, int M, int k, int d, int H, int Dh, int F, const fvo_weights *w,
                     float eps, float scale, float *Kc, float *Vc, int len, int r, const float *Wc,
                     const float *Gc, float *scores, int32_t *keep, int32_t *drop, float *y_keep,
                     float *Y);
int fvo_num_threads(void);

static uint32_t rng = 12345u;
static float rnd(void)
{
    rng = rng * 1664525u + 1013904223u;
    return (float)((int32_t)(rng >> 8) % 2001 - 1000) * 1e-3f;
}
static float *buf(size_t n)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    if (!p) exit(2);
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
static double sum(const float *p, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += (double)p[i];
    return s;
}

int main(void)
{
    enum { M = 37, d = 24, H = 3, Dh = 8, F = 40, k = 11, r = 5, len = 13 };
    double chk = 0.0;
    float *x = buf((size_t)M * d);
    fvo_weights w;
    float *ln1_g = buf(d), *ln1_b = buf(d), *ln2_g = buf(d), *ln2_b = buf(d);
    float *w_qkv = buf((size_t)3 * d * d), *b_qkv = buf(3 * d), *w_o = buf((size_t)d * d), *b_o = buf(d);
    float *w_fc1 = buf((size_t)F * d), *b_fc1 = buf(F), *w_fc2 = buf((size_t)d * F), *b_fc2 = buf(d);
    w.ln1_g = ln1_g; w.ln1_b = ln1_b; w.w_qkv = w_qkv; w.b_qkv = b_qkv; w.w_o = w_o; w.b_o = b_o;
    w.ln2_g = ln2_g; w.ln2_b = ln2_b; w.w_fc1 = w_fc1; w.b_fc1 = b_fc1; w.w_fc2 = w_fc2; w.b_fc2 = b_fc2;

    /* the whole pruned step: the cache holds exactly len + k rows */
    float *Kc = buf((size_t)(len + k) * d), *Vc = buf((size_t)(len + k) * d);
    float *Wc = buf((size_t)M * r), *Gc = buf((size_t)r * d);
    float *scores = buf(M), *y_keep = buf((size_t)k * d), *Y = buf((size_t)M * d);
    int32_t *keep = (int32_t *)malloc(sizeof(int32_t) * k);
    int32_t *drop = (int32_t *)malloc(sizeof(int32_t) * (M - k));
    fvo_pruned_step(x, M, k, d, H, Dh, F, &w, 1e-6f, 0.35f, Kc, Vc, len, r, Wc, Gc, scores, keep, drop,
                    y_keep, Y);
    chk += sum(Y, (size_t)M * d) + sum(scores, M) + keep[k - 1] + drop[M - k - 1];

    /* no affine, no biases; dense block on all rows with an empty cache prefix */
    fvo_weights w0 = {0, 0, w_qkv, 0, w_o, 0, 0, 0, w_fc1, 0, w_fc2, 0};
    float *K0 = buf((size_t)M * d), *V0 = buf((size_t)M * d), *y0 = buf((size_t)M * d);
    fvo_block_forward(x, M, d, H, Dh, F, &w0, 1e-6f, 0.35f, K0, V0, 0, y0);
    chk += sum(y0, (size_t)M * d);

    /* selection edge cases: nothing kept, everything kept, ties */
    float *P = buf(M);
    fvo_importance(scores, M, P);
    chk += sum(P, M);
    int32_t *all = (int32_t *)malloc(sizeof(int32_t) * M), *none = (int32_t *)malloc(sizeof(int32_t));
    fvo_topk(scores, M, M, all, none);
    fvo_topk(scores, M, 0, none, all);
    for (int i = 0; i < M; ++i) scores[i] = (float)(i % 3);
    fvo_topk(scores, M, k, keep, drop);
    chk += keep[0] + all[M - 1];

    /* masked attention with the optional outputs; one key only */
    enum { n = 5, L = 9 };
    float *q = buf((size_t)n * H * Dh), *Ka = buf((size_t)L * H * Dh), *Va = buf((size_t)L * H * Dh);
    float *o = buf((size_t)n * H * Dh), *lse = buf((size_t)n * H), *ps = buf((size_t)n * H);
    uint8_t *mask = (uint8_t *)malloc((size_t)n * L);
    for (int i = 0; i < n * L; ++i) mask[i] = (uint8_t)(i % L <= i / L + 2);
    fvo_attention(q, Ka, Va, n, L, H, Dh, 0.35f, mask, o, lse, ps);
    fvo_attention(q, Ka, Va, n, 1, H, Dh, 0.35f, NULL, o, NULL, NULL);
    chk += sum(o, (size_t)n * H * Dh) + sum(lse, (size_t)n * H);

    /* the row kernels on their own, a single row and a single column */
    float *g1 = buf(d), *l1 = buf(d), *lin = buf(7);
    fvo_gather_rows(x, keep, 1, d, g1);
    fvo_layernorm(g1, 1, d, NULL, NULL, 1e-6f, l1);
    fvo_linear(l1, 1, d, w_fc1, NULL, 7, lin);
    fvo_gelu_tanh(lin, 7);
    fvo_lowrank_fill(y_keep, keep, drop, M, k, d, r, Wc, Gc, Y);
    chk += sum(lin, 7) + sum(Y, (size_t)M * d);

    free(x); free(ln1_g); free(ln1_b); free(ln2_g); free(ln2_b); free(w_qkv); free(b_qkv); free(w_o);
    free(b_o); free(w_fc1); free(b_fc1); free(w_fc2); free(b_fc2); free(Kc); free(Vc); free(Wc); free(Gc);
    free(scores); free(y_keep); free(Y); free(keep); free(drop); free(K0); free(V0); free(y0); free(P);
    free(all); free(none); free(q); free(Ka); free(Va); free(o); free(lse); free(ps); free(mask);
    free(g1); free(l1); free(lin);
    printf("threads %d checksum %.6f\n", fvo_num_threads(), chk);
    return chk == chk ? 0 : 3;
}
