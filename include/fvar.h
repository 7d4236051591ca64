/*
 * fvar.h -- C ABI of the late-scale block of a next-scale-prediction (VAR)
 * model run with FasterVAR's training-free token reduction, for AMD MI355X
 * (gfx950).
 *
 * One call sequence processes one transformer block at one late scale for a
 * batch of B samples:
 *
 *     fvar_score_select          x[B,M,d]            -> idx_keep[B,k], idx_drop[B,M-k]
 *     fvar_block_forward_pruned  x, idx_keep, KV     -> y_keep[B,k,d]   (appends k K/V rows)
 *     fvar_lowrank_fill          y_keep, idx, W_c,G_c-> y[B,M,d]
 *
 * and fvar_block_forward_dense is the unreduced control (x[B,M,d] -> y[B,M,d],
 * appends M K/V rows).  fvar_cache_factors builds W_c, G_c from the cached
 * counterpart feature.  The variant with a random-projection input is
 *
 *     fvar_rp_project            Q^T, x[B,M,d]       -> f_r[B,r,d]
 *     fvar_block_forward_dense   f_r (as r tokens)   -> y_keep[B,r,d]   (appends r K/V rows)
 *     fvar_cache_fill            y_keep, idx, cache  -> y[B,M,d]
 *
 * fvar_upsample_tokens brings a cached token map (or the thin factor W_c of its
 * rank-r form) from the previous scale's grid to the current one.
 *
 * Conventions common to every call
 *  - Every tensor pointer is DEVICE memory owned by the caller, row-major,
 *    contiguous, 16-byte aligned, of element type `fvar_config.dtype`
 *    (bf16 or fp32) unless a different type is written in the signature.
 *    The library never allocates or frees device memory; scratch space is the
 *    caller's workspace buffer.
 *  - Linear weights are stored "out,in": W[out][in], y = x W^T + b.
 *  - `stream` is a hipStream_t (passed as void*; NULL = the null stream).  All
 *    calls only enqueue work on it and return without synchronising.  The
 *    returned status covers argument validation and launch errors, not kernel
 *    completion.
 *  - Arguments are validated before anything is enqueued: FVAR_ERR_INVALID_ARG,
 *    FVAR_ERR_UNSUPPORTED and FVAR_ERR_WORKSPACE mean that nothing has been
 *    launched.  FVAR_ERR_HIP reports a failed runtime call or kernel launch and
 *    may come after earlier kernels of the same call were enqueued; the outputs
 *    are then undefined.  fvar_last_error() returns a text for the last failing
 *    call on that context.
 *  - A context may be used from one thread at a time.  State outside a context:
 *    a per-device table of the address of the built-in scratch array used by
 *    fvar_score_select_static (filled under a mutex on a device's first call),
 *    and a thread-local pointer that exists only while a call with per-kernel
 *    timing switched on is enqueueing its kernels.
 *  - Index arrays are int32, strictly ascending per sample and in range; this is
 *    the caller's contract for fvar_block_forward_pruned / fvar_lowrank_fill /
 *    fvar_cache_fill (fvar_score_select produces arrays that satisfy it).
 *    fvar_debug_checks() makes the library verify it.
 *  - Size limits of the block calls: B*rows <= 2^24, B <= 8191, and every operand
 *    matrix (B*rows x max(hidden, ffn_hidden) elements) below 4 GiB, because the
 *    linear-layer kernels use 32-bit byte offsets inside a matrix; larger calls
 *    return FVAR_ERR_UNSUPPORTED.
 */
#ifndef FVAR_H
#define FVAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FVAR_OK = 0,
    FVAR_ERR_INVALID_ARG = 1,   /* null / misaligned pointer, size out of range, inconsistent geometry */
    FVAR_ERR_UNSUPPORTED = 2,   /* valid request outside what the kernels implement */
    FVAR_ERR_WORKSPACE = 3,     /* workspace missing or smaller than fvar_*_workspace_bytes() */
    FVAR_ERR_HIP = 4            /* a HIP runtime call or kernel launch failed */
} fvar_status;

typedef enum { FVAR_F32 = 0, FVAR_BF16 = 1 } fvar_dtype;

/* Immutable geometry of the model the block belongs to.
 * scale_hw holds 2*num_scales ints (h_1,w_1,...,h_K,w_K): the predefined scale schedule
 * (paper, Sec. "Preliminary": token map R_k has h_k x w_k tokens).  It is copied. */
typedef struct {
    int32_t hidden;        /* d */
    int32_t heads;         /* H, heads * head_dim == hidden */
    int32_t head_dim;      /* 64 or 128 */
    int32_t ffn_hidden;    /* F, MLP width */
    int32_t num_scales;    /* K (may be 0 if the schedule helpers are not used) */
    const int32_t *scale_hw;
    fvar_dtype dtype;      /* activations, weights, KV cache, factors */
    float ln_eps;          /* LayerNorm epsilon; 0 selects 1e-6 */
    float attn_scale;      /* softmax scale; 0 selects 1/sqrt(head_dim) */
} fvar_config;

/* Weights of one block phi (paper: F^o = phi(F~); phi itself is never opened there; this
 * library implements a plain pre-LayerNorm block:
 *   u = LN1(x); [q|k|v] = u W_qkv^T + b_qkv; o = softmax(scale q K^T) V over the whole cache;
 *   h = x + o W_o^T + b_o;  y = h + GELU_tanh(LN2(h) W_fc1^T + b_fc1) W_fc2^T + b_fc2 ).
 * Any LayerNorm affine pointer or bias pointer may be NULL (gamma=1, beta=0, bias=0). */
typedef struct {
    const void *ln1_g, *ln1_b;   /* [d] */
    const void *w_qkv, *b_qkv;   /* [3d][d], [3d]; output features ordered q | k | v, head h = columns [h*Dh,(h+1)*Dh) */
    const void *w_o, *b_o;       /* [d][d], [d] */
    const void *ln2_g, *ln2_b;   /* [d] */
    const void *w_fc1, *b_fc1;   /* [F][d], [F] */
    const void *w_fc2, *b_fc2;   /* [d][F], [d] */
} fvar_block_weights;

/* Multi-scale KV cache of one block: k and v are [B][capacity][H][Dh]; rows [0,len) of every
 * sample hold the keys/values of the earlier scales.  The forward calls write the new rows at
 * [len, len+rows) and read [0, len+rows); they do not change `len` (the caller advances it). */
typedef struct {
    void *k, *v;
    int32_t capacity;
    int32_t len;
} fvar_kv;

typedef struct fvar_ctx fvar_ctx;
typedef void *fvar_stream;

/* Create / destroy a context for one geometry on the current HIP device.  Host-only work. */
fvar_status fvar_create(const fvar_config *cfg, fvar_ctx **out);
void fvar_destroy(fvar_ctx *ctx);
const char *fvar_last_error(const fvar_ctx *ctx);
const char *fvar_status_string(fvar_status s);

/* k = ceil(M * keep_num / keep_den) in integer arithmetic, clamped to [1, M]; -1 on bad input.
 * (The paper fixes the number of rows r that enter the block; a keep ratio is turned into a
 * row count here so that no float rounding can change it.) */
int32_t fvar_keep_count(int32_t M, int32_t keep_num, int32_t keep_den);
/* M = h_k * w_k of scale `scale_index` (0-based) and L_prev = sum of the earlier scales' tokens;
 * -1 if the index is out of range. */
int32_t fvar_scale_tokens(const fvar_ctx *ctx, int32_t scale_index);
int32_t fvar_scale_prev_len(const fvar_ctx *ctx, int32_t scale_index);

/* Workspace sizes in bytes (multiples of 256).  `rows` is the number of rows per sample that
 * pass through the block: k for the pruned call, M for the dense call. */
size_t fvar_select_workspace_bytes(const fvar_ctx *ctx, int32_t B, int32_t M);
size_t fvar_block_workspace_bytes(const fvar_ctx *ctx, int32_t B, int32_t rows);

/* Representative-token selection (paper, Sec. "Representative Token Restoration": rows of the
 * block INPUT are ranked by their energy ||row_i||^2, the numerator of the sampling
 * probability P_i; the index set I holds the most important rows).  Deterministic reading:
 *   s_i = fl32(sum_j x_ij^2)   (products and sum in fp64, rounded once)
 *   I   = the k indices that come first under (s descending, index ascending).
 * x:[B,M,d] or NULL when scores_in is given.  scores_in:[B,M] fp32 or NULL: if given, scoring
 * is skipped and selection runs on these values (any finite floats; -0 == +0).
 * scores_out:[B,M] fp32 or NULL.  idx_keep:[B,k] and idx_drop:[B,M-k] (NULL allowed) receive
 * the kept / pruned token indices in ascending order.  1 <= k <= M <= 1<<20.
 * ws: at least fvar_select_workspace_bytes(ctx,B,M). */
fvar_status fvar_score_select(fvar_ctx *ctx, fvar_stream stream, const void *x, int32_t B,
                              int32_t M, int32_t k, const float *scores_in, float *scores_out,
                              int32_t *idx_keep, int32_t *idx_drop, void *ws, size_t ws_bytes);

/* The same selection for callers that cannot allocate device memory or carry a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * scores live in a fixed device array built into the library (4 MiB per GPU, held until the
 * process ends) instead of caller workspace.  No hipMalloc / hipFree, no workspace argument.
 * Requires B*M <= 1048576 (FVAR_ERR_UNSUPPORTED beyond that; use fvar_score_select).  x is
 * required; results are bit-identical to fvar_score_select.  Every call on one GPU uses the
 * same array: calls that overlap in time on one GPU (different streams or threads) race and
 * must be serialised by the caller.  The array keeps the previous call's scores; a call
 * rewrites every entry it reads, so nothing is cleared. */
fvar_status fvar_score_select_static(fvar_ctx *ctx, fvar_stream stream, const void *x, int32_t B,
                                     int32_t M, int32_t k, int32_t *idx_keep, int32_t *idx_drop);

/* Vanilla block on every token of the scale (paper, Alg. "FasterVAR", establishment stages:
 * F_k^o = phi(F~_{k-1})).  x:[B,M,d] -> y:[B,M,d]; writes M new K/V rows per sample at
 * kv->len and attends over kv->len + M rows.  Requires kv->len + M <= kv->capacity.
 * x and y must not overlap.  ws: at least fvar_block_workspace_bytes(ctx,B,M). */
fvar_status fvar_block_forward_dense(fvar_ctx *ctx, fvar_stream stream,
                                     const fvar_block_weights *w, const void *x, int32_t B,
                                     int32_t M, const fvar_kv *kv, void *y, void *ws,
                                     size_t ws_bytes);

/* Block on the reduced (k,d) feature (paper, Sec. "Plug-and-Play Acceleration": the (M,d) input
 * is replaced by k rows; Alg. "FasterVAR", fidelity stage: F_r^o = phi(.)).  The k rows are
 * the rows idx_keep of x, in idx_keep order; only they produce queries, keys and values, so
 * attention runs over kv->len + k rows and k rows are appended to the cache.
 * x:[B,M,d], idx_keep:[B,k] (NULL with k == M means identity), y_keep:[B,k,d] compact.
 * ws: at least fvar_block_workspace_bytes(ctx,B,k). */
fvar_status fvar_block_forward_pruned(fvar_ctx *ctx, fvar_stream stream,
                                      const fvar_block_weights *w, const void *x, int32_t B,
                                      int32_t M, const int32_t *idx_keep, int32_t k,
                                      const fvar_kv *kv, void *y_keep, void *ws, size_t ws_bytes);

/* Restoration of the full token map (paper, Eq. "redefine": rows in I come from the block
 * output, the others from the cached counterpart feature; here each cached row is given in the
 * rank-r restored form W_r F_r of Sec. "Random Projection" / Eq. "lstsq"):
 *   y[b,i,:] = y_keep[b,j,:]                  if i == idx_keep[b,j]
 *   y[b,i,:] = sum_t w_c[b,i,t] * g_c[b,t,:]  if i is in idx_drop[b,:]
 * y_keep:[B,k,d], w_c:[B,M,r], g_c:[B,r,d], y:[B,M,d] (must not overlap y_keep).
 * 1 <= r <= 256, r a multiple of 8 for bf16 (of 4 for fp32).  k == M (idx_drop unused) is a
 * plain scatter.  Accumulation in fp32.  No workspace. */
fvar_status fvar_lowrank_fill(fvar_ctx *ctx, fvar_stream stream, const void *y_keep,
                              const int32_t *idx_keep, const int32_t *idx_drop, int32_t B,
                              int32_t M, int32_t k, int32_t r, const void *w_c, const void *g_c,
                              void *y);

/* The same restoration that also returns the row energies of the map it writes,
 *   scores_out[b,i] = fl32(sum_j y[b,i,j]^2)   (exact products of the stored elements, fp64 sum),
 * i.e. the selection scores of the NEXT block (paper, Sec. "Representative Token Restoration":
 * rows are ranked by the energy of the block input, and this map is the next block's input):
 * fvar_score_select can then run with scores_in = scores_out and never reads the map.  The
 * kernels that write y accumulate the energy of what they store per 128-column slab; a second
 * small kernel adds the slabs in a fixed order, so the result is deterministic and, like
 * fvar_score_select's own scores, equal to the exactly rounded sum except in double-rounding
 * corner cases.  scores_out:[B,M] fp32.  ws: at least fvar_fill_scored_workspace_bytes(ctx,B,M). */
size_t fvar_fill_scored_workspace_bytes(const fvar_ctx *ctx, int32_t B, int32_t M);
fvar_status fvar_lowrank_fill_scored(fvar_ctx *ctx, fvar_stream stream, const void *y_keep,
                                     const int32_t *idx_keep, const int32_t *idx_drop, int32_t B,
                                     int32_t M, int32_t k, int32_t r, const void *w_c, const void *g_c,
                                     void *y, float *scores_out, void *ws, size_t ws_bytes);

/* Random projection to r rows (paper, Sec. "Random Projection (RP) for Low-Rank Feature":
 * F^_r = Q^T F~ with Q in R^{M x r}, Q_ij ~ N(0, 1/r); Alg. "FasterVAR", fidelity stage).
 *   out[b,t,:] = sum_i qt[t,i] * x[b,i,:]
 * qt is Q TRANSPOSED, [rows][M] row-major in the context's element type; the caller draws it
 * (the library holds no random generator).  q_per_sample != 0: qt is [B][rows][M], one matrix
 * per sample; otherwise one matrix serves every sample.  x:[B,M,d], out:[B,rows,d], fp32
 * accumulation.  1 <= rows <= M; M a multiple of 8 for bf16 (of 4 for fp32).  No workspace. */
fvar_status fvar_rp_project(fvar_ctx *ctx, fvar_stream stream, const void *qt, int32_t q_per_sample,
                            const void *x, int32_t B, int32_t M, int32_t rows, void *out);

/* Restoration of the full token map with the raw cached rows (paper, Eq. "redefine" as printed,
 * Alg. "FasterVAR"):
 *   y[b,i,:] = y_keep[b,j,:]   if i == idx_keep[b,j]
 *   y[b,i,:] = cache[b,i,:]    if i is in idx_drop[b,:]
 * y_keep:[B,k,d], cache:[B,M,d] (the cached counterpart feature, already at M rows),
 * y:[B,M,d].  y may be the very same buffer as cache (then only the kept rows are written,
 * the pruned rows being in place already); otherwise the buffers must not overlap.
 * 0 <= k <= M.  No workspace. */
fvar_status fvar_cache_fill(fvar_ctx *ctx, fvar_stream stream, const void *y_keep,
                            const int32_t *idx_keep, const int32_t *idx_drop, int32_t B, int32_t M,
                            int32_t k, const void *cache, void *y);

/* Rank-r factors of the cached counterpart feature (paper, Sec. "Random Projection": G = Q^T C;
 * Eq. "lstsq" posed on the cached feature as App. "Construction of W_r^o" prescribes):
 *   g_c[b] = store(qt[b] cache[b])                                   [r,d]
 *   w_c[b] = store(argmin_W || W g_c[b] - cache[b] ||_F)             [M,r]
 *          = store((cache g_c^T)(g_c g_c^T + ridge*trace/r*I)^{-1})
 * store() rounds to the context's element type; the least-squares problem is posed against the
 * stored g_c.  Gram matrix, its inverse (elimination without pivoting: the matrix is symmetric
 * positive definite) and the final product run in fp64.  A singular Gram matrix (r above the
 * rank of the cache with ridge == 0) gives non-finite w_c; pass a small ridge (e.g. 1e-10) then.  qt, q_per_sample as in fvar_rp_project.
 * 1 <= r <= min(M,128), r a multiple of 8 for bf16 (of 4 for fp32); M as in fvar_rp_project.
 * ws: at least fvar_factors_workspace_bytes(ctx,B,M,r). */
size_t fvar_factors_workspace_bytes(const fvar_ctx *ctx, int32_t B, int32_t M, int32_t r);
fvar_status fvar_cache_factors(fvar_ctx *ctx, fvar_stream stream, const void *cache, const void *qt,
                               int32_t q_per_sample, int32_t B, int32_t M, int32_t r, double ridge,
                               void *w_c, void *g_c, void *ws, size_t ws_bytes);

/* Up-sampling of a cached token map to the token grid of the next scale (paper, Eq. "upcache":
 * F^{o,cache}_{k-1} = Up(F^o_{k-1})).  The paper does not name the interpolation; this is
 * bilinear interpolation with half-pixel centres and clamped edges, applied to the token axis:
 *   src:[B][hs*ws][c] (row-major hs x ws grid)  ->  dst:[B][hd*wd][c]
 * It is linear in the tokens, so a cache kept as W_c G_c is up-sampled by passing W_c (c = r):
 * Up(W_c G_c) = Up(W_c) G_c.  c a multiple of 8 for bf16 (of 4 for fp32); any grid sizes >= 1
 * (hd < hs down-samples without anti-aliasing).  fp32 arithmetic.  No workspace; src and dst
 * must not overlap. */
fvar_status fvar_upsample_tokens(fvar_ctx *ctx, fvar_stream stream, const void *src, int32_t B,
                                 int32_t hs, int32_t ws, int32_t c, int32_t hd, int32_t wd,
                                 void *dst);

/* Debug checks, off by default.  While on, fvar_block_forward_pruned, fvar_lowrank_fill and
 * fvar_cache_fill copy their index arrays to the host and verify the contract (in range,
 * strictly ascending per sample, idx_keep and idx_drop disjoint, hence a partition of [0,M));
 * a violation returns FVAR_ERR_INVALID_ARG with nothing launched.  The block calls also put a
 * 256-byte canary behind their workspace (fvar_block_workspace_bytes grows by that much while
 * the checks are on) and return FVAR_ERR_WORKSPACE if a kernel overwrote it.  Calls made with
 * the checks on synchronise the stream and are not asynchronous. */
fvar_status fvar_debug_checks(fvar_ctx *ctx, int32_t on);

/* Per-kernel timing (hipEvent pairs around every launch while enabled).  Off by default and
 * outside any throughput measurement.  fvar_profile_read synchronises the recorded events,
 * writes up to `cap` entries (kernel label, launches, total milliseconds) and clears them;
 * returns the number of distinct labels. */
typedef struct {
    char label[48];
    int64_t launches;
    double total_ms;
} fvar_profile_entry;
fvar_status fvar_profile_enable(fvar_ctx *ctx, int32_t on);
int32_t fvar_profile_read(fvar_ctx *ctx, fvar_profile_entry *out, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* FVAR_H */
