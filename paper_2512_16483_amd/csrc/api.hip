// C ABI of the library: argument validation, workspace carving and the launch sequence of each
// entry point.  Host code only; every arithmetic step runs in the kernels of this directory.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/fvar.h"
#include "common.h"

using fvar::DType;

thread_local fvar::LaunchProbe *fvar::g_probe = nullptr;

// Scratch of fvar_score_select_static (the fp32 scores of one call): a fixed device array instead
// of caller workspace, so that the call needs no allocation anywhere.  Every GPU the library runs
// on holds its own copy; host code reaches it only through the per-device address below.
constexpr int kStaticScoreCap = 1 << 20;                       // floats: 4 MiB per device
static __device__ __align__(256) float scratch[kStaticScoreCap];
constexpr int kMaxDevices = 64;
static float *g_scratch_ptr[kMaxDevices];                      // resolved on a device's first call
static std::mutex g_scratch_mutex;

struct fvar_ctx {
    fvar_config cfg;
    std::vector<int32_t> scale_hw;
    float eps, scale;
    char err[256];
    bool debug_checks = false;
    // per-kernel timing
    bool profiling = false;
    struct Rec { std::string label; hipEvent_t a, b; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
};

namespace {

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
size_t esize(const fvar_ctx *c) { return c->cfg.dtype == FVAR_BF16 ? 2 : 4; }
DType dtype(const fvar_ctx *c) { return c->cfg.dtype == FVAR_BF16 ? DType::BF16 : DType::F32; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

fvar_status fail(fvar_ctx *c, fvar_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
    return s;
}

hipEvent_t get_event(fvar_ctx *c)
{
    if (!c->pool.empty()) {
        hipEvent_t e = c->pool.back();
        c->pool.pop_back();
        return e;
    }
    hipEvent_t e;
    (void)hipEventCreate(&e);
    return e;
}

// Runs `launch` (the kernels of one step) with their start/stop recorded in an event pair when
// profiling is on.
template <typename F>
void timed(fvar_ctx *c, hipStream_t st, const char *label, F &&launch)
{
    if (!c->profiling) { launch(); return; }
    fvar_ctx::Rec r{label, get_event(c), get_event(c)};
    fvar::LaunchProbe probe{r.a, r.b, false};
    fvar::g_probe = &probe;                   // the kernel launches inside record into it
    launch();
    fvar::g_probe = nullptr;
    (void)st;
    c->recs.push_back(r);
}

fvar_status launch_status(fvar_ctx *c, const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, FVAR_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    c->err[0] = 0;
    return FVAR_OK;
}

constexpr size_t kCanaryBytes = 256;
constexpr unsigned char kCanaryByte = 0xA5;

// Debug checks: the index arrays are the caller's contract in normal operation; with the checks
// switched on they are brought to the host (which synchronises the stream) and verified:
// in range, strictly ascending per sample, and -- when both lists are given -- together exactly
// the set [0, M).
fvar_status validate_indices(fvar_ctx *c, hipStream_t st, const int32_t *idx_keep,
                             const int32_t *idx_drop, int B, int M, int k, const char *who)
{
    if (hipStreamSynchronize(st) != hipSuccess)
        return fail(c, FVAR_ERR_HIP, "%s: stream synchronisation failed in the index check", who);
    std::vector<int32_t> hk, hd;
    if (idx_keep && k > 0) {
        hk.resize((size_t)B * k);
        if (hipMemcpy(hk.data(), idx_keep, hk.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
            return fail(c, FVAR_ERR_HIP, "%s: cannot read idx_keep", who);
    }
    if (idx_drop && k < M) {
        hd.resize((size_t)B * (M - k));
        if (hipMemcpy(hd.data(), idx_drop, hd.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
            return fail(c, FVAR_ERR_HIP, "%s: cannot read idx_drop", who);
    }
    auto ascending = [&](const int32_t *v, int n, const char *name, int b) -> bool {
        for (int j = 0; j < n; ++j) {
            if (v[j] < 0 || v[j] >= M) {
                fail(c, FVAR_ERR_INVALID_ARG, "%s: %s[%d,%d] = %d is outside [0,%d)", who, name, b, j, v[j], M);
                return false;
            }
            if (j > 0 && v[j] <= v[j - 1]) {
                fail(c, FVAR_ERR_INVALID_ARG, "%s: %s[%d,:] is not strictly ascending at position %d", who,
                     name, b, j);
                return false;
            }
        }
        return true;
    };
    for (int b = 0; b < B; ++b) {
        const int32_t *kp = hk.empty() ? nullptr : hk.data() + (size_t)b * k;
        const int32_t *dp = hd.empty() ? nullptr : hd.data() + (size_t)b * (M - k);
        if (kp && !ascending(kp, k, "idx_keep", b)) return FVAR_ERR_INVALID_ARG;
        if (dp && !ascending(dp, M - k, "idx_drop", b)) return FVAR_ERR_INVALID_ARG;
        if (kp && dp) {
            // two ascending in-range lists of k and M-k entries partition [0,M) iff they share no entry
            int i = 0, j = 0;
            while (i < k && j < M - k) {
                if (kp[i] == dp[j])
                    return fail(c, FVAR_ERR_INVALID_ARG, "%s: token %d of sample %d is in idx_keep and idx_drop",
                                who, kp[i], b);
                if (kp[i] < dp[j]) ++i; else ++j;
            }
        }
    }
    return FVAR_OK;
}

struct BlockWs {
    char *x_keep, *u, *q, *att, *h1, *hid, *att_part, *gemm_part;
    size_t total;
};

BlockWs carve(const fvar_ctx *c, void *ws, int B, int rows)
{
    const size_t es = esize(c), R = (size_t)B * rows, d = c->cfg.hidden, F = c->cfg.ffn_hidden;
    BlockWs w;
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align256(bytes); return r; };
    w.x_keep = take(R * d * es);
    w.u = take(R * d * es);
    w.q = take(R * d * es);
    w.att = take(R * d * es);
    w.h1 = take(R * d * sizeof(float));       // intermediate residual stream, always fp32
    w.hid = take(R * F * es);
    // partial attention results when the key axis is split between workgroups (small batches)
    const size_t part = fvar::attention_scratch_floats(dtype(c), B, rows, c->cfg.heads, c->cfg.head_dim);
    w.att_part = part ? take(part * sizeof(float)) : nullptr;
    // partial tiles of the linear layers whose contraction axis is divided between workgroups
    const DType dt = dtype(c);
    size_t gp = 0;
    const size_t shapes[3][2] = {{d, d}, {F, d}, {d, F}};            // (N, K) of O, FC1, FC2
    for (auto &sh : shapes) {
        const size_t need = fvar::gemm_scratch_floats(dt, (int)R, (int)sh[0], (int)sh[1]) * sizeof(float);
        if (need > gp) gp = need;
    }
    w.gemm_part = gp ? take(gp) : nullptr;
    w.total = off;
    return w;
}

// The block on `rows` rows per sample.  idx == nullptr: rows are x's own rows (rows == M).
fvar_status block_forward(fvar_ctx *c, hipStream_t st, const fvar_block_weights *w, const void *x,
                          int B, int M, const int32_t *idx, int rows, const fvar_kv *kv, void *y,
                          void *ws, size_t ws_bytes, const char *who)
{
    if (!w || !x || !kv || !y) return fail(c, FVAR_ERR_INVALID_ARG, "%s: null argument", who);
    if (B < 1 || M < 1 || rows < 1 || rows > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 1<=rows<=M (B=%d M=%d rows=%d)", who, B,
                    M, rows);
    if (!idx && rows != M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: idx_keep may be NULL only when k == M", who);
    if (!w->w_qkv || !w->w_o || !w->w_fc1 || !w->w_fc2)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: weight matrix pointer is NULL", who);
    if (!kv->k || !kv->v || kv->len < 0 || kv->capacity < 1 ||
        (int64_t)kv->len + rows > (int64_t)kv->capacity)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: KV cache too small (len=%d + rows=%d > capacity=%d)",
                    who, kv->len, rows, kv->capacity);
    const void *ptrs[] = {x, y, kv->k, kv->v, w->w_qkv, w->w_o, w->w_fc1, w->w_fc2, w->ln1_g, w->ln1_b,
                          w->ln2_g, w->ln2_b, w->b_qkv, w->b_o, w->b_fc1, w->b_fc2, ws};
    for (const void *p : ptrs)
        if (!aligned16(p)) return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    if ((int64_t)B * rows > (1 << 24))
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B*rows exceeds 2^24", who);
    {
        // the linear-layer kernels address their operand tiles with 32-bit byte offsets from the
        // matrix base, and the attention grid carries (sample, key range) in blockIdx.z
        const int64_t wide = c->cfg.hidden > c->cfg.ffn_hidden ? c->cfg.hidden : c->cfg.ffn_hidden;
        const int64_t es = (int64_t)esize(c);
        if ((int64_t)B * rows * wide * es >= ((int64_t)1 << 32) ||
            (int64_t)3 * c->cfg.hidden * c->cfg.hidden * es >= ((int64_t)1 << 32) ||
            (int64_t)c->cfg.ffn_hidden * c->cfg.hidden * es >= ((int64_t)1 << 32))
            return fail(c, FVAR_ERR_UNSUPPORTED,
                        "%s: an operand matrix of B*rows=%lld rows reaches 4 GiB (32-bit tile offsets)",
                        who, (long long)B * rows);
        if ((int64_t)B * 8 > 65535 || c->cfg.heads > 65535)
            return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B or heads exceeds the launch grid limits", who);
    }
    BlockWs s = carve(c, ws, B, rows);
    const size_t ws_need = s.total + (c->debug_checks ? kCanaryBytes : 0);
    if (!ws || ws_bytes < ws_need)
        return fail(c, FVAR_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, ws_need,
                    ws_bytes);
    if (c->debug_checks) {
        if (idx) {
            const fvar_status vs = validate_indices(c, st, idx, nullptr, B, M, rows, who);
            if (vs != FVAR_OK) return vs;
        }
        // canary behind the carved workspace, verified after the kernels have finished
        if (hipMemsetAsync(static_cast<char *>(ws) + s.total, kCanaryByte, kCanaryBytes, st) != hipSuccess)
            return fail(c, FVAR_ERR_HIP, "%s: cannot write the workspace canary", who);
    }

    const DType dt = dtype(c);
    const int d = c->cfg.hidden, H = c->cfg.heads, Dh = c->cfg.head_dim, F = c->cfg.ffn_hidden;
    const int R = B * rows, L = kv->len + rows;

    // gather (identity in the dense case) + LayerNorm 1; the dense case reads the residual from x
    const void *resid = idx ? (const void *)s.x_keep : x;
    timed(c, st, "gather_ln1", [&] {
        fvar::launch_gather_ln(dt, x, idx, B, M, rows, d, w->ln1_g, w->ln1_b, c->eps,
                               idx ? s.x_keep : nullptr, s.u, st);
    });
    // QKV projection; K and V rows land in the cache behind the valid prefix
    timed(c, st, "gemm_qkv", [&] {
        fvar::GemmEpilogue e;
        e.bias = w->b_qkv; e.out0 = s.q; e.ld0 = d; e.split = d;
        e.kcache = kv->k; e.vcache = kv->v; e.hd = d; e.cap = kv->capacity; e.len = kv->len;
        e.rows_per_sample = rows;
        fvar::launch_gemm(dt, s.u, w->w_qkv, R, 3 * d, d, e, st);
    });
    timed(c, st, "attention", [&] {
        fvar::launch_attention(dt, s.q, kv->k, kv->v, B, rows, L, kv->capacity, H, Dh, c->scale, s.att,
                               reinterpret_cast<float *>(s.att_part), st);
    });
    timed(c, st, "gemm_o", [&] {
        fvar::GemmEpilogue e;
        e.bias = w->b_o; e.residual = resid; e.out0 = s.h1; e.ld0 = d; e.split = d;
        e.out_f32 = 1;
        e.splitk_scratch = reinterpret_cast<float *>(s.gemm_part);
        fvar::launch_gemm(dt, s.att, w->w_o, R, d, d, e, st);
    });
    timed(c, st, "ln2", [&] {
        if (dt == DType::BF16)
            fvar::launch_ln_f32_to_bf16((const float *)s.h1, R, d, w->ln2_g, w->ln2_b, c->eps, s.u, st);
        else
            fvar::launch_gather_ln(dt, s.h1, nullptr, 1, R, R, d, w->ln2_g, w->ln2_b, c->eps, nullptr,
                                   s.u, st);
    });
    timed(c, st, "gemm_fc1", [&] {
        fvar::GemmEpilogue e;
        e.bias = w->b_fc1; e.gelu = 1; e.out0 = s.hid; e.ld0 = F; e.split = F;
        e.splitk_scratch = reinterpret_cast<float *>(s.gemm_part);
        fvar::launch_gemm(dt, s.u, w->w_fc1, R, F, d, e, st);
    });
    timed(c, st, "gemm_fc2", [&] {
        fvar::GemmEpilogue e;
        e.bias = w->b_fc2; e.residual = s.h1; e.res_f32 = 1; e.out0 = y; e.ld0 = d; e.split = d;
        e.splitk_scratch = reinterpret_cast<float *>(s.gemm_part);
        fvar::launch_gemm(dt, s.hid, w->w_fc2, R, d, F, e, st);
    });
    const fvar_status ls = launch_status(c, who);
    if (ls != FVAR_OK || !c->debug_checks) return ls;
    unsigned char canary[kCanaryBytes];
    if (hipStreamSynchronize(st) != hipSuccess ||
        hipMemcpy(canary, static_cast<char *>(ws) + s.total, kCanaryBytes, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(c, FVAR_ERR_HIP, "%s: kernels failed (seen at the debug-check synchronisation)", who);
    for (size_t i = 0; i < kCanaryBytes; ++i)
        if (canary[i] != kCanaryByte)
            return fail(c, FVAR_ERR_WORKSPACE, "%s: a kernel wrote past the end of its workspace (canary byte %zu)",
                        who, i);
    return FVAR_OK;
}

}  // namespace

extern "C" {

const char *fvar_status_string(fvar_status s)
{
    switch (s) {
    case FVAR_OK: return "ok";
    case FVAR_ERR_INVALID_ARG: return "invalid argument";
    case FVAR_ERR_UNSUPPORTED: return "unsupported";
    case FVAR_ERR_WORKSPACE: return "workspace too small";
    case FVAR_ERR_HIP: return "HIP error";
    }
    return "unknown";
}

fvar_status fvar_create(const fvar_config *cfg, fvar_ctx **out)
{
    if (!cfg || !out) return FVAR_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->hidden < 1 || cfg->heads < 1 || cfg->head_dim < 1 || cfg->ffn_hidden < 1 ||
        (int64_t)cfg->heads * cfg->head_dim != cfg->hidden)
        return FVAR_ERR_INVALID_ARG;
    if (cfg->dtype != FVAR_F32 && cfg->dtype != FVAR_BF16) return FVAR_ERR_INVALID_ARG;
    if (cfg->num_scales < 0 || (cfg->num_scales > 0 && !cfg->scale_hw)) return FVAR_ERR_INVALID_ARG;
    if (cfg->head_dim != 64 && cfg->head_dim != 128) return FVAR_ERR_UNSUPPORTED;
    // k-tiles of 64 in the GEMMs; one wavefront holds a whole row in the row kernels
    if (cfg->hidden % 64 || cfg->ffn_hidden % 64) return FVAR_ERR_UNSUPPORTED;
    const int max_hidden = cfg->dtype == FVAR_BF16 ? 8192 : 4096;
    if (cfg->hidden > max_hidden) return FVAR_ERR_UNSUPPORTED;
    for (int i = 0; i < 2 * cfg->num_scales; ++i)
        if (cfg->scale_hw[i] < 1) return FVAR_ERR_INVALID_ARG;
    fvar_ctx *c = new fvar_ctx();
    c->cfg = *cfg;
    c->scale_hw.assign(cfg->scale_hw, cfg->scale_hw + 2 * (size_t)cfg->num_scales);
    c->cfg.scale_hw = c->scale_hw.data();
    c->eps = cfg->ln_eps > 0.f ? cfg->ln_eps : 1e-6f;
    c->scale = cfg->attn_scale > 0.f ? cfg->attn_scale : 1.0f / sqrtf((float)cfg->head_dim);
    c->err[0] = 0;
    *out = c;
    return FVAR_OK;
}

void fvar_destroy(fvar_ctx *c)
{
    if (!c) return;
    for (auto &r : c->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : c->pool) (void)hipEventDestroy(e);
    delete c;
}

const char *fvar_last_error(const fvar_ctx *c) { return c ? c->err : "null context"; }

int32_t fvar_keep_count(int32_t M, int32_t num, int32_t den)
{
    if (M < 1 || den < 1 || num < 0) return -1;
    int64_t k = ((int64_t)M * num + den - 1) / den;
    if (k < 1) k = 1;
    if (k > M) k = M;
    return (int32_t)k;
}

int32_t fvar_scale_tokens(const fvar_ctx *c, int32_t i)
{
    if (!c || i < 0 || i >= c->cfg.num_scales) return -1;
    return c->scale_hw[2 * i] * c->scale_hw[2 * i + 1];
}

int32_t fvar_scale_prev_len(const fvar_ctx *c, int32_t i)
{
    if (!c || i < 0 || i >= c->cfg.num_scales) return -1;
    int64_t s = 0;
    for (int j = 0; j < i; ++j) s += (int64_t)c->scale_hw[2 * j] * c->scale_hw[2 * j + 1];
    return s > INT32_MAX ? -1 : (int32_t)s;
}

size_t fvar_select_workspace_bytes(const fvar_ctx *c, int32_t B, int32_t M)
{
    if (!c || B < 1 || M < 1) return 0;
    return align256((size_t)B * M * sizeof(float));
}

size_t fvar_block_workspace_bytes(const fvar_ctx *c, int32_t B, int32_t rows)
{
    if (!c || B < 1 || rows < 1) return 0;
    return carve(c, nullptr, B, rows).total + (c->debug_checks ? kCanaryBytes : 0);
}

fvar_status fvar_debug_checks(fvar_ctx *c, int32_t on)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    c->debug_checks = on != 0;
    return FVAR_OK;
}

fvar_status fvar_score_select(fvar_ctx *c, fvar_stream stream, const void *x, int32_t B, int32_t M,
                              int32_t k, const float *scores_in, float *scores_out,
                              int32_t *idx_keep, int32_t *idx_drop, void *ws, size_t ws_bytes)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    const char *who = "fvar_score_select";
    if (B < 1 || M < 1 || k < 1 || k > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 1<=k<=M (B=%d M=%d k=%d)", who, B, M, k);
    if (M > (1 << 20) || (int64_t)B * M > (int64_t)INT32_MAX / 2)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: M or B*M too large", who);
    if (!idx_keep) return fail(c, FVAR_ERR_INVALID_ARG, "%s: idx_keep is NULL", who);
    if (!x && !scores_in) return fail(c, FVAR_ERR_INVALID_ARG, "%s: x and scores_in both NULL", who);
    if (!aligned16(x) || !aligned16(ws))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float *scores = scores_in;
    if (!scores_in) {
        float *buf = scores_out;
        if (!buf) {
            if (!ws || ws_bytes < fvar_select_workspace_bytes(c, B, M))
                return fail(c, FVAR_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who,
                            fvar_select_workspace_bytes(c, B, M), ws_bytes);
            buf = static_cast<float *>(ws);
        }
        timed(c, st, "score", [&] { fvar::launch_scores(dtype(c), x, B * M, c->cfg.hidden, buf, st); });
        scores = buf;
    } else if (scores_out && scores_out != scores_in) {
        hipError_t e = hipMemcpyAsync(scores_out, scores_in, (size_t)B * M * sizeof(float),
                                      hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return fail(c, FVAR_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
    }
    timed(c, st, "select", [&] { fvar::launch_select(scores, B, M, k, idx_keep, idx_drop, st); });
    return launch_status(c, who);
}

fvar_status fvar_score_select_static(fvar_ctx *c, fvar_stream stream, const void *x, int32_t B,
                                     int32_t M, int32_t k, int32_t *idx_keep, int32_t *idx_drop)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    const char *who = "fvar_score_select_static";
    if (B < 1 || M < 1 || k < 1 || k > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 1<=k<=M (B=%d M=%d k=%d)", who, B, M, k);
    if ((int64_t)B * M > kStaticScoreCap)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B*M = %lld exceeds the built-in scratch of %d scores; use "
                    "fvar_score_select with a workspace", who, (long long)B * M, kStaticScoreCap);
    if (!x || !idx_keep) return fail(c, FVAR_ERR_INVALID_ARG, "%s: x or idx_keep is NULL", who);
    if (!aligned16(x)) return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(c, FVAR_ERR_HIP, "%s: no usable current device", who);
    float *buf;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            // the array's name is only a host-side handle; this is its address on the current device
            float *p = nullptr;
            const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p)
                return fail(c, FVAR_ERR_HIP, "%s: hipGetSymbolAddress: %s", who, hipGetErrorString(e));
            g_scratch_ptr[dev] = p;
        }
        buf = g_scratch_ptr[dev];
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    // every score of [0, B*M) is rewritten before the selection reads it: nothing to clear
    timed(c, st, "score", [&] { fvar::launch_scores(dtype(c), x, B * M, c->cfg.hidden, buf, st); });
    timed(c, st, "select", [&] { fvar::launch_select(buf, B, M, k, idx_keep, idx_drop, st); });
    return launch_status(c, who);
}

fvar_status fvar_block_forward_dense(fvar_ctx *c, fvar_stream stream, const fvar_block_weights *w,
                                     const void *x, int32_t B, int32_t M, const fvar_kv *kv, void *y,
                                     void *ws, size_t ws_bytes)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    return block_forward(c, static_cast<hipStream_t>(stream), w, x, B, M, nullptr, M, kv, y, ws,
                         ws_bytes, "fvar_block_forward_dense");
}

fvar_status fvar_block_forward_pruned(fvar_ctx *c, fvar_stream stream, const fvar_block_weights *w,
                                      const void *x, int32_t B, int32_t M, const int32_t *idx_keep,
                                      int32_t k, const fvar_kv *kv, void *y_keep, void *ws,
                                      size_t ws_bytes)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    return block_forward(c, static_cast<hipStream_t>(stream), w, x, B, M, idx_keep, k, kv, y_keep, ws,
                         ws_bytes, "fvar_block_forward_pruned");
}

static fvar_status lowrank_fill(fvar_ctx *c, fvar_stream stream, const void *y_keep,
                                const int32_t *idx_keep, const int32_t *idx_drop, int32_t B, int32_t M,
                                int32_t k, int32_t r, const void *w_c, const void *g_c, void *y,
                                float *scores_out, void *ws, size_t ws_bytes, const char *who)
{
    if (B < 1 || M < 1 || k < 0 || k > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 0<=k<=M (B=%d M=%d k=%d)", who, B, M, k);
    if (!y || (k > 0 && !y_keep)) return fail(c, FVAR_ERR_INVALID_ARG, "%s: null output or y_keep", who);
    if (k < M) {
        if (!idx_keep && k > 0) return fail(c, FVAR_ERR_INVALID_ARG, "%s: idx_keep is NULL", who);
        if (!idx_drop || !w_c || !g_c)
            return fail(c, FVAR_ERR_INVALID_ARG, "%s: idx_drop, w_c and g_c are required when k < M", who);
        const int mult = c->cfg.dtype == FVAR_BF16 ? 8 : 4;
        if (r < 1 || r > 256 || r % mult)
            return fail(c, FVAR_ERR_INVALID_ARG, "%s: rank %d must be in [1,256] and a multiple of %d",
                        who, r, mult);
    }
    if (!aligned16(y) || !aligned16(y_keep) || !aligned16(w_c) || !aligned16(g_c) || !aligned16(ws))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    if ((int64_t)B * M > (int64_t)INT32_MAX / 2)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B*M too large", who);
    double *parts = nullptr;
    if (scores_out) {
        const size_t need = fvar_fill_scored_workspace_bytes(c, B, M);
        if (!ws || ws_bytes < need)
            return fail(c, FVAR_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need,
                        ws_bytes);
        parts = static_cast<double *>(ws);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (c->debug_checks && k < M) {
        const fvar_status vs = validate_indices(c, st, idx_keep, idx_drop, B, M, k, who);
        if (vs != FVAR_OK) return vs;
    }
    timed(c, st, "fill", [&] {
        fvar::launch_fill(dtype(c), y_keep, idx_keep, idx_drop, B, M, k, r, c->cfg.hidden, w_c, g_c, y,
                          parts, scores_out, st);
    });
    return launch_status(c, who);
}

size_t fvar_fill_scored_workspace_bytes(const fvar_ctx *c, int32_t B, int32_t M)
{
    if (!c || B < 1 || M < 1) return 0;
    return align256((size_t)B * M * fvar::fill_score_parts(dtype(c), c->cfg.hidden) * sizeof(double));
}

fvar_status fvar_lowrank_fill(fvar_ctx *c, fvar_stream stream, const void *y_keep,
                              const int32_t *idx_keep, const int32_t *idx_drop, int32_t B, int32_t M,
                              int32_t k, int32_t r, const void *w_c, const void *g_c, void *y)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    return lowrank_fill(c, stream, y_keep, idx_keep, idx_drop, B, M, k, r, w_c, g_c, y, nullptr, nullptr,
                        0, "fvar_lowrank_fill");
}

fvar_status fvar_lowrank_fill_scored(fvar_ctx *c, fvar_stream stream, const void *y_keep,
                                     const int32_t *idx_keep, const int32_t *idx_drop, int32_t B,
                                     int32_t M, int32_t k, int32_t r, const void *w_c, const void *g_c,
                                     void *y, float *scores_out, void *ws, size_t ws_bytes)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    if (!scores_out)
        return fail(c, FVAR_ERR_INVALID_ARG, "fvar_lowrank_fill_scored: scores_out is NULL");
    return lowrank_fill(c, stream, y_keep, idx_keep, idx_drop, B, M, k, r, w_c, g_c, y, scores_out, ws,
                        ws_bytes, "fvar_lowrank_fill_scored");
}

fvar_status fvar_rp_project(fvar_ctx *c, fvar_stream stream, const void *qt, int32_t q_per_sample,
                            const void *x, int32_t B, int32_t M, int32_t rows, void *out)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    const char *who = "fvar_rp_project";
    if (B < 1 || M < 1 || rows < 1 || rows > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 1<=rows<=M (B=%d M=%d rows=%d)", who, B,
                    M, rows);
    if (!qt || !x || !out) return fail(c, FVAR_ERR_INVALID_ARG, "%s: null argument", who);
    if (!aligned16(qt) || !aligned16(x) || !aligned16(out))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    const int mult = c->cfg.dtype == FVAR_BF16 ? 8 : 4;
    if (M % mult)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: M=%d must be a multiple of %d", who, M, mult);
    if ((int64_t)B * M > (int64_t)INT32_MAX / 2 || B > 65535)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B or B*M too large", who);
    hipStream_t st = static_cast<hipStream_t>(stream);
    timed(c, st, "rp_project", [&] {
        fvar::launch_rp_project(dtype(c), qt, q_per_sample ? (size_t)rows * M : 0, x, B, M, rows,
                                c->cfg.hidden, out, st);
    });
    return launch_status(c, who);
}

fvar_status fvar_cache_fill(fvar_ctx *c, fvar_stream stream, const void *y_keep,
                            const int32_t *idx_keep, const int32_t *idx_drop, int32_t B, int32_t M,
                            int32_t k, const void *cache, void *y)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    const char *who = "fvar_cache_fill";
    if (B < 1 || M < 1 || k < 0 || k > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 0<=k<=M (B=%d M=%d k=%d)", who, B, M, k);
    if (!y || (k > 0 && (!y_keep || !idx_keep)))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: null output, y_keep or idx_keep", who);
    if (k < M && (!idx_drop || !cache))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: idx_drop and cache are required when k < M", who);
    if (!aligned16(y) || !aligned16(y_keep) || !aligned16(cache))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    if ((int64_t)B * M > (int64_t)INT32_MAX / 2)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B*M too large", who);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (c->debug_checks) {
        const fvar_status vs = validate_indices(c, st, idx_keep, idx_drop, B, M, k, who);
        if (vs != FVAR_OK) return vs;
    }
    timed(c, st, "cache_fill", [&] {
        fvar::launch_cache_fill(dtype(c), y_keep, idx_keep, idx_drop, B, M, k, c->cfg.hidden, cache, y,
                                st);
    });
    return launch_status(c, who);
}

size_t fvar_factors_workspace_bytes(const fvar_ctx *c, int32_t B, int32_t M, int32_t r)
{
    if (!c || B < 1 || M < 1 || r < 1) return 0;
    const size_t rr = (size_t)B * r * r * sizeof(double);
    return align256((size_t)B * M * r * sizeof(float) * fvar::factor_t_parts(dtype(c), B, M)) +
           align256(rr * fvar::gram_parts(dtype(c))) + align256(rr);
}

fvar_status fvar_cache_factors(fvar_ctx *c, fvar_stream stream, const void *cache, const void *qt,
                               int32_t q_per_sample, int32_t B, int32_t M, int32_t r, double ridge,
                               void *w_c, void *g_c, void *ws, size_t ws_bytes)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    const char *who = "fvar_cache_factors";
    const int mult = c->cfg.dtype == FVAR_BF16 ? 8 : 4;
    if (B < 1 || M < 1 || r < 1 || r > M)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: need B>=1 and 1<=r<=M (B=%d M=%d r=%d)", who, B, M, r);
    if (!cache || !qt || !w_c || !g_c) return fail(c, FVAR_ERR_INVALID_ARG, "%s: null argument", who);
    if (!(ridge >= 0.0)) return fail(c, FVAR_ERR_INVALID_ARG, "%s: ridge must be >= 0", who);
    if (r > 128 || r % mult)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: rank %d must be <= 128 and a multiple of %d", who, r,
                    mult);
    if (M % mult)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: M=%d must be a multiple of %d", who, M, mult);
    if ((int64_t)B * M > (int64_t)INT32_MAX / 2 || B > 65535)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: B or B*M too large", who);
    if (!aligned16(cache) || !aligned16(qt) || !aligned16(w_c) || !aligned16(g_c) || !aligned16(ws))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    const size_t need = fvar_factors_workspace_bytes(c, B, M, r);
    if (!ws || ws_bytes < need)
        return fail(c, FVAR_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need,
                    ws_bytes);
    char *p = static_cast<char *>(ws);
    float *T = reinterpret_cast<float *>(p);
    p += align256((size_t)B * M * r * sizeof(float) * fvar::factor_t_parts(dtype(c), B, M));
    double *S = reinterpret_cast<double *>(p);
    p += align256((size_t)B * r * r * sizeof(double) * fvar::gram_parts(dtype(c)));
    double *Sinv = reinterpret_cast<double *>(p);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const DType dt = dtype(c);
    const int d = c->cfg.hidden;
    timed(c, st, "factor_project", [&] {
        fvar::launch_rp_project(dt, qt, q_per_sample ? (size_t)r * M : 0, cache, B, M, r, d, g_c, st);
    });
    timed(c, st, "factor_t", [&] { fvar::launch_factor_t(dt, cache, g_c, B, M, r, d, T, st); });
    timed(c, st, "factor_gram", [&] { fvar::launch_factor_gram(dt, g_c, B, r, d, S, st); });
    timed(c, st, "factor_inverse", [&] { fvar::launch_factor_inverse(S, fvar::gram_parts(dt), B, r, ridge, Sinv, st); });
    timed(c, st, "factor_w", [&] { fvar::launch_factor_w(dt, T, Sinv, B, M, r, w_c, st); });
    return launch_status(c, who);
}

fvar_status fvar_upsample_tokens(fvar_ctx *c, fvar_stream stream, const void *src, int32_t B,
                                 int32_t hs, int32_t ws, int32_t ch, int32_t hd, int32_t wd,
                                 void *dst)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    const char *who = "fvar_upsample_tokens";
    if (B < 1 || hs < 1 || ws < 1 || hd < 1 || wd < 1 || ch < 1)
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: sizes must be >= 1", who);
    if (!src || !dst) return fail(c, FVAR_ERR_INVALID_ARG, "%s: null argument", who);
    if (!aligned16(src) || !aligned16(dst))
        return fail(c, FVAR_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
    const int mult = c->cfg.dtype == FVAR_BF16 ? 8 : 4;
    if (ch % mult)
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: channel count %d must be a multiple of %d", who, ch,
                    mult);
    if ((int64_t)hs * ws > (1 << 24) || (int64_t)hd * wd > (1 << 24) ||
        (int64_t)B * hd * wd * (ch / mult) > ((int64_t)1 << 38))
        return fail(c, FVAR_ERR_UNSUPPORTED, "%s: grid too large", who);
    hipStream_t st = static_cast<hipStream_t>(stream);
    timed(c, st, "upsample", [&] {
        fvar::launch_upsample(dtype(c), src, B, hs, ws, hd, wd, ch, dst, st);
    });
    return launch_status(c, who);
}

fvar_status fvar_profile_enable(fvar_ctx *c, int32_t on)
{
    if (!c) return FVAR_ERR_INVALID_ARG;
    c->profiling = on != 0;
    return FVAR_OK;
}

int32_t fvar_profile_read(fvar_ctx *c, fvar_profile_entry *out, int32_t cap)
{
    if (!c) return 0;
    std::map<std::string, std::pair<int64_t, double>> acc;
    std::vector<std::string> order;
    for (auto &r : c->recs) {
        (void)hipEventSynchronize(r.b);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, r.a, r.b);
        if (!acc.count(r.label)) order.push_back(r.label);
        auto &e = acc[r.label];
        e.first += 1;
        e.second += ms;
        c->pool.push_back(r.a);
        c->pool.push_back(r.b);
    }
    c->recs.clear();
    int32_t nlab = 0;
    for (auto &lab : order) {
        if (out && nlab < cap) {
            std::snprintf(out[nlab].label, sizeof(out[nlab].label), "%s", lab.c_str());
            out[nlab].launches = acc[lab].first;
            out[nlab].total_ms = acc[lab].second;
        }
        ++nlab;
    }
    return nlab;
}

}  // extern "C"
