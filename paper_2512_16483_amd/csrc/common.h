// Shared device helpers and the host-side launcher interface of the fvar kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#define FVAR_WAVE 64

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------- bf16 <-> fp32
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round-to-nearest-even pack of two floats into one dword (lo = a, hi = b)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    floatx2_t v = {a, b};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float a)
{
    return (uint16_t)(pack_bf16x2(a, 0.f) & 0xffffu);
}

// ---------------------------------------------------------------- element-type traits
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerChunk = 4;                 // elements per 16-byte chunk
    __device__ static __forceinline__ void unpack(const uint4 &c, float *f)
    {
        f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y);
        f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
    }
    __device__ static __forceinline__ uint4 pack(const float *f)
    {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                          __float_as_uint(f[3]));
    }
    __device__ static __forceinline__ float load(const float *p) { return *p; }
    __device__ static __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {                     // bf16 stored as raw 16-bit words
    static constexpr int kPerChunk = 8;
    __device__ static __forceinline__ void unpack(const uint4 &c, float *f)
    {
        f[0] = bf16_lo(c.x); f[1] = bf16_hi(c.x); f[2] = bf16_lo(c.y); f[3] = bf16_hi(c.y);
        f[4] = bf16_lo(c.z); f[5] = bf16_hi(c.z); f[6] = bf16_lo(c.w); f[7] = bf16_hi(c.w);
    }
    __device__ static __forceinline__ uint4 pack(const float *f)
    {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                          pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
    __device__ static __forceinline__ float load(const uint16_t *p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void store(uint16_t *p, float v) { *p = f32_to_bf16(v); }
};

// ---------------------------------------------------------------- wavefront reductions
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------- launcher interface
// Every launcher only enqueues kernels on `st`; shapes are validated by the callers in api.hip.
namespace fvar {

enum class DType : int { F32 = 0, BF16 = 1 };

// Kernel launch used by every launcher.  While per-kernel timing is switched on, the API layer
// points g_probe at an event pair and the launch records the kernel's own start and stop in it
// (hipExtLaunchKernel), which excludes the dispatch gap in front of the step.
// A step that launches several kernels records the start of its first and the stop of its last.
struct LaunchProbe { hipEvent_t start, stop; bool started; };
extern thread_local LaunchProbe *g_probe;
template <typename F, typename... Args>
inline void launch(F kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args)
{
    if (g_probe) {
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st,
                              g_probe->started ? nullptr : g_probe->start, g_probe->stop, 0, args...);
        g_probe->started = true;
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
    }
}

// scores[b,i] = fl32(sum_j x[b,i,j]^2), fp64 accumulation
void launch_scores(DType dt, const void *x, int rows, int d, float *scores, hipStream_t st);
// per-sample radix select of the k largest scores + stable compaction
void launch_select(const float *scores, int B, int M, int k, int32_t *idx_keep, int32_t *idx_drop,
                   hipStream_t st);
// rows of x (optionally gathered through idx) -> optional raw copy + LayerNorm output
//   x:[B,M,d]; idx:[B,n] or null (identity, then n == M); copy_out / ln_out: [B*n,d] or null
void launch_gather_ln(DType dt, const void *x, const int32_t *idx, int B, int M, int n, int d,
                      const void *gamma, const void *beta, float eps, void *copy_out, void *ln_out,
                      hipStream_t st);
// LayerNorm of fp32 rows h:[rows,d] into bf16 rows (gamma, beta bf16 or null)
void launch_ln_f32_to_bf16(const float *h, int rows, int d, const void *gamma, const void *beta,
                           float eps, void *ln_out, hipStream_t st);

// C = epilogue(A[rows,K] * W[N,K]^T + bias)
struct GemmEpilogue {
    const void *bias = nullptr;        // [N] or null
    const void *residual = nullptr;    // [rows,N] or null, added after the activation
    int gelu = 0;                      // tanh-GELU before the residual
    // output routing: columns [0,split) go to out0 (ld0); if split < N the remaining columns are
    // the K and V projections, written into the cache rows of each sample:
    //   col in [split, split+hd)      -> kcache[(b*cap + len + j) * hd + col-split]
    //   col in [split+hd, split+2hd)  -> vcache[...]
    // with b = row / rows_per_sample, j = row % rows_per_sample.
    void *out0 = nullptr;
    int ld0 = 0;
    int split = 0;                     // == N when there is no K/V routing
    void *kcache = nullptr, *vcache = nullptr;
    int hd = 0, cap = 0, len = 0, rows_per_sample = 1;
    // bf16 path only: out0 receives fp32 (no routing, no GELU) / the residual operand is fp32.
    // Used for the intermediate residual stream h = x + attention projection, which stays in
    // fp32 between the two halves of the block so that it is not rounded twice.
    int out_f32 = 0, res_f32 = 0;
    // bf16 path: scratch of gemm_scratch_floats() floats for dividing the contraction axis between
    // workgroups (every tile of a problem with too few tiles to fill the chip, or only the tiles
    // beyond the last full round of workgroups), or null (never divide).
    float *splitk_scratch = nullptr;
};
size_t gemm_scratch_floats(DType dt, int rows, int N, int K);
void launch_gemm(DType dt, const void *A, const void *W, int rows, int N, int K,
                 const GemmEpilogue &ep, hipStream_t st);

// o[b,i,h,:] = softmax_t(scale * q[b,i,h,:] . K[b,t,h,:]) V[b,t,h,:], t in [0,L)
//   q,o:[B,n,H,Dh]; K,V:[B,cap,H,Dh]
// `part`: scratch of attention_scratch_floats() floats for dividing the key axis between workgroups
// (every unit of a problem with too few (query block, head, sample) triples to fill the chip, or
// only the units of the last, mostly empty round of workgroups of a large problem), or null
// (never divide).  With more than one key range a second kernel merges the partial results.
size_t attention_scratch_floats(DType dt, int B, int n, int H, int Dh);
void launch_attention(DType dt, const void *q, const void *K, const void *V, int B, int n, int L,
                      int cap, int H, int Dh, float scale, void *o, float *part, hipStream_t st);

// y[b,idx_keep[b,j],:] = y_keep[b,j,:];  y[b,i,:] = w_c[b,i,:] g_c[b] for i in idx_drop[b,:]
// parts / scores_out: null, or scratch of B*M*fill_score_parts() doubles and a [B*M] fp32 array that
// receives the energy (sum of squares of the stored elements) of every row of y
int fill_score_parts(DType dt, int d);
void launch_fill(DType dt, const void *y_keep, const int32_t *idx_keep, const int32_t *idx_drop,
                 int B, int M, int k, int r, int d, const void *w_c, const void *g_c, void *y,
                 double *parts, float *scores_out, hipStream_t st);

// raw-cache variant of the fill: pruned rows are copied from cache:[B,M,d]
void launch_cache_fill(DType dt, const void *y_keep, const int32_t *idx_keep, const int32_t *idx_drop,
                       int B, int M, int k, int d, const void *cache, void *y, hipStream_t st);

// out[b] = qt[b] x[b]:  qt:[rows,M] (sample stride q_stride elements, 0 = shared), x:[B,M,d],
// out:[B,rows,d].  M must be a multiple of the 16-byte chunk (8 bf16 / 4 fp32 elements).
bool launch_gemm_bf16_batched_f32(const void *A, const void *W, int nbatch, int rows, int N, int K,
                                  float *out, hipStream_t st);
bool launch_gemm_bf16_kmajor(const void *qt, size_t q_stride, const void *x, int B, int M, int rows,
                             int d, void *out, hipStream_t st);
void launch_rp_project(DType dt, const void *qt, size_t q_stride, const void *x, int B, int M,
                       int rows, int d, void *out, hipStream_t st);

// bilinear up-sampling of token maps src:[B,hs*ws,c] -> dst:[B,hd*wd,c]; c a multiple of the
// 16-byte chunk
void launch_upsample(DType dt, const void *src, int B, int hs, int ws, int hd, int wd, int c,
                     void *dst, hipStream_t st);

// restoration matrix W_c = (C G_c^T)(G_c G_c^T)^{-1} in four steps; T:[factor_t_parts (1 or 2),B,M,r] fp32,
// S:[B,gram_parts(dt),r,r] and Sinv:[B,r,r] fp64 are scratch.  r <= 128.
int factor_t_parts(DType dt, int B, int M);
void launch_factor_t(DType dt, const void *cache, const void *g_c, int B, int M, int r, int d, float *T,
                     hipStream_t st);
void launch_factor_gram(DType dt, const void *g_c, int B, int r, int d, double *S, hipStream_t st);
int gram_parts(DType dt);
void launch_factor_inverse(const double *S, int parts, int B, int r, double ridge, double *Sinv,
                           hipStream_t st);
void launch_factor_w(DType dt, const float *T, const double *Sinv, int B, int M, int r, void *w_c,
                     hipStream_t st);

}  // namespace fvar
