// Restoration matrix of the cached counterpart feature by linear least squares (paper, Eq.
// "lstsq" with the cached feature in place of the input, App. "Construction of W_r^o"):
//
//     W_c = argmin_W || W G_c - C ||_F = (C G_c^T) (G_c G_c^T)^{-1},     G_c = Q^T C  as stored.
//
// Four kernels per call (the projection G_c itself is the kernel of rp.hip):
//   t_kernel      T = C G_c^T            [M,r]  fp32; bf16 inputs on MFMA, the only pass over C
//   gram_kernel   S = G_c G_c^T          [r,r]  fp64
//   chol_kernel   S^{-1} by Cholesky     one workgroup per sample, fp64 in LDS
//   w_kernel      W_c = T S^{-1}         [M,r]  fp64 accumulation, rounded to the storage type
#include "common.h"

namespace fvar {

// ------------------------------------------------------------------ T = C G^T, bf16 on MFMA
// Workgroup = 32 rows of C; its four wavefronts take the 64-element chunks of the contraction
// axis round-robin (each reads a 128-byte segment of every row per chunk), then the partial
// 32 x r tiles are added up through LDS.  RT = r / 32 rounded up.
template <int RT>
__global__ __launch_bounds__(256) void t_bf16_kernel(const uint16_t *__restrict__ cache,
                                                     const uint16_t *__restrict__ g_c, int M, int r,
                                                     int d, float *__restrict__ T)
{
    extern __shared__ float part[];                 // [4][32][32*RT]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    const int b = blockIdx.y, row0 = blockIdx.x * 32;
    const uint16_t *crow = cache + ((size_t)b * M + min(row0 + rl, M - 1)) * d;
    const uint16_t *G = g_c + (size_t)b * r * d;
    const uint16_t *grow[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j) grow[j] = G + (size_t)min(j * 32 + rl, r - 1) * d;

    floatx16_t acc[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j) acc[j] = floatx16_t{0};
    const int nchunks = d / 64;
    for (int c = wave; c < nchunks; c += 4) {
        uint4 a[4], bv[RT][4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int t = c * 64 + 16 * s + 8 * g;
            a[s] = *reinterpret_cast<const uint4 *>(crow + t);
#pragma unroll
            for (int j = 0; j < RT; ++j) bv[j][s] = *reinterpret_cast<const uint4 *>(grow[j] + t);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < RT; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[s]),
                                                                 __builtin_bit_cast(bf16x8_t, bv[j][s]),
                                                                 acc[j], 0, 0, 0);
    }
    constexpr int W = 32 * RT;
    float *mine = part + (size_t)wave * 32 * W;
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            mine[(8 * (e >> 2) + 4 * g + (e & 3)) * W + j * 32 + rl] = acc[j][e];
    __syncthreads();
    for (int idx = tid; idx < 32 * W; idx += 256) {
        const int lr = idx / W, col = idx % W;
        const float v = (part[idx] + part[32 * W + idx]) + (part[2 * 32 * W + idx] + part[3 * 32 * W + idx]);
        if (row0 + lr < M && col < r) T[((size_t)b * M + row0 + lr) * r + col] = v;
    }
}

// fp32 storage: one row of C per workgroup, fp64 accumulation
__global__ __launch_bounds__(256) void t_f32_kernel(const float *__restrict__ cache,
                                                    const float *__restrict__ g_c, int M, int r, int d,
                                                    float *__restrict__ T)
{
    const int b = blockIdx.y, i = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *crow = cache + ((size_t)b * M + i) * d;
    const float *G = g_c + (size_t)b * r * d;
    for (int t = wave; t < r; t += 4) {
        double acc = 0.0;
        for (int j = lane; j < d; j += 64) acc = fma((double)crow[j], (double)G[(size_t)t * d + j], acc);
        acc = wave_sum(acc);
        if (lane == 0) T[((size_t)b * M + i) * r + t] = (float)acc;
    }
}

// ------------------------------------------------------------------ S = G G^T in fp64
// One workgroup per (sample, row a); each wavefront takes columns a' = wave, wave+4, ...
template <typename TT>
__global__ __launch_bounds__(256) void gram_kernel(const TT *__restrict__ g_c, int r, int d,
                                                   double *__restrict__ S)
{
    const int b = blockIdx.y, a = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const TT *G = g_c + (size_t)b * r * d;
    for (int c = wave; c < r; c += 4) {
        double acc = 0.0;
        for (int j = lane; j < d; j += 64)
            acc = fma((double)Elem<TT>::load(G + (size_t)a * d + j), (double)Elem<TT>::load(G + (size_t)c * d + j), acc);
        acc = wave_sum(acc);
        if (lane == 0) S[((size_t)b * r + a) * r + c] = acc;
    }
}

// ------------------------------------------------------------------ S^{-1} by Cholesky
// One workgroup per sample; the matrix lives in LDS with an odd pitch.  Right-looking Cholesky
// S = L L^T into the lower triangle; Y = L^{-1} by forward substitution, one column per thread,
// kept transposed in the strict upper triangle (the diagonals of L and Y are reciprocals of each
// other and live in `dinv`); S^{-1} = Y^T Y.  `ridge` (relative to trace/r) is added to the
// diagonal first.  A Gram matrix that is not positive definite yields non-finite output.
__global__ __launch_bounds__(256) void chol_inverse_kernel(const double *__restrict__ S, int r,
                                                           double ridge, double *__restrict__ Sinv)
{
    extern __shared__ double A[];                 // [r][r+1], then dinv[r]
    const int P = r + 1;
    double *dinv = A + (size_t)r * P;
    __shared__ double red[4];
    const int tid = threadIdx.x, b = blockIdx.x;
    const double *Sb = S + (size_t)b * r * r;
    for (int idx = tid; idx < r * r; idx += 256) A[(idx / r) * P + idx % r] = Sb[idx];
    __syncthreads();
    if (ridge != 0.0) {
        double tr = 0.0;
        for (int i = tid; i < r; i += 256) tr += A[i * P + i];
        tr = wave_sum(tr);
        if ((tid & 63) == 0) red[tid >> 6] = tr;
        __syncthreads();
        const double add = ridge * ((red[0] + red[1]) + (red[2] + red[3])) / (double)r;
        for (int i = tid; i < r; i += 256) A[i * P + i] += add;
        __syncthreads();
    }
    for (int j = 0; j < r; ++j) {
        const double ljj = sqrt(A[j * P + j]);
        __syncthreads();                           // every thread has read the pivot
        for (int i = j + tid; i < r; i += 256) A[i * P + j] = (i == j) ? ljj : A[i * P + j] / ljj;
        __syncthreads();
        const int n = r - j - 1;
        for (int idx = tid; idx < n * n; idx += 256) {
            const int i = j + 1 + idx / n, k = j + 1 + idx % n;
            if (k <= i) A[i * P + k] -= A[i * P + j] * A[k * P + j];
        }
        __syncthreads();
    }
    for (int i = tid; i < r; i += 256) dinv[i] = 1.0 / A[i * P + i];
    __syncthreads();
    // Y = L^{-1}: thread c owns column c, stored as row c of the strict upper triangle
    for (int c = tid; c < r; c += 256) {
        for (int i = c + 1; i < r; ++i) {
            double s = A[i * P + c] * dinv[c];
            for (int k = c + 1; k < i; ++k) s = fma(A[i * P + k], A[c * P + k], s);
            A[c * P + i] = -s * dinv[i];
        }
    }
    __syncthreads();
    // S^{-1}[a][c] = sum_{i >= max(a,c)} Y[i][a] Y[i][c]
    double *out = Sinv + (size_t)b * r * r;
    for (int idx = tid; idx < r * r; idx += 256) {
        const int a = idx / r, c = idx % r;
        const int lo = a < c ? a : c, hi = a < c ? c : a;
        // i == hi: Y[hi][hi] = dinv[hi];  Y[hi][lo] = (lo == hi) ? dinv : A[lo][hi]
        double s = dinv[hi] * (lo == hi ? dinv[hi] : A[lo * P + hi]);
        for (int i = hi + 1; i < r; ++i) s = fma(A[a * P + i], A[c * P + i], s);
        out[idx] = s;
    }
}

// ------------------------------------------------------------------ W = T S^{-1}
template <typename TT>
__global__ __launch_bounds__(256) void w_kernel(const float *__restrict__ T,
                                                const double *__restrict__ Sinv, int M, int r,
                                                TT *__restrict__ w_c)
{
    const int b = blockIdx.y;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)M * r) return;
    const int i = (int)(idx / r), c = (int)(idx % r);
    const float *trow = T + ((size_t)b * M + i) * r;
    const double *Si = Sinv + (size_t)b * r * r;
    double acc = 0.0;
    for (int t = 0; t < r; ++t) acc = fma((double)trow[t], Si[(size_t)t * r + c], acc);
    Elem<TT>::store(w_c + ((size_t)b * M + i) * r + c, (float)acc);
}

void launch_factor_t(DType dt, const void *cache, const void *g_c, int B, int M, int r, int d, float *T,
                     hipStream_t st)
{
    if (dt == DType::BF16) {
        dim3 grid((M + 31) / 32, B);
        const int rt = (r + 31) / 32;
        const size_t lds = (size_t)4 * 32 * 32 * rt * sizeof(float);
#define FVAR_T(RT)                                                                                  \
    do {                                                                                            \
        if (lds > 48 * 1024)                                                                        \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(t_bf16_kernel<RT>),            \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);        \
        launch(t_bf16_kernel<RT>, grid, dim3(256), lds, st, (const uint16_t *)cache,                \
               (const uint16_t *)g_c, M, r, d, T);                                                  \
    } while (0)
        if (rt == 1) FVAR_T(1);
        else if (rt == 2) FVAR_T(2);
        else if (rt == 3) FVAR_T(3);
        else FVAR_T(4);
#undef FVAR_T
    } else {
        launch(t_f32_kernel, dim3(M, B), dim3(256), 0, st, (const float *)cache, (const float *)g_c, M, r,
               d, T);
    }
}

void launch_factor_gram(DType dt, const void *g_c, int B, int r, int d, double *S, hipStream_t st)
{
    if (dt == DType::BF16)
        launch(gram_kernel<uint16_t>, dim3(r, B), dim3(256), 0, st, (const uint16_t *)g_c, r, d, S);
    else
        launch(gram_kernel<float>, dim3(r, B), dim3(256), 0, st, (const float *)g_c, r, d, S);
}

void launch_factor_inverse(const double *S, int B, int r, double ridge, double *Sinv, hipStream_t st)
{
    const size_t lds = ((size_t)r * (r + 1) + r) * sizeof(double);
    if (lds > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(chol_inverse_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    launch(chol_inverse_kernel, dim3(B), dim3(256), lds, st, S, r, ridge, Sinv);
}

void launch_factor_w(DType dt, const float *T, const double *Sinv, int B, int M, int r, void *w_c,
                     hipStream_t st)
{
    dim3 grid((unsigned)(((size_t)M * r + 255) / 256), B);
    if (dt == DType::BF16)
        launch(w_kernel<uint16_t>, grid, dim3(256), 0, st, T, Sinv, M, r, (uint16_t *)w_c);
    else
        launch(w_kernel<float>, grid, dim3(256), 0, st, T, Sinv, M, r, (float *)w_c);
}

}  // namespace fvar
