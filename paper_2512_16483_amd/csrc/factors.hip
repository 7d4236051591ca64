// Restoration matrix of the cached counterpart feature by linear least squares (paper, Eq.
// "lstsq" with the cached feature in place of the input, App. "Construction of W_r^o"):
//
//     W_c = argmin_W || W G_c - C ||_F = (C G_c^T) (G_c G_c^T)^{-1},     G_c = Q^T C  as stored.
//
// Four kernels per call (the projection G_c itself is the kernel of rp.hip):
//   t_kernel      T = C G_c^T            [M,r]  fp32; bf16 inputs on MFMA, the second pass over C
//   gram_kernel   S = G_c G_c^T          [r,r]  fp64 (bf16: MFMA per 64-element chunk, fp64 across)
//   spd_inverse   S^{-1}                 Gauss-Jordan in registers, one workgroup per sample, fp64
//   w_kernel      W_c = T S^{-1}         [M,r]  fp64 accumulation, rounded to the storage type
#include "common.h"

namespace fvar {

// ------------------------------------------------------------------ T = C G^T, bf16 on MFMA
// Workgroup = 64 rows of C and one slice of the contraction axis: the 64-element chunks
// c = part*4 + wave, + 4*parts, ... go to its four wavefronts (each reads a 128-byte segment of
// every row per chunk, the next chunk's loads in flight under the current chunk's MFMAs); the
// four partial 64 x r tiles are added through LDS and written to Tpart[part].  The slices are
// summed by the kernel that consumes T.  RT = r / 32 rounded up.
template <int RT>
__global__ __launch_bounds__(256) void t_bf16_kernel(const uint16_t *__restrict__ cache,
                                                     const uint16_t *__restrict__ g_c, int B, int M,
                                                     int r, int d, float *__restrict__ Tpart)
{
    extern __shared__ float part_lds[];             // [4][64][32*RT]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    const int row0 = blockIdx.x * 64, part = blockIdx.y, parts = gridDim.y, b = blockIdx.z;
    const uint16_t *crow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        crow[i] = cache + ((size_t)b * M + min(row0 + 32 * i + rl, M - 1)) * d + 8 * g;
    const uint16_t *G = g_c + (size_t)b * r * d;
    const uint16_t *grow[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j) grow[j] = G + (size_t)min(j * 32 + rl, r - 1) * d + 8 * g;

    floatx16_t acc[2][RT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j) acc[i][j] = floatx16_t{0};
    const int nchunks = d / 64, stride = 4 * parts;
    uint4 a[2][4], bv[RT][4];
    auto load = [&](int c, uint4 (&av)[2][4], uint4 (&bw)[RT][4]) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int t = c * 64 + 16 * s;
#pragma unroll
            for (int i = 0; i < 2; ++i) av[i][s] = *reinterpret_cast<const uint4 *>(crow[i] + t);
#pragma unroll
            for (int j = 0; j < RT; ++j) bw[j][s] = *reinterpret_cast<const uint4 *>(grow[j] + t);
        }
    };
    int c = part * 4 + wave;
    if (c < nchunks) load(c, a, bv);
    for (; c < nchunks; c += stride) {
        uint4 an[2][4], bn[RT][4];
        const bool more = c + stride < nchunks;
        if (more) load(c + stride, an, bn);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < RT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, a[i][s]), __builtin_bit_cast(bf16x8_t, bv[j][s]),
                        acc[i][j], 0, 0, 0);
        if (more) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i][s] = an[i][s];
#pragma unroll
                for (int j = 0; j < RT; ++j) bv[j][s] = bn[j][s];
            }
        }
    }
    constexpr int W = 32 * RT;
    float *mine = part_lds + (size_t)wave * 64 * W;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                mine[(32 * i + 8 * (e >> 2) + 4 * g + (e & 3)) * W + j * 32 + rl] = acc[i][j][e];
    __syncthreads();
    float *T = Tpart + (size_t)part * B * M * r;
    for (int idx = tid; idx < 64 * W; idx += 256) {
        const int lr = idx / W, col = idx % W;
        const float v = (part_lds[idx] + part_lds[64 * W + idx]) +
                        (part_lds[2 * 64 * W + idx] + part_lds[3 * 64 * W + idx]);
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

// ------------------------------------------------------------------ S = G G^T
// fp32 storage: one workgroup of 16 wavefronts per (sample, row a); the row is parked in LDS,
// each wavefront takes columns c = wave, wave+16, ... <= a, fp64 products and sums.
constexpr int kGramThreads = 1024;
__global__ __launch_bounds__(kGramThreads) void gram_f32_kernel(const float *__restrict__ g_c, int r,
                                                                int d, double *__restrict__ S)
{
    extern __shared__ float rowa[];                 // [d]
    const int b = blockIdx.y, a = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *G = g_c + (size_t)b * r * d;
    for (int j = threadIdx.x; j < d; j += kGramThreads) rowa[j] = G[(size_t)a * d + j];
    __syncthreads();
    double *Sb = S + (size_t)b * r * r;
    for (int c = wave; c <= a; c += kGramThreads / 64) {
        double acc = 0.0;
        for (int j = lane; j < d; j += 64) acc = fma((double)G[(size_t)c * d + j], (double)rowa[j], acc);
        acc = wave_sum(acc);
        if (lane == 0) {
            Sb[(size_t)a * r + c] = acc;
            Sb[(size_t)c * r + a] = acc;
        }
    }
}

// bf16 storage, on MFMA.  A workgroup owns one 32x32 tile (ti >= tj) of S for one slice of the
// contraction axis: the 64-element chunks c = part, part + parts, ... are dealt round-robin to its
// four wavefronts.  Within a chunk the products (exact in fp32) are summed in fp32; chunk results
// are added in fp64.  The slices' partial matrices are written to Spart[b][part] (both triangles)
// and summed by the factorisation kernel, so the result does not depend on scheduling.
constexpr int kGramParts = 8;
__global__ __launch_bounds__(256) void gram_bf16_kernel(const uint16_t *__restrict__ g_c, int r, int d,
                                                        double *__restrict__ Spart)
{
    __shared__ double red[4][32 * 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    int ti = 0;
    while ((ti + 1) * (ti + 2) / 2 <= (int)blockIdx.x) ++ti;
    const int tj = blockIdx.x - ti * (ti + 1) / 2;
    const int part = blockIdx.y, parts = gridDim.y, b = blockIdx.z;
    const uint16_t *G = g_c + (size_t)b * r * d;
    const uint16_t *arow = G + (size_t)min(ti * 32 + rl, r - 1) * d;
    const uint16_t *brow = G + (size_t)min(tj * 32 + rl, r - 1) * d;
    double acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.0;
    const int nchunks = d / 64;
    for (int c = part + parts * wave; c < nchunks; c += parts * 4) {
        floatx16_t a32 = {0};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int t = c * 64 + 16 * s + 8 * g;
            const uint4 av = *reinterpret_cast<const uint4 *>(arow + t);
            const uint4 bv = *reinterpret_cast<const uint4 *>(brow + t);
            a32 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av),
                                                          __builtin_bit_cast(bf16x8_t, bv), a32, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] += (double)a32[e];
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][(8 * (e >> 2) + 4 * g + (e & 3)) * 32 + rl] = acc[e];
    __syncthreads();
    double *Sb = Spart + ((size_t)b * parts + part) * r * r;
    for (int idx = tid; idx < 32 * 32; idx += 256) {
        const int i = ti * 32 + idx / 32, j = tj * 32 + idx % 32;
        const double v = (red[0][idx] + red[1][idx]) + (red[2][idx] + red[3][idx]);
        if (i < r && j < r) {
            Sb[(size_t)i * r + j] = v;
            if (ti != tj) Sb[(size_t)j * r + i] = v;
        }
    }
}

// ------------------------------------------------------------------ S^{-1}
// One workgroup per sample inverts the symmetric positive definite Gram matrix (the sum of the
// `parts` partial matrices, plus ridge * trace / r on the diagonal) by in-place Gauss-Jordan
// elimination without pivoting, in fp64.  The matrix is padded to RP x RP with an identity block
// and lives in REGISTERS for the whole elimination: thread t owns the NC = RP*RP/256 consecutive
// columns [cb*NC, cb*NC+NC) of row i = t / TPR, cb = t % TPR.
//
// Step j with pivot p = 1/a_jj turns   a_ik -> a_ik - a_ij p a_jk   (i != j, k != j),
// a_ij -> -a_ij p,  a_jk -> a_jk p,  a_jj -> p.  It needs the pivot row, the pivot column and p
// from other threads; their owners publish them in LDS at the end of step j-1 (two buffers in
// turn, one barrier per step).  The published row carries a_jj + 1 at column j: then the general
// update f - f p (a_jj + 1) = -f p also covers the pivot column, and only the threads of the
// pivot row take a separate branch.  Steps are numbered j = jo*NC + ji with ji unrolled, so that
// the column a thread has to publish is a compile-time register index.
// A singular matrix yields non-finite output.
template <int RP>
__global__ __launch_bounds__(256) void spd_inverse_kernel(const double *__restrict__ S, int parts,
                                                          int r, double ridge,
                                                          double *__restrict__ Sinv)
{
    constexpr int TPR = 256 / RP;                  // threads per row
    constexpr int NC = RP / TPR;                   // columns per thread
    __shared__ __attribute__((aligned(16))) double rowbuf[2][RP];
    __shared__ double colbuf[2][RP], pinv[2], red[4];
    const int tid = threadIdx.x, b = blockIdx.x;
    const int i = tid / TPR, cb = tid % TPR, k0 = cb * NC;
    const double *Sb = S + (size_t)b * parts * r * r;
    double a[NC];
#pragma unroll
    for (int q = 0; q < NC; ++q) {
        const int k = k0 + q;
        double v = (i == k) ? 1.0 : 0.0;           // identity padding
        if (i < r && k < r) {
            v = 0.0;
            for (int p = 0; p < parts; ++p) v += Sb[((size_t)p * r + i) * r + k];
        }
        a[q] = v;
    }
    if (ridge != 0.0) {
        double tr = 0.0;
#pragma unroll
        for (int q = 0; q < NC; ++q) tr += (k0 + q == i && i < r) ? a[q] : 0.0;
        tr = wave_sum(tr);
        if ((tid & 63) == 0) red[tid >> 6] = tr;
        __syncthreads();
        const double add = ridge * ((red[0] + red[1]) + (red[2] + red[3])) / (double)r;
#pragma unroll
        for (int q = 0; q < NC; ++q) a[q] += (k0 + q == i && i < r) ? add : 0.0;
    }
    // row and column jo*NC + JI of the current matrix, and the reciprocal pivot, into buffer `buf`
#define FVAR_GJ_PUBLISH(jo_, JI, buf_)                                                            \
    do {                                                                                           \
        const bool own_col = cb == (jo_);                                                          \
        if (own_col) colbuf[buf_][i] = a[JI];                                                      \
        if (i == (jo_) * NC + (JI)) {                                                              \
            _Pragma("unroll") for (int q = 0; q < NC; ++q)                                         \
                rowbuf[buf_][k0 + q] = a[q] + ((own_col && q == (JI)) ? 1.0 : 0.0);                \
            if (own_col) pinv[buf_] = 1.0 / a[JI];                                                 \
        }                                                                                          \
    } while (0)
    FVAR_GJ_PUBLISH(0, 0, 0);
    __syncthreads();
    for (int jo = 0; jo * NC < r; ++jo) {
#pragma unroll
        for (int ji = 0; ji < NC; ++ji) {
            const int j = jo * NC + ji;            // uniform
            if (j < r) {
                const int buf = ji & 1;            // NC is even, so the parity of j is that of ji
                const double p = pinv[buf];
                const double fp = colbuf[buf][i] * p;
                if (i == j) {
#pragma unroll
                    for (int q = 0; q < NC; ++q) a[q] = (cb == jo && q == ji) ? p : a[q] * p;
                } else {
#pragma unroll
                    for (int q = 0; q < NC; ++q) a[q] = fma(-fp, rowbuf[buf][k0 + q], a[q]);
                }
                if (j + 1 < r) FVAR_GJ_PUBLISH(jo + (ji + 1 == NC ? 1 : 0), (ji + 1) % NC, buf ^ 1);
                __syncthreads();
            }
        }
    }
#undef FVAR_GJ_PUBLISH
    if (i < r) {
        double *out = Sinv + ((size_t)b * r + i) * r;
#pragma unroll
        for (int q = 0; q < NC; ++q)
            if (k0 + q < r) out[k0 + q] = a[q];
    }
}

// ------------------------------------------------------------------ W = T S^{-1}
// Workgroup = 64 * RPL rows of T; S^{-1} is staged in LDS (fp64).  Wavefront w produces the w-th
// quarter of the r columns, a lane owns RPL rows (64 apart): every lane of a wavefront reads the
// same S^{-1} entries (LDS broadcast, one read serves RPL FMAs) and walks its own rows of T (the
// sum of their one or two slices).  CQ = columns per wavefront (r / 4 rounded up).
template <typename TT, int CQ, int RPL>
__global__ __launch_bounds__(256) void w_kernel(const float *__restrict__ T, int t_parts,
                                                size_t t_part_stride,
                                                const double *__restrict__ Sinv, int M, int r,
                                                TT *__restrict__ w_c)
{
    extern __shared__ double Si[];                 // [r][4*CQ], zero padded columns
    constexpr int PW = 4 * CQ;
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double *Sg = Sinv + (size_t)b * r * r;
    for (int idx = tid; idx < r * PW; idx += 256) {
        const int t = idx / PW, c = idx % PW;
        Si[idx] = c < r ? Sg[(size_t)t * r + c] : 0.0;
    }
    __syncthreads();
    const int row0 = blockIdx.x * (64 * RPL) + lane;
    const float *trow[RPL];
#pragma unroll
    for (int p = 0; p < RPL; ++p) trow[p] = T + ((size_t)b * M + min(row0 + 64 * p, M - 1)) * r;
    double acc[RPL][CQ];
#pragma unroll
    for (int p = 0; p < RPL; ++p)
#pragma unroll
        for (int q = 0; q < CQ; ++q) acc[p][q] = 0.0;
    const double *sw = Si + wave * CQ;
    for (int t0 = 0; t0 < r; t0 += 4) {            // r is a multiple of 4
        float4 tv[RPL];
#pragma unroll
        for (int p = 0; p < RPL; ++p) {
            tv[p] = *reinterpret_cast<const float4 *>(trow[p] + t0);
            if (t_parts > 1) {                     // second slice of the contraction axis
                const float4 tp = *reinterpret_cast<const float4 *>(trow[p] + t_part_stride + t0);
                tv[p].x += tp.x; tv[p].y += tp.y; tv[p].z += tp.z; tv[p].w += tp.w;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            double td[RPL];
#pragma unroll
            for (int p = 0; p < RPL; ++p)
                td[p] = (double)(u == 0 ? tv[p].x : u == 1 ? tv[p].y : u == 2 ? tv[p].z : tv[p].w);
#pragma unroll
            for (int q = 0; q < CQ; ++q) {
                const double sv = sw[(t0 + u) * PW + q];
#pragma unroll
                for (int p = 0; p < RPL; ++p) acc[p][q] = fma(td[p], sv, acc[p][q]);
            }
        }
    }
#pragma unroll
    for (int p = 0; p < RPL; ++p) {
        const int row = row0 + 64 * p;
        if (row >= M) continue;
        TT *out = w_c + ((size_t)b * M + row) * r;
#pragma unroll
        for (int q = 0; q < CQ; ++q) {
            const int c = wave * CQ + q;
            if (c < r) Elem<TT>::store(out + c, (float)acc[p][q]);
        }
    }
}

// Slices of the contraction axis in the bf16 T kernel: enough workgroups to fill the chip when
// the batch is small, none extra when it is large.
int factor_t_parts(DType dt, int B, int M)
{
    if (dt != DType::BF16) return 1;
    const long wgs = (long)B * ((M + 63) / 64);
    int parts = (int)((512 + wgs - 1) / wgs);
    return parts < 1 ? 1 : (parts > 2 ? 2 : parts);
}

void launch_factor_t(DType dt, const void *cache, const void *g_c, int B, int M, int r, int d, float *T,
                     hipStream_t st)
{
    if (dt == DType::BF16) {
        // many samples at once (the caches of all blocks of a scale): T = C G^T is an ordinary
        // linear layer per sample, run on the tiled MFMA kernel with fp32 output
        if (factor_t_parts(dt, B, M) == 1 && launch_gemm_bf16_batched_f32(cache, g_c, B, M, r, d, T, st))
            return;
        dim3 grid((M + 63) / 64, factor_t_parts(dt, B, M), B);
        const int rt = (r + 31) / 32;
        const size_t lds = (size_t)4 * 64 * 32 * rt * sizeof(float);
#define FVAR_T(RT)                                                                                  \
    do {                                                                                            \
        if (lds > 48 * 1024)                                                                        \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(t_bf16_kernel<RT>),            \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);        \
        launch(t_bf16_kernel<RT>, grid, dim3(256), lds, st, (const uint16_t *)cache,                \
               (const uint16_t *)g_c, B, M, r, d, T);                                               \
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
    if (dt == DType::BF16) {
        const int rt = (r + 31) / 32;
        launch(gram_bf16_kernel, dim3(rt * (rt + 1) / 2, kGramParts, B), dim3(256), 0, st,
               (const uint16_t *)g_c, r, d, S);
    } else {
        launch(gram_f32_kernel, dim3(r, B), dim3(kGramThreads), (size_t)d * sizeof(float), st,
               (const float *)g_c, r, d, S);
    }
}

int gram_parts(DType dt) { return dt == DType::BF16 ? kGramParts : 1; }

void launch_factor_inverse(const double *S, int parts, int B, int r, double ridge, double *Sinv,
                           hipStream_t st)
{
    if (r <= 32)
        launch(spd_inverse_kernel<32>, dim3(B), dim3(256), 0, st, S, parts, r, ridge, Sinv);
    else if (r <= 64)
        launch(spd_inverse_kernel<64>, dim3(B), dim3(256), 0, st, S, parts, r, ridge, Sinv);
    else
        launch(spd_inverse_kernel<128>, dim3(B), dim3(256), 0, st, S, parts, r, ridge, Sinv);
}

template <typename TT>
static void launch_w_t(const float *T, int t_parts, const double *Sinv, int B, int M, int r, void *w_c,
                       hipStream_t st)
{
    const size_t t_stride = (size_t)B * M * r;
    // two rows per lane once that still leaves a workgroup for every CU
    const bool two = (long)B * ((M + 127) / 128) >= 256;
    dim3 grid(two ? (M + 127) / 128 : (M + 63) / 64, B);
    const int cq = (r + 3) / 4;
#define FVAR_W(CQ)                                                                                 \
    do {                                                                                           \
        const size_t lds = (size_t)r * 4 * CQ * sizeof(double);                                    \
        auto k1 = w_kernel<TT, CQ, 1>;                                                             \
        auto k2 = w_kernel<TT, CQ, 2>;                                                             \
        auto kern = two ? k2 : k1;                                                                 \
        if (lds > 48 * 1024)                                                                       \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                        \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);       \
        launch(kern, grid, dim3(256), lds, st, T, t_parts, t_stride, Sinv, M, r, (TT *)w_c);       \
    } while (0)
    if (cq <= 8) FVAR_W(8);
    else if (cq <= 16) FVAR_W(16);
    else if (cq <= 24) FVAR_W(24);
    else FVAR_W(32);
#undef FVAR_W
}

void launch_factor_w(DType dt, const float *T, const double *Sinv, int B, int M, int r, void *w_c,
                     hipStream_t st)
{
    const int tp = factor_t_parts(dt, B, M);
    if (dt == DType::BF16) launch_w_t<uint16_t>(T, tp, Sinv, B, M, r, w_c, st);
    else launch_w_t<float>(T, tp, Sinv, B, M, r, w_c, st);
}

}  // namespace fvar
