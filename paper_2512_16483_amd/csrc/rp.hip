// Random projection of a token map (paper, Sec. "Random Projection (RP) for Low-Rank Feature"):
//
//     out[b] = Q^T X[b],   Q^T given as qt[rows][M],  X[b]:[M][d]  ->  out[b]:[rows][d]
//
// used with rows = r on the block input (Alg. "FasterVAR": F^_r = Q^T F~) and on the cached
// counterpart feature (G_c = Q^T C).  The contraction runs over the token axis M, along which X
// is strided, so the bf16 kernel turns each 64-token chunk of X around on its way into LDS
// (4x8 blocks, byte permutes) to give the MFMA B operand its 8 consecutive k values per lane;
// the rows of Q^T are k-contiguous already and go from global memory straight into the A operand.
#include "common.h"

namespace fvar {

constexpr int kRpBM = 128, kRpBN = 128, kRpBK = 64;
constexpr int kRpPitch = kRpBK + 8;          // X^T row pitch (elements): 9 chunks of 16 bytes
constexpr int kRpOutPitch = kRpBN + 8;       // output staging pitch

__global__ __launch_bounds__(256) void rp_project_bf16_kernel(const uint16_t *__restrict__ qt,
                                                              size_t q_stride,
                                                              const uint16_t *__restrict__ x, int M,
                                                              int rows, int d,
                                                              uint16_t *__restrict__ out)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * kRpBN * kRpPitch];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int col0 = blockIdx.x * kRpBN, row0 = blockIdx.y * kRpBM, b = blockIdx.z;
    const uint16_t *Q = qt + (size_t)b * q_stride;
    const uint16_t *X = x + (size_t)b * M * d;
    uint16_t *O = out + (size_t)b * rows * d;

    // this thread's 4x8 block of every X chunk
    const int cb = tid & 15, tb = tid >> 4;
    const int xc = col0 + cb * 8;
    const bool col_ok = xc < d;
    auto load_x = [&](int k0, uint4 (&v)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = k0 + tb * 4 + j;
            v[j] = (col_ok && t < M) ? *reinterpret_cast<const uint4 *>(X + (size_t)t * d + xc)
                                     : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_xt = [&](uint16_t *buf, const uint4 (&v)[4]) {
        const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&v[0]);
        const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&v[1]);
        const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&v[2]);
        const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&v[3]);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            uint2 lo, hi;
            lo.x = __builtin_amdgcn_perm(w1[m], w0[m], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(w3[m], w2[m], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(w1[m], w0[m], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(w3[m], w2[m], 0x07060302u);
            *reinterpret_cast<uint2 *>(buf + (cb * 8 + 2 * m) * kRpPitch + tb * 4) = lo;
            *reinterpret_cast<uint2 *>(buf + (cb * 8 + 2 * m + 1) * kRpPitch + tb * 4) = hi;
        }
    };
    // A operand rows of this lane (clamped: rows past the end are computed and dropped)
    const uint16_t *qrow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        qrow[i] = Q + (size_t)min(row0 + wm * 64 + i * 32 + rl, rows - 1) * M;
    auto load_a = [&](int k0, uint4 (&a)[2][4]) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int t = k0 + 16 * s + 8 * g;
                a[i][s] = t < M ? *reinterpret_cast<const uint4 *>(qrow[i] + t) : make_uint4(0, 0, 0, 0);
            }
    };

    floatx16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = floatx16_t{0};

    const int nchunks = (M + kRpBK - 1) / kRpBK;
    uint4 xv[4], av[2][4];
    load_x(0, xv);
    load_a(0, av);
    store_xt(lds, xv);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        uint16_t *cur = lds + (c & 1) * (kRpBN * kRpPitch);
        uint16_t *nxt = lds + ((c + 1) & 1) * (kRpBN * kRpPitch);
        const bool more = c + 1 < nchunks;
        uint4 an[2][4];
        if (more) {
            load_x((c + 1) * kRpBK, xv);
            load_a((c + 1) * kRpBK, an);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8_t bf[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                bf[j] = *reinterpret_cast<const bf16x8_t *>(cur + (wn * 64 + j * 32 + rl) * kRpPitch +
                                                            16 * s + 8 * g);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, av[i][s]), bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            store_xt(nxt, xv);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int s = 0; s < 4; ++s) av[i][s] = an[i][s];
        }
        __syncthreads();
    }

    // accumulators -> bf16 row-major in LDS (neighbouring lanes swap one value per row pair so a
    // lane owns two adjacent columns), then 16-byte row chunks to global memory
    uint16_t *stage = lds;                    // 128 x kRpOutPitch elements fit the two X^T buffers
    const int odd = lane & 1;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int lcol = wn * 64 + j * 32 + rl - odd;
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float v0 = acc[i][j][e], v1 = acc[i][j][e + 1];
                const float recv = __shfl_xor(odd ? v0 : v1, 1);
                const int lrow = wm * 64 + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3) + odd;
                *reinterpret_cast<uint32_t *>(stage + lrow * kRpOutPitch + lcol) =
                    odd ? pack_bf16x2(recv, v1) : pack_bf16x2(v0, recv);
            }
        }
    __syncthreads();
    const int c8 = (tid & 15) * 8;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int lrow = it * 16 + (tid >> 4), rr = row0 + lrow;
        if (rr < rows && col0 + c8 < d)
            *reinterpret_cast<uint4 *>(O + (size_t)rr * d + col0 + c8) =
                *reinterpret_cast<const uint4 *>(stage + lrow * kRpOutPitch + c8);
    }
}

// fp32 path (parity configuration): eight output rows per workgroup, one column per thread
__global__ __launch_bounds__(256) void rp_project_f32_kernel(const float *__restrict__ qt,
                                                             size_t q_stride,
                                                             const float *__restrict__ x, int M,
                                                             int rows, int d, float *__restrict__ out)
{
    const int b = blockIdx.z, t0 = blockIdx.y * 8;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    const float *Q = qt + (size_t)b * q_stride;
    const float *X = x + (size_t)b * M * d;
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = 0; i < M; ++i) {
        const double xv = X[(size_t)i * d + j];
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = fma((double)Q[(size_t)min(t0 + t, rows - 1) * M + i], xv, acc[t]);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t0 + t < rows) out[((size_t)b * rows + t0 + t) * d + j] = (float)acc[t];
}

void launch_rp_project(DType dt, const void *qt, size_t q_stride, const void *x, int B, int M,
                       int rows, int d, void *out, hipStream_t st)
{
    if (dt == DType::BF16) {
        dim3 grid((d + kRpBN - 1) / kRpBN, (rows + kRpBM - 1) / kRpBM, B);
        launch(rp_project_bf16_kernel, grid, dim3(256), 0, st, (const uint16_t *)qt, q_stride,
               (const uint16_t *)x, M, rows, d, (uint16_t *)out);
    } else {
        dim3 grid((d + 255) / 256, (rows + 7) / 8, B);
        launch(rp_project_f32_kernel, grid, dim3(256), 0, st, (const float *)qt, q_stride,
               (const float *)x, M, rows, d, (float *)out);
    }
}

}  // namespace fvar
