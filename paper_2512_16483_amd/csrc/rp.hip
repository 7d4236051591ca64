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

constexpr int kRpBN = 128, kRpBK = 64;
constexpr int kRpPitch = kRpBK;              // X^T row = 8 chunks of 16 bytes, swizzled
constexpr int kRpOutPitch = kRpBN + 8;       // output staging pitch

// Chunk swizzle of the X^T tile (rows = columns of X, 8 chunks of 8 tokens).  MFMA operand reads
// fetch 16 consecutive rows at one logical chunk: (row/2)%8 spreads those over all 64 banks, and
// the other terms are constant inside an aligned group of 16 rows.  The transposing stores write
// 8-byte halves to rows 8 apart; the row/16 terms send those to different chunks.
__device__ __forceinline__ int xt_swz(int row)
{
    return ((row >> 1) & 7) ^ (((row >> 4) & 1) << 2) ^ ((row >> 5) & 3);
}

// BM = output rows per workgroup (128, or 64 when few rows are asked for); the four wavefronts
// form a 2 x 2 grid of (BM/2) x 64 tiles.
template <int BM>
__global__ __launch_bounds__(256) void rp_project_bf16_kernel(const uint16_t *__restrict__ qt,
                                                              size_t q_stride,
                                                              const uint16_t *__restrict__ x, int M,
                                                              int rows, int d,
                                                              uint16_t *__restrict__ out)
{
    // two X^T buffers during the main loop, the BM x kRpOutPitch output staging afterwards
    constexpr int kLdsElems = 2 * kRpBN * kRpPitch > BM * kRpOutPitch ? 2 * kRpBN * kRpPitch
                                                                      : BM * kRpOutPitch;
    __shared__ __attribute__((aligned(16))) uint16_t lds[kLdsElems];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int MI = BM / 64;                // 32-row MFMA tiles per wavefront
    const int col0 = blockIdx.x * kRpBN, row0 = blockIdx.y * BM, b = blockIdx.z;
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
            // threads of odd column blocks store the odd row first, so that one store instruction
            // touches rows of both parities (both halves of the banks)
            const int r0 = cb * 8 + 2 * m, r1 = r0 + 1;
            const int ra = (cb & 1) ? r1 : r0, rb = (cb & 1) ? r0 : r1;
            const int chunk = tb >> 1, sub = (tb & 1) * 4;
            *reinterpret_cast<uint2 *>(buf + ra * kRpPitch + ((chunk ^ xt_swz(ra)) << 3) + sub) =
                (cb & 1) ? hi : lo;
            *reinterpret_cast<uint2 *>(buf + rb * kRpPitch + ((chunk ^ xt_swz(rb)) << 3) + sub) =
                (cb & 1) ? lo : hi;
        }
    };
    // A operand rows of this lane (clamped: rows past the end are computed and dropped)
    const uint16_t *qrow[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
        qrow[i] = Q + (size_t)min(row0 + wm * (BM / 2) + i * 32 + rl, rows - 1) * M;
    auto load_a = [&](int k0, uint4 (&a)[MI][4]) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int t = k0 + 16 * s + 8 * g;
                a[i][s] = t < M ? *reinterpret_cast<const uint4 *>(qrow[i] + t) : make_uint4(0, 0, 0, 0);
            }
    };

    floatx16_t acc[MI][2];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = floatx16_t{0};

    const int nchunks = (M + kRpBK - 1) / kRpBK;
    uint4 xv[4], av[MI][4];
    load_x(0, xv);
    load_a(0, av);
    store_xt(lds, xv);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        uint16_t *cur = lds + (c & 1) * (kRpBN * kRpPitch);
        uint16_t *nxt = lds + ((c + 1) & 1) * (kRpBN * kRpPitch);
        const bool more = c + 1 < nchunks;
        uint4 an[MI][4];
        if (more) {
            load_x((c + 1) * kRpBK, xv);
            load_a((c + 1) * kRpBK, an);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8_t bf[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = wn * 64 + j * 32 + rl;
                bf[j] = *reinterpret_cast<const bf16x8_t *>(cur + row * kRpPitch +
                                                            (((2 * s + g) ^ xt_swz(row)) << 3));
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, av[i][s]), bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            store_xt(nxt, xv);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int s = 0; s < 4; ++s) av[i][s] = an[i][s];
        }
        __syncthreads();
    }

    // accumulators -> bf16 row-major in LDS (neighbouring lanes swap one value per row pair so a
    // lane owns two adjacent columns), then 16-byte row chunks to global memory
    uint16_t *stage = lds;
    const int odd = lane & 1;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int lcol = wn * 64 + j * 32 + rl - odd;
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float v0 = acc[i][j][e], v1 = acc[i][j][e + 1];
                const float recv = __shfl_xor(odd ? v0 : v1, 1);
                const int lrow = wm * (BM / 2) + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3) + odd;
                *reinterpret_cast<uint32_t *>(stage + lrow * kRpOutPitch + lcol) =
                    odd ? pack_bf16x2(recv, v1) : pack_bf16x2(v0, recv);
            }
        }
    __syncthreads();
    const int c8 = (tid & 15) * 8;
#pragma unroll
    for (int it = 0; it < BM / 16; ++it) {
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
        // large problems on whole k-tiles go to the tiled MFMA kernel of the linear layers
        if (launch_gemm_bf16_kmajor(qt, q_stride, x, B, M, rows, d, out, st)) return;
        if (rows <= 64 || (rows > 128 && rows <= 192)) {
            dim3 grid((d + kRpBN - 1) / kRpBN, (rows + 63) / 64, B);
            launch(rp_project_bf16_kernel<64>, grid, dim3(256), 0, st, (const uint16_t *)qt, q_stride,
                   (const uint16_t *)x, M, rows, d, (uint16_t *)out);
        } else {
            dim3 grid((d + kRpBN - 1) / kRpBN, (rows + 127) / 128, B);
            launch(rp_project_bf16_kernel<128>, grid, dim3(256), 0, st, (const uint16_t *)qt, q_stride,
                   (const uint16_t *)x, M, rows, d, (uint16_t *)out);
        }
    } else {
        dim3 grid((d + 255) / 256, (rows + 7) / 8, B);
        launch(rp_project_f32_kernel, grid, dim3(256), 0, st, (const float *)qt, q_stride,
               (const float *)x, M, rows, d, (float *)out);
    }
}

}  // namespace fvar
