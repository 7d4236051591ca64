// Row pass: (M,d) -> (k,d) gather of the kept token rows, fused with the LayerNorm that opens
// the block (paper, Sec. "Plug-and-Play Acceleration": the block sees k rows instead of M).
// One wavefront per output row; the row lives in registers between the statistics and the
// normalisation, every global access is a 16-byte chunk and a row is read exactly once.
#include "common.h"

namespace fvar {

// CH = 16-byte chunks per lane (row length <= 64 * CH chunks)
template <typename T, int CH>
__global__ __launch_bounds__(256) void gather_ln_kernel(const T *__restrict__ x,
                                                        const int32_t *__restrict__ idx, int M, int n,
                                                        int total_rows, int d,
                                                        const T *__restrict__ gamma,
                                                        const T *__restrict__ beta, float eps,
                                                        T *__restrict__ copy_out,
                                                        T *__restrict__ ln_out)
{
    constexpr int E = Elem<T>::kPerChunk;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;          // output row in [0, B*n)
    if (row >= total_rows) return;
    const int b = row / n;
    const int src_row = idx ? idx[row] : (row - b * n);
    const uint4 *src = reinterpret_cast<const uint4 *>(x + ((size_t)b * M + src_row) * d);
    const int nchunk = d / E;

    uint4 raw[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        int ci = lane + 64 * c;
        raw[c] = ci < nchunk ? src[ci] : make_uint4(0, 0, 0, 0);
    }
    if (copy_out) {
        uint4 *dst = reinterpret_cast<uint4 *>(copy_out + (size_t)row * d);
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            int ci = lane + 64 * c;
            if (ci < nchunk) dst[ci] = raw[c];
        }
    }
    if (!ln_out) return;

    float v[CH][E];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        Elem<T>::unpack(raw[c], v[c]);
#pragma unroll
        for (int e = 0; e < E; ++e) sum += v[c][e];        // padded chunks hold zeros
    }
    const float mu = wave_sum(sum) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const bool in = lane + 64 * c < nchunk;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float t = v[c][e] - mu;
            v[c][e] = t;
            sq += in ? t * t : 0.f;
        }
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);

    uint4 *dst = reinterpret_cast<uint4 *>(ln_out + (size_t)row * d);
    const uint4 *g4 = reinterpret_cast<const uint4 *>(gamma);
    const uint4 *b4 = reinterpret_cast<const uint4 *>(beta);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        int ci = lane + 64 * c;
        if (ci >= nchunk) continue;
        float o[E];
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = v[c][e] * rstd;
        if (gamma) {
            float g[E];
            Elem<T>::unpack(g4[ci], g);
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] *= g[e];
        }
        if (beta) {
            float bb[E];
            Elem<T>::unpack(b4[ci], bb);
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] += bb[e];
        }
        dst[ci] = Elem<T>::pack(o);
    }
}

// LayerNorm of the fp32 intermediate residual stream into the bf16 operand of the MLP.
// One wavefront per row; CH = 16-byte (4 float) chunks per lane.
template <int CH>
__global__ __launch_bounds__(256) void ln_f32_to_bf16_kernel(const float *__restrict__ h, int rows,
                                                             int d,
                                                             const uint16_t *__restrict__ gamma,
                                                             const uint16_t *__restrict__ beta,
                                                             float eps, uint16_t *__restrict__ out)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= rows) return;
    const uint4 *src = reinterpret_cast<const uint4 *>(h + (size_t)row * d);
    const int nchunk = d / 4;
    float v[CH][4];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int ci = lane + 64 * c;
        const uint4 raw = ci < nchunk ? src[ci] : make_uint4(0, 0, 0, 0);
        Elem<float>::unpack(raw, v[c]);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += v[c][e];
    }
    const float mu = wave_sum(sum) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const bool in = lane + 64 * c < nchunk;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float t = v[c][e] - mu;
            v[c][e] = t;
            sq += in ? t * t : 0.f;
        }
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
    uint2 *dst = reinterpret_cast<uint2 *>(out + (size_t)row * d);
    const uint2 *g2 = reinterpret_cast<const uint2 *>(gamma);
    const uint2 *b2 = reinterpret_cast<const uint2 *>(beta);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int ci = lane + 64 * c;
        if (ci >= nchunk) continue;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = v[c][e] * rstd;
        if (gamma) {
            const uint2 gv = g2[ci];
            o[0] *= bf16_lo(gv.x); o[1] *= bf16_hi(gv.x); o[2] *= bf16_lo(gv.y); o[3] *= bf16_hi(gv.y);
        }
        if (beta) {
            const uint2 bv = b2[ci];
            o[0] += bf16_lo(bv.x); o[1] += bf16_hi(bv.x); o[2] += bf16_lo(bv.y); o[3] += bf16_hi(bv.y);
        }
        dst[ci] = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
    }
}

void launch_ln_f32_to_bf16(const float *h, int rows, int d, const void *gamma, const void *beta,
                           float eps, void *ln_out, hipStream_t st)
{
    const int ch = (d / 4 + 63) / 64;
    dim3 grid((rows + 3) / 4), block(256);
#define FVAR_LN32(CH)                                                                          \
    launch(ln_f32_to_bf16_kernel<CH>, grid, block, 0, st, h, rows, d, (const uint16_t *)gamma,  \
           (const uint16_t *)beta, eps, (uint16_t *)ln_out)
    if (ch <= 4) FVAR_LN32(4);
    else if (ch <= 8) FVAR_LN32(8);
    else if (ch <= 16) FVAR_LN32(16);
    else FVAR_LN32(32);
#undef FVAR_LN32
}

template <typename T>
static void launch_gather_ln_t(const void *x, const int32_t *idx, int B, int M, int n, int d,
                               const void *gamma, const void *beta, float eps, void *copy_out,
                               void *ln_out, hipStream_t st)
{
    const int total = B * n;
    const int nchunk = d / Elem<T>::kPerChunk;
    const int ch = (nchunk + 63) / 64;
    dim3 grid((total + 3) / 4), block(256);
#define FVAR_GLN(CH)                                                                             \
    launch((gather_ln_kernel<T, CH>), grid, block, 0, st, (const T *)x, idx, M, n,    \
                       total, d, (const T *)gamma, (const T *)beta, eps, (T *)copy_out,           \
                       (T *)ln_out)
    if (ch <= 2) FVAR_GLN(2);
    else if (ch <= 4) FVAR_GLN(4);
    else if (ch <= 8) FVAR_GLN(8);
    else FVAR_GLN(16);
#undef FVAR_GLN
}

void launch_gather_ln(DType dt, const void *x, const int32_t *idx, int B, int M, int n, int d,
                      const void *gamma, const void *beta, float eps, void *copy_out, void *ln_out,
                      hipStream_t st)
{
    if (dt == DType::BF16)
        launch_gather_ln_t<uint16_t>(x, idx, B, M, n, d, gamma, beta, eps, copy_out, ln_out, st);
    else
        launch_gather_ln_t<float>(x, idx, B, M, n, d, gamma, beta, eps, copy_out, ln_out, st);
}

}  // namespace fvar
