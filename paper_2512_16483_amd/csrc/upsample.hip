// Up-sampling of a cached token map to the grid of the next scale (paper, Eq. "upcache").
// Bilinear, half-pixel centres, edges clamped; acts on the token axis only, so the rank-r form
// W G of the cache is up-sampled through its thin factor W ([M,r] instead of [M,d]).
// One thread per (destination token, 16-byte channel chunk); tap indices in integer arithmetic:
// the source coordinate of destination centre y is ((2y+1) n_src - n_dst) / (2 n_dst).
#include "common.h"

namespace fvar {

struct AxisTap { int i0, i1; float w1; };

__device__ __forceinline__ AxisTap axis_tap(int y, int n_src, int n_dst)
{
    long num = (long)(2 * y + 1) * n_src - n_dst;          // source coordinate * 2 n_dst
    if (num < 0) num = 0;
    const long den = 2L * n_dst;
    int i0 = (int)(num / den);
    if (i0 > n_src - 1) i0 = n_src - 1;
    AxisTap t;
    t.i0 = i0;
    t.i1 = min(i0 + 1, n_src - 1);
    t.w1 = (float)(num - (long)i0 * den) / (float)den;
    return t;
}

template <typename T>
__global__ __launch_bounds__(256) void upsample_kernel(const T *__restrict__ src, int hs, int ws,
                                                       int hd, int wd, int c, long total_chunks,
                                                       T *__restrict__ dst)
{
    constexpr int E = Elem<T>::kPerChunk;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total_chunks) return;
    const int cpr = c / E;                                  // chunks per token row
    const int ch = (int)(idx % cpr);
    const long tok = idx / cpr;                             // b * hd*wd + y * wd + x
    const int x = (int)(tok % wd), y = (int)((tok / wd) % hd);
    const long b = tok / ((long)wd * hd);
    const AxisTap ty = axis_tap(y, hs, hd), tx = axis_tap(x, ws, wd);
    const uint4 *S = reinterpret_cast<const uint4 *>(src + (size_t)b * hs * ws * c) + ch;
    float v00[E], v01[E], v10[E], v11[E], o[E];
    Elem<T>::unpack(S[(size_t)(ty.i0 * ws + tx.i0) * cpr], v00);
    Elem<T>::unpack(S[(size_t)(ty.i0 * ws + tx.i1) * cpr], v01);
    Elem<T>::unpack(S[(size_t)(ty.i1 * ws + tx.i0) * cpr], v10);
    Elem<T>::unpack(S[(size_t)(ty.i1 * ws + tx.i1) * cpr], v11);
    const float wx = tx.w1, wy = ty.w1;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const float top = (1.f - wx) * v00[e] + wx * v01[e];
        const float bot = (1.f - wx) * v10[e] + wx * v11[e];
        o[e] = (1.f - wy) * top + wy * bot;
    }
    reinterpret_cast<uint4 *>(dst)[idx] = Elem<T>::pack(o);
}

void launch_upsample(DType dt, const void *src, int B, int hs, int ws, int hd, int wd, int c,
                     void *dst, hipStream_t st)
{
    const int E = dt == DType::BF16 ? 8 : 4;
    const long total = (long)B * hd * wd * (c / E);
    dim3 grid((unsigned)((total + 255) / 256));
    if (dt == DType::BF16)
        launch(upsample_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)src, hs, ws, hd, wd,
               c, total, (uint16_t *)dst);
    else
        launch(upsample_kernel<float>, grid, dim3(256), 0, st, (const float *)src, hs, ws, hd, wd, c,
               total, (float *)dst);
}

}  // namespace fvar
