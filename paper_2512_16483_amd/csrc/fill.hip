// Restoration of the full token map (paper, Eq. "redefine"; cached rows in the rank-r restored
// form W_r F_r of Sec. "Random Projection (RP) for Low-Rank Feature" / Eq. "lstsq").
//
//   kept rows    y[b, idx_keep[b,j], :] = y_keep[b,j,:]         one wavefront per row, 16 B/lane
//   pruned rows  y[b, i, :] = w_c[b,i,:] . g_c[b]               thin GEMM, K = r
//
// The pruned part writes (M-k)*d elements per sample and does 2*r flops for each: at r = 64 that
// is 64 flop per written byte in bf16, far above what the vector ALUs can feed at HBM speed, so
// the bf16 path runs it on MFMA with fp32 accumulation and stays bound by the output write.
// A workgroup owns a 128-column slab of g_c[b], transposes it once into LDS (k-contiguous per
// column, which is what the MFMA B operand wants) and streams its share of the pruned rows past
// it; w_c rows go straight from global memory into the A operand.
#include "common.h"

namespace fvar {

// ------------------------------------------------------------------ kept rows: scatter
// Workgroup `blk` of the scatter part: four rows, one per wavefront.
template <typename T>
__device__ __forceinline__ void scatter_rows(int blk, const T *__restrict__ y_keep,
                                             const int32_t *__restrict__ idx_keep, int M, int k,
                                             int total_rows, int d, T *__restrict__ y)
{
    constexpr int E = Elem<T>::kPerChunk;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blk * 4 + wave;
    if (row >= total_rows) return;
    const int b = row / k;
    const int dst_row = idx_keep ? idx_keep[row] : row - b * k;
    const uint4 *src = reinterpret_cast<const uint4 *>(y_keep + (size_t)row * d);
    uint4 *dst = reinterpret_cast<uint4 *>(y + ((size_t)b * M + dst_row) * d);
    const int nchunk = d / E;
    for (int c = lane; c < nchunk; c += 64) dst[c] = src[c];
}

// ------------------------------------------------------------------ pruned rows, bf16 MFMA
constexpr int kFillCols = 128;     // column slab per workgroup
constexpr int kFillRows = 128;     // pruned rows per workgroup iteration (4 waves x 32)
constexpr int kFillPitch = kFillCols + 8;   // row pitch (elements) of the output staging

// One launch does both parts: workgroups [0, fill_blocks) restore pruned rows (slab, row share and
// sample decoded from the block id), the workgroups after them copy kept rows.
__global__ __launch_bounds__(256) void fill_bf16_kernel(const uint16_t *__restrict__ y_keep,
                                                        const int32_t *__restrict__ idx_keep,
                                                        const int32_t *__restrict__ idx_drop, int M,
                                                        int k, int B, int r, int d,
                                                        const uint16_t *__restrict__ w_c,
                                                        const uint16_t *__restrict__ g_c,
                                                        uint16_t *__restrict__ y, int slabs,
                                                        int row_split, int fill_blocks)
{
    if ((int)blockIdx.x >= fill_blocks) {
        scatter_rows<uint16_t>(blockIdx.x - fill_blocks, y_keep, idx_keep, M, k, B * k, d, y);
        return;
    }
    const int nd = M - k;
    const int slab = blockIdx.x % slabs, share = (blockIdx.x / slabs) % row_split;
    const int b = blockIdx.x / (slabs * row_split);
    extern __shared__ uint4 lds_raw[];
    uint16_t *gt = reinterpret_cast<uint16_t *>(lds_raw);     // [kFillCols][pitch]
    const int rp = (r + 15) & ~15;                            // k extent padded to the MFMA step
    const int pitch = rp + 8;                                 // odd number of 16 B chunks per row
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    uint16_t *wl = gt + (size_t)kFillCols * pitch + wave * (32 * kFillPitch);   // output staging
    const int col0 = slab * kFillCols;
    const uint16_t *G = g_c + (size_t)b * r * d;
    const uint16_t *W = w_c + (size_t)b * M * r;
    const int32_t *drop = idx_drop + (size_t)b * nd;
    uint16_t *Y = y + (size_t)b * M * d;

    // ---- stage the slab transposed: 4 (t) x 8 (col) blocks, one 8-byte LDS write per column
    const int tblocks = rp / 4;
    for (int blk = tid; blk < tblocks * (kFillCols / 8); blk += 256) {
        const int cb = blk % (kFillCols / 8), tb = blk / (kFillCols / 8);
        const int c = col0 + cb * 8;
        uint4 rows[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = tb * 4 + j;
            rows[j] = (t < r && c < d) ? *reinterpret_cast<const uint4 *>(G + (size_t)t * d + c)
                                       : make_uint4(0, 0, 0, 0);
        }
        const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&rows[0]);
        const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&rows[1]);
        const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&rows[2]);
        const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&rows[3]);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            // columns 2m (low halves) and 2m+1 (high halves)
            uint2 lo, hi;
            lo.x = __builtin_amdgcn_perm(w1[m], w0[m], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(w3[m], w2[m], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(w1[m], w0[m], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(w3[m], w2[m], 0x07060302u);
            *reinterpret_cast<uint2 *>(gt + (size_t)(cb * 8 + 2 * m) * pitch + tb * 4) = lo;
            *reinterpret_cast<uint2 *>(gt + (size_t)(cb * 8 + 2 * m + 1) * pitch + tb * 4) = hi;
        }
    }
    __syncthreads();

    const int ksteps = rp / 16;
    const int iters = (nd + kFillRows - 1) / kFillRows;
    for (int it = share; it < iters; it += row_split) {
        const int j0 = it * kFillRows + wave * 32;
        if (j0 >= nd) continue;                                // wave-uniform
        // A operand: lane (row rl, half g) holds w_c[row][16s + 8g .. +8)
        const int slot = min(j0 + rl, nd - 1);
        const uint16_t *wrow = W + (size_t)drop[slot] * r;
        uint4 afrag[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int t = 16 * s + 8 * g;
            afrag[s] = (s < ksteps && t < r) ? *reinterpret_cast<const uint4 *>(wrow + t)
                                             : make_uint4(0, 0, 0, 0);
        }
        // The four 32x32 accumulator tiles of this row block are packed to bf16 (adjacent lanes
        // swap one value per row pair so that a lane owns two neighbouring columns) and parked
        // row-major in this wavefront's private LDS region; they leave as 16-byte row chunks, so
        // a store instruction writes whole 256-byte row segments.
        const int odd = lane & 1;
#pragma unroll 1
        for (int cb = 0; cb < kFillCols / 32; ++cb) {
            floatx16_t acc = {0};
            const uint16_t *bsrc = gt + (size_t)(cb * 32 + rl) * pitch + 8 * g;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                if (s < ksteps) {
                    uint4 bv = *reinterpret_cast<const uint4 *>(bsrc + 16 * s);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, afrag[s]), __builtin_bit_cast(bf16x8_t, bv), acc,
                        0, 0, 0);
                }
            }
            const int lcol = cb * 32 + rl - odd;
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float v0 = acc[e], v1 = acc[e + 1];
                const float recv = __shfl_xor(odd ? v0 : v1, 1);
                const int lrow = 8 * (e >> 2) + 4 * g + (e & 3) + odd;
                *reinterpret_cast<uint32_t *>(wl + lrow * kFillPitch + lcol) =
                    odd ? pack_bf16x2(recv, v1) : pack_bf16x2(v0, recv);
            }
        }
        // same wavefront wrote and reads the region: LDS operations of a wavefront stay in order
        const int c = (lane & 15) * 8;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int lrow = it * 4 + (lane >> 4), rr = j0 + lrow;
            const uint4 v = *reinterpret_cast<const uint4 *>(wl + lrow * kFillPitch + c);
            if (rr < nd && col0 + c < d)
                *reinterpret_cast<uint4 *>(Y + (size_t)drop[rr] * d + col0 + c) = v;
        }
    }
}

// ------------------------------------------------------------------ pruned rows, fp32 FMA
__global__ __launch_bounds__(256) void fill_f32_kernel(const float *__restrict__ y_keep,
                                                       const int32_t *__restrict__ idx_keep,
                                                       const int32_t *__restrict__ idx_drop, int M,
                                                       int k, int B, int r, int d,
                                                       const float *__restrict__ w_c,
                                                       const float *__restrict__ g_c,
                                                       float *__restrict__ y, int fill_blocks)
{
    __shared__ float wrow[256];
    if ((int)blockIdx.x >= fill_blocks) {
        scatter_rows<float>(blockIdx.x - fill_blocks, y_keep, idx_keep, M, k, B * k, d, y);
        return;
    }
    const int nd = M - k;
    const int b = blockIdx.x / nd, j = blockIdx.x % nd;
    const int i = idx_drop[(size_t)b * nd + j];
    const float *W = w_c + ((size_t)b * M + i) * r;
    const float *G = g_c + (size_t)b * r * d;
    for (int t = threadIdx.x; t < r; t += 256) wrow[t] = W[t];
    __syncthreads();
    float *out = y + ((size_t)b * M + i) * d;
    for (int c = threadIdx.x * 4; c < d; c += 1024) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int t = 0; t < r; ++t) {
            const float w = wrow[t];
            const float4 gv = *reinterpret_cast<const float4 *>(G + (size_t)t * d + c);
            acc.x = fmaf(w, gv.x, acc.x); acc.y = fmaf(w, gv.y, acc.y);
            acc.z = fmaf(w, gv.z, acc.z); acc.w = fmaf(w, gv.w, acc.w);
        }
        *reinterpret_cast<float4 *>(out + c) = acc;
    }
}

// ------------------------------------------------------------------ raw cached rows
// Eq. "redefine" as printed: kept rows come from the block output, every other row is the cached
// counterpart row itself.  One wavefront per output row: the first B*k rows of the launch scatter
// y_keep, the remaining B*(M-k) copy row idx_drop[b,j] of the cache to the same position of y.
template <typename T>
__global__ __launch_bounds__(256) void cache_fill_kernel(const T *__restrict__ y_keep,
                                                         const int32_t *__restrict__ idx_keep,
                                                         const int32_t *__restrict__ idx_drop, int M,
                                                         int k, int B, int d,
                                                         const T *__restrict__ cache,
                                                         T *__restrict__ y)
{
    constexpr int E = Elem<T>::kPerChunk;
    const int kept_blocks = (B * k + 3) / 4;
    if ((int)blockIdx.x < kept_blocks) {
        scatter_rows<T>(blockIdx.x, y_keep, idx_keep, M, k, B * k, d, y);
        return;
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nd = M - k;
    const int j = (blockIdx.x - kept_blocks) * 4 + wave;
    if (j >= B * nd) return;                       // also covers nd == 0
    const int b = j / nd;
    const size_t row = (size_t)b * M + idx_drop[j];
    const uint4 *src = reinterpret_cast<const uint4 *>(cache + row * d);
    uint4 *dst = reinterpret_cast<uint4 *>(y + row * d);
    const int nchunk = d / E;
    for (int c = lane; c < nchunk; c += 64) dst[c] = src[c];
}

void launch_cache_fill(DType dt, const void *y_keep, const int32_t *idx_keep, const int32_t *idx_drop,
                       int B, int M, int k, int d, const void *cache, void *y, hipStream_t st)
{
    // cache == y: the pruned rows are in place already and only the kept rows are written
    const int copy_rows = cache == y ? 0 : B * (M - k);
    const int blocks = (B * k + 3) / 4 + (copy_rows + 3) / 4;
    if (blocks == 0) return;
    if (dt == DType::BF16)
        launch(cache_fill_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (const uint16_t *)y_keep,
               idx_keep, idx_drop, M, k, B, d, (const uint16_t *)cache, (uint16_t *)y);
    else
        launch(cache_fill_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float *)y_keep, idx_keep,
               idx_drop, M, k, B, d, (const float *)cache, (float *)y);
}

void launch_fill(DType dt, const void *y_keep, const int32_t *idx_keep, const int32_t *idx_drop,
                 int B, int M, int k, int r, int d, const void *w_c, const void *g_c, void *y,
                 hipStream_t st)
{
    const int nd = M - k;
    const int scatter_blocks = (B * k + 3) / 4;
    if (dt == DType::BF16) {
        const int slabs = (d + kFillCols - 1) / kFillCols;
        const int iters = (nd + kFillRows - 1) / kFillRows;
        // enough workgroups to cover the chip a few times, but keep the slab staging amortised
        int row_split = nd > 0 ? (1024 + slabs * B - 1) / (slabs * B) : 0;
        if (row_split > iters) row_split = iters;
        const int fill_blocks = slabs * row_split * B;
        const int rp = (r + 15) & ~15;
        const size_t lds = nd > 0 ? ((size_t)kFillCols * (rp + 8) + 4 * 32 * kFillPitch) * sizeof(uint16_t) : 0;
        if (lds > 48 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(fill_bf16_kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (fill_blocks + scatter_blocks == 0) return;
        launch(fill_bf16_kernel, dim3(fill_blocks + scatter_blocks), dim3(256), lds, st,
               (const uint16_t *)y_keep, idx_keep, idx_drop, M, k, B, r, d, (const uint16_t *)w_c,
               (const uint16_t *)g_c, (uint16_t *)y, slabs, row_split, fill_blocks);
    } else {
        const int fill_blocks = nd * B;
        if (fill_blocks + scatter_blocks == 0) return;
        launch(fill_f32_kernel, dim3(fill_blocks + scatter_blocks), dim3(256), 0, st,
               (const float *)y_keep, idx_keep, idx_drop, M, k, B, r, d, (const float *)w_c,
               (const float *)g_c, (float *)y, fill_blocks);
    }
}

}  // namespace fvar
