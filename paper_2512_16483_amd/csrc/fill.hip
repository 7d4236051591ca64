// Restoration of the full token map (paper, Eq. "redefine"; cached rows in the rank-r restored
// form W_r F_r of Sec. "Random Projection (RP) for Low-Rank Feature" / Eq. "lstsq").
//
//   kept rows    y[b, idx_keep[b,j], :] = y_keep[b,j,:]         one wavefront per row, 16 B/lane
//   pruned rows  y[b, i, :] = w_c[b,i,:] . g_c[b]               thin GEMM, K = r
//
// The pruned part writes (M-k)*d elements per sample and does 2*r flops for each: at r = 64 that
// is 64 flop per written byte in bf16, far above what the vector ALUs can feed at HBM speed, so
// the bf16 path runs it on MFMA with fp32 accumulation and stays bound by the output write.
// A workgroup owns a 128-column slab of g_c[b]: the slab travels global -> LDS by DMA once, in
// its own row-major layout, and the workgroup streams its share of the pruned rows past it.
// The product is formed transposed (slab columns are the MFMA rows, token rows the MFMA columns)
// so that a lane ends up with 4 consecutive output columns of one token row: the slab operand,
// which the MFMA wants k-contiguous, is fetched with the transposing LDS load
// (ds_read_b64_tr_b16), the w_c rows go straight from global memory into the other operand, one
// row group ahead of the MFMAs that use them.
//
// Optionally every workgroup also leaves, per output row, the sum of squares of the values it
// stored (exact products of the stored elements, fp64 sum): the row energies of the map, i.e. the
// selection scores of the NEXT block (paper, Sec. "Representative Token Restoration"), so that
// the next block does not have to read the map again.
#include "common.h"

namespace fvar {

// sum over the `width` (power of two, <= 64) consecutive lanes of a group
__device__ __forceinline__ double group_sum(double v, int width)
{
    for (int o = width >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// sum of squares of the 8 bf16 (4 fp32) elements of a 16-byte chunk, in fp64
template <typename T> __device__ __forceinline__ double chunk_energy(const uint4 &c)
{
    float f[Elem<T>::kPerChunk];
    Elem<T>::unpack(c, f);
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < Elem<T>::kPerChunk; ++e) acc = fma((double)f[e], (double)f[e], acc);
    return acc;
}

// ------------------------------------------------------------------ kept rows: scatter
// Workgroup `blk` of the scatter part: four rows, one per wavefront.  With `parts` the row's
// energy goes to part 0 of the row and zeros to its other parts.
template <typename T>
__device__ __forceinline__ void scatter_rows(int blk, const T *__restrict__ y_keep,
                                             const int32_t *__restrict__ idx_keep, int M, int k,
                                             int total_rows, int d, T *__restrict__ y,
                                             double *__restrict__ parts, int nparts)
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
    double e = 0.0;
    for (int c = lane; c < nchunk; c += 64) {
        const uint4 v = src[c];
        dst[c] = v;
        if (parts) e += chunk_energy<T>(v);
    }
    if (parts) {
        e = group_sum(e, 64);
        double *pr = parts + ((size_t)b * M + dst_row) * nparts;
        if (lane < nparts) pr[lane] = lane == 0 ? e : 0.0;
    }
}

// ------------------------------------------------------------------ pruned rows, bf16 MFMA
constexpr int kFillCols = 128;              // column slab per workgroup (16 chunks of 16 B per row)
constexpr int kFillStage = 64 + 8;          // row pitch (elements) of the per-wavefront output staging

typedef short fill_shortx4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void fill_dma_b128(const void *base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}

// One launch does both parts: workgroups [0, fill_blocks) restore pruned rows (slab, row share and
// sample decoded from the block id), the workgroups after them copy kept rows.
// KSTEPS = ceil(r / 16): 16-wide steps of the contraction.
template <int KSTEPS>
__global__ __launch_bounds__(256) void fill_bf16_kernel(const uint16_t *__restrict__ y_keep,
                                                        const int32_t *__restrict__ idx_keep,
                                                        const int32_t *__restrict__ idx_drop, int M,
                                                        int k, int B, int r, int d,
                                                        const uint16_t *__restrict__ w_c,
                                                        const uint16_t *__restrict__ g_c,
                                                        uint16_t *__restrict__ y, int slabs,
                                                        int row_split, int fill_blocks,
                                                        double *__restrict__ parts)
{
    if ((int)blockIdx.x >= fill_blocks) {
        scatter_rows<uint16_t>(blockIdx.x - fill_blocks, y_keep, idx_keep, M, k, B * k, d, y, parts, slabs);
        return;
    }
    constexpr int RP = KSTEPS * 16;                           // slab rows in LDS (k extent, padded)
    const int nd = M - k;
    const int slab = blockIdx.x % slabs, share = (blockIdx.x / slabs) % row_split;
    const int b = blockIdx.x / (slabs * row_split);
    extern __shared__ uint4 lds_raw[];
    uint16_t *gs = reinterpret_cast<uint16_t *>(lds_raw);     // [RP][kFillCols], chunks swizzled
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds_raw;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rl = lane & 31, g = lane >> 5;
    uint16_t *wl = gs + RP * kFillCols + wave * (32 * kFillStage);   // output staging of this wavefront
    const int col0 = slab * kFillCols;
    const uint16_t *G = g_c + (size_t)b * r * d;
    const uint16_t *W = w_c + (size_t)b * M * r;
    const int32_t *drop = idx_drop + (size_t)b * nd;
    uint16_t *Y = y + (size_t)b * M * d;

    // ---- the slab: rows t of g_c[b], columns col0 .. col0+127, 4 rows (1 KiB) per DMA instruction.
    // Lane l fills physical chunk l%16 of row 4*group + l/16 with the logical chunk that the
    // swizzle (chunk ^ 4*(row%4)) maps there.  Rows past r repeat row r-1 (their products meet
    // zeros of the other operand), columns past d repeat the last chunk (never stored).
    for (int grp = wave; grp < RP / 4; grp += 4) {
        const int t = min(grp * 4 + lane / 16, r - 1);
        const int lc = (lane % 16) ^ ((t & 3) << 2);
        const int col = min(col0 + lc * 8, d - 8);
        fill_dma_b128(G, (uint32_t)(((size_t)t * d + col) * 2), lds_base + grp * 1024);
    }

    // ---- operand addressing
    // transposing read of the slab: lane l = 16*Gq + 4*j + a points at slab row 8*(Gq/2) + j (+ 16s,
    // + 4 for the second read) and columns 16*(Gq%2) + 4*a .. +3 (+ 32*cb); it receives, for
    // MFMA row (slab column) 16*(Gq%2) + l%16 of block cb, the k-slots 8*(Gq/2) + 0..3 (+4)
    const int tG = lane >> 4, tj = (lane >> 2) & 3, ta = lane & 3;
    const int g_lane = (8 * (tG >> 1) + tj) * kFillCols + ((2 * (tG & 1) + (ta >> 1)) << 3) + (ta & 1) * 4;
    // rows of this workgroup: 32-row groups it, it + row_split*4 ... per wavefront
    const int groups = (nd + 31) / 32;
    const int gstep = row_split * 4;
    int grp_row = share * 4 + wave;                             // this wavefront's current group

    // other operand: lane (row rl, half g) holds w_c[row][16s + 8g .. +8)
    // The token row of a slot comes from idx_drop: that index is fetched two groups ahead of the
    // MFMAs (one group ahead of the w_c fragments it addresses), so neither the fragment loads nor
    // the stores wait for an index at the moment they are issued.
    uint4 afrag[2][KSTEPS];
    auto load_row = [&](int grpi) { return drop[min(grpi * 32 + rl, nd - 1)]; };
    auto load_a = [&](int row, uint4 *dst) {
        const uint16_t *wrow = W + (size_t)row * r;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const int t = 16 * s + 8 * g;
            dst[s] = t < r ? *reinterpret_cast<const uint4 *>(wrow + t) : make_uint4(0, 0, 0, 0);
        }
    };
    int row_next = 0;                                          // token row of this lane in the next group
    if (grp_row < groups) load_a(load_row(grp_row), afrag[0]);
    if (grp_row + gstep < groups) row_next = load_row(grp_row + gstep);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // one 32-row group: af holds its w_c fragments, af_next receives those of the next group
    auto group = [&](int grp_row, const uint4 *af, uint4 *af_next) {
        const int j0 = grp_row * 32;
        // destination rows of the 4 row-chunks this lane stores per half (rows it*8 + lane/8)
        int orow[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) orow[it] = drop[min(j0 + it * 8 + (lane >> 3), nd - 1)];
        if (grp_row + gstep < groups) load_a(row_next, af_next);
        if (grp_row + 2 * gstep < groups) row_next = load_row(grp_row + 2 * gstep);
        double erow[4] = {0.0, 0.0, 0.0, 0.0};
        // two halves of 64 columns: 2 x 32-column accumulator tiles each
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            floatx16_t acc[2] = {floatx16_t{0}, floatx16_t{0}};
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    typedef __attribute__((address_space(3))) fill_shortx4_t lds_shortx4_t;
                    const int cb = half * 2 + c2;
                    const uint16_t *src = gs + g_lane + 16 * s * kFillCols + ((cb ^ tj) << 5);
                    const fill_shortx4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t *)src);
                    const fill_shortx4_t hi =
                        __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t *)(src + 4 * kFillCols));
                    const bf16x8_t gf = __builtin_bit_cast(
                        bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    acc[c2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        gf, __builtin_bit_cast(bf16x8_t, af[s]), acc[c2], 0, 0, 0);
                }
            }
            // accumulator entry e of tile c2: token row rl, slab column 32*cb + 8*(e/4) + 4*g + e%4.
            // Pack 4 consecutive columns and park them row-major in this wavefront's staging tile.
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 pk;
                    pk.x = pack_bf16x2(acc[c2][4 * q], acc[c2][4 * q + 1]);
                    pk.y = pack_bf16x2(acc[c2][4 * q + 2], acc[c2][4 * q + 3]);
                    *reinterpret_cast<uint2 *>(wl + rl * kFillStage + c2 * 32 + 8 * q + 4 * g) = pk;
                }
            // same wavefront wrote and reads the region: LDS operations of a wavefront stay in order
            // in hardware; the compiler is told not to move them across these points (the stores
            // and loads use different vector types).
            // 8 lanes cover the 128 bytes of one row half: 8 rows per store instruction.
            asm volatile("" ::: "memory");
            const int c = (lane & 7) * 8;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int lrow = it * 8 + (lane >> 3), rr = j0 + lrow;
                const uint4 v = *reinterpret_cast<const uint4 *>(wl + lrow * kFillStage + c);
                const int col = col0 + half * 64 + c;
                const bool ok = rr < nd && col < d;
                if (ok) *reinterpret_cast<uint4 *>(Y + (size_t)orow[it] * d + col) = v;
                if (parts && ok) erow[it] += chunk_energy<uint16_t>(v);
            }
            asm volatile("" ::: "memory");
        }
        // the 8 lanes of a group hold the pieces of one row; the lane at their head owns rows
        // it*8 + lane/8 of the group
        double e8[4];
        if (parts) {
#pragma unroll
            for (int it = 0; it < 4; ++it) e8[it] = group_sum(erow[it], 8);
        }
        if (parts && (lane & 7) == 0) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int rr = j0 + it * 8 + (lane >> 3);
                if (rr < nd) parts[((size_t)b * M + orow[it]) * slabs + slab] = e8[it];
            }
        }
    };
    for (; grp_row < groups; grp_row += 2 * gstep) {
        group(grp_row, afrag[0], afrag[1]);
        if (grp_row + gstep < groups) group(grp_row + gstep, afrag[1], afrag[0]);
    }
}

// ------------------------------------------------------------------ pruned rows, fp32 FMA
__global__ __launch_bounds__(256) void fill_f32_kernel(const float *__restrict__ y_keep,
                                                       const int32_t *__restrict__ idx_keep,
                                                       const int32_t *__restrict__ idx_drop, int M,
                                                       int k, int B, int r, int d,
                                                       const float *__restrict__ w_c,
                                                       const float *__restrict__ g_c,
                                                       float *__restrict__ y, int fill_blocks,
                                                       double *__restrict__ parts)
{
    __shared__ float wrow[256];
    __shared__ double esum[4];
    if ((int)blockIdx.x >= fill_blocks) {
        scatter_rows<float>(blockIdx.x - fill_blocks, y_keep, idx_keep, M, k, B * k, d, y, parts, 1);
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
    double e = 0.0;
    for (int c = threadIdx.x * 4; c < d; c += 1024) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int t = 0; t < r; ++t) {
            const float w = wrow[t];
            const float4 gv = *reinterpret_cast<const float4 *>(G + (size_t)t * d + c);
            acc.x = fmaf(w, gv.x, acc.x); acc.y = fmaf(w, gv.y, acc.y);
            acc.z = fmaf(w, gv.z, acc.z); acc.w = fmaf(w, gv.w, acc.w);
        }
        *reinterpret_cast<float4 *>(out + c) = acc;
        e = fma((double)acc.x, (double)acc.x, e); e = fma((double)acc.y, (double)acc.y, e);
        e = fma((double)acc.z, (double)acc.z, e); e = fma((double)acc.w, (double)acc.w, e);
    }
    if (parts) {                                            // uniform
        e = group_sum(e, 64);
        if ((threadIdx.x & 63) == 0) esum[threadIdx.x >> 6] = e;
        __syncthreads();
        if (threadIdx.x == 0) parts[(size_t)b * M + i] = (esum[0] + esum[1]) + (esum[2] + esum[3]);
    }
}

// Row energies of the restored map from the per-slab parts: scores[row] = fl32(sum of the row's
// parts in slab order), one thread per row.
__global__ __launch_bounds__(256) void scores_from_parts_kernel(const double *__restrict__ parts,
                                                                int nparts, long rows,
                                                                float *__restrict__ scores)
{
    const long row = (long)blockIdx.x * 256 + threadIdx.x;
    if (row >= rows) return;
    const double *p = parts + (size_t)row * nparts;
    double acc = 0.0;
    for (int i = 0; i < nparts; ++i) acc += p[i];
    scores[row] = (float)acc;
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
        scatter_rows<T>(blockIdx.x, y_keep, idx_keep, M, k, B * k, d, y, nullptr, 0);
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

// parts per output row that launch_fill leaves when row energies are requested
int fill_score_parts(DType dt, int d)
{
    return dt == DType::BF16 ? (d + kFillCols - 1) / kFillCols : 1;
}

template <int KSTEPS>
static void launch_fill_bf16(const void *y_keep, const int32_t *idx_keep, const int32_t *idx_drop, int B,
                             int M, int k, int r, int d, const void *w_c, const void *g_c, void *y,
                             double *parts, hipStream_t st)
{
    const int nd = M - k;
    const int scatter_blocks = (B * k + 3) / 4;
    const int slabs = (d + kFillCols - 1) / kFillCols;
    const int groups = (nd + 31) / 32;                      // 32-row groups, one wavefront each
    // enough workgroups to cover the chip a few times while the slab staging stays amortised
    int row_split = nd > 0 ? (1536 + slabs * B - 1) / (slabs * B) : 0;
    const int max_split = (groups + 3) / 4;
    if (row_split > max_split) row_split = max_split;
    const int fill_blocks = slabs * row_split * B;
    const size_t lds = nd > 0 ? ((size_t)KSTEPS * 16 * kFillCols + 4 * 32 * kFillStage) * sizeof(uint16_t) : 0;
    auto kern = fill_bf16_kernel<KSTEPS>;
    if (lds > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (fill_blocks + scatter_blocks == 0) return;
    launch(kern, dim3(fill_blocks + scatter_blocks), dim3(256), lds, st, (const uint16_t *)y_keep, idx_keep,
           idx_drop, M, k, B, r, d, (const uint16_t *)w_c, (const uint16_t *)g_c, (uint16_t *)y, slabs,
           row_split, fill_blocks, parts);
}

// parts: null, or B*M*fill_score_parts() doubles that receive the energy of every output row in
// parts; scores_out (with parts): [B*M] fp32 row energies, summed from the parts by a second kernel
void launch_fill(DType dt, const void *y_keep, const int32_t *idx_keep, const int32_t *idx_drop,
                 int B, int M, int k, int r, int d, const void *w_c, const void *g_c, void *y,
                 double *parts, float *scores_out, hipStream_t st)
{
    const int nd = M - k;
    const int scatter_blocks = (B * k + 3) / 4;
    if (dt == DType::BF16) {
        const int ks = nd > 0 ? (r + 15) / 16 : 1;
#define FVAR_FILL(KS) launch_fill_bf16<KS>(y_keep, idx_keep, idx_drop, B, M, k, r, d, w_c, g_c, y, parts, st)
        if (ks <= 1) FVAR_FILL(1);
        else if (ks <= 2) FVAR_FILL(2);
        else if (ks <= 3) FVAR_FILL(3);
        else if (ks <= 4) FVAR_FILL(4);
        else if (ks <= 6) FVAR_FILL(6);
        else if (ks <= 8) FVAR_FILL(8);
        else if (ks <= 12) FVAR_FILL(12);
        else FVAR_FILL(16);
#undef FVAR_FILL
    } else {
        const int fill_blocks = nd * B;
        if (fill_blocks + scatter_blocks > 0)
            launch(fill_f32_kernel, dim3(fill_blocks + scatter_blocks), dim3(256), 0, st,
                   (const float *)y_keep, idx_keep, idx_drop, M, k, B, r, d, (const float *)w_c,
                   (const float *)g_c, (float *)y, fill_blocks, parts);
    }
    if (parts && scores_out) {
        const long rows = (long)B * M;
        launch(scores_from_parts_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st,
               (const double *)parts, fill_score_parts(dt, d), rows, scores_out);
    }
}

}  // namespace fvar
