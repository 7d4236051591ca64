// Linear layers of the block phi on the rows that pass through it (QKV, output projection,
// MLP): C = epilogue(A[rows,K] * W[N,K]^T).  Both operands are K-contiguous ("out,in" weights),
// which is the layout the MFMA operands want: a lane holds 8 consecutive k of one row.
//
// bf16: 256 threads = 4 wavefronts, workgroup tile BM x BN x 64, v_mfma_f32_32x32x16_bf16 with
// fp32 accumulation.  Tiles are staged global -> registers -> LDS with the next tile's global
// loads in flight during the current tile's MFMAs (double-buffered LDS, one barrier per k-tile).
// LDS rows are 128 B; the 16-byte chunk index is XOR-swizzled with (row/2)%8 so that the
// ds_read_b128 operand fetches of 16 consecutive rows cover all 64 banks exactly once.
// Workgroup ids are remapped so that each XCD (own L2) works on a compact patch of the tile grid.
//
// fp32: plain LDS-tiled FMA kernel, used only by the fp32 parity configuration.
#include <type_traits>

#include "common.h"

namespace fvar {

struct EpiParams {
    const void *bias;
    const void *residual;
    int gelu;
    void *out0;
    int ld0;
    int split;
    void *kcache, *vcache;
    int hd, cap, len, rows_per_sample;
    int N;
};

__device__ __forceinline__ float gelu_tanh(float v)
{
    // 0.5 v (1 + tanh(u)) = v / (1 + exp(-2u)),  u = sqrt(2/pi) (v + 0.044715 v^3)
    const float u = 0.7978845608028654f * (v + 0.044715f * v * v * v);
    return v / (1.0f + __expf(-2.0f * u));
}

// destination of element (row, col) in elements from the base pointer it returns
template <typename T>
__device__ __forceinline__ T *epi_dst(const EpiParams &ep, int row, int col)
{
    if (col < ep.split) return (T *)ep.out0 + (size_t)row * ep.ld0 + col;
    const int b = row / ep.rows_per_sample, j = row - b * ep.rows_per_sample;
    const size_t crow = (size_t)b * ep.cap + ep.len + j;
    int c = col - ep.split;
    if (c < ep.hd) return (T *)ep.kcache + crow * ep.hd + c;
    return (T *)ep.vcache + crow * ep.hd + (c - ep.hd);
}

// ------------------------------------------------------------------------------ bf16 MFMA
constexpr int BK = 64;

__device__ __forceinline__ int lds_off(int row, int chunk)      // in bf16 elements
{
    return row * BK + ((chunk ^ ((row >> 1) & 7)) << 3);
}

typedef int intx4_t __attribute__((ext_vector_type(4)));

// 16-byte global load whose position in the instruction stream is fixed.  The result must not be
// read before an explicit s_waitcnt vmcnt (the compiler does not count this load).
__device__ __forceinline__ intx4_t global_load_b128(const void *base, uint32_t byte_off)
{
    intx4_t v;
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(v) : "v"(byte_off), "s"(base) : "memory");
    return v;
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(const uint16_t *__restrict__ A,
                                                        const uint16_t *__restrict__ W, int rows,
                                                        int N, int K, int tiles_m, int tiles_n,
                                                        EpiParams ep)
{
    static_assert(WM * WN == 4, "four wavefronts");
    constexpr int TM = BM / WM, TN = BN / WN;       // wavefront tile
    constexpr int FM = TM / 32, FN = TN / 32;       // 32x32 MFMA tiles per wavefront
    constexpr int LA = BM * 8 / 256, LB = BN * 8 / 256;   // 16 B chunks per thread per tile
    extern __shared__ uint4 lds_raw[];
    uint16_t *lds = reinterpret_cast<uint16_t *>(lds_raw);
    // layout: [stage][A tile | B tile]
    constexpr int STAGE = (BM + BN) * BK;

    // ---- workgroup -> tile: XCD-contiguous ranges, then grouped rows
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = (gridDim.x + 7) / 8;
    int pid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (pid >= ntiles) return;
    constexpr int GROUP_M = 8;
    const int group = pid / (GROUP_M * tiles_n);
    const int first_m = group * GROUP_M;
    const int gsize = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % (GROUP_M * tiles_n)) % gsize;
    const int tn = (pid % (GROUP_M * tiles_n)) / gsize;
    const int row0 = tm * BM, col0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;

    // ---- global load assignment (rows beyond the matrix are clamped; their results are masked)
    // byte offsets from the (uniform) matrix base: one VGPR per load instead of a 64-bit pointer
    uint32_t a_src[LA], b_src[LB];
    int a_dst[LA], b_dst[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int id = tid + 256 * i, r = id >> 3, c = id & 7;
        a_src[i] = (uint32_t)(((size_t)min(row0 + r, rows - 1) * K + c * 8) * sizeof(uint16_t));
        a_dst[i] = lds_off(r, c);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int id = tid + 256 * i, r = id >> 3, c = id & 7;
        b_src[i] = (uint32_t)(((size_t)min(col0 + r, N - 1) * K + c * 8) * sizeof(uint16_t));
        b_dst[i] = BM * BK + lds_off(r, c);
    }

    floatx16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = floatx16_t{0};

    auto load_frags = [&](const uint16_t *tile, int kk, bf16x8_t *a, bf16x8_t *b) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int r = wm * TM + i * 32 + rl;
            a[i] = *reinterpret_cast<const bf16x8_t *>(tile + lds_off(r, kk * 2 + g));
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int r = wn * TN + j * 32 + rl;
            b[j] = *reinterpret_cast<const bf16x8_t *>(tile + BM * BK + lds_off(r, kk * 2 + g));
        }
    };

    // Pipeline: while k-tile kt is multiplied out of LDS stage kt%2, tile kt+1 travels global ->
    // registers -> the other stage.  The loads are issued through asm so that they stay at the
    // top of the iteration (the compiler would sink them next to the LDS stores otherwise); the
    // staging registers are written by the asm and read after the explicit vmcnt wait inside the
    // same straight-line block, so no in-flight register ever crosses a branch.  The last
    // iteration re-reads its own tile (the copy is never consumed).
    const int ktiles = K / BK;
    intx4_t ra[LA], rb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i)
        ra[i] = *reinterpret_cast<const intx4_t *>(reinterpret_cast<const char *>(A) + a_src[i]);
#pragma unroll
    for (int i = 0; i < LB; ++i)
        rb[i] = *reinterpret_cast<const intx4_t *>(reinterpret_cast<const char *>(W) + b_src[i]);
#pragma unroll
    for (int i = 0; i < LA; ++i) *reinterpret_cast<intx4_t *>(lds + a_dst[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < LB; ++i) *reinterpret_cast<intx4_t *>(lds + b_dst[i]) = rb[i];
    __syncthreads();

    for (int kt = 0; kt < ktiles; ++kt) {
        const uint16_t *cur = lds + (kt & 1) * STAGE;
        uint16_t *nxt = lds + ((kt + 1) & 1) * STAGE;
        const int koff = min(kt + 1, ktiles - 1) * BK;
#pragma unroll
        for (int i = 0; i < LA; ++i) ra[i] = global_load_b128(A + koff, a_src[i]);
#pragma unroll
        for (int i = 0; i < LB; ++i) rb[i] = global_load_b128(W + koff, b_src[i]);
        __builtin_amdgcn_sched_barrier(0);
        // operand fragments run one 16-wide k-step ahead of the MFMAs that consume them
        bf16x8_t af[2][FM], bfr[2][FN];
        load_frags(cur, 0, af[0], bfr[0]);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            if (kk + 1 < BK / 16) load_frags(cur, kk + 1, af[(kk + 1) & 1], bfr[(kk + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j],
                                                                        acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the asm loads above have landed
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<intx4_t *>(nxt + a_dst[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<intx4_t *>(nxt + b_dst[i]) = rb[i];
        __syncthreads();
    }

    // ---- epilogue.  Accumulator entry i of a 32x32 tile: row 8*(i/4) + 4*g + i%4, column rl.
    // Adjacent lanes swap one value per row pair so that every lane stores two neighbouring
    // columns of one row as a single dword.
    const uint16_t *bias = reinterpret_cast<const uint16_t *>(ep.bias);
    const uint16_t *res = reinterpret_cast<const uint16_t *>(ep.residual);
    const int odd = lane & 1;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int col = col0 + wn * TN + j * 32 + rl;
        const bool col_ok = col < N;
        const float bv = (bias && col_ok) ? bf16_to_f32(bias[col]) : 0.f;
        const int pcol = col - odd;                          // even column of the stored pair
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                float v0 = acc[i][j][e] + bv, v1 = acc[i][j][e + 1] + bv;
                if (ep.gelu) { v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); }
                const float send = odd ? v0 : v1;
                const float recv = __shfl_xor(send, 1);
                const int rbase = row0 + wm * TM + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                const int row = rbase + odd;
                float lo = odd ? recv : v0, hi = odd ? v1 : recv;
                if (row < rows && col_ok) {
                    if (res) {
                        const uint32_t rv =
                            *reinterpret_cast<const uint32_t *>(res + (size_t)row * N + pcol);
                        lo += bf16_lo(rv);
                        hi += bf16_hi(rv);
                    }
                    *reinterpret_cast<uint32_t *>(epi_dst<uint16_t>(ep, row, pcol)) =
                        pack_bf16x2(lo, hi);
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN>
static void launch_gemm_bf16_cfg(const void *A, const void *W, int rows, int N, int K,
                                 const EpiParams &ep, hipStream_t st)
{
    const int tiles_m = (rows + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int ntiles = tiles_m * tiles_n;
    const int grid = (ntiles + 7) / 8 * 8;
    const size_t lds = (size_t)2 * (BM + BN) * BK * sizeof(uint16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN>;
    static bool attr_set = false;
    if (!attr_set && lds > 48 * 1024) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, (const uint16_t *)A,
                       (const uint16_t *)W, rows, N, K, tiles_m, tiles_n, ep);
}

// ------------------------------------------------------------------------------ fp32 FMA
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A,
                                                       const float *__restrict__ W, int rows, int N,
                                                       int K, EpiParams ep)
{
    constexpr int T = 64, KB = 16;
    __shared__ float As[KB][T + 4];
    __shared__ float Bs[KB][T + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int row0 = blockIdx.y * T, col0 = blockIdx.x * T;
    // each thread loads one float4 of A and one of W per k-tile: row = tid/4, k = (tid%4)*4
    const int lr = tid >> 2, lk = (tid & 3) * 4;
    const float *a_src = A + (size_t)min(row0 + lr, rows - 1) * K + lk;
    const float *b_src = W + (size_t)min(col0 + lr, N - 1) * K + lk;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += KB) {
        const float4 av = *reinterpret_cast<const float4 *>(a_src + k0);
        const float4 bv = *reinterpret_cast<const float4 *>(b_src + k0);
        As[lk + 0][lr] = av.x; As[lk + 1][lr] = av.y; As[lk + 2][lr] = av.z; As[lk + 3][lr] = av.w;
        Bs[lk + 0][lr] = bv.x; Bs[lk + 1][lr] = bv.y; Bs[lk + 2][lr] = bv.z; Bs[lk + 3][lr] = bv.w;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KB; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    const float *bias = reinterpret_cast<const float *>(ep.bias);
    const float *res = reinterpret_cast<const float *>(ep.residual);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = row0 + ty * 4 + i;
        if (row >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = col0 + tx * 4 + j;
            if (col >= N) continue;
            float v = acc[i][j] + (bias ? bias[col] : 0.f);
            if (ep.gelu) {
                const float u = 0.7978845608028654f * (v + 0.044715f * v * v * v);
                v = 0.5f * v * (1.0f + tanhf(u));
            }
            if (res) v += res[(size_t)row * N + col];
            *epi_dst<float>(ep, row, col) = v;
        }
    }
}

void launch_gemm(DType dt, const void *A, const void *W, int rows, int N, int K,
                 const GemmEpilogue &e, hipStream_t st)
{
    EpiParams ep;
    ep.bias = e.bias; ep.residual = e.residual; ep.gelu = e.gelu;
    ep.out0 = e.out0; ep.ld0 = e.ld0; ep.split = e.split;
    ep.kcache = e.kcache; ep.vcache = e.vcache;
    ep.hd = e.hd; ep.cap = e.cap; ep.len = e.len;
    ep.rows_per_sample = e.rows_per_sample > 0 ? e.rows_per_sample : 1;
    ep.N = N;
    if (dt == DType::BF16) {
        launch_gemm_bf16_cfg<128, 128, 2, 2>(A, W, rows, N, K, ep, st);
    } else {
        dim3 grid((N + 63) / 64, (rows + 63) / 64), block(256);
        hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, st, (const float *)A, (const float *)W,
                           rows, N, K, ep);
    }
}

}  // namespace fvar
