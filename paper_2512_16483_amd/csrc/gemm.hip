// Linear layers of the block phi on the rows that pass through it (QKV, output projection,
// MLP): C = epilogue(A[rows,K] * W[N,K]^T).  Both operands are K-contiguous ("out,in" weights),
// which is the layout the MFMA operands want: a lane holds 8 consecutive k of one row.
//
// bf16: workgroup tile BM x BN x 64 computed by WM x WN wavefronts with v_mfma_f32_16x16x32_bf16
// (fp32 accumulation; on operands with realistic bit activity the chip sustains a higher clock
// on this shape than on 32x32x16: half the accumulator register traffic per flop).  Tiles are
// DMA-ed global -> LDS (no register staging) into a ring of stages ahead of the MFMAs; operand
// fragments are read from LDS a few MFMA groups ahead of their use.  LDS rows are 128 B; the
// 16-byte chunk index is XOR-swizzled with (row/2)%8 so that the ds_read_b128 operand fetches of
// 16 consecutive rows cover all 64 banks exactly once.
// Workgroup ids are remapped so that each XCD (own L2) works on a compact patch of the tile
// grid.  Bigger tiles cut the L1/LDS traffic per flop (a 128x128 tile needs the full 64 B/clk of
// the CU's vector L1 at peak MFMA rate, a 256x256 tile half of it) but quantise badly on the few
// thousand rows of a pruned scale, so the launcher picks the tile per problem with a small cost
// model.
//
// fp32: plain LDS-tiled FMA kernel, used only by the fp32 parity configuration.
#include <cmath>
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
    int out_f32;   // bf16 kernel: write fp32 instead of bf16 (the intermediate residual stream)
    int res_f32;   // bf16 kernel: the residual operand is fp32
};

__device__ __forceinline__ float gelu_tanh(float v)
{
    // 0.5 v (1 + tanh(u)) = v / (1 + exp(-2u)),  u = sqrt(2/pi) (v + 0.044715 v^3)
    // exp(-2u) = exp2(v * (a + b v^2)) with a = -2 sqrt(2/pi) log2(e), b = 0.044715 a
    const float t = v * fmaf(-0.10294324f, v * v, -2.3022082f);
    return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
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

// Chunk swizzle of a k-major operand tile (rows = k, 256 or 512 bytes each, all starting at the
// same bank).  The transposing load reads, per 32 lanes, the rows {0..3, 8..11} (or {4..7,
// 12..15}) + 16n, 32 contiguous bytes of each: the 8 rows go to 8 different 32-byte eighths of the
// 256-byte bank span.
__device__ __forceinline__ int bkm_swz(int row)
{
    return ((row & 3) | (((row >> 3) & 1) << 2)) << 1;
}

// Epilogue of the bf16 kernel.  The accumulators of a wavefront are kept per 32x32 region
// [i][j] as 2x2 blocks [bi][bj] of the 16x16 MFMA: entry e of a block holds row
// 16*bi + 4*(lane/16) + e, column 16*bj + lane%16 of the region.  Each wavefront applies bias
// and GELU, packs to bf16 (adjacent lanes swap one value per row pair so that a lane owns two
// neighbouring columns)
// and parks its sub-tile row-major in a private LDS region; it then reads the sub-tile back as
// 16-byte row chunks, adds the residual (16-byte loads) and stores 16 bytes per lane, so a store
// instruction covers whole 128-byte row segments.  The destination row pointers (plain output,
// or the K / V cache rows of the sample the row belongs to) are computed once per chunk.
template <int FM, int FN, bool F32_STAGED>
__device__ __forceinline__ void store_tile_epilogue(const floatx4_t (*acc)[FN][2][2], const EpiParams &ep,
                                                    int rows, int N, int wrow0, int wcol0, int lane,
                                                    uint16_t *wlds)
{
    constexpr int TM = FM * 32, TN = FN * 32, PITCH = TN + 8;
    const int c16 = lane & 15, q16 = lane >> 4;
    const uint16_t *bias = reinterpret_cast<const uint16_t *>(ep.bias);
    if constexpr (F32_STAGED) {
        // fp32 output (never routed, never GELU-ed; the residual operand is bf16): same two-phase
        // scheme with an fp32 staging tile, 16-byte (4 float) row chunks out
        const uint16_t *res = reinterpret_cast<const uint16_t *>(ep.residual);
        float *out = reinterpret_cast<float *>(ep.out0);
        constexpr int P32 = TN + 4;
        float *w32 = reinterpret_cast<float *>(wlds);
#pragma unroll
        for (int jj = 0; jj < 2 * FN; ++jj) {
            const int j = jj >> 1, bj = jj & 1;
            const int col = wcol0 + jj * 16 + c16;
            const float bv = (bias && col < N) ? bf16_to_f32(bias[col]) : 0.f;
#pragma unroll
            for (int ii = 0; ii < 2 * FM; ++ii)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w32[(ii * 16 + 4 * q16 + e) * P32 + jj * 16 + c16] = acc[ii >> 1][j][ii & 1][bj][e] + bv;
        }
        asm volatile("" ::: "memory");       // staging stores and loads use different vector types
        constexpr int CPR = TN / 4, RPI = 64 / CPR;
        const int lc = (lane % CPR) * 4, col = wcol0 + lc;
#pragma unroll
        for (int it = 0; it < TM / RPI; ++it) {
            const int lrow = it * RPI + lane / CPR, row = wrow0 + lrow;
            float4 v = *reinterpret_cast<const float4 *>(w32 + lrow * P32 + lc);
            if (row >= rows || col >= N) continue;
            if (res) {
                const uint2 rv = *reinterpret_cast<const uint2 *>(res + (size_t)row * N + col);
                v.x += bf16_lo(rv.x); v.y += bf16_hi(rv.x); v.z += bf16_lo(rv.y); v.w += bf16_hi(rv.y);
            }
            *reinterpret_cast<float4 *>(out + (size_t)row * ep.ld0 + col) = v;
        }
        asm volatile("" ::: "memory");
        return;
    }
    const int odd = lane & 1;
#pragma unroll
    for (int jj = 0; jj < 2 * FN; ++jj) {
        const int j = jj >> 1, bj = jj & 1;
        const int col = wcol0 + jj * 16 + c16;
        const float bv = (bias && col < N) ? bf16_to_f32(bias[col]) : 0.f;
        const int lcol = jj * 16 + c16 - odd;                // even column of the stored pair
#pragma unroll
        for (int ii = 0; ii < 2 * FM; ++ii) {
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
                float v0 = acc[ii >> 1][j][ii & 1][bj][e] + bv, v1 = acc[ii >> 1][j][ii & 1][bj][e + 1] + bv;
                if (ep.gelu) { v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); }
                const float send = odd ? v0 : v1;
                const float recv = __shfl_xor(send, 1);
                const int lrow = ii * 16 + 4 * q16 + e + odd;
                *reinterpret_cast<uint32_t *>(wlds + lrow * PITCH + lcol) =
                    odd ? pack_bf16x2(recv, v1) : pack_bf16x2(v0, recv);
            }
        }
    }
    // the region is private to this wavefront and LDS operations of one wavefront complete in
    // order, so no barrier is needed between the two phases (the compiler is kept from moving the
    // accesses across this point: the stores and loads use different vector types)
    asm volatile("" ::: "memory");
    constexpr int CPR = TN / 8, RPI = 64 / CPR;             // chunks per row, rows per instruction
    const uint16_t *res = reinterpret_cast<const uint16_t *>(ep.residual);
    const bool routed = ep.split < N;                       // K/V columns go to the cache
    const float inv_rps = 1.0f / (float)ep.rows_per_sample;
    const int lc = (lane % CPR) * 8, col = wcol0 + lc;
#pragma unroll
    for (int it = 0; it < TM / RPI; ++it) {
        const int lrow = it * RPI + lane / CPR, row = wrow0 + lrow;
        uint4 v = *reinterpret_cast<const uint4 *>(wlds + lrow * PITCH + lc);
        if (row >= rows || col >= N) continue;
        if (res) {
            float a[8], r[8];
            Elem<uint16_t>::unpack(v, a);
            if (ep.res_f32) {
                const float *rf = reinterpret_cast<const float *>(ep.residual) + (size_t)row * N + col;
                Elem<float>::unpack(*reinterpret_cast<const uint4 *>(rf), r);
                Elem<float>::unpack(*reinterpret_cast<const uint4 *>(rf + 4), r + 4);
            } else {
                Elem<uint16_t>::unpack(*reinterpret_cast<const uint4 *>(res + (size_t)row * N + col), r);
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) a[t] += r[t];
            v = Elem<uint16_t>::pack(a);
        }
        uint16_t *dst;
        const int c = col - ep.split;
        if (!routed || c < 0) {
            dst = (uint16_t *)ep.out0 + (size_t)row * ep.ld0 + col;
        } else {
            // sample index: float estimate, then one exact correction step
            int b = (int)(((float)row + 0.5f) * inv_rps);
            int j0 = row - b * ep.rows_per_sample;
            if (j0 < 0) { --b; j0 += ep.rows_per_sample; }
            else if (j0 >= ep.rows_per_sample) { ++b; j0 -= ep.rows_per_sample; }
            const size_t crow = (size_t)b * ep.cap + ep.len + j0;
            dst = (c < ep.hd) ? (uint16_t *)ep.kcache + crow * ep.hd + c
                              : (uint16_t *)ep.vcache + crow * ep.hd + (c - ep.hd);
        }
        *reinterpret_cast<uint4 *>(dst) = v;
    }
    asm volatile("" ::: "memory");
}

// The operand tiles travel global -> LDS directly (global_load_lds_dwordx4: 16 bytes per lane, a
// wavefront fills 1 KiB = 8 swizzled rows per instruction) into a ring of STAGES buffers,
// STAGES-1 k-tiles ahead of the MFMAs.  No staging registers, no LDS store instructions; the
// loads are counted by hand (vmcnt) because the compiler does not see them.
// M0 carries the LDS base of the instruction; nothing else in these kernels uses M0 (gfx9+ LDS
// instructions do not), and it is rewritten before every use.
__device__ __forceinline__ void dma_b128(const void *base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}

// LDS needed after the main loop: k-split reduction buffer + one staging tile per wavefront.
// A wavefront sends its sub-tile through the epilogue in passes of a few 32-row fragments:
// epi_frags() for bf16 output (a staging tile of at most 128 rows), epi_frags_f32() for fp32
// output (as many fragments as fit the LDS with 4-byte elements, at least one).
constexpr size_t kLdsLimit = 160 * 1024;
constexpr size_t gemm_red_bytes(int BM, int BN, int KS) { return KS > 1 ? (size_t)BM * BN * 4 : 0; }
constexpr int epi_frags(int FM) { return FM > 4 ? (FM + 1) / 2 : FM; }
constexpr size_t epi_bytes_bf16(int BM, int BN, int WM, int WN)
{
    return (size_t)32 * epi_frags(BM / WM / 32) * (BN / WN + 8) * 2 * WM * WN;
}
constexpr size_t epi_bytes_f32(int BN, int WM, int WN, int fe)
{
    return (size_t)32 * fe * (BN / WN + 4) * 4 * WM * WN;
}
constexpr int epi_frags_f32(int BM, int BN, int WM, int WN, int KS)
{
    int fe = epi_frags(BM / WM / 32);
    while (fe > 1 && gemm_red_bytes(BM, BN, KS) + epi_bytes_f32(BN, WM, WN, fe) > kLdsLimit) --fe;
    return fe;
}
constexpr size_t gemm_epi_lds_bytes(int BM, int BN, int WM, int WN, int KS)
{
    const size_t a = epi_bytes_bf16(BM, BN, WM, WN);
    const size_t b = epi_bytes_f32(BN, WM, WN, epi_frags_f32(BM, BN, WM, WN, KS));
    return gemm_red_bytes(BM, BN, KS) + (a > b ? a : b);
}

// KS > 1 splits every k-tile between KS groups of WM x WN wavefronts (group ks takes the 32-wide
// k-steps ks, ks+KS, ...); the groups' partial accumulators are summed through LDS before the
// epilogue.  This doubles the wavefronts per CU for problems that give a CU only one small tile.
//
// BKM ("B k-major"): the second operand is given as X[K][N] (row = contraction index, as a token
// map is when the contraction runs over tokens: paper, Sec. "Random Projection (RP) for Low-Rank
// Feature", Q^T X) instead of W[N][K].  Its tiles travel to LDS in their own row-major layout and
// the B fragments come from the transposing LDS load.  This mode runs `nbatch` independent
// problems of one shape in one launch (operands and output `*_bstride` elements apart), whole
// tiles only (no division of the contraction), K a multiple of 64 and N a multiple of 8.
// nbatch > 1 is also available with the ordinary operand layout (whole tiles only).
template <int BM, int BN, int WM, int WN, int STAGES, int KS, bool BKM = false>
__global__ __launch_bounds__(64 * WM * WN * KS) void gemm_bf16_kernel(
    const uint16_t *__restrict__ A_in, const uint16_t *__restrict__ W_in, int rows, int N, int K,
    int tiles_m, int tiles_n, int group_m, EpiParams ep, int nsplit, float *__restrict__ part,
    int full_tiles, int tail_split, int nbatch, size_t a_bstride, size_t w_bstride,
    size_t o_bstride)
{
    const uint16_t *A = A_in, *W = W_in;
    constexpr int NW = WM * WN * KS;                   // wavefronts per workgroup
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int NGA = BM / 8 / NW, NGB = BN / 8 / NW; // 1 KiB groups (8 rows) per wavefront
    constexpr int NG = NGA + NGB;                      // DMA instructions per lane per k-tile
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    extern __shared__ uint4 lds_raw[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds_raw;

    // Work decomposition.  Workgroups are dealt to the 8 XCDs round-robin; XCD x takes the x-th
    // eighth of the work in ascending order.  Three modes:
    //  * plain: one workgroup per tile;
    //  * nsplit > 1 (too few tiles to fill the chip): the contraction axis of every tile is divided
    //    between nsplit workgroups, partial tiles go to `part` in the output's [rows][N] layout;
    //  * tail_split > 1 (the tiles beyond the last full round of 256 would leave most CUs idle):
    //    the first full_tiles tiles run whole, each later tile is divided between tail_split
    //    workgroups whose partial tiles go to `part` tile by tile; every XCD gets an eighth of
    //    the whole tiles first and an eighth of the divided ones after them.
    // Partial tiles are summed and finished by a second kernel.
    const int ntiles = tiles_m * tiles_n * nbatch;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    int pid, split = 0, ranges = 1;
    if (tail_split > 1) {
        const int nf = full_tiles / 8, tail_units = (ntiles - full_tiles) * tail_split;
        const int nt = (tail_units + 7) / 8;
        if (slot < nf) {
            pid = xcd * nf + slot;
        } else {
            const int t = xcd * nt + (slot - nf);
            if (slot - nf >= nt || t >= tail_units) return;
            pid = full_tiles + t / tail_split;
            split = t % tail_split;
            ranges = tail_split;
        }
    } else {
        const int per_xcd = (gridDim.x + 7) / 8;
        pid = xcd * per_xcd + slot;
        if (pid >= ntiles * nsplit) return;
        split = pid % nsplit;
        pid /= nsplit;
        ranges = nsplit;
    }
    const int tile_id = pid;
    if (BKM || nbatch > 1) {
        const int per = tiles_m * tiles_n, bidx = pid / per;
        pid -= bidx * per;
        A += (size_t)bidx * a_bstride;
        W += (size_t)bidx * w_bstride;
        ep.out0 = reinterpret_cast<char *>(ep.out0) + (size_t)bidx * o_bstride * (ep.out_f32 ? 4 : 2);
    }
    // consecutive tile ids run down group_m row tiles, then across the columns: the contiguous
    // id range of one XCD is a patch of about group_m x (tiles/8/group_m) tiles
    const int group = pid / (group_m * tiles_n);
    const int first_m = group * group_m;
    const int gsize = min(tiles_m - first_m, group_m);
    const int tm = first_m + (pid % (group_m * tiles_n)) % gsize;
    const int tn = (pid % (group_m * tiles_n)) / gsize;
    const int row0 = tm * BM, col0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c16 = lane & 15, q16 = lane >> 4;
    const int ks = wave / (WM * WN), wsub = wave % (WM * WN);
    const int wm = wsub / WN, wn = wsub % WN;

    // ---- DMA assignment: wavefront w owns the 8-row groups w, w+NW, ... of each tile; lane l of a
    // group fills physical chunk l%8 of row 8*group + l/8, i.e. it fetches the logical chunk that
    // the swizzle maps there
    uint32_t a_off[NGA], b_off[NGB];                   // byte offsets of this lane's 16 B at k = 0
#pragma unroll
    for (int i = 0; i < NGA; ++i) {
        const int r = (wave + NW * i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        a_off[i] = (uint32_t)(((size_t)min(row0 + r, rows - 1) * K + c * 8) * sizeof(uint16_t));
    }
#pragma unroll
    for (int i = 0; i < NGB; ++i) {
        if (BKM) {
            // k-major tile [BK][BN]: a 1 KiB instruction fills 1024 / (2 BN) whole k-rows; lane l
            // fills physical chunk l % (BN/8) of its row with the logical chunk the swizzle maps there
            constexpr int CPR = BN / 8, RPI = 64 / CPR;
            const int r = (wave + NW * i) * RPI + lane / CPR;
            const int c = (lane % CPR) ^ bkm_swz(r);
            b_off[i] = (uint32_t)(((size_t)r * N + min(col0 + c * 8, N - 8)) * sizeof(uint16_t));
        } else {
            const int r = (wave + NW * i) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            b_off[i] = (uint32_t)(((size_t)min(col0 + r, N - 1) * K + c * 8) * sizeof(uint16_t));
        }
    }
    const int ktiles_all = K / BK, kper = (ktiles_all + ranges - 1) / ranges;
    const int kt0 = split * kper;
    const int ktiles = min(ktiles_all, kt0 + kper) - kt0;   // k-tiles of this workgroup (>= 1)
    // DMA instructions i0 .. i1-1 (of the NG that make up a k-tile) of k-tile kt into `stage`
    auto issue_part = [&](int kt, int stage, int i0, int i1) {
        const int koff = (kt0 + kt) * BK;
        const uint32_t sbase = lds_base + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < NGA; ++i)
            if (i >= i0 && i < i1) dma_b128(A + koff, a_off[i], sbase + i * (NW * 1024));
#pragma unroll
        for (int i = 0; i < NGB; ++i)
            if (NGA + i >= i0 && NGA + i < i1)
                dma_b128(BKM ? W + (size_t)koff * N : W + koff, b_off[i],
                         sbase + BM * BK * 2 + i * (NW * 1024));
    };
    // DMA of this workgroup's whole k-tile kt into `stage`
    auto issue = [&](int kt, int stage) { issue_part(kt, stage, 0, NG); };

    floatx4_t acc[FM][FN][2][2];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[i][j][b >> 1][b & 1] = floatx4_t{0};

    const uint16_t *lds = reinterpret_cast<const uint16_t *>(lds_raw);
    // Operand fragments (16x16x32 MFMA: lane l holds row l%16, k-values 8*(l/16) .. +7 of a 32-wide
    // k-step).  The MFMAs of a k-tile are walked as ROWS = steps x (TM/16) "rows": one A fragment
    // (16 tile rows) against the FN16 B fragments of its k-step.  A fragments go through a ring of
    // four slots filled three rows ahead of their use; the B fragments of a k-step are double
    // buffered.  The ring runs across k-tiles: the hand-over point of the loop (DMA of k-tile kt+1
    // landed, barrier) sits three rows before the end of k-tile kt, by which time every wavefront
    // holds all fragments of k-tile kt in registers, so the same barrier frees that tile's stage
    // for the DMA of k-tile kt+STAGES.
    constexpr int FM16 = TM / 16, FN16 = TN / 16;
    constexpr int SPW = BK / 32 / KS;                    // k-steps of this wavefront per k-tile
    constexpr int ROWS = SPW * FM16;
    static_assert(ROWS % 4 == 0 && ROWS >= 4, "ring of four A fragments");
    constexpr int SPREAD = ROWS >= 12 ? 6 : 1;           // rows over which a k-tile's DMA is issued
    static_assert(STAGES == 2 || STAGES == 3, "wait counts below are written for 2 or 3 stages");
    auto load_a = [&](const uint16_t *tile, int row) {   // row of the walk -> fragment
        const int q = row / FM16, i = row % FM16;
        const int r = wm * TM + i * 16 + c16;
        return *reinterpret_cast<const bf16x8_t *>(tile + lds_off(r, (q * KS + ks) * 4 + q16));
    };
    auto load_b = [&](const uint16_t *tile, int q, bf16x8_t *b) {
        if constexpr (BKM) {
            // lane l needs column 16j + l%16 at the k-values 8*(l/16) .. +7 of the k-step.  The
            // transposing load hands lane i of a 16-lane group element i%4 of the 8-byte chunks
            // that lanes 4t + i/4 (t = 0..3) point at: lane l points at k-row 8*(l/16) + (l%16)/4
            // (+4 for the second half) and at columns 16j + 4*(l%4) .. +3.
            typedef short bkm_shortx4_t __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) bkm_shortx4_t lds_shortx4_t;
            const int kr = (q * KS + ks) * 32 + 8 * q16 + (c16 >> 2);
#pragma unroll
            for (int j = 0; j < FN16; ++j) {
                const int chunk = (wn * TN + j * 16) / 8 + ((c16 & 3) >> 1);
                const uint16_t *src = tile + BM * BK + kr * BN + ((chunk ^ bkm_swz(kr)) << 3) + (c16 & 1) * 4;
                const bkm_shortx4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t *)src);
                const bkm_shortx4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t *)(src + 4 * BN));
                b[j] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        } else {
#pragma unroll
            for (int j = 0; j < FN16; ++j) {
                const int r = wn * TN + j * 16 + c16;
                b[j] = *reinterpret_cast<const bf16x8_t *>(tile + BM * BK + lds_off(r, (q * KS + ks) * 4 + q16));
            }
        }
    };

    issue(0, 0);
    if (ktiles > 1) issue(1, 1);
    if (STAGES == 3 && ktiles > 2) issue(2, 2);
    if (ktiles == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (STAGES == 3 && ktiles > 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NG) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NG) : "memory");
    __syncthreads();

    bf16x8_t ring[4], bb[2][FN16];
    load_b(lds, 0, bb[0]);
#pragma unroll
    for (int t = 0; t < 3; ++t) ring[t] = load_a(lds, t);
    int stage = 0;                                       // stage holding k-tile kt
    for (int kt = 0; kt < ktiles; ++kt) {
        const uint16_t *cur = lds + stage * (STAGE_BYTES / 2);
        const int nstage = stage + 1 == STAGES ? 0 : stage + 1;
        const uint16_t *nxt = lds + nstage * (STAGE_BYTES / 2);
        const bool more = kt + 1 < ktiles;               // uniform
#pragma unroll
        for (int row = 0; row < ROWS; ++row) {
            const int q = row / FM16, i = row % FM16;
            if (row == ROWS - 3 && more) {
                // own reads of this stage are complete before the barrier says so
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                // k-tile kt+1 has landed once only the requests of the tiles after it are outstanding
                if (STAGES == 3 && kt + 2 < ktiles) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NG) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (SPW % 2 == 0) load_b(nxt, 0, bb[0]);
            }
            // The DMA of k-tile kt+STAGES into the stage that the hand-over frees is issued a few
            // instructions per row over the SPREAD rows that follow the hand-over (they run into
            // the next k-tile): a burst of all NG instructions from all wavefronts at once fills
            // the CU's vector-memory queue and holds up the MFMAs queued behind them.
            if (row >= ROWS - 3) {
                const int w = row - (ROWS - 3);
                if (w < SPREAD && more && kt + STAGES < ktiles)
                    issue_part(kt + STAGES, stage, w * NG / SPREAD, (w + 1) * NG / SPREAD);
            } else if (row + 3 < SPREAD) {
                const int w = row + 3;
                if (kt >= 1 && kt - 1 + STAGES < ktiles)
                    issue_part(kt - 1 + STAGES, stage == 0 ? STAGES - 1 : stage - 1, w * NG / SPREAD,
                               (w + 1) * NG / SPREAD);
            }
            if (row + 3 < ROWS) ring[(row + 3) & 3] = load_a(cur, row + 3);
            else if (more) ring[(row + 3) & 3] = load_a(nxt, row + 3 - ROWS);
            // B fragments of the next k-step of this tile, fetched in the middle of the current one
            if (i == FM16 / 2 && q + 1 < SPW) load_b(cur, q + 1, bb[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < FN16; ++j)
                acc[i >> 1][j >> 1][i & 1][j & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    ring[row & 3], bb[q & 1][j], acc[i >> 1][j >> 1][i & 1][j & 1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // with an odd number of k-steps per tile the first B buffer is in use until the tile's end
        if (SPW % 2 == 1 && more) load_b(nxt, 0, bb[0]);
        stage = nstage;
    }
    // the stage buffers are reused below: every wavefront must be past its last operand read
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
    // every request has landed and every wavefront is past its last operand read (barrier above):
    // the stage buffers are free for the k-split reduction and the epilogue's staging
    constexpr int RED_FLOATS = KS > 1 ? WM * WN * FM * FN * 16 * 64 : 0;
    if (KS > 1) {
        // partial accumulators in lane-major order: entry (tile, e) of lane l at (tile*16+e)*64 + l
        float *red = reinterpret_cast<float *>(lds_raw) + wsub * (FM * FN * 16 * 64) + lane;
        if (ks != 0) {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) red[((i * FN + j) * 16 + e) * 64] = acc[i][j][(e >> 3) & 1][(e >> 2) & 1][e & 3];
        }
        __syncthreads();
        if (ks != 0) return;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][(e >> 3) & 1][(e >> 2) & 1][e & 3] += red[((i * FN + j) * 16 + e) * 64];
    }
    if (ranges > 1) {
        // partial tile, fp32: 16 neighbouring lanes cover 64 contiguous bytes of a row.
        // Divided problem: [range][rows][N]; divided tail: [tail tile][range][BM][BN].
        const bool tail = tail_split > 1;
        float *dst = tail ? part + ((size_t)(tile_id - full_tiles) * tail_split + split) * (BM * BN)
                          : part + (size_t)split * rows * N;
        const size_t pitch = tail ? BN : N;
        const int rbase = tail ? 0 : row0, cbase = tail ? 0 : col0;
#pragma unroll
        for (int jj = 0; jj < 2 * FN; ++jj) {
            const int lcol = wn * TN + jj * 16 + c16;
            if (col0 + lcol >= N) continue;
#pragma unroll
            for (int ii = 0; ii < 2 * FM; ++ii)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int lrow = wm * TM + ii * 16 + 4 * q16 + e;
                    if (row0 + lrow < rows)
                        dst[(size_t)(rbase + lrow) * pitch + cbase + lcol] = acc[ii >> 1][jj >> 1][ii & 1][jj & 1][e];
                }
        }
        return;
    }
    // per-wavefront staging region behind the reduction buffer; the sub-tile passes through it a few
    // fragments at a time (fewer per pass when the output is fp32)
    constexpr int FE = epi_frags(FM), FE32 = epi_frags_f32(BM, BN, WM, WN, KS);
    static_assert(gemm_red_bytes(BM, BN, KS) + epi_bytes_f32(BN, WM, WN, FE32) <= kLdsLimit, "fp32 staging");
    char *stage_base = reinterpret_cast<char *>(lds_raw) + RED_FLOATS * 4;
    if (ep.out_f32) {
        uint16_t *wlds = reinterpret_cast<uint16_t *>(stage_base + wsub * (FE32 * 32 * (TN + 4) * 4));
#pragma unroll
        for (int f0 = 0; f0 < FM; f0 += FE32) {
            constexpr int dummy = 0; (void)dummy;
            if (f0 + FE32 <= FM)
                store_tile_epilogue<FE32, FN, true>(acc + f0, ep, rows, N, row0 + wm * TM + f0 * 32,
                                                    col0 + wn * TN, lane, wlds);
            else
                store_tile_epilogue<(FM % FE32 ? FM % FE32 : FE32), FN, true>(
                    acc + f0, ep, rows, N, row0 + wm * TM + f0 * 32, col0 + wn * TN, lane, wlds);
        }
        return;
    }
    uint16_t *wlds = reinterpret_cast<uint16_t *>(stage_base + wsub * (FE * 32 * (TN + 8) * 2));
    store_tile_epilogue<FE, FN, false>(acc, ep, rows, N, row0 + wm * TM, col0 + wn * TN, lane, wlds);
    if constexpr (FE < FM)
        store_tile_epilogue<FM - FE, FN, false>(acc + FE, ep, rows, N, row0 + wm * TM + FE * 32,
                                                col0 + wn * TN, lane, wlds);
}

// Sum of the partial tiles of the divided tail + the epilogue (bias, GELU, residual, bf16 or fp32
// output; never the K/V routing).  One thread per 4 consecutive columns of one tile row.
__global__ __launch_bounds__(256) void gemm_tail_epilogue_kernel(const float *__restrict__ part,
                                                                 int ranges, int full_tiles,
                                                                 int tiles_m, int tiles_n, int group_m,
                                                                 int BM, int BN, int rows, int N,
                                                                 long total, EpiParams ep)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;       // over tail tiles * BM * BN/4
    if (idx >= total) return;
    const int cpr = BN / 4;
    const int lcol = (int)(idx % cpr) * 4;
    const long tr = idx / cpr;
    const int lrow = (int)(tr % BM), tt = (int)(tr / BM), pid = full_tiles + tt;
    const int group = pid / (group_m * tiles_n);
    const int first_m = group * group_m;
    const int gsize = min(tiles_m - first_m, group_m);
    const int tm = first_m + (pid % (group_m * tiles_n)) % gsize;
    const int tn = (pid % (group_m * tiles_n)) / gsize;
    const int row = tm * BM + lrow, col = tn * BN + lcol;
    if (row >= rows || col >= N) return;
    const float *src = part + (size_t)tt * ranges * BM * BN + (size_t)lrow * BN + lcol;
    float4 v = *reinterpret_cast<const float4 *>(src);
    for (int s = 1; s < ranges; ++s) {
        const float4 p = *reinterpret_cast<const float4 *>(src + (size_t)s * BM * BN);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (ep.bias) {
        const uint2 b = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(ep.bias) + col);
        v.x += bf16_lo(b.x); v.y += bf16_hi(b.x); v.z += bf16_lo(b.y); v.w += bf16_hi(b.y);
    }
    if (ep.gelu) { v.x = gelu_tanh(v.x); v.y = gelu_tanh(v.y); v.z = gelu_tanh(v.z); v.w = gelu_tanh(v.w); }
    const size_t off = (size_t)row * N + col;
    if (ep.residual) {
        if (ep.res_f32) {
            const float4 r = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(ep.residual) + off);
            v.x += r.x; v.y += r.y; v.z += r.z; v.w += r.w;
        } else {
            const uint2 r = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(ep.residual) + off);
            v.x += bf16_lo(r.x); v.y += bf16_hi(r.x); v.z += bf16_lo(r.y); v.w += bf16_hi(r.y);
        }
    }
    const size_t ooff = (size_t)row * ep.ld0 + col;
    if (ep.out_f32)
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(ep.out0) + ooff) = v;
    else
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(ep.out0) + ooff) =
            make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
}

// tail > 1: the tiles beyond the last full round of 256 are divided into `tail` ranges of the
// contraction axis each (nsplit must be 1 then)
template <int BM, int BN, int WM, int WN, int STAGES, int KS = 1>
static void launch_gemm_bf16_cfg(const void *A, const void *W, int rows, int N, int K,
                                 const EpiParams &ep, hipStream_t st, int nsplit = 1,
                                 float *part = nullptr, int tail = 1)
{
    const int tiles_m = (rows + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int ntiles = tiles_m * tiles_n;
    const int full_tiles = tail > 1 ? ntiles / 256 * 256 : ntiles;
    const int tail_units = (ntiles - full_tiles) * tail;
    const int grid = tail > 1 ? full_tiles + (tail_units + 7) / 8 * 8 : (ntiles * nsplit + 7) / 8 * 8;
    const size_t lds_stages = (size_t)STAGES * (BM + BN) * BK * sizeof(uint16_t);
    const size_t lds_epi = gemm_epi_lds_bytes(BM, BN, WM, WN, KS);
    const size_t lds = lds_stages > lds_epi ? lds_stages : lds_epi;
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, STAGES, KS>;
    // set on every launch: the attribute belongs to the current device's copy of the kernel
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    // patch height that minimises what one XCD has to pull through its own L2: a patch of g x c
    // tiles reads g row strips (BM x K) and c column strips (BN x K), with g * c = tiles / 8
    int group_m = (int)lround(sqrt((double)ntiles * BN / (8.0 * BM)));
    group_m = group_m < 1 ? 1 : (group_m > tiles_m ? tiles_m : group_m);
    launch(kern, dim3(grid), dim3(64 * WM * WN * KS), lds, st, (const uint16_t *)A,
                       (const uint16_t *)W, rows, N, K, tiles_m, tiles_n, group_m, ep, nsplit, part,
                       full_tiles, tail, 1, (size_t)0, (size_t)0, (size_t)0);
    if (tail > 1) {
        const long total = (long)(ntiles - full_tiles) * BM * (BN / 4);
        launch(gemm_tail_epilogue_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
               (const float *)part, tail, full_tiles, tiles_m, tiles_n, group_m, BM, BN, rows, N, total, ep);
    }
}

// out[b] = A[b] X[b] for nbatch problems with the second operand k-major (X[b]: [K][N], A[b]:
// [rows][K], `a_bstride` elements apart or shared when 0), bf16 output, no epilogue terms.
template <int BM, int BN, int WM, int WN, int STAGES>
static void launch_kmajor_cfg(const void *A, size_t a_bstride, const void *X, int nbatch, int rows,
                              int N, int K, void *out, hipStream_t st)
{
    EpiParams ep{};
    ep.out0 = out; ep.ld0 = N; ep.split = N; ep.N = N; ep.rows_per_sample = 1;
    const int tiles_m = (rows + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int ntiles = tiles_m * tiles_n * nbatch;
    const int grid = (ntiles + 7) / 8 * 8;
    const size_t lds_stages = (size_t)STAGES * (BM + BN) * BK * sizeof(uint16_t);
    const size_t lds_epi = gemm_epi_lds_bytes(BM, BN, WM, WN, 1);
    const size_t lds = lds_stages > lds_epi ? lds_stages : lds_epi;
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, STAGES, 1, true>;
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    int group_m = (int)lround(sqrt((double)tiles_m * tiles_n * BN / (8.0 * BM)));
    group_m = group_m < 1 ? 1 : (group_m > tiles_m ? tiles_m : group_m);
    launch(kern, dim3(grid), dim3(64 * WM * WN), lds, st, (const uint16_t *)A, (const uint16_t *)X, rows,
           N, K, tiles_m, tiles_n, group_m, ep, 1, (float *)nullptr, ntiles, 1, nbatch, a_bstride,
           (size_t)K * N, (size_t)rows * N);
}

// out[b] = A[b] W[b]^T in fp32 for nbatch problems of one shape (A[b]: [rows][K], W[b]: [N][K], both
// bf16 and `rows*K` / `N*K` elements apart; out[b]: [rows][N]) on the tiled MFMA kernel, when the
// shape suits it: K a multiple of the 64-wide k-tile, N <= 256 and enough tiles to fill three
// quarters of the chip.  Returns false (nothing launched) otherwise.
template <int BM, int BN, int WM, int WN, int STAGES>
static void launch_batched_f32_cfg(const void *A, const void *W, int nbatch, int rows, int N, int K,
                                   float *out, hipStream_t st)
{
    EpiParams ep{};
    ep.out0 = out; ep.ld0 = N; ep.split = N; ep.N = N; ep.rows_per_sample = 1; ep.out_f32 = 1;
    const int tiles_m = (rows + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int ntiles = tiles_m * tiles_n * nbatch;
    const int grid = (ntiles + 7) / 8 * 8;
    const size_t lds_stages = (size_t)STAGES * (BM + BN) * BK * sizeof(uint16_t);
    const size_t lds_epi = gemm_epi_lds_bytes(BM, BN, WM, WN, 1);
    const size_t lds = lds_stages > lds_epi ? lds_stages : lds_epi;
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, STAGES, 1, false>;
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    int group_m = (int)lround(sqrt((double)tiles_m * tiles_n * BN / (8.0 * BM)));
    group_m = group_m < 1 ? 1 : (group_m > tiles_m ? tiles_m : group_m);
    launch(kern, dim3(grid), dim3(64 * WM * WN), lds, st, (const uint16_t *)A, (const uint16_t *)W, rows,
           N, K, tiles_m, tiles_n, group_m, ep, 1, (float *)nullptr, ntiles, 1, nbatch,
           (size_t)rows * K, (size_t)N * K, (size_t)rows * N);
}

bool launch_gemm_bf16_batched_f32(const void *A, const void *W, int nbatch, int rows, int N, int K,
                                  float *out, hipStream_t st)
{
    if (K < BK || K % BK != 0 || N < 1 || N > 256 || rows < 1 || nbatch < 1) return false;
    if ((size_t)rows * K * sizeof(uint16_t) >= ((size_t)1 << 32)) return false;   // 32-bit operand offsets
    const bool narrow = N <= 128;
    const long tiles = (long)((rows + 255) / 256) * nbatch;
    if (tiles < 192) return false;
    if (narrow) launch_batched_f32_cfg<256, 128, 4, 2, 3>(A, W, nbatch, rows, N, K, out, st);
    else launch_batched_f32_cfg<256, 256, 2, 4, 2>(A, W, nbatch, rows, N, K, out, st);
    return true;
}

// Runs out[b] = qt[b] x[b] (qt: [rows][M] per sample or shared, x[b]: [M][d]) on the tiled MFMA
// kernel when the shape suits it: M a multiple of the 64-wide k-tile, d a multiple of 8, and
// enough tiles to fill three quarters of the chip.  Returns false (nothing launched) otherwise.
bool launch_gemm_bf16_kmajor(const void *qt, size_t q_stride, const void *x, int B, int M, int rows,
                             int d, void *out, hipStream_t st)
{
    if (M < BK || M % BK != 0 || d % 8 != 0 || d < 8 || rows < 1 || B < 1) return false;
    if ((size_t)rows * M * sizeof(uint16_t) >= ((size_t)1 << 32)) return false;   // 32-bit operand offsets
    struct Cand { int bm, bn; double rate; };
    // (no 320x256 tile here: with the transposing reads it would not fit the 256 registers)
    const Cand cands[4] = {{256, 256, 1155.0}, {128, 256, 1041.0}, {192, 256, 1100.0},
                           {256, 128, 1045.0}};
    int best = -1;
    double best_cost = 1e300;
    for (int i = 0; i < 4; ++i) {
        const long tiles = (long)((rows + cands[i].bm - 1) / cands[i].bm) *
                           ((d + cands[i].bn - 1) / cands[i].bn) * B;
        if (tiles < 192) continue;
        const double t_tile = 2.0 * cands[i].bm * cands[i].bn * (double)M * 256.0 / (cands[i].rate * 1e6);
        const double cost = (double)((tiles + 255) / 256) * t_tile;
        if (cost < best_cost) { best_cost = cost; best = i; }
    }
    switch (best) {
    case 0: launch_kmajor_cfg<256, 256, 2, 4, 2>(qt, q_stride, x, B, rows, d, M, out, st); break;
    case 1: launch_kmajor_cfg<128, 256, 2, 4, 3>(qt, q_stride, x, B, rows, d, M, out, st); break;
    case 2: launch_kmajor_cfg<192, 256, 2, 4, 2>(qt, q_stride, x, B, rows, d, M, out, st); break;
    case 3: launch_kmajor_cfg<256, 128, 4, 2, 3>(qt, q_stride, x, B, rows, d, M, out, st); break;
    default: return false;
    }
    return true;
}

// Sum of the partial tiles of a split contraction + the epilogue (bias, GELU, residual, bf16 or
// fp32 output; never the K/V routing).  One thread per 4 consecutive columns.
__global__ __launch_bounds__(256) void gemm_splitk_epilogue_kernel(const float *__restrict__ part,
                                                                   int nsplit, int rows, int N,
                                                                   EpiParams ep)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const int cpr = N / 4;
    if (idx >= (long)rows * cpr) return;
    const int row = (int)(idx / cpr), col = (int)(idx % cpr) * 4;
    const size_t off = (size_t)row * N + col;
    float4 v = *reinterpret_cast<const float4 *>(part + off);
    for (int s = 1; s < nsplit; ++s) {
        const float4 p = *reinterpret_cast<const float4 *>(part + (size_t)s * rows * N + off);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (ep.bias) {
        const uint2 b = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(ep.bias) + col);
        v.x += bf16_lo(b.x); v.y += bf16_hi(b.x); v.z += bf16_lo(b.y); v.w += bf16_hi(b.y);
    }
    if (ep.gelu) { v.x = gelu_tanh(v.x); v.y = gelu_tanh(v.y); v.z = gelu_tanh(v.z); v.w = gelu_tanh(v.w); }
    if (ep.residual) {
        if (ep.res_f32) {
            const float4 r = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(ep.residual) + off);
            v.x += r.x; v.y += r.y; v.z += r.z; v.w += r.w;
        } else {
            const uint2 r = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(ep.residual) + off);
            v.x += bf16_lo(r.x); v.y += bf16_hi(r.x); v.z += bf16_lo(r.y); v.w += bf16_hi(r.y);
        }
    }
    const size_t ooff = (size_t)row * ep.ld0 + col;
    if (ep.out_f32)
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(ep.out0) + ooff) = v;
    else
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(ep.out0) + ooff) =
            make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
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

// Tile configuration for a problem: rounds of workgroups over the 256 CUs (one workgroup per CU
// at these LDS sizes) x time of one tile at the sustained rate of the configuration (TFLOP/s
// measured on large problems).  With `allow_tail` the tiles beyond the last full round may be
// divided along the contraction axis into 2..8 ranges (each at least 8 k-tiles long) so that
// they fill the chip once more at a fraction of a tile's time; their fp32 partial tiles cost a
// write and a read at about 4 TB/s.
struct GemmPlan { int cfg; long tiles; int tail; size_t tail_floats; };
static GemmPlan plan_bf16(int rows, int N, int K, bool allow_tail)
{
    struct Cand { int bm, bn; double rate; };
    const Cand cands[6] = {{256, 256, 1155.0}, {256, 128, 1045.0}, {128, 256, 1041.0},
                           {128, 128, 1000.0}, {320, 256, 1300.0}, {192, 256, 1100.0}};
    GemmPlan best{0, 0, 1, 0};
    double best_cost = 1e300;
    for (int i = 0; i < 6; ++i) {
        const long tiles = (long)((rows + cands[i].bm - 1) / cands[i].bm) *
                           ((N + cands[i].bn - 1) / cands[i].bn);
        double rate = cands[i].rate;
        if (i == 3 && tiles > 256) rate = 650.0;       // small tiles pay per round
        const double area = (double)cands[i].bm * cands[i].bn;
        const double t_tile = 2.0 * area * K * 256.0 / (rate * 1e6);     // microseconds on one CU
        const double cost = (double)((tiles + 255) / 256) * t_tile;
        if (cost < best_cost) { best_cost = cost; best = GemmPlan{i, tiles, 1, 0}; }
        const long full = tiles / 256 * 256, rem = tiles - full;
        if (!allow_tail || i == 3 || full == 0 || rem == 0) continue;
        for (int s = 2; s <= 8; ++s) {
            if (rem * s > 256 || K / BK / s < 8) break;
            const double c2 = (double)(full / 256) * t_tile + t_tile / s + 10.0 +
                              (double)rem * s * area * 8.0 / 4e6;
            if (c2 < best_cost) {
                best_cost = c2;
                best = GemmPlan{i, tiles, s, (size_t)rem * s * (size_t)area};
            }
        }
    }
    return best;
}
static int pick_bf16_config(int rows, int N, long *tiles_out)
{
    const GemmPlan p = plan_bf16(rows, N, BK * 64, false);
    *tiles_out = p.tiles;
    return p.cfg;
}

// Workgroups per tile along the contraction axis: only when the tiles cover at most half of the
// CUs, every part at least 4 k-tiles long, at most 8 parts.
int gemm_splits(DType dt, int rows, int N, int K)
{
    if (dt != DType::BF16) return 1;
    long tiles;
    (void)pick_bf16_config(rows, N, &tiles);
    long s = 256 / tiles;
    const long kmax = K / BK / 4;
    if (s > kmax) s = kmax;
    if (s > 8) s = 8;
    if (s < 2) return 1;
    const long kt = K / BK, per = (kt + s - 1) / s;
    return (int)((kt + per - 1) / per);                  // no empty part
}

// Floats of scratch a bf16 linear layer may need for partial tiles (either way of dividing the
// contraction axis); 0 when every tile is computed by one workgroup.
size_t gemm_scratch_floats(DType dt, int rows, int N, int K)
{
    if (dt != DType::BF16) return 0;
    const int ns = gemm_splits(dt, rows, N, K);
    if (ns > 1) return (size_t)ns * rows * N;
    return plan_bf16(rows, N, K, true).tail_floats;
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
    ep.out_f32 = e.out_f32;
    ep.res_f32 = e.res_f32;
    if (dt == DType::BF16) {
        // the K/V routing lives in the in-kernel epilogue only, so the routed launch is never divided
        const bool may_divide = e.splitk_scratch && e.split == N;
        const int ns = may_divide ? gemm_splits(dt, rows, N, K) : 1;
        const GemmPlan plan = plan_bf16(rows, N, K, may_divide && ns == 1);
        const int best = ns > 1 ? plan_bf16(rows, N, K, false).cfg : plan.cfg;
        const int tail = ns > 1 ? 1 : plan.tail;
        float *part = (ns > 1 || tail > 1) ? e.splitk_scratch : nullptr;
        switch (best) {
        case 0: launch_gemm_bf16_cfg<256, 256, 2, 4, 2>(A, W, rows, N, K, ep, st, ns, part, tail); break;
        case 1: launch_gemm_bf16_cfg<256, 128, 4, 2, 3>(A, W, rows, N, K, ep, st, ns, part, tail); break;
        case 2: launch_gemm_bf16_cfg<128, 256, 2, 4, 3>(A, W, rows, N, K, ep, st, ns, part, tail); break;
        case 4: launch_gemm_bf16_cfg<320, 256, 2, 4, 2>(A, W, rows, N, K, ep, st, ns, part, tail); break;
        case 5: launch_gemm_bf16_cfg<192, 256, 2, 4, 2>(A, W, rows, N, K, ep, st, ns, part, tail); break;
        default: launch_gemm_bf16_cfg<128, 128, 2, 2, 3, 2>(A, W, rows, N, K, ep, st, ns, part, tail); break;
        }
        if (ns > 1) {
            const long total = (long)rows * (N / 4);
            launch(gemm_splitk_epilogue_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                   (const float *)part, ns, rows, N, ep);
        }
    } else {
        dim3 grid((N + 63) / 64, (rows + 63) / 64), block(256);
        launch(gemm_f32_kernel, grid, block, 0, st, (const float *)A, (const float *)W,
                           rows, N, K, ep);
    }
}

}  // namespace fvar
