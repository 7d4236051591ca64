// Attention of the rows that pass through the block over the whole multi-scale KV cache
// (every cached scale is <= the current one, so all L rows are visible to every query).
//
// bf16 kernel, flash style, written for 64-wide wavefronts and 32x32x16 MFMA:
//   * the score tile is computed TRANSPOSED, S^T = K Q^T (keys are the MFMA rows, queries the
//     columns).  In the 32x32 accumulator layout a lane then owns one query column, so the
//     running max / sum of the online softmax are lane-local scalars (one exchange with lane^32
//     per tile), the rescale of the output accumulator is a per-lane multiply, and the
//     probabilities are already laid out as the B operand of the second product
//     O^T = V^T P^T -- no trip through LDS for P.
//   * K and V tiles travel global -> LDS directly (global_load_lds_dwordx4, no staging registers,
//     no LDS store instructions), both row-major with XOR-swizzled 16-byte chunks; the swizzle is
//     applied on the global side (which chunk a lane fetches), since the DMA writes LDS in lane
//     order.  K rows feed the A operand of S^T with one ds_read_b128.  The A operand of the second
//     product needs V transposed (8 consecutive keys of one head-dim column per lane): it is read
//     with the transposing LDS load (ds_read_b64_tr_b16), which hands a lane 4 elements of one
//     column out of the 16 row chunks its 16-lane group points at -- V is never transposed in
//     memory.  The rows each lane points at follow the order in which the accumulator layout
//     hands out the keys of P.
//   * LDS is double buffered: the DMA of the next tile runs under the MFMAs of the current one,
//     one barrier per tile.
//
// fp32 kernel: plain tiled FMA version for the fp32 parity configuration.
#include <type_traits>

#include "common.h"

namespace fvar {

constexpr int BT = 64;                       // keys per tile

typedef short shortx4_t __attribute__((ext_vector_type(4)));
typedef short shortx8_t __attribute__((ext_vector_type(8)));

// 16 bytes per lane global -> LDS; the wavefront fills 1 KiB starting at `lds_addr` in lane order.
// M0 carries the LDS base and is rewritten before every use; no other instruction of these
// kernels reads it.  The loads are counted by hand (s_waitcnt vmcnt) because the compiler does
// not see them.
__device__ __forceinline__ void attn_dma_b128(const void *base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}

// Chunk swizzles (XOR on the 16-byte chunk index of a row).
//   K rows are read 16 rows at a time at one logical chunk (ds_read_b128): with 256-byte rows
//   (head_dim 128) all rows start at the same bank, so the 16 rows must land in 16 different
//   chunks; with 128-byte rows two neighbouring rows already differ by half the banks.
//   V rows are read by the transposing load 4 consecutive rows x 64 contiguous bytes at a time
//   (per 32 lanes): the 4 rows must land in different 64-byte quarters of the 256-byte bank span.
template <int DH> __device__ __forceinline__ int k_swz(int row)
{
    return DH == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int DH> __device__ __forceinline__ int v_swz(int row)
{
    return DH == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

// Position of workgroup `id` of `count` in a numbering that gives XCD x (= id % 8) the x-th
// contiguous share of [0, count): a bijection for any count.
__device__ __forceinline__ int xcd_contiguous(int id, int count)
{
    const int x = id & 7, pos = id >> 3, q = count >> 3, r = count & 7;
    return (x < r ? x * (q + 1) : r * (q + 1) + (x - r) * q) + pos;
}

template <int DH, int NQ>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(const uint16_t *__restrict__ q,
                                                        const uint16_t *__restrict__ Kc,
                                                        const uint16_t *__restrict__ Vc, int n, int L,
                                                        int cap, int H, float c_log2,
                                                        uint16_t *__restrict__ o, int nsplit,
                                                        int tiles_per_split,
                                                        float *__restrict__ part_o,
                                                        float *__restrict__ part_ml, int nqb,
                                                        int full_units, int tail_split)
{
    constexpr int KS = DH / 16;              // k16 steps of the QK product
    constexpr int DB = DH / 32;              // 32-row blocks of O^T
    constexpr int KCH = DH / 8;              // 16 B chunks per K / V row
    constexpr int RPD = 64 / KCH;            // tile rows filled by one DMA instruction (1 KiB)
    constexpr int NDMA = BT / RPD / 4;       // DMA instructions per wavefront per tile and tensor
    constexpr int KTILE = BT * DH, STAGE = 2 * KTILE;

    extern __shared__ uint4 lds_raw[];
    uint16_t *lds = reinterpret_cast<uint16_t *>(lds_raw);   // [stage][K tile | V tile]
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds_raw;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rl = lane & 31, g = lane >> 5;
    // Work decomposition.  A unit is one (query block, head, sample) triple, numbered with the
    // query block fastest.  Two ways of dividing the key axis between workgroups exist:
    //  * nsplit > 1 (problems with too few units to fill the chip): every unit is divided into
    //    nsplit key ranges, workgroup id = (sample * nsplit + range) * H * nqb + head * nqb + block;
    //  * tail_split > 1 (many units, but the last round of workgroups would leave most of the chip
    //    idle): the first full_units units run whole, each later unit is divided into tail_split
    //    ranges.
    // A workgroup with a partial key range [tile0, tile1) leaves an unnormalised partial result
    // (O, running max, running sum) for a merge kernel.
    // Workgroups are handed to the 8 XCDs in turn (id % 8), each with an L2 of its own, so ids
    // are first renumbered to give every XCD one contiguous run of the numbering above: the query
    // blocks of a head, which stream the same keys and values, then share one L2 instead of
    // fetching them from memory once per XCD.  Whole units and the divided last round are
    // renumbered separately, so the last round is still made of the short pieces on every XCD.
    int unit = blockIdx.x, split = 0, ranges = 1;
    size_t prow_base = 0;                                    // partial row of query 0 of this unit
    int prow_stride = 0;
    if (nsplit > 1) {
        unit = xcd_contiguous(unit, (int)gridDim.x);
        const int per = H * nqb, zz = unit / per;
        split = zz % nsplit;
        ranges = nsplit;
        unit = (zz / nsplit) * per + unit % per;
    } else if (unit < full_units) {
        unit = xcd_contiguous(unit, full_units);
    } else {
        const int t = xcd_contiguous(unit - full_units, (int)gridDim.x - full_units);
        unit = full_units + t / tail_split;
        split = t % tail_split;
        ranges = tail_split;
    }
    const int qb = unit % nqb, h = (unit / nqb) % H, b = unit / (nqb * H);
    if (nsplit > 1) {
        prow_base = (size_t)(b * nsplit + split) * n * H + h;
        prow_stride = H;
    } else if (ranges > 1) {
        prow_base = (size_t)((unit - full_units) * tail_split + split) * (128 * NQ) -
                    (size_t)qb * (128 * NQ);
        prow_stride = 1;
    }
    const int q0 = qb * (128 * NQ) + wave * (32 * NQ);
    const bool wave_active = __builtin_amdgcn_readfirstlane(q0 < n ? 1 : 0) != 0;
    const size_t rowpitch = (size_t)H * DH;
    const uint16_t *Kb = Kc + ((size_t)b * cap * H + h) * DH;
    const uint16_t *Vb = Vc + ((size_t)b * cap * H + h) * DH;

    // ---- Q fragments (B operand: lane = query column, 8 consecutive head-dim values)
    bf16x8_t qf[NQ][KS];
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const int row = min(q0 + j * 32 + rl, n - 1);
        const uint16_t *src = q + ((size_t)b * n + row) * rowpitch + (size_t)h * DH + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s)
            qf[j][s] = *reinterpret_cast<const bf16x8_t *>(src + 16 * s);
    }

    // ---- DMA assignment: wavefront w owns the 1 KiB row groups w, w+4, ... of each tile; lane l
    // fills physical chunk l % KCH of tile row RPD*group + l / KCH, i.e. it fetches the logical
    // chunk that the swizzle maps there.  Byte offsets from the tile's first row; a tile that
    // reaches past row L-1 recomputes them with the row clamped.
    int d_row[NDMA];
    uint32_t k_off[NDMA], v_off[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        d_row[i] = (wave + 4 * i) * RPD + lane / KCH;
        const int pc = lane % KCH;
        k_off[i] = (uint32_t)(((size_t)d_row[i] * rowpitch + ((pc ^ k_swz<DH>(d_row[i])) << 3)) * 2);
        v_off[i] = (uint32_t)(((size_t)d_row[i] * rowpitch + ((pc ^ v_swz<DH>(d_row[i])) << 3)) * 2);
    }
    auto issue_tile = [&](int t0, int stage) {
        const uint32_t sk = lds_base + stage * (STAGE * 2) + wave * 1024, sv = sk + KTILE * 2;
        if (t0 + BT <= L) {                                  // uniform
            const uint16_t *kt = Kb + (size_t)t0 * rowpitch, *vtile = Vb + (size_t)t0 * rowpitch;
#pragma unroll
            for (int i = 0; i < NDMA; ++i) attn_dma_b128(kt, k_off[i], sk + i * 4096);
#pragma unroll
            for (int i = 0; i < NDMA; ++i) attn_dma_b128(vtile, v_off[i], sv + i * 4096);
            return;
        }
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            const int t = min(t0 + d_row[i], L - 1), pc = lane % KCH;
            attn_dma_b128(Kb, (uint32_t)(((size_t)t * rowpitch + ((pc ^ k_swz<DH>(d_row[i])) << 3)) * 2),
                          sk + i * 4096);
        }
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            const int t = min(t0 + d_row[i], L - 1), pc = lane % KCH;
            attn_dma_b128(Vb, (uint32_t)(((size_t)t * rowpitch + ((pc ^ v_swz<DH>(d_row[i])) << 3)) * 2),
                          sv + i * 4096);
        }
    };

    // ---- transposing V read: lane l = 16*G + 4*j + a points at key row 4*(G/2) + j (+ 16u + 8h) and
    // the 4 head-dim values 16*(G%2) + 4*a (+ 32*db); it receives, for the output row
    // 16*(G%2) + (l%16) of block db, the keys 4*(G/2) + 0..3 (+ 16u + 8h): the k-slots 4h..4h+3 of
    // half G/2, in the order the P fragments hold them
    const int tG = lane >> 4, tj = (lane >> 2) & 3, ta = lane & 3;
    const int v_row = 4 * (tG >> 1) + tj;                    // key row inside a 16-key step (h = 0)
    const int v_swq = v_swz<DH>(v_row) >> 2;                 // depends on the lane only (rows +8, +16 keep it)
    const int v_lane = v_row * DH + ((2 * (tG & 1) + (ta >> 1)) << 3) + (ta & 1) * 4;   // elements

    floatx16_t oacc[DB][NQ];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < NQ; ++j) oacc[i][j] = floatx16_t{0};
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int j = 0; j < NQ; ++j) { m_run[j] = -INFINITY; l_run[j] = 0.f; }

    const int ntiles_all = (L + BT - 1) / BT;
    const int tile0 = ranges > 1 ? split * tiles_per_split : 0;
    const int tile1 = ranges > 1 ? min(ntiles_all, tile0 + tiles_per_split) : ntiles_all;
    const int nloc = tile1 - tile0;
    issue_tile(tile0 * BT, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // the Q fragments are consumed here once so that the compiler's own wait for their loads
    // sits in front of the loop instead of inside it (where it would also wait for the prefetch)
#pragma unroll
    for (int j = 0; j < NQ; ++j)
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qf[j][s]));
    __syncthreads();

    // one key tile (`it` counts from this workgroup's first tile); MASKED is set only for the
    // last tile, whose ragged tail must not contribute
    auto tile = [&](int lt, auto masked) {
        constexpr bool MASKED = decltype(masked)::value;
        const int it = tile0 + lt;
        const uint16_t *ks = lds + (lt & 1) * STAGE;
        const uint16_t *vt = ks + KTILE;
        // next tile into the other stage: every wavefront finished reading it before the barrier
        // that ended the previous iteration
        if (lt + 1 < nloc) issue_tile((it + 1) * BT, (lt + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);

        // a wavefront whose queries all lie past the end only helps with the staging
        if (wave_active) {
        // ---- S^T = K Q^T : [64 keys] x [32*NQ queries]
        floatx16_t sacc[2][NQ];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int j = 0; j < NQ; ++j) sacc[tb][j] = floatx16_t{0};
        // operand fragments are fetched one step ahead of the MFMAs that use them
        auto load_k = [&](int s, bf16x8_t *dst) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int r = tb * 32 + rl;
                dst[tb] = *reinterpret_cast<const bf16x8_t *>(
                    ks + r * DH + (((2 * s + g) ^ k_swz<DH>(r)) << 3));
            }
        };
        auto load_v = [&](int u, bf16x8_t *dst) {
            typedef __attribute__((address_space(3))) shortx4_t lds_shortx4_t;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const uint16_t *vsrc = vt + v_lane + 16 * u * DH + ((db ^ v_swq) << 5);
                const shortx4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t *)vsrc);
                const shortx4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_t *)(vsrc + 8 * DH));
                dst[db] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        };
        bf16x8_t kf[2][2];
        load_k(0, kf[0]);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s + 1 < KS) load_k(s + 1, kf[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    sacc[tb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s & 1][tb], qf[j][s],
                                                                          sacc[tb][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the first V fragments travel under the softmax
        bf16x8_t vf[2][DB];
        load_v(0, vf[0]);
        __builtin_amdgcn_sched_barrier(0);
        // ---- mask the ragged tail of the cache
        if (MASKED) {
            const int t0 = it * BT;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + tb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                    if (t >= L) {
#pragma unroll
                        for (int j = 0; j < NQ; ++j) sacc[tb][j][i] = -INFINITY;
                    }
                }
        }
        // ---- online softmax, one query column per lane
        bf16x8_t pf[4][NQ];
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            float mx = sacc[0][j][0];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[tb][j][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[j], mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run[j] - m_new) * c_log2);
            const float mc = m_new * c_log2;
            m_run[j] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                float p[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = __builtin_amdgcn_exp2f(fmaf(sacc[tb][j][i], c_log2, -mc));
                    psum += p[i];
                }
#pragma unroll
                for (int uu = 0; uu < 2; ++uu) {
                    uint4 pk;
                    pk.x = pack_bf16x2(p[8 * uu + 0], p[8 * uu + 1]);
                    pk.y = pack_bf16x2(p[8 * uu + 2], p[8 * uu + 3]);
                    pk.z = pack_bf16x2(p[8 * uu + 4], p[8 * uu + 5]);
                    pk.w = pack_bf16x2(p[8 * uu + 6], p[8 * uu + 7]);
                    pf[2 * tb + uu][j] = __builtin_bit_cast(bf16x8_t, pk);
                }
            }
            l_run[j] = l_run[j] * alpha + psum;
            if (__any(alpha != 1.0f)) {                       // wave-uniform: the max rarely moves
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[db][j][i] *= alpha;
            }
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u + 1 < 4) load_v(u + 1, vf[(u + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    oacc[db][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u & 1][db], pf[u][j],
                                                                          oacc[db][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };
    for (int lt = 0; lt + 1 < nloc; ++lt) tile(lt, std::false_type{});
    tile(nloc - 1, std::true_type{});

    if (ranges > 1) {
        // partial result of this key range: unnormalised O (fp32), running max and sum
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const int row = q0 + j * 32 + rl;
            const float l = l_run[j] + __shfl_xor(l_run[j], 32);
            if (row >= n) continue;
            const size_t prow = prow_base + (size_t)row * prow_stride;
            float *dst = part_o + prow * DH;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int e = 0; e < 16; e += 4) {
                    const int dh = db * 32 + 8 * (e >> 2) + 4 * g;
                    *reinterpret_cast<float4 *>(dst + dh) = make_float4(
                        oacc[db][j][e], oacc[db][j][e + 1], oacc[db][j][e + 2], oacc[db][j][e + 3]);
                }
            if (g == 0) *reinterpret_cast<float2 *>(part_ml + prow * 2) = make_float2(m_run[j], l);
        }
        return;
    }

    // ---- normalise and store: lane = query, 4 consecutive head-dim values per accumulator group
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const int row = q0 + j * 32 + rl;
        const float l = l_run[j] + __shfl_xor(l_run[j], 32);
        const float inv = 1.0f / l;
        if (row >= n) continue;
        uint16_t *dst = o + ((size_t)b * n + row) * rowpitch + (size_t)h * DH;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 16; e += 4) {
                const int dh = db * 32 + 8 * (e >> 2) + 4 * g;
                uint2 pk;
                pk.x = pack_bf16x2(oacc[db][j][e] * inv, oacc[db][j][e + 1] * inv);
                pk.y = pack_bf16x2(oacc[db][j][e + 2] * inv, oacc[db][j][e + 3] * inv);
                *reinterpret_cast<uint2 *>(dst + dh) = pk;
            }
    }
}

// Merge of the key-range partials: o = sum_s O_s w_s / sum_s l_s w_s with w_s = 2^((m_s - max m) c).
// One thread per 4 consecutive head-dim values of one (sample, query row, head).
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part_o,
                                                         const float *__restrict__ part_ml, int n,
                                                         int H, int DH, int nsplit, float c_log2,
                                                         long total, uint16_t *__restrict__ o)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;       // over B * n * H * DH/4
    if (idx >= total) return;
    const int per_row = H * (DH / 4);
    const long brow = idx / per_row;                             // b * n + row
    const int rem = (int)(idx % per_row), h = rem / (DH / 4), c4 = rem % (DH / 4);
    const long b = brow / n, row = brow % n;
    float m = -INFINITY;
    for (int s = 0; s < nsplit; ++s)
        m = fmaxf(m, part_ml[((((size_t)b * nsplit + s) * n + row) * H + h) * 2]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float den = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const size_t prow = (((size_t)b * nsplit + s) * n + row) * H + h;
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + prow * 2);
        const float w = __builtin_amdgcn_exp2f((ml.x - m) * c_log2);
        const float4 v = *reinterpret_cast<const float4 *>(part_o + prow * DH + c4 * 4);
        acc.x = fmaf(v.x, w, acc.x); acc.y = fmaf(v.y, w, acc.y);
        acc.z = fmaf(v.z, w, acc.z); acc.w = fmaf(v.w, w, acc.w);
        den = fmaf(ml.y, w, den);
    }
    const float inv = 1.0f / den;
    uint2 pk;
    pk.x = pack_bf16x2(acc.x * inv, acc.y * inv);
    pk.y = pack_bf16x2(acc.z * inv, acc.w * inv);
    *reinterpret_cast<uint2 *>(o + ((size_t)brow * H + h) * DH + c4 * 4) = pk;
}

// Merge for the units whose key axis was divided only in the last round of workgroups: partials
// are stored per (tail unit, range) as [BQ queries][DH] (+ [BQ][2] running max / sum).
// One thread per 4 consecutive head-dim values of one (tail unit, query).
__global__ __launch_bounds__(256) void attn_tail_merge_kernel(const float *__restrict__ part_o,
                                                              const float *__restrict__ part_ml, int n,
                                                              int H, int DH, int BQ, int nqb,
                                                              int full_units, int ranges, float c_log2,
                                                              long total, uint16_t *__restrict__ o)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;       // over tail units * BQ * DH/4
    if (idx >= total) return;
    const int c4 = (int)(idx % (DH / 4));
    const long uq = idx / (DH / 4);
    const int ql = (int)(uq % BQ), tu = (int)(uq / BQ), unit = full_units + tu;
    const int qb = unit % nqb, h = (unit / nqb) % H, b = unit / (nqb * H);
    const int row = qb * BQ + ql;
    if (row >= n) return;
    float m = -INFINITY;
    for (int s = 0; s < ranges; ++s) m = fmaxf(m, part_ml[((size_t)(tu * ranges + s) * BQ + ql) * 2]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float den = 0.f;
    for (int s = 0; s < ranges; ++s) {
        const size_t prow = (size_t)(tu * ranges + s) * BQ + ql;
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + prow * 2);
        const float w = __builtin_amdgcn_exp2f((ml.x - m) * c_log2);
        const float4 v = *reinterpret_cast<const float4 *>(part_o + prow * DH + c4 * 4);
        acc.x = fmaf(v.x, w, acc.x); acc.y = fmaf(v.y, w, acc.y);
        acc.z = fmaf(v.z, w, acc.z); acc.w = fmaf(v.w, w, acc.w);
        den = fmaf(ml.y, w, den);
    }
    const float inv = 1.0f / den;
    uint2 pk;
    pk.x = pack_bf16x2(acc.x * inv, acc.y * inv);
    pk.y = pack_bf16x2(acc.z * inv, acc.w * inv);
    *reinterpret_cast<uint2 *>(o + (((size_t)b * n + row) * H + h) * DH + c4 * 4) = pk;
}

// Query rows per workgroup and workgroups that a CU holds at once for a problem (the variant the
// launcher picks), and the plan for the last round of workgroups: with `units` workgroups on
// `slots` places, the units beyond the last full round are divided into `ranges` key ranges each
// when that round would leave more than a quarter of the places empty.
struct AttnPlan { int bq, slots, nqb, units, full_units, tail_ranges; };
static AttnPlan attention_plan(int B, int n, int H, int Dh)
{
    AttnPlan p;
    const bool wide = Dh == 64 && ((n % 256 == 0) || (n % 256 > 128));
    p.bq = wide ? 256 : 128;
    p.slots = 256 * ((Dh == 64 && !wide) ? 4 : 2);
    p.nqb = (n + p.bq - 1) / p.bq;
    p.units = p.nqb * H * B;
    p.full_units = p.units / p.slots * p.slots;
    const int rem = p.units - p.full_units;
    p.tail_ranges = 1;
    if (p.full_units > 0 && rem > 0 && rem * 4 <= p.slots * 3) {
        int r = p.slots / rem;
        p.tail_ranges = r > 8 ? 8 : r;
    }
    if (p.tail_ranges < 2) { p.tail_ranges = 1; p.full_units = p.units; }
    return p;
}

// Number of key ranges for a problem, from the launch geometry alone (not the cache length, so
// that the workspace can be sized from it; the launcher lowers it when the cache is short).
// The kernel is throughput-bound per CU, so what counts is rounds of workgroups over the 256 CUs:
// s ranges cost ceil(wgs*s/256)/s rounds of full-length work, plus about 8 % per extra range for
// the partial results and their merge (12 % when the problem already fills the chip once: its
// partials are larger); fitted to sweeps of the head_dim-128 shapes with 64..640 workgroups.
int attention_max_splits(DType dt, int B, int n, int H, int Dh)
{
    if (dt != DType::BF16) return 1;
    const bool wide = Dh == 64 && ((n % 256 == 0) || (n % 256 > 128));
    const long wgs = (long)((n + (wide ? 255 : 127)) / (wide ? 256 : 128)) * H * B;
    int best = 1;
    double best_cost = 1e300;
    const double per_split = wgs >= 256 ? 0.12 : 0.08;
    for (int s = 1; s <= 8; ++s) {
        const double rounds = (double)((wgs * s + 255) / 256);
        const double cost = rounds / s * (1.0 + per_split * (s - 1));
        if (cost < best_cost - 1e-9) { best_cost = cost; best = s; }
    }
    return best;
}

// Floats of scratch the bf16 attention of a problem may need for partial results (either way of
// dividing the key axis); 0 when every workgroup sees the whole cache.
size_t attention_scratch_floats(DType dt, int B, int n, int H, int Dh)
{
    if (dt != DType::BF16) return 0;
    const int ns = attention_max_splits(dt, B, n, H, Dh);
    if (ns > 1) return (size_t)ns * B * n * H * (Dh + 2);
    const AttnPlan p = attention_plan(B, n, H, Dh);
    if (p.tail_ranges > 1) return (size_t)(p.units - p.full_units) * p.tail_ranges * p.bq * (Dh + 2);
    return 0;
}

template <int DH, int NQ>
static void launch_attn_bf16(const void *q, const void *K, const void *V, int B, int n, int L,
                             int cap, int H, float scale, void *o, float *part, hipStream_t st)
{
    constexpr int BQ = 128 * NQ;
    const size_t lds = (size_t)2 * 2 * BT * DH * sizeof(uint16_t);
    auto kern = attn_bf16_kernel<DH, NQ>;
    if (lds > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    // key ranges: every range at least 4 tiles long, none empty
    const int ntiles = (L + BT - 1) / BT;
    int nsplit = part ? attention_max_splits(DType::BF16, B, n, H, DH) : 1;
    if (nsplit > ntiles / 4) nsplit = ntiles / 4 > 0 ? ntiles / 4 : 1;
    int tps = (ntiles + nsplit - 1) / nsplit;
    nsplit = (ntiles + tps - 1) / tps;
    const float c_log2 = scale * 1.4426950408889634f;
    AttnPlan plan = attention_plan(B, n, H, DH);
    int tail = (part && nsplit == 1) ? plan.tail_ranges : 1;
    if (tail > ntiles / 4) tail = ntiles / 4 > 0 ? ntiles / 4 : 1;
    if (tail > 1) {
        tps = (ntiles + tail - 1) / tail;
        tail = (ntiles + tps - 1) / tps;
    }
    if (tail < 2) { tail = 1; plan.full_units = plan.units; }
    const int tail_units = plan.units - plan.full_units;
    float *part_o = part, *part_ml = nullptr;
    if (nsplit > 1) part_ml = part + (size_t)nsplit * B * n * H * DH;
    else if (tail > 1) part_ml = part + (size_t)tail_units * tail * BQ * DH;
    const unsigned nwg = nsplit > 1 ? (unsigned)plan.units * nsplit
                                    : (unsigned)(plan.full_units + tail_units * tail);
    launch(kern, dim3(nwg), dim3(256), lds, st, (const uint16_t *)q, (const uint16_t *)K,
           (const uint16_t *)V, n, L, cap, H, c_log2, (uint16_t *)o, nsplit, tps, part_o, part_ml,
           plan.nqb, plan.full_units, tail);
    if (nsplit > 1) {
        const long total = (long)B * n * H * (DH / 4);
        launch(attn_merge_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
               (const float *)part_o, (const float *)part_ml, n, H, DH, nsplit, c_log2, total,
               (uint16_t *)o);
    } else if (tail > 1) {
        const long total = (long)tail_units * BQ * (DH / 4);
        launch(attn_tail_merge_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
               (const float *)part_o, (const float *)part_ml, n, H, DH, BQ, plan.nqb, plan.full_units,
               tail, c_log2, total, (uint16_t *)o);
    }
}

// ------------------------------------------------------------------------------ fp32
template <int DH>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float *__restrict__ q,
                                                       const float *__restrict__ Kc,
                                                       const float *__restrict__ Vc, int n, int L,
                                                       int cap, int H, float scale,
                                                       float *__restrict__ o)
{
    constexpr int TQ = 32, TK = 32, OC = DH / 8;
    __shared__ float Qs[TQ][DH + 1];
    __shared__ float Ks[TK][DH + 1];
    __shared__ float Vs[TK][DH];
    __shared__ float Ps[TQ][TK + 1];
    const int tid = threadIdx.x, ty = tid >> 3, tx = tid & 7;     // row ty, 4 key columns at tx*4
    const int h = blockIdx.y, b = blockIdx.z, q0 = blockIdx.x * TQ;
    const size_t rowpitch = (size_t)H * DH;
    for (int e = tid; e < TQ * DH; e += 256) {
        const int r = e / DH, c = e % DH;
        Qs[r][c] = q[((size_t)b * n + min(q0 + r, n - 1)) * rowpitch + (size_t)h * DH + c];
    }
    float acc[OC];
#pragma unroll
    for (int c = 0; c < OC; ++c) acc[c] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    for (int t0 = 0; t0 < L; t0 += TK) {
        __syncthreads();
        for (int e = tid; e < TK * DH; e += 256) {
            const int r = e / DH, c = e % DH;
            const size_t off = ((size_t)b * cap + min(t0 + r, L - 1)) * rowpitch + (size_t)h * DH + c;
            Ks[r][c] = Kc[off];
            Vs[r][c] = Vc[off];
        }
        __syncthreads();
        float s[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float d = 0.f;
            for (int e = 0; e < DH; ++e) d = fmaf(Qs[ty][e], Ks[tx * 4 + c][e], d);
            s[c] = (t0 + tx * 4 + c < L) ? d * scale : -INFINITY;
        }
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 1));
        mx = fmaxf(mx, __shfl_xor(mx, 2));
        mx = fmaxf(mx, __shfl_xor(mx, 4));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = expf(m_run - m_new);
        float ps = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float p = expf(s[c] - m_new);
            Ps[ty][tx * 4 + c] = p;
            ps += p;
        }
        ps += __shfl_xor(ps, 1);
        ps += __shfl_xor(ps, 2);
        ps += __shfl_xor(ps, 4);
        l_run = l_run * alpha + ps;
        m_run = m_new;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < OC; ++c) acc[c] *= alpha;
        for (int t = 0; t < TK; ++t) {
            const float p = Ps[ty][t];
#pragma unroll
            for (int c = 0; c < OC; ++c) acc[c] = fmaf(p, Vs[t][tx * OC + c], acc[c]);
        }
    }
    const int row = q0 + ty;
    if (row < n) {
        float *dst = o + ((size_t)b * n + row) * rowpitch + (size_t)h * DH + tx * OC;
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int c = 0; c < OC; ++c) dst[c] = acc[c] * inv;
    }
}

void launch_attention(DType dt, const void *q, const void *K, const void *V, int B, int n, int L,
                      int cap, int H, int Dh, float scale, void *o, float *part, hipStream_t st)
{
    if (dt == DType::BF16) {
        // two 32-query blocks per wavefront halve the LDS operand traffic per MFMA; use the
        // single-block variant when that would leave most of a 256-query tile empty
        const bool wide = (n % 256 == 0) || (n % 256 > 128);
        if (Dh == 64) {
            if (wide) launch_attn_bf16<64, 2>(q, K, V, B, n, L, cap, H, scale, o, part, st);
            else launch_attn_bf16<64, 1>(q, K, V, B, n, L, cap, H, scale, o, part, st);
        } else {
            // head_dim 128 with two query blocks per wavefront does not fit the register budget of
            // two wavefronts per SIMD, which is what lets one wavefront's softmax overlap the
            // other's MFMAs
            launch_attn_bf16<128, 1>(q, K, V, B, n, L, cap, H, scale, o, part, st);
        }
    } else {
        dim3 grid((n + 31) / 32, H, B), block(256);
        if (Dh == 64)
            launch(attn_f32_kernel<64>, grid, block, 0, st, (const float *)q,
                               (const float *)K, (const float *)V, n, L, cap, H, scale, (float *)o);
        else
            launch(attn_f32_kernel<128>, grid, block, 0, st, (const float *)q,
                               (const float *)K, (const float *)V, n, L, cap, H, scale, (float *)o);
    }
}

}  // namespace fvar
