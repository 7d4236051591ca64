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
//   * K tiles go to LDS row-major (swizzled 16 B chunks).  V tiles are transposed on their way
//     into LDS with a register 4x8 transpose (v_perm_b32), stored [Dh][t'] where t' orders the
//     keys the way the accumulator layout hands out P, so the V^T operand is one ds_read_b128.
//   * global -> register prefetch of the next K/V tile overlaps the MFMAs of the current one;
//     LDS is double buffered, one barrier per tile.
//
// fp32 kernel: plain tiled FMA version for the fp32 parity configuration.
#include <type_traits>

#include "common.h"

namespace fvar {

constexpr int BT = 64;                       // keys per tile

typedef int intx4_t __attribute__((ext_vector_type(4)));

// 16-byte global load whose position in the instruction stream is fixed.  The compiler does not
// count this load: the destination must be kept alive and unread until an explicit
// s_waitcnt vmcnt that the later uses are tied to (see wait_tile below).
__device__ __forceinline__ intx4_t global_load_b128(const void *base, uint32_t byte_off)
{
    intx4_t v;
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(v) : "v"(byte_off), "s"(base) : "memory");
    return v;
}

// Chunk swizzle of the V^T tile (rows = head-dim index, 8 chunks of 8 keys).  Readers fetch 16
// consecutive rows at one logical chunk: (row/2)%8 makes those 16 accesses cover all 64 banks
// once, and the extra term is constant inside an aligned group of 16 rows, so it keeps that.
// Writers store 8-byte halves to rows 8 apart (one per 8-column block of the transposed 4x8
// blocks): the extra term, a function of row/16, spreads those rows over different chunks.
__device__ __forceinline__ int vt_swz(int row)
{
    return ((row >> 1) & 7) ^ (((row >> 4) & 1) << 2) ^ ((row >> 5) & 3);
}

template <int DH, int NQ>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(const uint16_t *__restrict__ q,
                                                        const uint16_t *__restrict__ Kc,
                                                        const uint16_t *__restrict__ Vc, int n, int L,
                                                        int cap, int H, float c_log2,
                                                        uint16_t *__restrict__ o, int nsplit,
                                                        int tiles_per_split,
                                                        float *__restrict__ part_o,
                                                        float *__restrict__ part_ml)
{
    constexpr int KS = DH / 16;              // k16 steps of the QK product
    constexpr int DB = DH / 32;              // 32-row blocks of O^T
    constexpr int KCH = DH / 8;              // 16 B chunks per K row
    constexpr int LK = BT * KCH / 256;       // K chunks per thread per tile
    constexpr int VBLK = (BT / 4) * (DH / 8);        // 4x8 transpose blocks per V tile
    constexpr int LV = (VBLK + 255) / 256;       // V blocks per thread
    constexpr int KTILE = BT * DH, STAGE = 2 * KTILE;

    extern __shared__ uint4 lds_raw[];
    uint16_t *lds = reinterpret_cast<uint16_t *>(lds_raw);   // [stage][K tile | V^T tile]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rl = lane & 31, g = lane >> 5;
    // blockIdx.z = sample * nsplit + split: with nsplit > 1 this workgroup sees only the key tiles
    // [tile0, tile1) and leaves an unnormalised partial result for the merge kernel
    const int h = blockIdx.y, b = blockIdx.z / nsplit, split = blockIdx.z % nsplit;
    const int q0 = blockIdx.x * (128 * NQ) + wave * (32 * NQ);
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

    // ---- staging assignment
    int k_row[LK], k_chk[LK];
#pragma unroll
    for (int i = 0; i < LK; ++i) {
        const int id = tid + 256 * i;
        k_row[i] = id / KCH;
        k_chk[i] = id % KCH;
    }
    // V block: 4 key rows x 8 head-dim columns.  tb4 = 2*chunk + half; chunk = 2*w + gg covers
    // keys 16w + 8a + 4gg + jj (a = half, jj = 0..3): the order in which a lane's accumulator
    // entries enumerate the keys of a 16-key MFMA step.
    // When the tile has fewer blocks than threads (head_dim 64) the upper threads repeat the
    // lower ones' blocks: same loads, same LDS stores, no divergence.
    int v_t0[LV], v_col[LV], v_dst[LV];
#pragma unroll
    for (int i = 0; i < LV; ++i) {
        const int blk = (tid + 256 * i) % VBLK;
        const int cb = blk % (DH / 8), tb4 = blk / (DH / 8);
        const int chunk = tb4 >> 1, a = tb4 & 1, w = chunk >> 1, gg = chunk & 1;
        v_t0[i] = 16 * w + 8 * a + 4 * gg;
        v_col[i] = cb * 8;
        v_dst[i] = chunk * 8 + a * 4;        // element offset inside an unswizzled V^T row
    }

    // The tile loads are issued through asm so that they stay where they are written (the
    // compiler would sink them next to the LDS stores); their registers are read only after the
    // explicit vmcnt wait further down the same straight-line block.
    intx4_t kreg[LK];
    intx4_t vreg[LV][4];
    // byte offsets of this thread's chunks inside a tile that lies wholly inside the cache: such a
    // tile is fetched as (uniform tile base) + (these constants); only a tile that reaches past
    // row L-1 pays for the per-row clamp
    uint32_t k_off[LK], v_off[LV][4];
#pragma unroll
    for (int i = 0; i < LK; ++i) k_off[i] = (uint32_t)(((size_t)k_row[i] * rowpitch + k_chk[i] * 8) * 2);
#pragma unroll
    for (int i = 0; i < LV; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            v_off[i][jj] = (uint32_t)(((size_t)(v_t0[i] + jj) * rowpitch + v_col[i]) * 2);
    auto load_tile = [&](int t0) {
        if (t0 + BT <= L) {                                  // uniform
            const uint16_t *kt = Kb + (size_t)t0 * rowpitch, *vtile = Vb + (size_t)t0 * rowpitch;
#pragma unroll
            for (int i = 0; i < LK; ++i) kreg[i] = global_load_b128(kt, k_off[i]);
#pragma unroll
            for (int i = 0; i < LV; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) vreg[i][jj] = global_load_b128(vtile, v_off[i][jj]);
            return;
        }
#pragma unroll
        for (int i = 0; i < LK; ++i) {
            const int t = min(t0 + k_row[i], L - 1);
            kreg[i] = global_load_b128(Kb, (uint32_t)(((size_t)t * rowpitch + k_chk[i] * 8) * 2));
        }
#pragma unroll
        for (int i = 0; i < LV; ++i) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int t = min(t0 + v_t0[i] + jj, L - 1);
                vreg[i][jj] = global_load_b128(Vb, (uint32_t)(((size_t)t * rowpitch + v_col[i]) * 2));
            }
        }
    };
    // Wait for the asm loads and make every later use of the staging registers depend on that
    // wait: the empty asm statements "redefine" the registers, so neither the ALU work of the
    // transpose nor a reuse of the registers can be scheduled while the loads are in flight.
    auto wait_tile = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int i = 0; i < LK; ++i) asm volatile("" : "+v"(kreg[i]));
#pragma unroll
        for (int i = 0; i < LV; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) asm volatile("" : "+v"(vreg[i][jj]));
    };
    // Lanes of odd column blocks store the odd row of each row pair first, so that one store
    // instruction touches rows of both parities (both halves of the 64 banks); which half of the
    // byte permute goes first is folded into per-thread selector constants.
    uint32_t v_sel[LV][2];
#pragma unroll
    for (int i = 0; i < LV; ++i) {
        const bool flip = (v_col[i] >> 3) & 1;
        v_sel[i][0] = flip ? 0x07060302u : 0x05040100u;
        v_sel[i][1] = flip ? 0x05040100u : 0x07060302u;
    }
    auto store_tile = [&](uint16_t *st) {
#pragma unroll
        for (int i = 0; i < LK; ++i)
            *reinterpret_cast<intx4_t *>(st + k_row[i] * DH + ((k_chk[i] ^ ((k_row[i] >> 1) & 7)) << 3)) =
                kreg[i];
        uint16_t *vt = st + KTILE;
#pragma unroll
        for (int i = 0; i < LV; ++i) {
            const int chunk = v_dst[i] >> 3, sub = v_dst[i] & 7;
            const int par = (v_col[i] >> 3) & 1;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                uint2 first, second;
                first.x = __builtin_amdgcn_perm(vreg[i][1][m], vreg[i][0][m], v_sel[i][0]);
                first.y = __builtin_amdgcn_perm(vreg[i][3][m], vreg[i][2][m], v_sel[i][0]);
                second.x = __builtin_amdgcn_perm(vreg[i][1][m], vreg[i][0][m], v_sel[i][1]);
                second.y = __builtin_amdgcn_perm(vreg[i][3][m], vreg[i][2][m], v_sel[i][1]);
                const int ra = v_col[i] + 2 * m + par, rb = v_col[i] + 2 * m + (par ^ 1);
                *reinterpret_cast<uint2 *>(vt + ra * BT + ((chunk ^ vt_swz(ra)) << 3) + sub) = first;
                *reinterpret_cast<uint2 *>(vt + rb * BT + ((chunk ^ vt_swz(rb)) << 3) + sub) = second;
            }
        }
    };

    floatx16_t oacc[DB][NQ];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < NQ; ++j) oacc[i][j] = floatx16_t{0};
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int j = 0; j < NQ; ++j) { m_run[j] = -INFINITY; l_run[j] = 0.f; }

    const int tile0 = split * tiles_per_split;
    const int tile1 = min((L + BT - 1) / BT, tile0 + tiles_per_split);
    load_tile(tile0 * BT);
    wait_tile();
    store_tile(lds);
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
        // next tile (row indices are clamped, so the request past the end is harmless)
        load_tile((it + 1) * BT);
        __builtin_amdgcn_sched_barrier(0);

        // a wavefront whose queries all lie past the end only helps with the staging
        if (wave_active) {
        // ---- S^T = K Q^T : [64 keys] x [32*NQ queries]
        floatx16_t sacc[2][NQ];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int j = 0; j < NQ; ++j) sacc[tb][j] = floatx16_t{0};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int r = tb * 32 + rl;
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(
                    ks + r * DH + (((2 * s + g) ^ ((r >> 1) & 7)) << 3));
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    sacc[tb][j] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[j][s], sacc[tb][j], 0, 0, 0);
            }
        }
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
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const int dr = db * 32 + rl;
                const bf16x8_t vf = *reinterpret_cast<const bf16x8_t *>(
                    vt + dr * BT + (((2 * u + g) ^ vt_swz(dr)) << 3));
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    oacc[db][j] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u][j], oacc[db][j], 0, 0, 0);
            }
        }
        }
        wait_tile();
        store_tile(lds + ((lt + 1) & 1) * STAGE);
        __syncthreads();
    };
    const int nloc = tile1 - tile0;
    for (int lt = 0; lt + 1 < nloc; ++lt) tile(lt, std::false_type{});
    tile(nloc - 1, std::true_type{});

    if (nsplit > 1) {
        // partial result of this key range: unnormalised O (fp32), running max and sum
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const int row = q0 + j * 32 + rl;
            const float l = l_run[j] + __shfl_xor(l_run[j], 32);
            if (row >= n) continue;
            const size_t prow = ((size_t)(b * nsplit + split) * n + row) * H + h;
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
    float *part_o = part;
    float *part_ml = part ? part + (size_t)nsplit * B * n * H * DH : nullptr;
    dim3 grid((n + BQ - 1) / BQ, H, B * nsplit), block(256);
    launch(kern, grid, block, lds, st, (const uint16_t *)q, (const uint16_t *)K,
                       (const uint16_t *)V, n, L, cap, H, c_log2, (uint16_t *)o, nsplit, tps, part_o,
                       part_ml);
    if (nsplit > 1) {
        const long total = (long)B * n * H * (DH / 4);
        launch(attn_merge_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
               (const float *)part_o, (const float *)part_ml, n, H, DH, nsplit, c_log2, total,
               (uint16_t *)o);
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
