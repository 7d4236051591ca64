// Representative-token scoring and selection (paper, Sec. "Representative Token Restoration").
//
//   score   s_i = fl32(sum_j x_ij^2): one wavefront per token row, 16-byte loads, products and
//           the sum carried in fp64 (exact products; the order of the adds then changes the
//           stored fp32 value only in double-rounding corner cases), butterfly reduction.
//   select  one workgroup per sample: MSB-first radix select (4 passes of 8 bits) over the
//           order-preserving integer image of the scores held in LDS, which yields the k-th
//           largest key T and how many keys equal to T are still needed; then one ordered
//           sweep over the indices with block-wide prefix sums writes the kept and the pruned
//           indices, each ascending.  Ties at T go to the lower index.  No atomics touch the
//           outputs, so the result is deterministic.
#include "common.h"

namespace fvar {

template <typename T>
__global__ __launch_bounds__(256) void scores_kernel(const T *__restrict__ x, int rows, int d,
                                                     float *__restrict__ scores)
{
    constexpr int E = Elem<T>::kPerChunk;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= rows) return;
    const uint4 *src = reinterpret_cast<const uint4 *>(x + (size_t)row * d);
    const int nchunk = d / E;
    double acc0 = 0.0, acc1 = 0.0;
    int c = lane;
    // four chunks in flight per lane
    for (; c + 192 < nchunk; c += 256) {
        uint4 v0 = src[c], v1 = src[c + 64], v2 = src[c + 128], v3 = src[c + 192];
        float f[E];
        Elem<T>::unpack(v0, f);
#pragma unroll
        for (int e = 0; e < E; ++e) acc0 = fma((double)f[e], (double)f[e], acc0);
        Elem<T>::unpack(v1, f);
#pragma unroll
        for (int e = 0; e < E; ++e) acc1 = fma((double)f[e], (double)f[e], acc1);
        Elem<T>::unpack(v2, f);
#pragma unroll
        for (int e = 0; e < E; ++e) acc0 = fma((double)f[e], (double)f[e], acc0);
        Elem<T>::unpack(v3, f);
#pragma unroll
        for (int e = 0; e < E; ++e) acc1 = fma((double)f[e], (double)f[e], acc1);
    }
    for (; c < nchunk; c += 64) {
        uint4 v0 = src[c];
        float f[E];
        Elem<T>::unpack(v0, f);
#pragma unroll
        for (int e = 0; e < E; ++e) acc0 = fma((double)f[e], (double)f[e], acc0);
    }
    double acc = wave_sum(acc0 + acc1);
    if (lane == 0) scores[row] = (float)acc;
}

void launch_scores(DType dt, const void *x, int rows, int d, float *scores, hipStream_t st)
{
    dim3 grid((rows + 3) / 4), block(256);
    if (dt == DType::BF16)
        launch(scores_kernel<uint16_t>, grid, block, 0, st, (const uint16_t *)x, rows, d,
                           scores);
    else
        launch(scores_kernel<float>, grid, block, 0, st, (const float *)x, rows, d,
                           scores);
}

// Order-preserving map float -> uint32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// exclusive prefix sum of a 0/1 flag over the workgroup, in thread order; `total` = block sum
__device__ __forceinline__ int block_excl_scan_flag(bool flag, int *wave_tot, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long m = __ballot(flag);
    int in_wave = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(m);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        int t = wave_tot[w];
        before += (w < wave) ? t : 0;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return before + in_wave;
}

template <bool KEYS_IN_LDS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float *__restrict__ scores, int M,
                                                             int k, int32_t *__restrict__ idx_keep,
                                                             int32_t *__restrict__ idx_drop)
{
    extern __shared__ uint32_t lds_keys[];
    __shared__ int hist[256];
    __shared__ int wave_tot[kSelWaves];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_remaining;

    const int b = blockIdx.x;
    const float *s = scores + (size_t)b * M;
    const int tid = threadIdx.x;

    auto key_at = [&](int i) -> uint32_t {
        if constexpr (KEYS_IN_LDS) return lds_keys[i];
        else return score_key(s[i]);
    };

    if constexpr (KEYS_IN_LDS) {
        for (int i = tid; i < M; i += kSelThreads) lds_keys[i] = score_key(s[i]);
    }
    if (tid == 0) { sh_prefix = 0u; sh_remaining = k; }

    // ---- radix select of the k-th largest key
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh_prefix;
        const int remaining = sh_remaining;
        // keys whose already-fixed high bits equal the prefix
        const uint32_t himask = (pass == 0) ? 0u : (0xffffffffu << (shift + 8));
        for (int i = tid; i < M; i += kSelThreads) {
            uint32_t key = key_at(i);
            if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 0xffu], 1);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins 255-4l .. 252-4l (descending); `above` = keys in higher bins
            int c[4], sum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { c[j] = hist[255 - 4 * tid - j]; sum += c[j]; }
            int incl = sum;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                int t = __shfl_up(incl, o);
                if (tid >= o) incl += t;
            }
            int run = incl - sum;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (run < remaining && remaining <= run + c[j]) {
                    sh_prefix = prefix | ((uint32_t)(255 - 4 * tid - j) << shift);
                    sh_remaining = remaining - run;
                }
                run += c[j];
            }
        }
        __syncthreads();
    }
    const uint32_t T = sh_prefix;      // k-th largest key
    const int need_eq = sh_remaining;  // how many keys == T are kept (the lowest indices)

    // ---- ordered sweep: stable compaction of kept and pruned indices
    int run_eq = 0, run_keep = 0;
    int32_t *keep_out = idx_keep + (size_t)b * k;
    int32_t *drop_out = idx_drop ? idx_drop + (size_t)b * (M - k) : nullptr;
    for (int base = 0; base < M; base += kSelThreads) {
        const int i = base + tid;
        const bool valid = i < M;
        const uint32_t key = valid ? key_at(i) : 0u;
        const bool eq = valid && key == T;
        const bool gt = valid && key > T;
        int tot_eq, tot_keep;
        const int eq_rank = run_eq + block_excl_scan_flag(eq, wave_tot, tot_eq);
        const bool keep = gt || (eq && eq_rank < need_eq);
        const int keep_pos = run_keep + block_excl_scan_flag(keep, wave_tot, tot_keep);
        if (valid) {
            if (keep) keep_out[keep_pos] = i;
            else if (drop_out) drop_out[i - keep_pos] = i;
        }
        run_eq += tot_eq;
        run_keep += tot_keep;
    }
}

void launch_select(const float *scores, int B, int M, int k, int32_t *idx_keep, int32_t *idx_drop,
                   hipStream_t st)
{
    dim3 grid(B), block(kSelThreads);
    if (M <= 12288) {
        launch(select_kernel<true>, grid, block, (size_t)M * sizeof(uint32_t), st, scores,
                           M, k, idx_keep, idx_drop);
    } else {
        launch(select_kernel<false>, grid, block, 0, st, scores, M, k, idx_keep,
                           idx_drop);
    }
}

}  // namespace fvar
