// V-Major selection as the paper states it (Section III-D): a per-token scalar (L1 distance between the
// token's current and cached value vector), the fraction r with the smallest distance stays cached, the other
// tokens are active; r comes from the time-varying cache schedule (warm-up, linear ramp, periodic full update).
//
//   token_metric_kernel -- one wavefront per token streams the token's value vector from both tensors once
//                          (HBM-bound), fp32 sum of |cur - prev| per lane, wavefront tree reduction;
//   topk_kernel         -- one workgroup per segment (a logical rank's tokens), keys cached in LDS: 4-pass radix
//                          select (8 bits per pass, LDS histogram) of the K-th largest key, then an
//                          index-ordered compaction that takes every token above the threshold and the
//                          lowest-indexed tokens equal to it until K are taken.
#include "internal.h"

namespace cocodiff {

constexpr int kMetricWaves = 4;
constexpr int kMetricUnroll = 6;

// metric[n] = sum over slabs s and w of |cur[s][n][w] - prev[s][n][w]|
template <bool NT_CUR, bool NT_PREV>
__global__ void __launch_bounds__(64 * kMetricWaves) token_metric_kernel(const vec16* __restrict__ cur, const vec16* __restrict__ prev,
                                                                         float* __restrict__ metric, uint32_t S, uint32_t N, uint32_t W8) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t n = blockIdx.x * kMetricWaves + (threadIdx.x >> 6);
    if (n >= N) return;
    const uint32_t total = S * W8;
    float acc = 0.f;
    for (uint32_t g0 = lane; g0 < total; g0 += 64 * kMetricUnroll) {
        vec16 c[kMetricUnroll], p[kMetricUnroll];
#pragma unroll
        for (int k = 0; k < kMetricUnroll; ++k) {
            const uint32_t g = g0 + 64 * k;
            if (g < total) {
                const uint32_t s = g / W8, v = g - s * W8;
                const uint64_t at = ((uint64_t)s * N + n) * W8 + v;
                c[k] = ld_vec<NT_CUR>(cur + at);
                p[k] = ld_vec<NT_PREV>(prev + at);
            }
        }
#pragma unroll
        for (int k = 0; k < kMetricUnroll; ++k) {
            if (g0 + 64 * k < total) {
                const uint32_t cw[4] = {c[k].x, c[k].y, c[k].z, c[k].w};
                const uint32_t pw[4] = {p[k].x, p[k].y, p[k].z, p[k].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc += fabsf(bf16_lo(cw[i]) - bf16_lo(pw[i]));
                    acc += fabsf(bf16_hi(cw[i]) - bf16_hi(pw[i]));
                }
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) metric[n] = acc;
}

// Order-preserving key: larger metric <-> larger key; every NaN maps to the largest key; -0 and +0 share one.
__device__ __forceinline__ uint32_t metric_key(float m) {
    if (m != m) return 0xFFFFFFFFu;
    const uint32_t b = m == 0.f ? 0u : __float_as_uint(m);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kTopkThreads = 1024;
constexpr uint32_t kTopkCachedKeys = 32768;   // keys of one segment kept in LDS (128 KB) when they fit

// Exclusive prefix sum of `v` over the workgroup in thread order; `total` gets the workgroup's sum.
__device__ __forceinline__ uint32_t block_scan(uint32_t v, uint32_t* wave_tot, uint32_t& total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, 64);
        if (lane >= (uint32_t)off) incl += up;
    }
    __syncthreads();                               // wave_tot may still be read from the previous call
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kTopkThreads / 64; ++w) {
        const uint32_t c = wave_tot[w];
        before += (uint32_t)w < wave ? c : 0u;
        tot += c;
    }
    total = tot;
    return before + incl - v;
}

// One workgroup per segment (a logical rank's tokens).  CACHED: the segment's keys sit in LDS after one read of
// the metric; otherwise every pass reads the metric again (L2-resident).
template <bool CACHED>
__global__ void __launch_bounds__(kTopkThreads) topk_kernel(const float* __restrict__ metric, uint32_t N, uint32_t K,
                                                            int32_t* __restrict__ idx, int32_t* __restrict__ n_active,
                                                            uint32_t id_stride) {
    extern __shared__ uint32_t s_keys[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_tot[kTopkThreads / 64];
    __shared__ uint32_t s_prefix, s_remaining;
    metric += (size_t)blockIdx.x * N;
    idx += (size_t)blockIdx.x * N;
    const uint32_t id_base = blockIdx.x * id_stride;   // 0: ids local to the segment; N: ids in the whole metric array
    if (threadIdx.x == 0) n_active[blockIdx.x] = (int32_t)K;
    if (K == 0) return;
    if (CACHED) {
        for (uint32_t n = threadIdx.x; n < N; n += kTopkThreads) s_keys[n] = metric_key(metric[n]);
        __syncthreads();
    }
    auto key_at = [&](uint32_t n) { return CACHED ? s_keys[n] : metric_key(metric[n]); };
    // ---- the K-th largest key, one byte per pass from the top
    uint32_t prefix = 0, mask = 0, remaining = K;
    for (int pass = 3; pass >= 0; --pass) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        for (uint32_t n = threadIdx.x; n < N; n += kTopkThreads) {
            const uint32_t key = key_at(n);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        // bin of the `remaining`-th largest key: thread t looks at bin 255 - t; `above` = keys in higher bins
        const uint32_t mine = threadIdx.x < 256 ? hist[255 - threadIdx.x] : 0u;
        uint32_t in_play;
        const uint32_t above = block_scan(mine, wave_tot, in_play);
        if (above < remaining && above + mine >= remaining) {      // exactly one thread: 1 <= remaining <= in_play
            s_prefix = prefix | ((255u - threadIdx.x) << (8 * pass));
            s_remaining = remaining - above;       // how many keys of this bin (and, at the end, of this value) to take
        }
        __syncthreads();
        prefix = s_prefix;
        remaining = s_remaining;
        mask |= 0xFFu << (8 * pass);
        __syncthreads();
    }
    const uint32_t thr = prefix;                   // key of the K-th largest; `remaining` tokens equal to it are taken
    // ---- compaction in index order: thread t owns the contiguous run [t*per, (t+1)*per)
    const uint32_t per = (N + kTopkThreads - 1) / kTopkThreads;
    const uint32_t lo = threadIdx.x * per < N ? threadIdx.x * per : N;
    const uint32_t hi = lo + per < N ? lo + per : N;
    uint32_t n_gt = 0, n_eq = 0;
    for (uint32_t n = lo; n < hi; ++n) {
        const uint32_t key = key_at(n);
        n_gt += key > thr;
        n_eq += key == thr;
    }
    uint32_t eq_total, take_total;
    uint32_t eq_rank = block_scan(n_eq, wave_tot, eq_total);          // equal keys before this run
    const uint32_t eq_room = eq_rank < remaining ? remaining - eq_rank : 0u;
    const uint32_t n_take = n_gt + (n_eq < eq_room ? n_eq : eq_room);
    uint32_t pos = block_scan(n_take, wave_tot, take_total);
    for (uint32_t n = lo; n < hi; ++n) {
        const uint32_t key = key_at(n);
        const bool take = key > thr || (key == thr && eq_rank < remaining);
        eq_rank += key == thr;
        if (take) idx[pos++] = (int32_t)(id_base + n);
    }
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" int cocodiff_vmajor_token_metric(int32_t S, int32_t N, int32_t W, const cocodiff_bf16* v_cur,
                                            const cocodiff_bf16* v_prev, float* metric, void* stream) {
    if (S <= 0 || N <= 0 || W <= 0) return fail(COCODIFF_ERR_SHAPE, "token_metric: S, N, W must be positive");
    if (W % 8) return fail(COCODIFF_ERR_SHAPE, "token_metric: W (%d) must be a multiple of 8", W);
    if ((int64_t)S * (W / 8) >= ((int64_t)1 << 31)) return fail(COCODIFF_ERR_SHAPE, "token_metric: value vector too long");
    if (!v_cur || !v_prev || !metric) return fail(COCODIFF_ERR_NULL, "token_metric: NULL pointer");
    if (!aligned16(v_cur) || !aligned16(v_prev)) return fail(COCODIFF_ERR_ALIGN, "token_metric: tensors must be 16-byte aligned");
    const dim3 grid(((uint32_t)N + kMetricWaves - 1) / kMetricWaves), block(64 * kMetricWaves);
    const size_t touched = (size_t)S * N * W * 4;
    with_policy(stream_loads(touched), stream_loads_once(touched), [&](auto C, auto Pv) {
        hipLaunchKernelGGL((token_metric_kernel<decltype(C)::value, decltype(Pv)::value>), grid, block, 0, as_stream(stream),
                           (const vec16*)v_cur, (const vec16*)v_prev, metric, (uint32_t)S, (uint32_t)N, (uint32_t)(W / 8));
    });
    return check_launch("token_metric_kernel");
}

extern "C" int cocodiff_vmajor_topk(int32_t n_seg, int32_t N, const float* metric, int32_t n_keep, int32_t global_ids,
                                    int32_t* active_idx, int32_t* n_active, void* stream) {
    if (n_seg <= 0 || N <= 0) return fail(COCODIFF_ERR_SHAPE, "topk: n_seg and N must be positive");
    if ((int64_t)n_seg * N >= ((int64_t)1 << 31)) return fail(COCODIFF_ERR_SHAPE, "topk: n_seg * N must be below 2^31");
    if (n_keep < 0 || n_keep > N) return fail(COCODIFF_ERR_SHAPE, "topk: n_keep (%d) must be in [0, N = %d]", n_keep, N);
    if (!metric || !active_idx || !n_active) return fail(COCODIFF_ERR_NULL, "topk: NULL pointer");
    if ((uint32_t)N <= kTopkCachedKeys) {
        static int lds_ok = [] {
            return (int)hipFuncSetAttribute((const void*)topk_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)(kTopkCachedKeys * sizeof(uint32_t)));
        }();
        if (lds_ok != (int)hipSuccess) return fail(COCODIFF_ERR_HIP, "topk: cannot raise the kernel's LDS limit");
        hipLaunchKernelGGL(topk_kernel<true>, dim3(n_seg), dim3(kTopkThreads), (size_t)N * sizeof(uint32_t), as_stream(stream),
                           metric, (uint32_t)N, (uint32_t)n_keep, active_idx, n_active, global_ids ? (uint32_t)N : 0u);
    } else {
        hipLaunchKernelGGL(topk_kernel<false>, dim3(n_seg), dim3(kTopkThreads), 0, as_stream(stream), metric, (uint32_t)N,
                           (uint32_t)n_keep, active_idx, n_active, global_ids ? (uint32_t)N : 0u);
    }
    return check_launch("topk_kernel");
}

extern "C" int32_t cocodiff_cache_active_count(int32_t step, int32_t n_steps, int32_t warmup, int32_t sync_every,
                                               int32_t n_tokens) {
    if (n_tokens <= 0 || step < 1 || n_steps < 1 || warmup < 0) return -1;
    if (step <= warmup || n_steps <= warmup || (sync_every > 0 && step % sync_every == 0)) return n_tokens;   // full exchange
    const int64_t cached = (int64_t)n_tokens * (step - warmup) / (n_steps - warmup);   // floor(r * n_tokens), r = linear ramp
    return (int32_t)(n_tokens - (cached > n_tokens ? n_tokens : cached));
}
