// V-Major selection as the paper states it (Section III-D): a per-token scalar (L1 distance between the
// token's current and cached value vector), the fraction r with the smallest distance stays cached, the other
// tokens are active; r comes from the time-varying cache schedule (warm-up, linear ramp, periodic full update).
//
//   token_metric_kernel -- one wavefront per token streams the token's value vector from both tensors once
//                          (HBM-bound), fp32 sum of |cur - prev| per lane, wavefront tree reduction;
//   topk_kernel         -- one workgroup: 4-pass radix select (8 bits per pass, LDS histogram) of the K-th
//                          largest key, then an index-ordered compaction that takes every token above the
//                          threshold and the lowest-indexed tokens equal to it until K are taken.
#include "internal.h"

namespace cocodiff {

constexpr int kMetricWaves = 4;
constexpr int kMetricUnroll = 6;

// metric[n] = sum over slabs s and w of |cur[s][n][w] - prev[s][n][w]|
template <bool STREAM>
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
                c[k] = ld_vec<STREAM>(cur + at);
                p[k] = ld_vec<STREAM>(prev + at);
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

// Exclusive prefix count of `flag` over the workgroup; `total` gets the workgroup's count.
__device__ __forceinline__ uint32_t block_prefix(bool flag, uint32_t* wave_tot, uint32_t& total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t ball = __ballot(flag);
    const uint32_t below = __popcll(ball & ((1ull << lane) - 1ull));
    __syncthreads();                               // wave_tot may still be read from the previous call
    if (lane == 0) wave_tot[wave] = __popcll(ball);
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kTopkThreads / 64; ++w) {
        const uint32_t c = wave_tot[w];
        before += (uint32_t)w < wave ? c : 0u;
        tot += c;
    }
    total = tot;
    return before + below;
}

__global__ void __launch_bounds__(kTopkThreads) topk_kernel(const float* __restrict__ metric, uint32_t N, uint32_t K,
                                                            int32_t* __restrict__ idx, int32_t* __restrict__ n_active) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_tot[kTopkThreads / 64];
    __shared__ uint32_t s_prefix, s_remaining;
    if (threadIdx.x == 0) *n_active = (int32_t)K;
    if (K == 0) return;
    // ---- the K-th largest key, one byte per pass from the top
    uint32_t prefix = 0, mask = 0, remaining = K;
    for (int pass = 3; pass >= 0; --pass) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        for (uint32_t n = threadIdx.x; n < N; n += kTopkThreads) {
            const uint32_t key = metric_key(metric[n]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t cum = 0;
            int b = 255;
            for (; b > 0; --b) {
                if (cum + hist[b] >= remaining) break;
                cum += hist[b];
            }
            s_prefix = prefix | ((uint32_t)b << (8 * pass));
            s_remaining = remaining - cum;         // how many keys of this bin (and, at the end, of this value) to take
        }
        __syncthreads();
        prefix = s_prefix;
        remaining = s_remaining;
        mask |= 0xFFu << (8 * pass);
        __syncthreads();
    }
    const uint32_t thr = prefix;                   // key of the K-th largest; `remaining` tokens equal to it are taken
    // ---- compaction in index order
    uint32_t out_before = 0, eq_before = 0;
    for (uint32_t base = 0; base < N; base += kTopkThreads) {
        const uint32_t n = base + threadIdx.x;
        const uint32_t key = n < N ? metric_key(metric[n]) : 0u;
        const bool gt = n < N && key > thr;
        const bool eq = n < N && key == thr;
        uint32_t eq_total, take_total;
        const uint32_t eq_rank = eq_before + block_prefix(eq, wave_tot, eq_total);
        const bool take = gt || (eq && eq_rank < remaining);
        const uint32_t pos = out_before + block_prefix(take, wave_tot, take_total);
        if (take) idx[pos] = (int32_t)n;
        eq_before += eq_total;
        out_before += take_total;
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
    if (should_stream((size_t)S * N * W * 4))
        hipLaunchKernelGGL(token_metric_kernel<true>, grid, block, 0, as_stream(stream), (const vec16*)v_cur,
                           (const vec16*)v_prev, metric, (uint32_t)S, (uint32_t)N, (uint32_t)(W / 8));
    else
        hipLaunchKernelGGL(token_metric_kernel<false>, grid, block, 0, as_stream(stream), (const vec16*)v_cur,
                           (const vec16*)v_prev, metric, (uint32_t)S, (uint32_t)N, (uint32_t)(W / 8));
    return check_launch("token_metric_kernel");
}

extern "C" int cocodiff_vmajor_topk(int32_t N, const float* metric, int32_t n_keep, int32_t* active_idx,
                                    int32_t* n_active, void* stream) {
    if (N <= 0) return fail(COCODIFF_ERR_SHAPE, "topk: N must be positive");
    if (n_keep < 0 || n_keep > N) return fail(COCODIFF_ERR_SHAPE, "topk: n_keep (%d) must be in [0, N = %d]", n_keep, N);
    if (!metric || !active_idx || !n_active) return fail(COCODIFF_ERR_NULL, "topk: NULL pointer");
    hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(kTopkThreads), 0, as_stream(stream), metric, (uint32_t)N,
                       (uint32_t)n_keep, active_idx, n_active);
    return check_launch("topk_kernel");
}

extern "C" int32_t cocodiff_cache_active_count(int32_t step, int32_t n_steps, int32_t warmup, int32_t sync_every,
                                               int32_t n_tokens) {
    if (n_tokens <= 0 || step < 1 || n_steps < 1 || warmup < 0) return -1;
    if (step <= warmup || n_steps <= warmup || (sync_every > 0 && step % sync_every == 0)) return n_tokens;   // full exchange
    const int64_t cached = (int64_t)n_tokens * (step - warmup) / (n_steps - warmup);   // floor(r * n_tokens), r = linear ramp
    return (int32_t)(n_tokens - (cached > n_tokens ? n_tokens : cached));
}
