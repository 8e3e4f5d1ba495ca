// Error channel, shape validation, host helpers (RoPE table) and the calibration copy kernel.
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include "internal.h"

namespace cocodiff {

static thread_local char g_last_error[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return code;
}

int check_shape(const cocodiff_shape* s) {
    if (!s) return fail(COCODIFF_ERR_NULL, "shape is NULL");
    if (s->N <= 0 || s->D <= 0 || s->H <= 0 || s->d <= 0 || s->P <= 0)
        return fail(COCODIFF_ERR_SHAPE, "N, D, H, d, P must be positive (N=%d D=%d H=%d d=%d P=%d)",
                    s->N, s->D, s->H, s->d, s->P);
    if ((int64_t)s->H * s->d != s->D)
        return fail(COCODIFF_ERR_SHAPE, "D (%d) != H*d (%d*%d)", s->D, s->H, s->d);
    if (s->d % 8) return fail(COCODIFF_ERR_SHAPE, "d (%d) must be a multiple of 8", s->d);
    if (s->N % s->P) return fail(COCODIFF_ERR_SHAPE, "N (%d) must divide evenly over P (%d) ranks", s->N, s->P);
    if (s->H % s->P) return fail(COCODIFF_ERR_SHAPE, "H (%d) must divide evenly over P (%d) ranks", s->H, s->P);
    if ((s->N / s->P) % 16)
        return fail(COCODIFF_ERR_SHAPE, "tokens per rank (%d) must be a multiple of 16", s->N / s->P);
    if (s->rank_begin < 0 || s->rank_count < 1 || (int64_t)s->rank_begin + s->rank_count > s->P)
        return fail(COCODIFF_ERR_SHAPE, "rank range [%d, %d+%d) outside [0, %d)", s->rank_begin,
                    s->rank_begin, s->rank_count, s->P);
    return COCODIFF_OK;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(COCODIFF_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return COCODIFF_OK;
}

static int check_rope_desc(const cocodiff_rope* r) {
    if (!r) return fail(COCODIFF_ERR_NULL, "rope is NULL");
    if (r->n_axes < 1 || r->n_axes > 3) return fail(COCODIFF_ERR_SHAPE, "rope n_axes (%d) must be 1..3", r->n_axes);
    for (int a = 0; a < r->n_axes; ++a)
        if (r->grid[a] <= 0 || r->pairs[a] <= 0)
            return fail(COCODIFF_ERR_SHAPE, "rope axis %d: grid (%d) and pairs (%d) must be positive", a,
                        r->grid[a], r->pairs[a]);
    if (!(r->theta > 0.f)) return fail(COCODIFF_ERR_SHAPE, "rope theta must be positive");
    return COCODIFF_OK;
}

// One 16-byte vector per thread: small workgroups measured fastest on data that is not in the last-level cache.
template <bool NT_LD, bool NT_ST>
__global__ void __launch_bounds__(256) copy_kernel(const vec16* __restrict__ src, vec16* __restrict__ dst, size_t n_vec) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_vec) st_vec<NT_ST>(dst + i, ld_vec<NT_LD>(src + i));
}

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 mfma_in_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float mfma_acc_t;

constexpr int kRateNI = 4, kRateNJ = 8;   // the projection kernel's wavefront tile: 4 x 8 accumulator tiles of 16 x 16

// Register-only loop of the projection kernel's matrix-core work: v_mfma_f32_16x16x32_bf16 on a 4 x 8 outer product
// of operand fragments, token tile by token tile, 8 wavefronts per workgroup (two per SIMD), no memory traffic.  The fragments hold small pseudo-random bf16
// values that differ per lane and per fragment, so consecutive MFMAs see different operands as they do in a real
// product (with constant operands the matrix cores draw less power and the chip clocks higher than on real data).
__global__ void __launch_bounds__(512) mfma_rate_kernel(uint32_t iters, float* __restrict__ sink) {
    uint32_t h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
    union Operand { uint16_t u[8]; mfma_in_t v; };
    Operand a[kRateNI], b[kRateNJ];
    auto fill = [&](Operand& o) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            h = h * 1664525u + 1013904223u;
            o.u[i] = (uint16_t)(0x3C00u | ((h >> 9) & 0x83FFu));   // bf16 of magnitude 2^-7 .. 2, either sign
        }
    };
#pragma unroll
    for (int i = 0; i < kRateNI; ++i) fill(a[i]);
#pragma unroll
    for (int j = 0; j < kRateNJ; ++j) fill(b[j]);
    mfma_acc_t acc[kRateNI][kRateNJ];
#pragma unroll
    for (int i = 0; i < kRateNI; ++i)
#pragma unroll
        for (int j = 0; j < kRateNJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kRateNJ; ++j)
#pragma unroll
            for (int i = 0; i < kRateNI; ++i) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);      // the order as written, as in the projection kernel
            }
    }
    float total = 0.f;
#pragma unroll
    for (int i = 0; i < kRateNI; ++i)
#pragma unroll
        for (int j = 0; j < kRateNJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) total += acc[i][j][e];
    if (total == 123.456f) sink[0] = total;   // keeps the loop alive; practically never true
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" {

const char* cocodiff_version(void) { return "cocodiff-mi355x 0.1 (gfx950)"; }

const char* cocodiff_last_error(void) { return g_last_error; }

size_t cocodiff_rope_table_bytes(const cocodiff_rope* rope) {
    if (check_rope_desc(rope) != COCODIFF_OK) return 0;
    size_t n = 0;
    for (int a = 0; a < rope->n_axes; ++a) n += (size_t)rope->grid[a] * rope->pairs[a] * 2;
    return n * sizeof(float);
}

int cocodiff_rope_table_fill(const cocodiff_rope* rope, float* host_out) {
    int rc = check_rope_desc(rope);
    if (rc != COCODIFF_OK) return rc;
    if (!host_out) return fail(COCODIFF_ERR_NULL, "host_out is NULL");
    float* out = host_out;
    for (int a = 0; a < rope->n_axes; ++a) {
        const int pa = rope->pairs[a];
        for (int c = 0; c < rope->grid[a]; ++c)
            for (int j = 0; j < pa; ++j) {
                const double omega = std::pow((double)rope->theta, -(double)j / (double)pa);
                const double phi = (double)c * omega;
                *out++ = (float)std::cos(phi);
                *out++ = (float)std::sin(phi);
            }
    }
    return COCODIFF_OK;
}

int cocodiff_util_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst) return fail(COCODIFF_ERR_NULL, "copy: NULL pointer");
    if (!aligned16(src) || !aligned16(dst)) return fail(COCODIFF_ERR_ALIGN, "copy: pointers must be 16-byte aligned");
    if (bytes % 16) return fail(COCODIFF_ERR_SHAPE, "copy: bytes (%zu) must be a multiple of 16", bytes);
    if (bytes == 0) return COCODIFF_OK;
    const size_t n_vec = bytes / 16;
    const size_t blocks = (n_vec + 255) / 256;
    if (blocks >= ((size_t)1 << 31)) return fail(COCODIFF_ERR_SHAPE, "copy: %zu bytes is too much for one launch", bytes);
    with_policy(stream_loads(2 * bytes), stream_stores(2 * bytes), [&](auto L, auto S) {
        hipLaunchKernelGGL((copy_kernel<decltype(L)::value, decltype(S)::value>), dim3((unsigned)blocks), dim3(256), 0,
                           as_stream(stream), (const vec16*)src, (vec16*)dst, n_vec);
    });
    return check_launch("copy_kernel");
}

int64_t cocodiff_util_mfma_rate(int32_t blocks, int32_t iters, float* sink, void* stream) {
    if (blocks <= 0 || iters <= 0) return fail(COCODIFF_ERR_SHAPE, "mfma_rate: blocks and iters must be positive");
    if (!sink) return fail(COCODIFF_ERR_NULL, "mfma_rate: NULL sink");
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)blocks), dim3(512), 0, as_stream(stream), (uint32_t)iters, sink);
    const int rc = check_launch("mfma_rate_kernel");
    if (rc != COCODIFF_OK) return rc;
    return (int64_t)blocks * 8 * iters * (kRateNI * kRateNJ) * (2LL * 16 * 16 * 32);
}

}  // extern "C"
