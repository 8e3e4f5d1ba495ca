// V-Major active-tile selection (paper Section III-D), threshold-per-tile form:
//   flag[t] = any element of tile t with NOT(|v_cur - v_prev| <= tau)   (fp32 decision)
//   idx     = ascending list of flagged tiles, n_active = its length
//   compact = v_cur of the flagged tiles gathered densely in list order.
//
// Three launches on the caller's stream:
//   1. flag pass   -- one wavefront per piece (<= 256 16-byte vectors) of a (tile, slab) segment,
//                     streams v_cur and v_prev once, writes one partial flag per piece;
//   2. scan        -- one workgroup ORs the partials of each tile, ballot/prefix-scans the flags
//                     and writes flags, idx and n_active;
//   3. gather      -- one wavefront per (active tile, slab, piece) copies v_cur into `compact`;
//                     wavefronts beyond n_active exit at once.
// HBM traffic: 2 tensors read once + the active fraction read once more and written once.
#include "internal.h"

namespace cocodiff {

constexpr int kPieceVec = 256;   // 16-byte vectors per piece: 64 lanes x 4
constexpr int kWavesPerBlock = 4;

struct SelectShape {
    uint32_t S, NT, seg8, pieces;   // seg8: vectors per (tile, slab) segment; pieces per segment
    uint64_t slab8;                 // vectors per slab = N*W/8
};

__device__ __forceinline__ bool vec_changed(const vec16& c, const vec16& p, float tau) {
    const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
    const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
    bool changed = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float dl = fabsf(bf16_lo(cw[i]) - bf16_lo(pw[i]));
        const float dh = fabsf(bf16_hi(cw[i]) - bf16_hi(pw[i]));
        changed |= !(dl <= tau);
        changed |= !(dh <= tau);
    }
    return changed;
}

// partial[(t*S + s)*pieces + q] = 1 if piece q of segment (t, s) holds a changed element.
__global__ void __launch_bounds__(64 * kWavesPerBlock) select_flag_kernel(
    const vec16* __restrict__ cur, const vec16* __restrict__ prev, float tau, int32_t* __restrict__ partial,
    SelectShape sh, uint32_t n_items) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t item = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (item >= n_items) return;
    const uint32_t q = item % sh.pieces;
    const uint32_t ts = item / sh.pieces;
    const uint32_t s = ts % sh.S;
    const uint32_t t = ts / sh.S;
    const uint64_t seg = (uint64_t)s * sh.slab8 + (uint64_t)t * sh.seg8;
    const uint32_t v0 = q * kPieceVec + lane;
    vec16 c[4], p[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t v = v0 + k * 64;
        if (v < sh.seg8) {
            c[k] = ld_nt(cur + seg + v);
            p[k] = ld_nt(prev + seg + v);
        }
    }
    bool changed = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t v = v0 + k * 64;
        if (v < sh.seg8) changed |= vec_changed(c[k], p[k], tau);
    }
    const bool any = __ballot(changed) != 0ull;
    if (lane == 0) partial[item] = any ? 1 : 0;
}

// One workgroup of 1024 lanes walks the tiles in order, 1024 at a time.
__global__ void __launch_bounds__(1024) select_scan_kernel(const int32_t* __restrict__ partial, int32_t* __restrict__ flags,
                                                           int32_t* __restrict__ idx, int32_t* __restrict__ n_active,
                                                           uint32_t NT, uint32_t per_tile) {
    __shared__ uint32_t wave_count[16];
    __shared__ uint32_t running;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) running = 0;
    __syncthreads();
    for (uint32_t t0 = 0; t0 < NT; t0 += 1024) {
        const uint32_t t = t0 + threadIdx.x;
        bool f = false;
        if (t < NT) {
            const int32_t* pt = partial + (size_t)t * per_tile;
            int32_t acc = 0;
            for (uint32_t i = 0; i < per_tile; ++i) acc |= pt[i];
            f = acc != 0;
            if (flags) flags[t] = f ? 1 : 0;
        }
        const uint64_t ball = __ballot(f);
        const uint32_t below = __popcll(ball & ((1ull << lane) - 1ull));
        if (lane == 0) wave_count[wave] = __popcll(ball);
        __syncthreads();
        uint32_t before = running;
        for (uint32_t w = 0; w < wave; ++w) before += wave_count[w];
        if (f) idx[before + below] = (int32_t)t;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t tot = running;
            for (uint32_t w = 0; w < 16; ++w) tot += wave_count[w];
            running = tot;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *n_active = (int32_t)running;
}

// item = (j*S + s)*pieces + q over j < cap_tiles; wavefronts with j >= n_active leave at once.
__global__ void __launch_bounds__(64 * kWavesPerBlock) select_gather_kernel(
    const vec16* __restrict__ cur, const int32_t* __restrict__ idx, const int32_t* __restrict__ n_active,
    vec16* __restrict__ compact, SelectShape sh, uint32_t cap_tiles, uint32_t n_items) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t item = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (item >= n_items) return;
    const uint32_t q = item % sh.pieces;
    const uint32_t js = item / sh.pieces;
    const uint32_t s = js % sh.S;
    const uint32_t j = js / sh.S;
    if ((int32_t)j >= *n_active) return;
    const uint32_t t = (uint32_t)idx[j];
    const uint64_t src = (uint64_t)s * sh.slab8 + (uint64_t)t * sh.seg8;
    const uint64_t dst = ((uint64_t)s * cap_tiles + j) * sh.seg8;
    const uint32_t v0 = q * kPieceVec + lane;
    vec16 c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t v = v0 + k * 64;
        if (v < sh.seg8) c[k] = cur[src + v];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t v = v0 + k * 64;
        if (v < sh.seg8) st_nt(compact + dst + v, c[k]);
    }
}

static int select_shape(int32_t S, int32_t N, int32_t W, int32_t T, SelectShape* out) {
    if (S <= 0 || N <= 0 || W <= 0 || T <= 0) return fail(COCODIFF_ERR_SHAPE, "select: S, N, W, tile_tokens must be positive");
    if (W % 8) return fail(COCODIFF_ERR_SHAPE, "select: W (%d) must be a multiple of 8", W);
    if (N % T) return fail(COCODIFF_ERR_SHAPE, "select: N (%d) must be a multiple of tile_tokens (%d)", N, T);
    const int64_t seg8 = (int64_t)T * W / 8;
    const int64_t pieces = (seg8 + kPieceVec - 1) / kPieceVec;
    const int64_t NT = N / T;
    if (NT * S * pieces >= ((int64_t)1 << 31) || seg8 >= ((int64_t)1 << 31))
        return fail(COCODIFF_ERR_SHAPE, "select: too many (tile, slab, piece) work items");
    out->S = (uint32_t)S;
    out->NT = (uint32_t)NT;
    out->seg8 = (uint32_t)seg8;
    out->pieces = (uint32_t)pieces;
    out->slab8 = (uint64_t)N * W / 8;
    return COCODIFF_OK;
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" size_t cocodiff_vmajor_select_workspace_bytes(int32_t S, int32_t N, int32_t W, int32_t tile_tokens) {
    SelectShape sh;
    if (select_shape(S, N, W, tile_tokens, &sh) != COCODIFF_OK) return 0;
    return (size_t)sh.NT * sh.S * sh.pieces * sizeof(int32_t);
}

extern "C" int cocodiff_vmajor_select(int32_t S, int32_t N, int32_t W, int32_t tile_tokens,
                                      const cocodiff_bf16* v_cur, const cocodiff_bf16* v_prev, float tau,
                                      int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                      cocodiff_bf16* compact, int32_t cap_tiles,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    SelectShape sh;
    int rc = select_shape(S, N, W, tile_tokens, &sh);
    if (rc != COCODIFF_OK) return rc;
    if (!v_cur || !v_prev || !active_idx || !n_active || !workspace)
        return fail(COCODIFF_ERR_NULL, "select: v_cur, v_prev, active_idx, n_active and workspace are required");
    if (!aligned16(v_cur) || !aligned16(v_prev) || !aligned16(workspace) || (compact && !aligned16(compact)))
        return fail(COCODIFF_ERR_ALIGN, "select: tensors and workspace must be 16-byte aligned");
    if (compact && cap_tiles < 1) return fail(COCODIFF_ERR_CAPACITY, "select: cap_tiles (%d) must be >= 1", cap_tiles);
    const size_t need = (size_t)sh.NT * sh.S * sh.pieces * sizeof(int32_t);
    if (workspace_bytes < need)
        return fail(COCODIFF_ERR_CAPACITY, "select: workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    hipStream_t st = as_stream(stream);
    int32_t* partial = (int32_t*)workspace;

    const uint32_t n_items = sh.NT * sh.S * sh.pieces;
    hipLaunchKernelGGL(select_flag_kernel, dim3((n_items + kWavesPerBlock - 1) / kWavesPerBlock), dim3(64 * kWavesPerBlock),
                       0, st, (const vec16*)v_cur, (const vec16*)v_prev, tau, partial, sh, n_items);
    rc = check_launch("select_flag_kernel");
    if (rc != COCODIFF_OK) return rc;
    hipLaunchKernelGGL(select_scan_kernel, dim3(1), dim3(1024), 0, st, (const int32_t*)partial, flags, active_idx,
                       n_active, sh.NT, sh.S * sh.pieces);
    rc = check_launch("select_scan_kernel");
    if (rc != COCODIFF_OK) return rc;
    if (compact) {
        const uint32_t cap = (uint32_t)cap_tiles < sh.NT ? (uint32_t)cap_tiles : sh.NT;
        const uint64_t items64 = (uint64_t)cap * sh.S * sh.pieces;
        const uint32_t g_items = (uint32_t)items64;
        hipLaunchKernelGGL(select_gather_kernel, dim3((g_items + kWavesPerBlock - 1) / kWavesPerBlock),
                           dim3(64 * kWavesPerBlock), 0, st, (const vec16*)v_cur, (const int32_t*)active_idx,
                           (const int32_t*)n_active, (vec16*)compact, sh, (uint32_t)cap_tiles, g_items);
        rc = check_launch("select_gather_kernel");
    }
    return rc;
}
