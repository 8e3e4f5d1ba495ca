// QKV projection (paper Section II-B): Y[n][o] = sum_k X[n][k] * W[o][k], bf16 in, fp32 accumulate on the
// gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), one RNE rounding to bf16.
//
// Both operands are K-contiguous, so a tile of either is a set of 128-byte row segments.
// Workgroup = 256 lanes = 4 wavefronts (2 x 2), output tile 256 tokens x 256 features, K step 64,
// two LDS stages of (32 KB of X + 32 KB of W).  A wavefront owns 128 x 128 outputs = 4 x 4 MFMA tiles
// (256 accumulator registers per lane).  W rides the MFMA "A" side, so an accumulator lane holds four
// consecutive features of one token.  LDS rows are 128 B = eight 16-byte columns; column c of row r
// is stored at column c ^ swz(r), which makes the 128-bit fragment reads bank-conflict free.
// The epilogue rounds to bf16, transposes through the (now idle) LDS and writes whole 256-byte rows.
#include "internal.h"

namespace cocodiff {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 256;          // tokens per workgroup tile
constexpr int BN = 256;          // features per workgroup tile
constexpr int BK = 64;           // K elements per stage
constexpr int kGemmThreads = 256;
constexpr int kStageBytes = (BM + BN) * BK * 2;   // 64 KB
constexpr int kVecPerOperand = BM * (BK / 8) / kGemmThreads;   // 16-byte vectors per lane per operand per stage: 8

struct GemmArgs {
    const uint16_t* x;
    const uint16_t* w[3];
    uint16_t* y[3];
    int32_t n_tensors;
    int32_t row_begin, M;      // token rows [row_begin, row_begin + M)
    int32_t D;                 // features per tensor = K
    int32_t tiles_m, tiles_n_per_tensor;
};

__device__ __forceinline__ uint32_t swz(uint32_t row) { return (row & 7u) ^ ((row >> 3) & 1u); }

// Byte offset of 16-byte column c of row r inside a [rows][64] bf16 LDS tile.
__device__ __forceinline__ uint32_t lds_off(uint32_t row, uint32_t c) { return row * 128u + ((c ^ swz(row)) << 4); }

__global__ void __launch_bounds__(kGemmThreads) qkv_gemm_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // ---- which tile: blocks are dealt round-robin to the 8 XCDs, so give each XCD a contiguous run
    //      of tiles, ordered so that tiles running together share rows of X and W in that XCD's L2.
    const uint32_t n_tiles = gridDim.x;
    const uint32_t tiles_n = (uint32_t)a.tiles_n_per_tensor * a.n_tensors;
    uint32_t vt;
    {
        const uint32_t xcd = blockIdx.x & 7u, li = blockIdx.x >> 3;
        const uint32_t per = n_tiles >> 3, rem = n_tiles & 7u;   // XCD x gets per + (x < rem) tiles
        vt = xcd * per + (xcd < rem ? xcd : rem) + li;
    }
    // groups of 8 tile rows, walked column by column
    constexpr uint32_t GROUP = 8;
    const uint32_t per_group = GROUP * tiles_n;
    const uint32_t grp = vt / per_group;
    const uint32_t first_m = grp * GROUP;
    const uint32_t rows_here = min((uint32_t)a.tiles_m - first_m, GROUP);
    const uint32_t in_grp = vt - grp * per_group;
    const uint32_t tm = first_m + in_grp % rows_here;
    const uint32_t tn = in_grp / rows_here;

    const uint32_t tensor = tn / a.tiles_n_per_tensor;
    const uint32_t tn_local = tn - tensor * a.tiles_n_per_tensor;
    const uint16_t* __restrict__ W = a.w[tensor];
    uint16_t* __restrict__ Y = a.y[tensor];
    const uint32_t K = (uint32_t)a.D;
    const uint32_t m0 = tm * BM;          // first token of the tile, relative to row_begin
    const uint32_t f0 = tn_local * BN;    // first feature of the tile

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t wave_f = (wave & 1u) * 128u;    // wavefront's feature offset in the tile
    const uint32_t wave_t = (wave >> 1) * 128u;    // wavefront's token offset in the tile

    // ---- global -> register staging: lane moves vectors v = tid + 256*i, row = v/8, column = v%8
    const uint32_t ld_c = tid & 7u;
    const uint32_t ld_r = tid >> 3;       // + 32*i
    const uint16_t* xg[kVecPerOperand];
    const uint16_t* wg[kVecPerOperand];
#pragma unroll
    for (int i = 0; i < kVecPerOperand; ++i) {
        const uint32_t r = ld_r + 32u * i;
        const uint32_t xr = min(m0 + r, (uint32_t)a.M - 1u);       // rows past the end re-read the last row; never stored
        const uint32_t wr = min(f0 + r, (uint32_t)a.D - 1u);
        xg[i] = a.x + ((size_t)a.row_begin + xr) * K + ld_c * 8u;
        wg[i] = W + (size_t)wr * K + ld_c * 8u;
    }
    const bool k_tail = (K % BK) != 0;    // last stage partly beyond K: those vectors are zero

    vec16 xs[kVecPerOperand], ws[kVecPerOperand];
    auto load_stage = [&](uint32_t k0) {
#pragma unroll
        for (int i = 0; i < kVecPerOperand; ++i) {
            if (k_tail && k0 + ld_c * 8u >= K) {
                xs[i] = vec16{0u, 0u, 0u, 0u};
                ws[i] = vec16{0u, 0u, 0u, 0u};
            } else {
                xs[i] = *reinterpret_cast<const vec16*>(xg[i] + k0);
                ws[i] = *reinterpret_cast<const vec16*>(wg[i] + k0);
            }
        }
    };
    auto store_stage = [&](uint32_t stage) {
        unsigned char* xb = smem + stage * kStageBytes;
        unsigned char* wb = xb + BM * BK * 2;
#pragma unroll
        for (int i = 0; i < kVecPerOperand; ++i) {
            const uint32_t r = ld_r + 32u * i;
            *reinterpret_cast<vec16*>(xb + lds_off(r, ld_c)) = xs[i];
            *reinterpret_cast<vec16*>(wb + lds_off(r, ld_c)) = ws[i];
        }
    };

    f32x16 acc[4][4];   // [feature tile][token tile]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const uint32_t n_k = (K + BK - 1) / BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    const uint32_t frag_row = lane & 31u, frag_half = lane >> 5;
    for (uint32_t kt = 0; kt < n_k; ++kt) {
        const uint32_t cur = kt & 1u;
        if (kt + 1 < n_k) load_stage((kt + 1) * BK);
        const unsigned char* xb = smem + cur * kStageBytes;
        const unsigned char* wb = xb + BM * BK * 2;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 wf[4], xf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wf[i] = *reinterpret_cast<const bf16x8*>(wb + lds_off(wave_f + 32u * i + frag_row, 2u * kk + frag_half));
                xf[i] = *reinterpret_cast<const bf16x8*>(xb + lds_off(wave_t + 32u * i + frag_row, 2u * kk + frag_half));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < n_k) store_stage(cur ^ 1u);
        __syncthreads();
    }

    // ---- epilogue: bf16, transpose through this wavefront's private 32 KB of LDS, 256-byte row stores.
    // Accumulator element e of lane l in MFMA tile (i, j): feature 32i + 8*(e/4) + 4*(l/32) + e%4,
    // token 32j + l%32.  LDS row = token (256 B = sixteen 16-byte columns, column c stored at c ^ (row & 15)).
    unsigned char* ep = smem + wave * (128 * 256);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t row = 32u * j + frag_row;
                const uint32_t feat = 32u * i + 8u * g + 4u * frag_half;   // multiple of 4
                const uint32_t c16 = feat >> 3, half8 = (feat >> 2) & 1u;
                uint2 v;
                v.x = pack_bf16x2(acc[i][j][4 * g + 0], acc[i][j][4 * g + 1]);
                v.y = pack_bf16x2(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                *reinterpret_cast<uint2*>(ep + row * 256u + (((c16 ^ (row & 15u)) << 4) | (half8 << 3))) = v;
            }
    // the same wavefront reads back what it wrote, and a wavefront's LDS accesses complete in order:
    // no workgroup barrier is needed
    const uint32_t c16 = lane & 15u, rsub = lane >> 4;
#pragma unroll 8
    for (int it = 0; it < 32; ++it) {
        const uint32_t row = 4u * it + rsub;
        const vec16 v = *reinterpret_cast<const vec16*>(ep + row * 256u + ((c16 ^ (row & 15u)) << 4));
        const uint32_t tok = m0 + wave_t + row;
        const uint32_t feat = f0 + wave_f + c16 * 8u;
        if (tok < (uint32_t)a.M && feat < (uint32_t)a.D)
            *reinterpret_cast<vec16*>(Y + ((size_t)a.row_begin + tok) * K + feat) = v;
    }
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" int cocodiff_qkv_proj(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                 const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                 cocodiff_bf16* q, cocodiff_bf16* k, cocodiff_bf16* v, void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (!x) return fail(COCODIFF_ERR_NULL, "qkv_proj: x is NULL");
    if ((wq == nullptr) != (q == nullptr) || (wk == nullptr) != (k == nullptr) || (wv == nullptr) != (v == nullptr))
        return fail(COCODIFF_ERR_NULL, "qkv_proj: a weight and its output must be given together");
    if (!q && !k && !v) return fail(COCODIFF_ERR_NULL, "qkv_proj: no (weight, output) pair given");
    if (!aligned16(x) || !aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(q) || !aligned16(k) || !aligned16(v))
        return fail(COCODIFF_ERR_ALIGN, "qkv_proj: pointers must be 16-byte aligned");

    GemmArgs a;
    a.x = x;
    a.n_tensors = 0;
    const cocodiff_bf16* ws[3] = {wv, wq, wk};   // V first: its tiles are dealt out before Q's and K's
    cocodiff_bf16* ys[3] = {v, q, k};
    for (int i = 0; i < 3; ++i) {
        a.w[i] = nullptr;
        a.y[i] = nullptr;
    }
    for (int i = 0; i < 3; ++i)
        if (ws[i]) {
            a.w[a.n_tensors] = ws[i];
            a.y[a.n_tensors] = ys[i];
            ++a.n_tensors;
        }
    const int32_t Ns = shape->N / shape->P;
    a.row_begin = shape->rank_begin * Ns;
    a.M = shape->rank_count * Ns;
    a.D = shape->D;
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n_per_tensor = (a.D + BN - 1) / BN;
    const uint32_t n_tiles = (uint32_t)a.tiles_m * a.tiles_n_per_tensor * a.n_tensors;

    static bool attr_set = false;   // dynamic LDS above 64 KB needs the attribute once per process
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)qkv_gemm_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStageBytes);
        if (e != hipSuccess) return fail(COCODIFF_ERR_HIP, "qkv_proj: cannot reserve %d bytes of LDS: %s", 2 * kStageBytes, hipGetErrorString(e));
        attr_set = true;
    }
    hipLaunchKernelGGL(qkv_gemm_kernel, dim3(n_tiles), dim3(kGemmThreads), 2 * kStageBytes, as_stream(stream), a);
    return check_launch("qkv_gemm_kernel");
}
