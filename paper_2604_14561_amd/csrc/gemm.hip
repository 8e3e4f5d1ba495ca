// QKV projection (paper Section II-B): Y[n][o] = sum_k X[n][k] * W[o][k], bf16 in, fp32 accumulate on the
// gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), one RNE rounding to bf16.
//
// Workgroup tile: 256 tokens x 256 features, K step 64 (a row segment of either operand is one whole
// 128-byte line; half lines halve the L1 fill rate).  W rides the MFMA "A" side, so an accumulator lane
// holds four consecutive features of one token.  Both operands are K-contiguous; LDS tiles keep rows
// contiguous and store 16-byte column c of row r at column c ^ swz(r), which makes the 128-bit fragment
// reads bank-conflict free.
//
// Main kernel (K a multiple of 64): global -> LDS directly (no staging registers), two 64 KB stages.
// WN wavefronts along the features x 2 along the tokens: WN = 4 gives 8 wavefronts of 128 x 64 outputs,
// two per SIMD, so one can multiply while the other waits for LDS, memory or the barrier.
// Fallback kernel (any K that is a multiple of 8): global -> registers -> LDS, zero-filled K tail.
// The epilogue rounds to bf16, transposes through the (now idle) LDS and writes whole rows.
#include <type_traits>

#include "internal.h"

namespace cocodiff {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 256;          // tokens per workgroup tile
constexpr int BN = 256;          // features per workgroup tile
constexpr int BK = 64;           // K elements per step
constexpr int kTileBytes = BM * BK * 2;                  // one operand tile of one K step: 32 KB (BM == BN)
constexpr int kStageBytes = 2 * kTileBytes;              // 64 KB
constexpr int kLdsBytes = 2 * kStageBytes;               // 128 KB

struct GemmArgs {
    const uint16_t* x;
    const uint16_t* w[3];
    uint16_t* y[3];
    int32_t n_tensors;
    int32_t row_begin, M;      // token rows [row_begin, row_begin + M)
    int32_t D;                 // features per tensor = K
    int32_t tiles_m, tiles_n_per_tensor;
};

// [rows][64] bf16 tiles (128-byte rows): any 16 consecutive rows of one column land in 16 different
// 16-byte slots of the 256-byte bank span.
__device__ __forceinline__ uint32_t swz(uint32_t row) { return (row & 7u) ^ ((row >> 3) & 1u); }

// Byte offset of 16-byte column c of row r inside a [rows][64] bf16 LDS tile.
__device__ __forceinline__ uint32_t lds_off(uint32_t row, uint32_t c) { return row * 128u + ((c ^ swz(row)) << 4); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

struct TileCoord {
    uint32_t tensor, m0, f0;
};

// Blocks are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of tiles, ordered in groups
// of 8 tile rows walked column by column, so tiles running together share rows of X and W in that XCD's L2.
__device__ __forceinline__ TileCoord tile_of_block(const GemmArgs& a) {
    const uint32_t n_tiles = gridDim.x;
    const uint32_t tiles_n = (uint32_t)a.tiles_n_per_tensor * a.n_tensors;
    const uint32_t xcd = blockIdx.x & 7u, li = blockIdx.x >> 3;
    const uint32_t per = n_tiles >> 3, rem = n_tiles & 7u;   // XCD x gets per + (x < rem) tiles
    const uint32_t vt = xcd * per + (xcd < rem ? xcd : rem) + li;
    constexpr uint32_t GROUP = 8;
    const uint32_t per_group = GROUP * tiles_n;
    const uint32_t grp = vt / per_group;
    const uint32_t first_m = grp * GROUP;
    const uint32_t rows_here = min((uint32_t)a.tiles_m - first_m, GROUP);
    const uint32_t in_grp = vt - grp * per_group;
    const uint32_t tm = first_m + in_grp % rows_here;
    const uint32_t tn = in_grp / rows_here;
    TileCoord t;
    t.tensor = tn / a.tiles_n_per_tensor;
    t.m0 = tm * BM;
    t.f0 = (tn - t.tensor * a.tiles_n_per_tensor) * BN;
    return t;
}

// A wavefront's accumulators: NI feature tiles x 4 token tiles of 32 x 32.
template <int NI>
__device__ __forceinline__ void mfma_slice(f32x16 (&acc)[NI][4], const bf16x8 (&wf)[NI], const bf16x8 (&xf)[4]) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
}

// Round to bf16, transpose through this wavefront's private LDS region (128 token rows of NI*32 features),
// write whole rows.  Accumulator element e of lane l in MFMA tile (i, j): feature 32i + 8*(e/4) + 4*(l/32)
// + e%4, token 32j + l%32.  16-byte column c of LDS row r is stored at column c ^ (r & (columns - 1)).
template <int NI>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[NI][4], unsigned char* ep, uint32_t lane,
                                           uint16_t* __restrict__ Y, size_t row0, uint32_t tok0, uint32_t feat0,
                                           uint32_t M, uint32_t D) {
    constexpr uint32_t COLS = NI * 4;            // 16-byte columns per row
    constexpr uint32_t ROWB = COLS * 16;         // bytes per row
    const uint32_t frag_row = lane & 31u, frag_half = lane >> 5;
#pragma unroll
    for (int i = 0; i < NI; ++i)
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
                *reinterpret_cast<uint2*>(ep + row * ROWB + (((c16 ^ (row & (COLS - 1u))) << 4) | (half8 << 3))) = v;
            }
    // the same wavefront reads back what it wrote, and a wavefront's LDS accesses complete in order:
    // no workgroup barrier is needed
    constexpr uint32_t RPI = 64 / COLS;          // rows per read instruction
    const uint32_t c16 = lane % COLS, rsub = lane / COLS;
#pragma unroll 8
    for (uint32_t it = 0; it < 128 / RPI; ++it) {
        const uint32_t row = RPI * it + rsub;
        const vec16 v = *reinterpret_cast<const vec16*>(ep + row * ROWB + ((c16 ^ (row & (COLS - 1u))) << 4));
        const uint32_t tok = tok0 + row;
        const uint32_t feat = feat0 + c16 * 8u;
        if (tok < M && feat < D) *reinterpret_cast<vec16*>(Y + (row0 + tok) * D + feat) = v;
    }
}

// s_waitcnt: at most WAIT global->LDS loads of this wavefront still in flight (LDS-read counter untouched)
template <int WAIT>
__device__ __forceinline__ void wait_loads() {
    static_assert(WAIT >= 0 && WAIT < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (WAIT & 15) | ((WAIT >> 4) << 14));
}

// ---------------------------------------------------------------------------------------------
// Main kernel.  K step kt lives in LDS stage kt & 1.  In step kt a wavefront multiplies slices 0..2 (each
// while reading the next slice's fragments), waits until step kt+1 has landed (its own loads; the barrier
// covers the other wavefronts'), then multiplies slice 3 while reading slice 0 of step kt+1 and issuing
// the loads of step kt+2 into the stage step kt used (every wavefront is past its last read of it).
// Instruction order inside a slice is pinned with scheduling groups (0x008 MFMA, 0x100 LDS read,
// 0x020 VMEM read): the fragment reads of the next slice are slotted one per MFMA from the start.
// ---------------------------------------------------------------------------------------------
template <int WN>
__global__ void __launch_bounds__(128 * WN) qkv_gemm_direct_kernel(GemmArgs a) {
    constexpr int WAVES = 2 * WN;
    constexpr int NI = BN / WN / 32;               // feature tiles per wavefront: 4 or 2
    constexpr int NMFMA = NI * 4, NREAD = NI + 4;
    constexpr int LOADS = 32 / WAVES;              // global->LDS instructions per lane per operand per step
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const TileCoord tc = tile_of_block(a);
    const uint16_t* __restrict__ W = a.w[tc.tensor];
    const uint32_t K = (uint32_t)a.D;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t wave_f = (wave % WN) * (NI * 32u), wave_t = (wave / WN) * 128u;

    // load i of this wavefront fills LDS rows (WAVES*i + wave)*8 .. +8 of a tile: lane -> row lane>>3, stored column lane&7
    const unsigned char* xbase = reinterpret_cast<const unsigned char*>(a.x + ((size_t)a.row_begin + tc.m0) * K);
    const unsigned char* wbase = reinterpret_cast<const unsigned char*>(W + (size_t)tc.f0 * K);
    uint32_t xoff[LOADS], woff[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const uint32_t r = (WAVES * i + wave) * 8u + (lane >> 3);
        const uint32_t c = (lane & 7u) ^ swz(r);
        const uint32_t xr = min(r, (uint32_t)a.M - 1u - tc.m0);     // rows past the end re-read the last row; never stored
        const uint32_t wr = min(r, (uint32_t)a.D - 1u - tc.f0);
        xoff[i] = xr * K * 2u + c * 16u;
        woff[i] = wr * K * 2u + c * 16u;
    }
    auto issue_loads = [&](uint32_t kt) {
        const unsigned char* xk = xbase + (size_t)kt * (BK * 2);
        const unsigned char* wk = wbase + (size_t)kt * (BK * 2);
        unsigned char* xl = smem + (kt & 1u) * kStageBytes + wave * 1024u;
        unsigned char* wl = xl + kTileBytes;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            __builtin_amdgcn_global_load_lds((gptr_t)(xk + xoff[i]), (lptr_t)(xl + i * (WAVES * 1024)), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(wk + woff[i]), (lptr_t)(wl + i * (WAVES * 1024)), 16, 0, 0);
        }
    };

    // fragment addresses: row = wave offset + 32i + (lane & 31); the swizzle depends on the lane only
    const uint32_t frag_row = lane & 31u, frag_half = lane >> 5;
    const uint32_t sw = swz(frag_row);
    const uint32_t x_frag = (wave_t + frag_row) * 128u;
    const uint32_t w_frag = kTileBytes + (wave_f + frag_row) * 128u;
    auto read_frags = [&](uint32_t stage, uint32_t kk, bf16x8 (&wf)[NI], bf16x8 (&xf)[4]) {
        const unsigned char* sb = smem + stage * kStageBytes + (((2u * kk + frag_half) ^ sw) << 4);
        wf[0] = *reinterpret_cast<const bf16x8*>(sb + w_frag);     // in the order the MFMAs consume them
#pragma unroll
        for (int i = 0; i < 4; ++i) xf[i] = *reinterpret_cast<const bf16x8*>(sb + x_frag + i * 4096);
#pragma unroll
        for (int i = 1; i < NI; ++i) wf[i] = *reinterpret_cast<const bf16x8*>(sb + w_frag + i * 4096);
    };

    f32x16 acc[NI][4];   // [feature tile][token tile]
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const uint32_t n_k = K / BK;   // >= 2 (the host sends shorter K to the fallback kernel)
    issue_loads(0);
    issue_loads(1);
    wait_loads<2 * LOADS>();       // step 0 has landed; step 1 may still be in flight
    __syncthreads();

    bf16x8 wf0[NI], xf0[4], wf1[NI], xf1[4];
    read_frags(0, 0, wf0, xf0);

    auto pin_slice = [&]() {       // NMFMA MFMAs with the NREAD fragment reads slotted after the first ones
#pragma unroll
        for (int g = 0; g < NREAD; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NREAD, 0);
    };
    auto k_step = [&](uint32_t kt, auto next_frags, auto next_loads) {
        constexpr bool NEXT = decltype(next_frags)::value, LOAD = decltype(next_loads)::value;
        const uint32_t cur = kt & 1u;
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            __builtin_amdgcn_sched_barrier(0);
            if (kk & 1) {
                read_frags(cur, kk + 1, wf0, xf0);
                mfma_slice<NI>(acc, wf1, xf1);
            } else {
                read_frags(cur, kk + 1, wf1, xf1);
                mfma_slice<NI>(acc, wf0, xf0);
            }
            pin_slice();
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (NEXT) {
            wait_loads<0>();
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (NEXT) read_frags(cur ^ 1u, 0, wf0, xf0);
        if constexpr (LOAD) issue_loads(kt + 2);
        mfma_slice<NI>(acc, wf1, xf1);
        if constexpr (NEXT) {
#pragma unroll
            for (int g = 0; g < NREAD; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            if constexpr (LOAD) {
#pragma unroll
                for (int g = 0; g < NMFMA - NREAD; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, (2 * LOADS + NMFMA - NREAD - 1) / (NMFMA - NREAD), 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    using yes = std::true_type;
    using no = std::false_type;
    uint32_t kt = 0;
    for (; kt + 2 < n_k; ++kt) k_step(kt, yes{}, yes{});
    k_step(kt, yes{}, no{});       // step n_k-2: nothing left to issue
    k_step(kt + 1, no{}, no{});    // step n_k-1
    __syncthreads();
    store_tile<NI>(acc, smem + wave * (128 * NI * 64), lane, a.y[tc.tensor], (size_t)a.row_begin,
                   tc.m0 + wave_t, tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D);
}

// ---------------------------------------------------------------------------------------------
// General path, any K that is a multiple of 8: global -> registers -> LDS, vectors beyond K are zero.
// Four wavefronts (2 x 2) of 128 x 128 outputs.
// ---------------------------------------------------------------------------------------------
constexpr int kStagedThreads = 256;
constexpr int kVecPerOperand = BM * (BK / 8) / kStagedThreads;   // 16-byte vectors per lane per operand per stage: 8

__global__ void __launch_bounds__(kStagedThreads) qkv_gemm_staged_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const TileCoord tc = tile_of_block(a);
    const uint16_t* __restrict__ W = a.w[tc.tensor];
    const uint32_t K = (uint32_t)a.D;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t wave_f = (wave & 1u) * 128u, wave_t = (wave >> 1) * 128u;

    // lane moves vectors v = tid + 256*i of a tile: row = v/8, column = v%8
    const uint32_t ld_c = tid & 7u, ld_r = tid >> 3;
    const uint16_t* xg[kVecPerOperand];
    const uint16_t* wg[kVecPerOperand];
#pragma unroll
    for (int i = 0; i < kVecPerOperand; ++i) {
        const uint32_t r = ld_r + 32u * i;
        const uint32_t xr = min(tc.m0 + r, (uint32_t)a.M - 1u);
        const uint32_t wr = min(tc.f0 + r, (uint32_t)a.D - 1u);
        xg[i] = a.x + ((size_t)a.row_begin + xr) * K + ld_c * 8u;
        wg[i] = W + (size_t)wr * K + ld_c * 8u;
    }
    vec16 xs[kVecPerOperand], ws[kVecPerOperand];
    auto load_stage = [&](uint32_t k0) {
        const bool inside = k0 + ld_c * 8u < K;
#pragma unroll
        for (int i = 0; i < kVecPerOperand; ++i) {
            xs[i] = inside ? *reinterpret_cast<const vec16*>(xg[i] + k0) : vec16{0u, 0u, 0u, 0u};
            ws[i] = inside ? *reinterpret_cast<const vec16*>(wg[i] + k0) : vec16{0u, 0u, 0u, 0u};
        }
    };
    auto store_stage = [&](uint32_t stage) {
        unsigned char* xb = smem + stage * kStageBytes;
        unsigned char* wb = xb + kTileBytes;
#pragma unroll
        for (int i = 0; i < kVecPerOperand; ++i) {
            const uint32_t r = ld_r + 32u * i;
            *reinterpret_cast<vec16*>(xb + lds_off(r, ld_c)) = xs[i];
            *reinterpret_cast<vec16*>(wb + lds_off(r, ld_c)) = ws[i];
        }
    };

    f32x16 acc[4][4];
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
        const unsigned char* wb = xb + kTileBytes;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 wf[4], xf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wf[i] = *reinterpret_cast<const bf16x8*>(wb + lds_off(wave_f + 32u * i + frag_row, 2u * kk + frag_half));
                xf[i] = *reinterpret_cast<const bf16x8*>(xb + lds_off(wave_t + 32u * i + frag_row, 2u * kk + frag_half));
            }
            mfma_slice<4>(acc, wf, xf);
        }
        if (kt + 1 < n_k) store_stage(cur ^ 1u);
        __syncthreads();
    }
    store_tile<4>(acc, smem + wave * (128 * 256), lane, a.y[tc.tensor], (size_t)a.row_begin, tc.m0 + wave_t,
                  tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D);
}

constexpr int kMainWN = 4;   // 8 wavefronts per workgroup in the main kernel

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
    if ((int64_t)BM * a.D * 2 >= ((int64_t)1 << 32)) return fail(COCODIFF_ERR_SHAPE, "qkv_proj: D (%d) too large", a.D);

    static bool attr_set = false;   // dynamic LDS above 64 KB needs the attribute once per process
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)qkv_gemm_direct_kernel<kMainWN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)qkv_gemm_staged_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return fail(COCODIFF_ERR_HIP, "qkv_proj: cannot reserve LDS: %s", hipGetErrorString(e));
        attr_set = true;
    }
    if (a.D % BK == 0 && a.D >= 2 * BK)
        hipLaunchKernelGGL(qkv_gemm_direct_kernel<kMainWN>, dim3(n_tiles), dim3(128 * kMainWN), kLdsBytes, as_stream(stream), a);
    else
        hipLaunchKernelGGL(qkv_gemm_staged_kernel, dim3(n_tiles), dim3(kStagedThreads), kLdsBytes, as_stream(stream), a);
    return check_launch("qkv_gemm_kernel");
}
