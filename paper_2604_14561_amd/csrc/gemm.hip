// QKV projection (paper Section II-B): Y[n][o] = sum_k X[n][k] * W[o][k], bf16 in, fp32 accumulate on the
// gfx950 matrix cores, one RNE rounding to bf16.  The main kernel multiplies with v_mfma_f32_16x16x32_bf16: on this
// power-limited part it sustains 1.91 PFLOP/s at 0.70 pJ/flop in a register-only loop against 1.72 PFLOP/s at
// 0.77 pJ/flop for v_mfma_f32_32x32x16_bf16, for the same LDS traffic per flop (a wavefront's tile decides that).
//
// Workgroup tile: 256 tokens x 256 features (192 x 192 when that fills the compute units much better: small
// token counts), K step 64 (a row segment of either operand is one whole 128-byte line; half lines halve the L1
// fill rate).  W rides the MFMA "A" side, so an accumulator lane
// holds four consecutive features of one token.  Both operands are K-contiguous; LDS tiles keep rows
// contiguous and store 16-byte column c of row r at column c ^ swz(r), which makes the 128-bit fragment
// reads bank-conflict free.
//
// Main kernel (K a multiple of 64): global -> LDS directly (no staging registers) through a ring of five
// slots (X and W tiles of a step travel separately; 32 KB each for the 256 x 256 tile).  WN wavefronts along the
// features x 2 along the tokens: WN = 4 gives 8 wavefronts of 128 x 64 outputs, two per SIMD, so one can multiply
// while the other waits for LDS, memory or the barrier.  The epilogue writes [N][D] rows or, for the fused call,
// the rows' pieces straight into their chunks of the exchange buffer.
// Fallback kernel (any K that is a multiple of 8): global -> registers -> LDS, zero-filled K tail.
// The epilogue rounds to bf16, transposes through the (now idle) LDS and writes whole rows.
#include <type_traits>

#include "internal.h"

namespace cocodiff {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

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
    int32_t bm, bn;            // tile of the launch: tokens x features
    // outputs in exchange-buffer (chunk) order instead of [N][D]: tokens per rank, ranks, 16-byte vectors per
    // chunk row and per chunk, slot order
    uint32_t Ns, P, row8, chunk8;
    int32_t recv_major;
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
    t.m0 = tm * (uint32_t)a.bm;
    t.f0 = (tn - t.tensor * a.tiles_n_per_tensor) * (uint32_t)a.bn;
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

// Epilogue: round to bf16, transpose through this wavefront's private LDS region (ROWS token rows of COLS 16-byte
// feature columns), write whole rows.  An LDS row has CP >= COLS columns, CP a power of two; column c of row r is
// stored at column c ^ (r & (CP - 1)).
template <uint32_t COLS>
struct EpilogueRows {
    static constexpr uint32_t CP = COLS <= 4 ? 4 : COLS <= 8 ? 8 : 16;   // columns per LDS row
    static constexpr uint32_t ROWB = CP * 16;                            // bytes per LDS row
    // four consecutive features (feat a multiple of 4) of LDS row `row`
    static __device__ __forceinline__ void put4(unsigned char* ep, uint32_t row, uint32_t feat, float f0, float f1, float f2, float f3) {
        const uint32_t c16 = feat >> 3, half8 = (feat >> 2) & 1u;
        uint2 v;
        v.x = pack_bf16x2(f0, f1);
        v.y = pack_bf16x2(f2, f3);
        *reinterpret_cast<uint2*>(ep + row * ROWB + (((c16 ^ (row & (CP - 1u))) << 4) | (half8 << 3))) = v;
    }
};

// Second half of the epilogue: the wavefront reads back the rows it staged (a wavefront's LDS accesses complete in
// order: no workgroup barrier is needed) and writes them out.
// PACKED: the 8 features a lane writes for token n = r*Ns + m go to chunk (sender r, receiver p = feature / (Hp*d))
// of the exchange buffer Y, row m (Hp*d is a multiple of 8, so a 16-byte vector never straddles two chunks).
template <uint32_t COLS, uint32_t ROWS, bool PACKED>
__device__ __forceinline__ void store_rows(const unsigned char* ep, uint32_t lane, uint16_t* __restrict__ Y, size_t row0,
                                           uint32_t tok0, uint32_t feat0, uint32_t M, uint32_t D, const GemmArgs& a) {
    constexpr uint32_t CP = EpilogueRows<COLS>::CP, ROWB = EpilogueRows<COLS>::ROWB;
    constexpr uint32_t RPI = 64 / CP;            // rows per read instruction
    const uint32_t c16 = lane % CP, rsub = lane / CP;
#pragma unroll 8
    for (uint32_t it = 0; it < ROWS / RPI; ++it) {
        const uint32_t row = RPI * it + rsub;
        const uint32_t tok = tok0 + row;
        const uint32_t feat = feat0 + c16 * 8u;
        if (c16 < COLS && tok < M && feat < D) {
            const vec16 v = *reinterpret_cast<const vec16*>(ep + row * ROWB + ((c16 ^ (row & (CP - 1u))) << 4));
            if (PACKED) {
                const uint32_t n = (uint32_t)row0 + tok, r = n / a.Ns, m = n - r * a.Ns;
                const uint32_t v8 = feat >> 3, p = v8 / a.row8, c = v8 - p * a.row8;
                const size_t slot = a.recv_major ? (size_t)p * a.P + r : (size_t)r * a.P + p;
                reinterpret_cast<vec16*>(Y)[slot * a.chunk8 + (size_t)m * a.row8 + c] = v;
            } else {
                *reinterpret_cast<vec16*>(Y + (row0 + tok) * D + feat) = v;
            }
        }
    }
}

// 32 x 32 accumulator tiles (v_mfma_f32_32x32x16_bf16): element e of lane l in tile (i, j) is feature
// 32i + 8*(e/4) + 4*(l/32) + e%4 of token 32j + l%32.
template <int NI, int NJ, bool PACKED>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[NI][NJ], unsigned char* ep, uint32_t lane,
                                           uint16_t* __restrict__ Y, size_t row0, uint32_t tok0, uint32_t feat0,
                                           uint32_t M, uint32_t D, const GemmArgs& a) {
    const uint32_t frag_row = lane & 31u, frag_half = lane >> 5;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                EpilogueRows<NI * 4>::put4(ep, 32u * j + frag_row, 32u * i + 8u * g + 4u * frag_half, acc[i][j][4 * g + 0],
                                           acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
    store_rows<NI * 4, NJ * 32, PACKED>(ep, lane, Y, row0, tok0, feat0, M, D, a);
}

// 16 x 16 accumulator tiles (v_mfma_f32_16x16x32_bf16): element e of lane l in tile (i, j) is feature
// 16i + 4*(l/16) + e of token 16j + l%16.
template <int NI, int NJ, bool PACKED>
__device__ __forceinline__ void store_tile16(const f32x4 (&acc)[NI][NJ], unsigned char* ep, uint32_t lane,
                                             uint16_t* __restrict__ Y, size_t row0, uint32_t tok0, uint32_t feat0,
                                             uint32_t M, uint32_t D, const GemmArgs& a) {
    const uint32_t frag_row = lane & 15u, frag_q = lane >> 4;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            EpilogueRows<NI * 2>::put4(ep, 16u * j + frag_row, 16u * i + 4u * frag_q, acc[i][j][0], acc[i][j][1], acc[i][j][2],
                                       acc[i][j][3]);
    store_rows<NI * 2, NJ * 16, PACKED>(ep, lane, Y, row0, tok0, feat0, M, D, a);
}

// s_waitcnt: at most WAIT global->LDS loads of this wavefront still in flight (LDS-read counter untouched)
template <int WAIT>
__device__ __forceinline__ void wait_loads() {
    static_assert(WAIT >= 0 && WAIT < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (WAIT & 15) | ((WAIT >> 4) << 14));
}

// ---------------------------------------------------------------------------------------------
// Main kernel.  A step's X tile and W tile (32 KB each) travel separately through a ring of five LDS
// slots: X of K step kt lives in slot (2kt) % 5, W in slot (2kt + 1) % 5.  A K step is two halves of 32 K
// elements, one v_mfma_f32_16x16x32_bf16 per 16 x 16 output tile and half.  In step kt a wavefront multiplies half 0
// while reading the fragments of half 1, waits until step kt+1 has landed (its own loads; the barrier covers the
// other wavefronts'), then multiplies half 1 while reading half 0 of step kt+1.  After that barrier every
// wavefront is past its last read of step kt, so W of step kt+2 goes into the slot X of step kt used and X of
// step kt+3 into the slot W of step kt used.  The X loads are issued one at a time during half 0, the W loads
// during half 1: a wavefront that issues its eight loads of a step in one burst stalls on the address unit, and the
// MFMAs behind them in program order with it (measured: +340 cycles per step).
// The MFMAs of a half run token tile by token tile: the X fragment of a token tile is dead after NI MFMAs and is
// read again for the next half right there (X fragments need one register set), the NI W fragments live through
// the half and have two sets.  Instruction order inside a half is pinned by a scheduling barrier after every
// instruction group.
// ---------------------------------------------------------------------------------------------
constexpr int kRingSlots = 5;
constexpr int kRingLdsBytes256 = kRingSlots * 256 * BK * 2;   // 160 KB: tiles of 256 x 256
constexpr int kRingLdsBytes192 = kRingSlots * 192 * BK * 2;   // 120 KB: tiles of 192 x 192

__device__ __forceinline__ uint32_t ring_add(uint32_t slot, uint32_t n) {   // (slot + n) % 5 for n <= 5
    const uint32_t t = slot + n;
    return t >= kRingSlots ? t - kRingSlots : t;
}

// One global -> LDS load of 16 bytes per lane: lane l's vector lands at lds_addr + 16*l.  Written as inline
// assembly so that the compiler does not tie later LDS reads to it with a full vmcnt wait (it cannot tell
// that the ring slot being filled is not the one being read); completion is awaited by wait_loads().
__device__ __forceinline__ void load_to_lds(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}

// Tile = (2 * NJ * 16) tokens x (WN * NI * 16) features, square: 256 x 256 with WN = 4, NI = 4, NJ = 8 (8 wavefronts
// of 64 features x 128 tokens) or 192 x 192 with WN = 2, NI = 6, NJ = 6 (4 wavefronts of 96 x 96).
template <int WN, int NI, int NJ, bool PACKED>
__global__ void __launch_bounds__(128 * WN) qkv_gemm_direct_kernel(GemmArgs a) {
    constexpr int WAVES = 2 * WN;
    constexpr int TILE = 2 * NJ * 16;              // tokens = features per tile
    static_assert(TILE == WN * NI * 16, "square tiles only: the ring slots of X and W have one size");
    constexpr int kTileBytes = TILE * BK * 2;      // one operand tile of one K step
    constexpr int NMFMA = NI * NJ;
    constexpr int LOADS = TILE / 8 / WAVES;        // global->LDS instructions per lane per operand per step
    static_assert(LOADS * WAVES * 8 == TILE && NI >= 3 && LOADS <= 2 * NJ && NI <= NJ, "tile shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const TileCoord tc = tile_of_block(a);
    const uint16_t* __restrict__ W = a.w[tc.tensor];
    const uint32_t K = (uint32_t)a.D;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t wave_f = (wave % WN) * (NI * 16u), wave_t = (wave / WN) * (NJ * 16u);

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
    // load i of one operand tile of K step kt into ring slot `slot`
    auto issue_one = [&](const unsigned char* base, const uint32_t (&off)[LOADS], uint32_t kt, uint32_t slot, int i) {
        load_to_lds(base + (size_t)kt * (BK * 2) + off[i], lds0 + slot * kTileBytes + (WAVES * i + wave) * 1024u);
    };
    auto issue_tile = [&](const unsigned char* base, const uint32_t (&off)[LOADS], uint32_t kt, uint32_t slot) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) issue_one(base, off, kt, slot, i);
    };

    // MFMA operand layout: lane l holds 8 K elements (one 16-byte LDS column) of row l%16 of a 16-row fragment, lane
    // group l/16 the g-th eight of the instruction's 32.  Which column of the half a lane group takes is free as long as
    // W and X agree: groups 0, 1, 2, 3 take columns 0, 2, 1, 3, because a 128-bit LDS read serves lanes 8p .. 8p+7
    // together with lanes 32+8p .. 32+8p+7 (groups g and g+2), and rows 0 .. 7 of two columns share no bank only when
    // the columns differ in their lowest bit (measured: 4 conflict cycles per read with columns 0, 1, 2, 3).
    // Fragment addresses: row = wave offset + 16 i + (lane & 15); the swizzle depends on the lane only.
    const uint32_t frag_row = lane & 15u, frag_kg = ((lane >> 3) & 2u) | (lane >> 5);
    const uint32_t sw = swz(frag_row);
    const uint32_t x_frag = (wave_t + frag_row) * 128u;
    const uint32_t w_frag = (wave_f + frag_row) * 128u;
    // X fragment j / W fragment i of half kk of the step whose X tile sits in slot_x (W: the next slot)
    auto read_x = [&](uint32_t slot_x, uint32_t kk, int j) {
        return *reinterpret_cast<const bf16x8*>(smem + slot_x * kTileBytes + x_frag + (((4u * kk + frag_kg) ^ sw) << 4) + j * 2048);
    };
    auto read_w = [&](uint32_t slot_x, uint32_t kk, int i) {
        return *reinterpret_cast<const bf16x8*>(smem + ring_add(slot_x, 1) * kTileBytes + w_frag + (((4u * kk + frag_kg) ^ sw) << 4) + i * 2048);
    };

    f32x4 acc[NI][NJ];   // [feature tile][token tile]
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

    const uint32_t n_k = K / BK;   // >= 3 (the host sends shorter K to the fallback kernel)
    issue_tile(xbase, xoff, 0, 0);
    issue_tile(wbase, woff, 0, 1);
    issue_tile(xbase, xoff, 1, 2);
    issue_tile(wbase, woff, 1, 3);
    wait_loads<2 * LOADS>();       // step 0 has landed; X1, W1 may still be in flight
    __syncthreads();

    bf16x8 wf0[NI], wf1[NI], xf[NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i) wf0[i] = read_w(0, 0, i);
#pragma unroll
    for (int j = 0; j < NJ; ++j) xf[j] = read_x(0, 0, j);

    // One half: MFMA m multiplies W fragment i = m % NI with X fragment j = m / NI.  After the first MFMA of token
    // tile j < NI, W fragment j of the next half is read into wf_n; after the last MFMA of token tile j its X
    // fragment is read again for the next half; after the second (then the third) MFMA of token tile j load
    // number j (NJ + j) of the N_LOADS loads of `base` is issued.  sched_barrier(0) after every group keeps the order.
    auto half = [&](const bf16x8 (&wf)[NI], bf16x8 (&wf_n)[NI], bool read_next, uint32_t slot_n, uint32_t kk_n, auto n_loads_c,
                    const unsigned char* base, const uint32_t (&off)[LOADS], uint32_t kt_l, uint32_t slot_l) {
        constexpr int N_LOADS = decltype(n_loads_c)::value;
#pragma unroll
        for (int m = 0; m < NMFMA; ++m) {
            const int q = m % NI, j = m / NI;                 // q-th MFMA of token tile j
            const int i = (j & 1) ? NI - 1 - q : q;           // W fragments up, then down: one operand is kept at every turn
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (q == 0) {
                if (j < NI && read_next) wf_n[j] = read_w(slot_n, kk_n, j);
            } else if (q == NI - 1) {
                if (read_next) xf[j] = read_x(slot_n, kk_n, j);
            } else if (q <= 2) {
                const int l = (q - 1) * NJ + j;
                if (l < N_LOADS) issue_one(base, off, kt_l, slot_l, l);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // `slot` is the ring slot of X of step kt; W of step kt sits in the next slot.
    // LOAD_X: X of step kt+2 is issued during half 0 (into the slot W of step kt-1 used);
    // LOAD_W: W of step kt+2 is issued during half 1 (into the slot X of step kt used).
    auto k_step = [&](uint32_t kt, uint32_t slot, auto load_x, auto load_w, auto wait, auto next) {
        constexpr bool LOAD_X = decltype(load_x)::value, LOAD_W = decltype(load_w)::value, NEXT = decltype(next)::value;
        constexpr int WAIT = decltype(wait)::value;
        using xl = std::integral_constant<int, LOAD_X ? LOADS : 0>;
        using wl = std::integral_constant<int, LOAD_W ? LOADS : 0>;
        half(wf0, wf1, true, slot, 1, xl{}, xbase, xoff, kt + 2, ring_add(slot, 4));
        if constexpr (NEXT) {
            wait_loads<WAIT>();
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
        half(wf1, wf0, NEXT, ring_add(slot, 2), 0, wl{}, wbase, woff, kt + 2, slot);
    };
    using yes = std::true_type;
    using no = std::false_type;
    const std::integral_constant<int, 0> w0;
    const std::integral_constant<int, LOADS> w1;      // the X tile of the step after next may still be in flight
    uint32_t kt = 0, slot = 0;
    auto advance = [&]() {
        ++kt;
        slot = ring_add(slot, 2);
    };
    // At the barrier of step kt the loads in flight, oldest first, are X(kt+1), W(kt+1), X(kt+2): the last may stay.
    while (kt + 2 < n_k) {
        k_step(kt, slot, yes{}, yes{}, w1, yes{});
        advance();
    }
    k_step(kt, slot, no{}, no{}, w0, yes{});     // step n_k-2: the last step must have landed completely
    advance();
    k_step(kt, slot, no{}, no{}, w0, no{});      // step n_k-1
    __syncthreads();
    constexpr int kEpilogueBytes = NJ * 16 * EpilogueRows<NI * 2>::ROWB;   // per wavefront, see store_tile16
    static_assert(WAVES * kEpilogueBytes <= kRingSlots * kTileBytes, "the epilogue reuses the ring's LDS");
    store_tile16<NI, NJ, PACKED>(acc, smem + wave * kEpilogueBytes, lane, a.y[tc.tensor], (size_t)a.row_begin,
                                 tc.m0 + wave_t, tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D, a);
}

// ---------------------------------------------------------------------------------------------
// General path, any K that is a multiple of 8: global -> registers -> LDS, vectors beyond K are zero.
// Four wavefronts (2 x 2) of 128 x 128 outputs.
// ---------------------------------------------------------------------------------------------
constexpr int kStagedThreads = 256;
constexpr int kVecPerOperand = BM * (BK / 8) / kStagedThreads;   // 16-byte vectors per lane per operand per stage: 8

template <bool PACKED>
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
    store_tile<4, 4, PACKED>(acc, smem + wave * (128 * 256), lane, a.y[tc.tensor], (size_t)a.row_begin, tc.m0 + wave_t,
                          tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D, a);
}


}  // namespace cocodiff

using namespace cocodiff;

// packed = false: q, k, v are [N][D].  packed = true: they are exchange buffers, written in chunk order.
static int proj_launch(const cocodiff_shape* shape, const cocodiff_bf16* x,
                       const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                       cocodiff_bf16* q, cocodiff_bf16* k, cocodiff_bf16* v, bool packed, int slot_order, void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (packed && slot_order != COCODIFF_SEND_MAJOR && slot_order != COCODIFF_RECV_MAJOR)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_pack: slot_order (%d) must be SEND_MAJOR or RECV_MAJOR", slot_order);
    if (!x) return fail(COCODIFF_ERR_NULL, "qkv_proj: x is NULL");
    if ((wq == nullptr) != (q == nullptr) || (wk == nullptr) != (k == nullptr) || (wv == nullptr) != (v == nullptr))
        return fail(COCODIFF_ERR_NULL, "qkv_proj: a weight and its output must be given together");
    if (!q && !k && !v) return fail(COCODIFF_ERR_NULL, "qkv_proj: no (weight, output) pair given");
    if (!aligned16(x) || !aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(q) || !aligned16(k) || !aligned16(v))
        return fail(COCODIFF_ERR_ALIGN, "qkv_proj: pointers must be 16-byte aligned");

    GemmArgs a;
    a.Ns = (uint32_t)(shape->N / shape->P);
    a.P = (uint32_t)shape->P;
    a.row8 = (uint32_t)(shape->H / shape->P) * (uint32_t)(shape->d / 8);
    a.chunk8 = a.Ns * a.row8;
    a.recv_major = slot_order == COCODIFF_RECV_MAJOR;
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
    if ((int64_t)BM * a.D * 2 >= ((int64_t)1 << 32)) return fail(COCODIFF_ERR_SHAPE, "qkv_proj: D (%d) too large", a.D);
    const bool ring_kernel = a.D % BK == 0 && a.D >= 3 * BK;

    // Tile shape: 256 x 256 does the least operand traffic per flop; 192 x 192 is taken when its tile count fills
    // the compute units so much better that it wins all the same (small token counts).  Cost = rounds x tile area,
    // x 1.2 for the smaller tile (measured: per flop it is that much slower on this power-limited part, so three
    // full rounds of it only tie with two ragged rounds of the large one), a round being one tile on every unit.
    static const int n_cu = [] {     // asked once (thread-safe initialisation); 0 = could not be read
        int dev = 0, val = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&val, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return val;
    }();
    if (n_cu <= 0) return fail(COCODIFF_ERR_HIP, "qkv_proj: cannot read the compute-unit count");
    auto tiles_of = [&](int t) { return (int64_t)((a.M + t - 1) / t) * ((a.D + t - 1) / t) * a.n_tensors; };
    auto rounds_of = [&](int t) { return (tiles_of(t) + n_cu - 1) / n_cu; };
    const double cost256 = (double)rounds_of(256) * 256.0 * 256.0;
    const double cost192 = (double)rounds_of(192) * 192.0 * 192.0 * 1.2;
    static const int forced_tile = (int)tune_value("COCODIFF_GEMM_TILE", 0);      // tuning knob: 192 or 256
    const bool small_tile = ring_kernel && (forced_tile ? forced_tile == 192 : cost192 < cost256);
    a.bm = a.bn = small_tile ? 192 : 256;
    a.tiles_m = (a.M + a.bm - 1) / a.bm;
    a.tiles_n_per_tensor = (a.D + a.bn - 1) / a.bn;
    const uint32_t n_tiles = (uint32_t)a.tiles_m * a.tiles_n_per_tensor * a.n_tensors;

    // dynamic LDS above 64 KB needs the attribute, once per process (thread-safe initialisation)
    static const hipError_t attr_rc = [] {
        hipError_t e = hipSuccess;
        const void* big[2] = {(const void*)qkv_gemm_direct_kernel<4, 4, 8, false>, (const void*)qkv_gemm_direct_kernel<4, 4, 8, true>};
        const void* small[2] = {(const void*)qkv_gemm_direct_kernel<2, 6, 6, false>, (const void*)qkv_gemm_direct_kernel<2, 6, 6, true>};
        const void* staged[2] = {(const void*)qkv_gemm_staged_kernel<false>, (const void*)qkv_gemm_staged_kernel<true>};
        for (int i = 0; i < 2 && e == hipSuccess; ++i) {
            e = hipFuncSetAttribute(big[i], hipFuncAttributeMaxDynamicSharedMemorySize, kRingLdsBytes256);
            if (e == hipSuccess) e = hipFuncSetAttribute(small[i], hipFuncAttributeMaxDynamicSharedMemorySize, kRingLdsBytes192);
            if (e == hipSuccess) e = hipFuncSetAttribute(staged[i], hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        }
        return e;
    }();
    if (attr_rc != hipSuccess) return fail(COCODIFF_ERR_HIP, "qkv_proj: cannot reserve LDS: %s", hipGetErrorString(attr_rc));
    hipStream_t st = as_stream(stream);
    if (ring_kernel && small_tile && packed)
        hipLaunchKernelGGL((qkv_gemm_direct_kernel<2, 6, 6, true>), dim3(n_tiles), dim3(256), kRingLdsBytes192, st, a);
    else if (ring_kernel && small_tile)
        hipLaunchKernelGGL((qkv_gemm_direct_kernel<2, 6, 6, false>), dim3(n_tiles), dim3(256), kRingLdsBytes192, st, a);
    else if (ring_kernel && packed)
        hipLaunchKernelGGL((qkv_gemm_direct_kernel<4, 4, 8, true>), dim3(n_tiles), dim3(512), kRingLdsBytes256, st, a);
    else if (ring_kernel)
        hipLaunchKernelGGL((qkv_gemm_direct_kernel<4, 4, 8, false>), dim3(n_tiles), dim3(512), kRingLdsBytes256, st, a);
    else if (packed)
        hipLaunchKernelGGL(qkv_gemm_staged_kernel<true>, dim3(n_tiles), dim3(kStagedThreads), kLdsBytes, st, a);
    else
        hipLaunchKernelGGL(qkv_gemm_staged_kernel<false>, dim3(n_tiles), dim3(kStagedThreads), kLdsBytes, st, a);
    return check_launch("qkv_gemm_kernel");
}

extern "C" int cocodiff_qkv_proj(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                 const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                 cocodiff_bf16* q, cocodiff_bf16* k, cocodiff_bf16* v, void* stream) {
    return proj_launch(shape, x, wq, wk, wv, q, k, v, false, COCODIFF_SEND_MAJOR, stream);
}

extern "C" int cocodiff_qkv_proj_pack(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                      const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                      cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order, void* stream) {
    return proj_launch(shape, x, wq, wk, wv, qbuf, kbuf, vbuf, true, slot_order, stream);
}
