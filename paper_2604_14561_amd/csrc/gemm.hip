// QKV projection (paper Section II-B): Y[n][o] = sum_k X[n][k] * W[o][k], bf16 in, fp32 accumulate on the
// gfx950 matrix cores, one RNE rounding to bf16.  The main kernel multiplies with v_mfma_f32_16x16x32_bf16: on this
// power-limited part it sustains 1.91 PFLOP/s at 0.70 pJ/flop in a register-only loop against 1.72 PFLOP/s at
// 0.77 pJ/flop for v_mfma_f32_32x32x16_bf16, for the same LDS traffic per flop (a wavefront's tile decides that).
//
// Workgroup tile (tokens x features): 256 x 256, 288 x 192 or 192 x 192 -- the host takes the one with the fewest
// rounds of tiles over the compute units, weighted by a measured per-flop cost (plan_launch).  K step 64: a row
// segment of either operand is one whole 128-byte line (half lines halve the L1 fill rate).  W rides the MFMA "A"
// side, so an accumulator lane holds four consecutive features of one token.  Both operands are K-contiguous; LDS
// tiles keep rows contiguous and store 16-byte column c of row r at column c ^ swz(r), which makes the 128-bit
// fragment reads bank-conflict free.
//
// Main kernel (K a multiple of 64, at least three steps): global -> LDS directly (no staging registers) through two
// rings, three slots for X tiles and two for W tiles (160 KB for the 256 x 256 tile).  Eight wavefronts, four along
// the features x two along the tokens, two per SIMD, so one can multiply while the other waits for LDS, memory or
// the barrier.  General kernel (any K that is a multiple of 8): global -> registers -> LDS, zero-filled K tail.
// The epilogue rounds to bf16, transposes through the (now idle) LDS and writes 16-byte vectors: rows of [N][D],
// row pieces straight into their chunks of the exchange buffer, or row pieces of the head-parallel tensor -- or, in
// the fused form (tiles 256 features wide, so that they hold whole heads), it first RMS-normalises and rotates Q and K
// on the fp32 accumulators (paper Section II-B's norm and RoPE, one rounding in all) and writes both the chunks and
// the head-parallel tensor.
#include <initializer_list>
#include <type_traits>

#include "internal.h"

namespace cocodiff {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int BM = 256;          // tokens per workgroup tile
constexpr int BK = 64;           // K elements per step
constexpr int kTileBytes = BM * BK * 2;                  // one operand tile of one K step of the fallback kernel: 32 KB
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
    // outputs in head-parallel order [H][N][d]: all tokens, 16-byte vectors per head row
    uint32_t N_all, d8;
    // OUT_FUSED: second destination (head-parallel; y[] is then the exchange buffer; either may be null), RMSNorm + RoPE
    // of the tensors that have a gamma
    uint16_t* y2[3];
    const uint16_t* gamma[3];
    uint32_t d;                // features per head
    float inv_d, eps;
    RopeDev rope;
    // How the normalising epilogue walks the rotation table, in floats: axis x' rows start at row_base[x], row_stride[x]
    // apart, row_span[x] = grid x stride in all, up to row_end[x] (absent axes: never reached); row_step16[x] = the axis' digit of 16 tokens in the grid's mixed radix
    // (last axis fastest) times the stride.  tab_lds != 0: every workgroup that normalises stages the table in LDS, rows
    // 2 pairs + 2 floats apart (the two extra floats spread consecutive rows over the banks), and the four arrays describe
    // that copy; axis x is pairs [tab_cum[x], ...) of the caller's table and tab_magic[x] = ceil(2^32 / pairs[x])
    // divides a pair index by the row length.  tab_lds == 0: the arrays describe the caller's table in global memory.
    // The fused call that also flags V for the selection (sel_prev != nullptr): the previous step's V in the head-parallel
    // layout, the decision's thresholds, and the flag records: 16 bytes per 16-token tile, byte c written by the workgroup
    // of V's feature tile c.  sel_tiles = N / 16.
    const uint16_t* sel_prev;
    uint8_t* sel_flag_bytes;
    Thresholds sel_th;
    uint32_t sel_tiles;
    uint32_t tab_lds, row_base[3], row_stride[3], row_span[3], row_end[3], row_step16[3], tab_cum[3], tab_magic[3];
};

// Where the epilogue writes: token-major [N][D]; the exchange-buffer chunks of the first all-to-all; or the
// head-parallel tensor [H][N][d] that all-to-all ends in (pack, exchange and unpack folded into the store address).
// OUT_FUSED: Q and K are normalised and rotated in the epilogue (on the fp32 accumulators), and every tensor goes to its
// exchange buffer and to its head-parallel tensor (whichever are given).
enum OutLayout { OUT_SEQ = 0, OUT_CHUNKS = 1, OUT_HEADS = 2, OUT_FUSED = 3 };

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
// order: no workgroup barrier is needed) and writes them out, RPI rows per instruction.  A lane keeps its 16-byte
// feature column and walks down the rows, so every destination address is formed once (the divisions below) and then
// stepped: the epilogue's time is its instruction count, not the stores' bandwidth.
// OUT_CHUNKS: the 8 features a lane writes for token n = r*Ns + m go to chunk (sender r, receiver p = feature / (Hp*d))
// of the exchange buffer Y, row m (Hp*d is a multiple of 8, so a 16-byte vector never straddles two chunks); RPI rows
// further down is RPI chunk rows further, and into sender r+1's chunk where m passes Ns (Ns >= 16 >= RPI: once at most).
// OUT_HEADS: they go to row n of head feature / d of Y = [H][N][d] (d is a multiple of 8).
// Cache policy of the stores: what a kernel of the same step reads next stays cached -- [N][D], the head-parallel V (the
// selection reads it), and the exchange buffer of cocodiff_qkv_proj_pack (its unpack follows: with streaming stores the
// steps through it were 2 - 3.5 % slower).  In the fused call nothing on this GPU reads the exchange buffers (they are
// what the all-to-all would send) or, within the step, the head-parallel Q and K (NT_HEADS): streamed past the caches
// they leave nothing dirty in L2 to be written back under the next round's loads (three-weight launch at 20736 tokens:
// 970 -> 941 us).
template <uint32_t COLS, uint32_t ROWS, int LAYOUT, bool NT_HEADS = false>
__device__ __forceinline__ void store_rows(const unsigned char* ep, uint32_t lane, uint16_t* __restrict__ Y, uint16_t* __restrict__ Y2,
                                           size_t row0, uint32_t tok0, uint32_t feat0, uint32_t M, uint32_t D, const GemmArgs& a) {
    constexpr uint32_t CP = EpilogueRows<COLS>::CP, ROWB = EpilogueRows<COLS>::ROWB;
    constexpr uint32_t RPI = 64 / CP;            // rows per read instruction
    static_assert(RPI <= 16 && ROWS % RPI == 0, "a lane moves at most one sender's chunk further per step");
    const uint32_t c16 = lane % CP, rsub = lane / CP;
    const uint32_t feat = feat0 + c16 * 8u;
    if (c16 >= COLS || feat >= D) return;
    const bool to_chunks = LAYOUT == OUT_CHUNKS || (LAYOUT == OUT_FUSED && Y);
    const bool to_heads = LAYOUT == OUT_HEADS || (LAYOUT == OUT_FUSED && Y2);
    uint32_t tok = tok0 + rsub;
    const uint32_t n = (uint32_t)row0 + tok, v8 = feat >> 3;
    vec16* yc = nullptr;       // exchange buffer
    vec16* yh = nullptr;       // head-parallel tensor, or the token-major one
    uint32_t m = 0;
    size_t step_c = 0, wrap_c = 0, step_h = 0;
    if (to_chunks) {
        const uint32_t r = n / a.Ns, p = v8 / a.row8, c = v8 - p * a.row8;
        m = n - r * a.Ns;
        const size_t slot = a.recv_major ? (size_t)p * a.P + r : (size_t)r * a.P + p;
        yc = reinterpret_cast<vec16*>(Y) + slot * a.chunk8 + (size_t)m * a.row8 + c;
        step_c = (size_t)RPI * a.row8;
        wrap_c = a.recv_major ? 0 : (size_t)(a.P - 1u) * a.chunk8;      // slot(r + 1) - slot(r) chunks, less the Ns rows stepped over
    }
    if (to_heads) {
        const uint32_t h = v8 / a.d8, c = v8 - h * a.d8;
        yh = reinterpret_cast<vec16*>(LAYOUT == OUT_HEADS ? Y : Y2) + ((size_t)h * a.N_all + n) * a.d8 + c;
        step_h = (size_t)RPI * a.d8;
    }
    if (LAYOUT == OUT_SEQ) {
        yh = reinterpret_cast<vec16*>(Y + (row0 + tok) * D + feat);
        step_h = (size_t)RPI * (D / 8u);
    }
#pragma unroll 8
    for (uint32_t it = 0; it < ROWS / RPI; ++it) {
        if (tok < M) {
            const uint32_t row = RPI * it + rsub;
            const vec16 v = *reinterpret_cast<const vec16*>(ep + row * ROWB + ((c16 ^ (row & (CP - 1u))) << 4));
            if (to_chunks) st_vec<LAYOUT == OUT_FUSED>(yc, v);
            if (to_heads || LAYOUT == OUT_SEQ) st_vec<NT_HEADS>(yh, v);
        }
        tok += RPI;
        yh += step_h;
        if (to_chunks) {
            yc += step_c;
            m += RPI;
            if (m >= a.Ns) {
                m -= a.Ns;
                yc += wrap_c;
            }
        }
    }
}

// store_rows for V in the fused call when the selection's flags are wanted too (paper Section III-D): every vector on
// its way out is compared with the previous step's vector at the same place of the head-parallel layout (the decision
// of the selection's flag pass: one streaming compare per element, the exact rule for suspects), and the wavefront
// notes per 16-token tile -- two consecutive row groups -- whether anything changed, in `changed_lds`
// ([wavefront][tile]: one byte-sized word each).  Both destinations must be given.
// prev_rows: the lane's vectors of the previous step's V, fetched by load_prev_rows before the tile was staged (one
// trip to memory for the whole tile, under the staging work, instead of one per group of rows).
template <uint32_t ROWS>
__device__ __forceinline__ void load_prev_rows(vec16 (&prev_rows)[ROWS / 8], uint32_t lane, size_t row0, uint32_t tok0, uint32_t feat0,
                                               uint32_t M, uint32_t D, const GemmArgs& a) {
    const uint32_t c16 = lane % 8u, rsub = lane / 8u;
    const uint32_t feat = min(feat0 + c16 * 8u, D - 8u);
    const bool live = feat0 + c16 * 8u < D;
    const uint32_t tok = tok0 + rsub, n = (uint32_t)row0 + tok, v8 = feat >> 3;
    const uint32_t h = v8 / a.d8, ch = v8 - h * a.d8;
    const vec16* yp = reinterpret_cast<const vec16*>(a.sel_prev) + ((size_t)h * a.N_all + n) * a.d8 + ch;
#pragma unroll
    for (uint32_t it = 0; it < ROWS / 8; ++it)
        if (live && tok + 8u * it < M) prev_rows[it] = ld_nt(yp + (size_t)(8u * it) * a.d8);
}

template <uint32_t ROWS>
__device__ __forceinline__ void store_rows_select(const unsigned char* ep, uint32_t lane, uint32_t wave, uint16_t* __restrict__ Y,
                                                  uint16_t* __restrict__ Y2, size_t row0, uint32_t tok0, uint32_t feat0, uint32_t M,
                                                  uint32_t D, const GemmArgs& a, uint32_t* changed_lds, const vec16 (&prev_rows)[ROWS / 8]) {
    constexpr uint32_t COLS = 8, ROWB = EpilogueRows<COLS>::ROWB, RPI = 8;
    static_assert(EpilogueRows<COLS>::CP == 8 && ROWS % 16 == 0, "eight rows per read instruction, whole 16-token tiles");
    const uint32_t c16 = lane % 8u, rsub = lane / 8u;
    const uint32_t feat = min(feat0 + c16 * 8u, D - 8u);         // lanes past the last feature idle on a valid address
    const bool live = feat0 + c16 * 8u < D;
    uint32_t tok = tok0 + rsub;
    const uint32_t n = (uint32_t)row0 + tok, v8 = feat >> 3;
    const uint32_t r = n / a.Ns, p = v8 / a.row8, c = v8 - p * a.row8;
    uint32_t m = n - r * a.Ns;
    const size_t slot = a.recv_major ? (size_t)p * a.P + r : (size_t)r * a.P + p;
    vec16* yc = reinterpret_cast<vec16*>(Y) + slot * a.chunk8 + (size_t)m * a.row8 + c;
    const size_t step_c = (size_t)RPI * a.row8, wrap_c = a.recv_major ? 0 : (size_t)(a.P - 1u) * a.chunk8;
    const uint32_t h = v8 / a.d8, ch = v8 - h * a.d8;
    const size_t hs_at = ((size_t)h * a.N_all + n) * a.d8 + ch;
    vec16* yh = reinterpret_cast<vec16*>(Y2) + hs_at;
    const size_t step_h = (size_t)RPI * a.d8;
    bool changed = false;
#pragma unroll
    for (uint32_t it = 0; it < ROWS / RPI; ++it) {
        if (live && tok < M) {
            const uint32_t row = RPI * it + rsub;
            const vec16 v = *reinterpret_cast<const vec16*>(ep + row * ROWB + ((c16 ^ (row & 7u)) << 4));
            const vec16 pv = prev_rows[it];
            st_nt(yc, v);
            *yh = v;
            if (vec_suspect(v, pv, a.sel_th.tau_s)) {
                bool tie = false;
                bool chg = vec_changed(v, pv, a.sel_th.tau, a.sel_th.tau_tie, tie);
                if (tie && !chg) chg = vec_changed_double(v, pv, a.sel_th.tau);
                changed |= chg;
            }
        }
        tok += RPI;
        yh += step_h;
        yc += step_c;
        m += RPI;
        if (m >= a.Ns) {
            m -= a.Ns;
            yc += wrap_c;
        }
        if (it & 1u) {        // rows 16 (it/2) .. +15 are done: one tile of the selection
            const bool any = __ballot(changed) != 0;
            if (lane == 0) changed_lds[wave * (ROWS / 16u) + it / 2u] = any ? 1u : 0u;
            changed = false;
        }
    }
}

// 32 x 32 accumulator tiles (v_mfma_f32_32x32x16_bf16): element e of lane l in tile (i, j) is feature
// 32i + 8*(e/4) + 4*(l/32) + e%4 of token 32j + l%32.
template <int NI, int NJ, int LAYOUT>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[NI][NJ], unsigned char* ep, uint32_t lane,
                                           uint16_t* __restrict__ Y, uint16_t* __restrict__ Y2, size_t row0, uint32_t tok0,
                                           uint32_t feat0, uint32_t M, uint32_t D, const GemmArgs& a) {
    const uint32_t frag_row = lane & 31u, frag_half = lane >> 5;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                EpilogueRows<NI * 4>::put4(ep, 32u * j + frag_row, 32u * i + 8u * g + 4u * frag_half, acc[i][j][4 * g + 0],
                                           acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
    store_rows<NI * 4, NJ * 32, LAYOUT>(ep, lane, Y, Y2, row0, tok0, feat0, M, D, a);
}

// 16 x 16 accumulator tiles (v_mfma_f32_16x16x32_bf16): element e of lane l in tile (i, j) is feature
// 16i + 4*(l/16) + e of token 16j + l%16.
template <int NI, int NJ>
__device__ __forceinline__ void stage_tile16(const f32x4 (&acc)[NI][NJ], unsigned char* ep, uint32_t lane) {
    const uint32_t frag_row = lane & 15u, frag_q = lane >> 4;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            EpilogueRows<NI * 2>::put4(ep, 16u * j + frag_row, 16u * i + 4u * frag_q, acc[i][j][0], acc[i][j][1], acc[i][j][2],
                                       acc[i][j][3]);
}

// RMSNorm over every head row and RoPE, on a wavefront's fp32 accumulators (NI feature tiles x NJ token tiles of 16 x 16:
// lane l holds features 16i + 4(l/16) + e, e = 0..3, of token 16j + l%16), in the arithmetic order of the stand-alone
// norm + RoPE kernel (x * rinv * gamma, then the rotation) -- but on the unrounded projection, so Q and K are rounded
// to bf16 once instead of twice -- and straight on through the epilogue's staging rows to both destinations.
// A head of d features is `d / (16 NI)` wavefronts wide (1, 2 or 4, neighbours along the features): each writes its
// partial sums of squares to `xch` ([wavefront][token]) and, after a workgroup barrier, adds the group's partial sums
// in a fixed order, so every wavefront of a head works with the same bits.
// The rotation table: where it fits beside the staging rows (IN_LDS) the workgroup copies it into LDS (`tab`) while the
// sums of squares are formed, and the barrier publishes it; a token's (cos, sin) values then cost an LDS read instead
// of a trip to L2.  Otherwise they are loaded from global memory one token tile ahead.
// This stage's time is its instruction count (the workgroup's successor cannot start before it ends, and nothing else
// runs on the unit), so the token's grid coordinates are divided out once, for token tile 0, and then stepped as table
// row offsets: 16 tokens further is a.row_step16[] further in mixed radix, with carries (the absent axes of a one- or
// two-axis grid are grids of one cell behind the last axis: they never carry).
// The token tiles go through the staging rows in two halves (the first (NJ+1)/2, then the rest), which is what leaves
// room for the table; a token tile's accumulators are dead once it is staged, so the whole thing fits the registers
// the K loop had.
// tile_m0: the tile's first token within the launch's rows; tok0 / feat0: the wavefront's first token within the launch's
// rows / first feature within its tensor.  Rows past the
// launch's last token (ragged tile; never stored) rotate by some row of the table.
template <int NI, int NJ, int WN, bool IN_LDS>
__device__ __forceinline__ void norm_rope_store(f32x4 (&acc)[NI][NJ], unsigned char* ep, float* xch, float* tab, const GemmArgs& a,
                                                const uint16_t* __restrict__ gamma, uint16_t* __restrict__ Y, uint16_t* __restrict__ Y2,
                                                uint32_t lane, uint32_t wave, uint32_t tile_m0, uint32_t tok0, uint32_t feat0) {
    constexpr uint32_t WF = NI * 16;                 // features per wavefront
    constexpr int JH = (NJ + 1) / 2;                 // token tiles in the first half
    const uint32_t g4 = lane >> 4, tl = lane & 15u;
    if (IN_LDS) {
        // Only the table rows the tile's tokens touch are copied (each to its usual place): along an axis the tile's
        // consecutive tokens cover consecutive coordinates, `span` of them from `first` on, wrapping -- all rows of the
        // fastest axis as a rule, two to four of the others: about half of the table.
        const float2* __restrict__ src = reinterpret_cast<const float2*>(a.rope.cs);
        uint32_t lo = (uint32_t)a.row_begin + tile_m0;
        uint32_t hi = min(lo + 2u * NJ * 16u, (uint32_t)a.row_begin + (uint32_t)a.M) - 1u;
        uint32_t first[3], span[3];
#pragma unroll
        for (int x = 2; x >= 0; --x) {
            const uint32_t g = (uint32_t)a.rope.grid[x];      // absent axes: 1
            first[x] = lo % g;
            span[x] = min(hi - lo + 1u, g);
            lo /= g;
            hi /= g;
        }
#pragma unroll
        for (int x = 0; x < 3; ++x) {
            if (x >= a.rope.n_axes) continue;
            const uint32_t g = (uint32_t)a.rope.grid[x], pr = (uint32_t)a.rope.pairs[x], count = span[x] * pr;
            float* dst = tab + a.row_base[x];
#pragma unroll 4
            for (uint32_t e = wave * 64u + lane; e < count; e += 128u * WN) {
                const uint32_t k = __umulhi(e, a.tab_magic[x]);             // e / pairs[x]
                const uint32_t p = e - k * pr;
                uint32_t r = first[x] + k;
                r -= r >= g ? g : 0u;
                *reinterpret_cast<float2*>(dst + r * a.row_stride[x] + 2u * p) = src[a.tab_cum[x] + r * pr + p];
            }
        }
    }
    float rinv[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) s += acc[i][j][e] * acc[i][j][e];
        s += __shfl_xor(s, 16, 64);
        s += __shfl_xor(s, 32, 64);
        rinv[j] = s;
    }
    const uint32_t group = a.d / WF;                 // the same for the whole launch
    if (group > 1 && lane < 16) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) xch[wave * (NJ * 16) + 16 * j + lane] = rinv[j];
    }
    if (IN_LDS || group > 1) __syncthreads();
    if (group > 1) {
        const uint32_t wf = wave % WN;
        const uint32_t w0 = wave - wf + (wf / group) * group;     // the head's first wavefront (same token half)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float s = 0.f;
            for (uint32_t w = 0; w < group; ++w) s += xch[(w0 + w) * (NJ * 16) + 16 * j + tl];
            rinv[j] = s;
        }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) rinv[j] = 1.0f / sqrtf(rinv[j] * a.inv_d + a.eps);

    // the lane's 2 NI rotary pairs (two per feature tile): which axis' table, and the float offset inside a table row
    const uint32_t fh0 = feat0 % a.d + 4u * g4;      // this lane's first feature inside its head, for feature tile 0
    const uint32_t p0 = (uint32_t)a.rope.pairs[0], p01 = p0 + (uint32_t)a.rope.pairs[1];
    uint32_t axis[NI][2], col[NI][2];
    float g[NI][4];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const uint2 gw = *reinterpret_cast<const uint2*>(gamma + fh0 + 16u * i);
        g[i][0] = bf16_lo(gw.x); g[i][1] = bf16_hi(gw.x); g[i][2] = bf16_lo(gw.y); g[i][3] = bf16_hi(gw.y);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const uint32_t jl = (fh0 + 16u * i) / 2u + q;         // pair index inside the head
            axis[i][q] = a.rope.n_axes > 2 && jl >= p01 ? 2u : a.rope.n_axes > 1 && jl >= p0 ? 1u : 0u;
            col[i][q] = 2u * (jl - (axis[i][q] == 2u ? p01 : axis[i][q] == 1u ? p0 : 0u));
        }
    }
    // float offsets of the token's row in each axis' table, for this lane's token of token tile 0
    uint32_t row_a[3];
    {
        uint32_t rem = (uint32_t)a.row_begin + tok0 + tl;
        const uint32_t c2 = rem % (uint32_t)a.rope.grid[2];
        rem /= (uint32_t)a.rope.grid[2];
        const uint32_t c1 = rem % (uint32_t)a.rope.grid[1];
        rem /= (uint32_t)a.rope.grid[1];
        row_a[0] = a.row_base[0] + rem * a.row_stride[0];
        row_a[1] = a.row_base[1] + c1 * a.row_stride[1];
        row_a[2] = a.row_base[2] + c2 * a.row_stride[2];
    }
    const uint32_t end0 = a.row_end[0] - a.row_stride[0];     // the table's last row of axis 0
    // (cos, sin) of the lane's pairs for its token of the current token tile; then on to the next tile's token
    auto load_cs = [&](float2 (&cs)[NI][2]) {
        const uint32_t r0 = min(row_a[0], end0), r1 = row_a[1], r2 = row_a[2];
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const uint32_t off = (axis[i][q] == 0 ? r0 : axis[i][q] == 1 ? r1 : r2) + col[i][q];
                if (IN_LDS)
                    cs[i][q] = *reinterpret_cast<const float2*>(tab + off);
                else
                    cs[i][q] = *reinterpret_cast<const float2*>(a.rope.cs + off);
            }
        row_a[2] += a.row_step16[2];
        const bool carry2 = row_a[2] >= a.row_end[2];
        row_a[2] -= carry2 ? a.row_span[2] : 0u;
        row_a[1] += a.row_step16[1] + (carry2 ? a.row_stride[1] : 0u);
        const bool carry1 = row_a[1] >= a.row_end[1];
        row_a[1] -= carry1 ? a.row_span[1] : 0u;
        row_a[0] += a.row_step16[0] + (carry1 ? a.row_stride[0] : 0u);
    };
    auto rotate_stage = [&](int j, const float2 (&cs)[NI][2]) {
        const uint32_t row = 16u * (j < JH ? j : j - JH) + tl;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            float o[4];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const float ev = acc[i][j][2 * q] * rinv[j] * g[i][2 * q];
                const float od = acc[i][j][2 * q + 1] * rinv[j] * g[i][2 * q + 1];
                o[2 * q] = ev * cs[i][q].x - od * cs[i][q].y;
                o[2 * q + 1] = ev * cs[i][q].y + od * cs[i][q].x;
            }
            EpilogueRows<NI * 2>::put4(ep, row, 16u * i + 4u * g4, o[0], o[1], o[2], o[3]);
        }
        // a half is complete: out it goes (this wavefront's LDS accesses complete in order, so the next half may
        // overwrite the rows right away)
        if (j == JH - 1)
            store_rows<NI * 2, JH * 16, OUT_FUSED, true>(ep, lane, Y, Y2, (size_t)a.row_begin, tok0, feat0, (uint32_t)a.M, (uint32_t)a.D, a);
        if (j == NJ - 1 && NJ > JH)
            store_rows<NI * 2, (NJ - JH) * 16, OUT_FUSED, true>(ep, lane, Y, Y2, (size_t)a.row_begin, tok0 + JH * 16u, feat0, (uint32_t)a.M,
                                                          (uint32_t)a.D, a);
    };
    float2 cs_a[NI][2], cs_b[NI][2];
    load_cs(cs_a);
#pragma unroll
    for (int j = 0; j < NJ; j += 2) {
        if (j + 1 < NJ) load_cs(cs_b);
        __builtin_amdgcn_sched_barrier(0);
        rotate_stage(j, cs_a);
        __builtin_amdgcn_sched_barrier(0);
        if (j + 1 < NJ) {
            if (j + 2 < NJ) load_cs(cs_a);
            __builtin_amdgcn_sched_barrier(0);
            rotate_stage(j + 1, cs_b);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// s_waitcnt: at most WAIT global->LDS loads of this wavefront still in flight (LDS-read counter untouched)
template <int WAIT>
__device__ __forceinline__ void wait_loads() {
    static_assert(WAIT >= 0 && WAIT < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (WAIT & 15) | ((WAIT >> 4) << 14));
}

// ---------------------------------------------------------------------------------------------
// Main kernel.  A step's X tile and W tile travel through two rings in LDS: three slots for X (X of K step kt in
// slot kt % 3) and two for W (slot kt % 2) -- 160 KB for a 256 x 256 tile (five times 32 KB), 156 KB for 288 tokens x
// 192 features (3 x 36 + 2 x 24 KB).  A K step is two halves of 32 K elements, one v_mfma_f32_16x16x32_bf16 per
// 16 x 16 output tile and half.  In step kt a wavefront multiplies half 0 while reading the fragments of half 1,
// waits until step kt+1 has landed (its own loads; the barrier covers the other wavefronts'), then multiplies half 1
// while reading half 0 of step kt+1.  After that barrier every wavefront is past its last read of step kt, so W of
// step kt+2 goes into the W slot of step kt (during half 1 of step kt) and X of step kt+3 into its X slot (during
// half 0 of step kt+1).  The loads are issued one at a time between the MFMAs: a wavefront that issues its eight
// loads of a step in one burst stalls on the address unit, and the MFMAs behind them in program order with it
// (measured: +340 cycles per step).
// The MFMAs of a half run token tile by token tile: the X fragment of a token tile is dead after NI MFMAs and is
// read again for the next half right there (X fragments need one register set), the NI W fragments live through
// the half and have two sets.  Instruction order inside a half is pinned by a scheduling barrier after every
// instruction group.
// ---------------------------------------------------------------------------------------------
constexpr int kXSlots = 3, kWSlots = 2;
constexpr double kPenalty288 = 1.07;   // measured per-flop cost of the 288 x 192 tile against 256 x 256 (4.5 - 8 %):
                                       // 11 % more operand bytes into LDS and 18 % more fragment reads per flop
constexpr double kPenalty192 = 1.2;    // 192 x 192: a third more operand bytes and twice the fragment reads per flop
constexpr int ring_lds_bytes(int bm, int bn) { return (kXSlots * bm + kWSlots * bn) * BK * 2; }
// Floats of LDS left for the rotation table in a normalising tile of the fused call (bn = 256: 8 wavefronts of 64
// features x bm/2 tokens): the ring minus a half tile of 128-byte staging rows and bm/2 partial sums per wavefront.
constexpr int fused_table_floats(int bm, int bn) { return (ring_lds_bytes(bm, bn) - 8 * ((bm / 32 + 1) / 2 * 16 * 128 + bm / 2 * 4)) / 4; }

// One global -> LDS load of 16 bytes per lane: lane l's vector lands at lds_addr + 16*l.  Written as inline
// assembly so that the compiler does not tie later LDS reads to it with a full vmcnt wait (it cannot tell
// that the ring slot being filled is not the one being read); completion is awaited by wait_loads().
__device__ __forceinline__ void load_to_lds(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}

// Tile = (2 * NJ * 16) tokens x (WN * NI * 16) features, WN wavefronts along the features x 2 along the tokens:
//   256 x 256: WN = 4, NI = 4, NJ = 8 (8 wavefronts of 64 features x 128 tokens);
//   288 x 192: WN = 4, NI = 3, NJ = 9 (8 wavefronts of 48 x 144) -- 9216 tokens x 3072 features are exactly 512 such
//              tiles, two rounds of 256 compute units, where 432 square tiles are 1.69;
//   192 x 192: WN = 4, NI = 3, NJ = 6 (8 wavefronts of 48 x 96; 2 - 5 % faster than 4 wavefronts of 96 x 96).
template <int WN, int NI, int NJ, int LAYOUT>
__global__ void __launch_bounds__(128 * WN) qkv_gemm_direct_kernel(GemmArgs a) {
    constexpr int WAVES = 2 * WN;
    constexpr int TM = 2 * NJ * 16, TN = WN * NI * 16;      // tokens, features per tile
    constexpr int kXBytes = TM * BK * 2, kWBytes = TN * BK * 2;   // one operand tile of one K step
    constexpr int NMFMA = NI * NJ;
    // global->LDS instructions per lane and step: a load fills 8 tile rows; the last one of X may exist only for the
    // first wavefronts (288 rows = 36 loads over 8 wavefronts)
    constexpr int XLOADS = (TM / 8 + WAVES - 1) / WAVES, WLOADS = TN / 8 / WAVES;
    constexpr int XLOADS_ALL = TM / 8 / WAVES;              // loads every wavefront issues
    static_assert(WLOADS * WAVES * 8 == TN && NI >= 3 && NI <= NJ && TM % 8 == 0, "tile shape");
    static_assert(XLOADS <= (NI > 3 ? 2 : 1) * NJ && WLOADS <= (NI > 3 ? 2 : 1) * NJ, "not enough MFMAs in a half to issue the loads between");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    constexpr uint32_t kWRing = kXSlots * kXBytes;          // the W slots follow the X slots
    const TileCoord tc = tile_of_block(a);
    const uint16_t* __restrict__ W = a.w[tc.tensor];
    const uint32_t K = (uint32_t)a.D;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t wave_f = (wave % WN) * (NI * 16u), wave_t = (wave / WN) * (NJ * 16u);

    // load i of this wavefront fills LDS rows (WAVES*i + wave)*8 .. +8 of a tile: lane -> row lane>>3, stored column lane&7
    const unsigned char* xbase = reinterpret_cast<const unsigned char*>(a.x + ((size_t)a.row_begin + tc.m0) * K);
    const unsigned char* wbase = reinterpret_cast<const unsigned char*>(W + (size_t)tc.f0 * K);
    uint32_t xoff[XLOADS], woff[WLOADS];
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) {
        const uint32_t r = (WAVES * i + wave) * 8u + (lane >> 3);
        const uint32_t c = (lane & 7u) ^ swz(r);
        const uint32_t xr = min(r, (uint32_t)a.M - 1u - tc.m0);     // rows past the end re-read the last row; never stored
        xoff[i] = xr * K * 2u + c * 16u;
    }
#pragma unroll
    for (int i = 0; i < WLOADS; ++i) {
        const uint32_t r = (WAVES * i + wave) * 8u + (lane >> 3);
        const uint32_t c = (lane & 7u) ^ swz(r);
        const uint32_t wr = min(r, (uint32_t)a.D - 1u - tc.f0);
        woff[i] = wr * K * 2u + c * 16u;
    }
    const bool last_x_load = XLOADS == XLOADS_ALL || (WAVES * (XLOADS - 1) + wave) * 8u < (uint32_t)TM;   // per wavefront
    // load i of the X / W tile of K step kt into slot `slot` of its ring
    auto issue_x = [&](uint32_t kt, uint32_t slot, int i) {
        if (i < XLOADS_ALL || last_x_load)
            load_to_lds(xbase + (size_t)kt * (BK * 2) + xoff[i], lds0 + slot * kXBytes + (WAVES * i + wave) * 1024u);
    };
    auto issue_w = [&](uint32_t kt, uint32_t slot, int i) {
        load_to_lds(wbase + (size_t)kt * (BK * 2) + woff[i], lds0 + kWRing + slot * kWBytes + (WAVES * i + wave) * 1024u);
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
    const uint32_t w_frag = kWRing + (wave_f + frag_row) * 128u;
    // X fragment j / W fragment i of half kk of the step that sits in slot xs of the X ring / ws of the W ring
    auto read_x = [&](uint32_t xs, uint32_t kk, int j) {
        return *reinterpret_cast<const bf16x8*>(smem + xs * kXBytes + x_frag + (((4u * kk + frag_kg) ^ sw) << 4) + j * 2048);
    };
    auto read_w = [&](uint32_t ws, uint32_t kk, int i) {
        return *reinterpret_cast<const bf16x8*>(smem + ws * kWBytes + w_frag + (((4u * kk + frag_kg) ^ sw) << 4) + i * 2048);
    };

    f32x4 acc[NI][NJ];   // [feature tile][token tile]
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

    const uint32_t n_k = K / BK;   // >= 3 (the host sends shorter K to the fallback kernel)
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) issue_x(0, 0, i);
#pragma unroll
    for (int i = 0; i < WLOADS; ++i) issue_w(0, 0, i);
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) issue_x(1, 1, i);
#pragma unroll
    for (int i = 0; i < WLOADS; ++i) issue_w(1, 1, i);
    // step 0 has landed; X1, W1 may still be in flight (counted with the loads every wavefront issues: a wavefront
    // that issues one more waits for a little more than it has to)
    wait_loads<XLOADS_ALL + WLOADS>();
    __syncthreads();

    bf16x8 wf0[NI], wf1[NI], xf[NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i) wf0[i] = read_w(0, 0, i);
#pragma unroll
    for (int j = 0; j < NJ; ++j) xf[j] = read_x(0, 0, j);

    // One half: MFMA m multiplies W fragment i with X fragment j = m / NI.  After the first MFMA of token tile j < NI,
    // W fragment j of the next half is read into wf_n; after the last MFMA of token tile j its X fragment is read
    // again for the next half; after the second (and, where NI > 3, the third) MFMA of token tile j one load is
    // issued: X loads of step kt_l into X slot slot_l (LOAD_X) or W loads into W slot slot_l.
    // sched_barrier(0) after every group keeps the order.
    auto half = [&](const bf16x8 (&wf)[NI], bf16x8 (&wf_n)[NI], bool read_next, uint32_t xs_n, uint32_t ws_n, uint32_t kk_n,
                    auto load_x_c, auto n_loads_c, uint32_t kt_l, uint32_t slot_l) {
        constexpr int N_LOADS = decltype(n_loads_c)::value;
        constexpr bool LOAD_X = decltype(load_x_c)::value;
#pragma unroll
        for (int m = 0; m < NMFMA; ++m) {
            const int q = m % NI, j = m / NI;                 // q-th MFMA of token tile j
            const int i = (j & 1) ? NI - 1 - q : q;           // W fragments up, then down: one operand is kept at every turn
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (q == 0) {
                if (j < NI && read_next) wf_n[j] = read_w(ws_n, kk_n, j);
            } else if (q == NI - 1) {
                if (read_next) xf[j] = read_x(xs_n, kk_n, j);
            } else if (q <= 2) {
                const int l = (q - 1) * NJ + j;
                if (l < N_LOADS) {
                    if constexpr (LOAD_X) issue_x(kt_l, slot_l, l);
                    else issue_w(kt_l, slot_l, l);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // xs / ws: the ring slots of X / W of step kt.
    // LOAD_X: X of step kt+2 is issued during half 0 (into the X slot step kt-1 used);
    // LOAD_W: W of step kt+2 is issued during half 1 (into the W slot of step kt itself).
    auto k_step = [&](uint32_t kt, uint32_t xs, uint32_t ws, auto load_x, auto load_w, auto wait, auto next) {
        constexpr bool LOAD_X = decltype(load_x)::value, LOAD_W = decltype(load_w)::value, NEXT = decltype(next)::value;
        constexpr int WAIT = decltype(wait)::value;
        using xl = std::integral_constant<int, LOAD_X ? XLOADS : 0>;
        using wl = std::integral_constant<int, LOAD_W ? WLOADS : 0>;
        const uint32_t xs_next = xs == kXSlots - 1 ? 0u : xs + 1u, xs_prev = xs == 0 ? kXSlots - 1u : xs - 1u;
        half(wf0, wf1, true, xs, ws, 1, std::true_type{}, xl{}, kt + 2, xs_prev);
        if constexpr (NEXT) {
            wait_loads<WAIT>();
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
        half(wf1, wf0, NEXT, xs_next, ws ^ 1u, 0, std::false_type{}, wl{}, kt + 2, ws);
    };
    using yes = std::true_type;
    using no = std::false_type;
    const std::integral_constant<int, 0> w0;
    const std::integral_constant<int, XLOADS_ALL> w1;      // the X tile of the step after next may still be in flight
    uint32_t kt = 0, xs = 0, ws = 0;
    auto advance = [&]() {
        ++kt;
        xs = xs == kXSlots - 1 ? 0u : xs + 1u;
        ws ^= 1u;
    };
    // At the barrier of step kt the loads in flight, oldest first, are X(kt+1), W(kt+1), X(kt+2): the last may stay.
    while (kt + 2 < n_k) {
        k_step(kt, xs, ws, yes{}, yes{}, w1, yes{});
        advance();
    }
    k_step(kt, xs, ws, no{}, no{}, w0, yes{});     // step n_k-2: the last step must have landed completely
    advance();
    k_step(kt, xs, ws, no{}, no{}, w0, no{});      // step n_k-1
    __syncthreads();
    constexpr int kEpilogueBytes = NJ * 16 * EpilogueRows<NI * 2>::ROWB;   // per wavefront, see stage_tile16
    static_assert(WAVES * kEpilogueBytes <= ring_lds_bytes(TM, TN), "the epilogue reuses the ring's LDS");
    if constexpr (LAYOUT == OUT_FUSED) {
        if (a.gamma[tc.tensor]) {     // the same for the whole workgroup: its barrier is taken by all or by none
            // LDS of a normalising tile: a half tile of staging rows per wavefront, the partial sums of squares, the table
            constexpr int kHalfBytes = (NJ + 1) / 2 * 16 * EpilogueRows<NI * 2>::ROWB;
            static_assert(fused_table_floats(TM, TN) >= 0, "the staging rows and the partial sums fit the ring's LDS");
            float* xch = reinterpret_cast<float*>(smem + WAVES * kHalfBytes);
            if (a.tab_lds)
                norm_rope_store<NI, NJ, WN, true>(acc, smem + wave * kHalfBytes, xch, xch + WAVES * NJ * 16, a, a.gamma[tc.tensor],
                                                  a.y[tc.tensor], a.y2[tc.tensor], lane, wave, tc.m0, tc.m0 + wave_t, tc.f0 + wave_f);
            else
                norm_rope_store<NI, NJ, WN, false>(acc, smem + wave * kHalfBytes, xch, nullptr, a, a.gamma[tc.tensor], a.y[tc.tensor],
                                                   a.y2[tc.tensor], lane, wave, tc.m0, tc.m0 + wave_t, tc.f0 + wave_f);
            return;
        }
    }
    unsigned char* ep = smem + wave * kEpilogueBytes;
    if constexpr (LAYOUT == OUT_FUSED) {
        if (a.sel_prev && tc.tensor == 0) {     // V (the first tensor of the launch), flagged on its way out
            static_assert(WAVES * kEpilogueBytes + WAVES * NJ * 4 <= ring_lds_bytes(TM, TN), "room for the wavefronts' verdicts");
            uint32_t* verdicts = reinterpret_cast<uint32_t*>(smem + WAVES * kEpilogueBytes);      // [wavefront][tile of 16 tokens]
            vec16 prev_rows[NJ * 2];
            load_prev_rows<NJ * 16>(prev_rows, lane, (size_t)a.row_begin, tc.m0 + wave_t, tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D, a);
            stage_tile16<NI, NJ>(acc, ep, lane);
            store_rows_select<NJ * 16>(ep, lane, wave, a.y[0], a.y2[0], (size_t)a.row_begin, tc.m0 + wave_t, tc.f0 + wave_f, (uint32_t)a.M,
                                       (uint32_t)a.D, a, verdicts, prev_rows);
            __syncthreads();
            // one lane per 16-token tile of the workgroup's 2 NJ: the verdicts of the WN wavefronts that share its tokens
            const uint32_t sel = threadIdx.x;
            if (sel < 2u * NJ) {
                const uint32_t half = sel / NJ, j = sel - half * NJ;
                uint32_t any = 0;
#pragma unroll
                for (uint32_t wf = 0; wf < (uint32_t)WN; ++wf) any |= verdicts[(half * WN + wf) * NJ + j];
                const uint32_t tok = tc.m0 + sel * 16u;
                if (tok < (uint32_t)a.M)
                    a.sel_flag_bytes[(size_t)(((uint32_t)a.row_begin + tok) / 16u) * 16u + tc.f0 / (uint32_t)TN] = (uint8_t)any;
            }
            return;
        }
    }
    stage_tile16<NI, NJ>(acc, ep, lane);
    store_rows<NI * 2, NJ * 16, LAYOUT>(ep, lane, a.y[tc.tensor], LAYOUT == OUT_FUSED ? a.y2[tc.tensor] : nullptr, (size_t)a.row_begin,
                                        tc.m0 + wave_t, tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D, a);
}

// ---------------------------------------------------------------------------------------------
// General path, any K that is a multiple of 8: global -> registers -> LDS, vectors beyond K are zero.
// Four wavefronts (2 x 2) of 128 x 128 outputs.
// ---------------------------------------------------------------------------------------------
constexpr int kStagedThreads = 256;
constexpr int kVecPerOperand = BM * (BK / 8) / kStagedThreads;   // 16-byte vectors per lane per operand per stage: 8

template <int LAYOUT>
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
    store_tile<4, 4, LAYOUT>(acc, smem + wave * (128 * 256), lane, a.y[tc.tensor], nullptr, (size_t)a.row_begin, tc.m0 + wave_t,
                          tc.f0 + wave_f, (uint32_t)a.M, (uint32_t)a.D, a);
}


// A tile shape of the main kernel with its two epilogues and launch parameters.
struct TileKernel {
    int bm, bn, threads, lds;
    double penalty;               // measured per-flop cost against the 256 x 256 tile
    const void* entry[4];         // by OutLayout (OUT_FUSED only for the shapes of whole 256-feature tiles)
};
template <int WN, int NI, int NJ>
TileKernel tile_kernel(double penalty) {
    return {2 * NJ * 16, WN * NI * 16, 128 * WN, ring_lds_bytes(2 * NJ * 16, WN * NI * 16), penalty,
            {(const void*)qkv_gemm_direct_kernel<WN, NI, NJ, OUT_SEQ>, (const void*)qkv_gemm_direct_kernel<WN, NI, NJ, OUT_CHUNKS>,
             (const void*)qkv_gemm_direct_kernel<WN, NI, NJ, OUT_HEADS>, nullptr}};
}
// a shape for the fused call only (tiles 256 features wide: whole heads of 64, 128 or 256)
template <int WN, int NI, int NJ>
TileKernel fused_tile_kernel(double penalty) {
    return {2 * NJ * 16, WN * NI * 16, 128 * WN, ring_lds_bytes(2 * NJ * 16, WN * NI * 16), penalty,
            {nullptr, nullptr, nullptr, (const void*)qkv_gemm_direct_kernel<WN, NI, NJ, OUT_FUSED>}};
}

// The tile shapes of the main kernel, and which one a launch of M tokens x D features x n_tensors weights takes.
// 256 x 256 does the least operand traffic per flop; the others are taken when their tile count fills the compute
// units so much better that they win all the same.  Cost = rounds x tile area x a measured per-flop penalty, a round
// being one tile on every unit.  (Measured and left out: 224 x 256 equals 288 x 192 at 9216 tokens and nothing else
// gains from it; 160 x 192, 256 x 192 and 192 x 256 win a few percent at 2304 tokens only.)
// whole_heads: the shapes of the fused call, all 256 features wide (a head row must lie inside one tile); their
// penalties follow the same two ratios (operand bytes and fragment reads per flop) as the measured ones.
static const TileKernel* tile_shapes(bool whole_heads, int* count) {
    static const TileKernel shapes[] = {tile_kernel<4, 4, 8>(1.0), tile_kernel<4, 3, 9>(kPenalty288), tile_kernel<4, 3, 6>(kPenalty192)};
    static const TileKernel fused[] = {fused_tile_kernel<4, 4, 8>(1.0), fused_tile_kernel<4, 4, 7>(1.035), fused_tile_kernel<4, 4, 6>(1.08)};
    *count = 3;
    return whole_heads ? fused : shapes;
}

struct LaunchPlan {
    const TileKernel* pick;    // nullptr: the compute-unit count could not be read
    bool ring_kernel;          // false: the general kernel (K not a multiple of 64, or shorter than three steps)
    int32_t bm, bn, tiles_m, tiles_n_per_tensor, n_cu;
};

static LaunchPlan plan_launch(int32_t M, int32_t D, int32_t n_tensors, bool whole_heads) {
    static const int n_cu = [] {     // asked once (thread-safe initialisation); 0 = could not be read
        int dev = 0, val = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&val, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        return val;
    }();
    LaunchPlan p{};
    p.n_cu = n_cu;
    if (n_cu <= 0) return p;
    int n_shapes = 0;
    const TileKernel* shapes = tile_shapes(whole_heads, &n_shapes);
    p.pick = &shapes[0];
    static const int forced_tile = (int)tune_value("COCODIFF_GEMM_TILE", 0);     // tuning builds only
    double best = 0.0;
    for (int i = 0; i < n_shapes; ++i) {
        const TileKernel& t = shapes[i];
        const int64_t tiles = (int64_t)((M + t.bm - 1) / t.bm) * ((D + t.bn - 1) / t.bn) * n_tensors;
        const double cost = (double)((tiles + n_cu - 1) / n_cu) * t.bm * t.bn * t.penalty;
        if (forced_tile ? forced_tile == t.bm * 1000 + t.bn : (i == 0 || cost < best)) {
            p.pick = &t;
            best = cost;
        }
    }
    p.ring_kernel = D % BK == 0 && D >= 3 * BK;
    p.bm = p.ring_kernel ? p.pick->bm : BM;      // the general kernel has one tile shape
    p.bn = p.ring_kernel ? p.pick->bn : BM;
    p.tiles_m = (M + p.bm - 1) / p.bm;
    p.tiles_n_per_tensor = (D + p.bn - 1) / p.bn;
    return p;
}

}  // namespace cocodiff

using namespace cocodiff;

// layout OUT_SEQ: q, k, v are [N][D]; OUT_CHUNKS: they are exchange buffers, written in chunk order; OUT_HEADS: [H][N][d].
// OUT_FUSED: q, k, v are the exchange buffers and `fused` holds the head-parallel tensors, the gammas and the rotation.
struct FusedExtras {
    cocodiff_bf16* hs[3];              // q_hs, k_hs, v_hs
    const cocodiff_bf16* gamma[2];     // gamma_q, gamma_k
    float eps;
    RopeDev rope;
    // V flagged for the selection on its way out (cocodiff_qkv_proj_fused_select): previous-step V, threshold, flag records
    const cocodiff_bf16* sel_prev;
    uint8_t* sel_flag_bytes;
    float sel_tau;
};

static int proj_launch(const cocodiff_shape* shape, const cocodiff_bf16* x,
                       const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                       cocodiff_bf16* q, cocodiff_bf16* k, cocodiff_bf16* v, OutLayout layout, int slot_order, void* stream,
                       const FusedExtras* fused = nullptr) {
    const bool packed = layout == OUT_CHUNKS || layout == OUT_FUSED;
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (packed && slot_order != COCODIFF_SEND_MAJOR && slot_order != COCODIFF_RECV_MAJOR)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_pack: slot_order (%d) must be SEND_MAJOR or RECV_MAJOR", slot_order);
    if (!x) return fail(COCODIFF_ERR_NULL, "qkv_proj: x is NULL");
    if (fused) {
        const cocodiff_bf16* w3[3] = {wq, wk, wv};
        cocodiff_bf16* b3[3] = {q, k, v};
        for (int i = 0; i < 3; ++i) {
            const bool any_out = b3[i] || fused->hs[i];
            if ((w3[i] != nullptr) != any_out)
                return fail(COCODIFF_ERR_NULL, "qkv_proj_fused: a weight needs at least one of its two outputs, and outputs need their weight");
            if (i < 2 && w3[i] && !fused->gamma[i]) return fail(COCODIFF_ERR_NULL, "qkv_proj_fused: gamma missing for a given Q or K");
            if (!aligned16(fused->hs[i]) || (i < 2 && !aligned16(fused->gamma[i])))
                return fail(COCODIFF_ERR_ALIGN, "qkv_proj_fused: pointers must be 16-byte aligned");
        }
        if (!wq && !wk && !wv) return fail(COCODIFF_ERR_NULL, "qkv_proj_fused: no weight given");
    } else {
        if ((wq == nullptr) != (q == nullptr) || (wk == nullptr) != (k == nullptr) || (wv == nullptr) != (v == nullptr))
            return fail(COCODIFF_ERR_NULL, "qkv_proj: a weight and its output must be given together");
        if (!q && !k && !v) return fail(COCODIFF_ERR_NULL, "qkv_proj: no (weight, output) pair given");
    }
    if (!aligned16(x) || !aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(q) || !aligned16(k) || !aligned16(v))
        return fail(COCODIFF_ERR_ALIGN, "qkv_proj: pointers must be 16-byte aligned");

    GemmArgs a;
    a.Ns = (uint32_t)(shape->N / shape->P);
    a.P = (uint32_t)shape->P;
    a.row8 = (uint32_t)(shape->H / shape->P) * (uint32_t)(shape->d / 8);
    a.chunk8 = a.Ns * a.row8;
    a.recv_major = slot_order == COCODIFF_RECV_MAJOR;
    a.N_all = (uint32_t)shape->N;
    a.d8 = (uint32_t)(shape->d / 8);
    a.x = x;
    a.n_tensors = 0;
    const cocodiff_bf16* ws[3] = {wv, wq, wk};   // V first: its tiles are dealt out before Q's and K's
    cocodiff_bf16* ys[3] = {v, q, k};
    cocodiff_bf16* y2s[3] = {fused ? fused->hs[2] : nullptr, fused ? fused->hs[0] : nullptr, fused ? fused->hs[1] : nullptr};
    const cocodiff_bf16* gs[3] = {nullptr, fused ? fused->gamma[0] : nullptr, fused ? fused->gamma[1] : nullptr};
    for (int i = 0; i < 3; ++i) {
        a.w[i] = nullptr;
        a.y[i] = nullptr;
        a.y2[i] = nullptr;
        a.gamma[i] = nullptr;
    }
    for (int i = 0; i < 3; ++i)
        if (ws[i]) {
            a.w[a.n_tensors] = ws[i];
            a.y[a.n_tensors] = ys[i];
            a.y2[a.n_tensors] = y2s[i];
            a.gamma[a.n_tensors] = gs[i];
            ++a.n_tensors;
        }
    a.d = (uint32_t)shape->d;
    a.inv_d = 1.0f / (float)shape->d;
    a.eps = fused ? fused->eps : 0.f;
    a.rope = fused ? fused->rope : RopeDev{};
    a.tab_lds = 0;
    a.sel_prev = fused ? fused->sel_prev : nullptr;
    a.sel_flag_bytes = fused ? fused->sel_flag_bytes : nullptr;
    a.sel_th = make_thresholds(fused ? fused->sel_tau : 0.f);
    a.sel_tiles = (uint32_t)shape->N / 16u;
    const int32_t Ns = shape->N / shape->P;
    a.row_begin = shape->rank_begin * Ns;
    a.M = shape->rank_count * Ns;
    a.D = shape->D;
    if ((int64_t)288 * a.D * 2 >= ((int64_t)1 << 32)) return fail(COCODIFF_ERR_SHAPE, "qkv_proj: D (%d) too large", a.D);
    const LaunchPlan plan = plan_launch(a.M, a.D, a.n_tensors, layout == OUT_FUSED);
    if (!plan.pick) return fail(COCODIFF_ERR_HIP, "qkv_proj: cannot read the compute-unit count");
    if (layout == OUT_FUSED && !plan.ring_kernel)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_fused: D (%d) must be a multiple of 64 and at least 192", a.D);
    const TileKernel* pick = plan.pick;
    const bool ring_kernel = plan.ring_kernel;
    a.bm = plan.bm;
    a.bn = plan.bn;
    a.tiles_m = plan.tiles_m;
    a.tiles_n_per_tensor = plan.tiles_n_per_tensor;
    const uint32_t n_tiles = (uint32_t)a.tiles_m * a.tiles_n_per_tensor * a.n_tensors;
    for (int ax = 0; ax < 3; ++ax)
        a.row_base[ax] = a.row_stride[ax] = a.row_span[ax] = a.row_end[ax] = a.row_step16[ax] = a.tab_cum[ax] = a.tab_magic[ax] = 0;
    if (layout == OUT_FUSED && (a.gamma[0] || a.gamma[1] || a.gamma[2])) {      // (V alone comes without a rotation)
        // the rotation table goes through LDS when it fits beside the tile's staging rows, padded by two floats a row
        // (a row of one pair would need a divisor of 2^32: such tables stay in global memory)
        uint32_t pairs_total = 0, floats = 0;
        bool can = true;
        for (int ax = 0; ax < 3; ++ax) {
            const uint32_t pr = (uint32_t)a.rope.pairs[ax], rows = (uint32_t)a.rope.grid[ax];     // absent axes: 0 pairs, 1 row
            can = can && (pr >= 2 || ax >= a.rope.n_axes);
            a.tab_cum[ax] = pairs_total;
            a.tab_magic[ax] = pr >= 2 ? (uint32_t)((((uint64_t)1 << 32) + pr - 1) / pr) : 0u;
            a.row_base[ax] = floats;
            a.row_stride[ax] = ax < a.rope.n_axes ? 2u * pr + 2u : 0u;
            pairs_total += rows * pr;
            if (floats <= (uint32_t)fused_table_floats(256, 256)) floats += rows * a.row_stride[ax];     // (no overflow: rows, pr < 2^31 / 2)
            can = can && floats <= (uint32_t)fused_table_floats(256, 256);
        }
        const int room = pick->bm == 256 ? fused_table_floats(256, 256) : pick->bm == 224 ? fused_table_floats(224, 256) : fused_table_floats(192, 256);
        a.tab_lds = can && (int)floats <= room;
        if (!a.tab_lds)
            for (int ax = 0; ax < 3; ++ax) {
                a.row_base[ax] = (uint32_t)a.rope.offset[ax];
                a.row_stride[ax] = 2u * (uint32_t)a.rope.pairs[ax];
            }
        uint32_t rest = 16;     // 16 tokens in the grid's mixed radix, last axis fastest
        for (int ax = 2; ax >= 0; --ax) {
            const uint32_t rows = (uint32_t)a.rope.grid[ax];
            a.row_span[ax] = rows * a.row_stride[ax];
            a.row_end[ax] = ax < a.rope.n_axes ? a.row_base[ax] + a.row_span[ax] : UINT32_MAX;     // an absent axis never carries
            a.row_step16[ax] = (ax > 0 ? rest % rows : rest) * a.row_stride[ax];
            rest /= rows;
        }
    }

    // dynamic LDS above 64 KB needs the attribute, once per process (thread-safe initialisation)
    static const hipError_t attr_rc = [] {
        hipError_t e = hipSuccess;
        for (bool whole_heads : {false, true}) {
            int n_shapes = 0;
            const TileKernel* shapes = tile_shapes(whole_heads, &n_shapes);
            for (int i = 0; i < n_shapes; ++i)
                for (const void* k : shapes[i].entry)
                    if (k && e == hipSuccess) e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, shapes[i].lds);
        }
        for (const void* k : {(const void*)qkv_gemm_staged_kernel<OUT_SEQ>, (const void*)qkv_gemm_staged_kernel<OUT_CHUNKS>,
                              (const void*)qkv_gemm_staged_kernel<OUT_HEADS>})
            if (e == hipSuccess) e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        return e;
    }();
    if (attr_rc != hipSuccess) return fail(COCODIFF_ERR_HIP, "qkv_proj: cannot reserve LDS: %s", hipGetErrorString(attr_rc));
    hipStream_t st = as_stream(stream);
    void* kernel_args[] = {&a};
    hipError_t le;
    static const void* const staged[4] = {(const void*)qkv_gemm_staged_kernel<OUT_SEQ>, (const void*)qkv_gemm_staged_kernel<OUT_CHUNKS>,
                                          (const void*)qkv_gemm_staged_kernel<OUT_HEADS>, nullptr};
    if (ring_kernel)
        le = hipLaunchKernel(pick->entry[layout], dim3(n_tiles), dim3(pick->threads), kernel_args, pick->lds, st);
    else
        le = hipLaunchKernel(staged[layout], dim3(n_tiles), dim3(kStagedThreads), kernel_args, kLdsBytes, st);
    if (le != hipSuccess) return fail(COCODIFF_ERR_HIP, "qkv_proj: launch failed: %s", hipGetErrorString(le));
    return check_launch("qkv_gemm_kernel");
}

extern "C" int cocodiff_qkv_proj(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                 const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                 cocodiff_bf16* q, cocodiff_bf16* k, cocodiff_bf16* v, void* stream) {
    return proj_launch(shape, x, wq, wk, wv, q, k, v, OUT_SEQ, COCODIFF_SEND_MAJOR, stream);
}

extern "C" int cocodiff_qkv_proj_pack(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                      const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                      cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order, void* stream) {
    return proj_launch(shape, x, wq, wk, wv, qbuf, kbuf, vbuf, OUT_CHUNKS, slot_order, stream);
}

extern "C" int cocodiff_qkv_proj_hs(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                    const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                    cocodiff_bf16* q_hs, cocodiff_bf16* k_hs, cocodiff_bf16* v_hs, void* stream) {
    return proj_launch(shape, x, wq, wk, wv, q_hs, k_hs, v_hs, OUT_HEADS, COCODIFF_SEND_MAJOR, stream);
}

extern "C" int cocodiff_qkv_proj_fused(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                       const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                       const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps, const cocodiff_rope* rope,
                                       cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order,
                                       cocodiff_bf16* q_hs, cocodiff_bf16* k_hs, cocodiff_bf16* v_hs, void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (shape->d != 64 && shape->d != 128 && shape->d != 256)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_fused: d (%d) must be 64, 128 or 256 (a head row must fill whole wavefront tiles of 64 features)", shape->d);
    FusedExtras f{};
    f.hs[0] = q_hs;
    f.hs[1] = k_hs;
    f.hs[2] = v_hs;
    f.gamma[0] = gamma_q;
    f.gamma[1] = gamma_k;
    f.eps = eps;
    if (wq || wk) {
        rc = fill_rope(shape, rope, "qkv_proj_fused", &f.rope);
        if (rc != COCODIFF_OK) return rc;
    }
    return proj_launch(shape, x, wq, wk, wv, qbuf, kbuf, vbuf, OUT_FUSED, slot_order, stream, &f);
}

// Flag records of the projection that flags V: 16 bytes per 16-token tile, one byte per 256-feature tile of V.
static bool flags_in_projection(const cocodiff_shape* shape, int32_t tile_tokens) {
    return tile_tokens == 16 && (shape->D + 255) / 256 <= 16;
}

extern "C" size_t cocodiff_qkv_proj_fused_select_workspace_bytes(const cocodiff_shape* shape, int32_t tile_tokens) {
    if (check_shape(shape) != COCODIFF_OK || tile_tokens <= 0 || shape->N % tile_tokens) return 0;
    if (flags_in_projection(shape, tile_tokens)) return (size_t)(shape->N / 16) * 16;
    return cocodiff_vmajor_select_workspace_bytes(shape->H, shape->N, shape->d, tile_tokens);
}

extern "C" int cocodiff_qkv_proj_fused_select(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                              const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                              const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                              const cocodiff_rope* rope,
                                              cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order,
                                              cocodiff_bf16* q_hs, cocodiff_bf16* k_hs, cocodiff_bf16* v_hs,
                                              const cocodiff_bf16* v_prev, int32_t tile_tokens, float tau,
                                              int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                              cocodiff_bf16* compact, int32_t cap_tiles,
                                              void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (shape->rank_begin != 0 || shape->rank_count != shape->P)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_fused_select: a tile's flag needs every head, so the rank range must be all P ranks");
    if (!wv || !vbuf || !v_hs)
        return fail(COCODIFF_ERR_NULL, "qkv_proj_fused_select: wv, vbuf and v_hs are required (the selection reads V in the head-parallel layout)");
    if (!v_prev || !active_idx || !n_active || !workspace)
        return fail(COCODIFF_ERR_NULL, "qkv_proj_fused_select: v_prev, active_idx, n_active and workspace are required");
    if (!aligned16(v_prev) || !aligned16(workspace) || !aligned16(compact))
        return fail(COCODIFF_ERR_ALIGN, "qkv_proj_fused_select: tensors and workspace must be 16-byte aligned");
    if (tile_tokens <= 0 || shape->N % tile_tokens)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_fused_select: N (%d) must be a multiple of tile_tokens (%d)", shape->N, tile_tokens);
    if (compact && cap_tiles < 1) return fail(COCODIFF_ERR_CAPACITY, "qkv_proj_fused_select: cap_tiles (%d) must be >= 1", cap_tiles);
    const size_t need = cocodiff_qkv_proj_fused_select_workspace_bytes(shape, tile_tokens);
    if (workspace_bytes < need)
        return fail(COCODIFF_ERR_CAPACITY, "qkv_proj_fused_select: workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    if (!flags_in_projection(shape, tile_tokens)) {
        // other tile heights, or more than 16 feature tiles: the two calls this one stands for
        rc = cocodiff_qkv_proj_fused(shape, x, wq, wk, wv, gamma_q, gamma_k, eps, rope, qbuf, kbuf, vbuf, slot_order, q_hs, k_hs, v_hs, stream);
        if (rc != COCODIFF_OK) return rc;
        return cocodiff_vmajor_select(shape->H, shape->N, shape->d, tile_tokens, v_hs, v_prev, tau, flags, active_idx, n_active, compact,
                                      cap_tiles, workspace, workspace_bytes, stream);
    }
    if (shape->d != 64 && shape->d != 128 && shape->d != 256)
        return fail(COCODIFF_ERR_SHAPE, "qkv_proj_fused: d (%d) must be 64, 128 or 256 (a head row must fill whole wavefront tiles of 64 features)", shape->d);
    FusedExtras f{};
    f.hs[0] = q_hs;
    f.hs[1] = k_hs;
    f.hs[2] = v_hs;
    f.gamma[0] = gamma_q;
    f.gamma[1] = gamma_k;
    f.eps = eps;
    f.sel_prev = v_prev;
    f.sel_flag_bytes = static_cast<uint8_t*>(workspace);
    f.sel_tau = tau;
    if (wq || wk) {
        rc = fill_rope(shape, rope, "qkv_proj_fused_select", &f.rope);
        if (rc != COCODIFF_OK) return rc;
    }
    rc = proj_launch(shape, x, wq, wk, wv, qbuf, kbuf, vbuf, OUT_FUSED, slot_order, stream, &f);
    if (rc != COCODIFF_OK) return rc;
    TileFlags tf;
    tf.words_ptr = static_cast<const uint32_t*>(workspace);
    tf.words = 4;
    const uint32_t parts = (uint32_t)(shape->D + 255) / 256u;        // bytes of a record that the projection wrote
    for (uint32_t w = 0; w < 4; ++w) {
        const uint32_t n = parts > 4 * w ? (parts - 4 * w < 4 ? parts - 4 * w : 4u) : 0u;
        tf.mask[w] = n >= 4 ? 0xffffffffu : (1u << (8 * n)) - 1u;
    }
    return select_finish_launch(shape->H, shape->N, shape->d, tile_tokens, v_hs, tf, flags, active_idx, n_active, compact, cap_tiles, stream);
}

extern "C" int cocodiff_qkv_proj_plan(const cocodiff_shape* shape, int32_t n_tensors, int32_t whole_heads, int32_t* tile_tokens,
                                      int32_t* tile_features, int32_t* n_tiles, int32_t* n_compute_units) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (n_tensors < 1 || n_tensors > 3) return fail(COCODIFF_ERR_SHAPE, "qkv_proj_plan: n_tensors (%d) must be 1, 2 or 3", n_tensors);
    const LaunchPlan p = plan_launch(shape->rank_count * (shape->N / shape->P), shape->D, n_tensors, whole_heads != 0);
    if (!p.pick) return fail(COCODIFF_ERR_HIP, "qkv_proj_plan: cannot read the compute-unit count");
    if (tile_tokens) *tile_tokens = p.bm;
    if (tile_features) *tile_features = p.bn;
    if (n_tiles) *n_tiles = p.tiles_m * p.tiles_n_per_tensor * n_tensors;
    if (n_compute_units) *n_compute_units = p.n_cu;
    return COCODIFF_OK;
}
