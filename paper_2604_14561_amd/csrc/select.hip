// V-Major active-tile selection (paper Section III-D), threshold-per-tile form:
//   flag[t] = any element of tile t with NOT(|v_cur - v_prev| <= tau)   (decided on the difference in double)
//   idx     = ascending list of flagged tiles, n_active = its length
//   compact = v_cur of the flagged tiles gathered densely in list order.
//
// Two launches on the caller's stream:
//   1. flag pass -- up to four workgroups of 256 lanes per tile, each streaming a contiguous share of the tile's
//                   S segments of v_cur and v_prev once and writing its verdict into its own byte of the tile's
//                   4-byte flag word (small workgroups: many fit a compute unit, so loads of one overlap the
//                   stores and the tail of another, and a launch of a few hundred tiles still spreads evenly);
//   2. gather    -- one workgroup per tile: a flagged tile's workgroup counts the flagged words before it (its
//                   slot in the list), writes its id there and copies its v_cur segments into `compact`;
//                   unflagged tiles leave at once; the last tile's workgroup also writes n_active.
// HBM traffic: 2 tensors read once + the active fraction read once more and written once (the flag words,
// 4 bytes per tile, are re-read by the flagged workgroups out of L2).
// The flag pass can take the current values from the exchange buffer of the first all-to-all instead and write
// the head-parallel tensor on the way (the receiver's unpack and the selection in one pass).
// The same file holds the gather / scatter of listed tiles (sender-side extraction, receiver-side overwrite).
#include <mutex>

#include "internal.h"

namespace cocodiff {

// Library-owned flag words for cocodiff_vmajor_select_static: one word per tile, up to kStaticMaxTiles tiles
// (256 KiB per GPU, held until the process ends).  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and host calls use the per-device address static_scratch() returns.
constexpr uint32_t kStaticMaxTiles = 1u << 16;
static __device__ __align__(256) uint32_t scratch[kStaticMaxTiles];

constexpr int kSelThreads = 256;
constexpr int kSelUnroll = 6;     // 16-byte vectors a lane of the gather / move kernels keeps in flight; a flag-pass share is up to 6 x 256
// vectors per tensor and lane in one round of the flag pass: plain, and with the unpack inside (measured on tensors of
// 57, 127 and 613 MB against rounds of 1, 2 and 6)
#ifndef COCODIFF_FLAG_UNROLL
#define COCODIFF_FLAG_UNROLL 3
#endif
#ifndef COCODIFF_FLAG_UNROLL_PLAIN
#define COCODIFF_FLAG_UNROLL_PLAIN 3
#endif
constexpr int kFlagUnroll = COCODIFF_FLAG_UNROLL, kFlagUnrollPlain = COCODIFF_FLAG_UNROLL_PLAIN;

struct SelectShape {
    uint32_t S, NT, seg8;   // seg8: 16-byte vectors per (tile, slab) segment
    uint64_t slab8;         // vectors per slab = N*W/8
};

// Where the current tensor comes from when the flag pass also does the receiver-side unpack of the first
// all-to-all: the exchange buffer, chunk (sender r -> receiver p) = [Ns tokens][Hp heads][d].
struct UnpackSource {
    const vec16* buf;
    vec16* hs_out;               // the head-parallel tensor being produced ([H][N][d])
    uint32_t Ns, P, Hp, d8, T;   // tokens per rank, ranks, heads per rank, vectors per head row, tokens per tile
    uint32_t row8, chunk8;
    int recv_major;
};

// Division of an index by a launch constant: multiply-high by ceil(2^32 / d), exact while n * d < 2^32 (the host
// checks the largest n of every use and falls back to the hardware-free plain division otherwise); d = 1 has no magic.
struct Divisor {
    uint32_t d, magic;
};
template <bool MAGIC>
__device__ __forceinline__ uint32_t div_by(uint32_t n, const Divisor& f) {
    if (!MAGIC) return n / f.d;
    return f.d == 1u ? n : __umulhi(n, f.magic);
}

// Workgroup (t, part): verdict over vectors [part * share, (part + 1) * share) of tile t's index space
// g = s * seg8 + v (S segments of seg8 vectors), written to byte `part` of the tile's flag word.
// FROM_BUF: the current values are read from the exchange buffer (and written to their place in the
// head-parallel tensor on the way) instead of from `cur`.
struct FlagPass {
    const vec16* cur;
    const vec16* prev;
    uint8_t* flag_bytes;
    SelectShape sh;
    uint32_t share;
    Thresholds th;
    UnpackSource u;
    Divisor seg8, d8, Ns, Hp;
};

// The share goes in rounds of U vectors per lane.  In a round the streaming part does one compare per element; the
// workgroup then agrees (one barrier) whether the round holds a suspect.  Without one -- the common case -- its part
// of the head-parallel tensor is streamed out non-temporally (nobody reads it again soon, nothing stays dirty in L2);
// with one (a changed tile, as a rule) it is stored cached -- the gather pass reads those vectors again -- and the
// lanes settle their verdict from the registers.
// FAST: multiply-high divisions and 32-bit byte offsets from the tensors' base addresses (one address register per
// vector instead of three 64-bit pointers); the host takes it when every tensor is below 4 GiB and the divisions are
// exact, else the plain form.
template <bool FAST> struct OffsetType { typedef uint64_t type; };
template <> struct OffsetType<true> { typedef uint32_t type; };

template <bool NT_PREV, bool FROM_BUF, int U, bool FAST>
__global__ void __launch_bounds__(kSelThreads) select_flag_kernel(FlagPass a) {
    typedef typename OffsetType<FAST>::type off_t;     // byte offsets
    const uint32_t t = blockIdx.x, part = blockIdx.y;
    const uint32_t total = a.sh.S * a.sh.seg8;
    const uint32_t begin = part * a.share, end = min(total, begin + a.share);
    const char* cur_b = reinterpret_cast<const char*>(a.cur);
    const char* prev_b = reinterpret_cast<const char*>(a.prev);
    const char* buf_b = reinterpret_cast<const char*>(a.u.buf);
    char* hs_b = reinterpret_cast<char*>(a.u.hs_out);
    const off_t tile_at = (off_t)t * a.sh.seg8;
    bool changed = false, ever_suspect = false;
    // the round count is the same for every lane (the barrier inside a round needs the whole workgroup)
    for (uint32_t base = begin; base < end; base += U * kSelThreads) {
        vec16 c[U], p[U];
        off_t at[U];
        // a vector beyond the share's end reads the share's last vector again (same verdict) and is not stored
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const uint32_t g = min(base + threadIdx.x + k * kSelThreads, end - 1u);
            const uint32_t s = div_by<FAST>(g, a.seg8), v = g - s * a.sh.seg8;
            at[k] = ((off_t)s * (off_t)a.sh.slab8 + tile_at + v) * 16u;
            if (FROM_BUF) {
                // s is the head, v = (token in tile) * d8 + i8
                const uint32_t tl = div_by<FAST>(v, a.d8), i8 = v - tl * a.u.d8;
                const uint32_t n = t * a.u.T + tl, r = div_by<FAST>(n, a.Ns), m = n - r * a.u.Ns;
                const uint32_t pr = div_by<FAST>(s, a.Hp), hl = s - pr * a.u.Hp;
                const uint32_t slot = a.u.recv_major ? pr * a.u.P + r : r * a.u.P + pr;
                const off_t from = ((off_t)slot * a.u.chunk8 + (off_t)m * a.u.row8 + hl * a.u.d8 + i8) * 16u;
                c[k] = ld_nt(reinterpret_cast<const vec16*>(buf_b + from));
            } else {
                c[k] = *reinterpret_cast<const vec16*>(cur_b + at[k]);
            }
            p[k] = ld_vec<NT_PREV>(reinterpret_cast<const vec16*>(prev_b + at[k]));
        }
        bool suspect = false;
#pragma unroll
        for (int k = 0; k < U; ++k) suspect |= vec_suspect(c[k], p[k], a.th.tau_s);
        // the store policy needs the workgroup's verdict; without stores every lane settles its own suspects
        const bool any_suspect = FROM_BUF ? __syncthreads_or(suspect ? 1 : 0) != 0 : suspect;
        if (FROM_BUF) {
            if (any_suspect) {
#pragma unroll
                for (int k = 0; k < U; ++k)
                    if (base + threadIdx.x + k * kSelThreads < end) *reinterpret_cast<vec16*>(hs_b + at[k]) = c[k];
            } else {
#pragma unroll
                for (int k = 0; k < U; ++k)
                    if (base + threadIdx.x + k * kSelThreads < end) st_nt(reinterpret_cast<vec16*>(hs_b + at[k]), c[k]);
            }
        }
        if (any_suspect) {
            ever_suspect = true;
            bool tie = false, ch = false;
            // (the empty asm hides the values' origin, or the compiler keeps all 8 * U differences of the streaming
            // part alive across the barrier to reuse them here: three times the registers)
#pragma unroll
            for (int k = 0; k < U; ++k) {
                asm volatile("" : "+v"(c[k]), "+v"(p[k]));
                ch |= vec_changed(c[k], p[k], a.th.tau, a.th.tau_tie, tie);
            }
            if (tie && !ch) {
#pragma unroll
                for (int k = 0; k < U; ++k) ch |= vec_changed_double(c[k], p[k], a.th.tau);
            }
            changed |= ch;
        }
    }
    // with FROM_BUF ever_suspect is the same in every lane: the workgroup takes the barrier together, or not at all
    const int any = (!FROM_BUF || ever_suspect) ? (__syncthreads_or(changed ? 1 : 0) ? 1 : 0) : 0;
    if (threadIdx.x == 0) a.flag_bytes[4u * t + part] = (uint8_t)any;
}

// Sum over the workgroup of one count per lane; every lane gets the total.
template <int THREADS>
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t* wave_tot) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t tot = 0;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) tot += wave_tot[w];
    return tot;
}

// Is tile t active by its flag record (WORDS words, the bytes in f.mask written by the pass before)?
template <int WORDS>
__device__ __forceinline__ bool tile_active(const TileFlags& f, uint32_t t) {
    if (WORDS == 1) return (f.words_ptr[t] & f.mask[0]) != 0;
    const uint4 w = reinterpret_cast<const uint4*>(f.words_ptr)[t];
    return ((w.x & f.mask[0]) | (w.y & f.mask[1]) | (w.z & f.mask[2]) | (w.w & f.mask[3])) != 0;
}

// Workgroup t: if tile t is flagged, its list slot is the number of flagged tiles before it.
template <int THREADS, int WORDS>
__global__ void __launch_bounds__(THREADS) select_gather_kernel(const vec16* __restrict__ cur, TileFlags tf,
                                                                    int32_t* __restrict__ user_flags,
                                                                    int32_t* __restrict__ idx, int32_t* __restrict__ n_active,
                                                                    vec16* __restrict__ compact, SelectShape sh, uint32_t cap_tiles) {
    __shared__ uint32_t wave_tot[THREADS / 64];
    const uint32_t t = blockIdx.x;
    const bool mine = tile_active<WORDS>(tf, t);
    const bool last = t + 1 == sh.NT;
    const bool lead = blockIdx.y == 0;        // with several workgroups per tile (gridDim.y), the first one also writes the lists
    if (user_flags && lead && threadIdx.x == 0) user_flags[t] = mine ? 1 : 0;
    if (!mine && !(last && lead)) return;
    uint32_t before = 0;
    for (uint32_t u = threadIdx.x; u < t; u += THREADS) before += tile_active<WORDS>(tf, u) ? 1u : 0u;
    const uint32_t slot = block_sum<THREADS>(before, wave_tot);
    if (lead && threadIdx.x == 0) {
        if (mine) idx[slot] = (int32_t)t;
        if (last) *n_active = (int32_t)(slot + (mine ? 1u : 0u));
    }
    if (!mine || !compact || slot >= cap_tiles) return;
    const uint32_t total = sh.S * sh.seg8;
    for (uint32_t g0 = blockIdx.y * (kSelUnroll * THREADS) + threadIdx.x; g0 < total; g0 += gridDim.y * (kSelUnroll * THREADS)) {
        vec16 c[kSelUnroll];
        uint64_t dst[kSelUnroll];
#pragma unroll
        for (int k = 0; k < kSelUnroll; ++k) {
            const uint32_t g = g0 + k * THREADS;
            if (g < total) {
                const uint32_t s = g / sh.seg8, v = g - s * sh.seg8;
                c[k] = cur[(uint64_t)s * sh.slab8 + (uint64_t)t * sh.seg8 + v];
                dst[k] = ((uint64_t)s * cap_tiles + slot) * sh.seg8 + v;
            }
        }
#pragma unroll
        for (int k = 0; k < kSelUnroll; ++k)
            if (g0 + k * THREADS < total) st_nt(compact + dst[k], c[k]);
    }
}

// Workgroup j moves tile idx[j] (j < n_active, j < cap_tiles) between x [S][N][W] and compact [S][cap*T][W]:
// GATHER compact <- x (sender-side extraction of the active tiles), else x <- compact (receiver-side overwrite
// of the cached tensor).  A list entry outside [0, NT) is skipped, so a corrupt list cannot fault.
template <bool GATHER>
__global__ void __launch_bounds__(kSelThreads) tile_move_kernel(vec16* __restrict__ x, vec16* __restrict__ compact,
                                                                const int32_t* __restrict__ idx, const int32_t* __restrict__ n_active,
                                                                SelectShape sh, uint32_t cap_tiles) {
    const uint32_t j = blockIdx.x;
    const int32_t n = *n_active;
    if (n <= 0 || j >= (uint32_t)n) return;
    const uint32_t t = (uint32_t)idx[j];
    if (t >= sh.NT) return;
    const uint32_t total = sh.S * sh.seg8;
    // blockIdx.y strides over the tile's vectors in pieces of kSelUnroll * kSelThreads, so that a short list
    // still spreads over the whole chip
    for (uint32_t g0 = blockIdx.y * (kSelUnroll * kSelThreads) + threadIdx.x; g0 < total; g0 += gridDim.y * (kSelUnroll * kSelThreads)) {
        vec16 c[kSelUnroll];
        uint64_t dst[kSelUnroll];
#pragma unroll
        for (int k = 0; k < kSelUnroll; ++k) {
            const uint32_t g = g0 + k * kSelThreads;
            if (g < total) {
                const uint32_t s = g / sh.seg8, v = g - s * sh.seg8;
                const uint64_t x_at = (uint64_t)s * sh.slab8 + (uint64_t)t * sh.seg8 + v;
                const uint64_t c_at = ((uint64_t)s * cap_tiles + j) * sh.seg8 + v;
                c[k] = GATHER ? x[x_at] : compact[c_at];
                dst[k] = GATHER ? c_at : x_at;
            }
        }
#pragma unroll
        for (int k = 0; k < kSelUnroll; ++k)
            if (g0 + k * kSelThreads < total) st_nt((GATHER ? compact : x) + dst[k], c[k]);
    }
}

static int select_shape(int32_t S, int32_t N, int32_t W, int32_t T, SelectShape* out) {
    if (S <= 0 || N <= 0 || W <= 0 || T <= 0) return fail(COCODIFF_ERR_SHAPE, "select: S, N, W, tile_tokens must be positive");
    if (W % 8) return fail(COCODIFF_ERR_SHAPE, "select: W (%d) must be a multiple of 8", W);
    if (N % T) return fail(COCODIFF_ERR_SHAPE, "select: N (%d) must be a multiple of tile_tokens (%d)", N, T);
    const int64_t seg8 = (int64_t)T * W / 8;
    if (seg8 * S >= ((int64_t)1 << 31)) return fail(COCODIFF_ERR_SHAPE, "select: a tile of %lld vectors is too large", (long long)(seg8 * S));
    out->S = (uint32_t)S;
    out->NT = (uint32_t)(N / T);
    out->seg8 = (uint32_t)seg8;
    out->slab8 = (uint64_t)N * W / 8;
    return COCODIFF_OK;
}

template <int WORDS>
static void gather_launch(const SelectShape& sh, hipStream_t st, const cocodiff_bf16* v_cur, const TileFlags& tf, int32_t* flags,
                          int32_t* active_idx, int32_t* n_active, cocodiff_bf16* compact, uint32_t cap) {
    // one workgroup per tile, a tile in as few passes as possible (kSelUnroll vectors per lane and pass) -- or, when
    // there are too few tiles for the flagged ones to occupy the chip, several 256-lane workgroups per tile, each of
    // which counts the tile's slot for itself
    const uint32_t per_tile = sh.S * sh.seg8;
    constexpr uint32_t kSplitBelowTiles = 2048;     // measured: 27.4 -> 26.2 us at 576 tiles, 49.0 -> 48.4 at 1296, nothing at 6240
    if (sh.NT <= kSplitBelowTiles && per_tile > 256 * kSelUnroll) {
        const uint32_t parts = (uint32_t)((per_tile + 256 * kSelUnroll - 1) / (256 * kSelUnroll));
        hipLaunchKernelGGL((select_gather_kernel<256, WORDS>), dim3(sh.NT, parts < 8 ? parts : 8), dim3(256), 0, st, (const vec16*)v_cur,
                           tf, flags, active_idx, n_active, (vec16*)compact, sh, cap);
        return;
    }
    const int threads = per_tile > 512 * kSelUnroll ? 1024 : per_tile > 256 * kSelUnroll ? 512 : 256;
    if (threads == 1024)
        hipLaunchKernelGGL((select_gather_kernel<1024, WORDS>), dim3(sh.NT), dim3(1024), 0, st, (const vec16*)v_cur, tf, flags,
                           active_idx, n_active, (vec16*)compact, sh, cap);
    else if (threads == 512)
        hipLaunchKernelGGL((select_gather_kernel<512, WORDS>), dim3(sh.NT), dim3(512), 0, st, (const vec16*)v_cur, tf, flags,
                           active_idx, n_active, (vec16*)compact, sh, cap);
    else
        hipLaunchKernelGGL((select_gather_kernel<256, WORDS>), dim3(sh.NT), dim3(256), 0, st, (const vec16*)v_cur, tf, flags,
                           active_idx, n_active, (vec16*)compact, sh, cap);
}

int select_finish_launch(int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const cocodiff_bf16* v_cur, TileFlags tf,
                         int32_t* flags, int32_t* active_idx, int32_t* n_active, cocodiff_bf16* compact, int32_t cap_tiles,
                         void* stream) {
    SelectShape sh;
    int rc = select_shape(S, N, W, tile_tokens, &sh);
    if (rc != COCODIFF_OK) return rc;
    const uint32_t cap = compact ? (uint32_t)cap_tiles : 0u;
    if (tf.words == 1)
        gather_launch<1>(sh, as_stream(stream), v_cur, tf, flags, active_idx, n_active, compact, cap);
    else
        gather_launch<4>(sh, as_stream(stream), v_cur, tf, flags, active_idx, n_active, compact, cap);
    return check_launch("select_gather_kernel");
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" size_t cocodiff_vmajor_select_workspace_bytes(int32_t S, int32_t N, int32_t W, int32_t tile_tokens) {
    SelectShape sh;
    if (select_shape(S, N, W, tile_tokens, &sh) != COCODIFF_OK) return 0;
    return (size_t)sh.NT * sizeof(int32_t);   // one flag per tile
}

// from_buf == nullptr: v_cur is read.  Otherwise v_cur is WRITTEN (the unpacked tensor) from from_buf->buf.
static int select_launch(int32_t S, int32_t N, int32_t W, int32_t tile_tokens,
                         const cocodiff_bf16* v_cur, const cocodiff_bf16* v_prev, float tau,
                         int32_t* flags, int32_t* active_idx, int32_t* n_active,
                         cocodiff_bf16* compact, int32_t cap_tiles,
                         void* workspace, size_t workspace_bytes, const UnpackSource* from_buf, void* stream) {
    SelectShape sh;
    int rc = select_shape(S, N, W, tile_tokens, &sh);
    if (rc != COCODIFF_OK) return rc;
    if (!v_cur || !v_prev || !active_idx || !n_active || !workspace)
        return fail(COCODIFF_ERR_NULL, "select: v_cur, v_prev, active_idx, n_active and workspace are required");
    if (!aligned16(v_cur) || !aligned16(v_prev) || !aligned16(workspace) || (compact && !aligned16(compact)))
        return fail(COCODIFF_ERR_ALIGN, "select: tensors and workspace must be 16-byte aligned");
    if (compact && cap_tiles < 1) return fail(COCODIFF_ERR_CAPACITY, "select: cap_tiles (%d) must be >= 1", cap_tiles);
    const size_t need = (size_t)sh.NT * sizeof(int32_t);
    if (workspace_bytes < need)
        return fail(COCODIFF_ERR_CAPACITY, "select: workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    hipStream_t st = as_stream(stream);
    uint32_t* tile_flag = (uint32_t*)workspace;    // one word per tile, a byte per workgroup of the flag pass

    const size_t touched = (size_t)S * sh.slab8 * 32;
    // flag pass: a tile is cut into at most 4 shares of whole 256-vector rows, about kSelUnroll vectors per lane
    const uint32_t per_tile = sh.S * sh.seg8;
    const uint32_t want = (per_tile + kSelUnroll * kSelThreads - 1) / (kSelUnroll * kSelThreads);
    const uint32_t parts_max = want < 1 ? 1 : want > 4 ? 4 : want;
    const uint32_t share = ((per_tile + parts_max - 1) / parts_max + kSelThreads - 1) / kSelThreads * kSelThreads;
    const uint32_t parts = (per_tile + share - 1) / share;                  // every share non-empty
    const uint32_t mask = parts >= 4 ? 0xffffffffu : (1u << (8 * parts)) - 1u;
    // v_cur stays cached: the second launch reads the active tiles again (streaming loads of v_cur were measured on
    // tensors of 127 and 613 MB too: 5 % slower and equal)
    FlagPass fp;
    fp.cur = (const vec16*)v_cur;
    fp.prev = (const vec16*)v_prev;
    fp.flag_bytes = (uint8_t*)tile_flag;
    fp.sh = sh;
    fp.share = share;
    fp.th = make_thresholds(tau);
    fp.u = from_buf ? *from_buf : UnpackSource{};
    // the fast form: multiply-high division is exact while (largest dividend) * divisor < 2^32; 32-bit byte offsets
    // need every tensor below 4 GiB
    bool magic = (uint64_t)S * sh.slab8 * 16u < ((uint64_t)1 << 32);
    auto divisor = [&](uint32_t d, uint64_t max_n) {
        Divisor f{d ? d : 1u, 0u};
        if (f.d > 1u) f.magic = (uint32_t)((((uint64_t)1 << 32) + f.d - 1) / f.d);
        if (max_n * f.d >= ((uint64_t)1 << 32)) magic = false;
        return f;
    };
    fp.seg8 = divisor(sh.seg8, per_tile);
    fp.d8 = divisor(from_buf ? fp.u.d8 : 1u, sh.seg8);
    fp.Ns = divisor(from_buf ? fp.u.Ns : 1u, (uint64_t)N);
    fp.Hp = divisor(from_buf ? fp.u.Hp : 1u, sh.S);
    with_policy(from_buf != nullptr, stream_loads_once(touched), [&](auto F, auto Pv) {
        constexpr bool fb = decltype(F)::value, pv = decltype(Pv)::value;
        constexpr int unroll = fb ? kFlagUnroll : kFlagUnrollPlain;
        if (magic)
            hipLaunchKernelGGL((select_flag_kernel<pv, fb, unroll, true>), dim3(sh.NT, parts), dim3(kSelThreads), 0, st, fp);
        else
            hipLaunchKernelGGL((select_flag_kernel<pv, fb, unroll, false>), dim3(sh.NT, parts), dim3(kSelThreads), 0, st, fp);
    });
    rc = check_launch("select_flag_kernel");
    if (rc != COCODIFF_OK) return rc;
    TileFlags tf;
    tf.words_ptr = tile_flag;
    tf.words = 1;
    tf.mask[0] = mask;
    tf.mask[1] = tf.mask[2] = tf.mask[3] = 0;
    return select_finish_launch(S, N, W, tile_tokens, v_cur, tf, flags, active_idx, n_active, compact, cap_tiles, stream);
}

extern "C" int cocodiff_vmajor_select(int32_t S, int32_t N, int32_t W, int32_t tile_tokens,
                                      const cocodiff_bf16* v_cur, const cocodiff_bf16* v_prev, float tau,
                                      int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                      cocodiff_bf16* compact, int32_t cap_tiles,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    return select_launch(S, N, W, tile_tokens, v_cur, v_prev, tau, flags, active_idx, n_active, compact, cap_tiles, workspace,
                         workspace_bytes, nullptr, stream);
}

// Address of `scratch` on the current device; asked once per device (every GPU holds its own copy of the array).
static int static_scratch(uint32_t** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static uint32_t* ptrs[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(COCODIFF_ERR_HIP, "select_static: no current device: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(COCODIFF_ERR_HIP, "select_static: device %d is outside the %d supported", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(COCODIFF_ERR_HIP, "select_static: cannot resolve the scratch array on device %d: %s", dev, hipGetErrorString(e));
        ptrs[dev] = static_cast<uint32_t*>(p);
    }
    *out = ptrs[dev];
    return COCODIFF_OK;
}

extern "C" int cocodiff_vmajor_select_static(int32_t S, int32_t N, int32_t W, int32_t tile_tokens,
                                             const cocodiff_bf16* v_cur, const cocodiff_bf16* v_prev, float tau,
                                             int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                             cocodiff_bf16* compact, int32_t cap_tiles, void* stream) {
    SelectShape sh;
    int rc = select_shape(S, N, W, tile_tokens, &sh);
    if (rc != COCODIFF_OK) return rc;
    if (sh.NT > kStaticMaxTiles)
        return fail(COCODIFF_ERR_CAPACITY, "select_static: %u tiles exceed the %u the library-owned scratch holds; "
                    "use cocodiff_vmajor_select with a caller workspace", sh.NT, kStaticMaxTiles);
    uint32_t* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != COCODIFF_OK) return rc;
    // the flag pass overwrites every byte of the flag words the gather pass reads: nothing of an earlier call survives
    return select_launch(S, N, W, tile_tokens, v_cur, v_prev, tau, flags, active_idx, n_active, compact, cap_tiles, ws,
                         (size_t)kStaticMaxTiles * sizeof(uint32_t), nullptr, stream);
}

extern "C" int cocodiff_a2a_unpack_select(const cocodiff_shape* shape, const cocodiff_bf16* vbuf, int slot_order,
                                          cocodiff_bf16* v_hs, const cocodiff_bf16* v_prev, int32_t tile_tokens, float tau,
                                          int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                          cocodiff_bf16* compact, int32_t cap_tiles,
                                          void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (shape->rank_begin != 0 || shape->rank_count != shape->P)
        return fail(COCODIFF_ERR_SHAPE, "unpack_select: a tile's flag needs every head, so the rank range must be all P ranks");
    if (slot_order != COCODIFF_SEND_MAJOR && slot_order != COCODIFF_RECV_MAJOR)
        return fail(COCODIFF_ERR_SHAPE, "unpack_select: slot_order (%d) must be SEND_MAJOR or RECV_MAJOR", slot_order);
    if (!vbuf) return fail(COCODIFF_ERR_NULL, "unpack_select: vbuf is NULL");
    if (!aligned16(vbuf)) return fail(COCODIFF_ERR_ALIGN, "unpack_select: vbuf must be 16-byte aligned");
    UnpackSource u;
    u.buf = (const vec16*)vbuf;
    u.hs_out = (vec16*)v_hs;
    u.Ns = (uint32_t)(shape->N / shape->P);
    u.P = (uint32_t)shape->P;
    u.Hp = (uint32_t)(shape->H / shape->P);
    u.d8 = (uint32_t)(shape->d / 8);
    u.T = (uint32_t)tile_tokens;
    u.row8 = u.Hp * u.d8;
    u.chunk8 = u.Ns * u.row8;
    u.recv_major = slot_order == COCODIFF_RECV_MAJOR;
    return select_launch(shape->H, shape->N, shape->d, tile_tokens, v_hs, v_prev, tau, flags, active_idx, n_active, compact,
                         cap_tiles, workspace, workspace_bytes, &u, stream);
}

static int tile_move(bool gather, int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const void* x, const void* compact,
                     const int32_t* active_idx, const int32_t* n_active, int32_t cap_tiles, void* stream) {
    const char* who = gather ? "vmajor_gather" : "vmajor_scatter";
    SelectShape sh;
    int rc = select_shape(S, N, W, tile_tokens, &sh);
    if (rc != COCODIFF_OK) return rc;
    if (!x || !compact || !active_idx || !n_active) return fail(COCODIFF_ERR_NULL, "%s: NULL pointer", who);
    if (!aligned16(x) || !aligned16(compact)) return fail(COCODIFF_ERR_ALIGN, "%s: tensors must be 16-byte aligned", who);
    if (cap_tiles < 1) return fail(COCODIFF_ERR_CAPACITY, "%s: cap_tiles (%d) must be >= 1", who, cap_tiles);
    const uint32_t blocks = (uint32_t)cap_tiles < sh.NT ? (uint32_t)cap_tiles : sh.NT;
    const uint32_t pieces = (sh.S * sh.seg8 + kSelUnroll * kSelThreads - 1) / (kSelUnroll * kSelThreads);
    const dim3 grid(blocks, pieces < 64 ? pieces : 64);
    if (gather)
        hipLaunchKernelGGL(tile_move_kernel<true>, grid, dim3(kSelThreads), 0, as_stream(stream), (vec16*)x,
                           (vec16*)compact, active_idx, n_active, sh, (uint32_t)cap_tiles);
    else
        hipLaunchKernelGGL(tile_move_kernel<false>, grid, dim3(kSelThreads), 0, as_stream(stream), (vec16*)x,
                           (vec16*)compact, active_idx, n_active, sh, (uint32_t)cap_tiles);
    return check_launch(who);
}

extern "C" int cocodiff_vmajor_gather(int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const cocodiff_bf16* x,
                                      const int32_t* active_idx, const int32_t* n_active, cocodiff_bf16* compact,
                                      int32_t cap_tiles, void* stream) {
    return tile_move(true, S, N, W, tile_tokens, x, compact, active_idx, n_active, cap_tiles, stream);
}

extern "C" int cocodiff_vmajor_scatter(int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const cocodiff_bf16* compact,
                                       const int32_t* active_idx, const int32_t* n_active, cocodiff_bf16* cache,
                                       int32_t cap_tiles, void* stream) {
    return tile_move(false, S, N, W, tile_tokens, cache, compact, active_idx, n_active, cap_tiles, stream);
}
