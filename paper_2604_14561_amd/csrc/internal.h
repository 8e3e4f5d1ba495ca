// Internal helpers shared by the HIP sources of libcocodiff (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <cstdlib>
#include <type_traits>
#include <stddef.h>
#include <stdint.h>

#include "../../include/cocodiff.h"

namespace cocodiff {

// Record a message for cocodiff_last_error() on this thread and return `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Shape rules of cocodiff_shape; returns COCODIFF_OK or records the violated rule.
int check_shape(const cocodiff_shape* s);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Check the launch that was just issued.
int check_launch(const char* what);

// The rotary description as the kernels take it: per-axis float offsets into the cos/sin table.
struct RopeDev {
    int32_t n_axes;
    int32_t grid[3];
    int32_t pairs[3];
    int32_t offset[3];   // float offset of each axis' [grid][pairs][2] table
    const float* cs;
};

// Rules of cocodiff_rope against `shape` (table present and aligned, 1..3 axes, grid cells == N, pairs == d/2);
// fills `out` or records the violated rule under the caller's name `who`.
int fill_rope(const cocodiff_shape* shape, const cocodiff_rope* rope, const char* who, RopeDev* out);

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// Cache policy of the HBM-bound kernels, from measurements on data that is not in the 256 MB last-level cache
// (rotating buffer sets) and on data that is:
//   * stores are non-temporal: nothing of the output stays in L2 to be written back when the kernel ends;
//   * loads of data that no later kernel reads again (the cached previous-step tensor, a tensor rewritten in
//     place) are non-temporal;
//   * other loads are cached while the launch touches less than ~192 MB (a consumer may find its producer's
//     output on chip) and non-temporal above.
// The library as shipped reads no environment variable.  A build with -DCOCODIFF_TUNING (measurement sweeps only)
// reads, once: COCODIFF_STREAM_LD_MB / _ST_MB / _ONCE_MB (the three thresholds below), COCODIFF_GEMM_TILE
// (tokens * 1000 + features: forces a projection tile shape) and COCODIFF_UNPACK_HPZ (heads per lane batch of the
// normalising unpack).
inline size_t tune_value(const char* name, size_t dflt) {
#ifdef COCODIFF_TUNING
    const char* e = getenv(name);
    return e ? (size_t)strtoull(e, nullptr, 10) : dflt;
#else
    (void)name;
    return dflt;
#endif
}
inline bool stream_loads(size_t bytes_touched) {
    static const size_t threshold = tune_value("COCODIFF_STREAM_LD_MB", 192) << 20;
    return bytes_touched > threshold;
}
inline bool stream_stores(size_t bytes_touched) {
    static const size_t threshold = tune_value("COCODIFF_STREAM_ST_MB", 0) << 20;
    return bytes_touched > threshold;
}
inline bool stream_loads_once(size_t bytes_touched) {
    static const size_t threshold = tune_value("COCODIFF_STREAM_ONCE_MB", 0) << 20;
    return bytes_touched > threshold;
}

// Calls f(std::bool_constant<nt_ld>{}, std::bool_constant<nt_st>{}): run-time policy -> template arguments.
template <typename F>
inline void with_policy(bool nt_ld, bool nt_st, F&& f) {
    if (nt_ld) {
        if (nt_st) f(std::true_type{}, std::true_type{});
        else f(std::true_type{}, std::false_type{});
    } else {
        if (nt_st) f(std::false_type{}, std::true_type{});
        else f(std::false_type{}, std::false_type{});
    }
}

// ---- device helpers -------------------------------------------------------

// One 16-byte vector (8 bf16), the unit every kernel moves; a native vector type, so the
// non-temporal load/store builtins accept it.
typedef uint32_t __attribute__((ext_vector_type(4))) vec16;

__device__ __forceinline__ vec16 ld_nt(const vec16* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_nt(vec16* p, vec16 v) { __builtin_nontemporal_store(v, p); }

// Streaming (non-temporal) or cached access, chosen at compile time.
template <bool STREAM> __device__ __forceinline__ vec16 ld_vec(const vec16* p) { return STREAM ? ld_nt(p) : *p; }
template <bool STREAM> __device__ __forceinline__ void st_vec(vec16* p, vec16 v) {
    if (STREAM) st_nt(p, v); else *p = v;
}

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Two bf16 packed in a 32-bit word: element 0 in the low half.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Round two floats to bf16 (nearest even; gfx950 has a packed convert) and pack them, a in the low half.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
    f32x2_t f = {a, b};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}


// ---- the selection's decision (used by the flag pass and by the projection that flags V on its way out) ----------

// The decision is NOT(|double(c) - double(p)| <= double(tau)).  The fp32 difference d = fl(c - p) decides it whenever
// |d| != tau (rounding is monotonic and tau is an fp32 value: |x| <= tau gives |d| <= tau, |d| > tau gives |x| > tau);
// only |d| == tau can hide a difference that exceeds tau by less than half an fp32 ulp, and only vectors with such a
// tie and no change are compared again in double.
//   vec_suspect: one compare per element for the streaming loop, NOT(|d| < tau_s): true for every change and every tie
//                (tau_s = tau, or the smallest positive fp32 when tau is 0, so that equal values are no suspects);
//   vec_changed: the fp32 decision plus a note of ties (tau_tie = tau, or NaN when tau is 0: a zero fp32 difference of
//                two bf16 values is exactly zero).
__device__ __forceinline__ bool vec_suspect(const vec16& c, const vec16& p, float tau_s) {
    const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
    const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
    bool suspect = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        suspect |= !(fabsf(bf16_lo(cw[i]) - bf16_lo(pw[i])) < tau_s);
        suspect |= !(fabsf(bf16_hi(cw[i]) - bf16_hi(pw[i])) < tau_s);
    }
    return suspect;
}

__device__ __forceinline__ bool vec_changed(const vec16& c, const vec16& p, float tau, float tau_tie, bool& tie) {
    const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
    const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
    bool changed = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float dl = fabsf(bf16_lo(cw[i]) - bf16_lo(pw[i]));
        const float dh = fabsf(bf16_hi(cw[i]) - bf16_hi(pw[i]));
        changed |= !(dl <= tau);
        changed |= !(dh <= tau);
        tie |= dl == tau_tie;
        tie |= dh == tau_tie;
    }
    return changed;
}

__device__ __forceinline__ bool vec_changed_double(const vec16& c, const vec16& p, float tau) {
    const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
    const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
    const double tau_d = (double)tau;
    bool changed = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        changed |= !(fabs((double)bf16_lo(cw[i]) - (double)bf16_lo(pw[i])) <= tau_d);
        changed |= !(fabs((double)bf16_hi(cw[i]) - (double)bf16_hi(pw[i])) <= tau_d);
    }
    return changed;
}

struct Thresholds {
    float tau, tau_s, tau_tie;   // see vec_suspect / vec_changed
};

inline Thresholds make_thresholds(float tau) {
    Thresholds th;
    th.tau = tau;
    th.tau_s = tau > 0.f ? tau : (tau == 0.f ? __builtin_bit_cast(float, 1u) : tau);
    th.tau_tie = tau > 0.f ? tau : __builtin_nanf("");
    return th;
}

// Flag records of the selection: `words` 32-bit words per tile (1 or 4), of which the bytes set in mask[] were
// written, each by one workgroup of whichever pass produced the flags; a tile is active if any of them is non-zero.
struct TileFlags {
    const uint32_t* words_ptr;
    uint32_t words;
    uint32_t mask[4];
};

// Second pass of the selection on `stream`: list, count, optional per-tile flags and the compact copy of v_cur's
// active tiles, from flag records some earlier kernel on the same stream wrote.  Arguments as cocodiff_vmajor_select
// (validated there or by the caller).
int select_finish_launch(int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const cocodiff_bf16* v_cur, TileFlags tf,
                         int32_t* flags, int32_t* active_idx, int32_t* n_active, cocodiff_bf16* compact, int32_t cap_tiles,
                         void* stream);

}  // namespace cocodiff
