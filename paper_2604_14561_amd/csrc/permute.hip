// The two Ulysses all-to-alls on one GPU (paper Section II-A): before attention, sequence-parallel ->
// head-parallel (pack the send chunks, unpack the received chunks head-major); after attention the way back
// (pack from the head-parallel tensor, unpack token-major).  Pure 128-bit permutation copies; HBM-bound.
//
// Units below are 16-byte vectors (8 bf16).  d8 = d/8 vectors per head row, D8 = D/8 per token row,
// row8 = Hp*d8 per chunk row, chunk8 = Ns*row8 per chunk.  A chunk always holds [Ns tokens][Hp heads][d] of
// one (token owner r, head owner p) pair; which of the two is the sender depends on the direction.
#include "internal.h"

namespace cocodiff {

constexpr int kThreads = 256;

struct PermuteArgs {
    uint32_t Ns, P, D8, d8, row8, chunk8;
    uint32_t N;           // tokens in total
    uint32_t first;       // token-major walk: first token of the range; head-major walk: first head of the range
    uint32_t n_vec;       // vectors this launch moves
    int recv_major;
};

__device__ __forceinline__ uint32_t slot_of(uint32_t sender, uint32_t receiver, uint32_t P, int recv_major) {
    return recv_major ? receiver * P + sender : sender * P + receiver;
}

// Walks the sequence-parallel tensor [N][H][d] linearly over the token range of the launch, one vector per thread
// (small workgroups measured fastest on cold data and disturb a concurrent projection least).
// TO_BUF: x_seq -> exchange buffer (first all-to-all, sender = token owner r, receiver = head owner p);
// else:   exchange buffer -> x_seq (second all-to-all, sender = head owner p, receiver = token owner r).
template <bool NT_LD, bool NT_ST, bool TO_BUF>
__global__ void __launch_bounds__(kThreads) seq_side_kernel(const vec16* __restrict__ in, vec16* __restrict__ out, PermuteArgs a) {
    const uint32_t g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= a.n_vec) return;
    const uint32_t tl = g / a.D8;            // token within the range
    const uint32_t v = g - tl * a.D8;        // vector within the token row
    const uint32_t n = a.first + tl;         // global token
    const uint32_t r = n / a.Ns;             // token owner
    const uint32_t m = n - r * a.Ns;         // token within the rank
    const uint32_t p = v / a.row8;           // head owner
    const uint32_t c = v - p * a.row8;       // (hl, i) within the chunk row
    const size_t seq_at = (size_t)n * a.D8 + v;
    const size_t buf_at = (size_t)(TO_BUF ? slot_of(r, p, a.P, a.recv_major) : slot_of(p, r, a.P, a.recv_major)) * a.chunk8 +
                          m * a.row8 + c;
    st_vec<NT_ST>(out + (TO_BUF ? buf_at : seq_at), ld_vec<NT_LD>(in + (TO_BUF ? seq_at : buf_at)));
}

// Walks the head-parallel tensor [H][N][d] linearly over the head range of the launch.
// TO_BUF: x_hs -> exchange buffer (second all-to-all, sender = head owner p, receiver = token owner r);
// else:   exchange buffer -> x_hs (first all-to-all, sender = token owner r, receiver = head owner p).
template <bool NT_LD, bool NT_ST, bool TO_BUF>
__global__ void __launch_bounds__(kThreads) head_side_kernel(const vec16* __restrict__ in, vec16* __restrict__ out, PermuteArgs a) {
    const uint32_t g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= a.n_vec) return;
    const uint32_t head8 = a.N * a.d8;       // vectors per head slab
    const uint32_t Hp = a.row8 / a.d8;
    const uint32_t hl_range = g / head8;
    const uint32_t rem = g - hl_range * head8;
    const uint32_t h = a.first + hl_range;   // global head
    const uint32_t n = rem / a.d8;           // global token
    const uint32_t i8 = rem - n * a.d8;
    const uint32_t p = h / Hp;               // head owner
    const uint32_t hl = h - p * Hp;
    const uint32_t r = n / a.Ns;             // token owner
    const uint32_t m = n - r * a.Ns;
    const size_t hs_at = (size_t)a.first * head8 + g;
    const size_t buf_at = (size_t)(TO_BUF ? slot_of(p, r, a.P, a.recv_major) : slot_of(r, p, a.P, a.recv_major)) * a.chunk8 +
                          m * a.row8 + hl * a.d8 + i8;
    st_vec<NT_ST>(out + (TO_BUF ? buf_at : hs_at), ld_vec<NT_LD>(in + (TO_BUF ? hs_at : buf_at)));
}

static int check_permute(const cocodiff_shape* s, const void* in, const void* out, int slot_order, const char* who) {
    int rc = check_shape(s);
    if (rc != COCODIFF_OK) return rc;
    if (!in || !out) return fail(COCODIFF_ERR_NULL, "%s: NULL tensor pointer", who);
    if (!aligned16(in) || !aligned16(out)) return fail(COCODIFF_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
    if (slot_order != COCODIFF_SEND_MAJOR && slot_order != COCODIFF_RECV_MAJOR)
        return fail(COCODIFF_ERR_SHAPE, "%s: slot_order (%d) must be SEND_MAJOR or RECV_MAJOR", who, slot_order);
    if ((int64_t)s->N * s->D / 8 >= (int64_t)1 << 31)
        return fail(COCODIFF_ERR_SHAPE, "%s: N*D/8 must be below 2^31", who);
    return COCODIFF_OK;
}

static PermuteArgs make_args(const cocodiff_shape* s, int slot_order) {
    PermuteArgs a;
    a.Ns = s->N / s->P;
    a.P = s->P;
    a.D8 = s->D / 8;
    a.d8 = s->d / 8;
    a.row8 = (s->H / s->P) * a.d8;
    a.chunk8 = a.Ns * a.row8;
    a.N = s->N;
    a.first = 0;
    a.n_vec = 0;
    a.recv_major = slot_order == COCODIFF_RECV_MAJOR;
    return a;
}

// Token-major walk over the ranks of the shape's range (they are token owners).
template <bool TO_BUF>
static int launch_seq_side(const cocodiff_shape* shape, const void* in, void* out, int slot_order, void* stream, const char* who) {
    int rc = check_permute(shape, in, out, slot_order, who);
    if (rc != COCODIFF_OK) return rc;
    PermuteArgs a = make_args(shape, slot_order);
    a.first = shape->rank_begin * a.Ns;
    a.n_vec = (uint32_t)shape->rank_count * a.Ns * a.D8;
    const dim3 grid((a.n_vec + kThreads - 1) / kThreads), block(kThreads);
    with_policy(stream_loads((size_t)a.n_vec * 32), stream_stores((size_t)a.n_vec * 32), [&](auto L, auto S) {
        hipLaunchKernelGGL((seq_side_kernel<decltype(L)::value, decltype(S)::value, TO_BUF>), grid, block, 0, as_stream(stream),
                           (const vec16*)in, (vec16*)out, a);
    });
    return check_launch(who);
}

// Head-major walk over the ranks of the shape's range (they are head owners).
template <bool TO_BUF>
static int launch_head_side(const cocodiff_shape* shape, const void* in, void* out, int slot_order, void* stream, const char* who) {
    int rc = check_permute(shape, in, out, slot_order, who);
    if (rc != COCODIFF_OK) return rc;
    PermuteArgs a = make_args(shape, slot_order);
    const uint32_t Hp = shape->H / shape->P;
    a.first = shape->rank_begin * Hp;
    a.n_vec = (uint32_t)shape->rank_count * Hp * a.N * a.d8;
    const dim3 grid((a.n_vec + kThreads - 1) / kThreads), block(kThreads);
    with_policy(stream_loads((size_t)a.n_vec * 32), stream_stores((size_t)a.n_vec * 32), [&](auto L, auto S) {
        hipLaunchKernelGGL((head_side_kernel<decltype(L)::value, decltype(S)::value, TO_BUF>), grid, block, 0, as_stream(stream),
                           (const vec16*)in, (vec16*)out, a);
    });
    return check_launch(who);
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" int cocodiff_a2a_pack(const cocodiff_shape* shape, const cocodiff_bf16* x_seq, cocodiff_bf16* xbuf,
                                 int slot_order, void* stream) {
    return launch_seq_side<true>(shape, x_seq, xbuf, slot_order, stream, "a2a_pack");
}

extern "C" int cocodiff_a2a_unpack(const cocodiff_shape* shape, const cocodiff_bf16* xbuf, cocodiff_bf16* x_hs,
                                   int slot_order, void* stream) {
    return launch_head_side<false>(shape, xbuf, x_hs, slot_order, stream, "a2a_unpack");
}

extern "C" int cocodiff_a2a_pack_hs(const cocodiff_shape* shape, const cocodiff_bf16* y_hs, cocodiff_bf16* xbuf,
                                    int slot_order, void* stream) {
    return launch_head_side<true>(shape, y_hs, xbuf, slot_order, stream, "a2a_pack_hs");
}

extern "C" int cocodiff_a2a_unpack_seq(const cocodiff_shape* shape, const cocodiff_bf16* xbuf, cocodiff_bf16* y_seq,
                                       int slot_order, void* stream) {
    return launch_seq_side<false>(shape, xbuf, y_seq, slot_order, stream, "a2a_unpack_seq");
}
