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
    uint32_t first;       // walk over x_seq: first token of the range; walk over x_hs: first head of the range
    uint32_t n_vec;       // vectors this launch moves
    int recv_major;
    uint32_t rank_begin, rank_count;     // the launch's ranks (buffer walks)
};

__device__ __forceinline__ uint32_t slot_of(uint32_t sender, uint32_t receiver, uint32_t P, int recv_major) {
    return recv_major ? receiver * P + sender : sender * P + receiver;
}

// Every kernel walks its OUTPUT linearly, one 16-byte vector per thread (small workgroups measured fastest on cold
// data and disturb a concurrent projection least): stores that run linearly through memory and loads that gather
// 512- or 256-byte pieces are faster than the other way round (cold, 57 MB tensors: 20 against 21.5 us).

// Exchange buffer -> sequence-parallel tensor [N][H][d] (second all-to-all: sender = head owner p, receiver = token
// owner r), linearly over the token range of the launch.
template <bool NT_LD, bool NT_ST>
__global__ void __launch_bounds__(kThreads) seq_from_buf_kernel(const vec16* __restrict__ in, vec16* __restrict__ out, PermuteArgs a) {
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
    const size_t buf_at = (size_t)slot_of(p, r, a.P, a.recv_major) * a.chunk8 + m * a.row8 + c;
    st_vec<NT_ST>(out + seq_at, ld_vec<NT_LD>(in + buf_at));
}

// Exchange buffer -> head-parallel tensor [H][N][d] (first all-to-all: sender = token owner r, receiver = head owner
// p), linearly over the head range of the launch.
template <bool NT_LD, bool NT_ST>
__global__ void __launch_bounds__(kThreads) heads_from_buf_kernel(const vec16* __restrict__ in, vec16* __restrict__ out, PermuteArgs a) {
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
    const size_t buf_at = (size_t)slot_of(r, p, a.P, a.recv_major) * a.chunk8 + m * a.row8 + hl * a.d8 + i8;
    st_vec<NT_ST>(out + hs_at, ld_vec<NT_LD>(in + buf_at));
}

// The packing directions: thread g of the launch is vector g of the chunks the launch's ranks send, in buffer order.
// Sequence-parallel tensor -> exchange buffer (first all-to-all): the senders are the token owners r of the rank range.
template <bool NT_LD, bool NT_ST>
__global__ void __launch_bounds__(kThreads) buf_from_seq_kernel(const vec16* __restrict__ in, vec16* __restrict__ out, PermuteArgs a) {
    const uint32_t g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= a.n_vec) return;
    const uint32_t ch = g / a.chunk8, rem = g - ch * a.chunk8;       // chunk of the launch, vector inside it
    // send-major: chunks (r, p) with p fastest; receive-major: (p, r) with r fastest
    const uint32_t r = a.rank_begin + (a.recv_major ? ch % a.rank_count : ch / a.P);
    const uint32_t p = a.recv_major ? ch / a.rank_count : ch % a.P;
    const uint32_t m = rem / a.row8, c = rem - m * a.row8;
    const size_t seq_at = (size_t)(r * a.Ns + m) * a.D8 + p * a.row8 + c;
    const size_t buf_at = (size_t)slot_of(r, p, a.P, a.recv_major) * a.chunk8 + rem;
    st_vec<NT_ST>(out + buf_at, ld_vec<NT_LD>(in + seq_at));
}

// Head-parallel tensor -> exchange buffer (second all-to-all): the senders are the head owners p of the rank range.
template <bool NT_LD, bool NT_ST>
__global__ void __launch_bounds__(kThreads) buf_from_heads_kernel(const vec16* __restrict__ in, vec16* __restrict__ out, PermuteArgs a) {
    const uint32_t g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= a.n_vec) return;
    const uint32_t ch = g / a.chunk8, rem = g - ch * a.chunk8;
    // send-major: chunks (p, r) with r fastest; receive-major: (r, p) with p fastest
    const uint32_t p = a.rank_begin + (a.recv_major ? ch % a.rank_count : ch / a.P);
    const uint32_t r = a.recv_major ? ch / a.rank_count : ch % a.P;
    const uint32_t m = rem / a.row8, c = rem - m * a.row8;           // token within the rank; (hl, i) within the chunk row
    const uint32_t hl = c / a.d8, i8 = c - hl * a.d8;
    const uint32_t Hp = a.row8 / a.d8;
    const size_t hs_at = ((size_t)(p * Hp + hl) * a.N + r * a.Ns + m) * a.d8 + i8;
    const size_t buf_at = (size_t)slot_of(p, r, a.P, a.recv_major) * a.chunk8 + rem;
    st_vec<NT_ST>(out + buf_at, ld_vec<NT_LD>(in + hs_at));
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
    a.rank_begin = (uint32_t)s->rank_begin;
    a.rank_count = (uint32_t)s->rank_count;
    return a;
}

// Between the sequence-parallel tensor and the buffer; the ranks of the shape's range are token owners.
template <bool TO_BUF>
static int launch_seq_side(const cocodiff_shape* shape, const void* in, void* out, int slot_order, void* stream, const char* who) {
    int rc = check_permute(shape, in, out, slot_order, who);
    if (rc != COCODIFF_OK) return rc;
    PermuteArgs a = make_args(shape, slot_order);
    a.first = shape->rank_begin * a.Ns;
    a.n_vec = (uint32_t)shape->rank_count * a.Ns * a.D8;
    const dim3 grid((a.n_vec + kThreads - 1) / kThreads), block(kThreads);
    with_policy(stream_loads((size_t)a.n_vec * 32), stream_stores((size_t)a.n_vec * 32), [&](auto L, auto S) {
        if (TO_BUF)      // (the same vectors, counted along the buffer)
            hipLaunchKernelGGL((buf_from_seq_kernel<decltype(L)::value, decltype(S)::value>), grid, block, 0, as_stream(stream),
                               (const vec16*)in, (vec16*)out, a);
        else
            hipLaunchKernelGGL((seq_from_buf_kernel<decltype(L)::value, decltype(S)::value>), grid, block, 0, as_stream(stream),
                               (const vec16*)in, (vec16*)out, a);
    });
    return check_launch(who);
}

// Between the head-parallel tensor and the buffer; the ranks of the shape's range are head owners.
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
        if (TO_BUF)
            hipLaunchKernelGGL((buf_from_heads_kernel<decltype(L)::value, decltype(S)::value>), grid, block, 0, as_stream(stream),
                               (const vec16*)in, (vec16*)out, a);
        else
            hipLaunchKernelGGL((heads_from_buf_kernel<decltype(L)::value, decltype(S)::value>), grid, block, 0, as_stream(stream),
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
