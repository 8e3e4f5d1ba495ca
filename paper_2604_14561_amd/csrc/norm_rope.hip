// Q/K RMSNorm fused with axial RoPE, in place (paper Section II-B; RMSNorm per Section III-C).
//
// One 16-byte vector (8 bf16 = 4 rotary pairs) per lane per step.  A head row of d elements is
// d8 = d/8 adjacent lanes; its sum of squares is reduced with cross-lane moves inside the wavefront.
// A wavefront owns a run of whole token rows: one token (D8 = D/8 vectors, a multiple of 64) walked in
// D8/64 steps, or 64/D8 short tokens in one step.  In both cases a lane keeps the same position inside
// its head and the same token for every step, so gamma and the token's cos/sin values are fetched
// once per lane and reused for every head.  HBM traffic: each element read once and written once.
// Variants of the same arithmetic (one shared device function): the result stored into the exchange buffer's
// chunks instead of in place (sender side), or the rows read from the chunks and stored head-parallel (receiver
// side: the unpack of the first all-to-all with norm + RoPE inside).
#include "internal.h"

namespace cocodiff {

struct NormRopeArgs {
    uint16_t* tensor[2];
    uint16_t* packed[2];              // PACK: the exchange buffers the result goes to (tensor[] is then read only)
    uint32_t Ns, P, row8, chunk8;     // PACK: tokens per rank, ranks, vectors per chunk row and per chunk
    int recv_major;
    const uint16_t* gamma[2];
    uint32_t D8, d8;
    uint32_t first_token, n_tokens;   // token range of this launch
    uint32_t steps;                   // D8/64 when D8 >= 64, else 1
    float inv_d, eps;
    RopeDev rope;
};

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over groups of `width` adjacent lanes (width a power of two, 1..64); every lane gets its group's sum.
__device__ __forceinline__ float group_sum(float v, uint32_t width) {
    if (width > 1) v += dpp<0xB1>(v);    // quad_perm [1,0,3,2]
    if (width > 2) v += dpp<0x4E>(v);    // quad_perm [2,3,0,1]
    if (width > 4) v += dpp<0x141>(v);   // row_half_mirror: the other quad of the 8-lane half row
    if (width > 8) v += dpp<0x140>(v);   // row_mirror: the other half of the 16-lane row
    if (width > 16) v += __shfl_xor(v, 16, 64);
    if (width > 32) v += __shfl_xor(v, 32, 64);
    return v;
}

// One 16-byte vector (8 elements = 4 rotary pairs) of a head row: RMSNorm over the row's d8 vectors (one per lane,
// adjacent lanes), scale by gamma, rotate.  Every kernel that normalises goes through this function, so the same
// row gives the same bits wherever it is done.
__device__ __forceinline__ vec16 norm_rope_vec(const vec16& in, const float (&g)[8], const float (&cs_c)[4],
                                               const float (&cs_s)[4], uint32_t d8, float inv_d, float eps) {
    const uint32_t w[4] = {in.x, in.y, in.z, in.w};
    float x[8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = bf16_lo(w[i]);
        x[2 * i + 1] = bf16_hi(w[i]);
        ss += x[2 * i] * x[2 * i] + x[2 * i + 1] * x[2 * i + 1];
    }
    ss = group_sum(ss, d8);
    const float rinv = 1.0f / sqrtf(ss * inv_d + eps);
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float e = x[2 * i] * rinv * g[2 * i];
        const float od = x[2 * i + 1] * rinv * g[2 * i + 1];
        o[i] = pack_bf16x2(e * cs_c[i] - od * cs_s[i], e * cs_s[i] + od * cs_c[i]);
    }
    return vec16{o[0], o[1], o[2], o[3]};
}

// gamma of the 8 elements of vector l of a head row, and (cos, sin) of its 4 pairs for the token with grid
// coordinates `coord`
__device__ __forceinline__ void load_gamma(const uint16_t* __restrict__ gamma, uint32_t l, float (&g)[8]) {
    const vec16 gv = *reinterpret_cast<const vec16*>(gamma + l * 8);
    g[0] = bf16_lo(gv.x); g[1] = bf16_hi(gv.x); g[2] = bf16_lo(gv.y); g[3] = bf16_hi(gv.y);
    g[4] = bf16_lo(gv.z); g[5] = bf16_hi(gv.z); g[6] = bf16_lo(gv.w); g[7] = bf16_hi(gv.w);
}

__device__ __forceinline__ void load_cos_sin(const RopeDev& rope, uint32_t n, uint32_t l, float (&cs_c)[4], float (&cs_s)[4]) {
    // grid coordinates of the token (last axis fastest)
    uint32_t coord[3] = {0, 0, 0};
    uint32_t rem = n;
    for (int ax = rope.n_axes - 1; ax >= 0; --ax) {
        const uint32_t gsz = (uint32_t)rope.grid[ax];
        coord[ax] = rem % gsz;
        rem /= gsz;
    }
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        uint32_t j = l * 4 + jj;
        int ax = 0;
        while (ax < rope.n_axes - 1 && j >= (uint32_t)rope.pairs[ax]) {
            j -= (uint32_t)rope.pairs[ax];
            ++ax;
        }
        const float2 v = *reinterpret_cast<const float2*>(rope.cs + rope.offset[ax] + ((size_t)coord[ax] * rope.pairs[ax] + j) * 2);
        cs_c[jj] = v.x;
        cs_s[jj] = v.y;
    }
}

constexpr int kMaxSteps = 8;

template <int STEPS, bool NT_LD, bool NT_ST, bool PACK>   // STEPS 0 = any number of steps, taken kMaxSteps at a time
__global__ void __launch_bounds__(256) norm_rope_kernel(NormRopeArgs a) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t run = blockIdx.x * 4 + (threadIdx.x >> 6);
    uint16_t* __restrict__ base = a.tensor[blockIdx.y];
    const uint16_t* __restrict__ gamma = a.gamma[blockIdx.y];

    // which token this lane works on, and where in its row the lane starts
    uint32_t tok_local, v_first;
    if (a.D8 >= 64) {
        tok_local = run;
        v_first = lane;
    } else {
        const uint32_t per_wave = 64 / a.D8;
        tok_local = run * per_wave + lane / a.D8;
        v_first = lane % a.D8;
    }
    if (tok_local >= a.n_tokens) return;   // whole groups of d8 lanes leave together (d8 divides D8)
    const uint32_t n = a.first_token + tok_local;
    const uint32_t l = lane % a.d8;        // vector index inside the head row; pairs 4l .. 4l+3

    float g[8], cs_c[4], cs_s[4];
    load_gamma(gamma, l, g);
    load_cos_sin(a.rope, n, l, cs_c, cs_s);

    vec16* row = reinterpret_cast<vec16*>(base) + (size_t)n * a.D8 + v_first;
    // PACK: vector v of token n = r*Ns + m goes to chunk (sender r, receiver p = v / row8), row m, column v % row8
    vec16* const pbase = PACK ? reinterpret_cast<vec16*>(a.packed[blockIdx.y]) : nullptr;
    const uint32_t r_own = PACK ? n / a.Ns : 0u;
    const uint32_t m_in = PACK ? n - r_own * a.Ns : 0u;
    const uint32_t total_steps = STEPS ? (uint32_t)STEPS : a.steps;
    for (uint32_t s0 = 0; s0 < total_steps; s0 += kMaxSteps) {
        constexpr int UN = STEPS ? (STEPS < kMaxSteps ? STEPS : kMaxSteps) : kMaxSteps;
        vec16 in[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k)
            if (STEPS || s0 + k < total_steps) in[k] = ld_vec<NT_LD>(row + (size_t)(s0 + k) * 64);
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            if (!(STEPS || s0 + k < total_steps)) continue;
            const vec16 out = norm_rope_vec(in[k], g, cs_c, cs_s, a.d8, a.inv_d, a.eps);
            if (PACK) {
                const uint32_t v = v_first + (s0 + k) * 64u;
                const uint32_t p = v / a.row8, c = v - p * a.row8;
                const size_t slot = a.recv_major ? (size_t)p * a.P + r_own : (size_t)r_own * a.P + p;
                st_vec<NT_ST>(pbase + slot * a.chunk8 + (size_t)m_in * a.row8 + c, out);
            } else {
                st_vec<NT_ST>(row + (size_t)(s0 + k) * 64, out);
            }
        }
    }
}

// Receiver-side unpack of the first all-to-all with the normalisation and the rotation done on the way: walks the
// head-parallel tensor [H][N][d] linearly over the head range of the launch, one vector per lane (a head row is d8
// adjacent lanes), reads the vector from its chunk of the exchange buffer, which holds the projection as it came
// out of the matrix cores.  The pass is HBM-bound, so the arithmetic rides along for nothing.
struct UnpackNormArgs {
    const uint16_t* buf[2];
    uint16_t* hs[2];
    const uint16_t* gamma[2];
    uint32_t N, Ns, P, Hp, d8, row8, chunk8;
    uint32_t first_head, n_heads;     // head range of the launch
    uint32_t heads_per_z;             // heads one workgroup handles (blockIdx.z walks the range in such groups)
    int recv_major;
    float inv_d, eps;
    RopeDev rope;
};

constexpr int kUnpackHeads = 6;   // vectors a lane keeps in flight

// A lane owns vector i8 of token n for every head of the launch's range, so gamma and the token's cos / sin are
// fetched once per lane; kUnpackHeads heads are in flight at a time.
template <bool NT_LD, bool NT_ST>
__global__ void __launch_bounds__(256) unpack_norm_rope_kernel(UnpackNormArgs a) {
    const uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g >= a.N * a.d8) return;           // whole head rows leave together: d8 divides 64
    const vec16* __restrict__ buf = reinterpret_cast<const vec16*>(a.buf[blockIdx.y]);
    vec16* __restrict__ hs = reinterpret_cast<vec16*>(a.hs[blockIdx.y]);
    const uint32_t n = g / a.d8, i8 = g - n * a.d8;
    const uint32_t r = n / a.Ns, m = n - r * a.Ns;
    float gm[8], cs_c[4], cs_s[4];
    load_gamma(a.gamma[blockIdx.y], i8, gm);
    load_cos_sin(a.rope, n, i8, cs_c, cs_s);
    const size_t head8 = (size_t)a.N * a.d8;
    const size_t row_at = (size_t)m * a.row8 + i8;
    const uint32_t h_end = min(a.n_heads, (blockIdx.z + 1u) * a.heads_per_z);
    for (uint32_t h0 = blockIdx.z * a.heads_per_z; h0 < h_end; h0 += kUnpackHeads) {
        vec16 in[kUnpackHeads];
#pragma unroll
        for (int u = 0; u < kUnpackHeads; ++u) {
            if (h0 + u < h_end) {
                const uint32_t h = a.first_head + h0 + u;
                const uint32_t p = h / a.Hp, hl = h - p * a.Hp;
                const size_t slot = a.recv_major ? (size_t)p * a.P + r : (size_t)r * a.P + p;
                in[u] = ld_vec<NT_LD>(buf + slot * a.chunk8 + row_at + hl * a.d8);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnpackHeads; ++u)
            if (h0 + u < h_end)
                st_vec<NT_ST>(hs + (a.first_head + h0 + u) * head8 + g, norm_rope_vec(in[u], gm, cs_c, cs_s, a.d8, a.inv_d, a.eps));
    }
}

int fill_rope(const cocodiff_shape* shape, const cocodiff_rope* rope, const char* who, RopeDev* out) {
    if (!rope || !rope->cs) return fail(COCODIFF_ERR_NULL, "%s: rope description or its table is NULL", who);
    if (!aligned16(rope->cs)) return fail(COCODIFF_ERR_ALIGN, "%s: the rope table must be 16-byte aligned", who);
    if (rope->n_axes < 1 || rope->n_axes > 3) return fail(COCODIFF_ERR_SHAPE, "%s: rope n_axes (%d) must be 1..3", who, rope->n_axes);
    int64_t cells = 1, npairs = 0;
    for (int ax = 0; ax < rope->n_axes; ++ax) {
        if (rope->grid[ax] <= 0 || rope->pairs[ax] <= 0)
            return fail(COCODIFF_ERR_SHAPE, "%s: rope axis %d needs positive grid and pairs", who, ax);
        cells *= rope->grid[ax];
        npairs += rope->pairs[ax];
    }
    if (cells != shape->N) return fail(COCODIFF_ERR_SHAPE, "%s: grid has %lld cells, N is %d", who, (long long)cells, shape->N);
    if (npairs * 2 != shape->d) return fail(COCODIFF_ERR_SHAPE, "%s: rope pairs sum to %lld, d/2 is %d", who, (long long)npairs, shape->d / 2);
    out->n_axes = rope->n_axes;
    int32_t off = 0;
    for (int ax = 0; ax < 3; ++ax) {
        out->grid[ax] = ax < rope->n_axes ? rope->grid[ax] : 1;
        out->pairs[ax] = ax < rope->n_axes ? rope->pairs[ax] : 0;
        out->offset[ax] = off;
        if (ax < rope->n_axes) off += rope->grid[ax] * rope->pairs[ax] * 2;
    }
    out->cs = rope->cs;
    return COCODIFF_OK;
}

}  // namespace cocodiff

using namespace cocodiff;

extern "C" int cocodiff_a2a_unpack_norm_rope(const cocodiff_shape* shape, const cocodiff_bf16* qbuf, const cocodiff_bf16* kbuf,
                                             cocodiff_bf16* q_hs, cocodiff_bf16* k_hs,
                                             const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                             const cocodiff_rope* rope, int slot_order, void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (!qbuf && !kbuf) return fail(COCODIFF_ERR_NULL, "unpack_norm_rope: qbuf and kbuf are both NULL");
    if ((qbuf && (!q_hs || !gamma_q)) || (kbuf && (!k_hs || !gamma_k)))
        return fail(COCODIFF_ERR_NULL, "unpack_norm_rope: a given buffer needs its output tensor and its gamma");
    if (!aligned16(qbuf) || !aligned16(kbuf) || !aligned16(q_hs) || !aligned16(k_hs) || !aligned16(gamma_q) || !aligned16(gamma_k))
        return fail(COCODIFF_ERR_ALIGN, "unpack_norm_rope: pointers must be 16-byte aligned");
    if (slot_order != COCODIFF_SEND_MAJOR && slot_order != COCODIFF_RECV_MAJOR)
        return fail(COCODIFF_ERR_SHAPE, "unpack_norm_rope: slot_order (%d) must be SEND_MAJOR or RECV_MAJOR", slot_order);
    const uint32_t d8 = shape->d / 8;
    if ((d8 & (d8 - 1)) || d8 > 64)
        return fail(COCODIFF_ERR_SHAPE, "unpack_norm_rope: d (%d) must be 8 times a power of two, at most 512", shape->d);
    if ((int64_t)shape->N * shape->D / 8 >= (int64_t)1 << 31) return fail(COCODIFF_ERR_SHAPE, "unpack_norm_rope: N*D/8 must be below 2^31");
    UnpackNormArgs a;
    rc = fill_rope(shape, rope, "unpack_norm_rope", &a.rope);
    if (rc != COCODIFF_OK) return rc;
    int nt = 0;
    if (qbuf) { a.buf[nt] = qbuf; a.hs[nt] = q_hs; a.gamma[nt] = gamma_q; ++nt; }
    if (kbuf) { a.buf[nt] = kbuf; a.hs[nt] = k_hs; a.gamma[nt] = gamma_k; ++nt; }
    if (nt == 1) { a.buf[1] = a.buf[0]; a.hs[1] = a.hs[0]; a.gamma[1] = a.gamma[0]; }
    a.N = (uint32_t)shape->N;
    a.Ns = (uint32_t)(shape->N / shape->P);
    a.P = (uint32_t)shape->P;
    a.Hp = (uint32_t)(shape->H / shape->P);
    a.d8 = d8;
    a.row8 = a.Hp * d8;
    a.chunk8 = a.Ns * a.row8;
    a.first_head = (uint32_t)shape->rank_begin * a.Hp;
    a.n_heads = (uint32_t)shape->rank_count * a.Hp;
    a.recv_major = slot_order == COCODIFF_RECV_MAJOR;
    a.inv_d = 1.0f / (float)shape->d;
    a.eps = eps;
    static const uint32_t hpz = (uint32_t)tune_value("COCODIFF_UNPACK_HPZ", kUnpackHeads);   // measured best: one batch per lane
    a.heads_per_z = hpz < 1 ? 1 : hpz;
    const dim3 grid((a.N * d8 + 255u) / 256u, nt, (a.n_heads + a.heads_per_z - 1) / a.heads_per_z), block(256);
    const size_t touched = (size_t)nt * a.n_heads * a.N * d8 * 32;
    with_policy(stream_loads_once(touched), stream_stores(touched), [&](auto L, auto S) {
        hipLaunchKernelGGL((unpack_norm_rope_kernel<decltype(L)::value, decltype(S)::value>), grid, block, 0, as_stream(stream), a);
    });
    return check_launch("unpack_norm_rope_kernel");
}

// pack = false: in place on q / k.  pack = true: q / k are read, the result goes to qbuf / kbuf in chunk order.
static int norm_rope_launch(const cocodiff_shape* shape, cocodiff_bf16* q, cocodiff_bf16* k,
                            const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                            const cocodiff_rope* rope, cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, int slot_order, bool pack,
                            void* stream) {
    int rc = check_shape(shape);
    if (rc != COCODIFF_OK) return rc;
    if (pack) {
        if ((q && !qbuf) || (k && !kbuf)) return fail(COCODIFF_ERR_NULL, "qk_norm_rope_pack: exchange buffer missing for a given tensor");
        if (!aligned16(qbuf) || !aligned16(kbuf)) return fail(COCODIFF_ERR_ALIGN, "qk_norm_rope_pack: buffers must be 16-byte aligned");
        if (slot_order != COCODIFF_SEND_MAJOR && slot_order != COCODIFF_RECV_MAJOR)
            return fail(COCODIFF_ERR_SHAPE, "qk_norm_rope_pack: slot_order (%d) must be SEND_MAJOR or RECV_MAJOR", slot_order);
    }
    if (!q && !k) return fail(COCODIFF_ERR_NULL, "qk_norm_rope: q and k are both NULL");
    if ((q && !gamma_q) || (k && !gamma_k)) return fail(COCODIFF_ERR_NULL, "qk_norm_rope: gamma missing for a given tensor");
    if (!aligned16(q) || !aligned16(k) || !aligned16(gamma_q) || !aligned16(gamma_k))
        return fail(COCODIFF_ERR_ALIGN, "qk_norm_rope: pointers must be 16-byte aligned");
    const uint32_t d8 = shape->d / 8, D8 = shape->D / 8;
    if ((d8 & (d8 - 1)) || d8 > 64)
        return fail(COCODIFF_ERR_SHAPE, "qk_norm_rope: d (%d) must be 8 times a power of two, at most 512", shape->d);
    if (!(D8 % 64 == 0 || 64 % D8 == 0))
        return fail(COCODIFF_ERR_SHAPE, "qk_norm_rope: D/8 (%u) must divide 64 or be a multiple of 64", D8);
    RopeDev rope_dev;
    rc = fill_rope(shape, rope, "qk_norm_rope", &rope_dev);
    if (rc != COCODIFF_OK) return rc;

    NormRopeArgs a;
    int nt = 0;
    if (q) { a.tensor[nt] = q; a.gamma[nt] = gamma_q; a.packed[nt] = qbuf; ++nt; }
    if (k) { a.tensor[nt] = k; a.gamma[nt] = gamma_k; a.packed[nt] = kbuf; ++nt; }
    if (nt == 1) { a.tensor[1] = a.tensor[0]; a.gamma[1] = a.gamma[0]; a.packed[1] = a.packed[0]; }
    const uint32_t Ns = shape->N / shape->P;
    a.Ns = Ns;
    a.P = (uint32_t)shape->P;
    a.row8 = (uint32_t)(shape->H / shape->P) * d8;
    a.chunk8 = Ns * a.row8;
    a.recv_major = slot_order == COCODIFF_RECV_MAJOR;
    a.D8 = D8;
    a.d8 = d8;
    a.first_token = shape->rank_begin * Ns;
    a.n_tokens = shape->rank_count * Ns;
    a.steps = D8 >= 64 ? D8 / 64 : 1;
    a.inv_d = 1.0f / (float)shape->d;
    a.eps = eps;
    a.rope = rope_dev;

    const uint32_t tokens_per_wave = D8 >= 64 ? 1 : 64 / D8;
    const uint32_t runs = (a.n_tokens + tokens_per_wave - 1) / tokens_per_wave;
    const dim3 grid((runs + 3) / 4, nt), block(256);
    hipStream_t st = as_stream(stream);
    const size_t touched = (size_t)nt * a.n_tokens * D8 * 32;
    const bool nt_ld = stream_loads_once(touched), nt_st = stream_stores(touched);   // in place: every element read once
#define COCODIFF_NR_LAUNCH(S)                                                                                                \
    with_policy(nt_ld, nt_st, [&](auto L, auto W) {                                                                          \
        if (pack) hipLaunchKernelGGL((norm_rope_kernel<S, decltype(L)::value, decltype(W)::value, true>), grid, block, 0, st, a);  \
        else hipLaunchKernelGGL((norm_rope_kernel<S, decltype(L)::value, decltype(W)::value, false>), grid, block, 0, st, a);      \
    })
    switch (a.steps) {
        case 1: COCODIFF_NR_LAUNCH(1); break;
        case 2: COCODIFF_NR_LAUNCH(2); break;
        case 4: COCODIFF_NR_LAUNCH(4); break;
        case 6: COCODIFF_NR_LAUNCH(6); break;
        case 8: COCODIFF_NR_LAUNCH(8); break;
        default: COCODIFF_NR_LAUNCH(0); break;
    }
#undef COCODIFF_NR_LAUNCH
    return check_launch("norm_rope_kernel");
}

extern "C" int cocodiff_qk_norm_rope(const cocodiff_shape* shape, cocodiff_bf16* q, cocodiff_bf16* k,
                                     const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                     const cocodiff_rope* rope, void* stream) {
    return norm_rope_launch(shape, q, k, gamma_q, gamma_k, eps, rope, nullptr, nullptr, COCODIFF_SEND_MAJOR, false, stream);
}

extern "C" int cocodiff_qk_norm_rope_pack(const cocodiff_shape* shape, const cocodiff_bf16* q, const cocodiff_bf16* k,
                                          const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                          const cocodiff_rope* rope, cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, int slot_order,
                                          void* stream) {
    return norm_rope_launch(shape, const_cast<cocodiff_bf16*>(q), const_cast<cocodiff_bf16*>(k), gamma_q, gamma_k, eps, rope,
                            qbuf, kbuf, slot_order, true, stream);
}
