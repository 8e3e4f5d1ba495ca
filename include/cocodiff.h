/*
 * cocodiff.h -- C ABI of the MI355X (gfx950) library for the per-rank Ulysses
 * attention-input path that CoCoDiff reorganises.
 *
 * The path, per transformer layer (paper Sections II-A, II-B, III-C, III-D):
 *   1. project a shard of hidden states to Q, K, V (V can be computed alone,
 *      first: the V-First schedule),
 *   2. RMS-normalise Q and K per (token, head) and rotate them by the token's
 *      grid position (axial RoPE); V gets neither,
 *   3. build the all-to-all send chunks ("pack"), and lay the received chunks
 *      out head-major ("unpack"): sequence-parallel -> head-parallel layout,
 *   4. V-Major selection: find the 16-token tiles of V that changed since the
 *      cached previous denoising step, list them in ascending order and gather
 *      their current values densely.
 *
 * One GPU runs all P logical ranks' shares; `rank_begin`/`rank_count` choose
 * which ranks' shares one call covers, so a caller can run one rank alone or
 * all P at once.  With all ranks in one HBM the exchange between pack and
 * unpack is a re-indexing of the same buffer (see `slot_order`).
 *
 * Conventions for every entry point
 *   - returns 0 (COCODIFF_OK) or a negative COCODIFF_ERR_* code; on error nothing
 *     has been enqueued and cocodiff_last_error() holds a message (thread-local);
 *   - every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned,
 *     unless the comment says "host"; `shape`/`rope` structs are HOST pointers read
 *     during the call;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream); the call does not synchronise, does not allocate and issues no memset, so a
 *     sequence of calls can be captured into a HIP graph -- with one exception: the first
 *     call of the projection entry points and of cocodiff_vmajor_topk in a process sets a
 *     kernel attribute (LDS above 64 KB) and must happen outside a capture;
 *   - inputs are not modified; outputs must not alias inputs unless "in place" is stated;
 *   - bf16 values are raw 16-bit patterns (cocodiff_bf16); float arithmetic is fp32
 *     inside the kernels with one round-to-nearest-even to bf16 at each kernel's output;
 *   - the library reads no environment variable: which kernel runs depends on the arguments and the
 *     device only (measurement builds compiled with -DCOCODIFF_TUNING read a few COCODIFF_* tuning
 *     variables; the shipped build does not).
 */
#ifndef COCODIFF_H
#define COCODIFF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COCODIFF_API __attribute__((visibility("default")))

typedef uint16_t cocodiff_bf16;

enum {
    COCODIFF_OK = 0,
    COCODIFF_ERR_NULL = -1,     /* a required pointer is NULL */
    COCODIFF_ERR_SHAPE = -2,    /* shape rule violated (see cocodiff_shape) */
    COCODIFF_ERR_ALIGN = -3,    /* a data pointer is not 16-byte aligned */
    COCODIFF_ERR_CAPACITY = -4, /* workspace too small or cap_tiles < 1 */
    COCODIFF_ERR_HIP = -5       /* a launch failed; the message holds the HIP error string */
};

/* Where chunk(r -> p), the block rank r sends to rank p, lives in the exchange buffer. */
enum {
    COCODIFF_SEND_MAJOR = 0, /* slot r*P + p: rank r's contiguous send buffer (state before the exchange) */
    COCODIFF_RECV_MAJOR = 1  /* slot p*P + r: rank p's contiguous receive buffer (pack does a one-sided put) */
};

/*
 * Problem shape (Section II-A notation: N tokens, H heads of d, P ranks).
 * Rules (else COCODIFF_ERR_SHAPE): all > 0; D == H*d; d % 8 == 0; N % P == 0; H % P == 0;
 * (N/P) % 16 == 0 (the paper's even-split rule, plus whole 16-token tiles per rank);
 * 0 <= rank_begin, rank_count >= 1, rank_begin + rank_count <= P.
 * Rank r owns tokens [r*N/P, (r+1)*N/P) in the sequence-parallel layout and heads
 * [r*H/P, (r+1)*H/P) in the head-parallel layout.
 */
typedef struct cocodiff_shape {
    int32_t N, D, H, d, P;
    int32_t rank_begin, rank_count;
} cocodiff_shape;

/*
 * Axial rotary embedding (Section II-B).  Token n has grid coordinates in row-major order,
 * last axis fastest.  Adjacent elements (2j, 2j+1) of a head form pair j; the first pairs[0]
 * pairs rotate with axis 0, the next pairs[1] with axis 1, ...; pair j' (local index) of axis a
 * turns by coord_a * theta^(-j'/pairs[a]).
 * Rules: n_axes in {1,2,3}; product of grid[0..n_axes) == N; sum of pairs == d/2.
 * `cs` is a DEVICE table: for axis a at float offset 2 * sum_{b<a} grid[b]*pairs[b],
 * [grid[a]][pairs[a]][2] = (cos, sin) in fp32 -- exactly what cocodiff_rope_table_fill writes.
 */
typedef struct cocodiff_rope {
    int32_t n_axes;
    int32_t grid[3];
    int32_t pairs[3];
    float theta;
    const float* cs;
} cocodiff_rope;

/*
 * Step 1 -- projection (Section II-B: q_i = h_i W_Q, k_i = h_i W_K, v_i = h_i W_V; no bias).
 * x [N][D]; w* [D_out = D][D_in = D] (output-major: y[n][o] = sum_k x[n][k] * w[o][k]);
 * q, k, v [N][D] = [N][H][d].  Rows of the ranks in the range are computed; other rows untouched.
 * Any of the pairs (wq,q), (wk,k), (wv,v) may be NULL/NULL = skip that tensor, so V alone first
 * and then Q,K is the V-First order of Section III-C; at least one pair must be given, and a
 * pair given half (weight without output or the reverse) is COCODIFF_ERR_NULL.
 * bf16 inputs, fp32 accumulation on the matrix cores, one RNE rounding to bf16.
 */
COCODIFF_API int cocodiff_qkv_proj(const cocodiff_shape* shape, const cocodiff_bf16* x,
                      const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                      cocodiff_bf16* q, cocodiff_bf16* k, cocodiff_bf16* v, void* stream);

/*
 * Step 2 -- Q/K normalisation + RoPE (Section II-B; RMSNorm as in Section III-C), IN PLACE.
 * For each given tensor t in {q, k} ([N][H][d]), each token of the rank range, each head:
 * y = x / sqrt(mean(x^2) + eps) * gamma_t, then the rotation of cocodiff_rope at the token's
 * GLOBAL index.  gamma_q, gamma_k: [d] bf16, shared by all heads.  q or k may be NULL (skipped,
 * its gamma is then ignored); both NULL is COCODIFF_ERR_NULL.  V is never touched.
 * Extra shape rule: d/8 must be a power of two (d in 8..512) and D/8 a divisor or multiple of 64.
 */
COCODIFF_API int cocodiff_qk_norm_rope(const cocodiff_shape* shape, cocodiff_bf16* q, cocodiff_bf16* k,
                          const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                          const cocodiff_rope* rope, void* stream);

/*
 * Fusions of the steps above (same arithmetic, fewer passes over HBM; Section III-C keeps tensor preparation for
 * the exchange off the critical path -- here it disappears into the producing kernel):
 *
 * cocodiff_qkv_proj_pack  = cocodiff_qkv_proj followed by cocodiff_a2a_pack of every given tensor: the projection
 *   writes its rows straight into the exchange buffers qbuf / kbuf / vbuf ([P*P slots][N/P][H/P][d], slot order as
 *   in cocodiff_a2a_pack); no [N][D] tensor is written.  Bit-identical to the two calls.
 * cocodiff_qk_norm_rope_pack = cocodiff_qk_norm_rope followed by cocodiff_a2a_pack: q / k ([N][D], read only, not
 *   modified) are normalised and rotated on the way into qbuf / kbuf.  Bit-identical to the two calls.
 * Argument rules of the calls they replace apply; a given tensor needs its buffer (COCODIFF_ERR_NULL otherwise).
 */
COCODIFF_API int cocodiff_qkv_proj_pack(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                        const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                        cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order,
                                        void* stream);
COCODIFF_API int cocodiff_qk_norm_rope_pack(const cocodiff_shape* shape, const cocodiff_bf16* q, const cocodiff_bf16* k,
                                            const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                            const cocodiff_rope* rope, cocodiff_bf16* qbuf, cocodiff_bf16* kbuf,
                                            int slot_order, void* stream);

/*
 * cocodiff_qkv_proj_hs = cocodiff_qkv_proj followed by cocodiff_a2a_pack and cocodiff_a2a_unpack of every given
 * tensor, for ranks that share one memory (this library's case: all P logical ranks on one GPU): the projection's
 * epilogue writes each 16-byte row piece to its place in the head-parallel tensor q_hs / k_hs / v_hs [H][N][d]
 * (Section II-A: the layout the first all-to-all ends in), so pack, exchange and unpack are the store address and no
 * exchange buffer exists.  Bit-identical to the three calls.  Rows (tokens) of the rank range are computed, every
 * head of them; other tokens' rows are untouched.  Argument rules as for cocodiff_qkv_proj.
 */
COCODIFF_API int cocodiff_qkv_proj_hs(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                      const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                      cocodiff_bf16* q_hs, cocodiff_bf16* k_hs, cocodiff_bf16* v_hs, void* stream);

/*
 * cocodiff_qkv_proj_fused: the sender's whole share in the projection kernel.  For every given weight the epilogue
 * writes the result to its exchange buffer (qbuf / kbuf / vbuf, chunk order as cocodiff_a2a_pack writes it) AND to its
 * head-parallel tensor (q_hs / k_hs / v_hs [H][N][d], what cocodiff_a2a_unpack of that buffer gives); either of the
 * two destinations of a tensor may be NULL.  Q and K are RMS-normalised per (token, head) and rotated (Section II-B,
 * the rules of cocodiff_qk_norm_rope) on the fp32 accumulators before the one rounding to bf16, so their exchange
 * buffers carry normalised values (norm + RoPE on the sending side, the order of Section III-C) and they are rounded
 * once where the chain cocodiff_qkv_proj -> cocodiff_qk_norm_rope rounds twice: the results agree with that chain
 * to within the float tolerance, not bit for bit.  V is bit-identical to cocodiff_qkv_proj_pack / cocodiff_qkv_proj_hs.
 * The two destinations of a tensor hold the same bits.
 * Rules: as cocodiff_qkv_proj and cocodiff_qk_norm_rope; gamma_q / gamma_k required with wq / wk; rope required when Q
 * or K is given; d must be 64, 128 or 256; D a multiple of 64, at least 192 (COCODIFF_ERR_SHAPE otherwise).
 */
COCODIFF_API int cocodiff_qkv_proj_fused(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                         const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                         const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                         const cocodiff_rope* rope,
                                         cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order,
                                         cocodiff_bf16* q_hs, cocodiff_bf16* k_hs, cocodiff_bf16* v_hs, void* stream);

/*
 * cocodiff_qkv_proj_fused_select = cocodiff_qkv_proj_fused followed by cocodiff_vmajor_select on v_hs (head-parallel:
 * S = H, W = d) against v_prev ([H][N][d], the previous step's V): with tile_tokens = 16 (the tile of Section III-D) the
 * projection compares every vector of V with v_prev's as it writes it out, so the selection's first pass -- a read of
 * both tensors -- does not run; the selection's second pass (list, count, compact copy) follows on the same stream.
 * Bit-identical to the two calls in every output.  Other tile heights, or D above 4096, run as the two calls.
 * wv, vbuf and v_hs are required (Q and K stay optional); the rank range of `shape` must be all P ranks (a tile's flag
 * needs every head).  workspace: cocodiff_qkv_proj_fused_select_workspace_bytes(shape, tile_tokens) bytes (0 for bad
 * arguments), 16-byte aligned; nothing in it needs clearing and nothing survives the call.  Other arguments and error
 * behaviour as for the two calls.
 */
COCODIFF_API size_t cocodiff_qkv_proj_fused_select_workspace_bytes(const cocodiff_shape* shape, int32_t tile_tokens);
COCODIFF_API int cocodiff_qkv_proj_fused_select(const cocodiff_shape* shape, const cocodiff_bf16* x,
                                                const cocodiff_bf16* wq, const cocodiff_bf16* wk, const cocodiff_bf16* wv,
                                                const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                                const cocodiff_rope* rope,
                                                cocodiff_bf16* qbuf, cocodiff_bf16* kbuf, cocodiff_bf16* vbuf, int slot_order,
                                                cocodiff_bf16* q_hs, cocodiff_bf16* k_hs, cocodiff_bf16* v_hs,
                                                const cocodiff_bf16* v_prev, int32_t tile_tokens, float tau,
                                                int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                                cocodiff_bf16* compact, int32_t cap_tiles,
                                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * cocodiff_a2a_unpack_select = cocodiff_a2a_unpack of V followed by cocodiff_vmajor_select on the unpacked tensor
 * (head-parallel: S = H, W = d): the selection's first pass reads the current values from the exchange buffer
 * vbuf, writes them to their place in v_hs [H][N][d] and compares them with v_prev on the way, so the unpacked
 * tensor is not read again for the flags.  Bit-identical to the two calls (v_hs, flags, active_idx, n_active,
 * compact).  The rank range of `shape` must be all P ranks (a tile's flag needs every head).  Other arguments
 * and rules as for cocodiff_vmajor_select with S = H, N, W = d.
 */
COCODIFF_API int cocodiff_a2a_unpack_select(const cocodiff_shape* shape, const cocodiff_bf16* vbuf, int slot_order,
                                            cocodiff_bf16* v_hs, const cocodiff_bf16* v_prev, int32_t tile_tokens, float tau,
                                            int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                            cocodiff_bf16* compact, int32_t cap_tiles,
                                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * cocodiff_a2a_unpack_norm_rope: normalisation and rotation moved to the receiver side of the first all-to-all.
 * qbuf / kbuf hold the projection itself in chunk order (what cocodiff_qkv_proj_pack writes); the unpack pass
 * applies RMSNorm and RoPE (same arithmetic as cocodiff_qk_norm_rope, token index taken from the chunk) while it
 * moves the rows into q_hs / k_hs [H][N][d].  The result is bit-identical to cocodiff_qk_norm_rope followed by
 * cocodiff_a2a_pack and cocodiff_a2a_unpack; the exchange buffer carries un-normalised values instead.  The rank
 * range of `shape` names the RECEIVING ranks (head owners), as for cocodiff_a2a_unpack.  (qbuf, q_hs, gamma_q) or
 * (kbuf, k_hs, gamma_k) may be NULL together = skip that tensor.  d/8 must be a power of two.
 */
COCODIFF_API int cocodiff_a2a_unpack_norm_rope(const cocodiff_shape* shape, const cocodiff_bf16* qbuf, const cocodiff_bf16* kbuf,
                                               cocodiff_bf16* q_hs, cocodiff_bf16* k_hs,
                                               const cocodiff_bf16* gamma_q, const cocodiff_bf16* gamma_k, float eps,
                                               const cocodiff_rope* rope, int slot_order, void* stream);

/*
 * Step 3a -- pack (Section II-A all-to-all, sender side; Section III-B "tensor preparation").
 * x_seq [N][H][d] -> xbuf, P*P chunks of [N/P][H/P][d]:
 *   chunk(r->p)[n][hl][i] = x_seq[r*N/P + n][p*H/P + hl][i]   for SOURCE ranks r in the range.
 * xbuf holds N*D elements; chunks of other source ranks are not written.
 */
COCODIFF_API int cocodiff_a2a_pack(const cocodiff_shape* shape, const cocodiff_bf16* x_seq, cocodiff_bf16* xbuf,
                      int slot_order, void* stream);

/*
 * Step 3b -- unpack (receiver side): xbuf -> x_hs [H][N][d] (head-parallel, head-major):
 *   x_hs[p*H/P + hl][r*N/P + n][i] = chunk(r->p)[n][hl][i]   for DESTINATION ranks p in the range.
 * With the same slot_order as the pack, pack + unpack is the whole all-to-all:
 * x_hs[h][n][i] == x_seq[n][h][i].
 */
COCODIFF_API int cocodiff_a2a_unpack(const cocodiff_shape* shape, const cocodiff_bf16* xbuf, cocodiff_bf16* x_hs,
                        int slot_order, void* stream);

/*
 * Step 4 -- V-Major active-tile selection (Section III-D, threshold-per-tile form).
 * v_cur, v_prev: [S][N][W] bf16 (head-parallel: S = H, W = d; sequence layout: S = 1, W = D).
 * Tile t = tokens [t*tile_tokens, (t+1)*tile_tokens) of every slab s; NT = N / tile_tokens.
 *   flags[t]      = 1 if some element of the tile has NOT(|v_cur - v_prev| <= tau), else 0, decided on the
 *                   difference of the widened values in double precision, tau widened too (NaN counts as
 *                   changed; |diff| == tau does not; a difference that an fp32 subtraction would round
 *                   onto tau still counts as what it is).  [NT] int32, may be NULL.
 *   active_idx[j] = id of the j-th active tile, ascending, j < n_active.  [NT] int32.
 *   *n_active     = number of active tiles (device int32), also when it exceeds cap_tiles.
 *   compact[s][j*tile_tokens + m][w] = v_cur[s][active_idx[j]*tile_tokens + m][w] for
 *                   j < min(n_active, cap_tiles); [S][cap_tiles*tile_tokens][W]; NULL = indices only.
 * Entries of active_idx and compact beyond n_active are unspecified.  v_prev is read-only.
 * Rules: S, N, W, tile_tokens > 0; W % 8 == 0; N % tile_tokens == 0 (else COCODIFF_ERR_SHAPE);
 * cap_tiles >= 1 when compact != NULL (else COCODIFF_ERR_CAPACITY).
 * workspace: device scratch of at least cocodiff_vmajor_select_workspace_bytes(...) bytes; its contents on entry
 * are ignored (no clearing needed) and it may be reused by the next call on the same stream.
 */
COCODIFF_API int cocodiff_vmajor_select(int32_t S, int32_t N, int32_t W, int32_t tile_tokens,
                           const cocodiff_bf16* v_cur, const cocodiff_bf16* v_prev, float tau,
                           int32_t* flags, int32_t* active_idx, int32_t* n_active,
                           cocodiff_bf16* compact, int32_t cap_tiles,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * cocodiff_vmajor_select for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, results and rules, but no workspace -- the
 * flag words live in an array the library owns on each GPU (256 KiB per GPU, held until the process ends), so
 * nothing is allocated or freed by the call, here or by the caller.  Limit: N / tile_tokens <= 65536 tiles
 * (COCODIFF_ERR_CAPACITY beyond, nothing enqueued).  The device of `stream` must be the current device.  All
 * calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams without
 * an ordering between them) race and must use cocodiff_vmajor_select with separate workspaces instead; calls on
 * one stream, or otherwise ordered, are safe (nothing needs clearing between them).  The first call on a device
 * resolves the array's address (no allocation; do it outside a graph capture).
 */
COCODIFF_API int cocodiff_vmajor_select_static(int32_t S, int32_t N, int32_t W, int32_t tile_tokens,
                                  const cocodiff_bf16* v_cur, const cocodiff_bf16* v_prev, float tau,
                                  int32_t* flags, int32_t* active_idx, int32_t* n_active,
                                  cocodiff_bf16* compact, int32_t cap_tiles, void* stream);

/* Bytes of device scratch cocodiff_vmajor_select needs for this shape (0 on a bad shape). */
COCODIFF_API size_t cocodiff_vmajor_select_workspace_bytes(int32_t S, int32_t N, int32_t W, int32_t tile_tokens);

/*
 * V-Major, sender side (Section III-D: Q and K send only their active part; the list comes from V's selection).
 * compact[s][j*tile_tokens + m][w] = x[s][active_idx[j]*tile_tokens + m][w] for j < min(*n_active, cap_tiles).
 * x [S][N][W] (sequence layout: S = 1, W = D; head-parallel: S = H, W = d); compact [S][cap_tiles*tile_tokens][W];
 * active_idx, n_active: DEVICE data as written by cocodiff_vmajor_select (no host read, no synchronisation).
 * List entries outside [0, N/tile_tokens) are skipped.  Shape rules as for the selection; cap_tiles >= 1.
 */
COCODIFF_API int cocodiff_vmajor_gather(int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const cocodiff_bf16* x,
                                        const int32_t* active_idx, const int32_t* n_active, cocodiff_bf16* compact,
                                        int32_t cap_tiles, void* stream);

/*
 * V-Major, receiver side (Section III-D: indexed overwrite of the cached tensor), IN PLACE on `cache`:
 * cache[s][active_idx[j]*tile_tokens + m][w] = compact[s][j*tile_tokens + m][w] for j < min(*n_active, cap_tiles);
 * every other tile of cache [S][N][W] keeps its value.  Same argument rules as cocodiff_vmajor_gather.
 */
COCODIFF_API int cocodiff_vmajor_scatter(int32_t S, int32_t N, int32_t W, int32_t tile_tokens, const cocodiff_bf16* compact,
                                         const int32_t* active_idx, const int32_t* n_active, cocodiff_bf16* cache,
                                         int32_t cap_tiles, void* stream);

/*
 * V-Major selection as the paper states it (Section III-D), step 1: one scalar per token,
 * metric[n] = sum over the token's whole value vector (all slabs s, all w) of |v_cur - v_prev|, the L1 distance
 * to the cached value vector, accumulated in fp32.  v_cur, v_prev [S][N][W] bf16; metric [N] fp32 (device).
 * Rules: S, N, W > 0, W % 8 == 0.
 */
COCODIFF_API int cocodiff_vmajor_token_metric(int32_t S, int32_t N, int32_t W, const cocodiff_bf16* v_cur,
                                              const cocodiff_bf16* v_prev, float* metric, void* stream);

/*
 * Step 2, for n_seg independent segments of N tokens each (one per logical rank: a rank ranks its own tokens):
 * in every segment the n_keep tokens with the largest metric are active (the others stay cached).  NaN ranks
 * above every number; among equal metrics the lower token index is taken first, so the answer is unique.
 * metric [n_seg][N] fp32; active_idx [n_seg][N] int32: the first n_keep entries of row g receive segment g's
 * active token ids in ascending order, the rest of the row is left alone; the ids are local to the segment
 * (0 .. N-1) when global_ids == 0 and positions in the whole metric array (g*N + local) otherwise; n_active [n_seg],
 * every entry = n_keep (all DEVICE).  With global ids, (active_idx + g*N, n_active + g) is the list / count pair
 * cocodiff_vmajor_gather and _scatter take with tile_tokens = 1 on the tensor the metric was computed from, so
 * the chain metric -> top-k -> gather needs no host step.
 * Rules: n_seg, N > 0, n_seg * N < 2^31, 0 <= n_keep <= N.
 */
COCODIFF_API int cocodiff_vmajor_topk(int32_t n_seg, int32_t N, const float* metric, int32_t n_keep, int32_t global_ids,
                                      int32_t* active_idx, int32_t* n_active, void* stream);

/*
 * Time-varying cache schedule (Section III-D), host arithmetic: number of active tokens at denoising step `step`
 * (1-based, 1..n_steps).  Steps up to `warmup` and every sync_every-th step exchange everything (n_tokens);
 * otherwise the cache ratio r rises linearly from 0 at the warm-up boundary to 1 at the last step and
 * floor(r * n_tokens) tokens stay cached.  sync_every <= 0 disables the periodic full update.  Returns -1 on
 * bad arguments.  The paper's setup is n_steps = 50, warmup = 5, sync_every = 10.
 */
COCODIFF_API int32_t cocodiff_cache_active_count(int32_t step, int32_t n_steps, int32_t warmup, int32_t sync_every,
                                                 int32_t n_tokens);

/*
 * Second all-to-all (Section II-A: after attention, head-parallel back to sequence-parallel), sender side.
 * y_hs [H][N][d] -> xbuf, P*P chunks of [N/P][H/P][d]:
 *   chunk(p->r)[n][hl][i] = y_hs[p*H/P + hl][r*N/P + n][i]   for SOURCE ranks p (head owners) in the range.
 * Slot of chunk(p->r): p*P + r (SEND_MAJOR) or r*P + p (RECV_MAJOR).
 */
COCODIFF_API int cocodiff_a2a_pack_hs(const cocodiff_shape* shape, const cocodiff_bf16* y_hs, cocodiff_bf16* xbuf,
                                      int slot_order, void* stream);

/*
 * Second all-to-all, receiver side: xbuf -> y_seq [N][H][d]:
 *   y_seq[r*N/P + n][p*H/P + hl][i] = chunk(p->r)[n][hl][i]   for DESTINATION ranks r (token owners) in the range.
 * With the same slot_order, pack_hs + unpack_seq gives y_seq[n][h][i] == y_hs[h][n][i]; after
 * cocodiff_a2a_pack + cocodiff_a2a_unpack it returns the original tensor.
 */
COCODIFF_API int cocodiff_a2a_unpack_seq(const cocodiff_shape* shape, const cocodiff_bf16* xbuf, cocodiff_bf16* y_seq,
                                         int slot_order, void* stream);

/* Host helpers (not on the hot path). */

/* Which tile the projection takes for this shape's rank range and n_tensors (1..3) weights in one launch, on the
 * current device: tile extent in tokens and features, number of workgroups (= tiles), compute units of the device.
 * whole_heads != 0: the choice cocodiff_qkv_proj_fused makes (its tiles are 256 features wide), else that of the
 * other projection calls.  Any out pointer may be NULL.  Host arithmetic only; it needs a current HIP device for
 * the unit count (COCODIFF_ERR_HIP without one).  For reports and for tests that must land on a given tile shape. */
COCODIFF_API int cocodiff_qkv_proj_plan(const cocodiff_shape* shape, int32_t n_tensors, int32_t whole_heads,
                                        int32_t* tile_tokens, int32_t* tile_features, int32_t* n_tiles,
                                        int32_t* n_compute_units);

/* Bytes of the cos/sin table described at cocodiff_rope (0 on a bad description; `cs` is ignored). */
COCODIFF_API size_t cocodiff_rope_table_bytes(const cocodiff_rope* rope);

/* Fill a HOST buffer of cocodiff_rope_table_bytes(rope) bytes; angles and cos/sin are computed in
 * fp64 and stored as fp32.  The caller uploads it and points rope->cs at the device copy. */
COCODIFF_API int cocodiff_rope_table_fill(const cocodiff_rope* rope, float* host_out);

/* Plain 128-bit copy kernel (dst[i] = src[i], `bytes` a multiple of 16): the calibration kernel the
 * HBM-bound steps are priced against; used by the benchmark and the profiler-counter scaling. */
COCODIFF_API int cocodiff_util_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Register-only matrix-core loop (v_mfma_f32_16x16x32_bf16, the projection kernel's instruction, on a 4 x 8 outer
 * product of pseudo-random operand fragments as in that kernel; no memory traffic): the calibration kernel the
 * projection is priced against besides the published peak.  Launches `blocks` workgroups of 8 wavefronts, each
 * wavefront issuing iters * 32 MFMAs; `sink` is one DEVICE float that is practically never written.  Returns the
 * floating-point operations of the launch (> 0) or a negative error code; the caller times the launch. */
COCODIFF_API int64_t cocodiff_util_mfma_rate(int32_t blocks, int32_t iters, float* sink, void* stream);

COCODIFF_API const char* cocodiff_version(void);
COCODIFF_API const char* cocodiff_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* COCODIFF_H */
