/*
 * CPU oracle, integer/index part (TEST INFRASTRUCTURE ONLY; never linked into
 * or called by the product library).
 *
 * Explicit index loops, one statement per definition:
 *   - the Ulysses all-to-all that turns the sequence-parallel layout (each rank
 *     holds N/P tokens, all H heads) into the head-parallel layout (each rank
 *     holds all N tokens, H/P heads) -- Section II-A -- written as its three
 *     literal steps: build the send chunks, exchange them, lay the received
 *     chunks out head-major;
 *   - the V-Major active-projection selection of Section III-D in the
 *     threshold-per-tile form this build measures: a tile of `T` consecutive
 *     tokens is active when any element of the current value vectors differs
 *     from the cached one by more than tau; active tiles are listed in
 *     ascending order and their current values are gathered densely.
 *
 * All data are 16-bit patterns (bf16) copied without interpretation, except
 * the selection's comparison, which widens both bf16 values and the fp32
 * threshold to double exactly and takes the decision on the double difference
 * (exact whenever the two exponents are less than 45 binary orders apart).
 *
 * Outer loops carry an OpenMP pragma; nothing is blocked, fused or reordered.
 */
#include <stdint.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the OpenMP loops below run on (for the benchmark's report of the CPU baseline). */
int oracle_omp_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

#define SLOT_SEND_MAJOR 0
#define SLOT_RECV_MAJOR 1

static inline int64_t slot_of(int r, int p, int P, int slot_order) {
    /* chunk(r -> p): in rank r's send buffer (SEND_MAJOR) or rank p's receive buffer (RECV_MAJOR) */
    return slot_order == SLOT_SEND_MAJOR ? (int64_t)r * P + p : (int64_t)p * P + r;
}

/* chunk(r->p)[n][hl][i] = X[r*Ns + n][p*Hp + hl][i], for source ranks r in the range */
void oracle_a2a_pack(const uint16_t* x, uint16_t* xbuf, int N, int H, int d, int P,
                     int rank_begin, int rank_count, int slot_order) {
    const int Ns = N / P, Hp = H / P;
    const int64_t chunk = (int64_t)Ns * Hp * d;
#pragma omp parallel for schedule(static)
    for (int r = rank_begin; r < rank_begin + rank_count; ++r)
        for (int p = 0; p < P; ++p) {
            uint16_t* c = xbuf + slot_of(r, p, P, slot_order) * chunk;
            for (int n = 0; n < Ns; ++n)
                for (int hl = 0; hl < Hp; ++hl)
                    for (int i = 0; i < d; ++i)
                        c[((int64_t)n * Hp + hl) * d + i] =
                            x[((int64_t)(r * Ns + n) * H + (p * Hp + hl)) * d + i];
        }
}

/* The exchange itself: what rank r sent to p becomes the r-th block rank p received. */
void oracle_a2a_exchange(const uint16_t* send_major, uint16_t* recv_major, int N, int H, int d, int P) {
    const int64_t chunk = (int64_t)(N / P) * (H / P) * d;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < P; ++r)
        for (int p = 0; p < P; ++p)
            memcpy(recv_major + ((int64_t)p * P + r) * chunk,
                   send_major + ((int64_t)r * P + p) * chunk, (size_t)chunk * sizeof(uint16_t));
}

/* Y[p*Hp + hl][r*Ns + n][i] = chunk(r->p)[n][hl][i], for destination ranks p in the range */
void oracle_a2a_unpack(const uint16_t* xbuf, uint16_t* y, int N, int H, int d, int P,
                       int rank_begin, int rank_count, int slot_order) {
    const int Ns = N / P, Hp = H / P;
    const int64_t chunk = (int64_t)Ns * Hp * d;
#pragma omp parallel for schedule(static)
    for (int p = rank_begin; p < rank_begin + rank_count; ++p)
        for (int r = 0; r < P; ++r) {
            const uint16_t* c = xbuf + slot_of(r, p, P, slot_order) * chunk;
            for (int n = 0; n < Ns; ++n)
                for (int hl = 0; hl < Hp; ++hl)
                    for (int i = 0; i < d; ++i)
                        y[((int64_t)(p * Hp + hl) * N + (r * Ns + n)) * d + i] =
                            c[((int64_t)n * Hp + hl) * d + i];
        }
}

static inline double bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * cur, prev: [S][N][W].  Tile t = tokens [t*T, (t+1)*T) of every slab s.
 * flag[t] = 1 iff some element has NOT(|double(cur) - double(prev)| <= double(tau))   (so NaN counts as changed).
 * idx: ascending active tile ids; compact[s][j*T + (n - t*T)][w] = cur[s][n][w] for the j-th
 * active tile t, for j < cap_tiles; the compact buffer is [S][cap_tiles*T][W].
 * Returns the number of active tiles (also beyond cap_tiles).
 */
int oracle_vmajor_select(int S, int N, int W, int T, const uint16_t* cur, const uint16_t* prev,
                         float tau, int32_t* flags, int32_t* idx, uint16_t* compact, int cap_tiles) {
    const int NT = N / T;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < NT; ++t) {
        int active = 0;
        for (int s = 0; s < S; ++s)
            for (int n = t * T; n < (t + 1) * T; ++n)
                for (int w = 0; w < W; ++w) {
                    const int64_t e = ((int64_t)s * N + n) * W + w;
                    const double diff = fabs(bf16_to_f64(cur[e]) - bf16_to_f64(prev[e]));
                    if (!(diff <= (double)tau)) active = 1;
                }
        flags[t] = active;
    }
    int n_active = 0;
    for (int t = 0; t < NT; ++t) {
        if (!flags[t]) continue;
        const int j = n_active++;
        idx[j] = t;
        if (compact && j < cap_tiles)
            for (int s = 0; s < S; ++s)
                for (int n = 0; n < T; ++n)
                    for (int w = 0; w < W; ++w)
                        compact[((int64_t)s * cap_tiles * T + (int64_t)j * T + n) * W + w] =
                            cur[((int64_t)s * N + (int64_t)t * T + n) * W + w];
    }
    return n_active;
}

/*
 * V-Major, sender side (Section III-D: Q and K send only their active part): gather the tiles listed
 * in idx[0..n_active) of x [S][N][W] into compact [S][cap_tiles*T][W], tile j of the list at rows j*T .. ;
 * tiles beyond cap_tiles are not gathered.
 */
void oracle_vmajor_gather(int S, int N, int W, int T, const uint16_t* x, const int32_t* idx, int n_active,
                          uint16_t* compact, int cap_tiles) {
    for (int j = 0; j < n_active && j < cap_tiles; ++j)
        for (int s = 0; s < S; ++s)
            for (int m = 0; m < T; ++m)
                for (int w = 0; w < W; ++w)
                    compact[((int64_t)s * cap_tiles * T + (int64_t)j * T + m) * W + w] =
                        x[((int64_t)s * N + (int64_t)idx[j] * T + m) * W + w];
}

/*
 * V-Major, receiver side (Section III-D: the receiver rebuilds the step's tensor from its cache): overwrite the
 * tiles listed in idx of the cached tensor [S][N][W] with the received active tiles; every other tile keeps
 * its cached value.
 */
void oracle_vmajor_scatter(int S, int N, int W, int T, const uint16_t* compact, const int32_t* idx, int n_active,
                           uint16_t* cache, int cap_tiles) {
    for (int j = 0; j < n_active && j < cap_tiles; ++j)
        for (int s = 0; s < S; ++s)
            for (int m = 0; m < T; ++m)
                for (int w = 0; w < W; ++w)
                    cache[((int64_t)s * N + (int64_t)idx[j] * T + m) * W + w] =
                        compact[((int64_t)s * cap_tiles * T + (int64_t)j * T + m) * W + w];
}

/*
 * Second Ulysses all-to-all (Section II-A: after attention, head-parallel layout back to sequence-parallel
 * layout), as its steps.  Rank p holds y [Hp][N][d] for its heads; the chunk it sends to rank r carries the
 * tokens r owns: chunk(p->r)[n][hl][i] = y[p*Hp + hl][r*Ns + n][i].
 * Slot of chunk(p->r): SEND_MAJOR p*P + r (sender p's buffer), RECV_MAJOR r*P + p (receiver r's buffer).
 */
void oracle_a2a_pack_hs(const uint16_t* y_hs, uint16_t* xbuf, int N, int H, int d, int P,
                        int rank_begin, int rank_count, int slot_order) {
    const int Ns = N / P, Hp = H / P;
    const int64_t chunk = (int64_t)Ns * Hp * d;
#pragma omp parallel for schedule(static)
    for (int p = rank_begin; p < rank_begin + rank_count; ++p)      /* source ranks: head owners */
        for (int r = 0; r < P; ++r) {
            uint16_t* c = xbuf + slot_of(p, r, P, slot_order) * chunk;
            for (int n = 0; n < Ns; ++n)
                for (int hl = 0; hl < Hp; ++hl)
                    for (int i = 0; i < d; ++i)
                        c[((int64_t)n * Hp + hl) * d + i] =
                            y_hs[((int64_t)(p * Hp + hl) * N + (r * Ns + n)) * d + i];
        }
}

/* x_seq[r*Ns + n][p*Hp + hl][i] = chunk(p->r)[n][hl][i], for destination ranks r (token owners) in the range */
void oracle_a2a_unpack_seq(const uint16_t* xbuf, uint16_t* x_seq, int N, int H, int d, int P,
                           int rank_begin, int rank_count, int slot_order) {
    const int Ns = N / P, Hp = H / P;
    const int64_t chunk = (int64_t)Ns * Hp * d;
#pragma omp parallel for schedule(static)
    for (int r = rank_begin; r < rank_begin + rank_count; ++r)
        for (int p = 0; p < P; ++p) {
            const uint16_t* c = xbuf + slot_of(p, r, P, slot_order) * chunk;
            for (int n = 0; n < Ns; ++n)
                for (int hl = 0; hl < Hp; ++hl)
                    for (int i = 0; i < d; ++i)
                        x_seq[((int64_t)(r * Ns + n) * H + (p * Hp + hl)) * d + i] =
                            c[((int64_t)n * Hp + hl) * d + i];
        }
}
