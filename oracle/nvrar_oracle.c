/*
 * CPU oracle for the hierarchical recursive-doubling all-reduce (NVRAR, Algorithm 1 and
 * Section 4.1 of the paper).  TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the
 * benchmark's cpu_baseline leg call it; the product path (the HIP library) never does, and
 * the two share no code.
 *
 * Plain, slow and meant to be checked against the paper by eye.  All P = G*N ranks live in
 * one process as P arrays.  Every rank keeps its own message M, its own reduce-scatter
 * result M' and its own per-step send buffers B_send[0..L] (Section 4.2.1: one buffer per
 * inter-node step), and every phase is a loop over ranks, each rank doing what Algorithm 1
 * makes that rank do:
 *
 *   phase 1 (Section 4.1, reduce-scatter):  rank (r_n, r_g) ends with chunk r_g of the sum
 *            over the G ranks of node r_n;
 *   phase 2 (Algorithm 1, function RD_inter): for l = 0 .. log2(N)-1 the rank takes the
 *            buffer of peer (r_n XOR 2^l, r_g) ("dst", what the put delivered) and its own
 *            ("src") and forms B_send[l+1] = dst + src;
 *   phase 3 (Section 4.1, all-gather):  every rank of node r_n receives chunk r_g from rank
 *            (r_n, r_g), for all r_g.
 *
 * Arithmetic (the paper fixes the data type, bf16 models, but not the order; these are the
 * readings this build takes):
 *   - values are widened to IEEE binary32 (exact for bf16), added in binary32 with
 *     round-to-nearest-even and gradual underflow;
 *   - the reduce-scatter accumulates local ranks 0, 1, .., G-1 in that order in binary32 and
 *     narrows once to the message type;
 *   - every inter-node step narrows its result to the message type (the per-step message is
 *     |M|/G bytes, so the buffers hold the message type);
 *   - narrowing to bf16 is round-to-nearest, ties to even; overflow gives +-Inf.
 *   - NaN: only "is NaN" is meaningful; payload and sign of a NaN result are not pinned.
 *
 * N that is not a power of two is outside the paper; see the comment at sits_out() below for
 * the extension taken.
 *
 * The chunk partition (needed when G does not divide n): chunk length is ceil(n/G) rounded
 * up to a whole number of 16-byte groups; chunk c covers [min(c*len,n), min((c+1)*len,n)).
 * Results do not depend on the partition because every element is reduced independently.
 *
 * Pins: tests/test_oracle_pins.py (exact rational arithmetic on tiny cases, closed forms,
 * integer-valued inputs, identity at P = 1, a second formulation as a balanced tree).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#if defined(__SSE__)
#include <xmmintrin.h>
#endif
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ARG = -1,   /* NULL pointer, G < 1, N < 1, n == 0, unknown dtype */
    ORACLE_BAD_N = -2,     /* (unused since N may be any positive number) */
    ORACLE_NO_MEM = -3
};

/* ---- scalar helpers ---------------------------------------------------------------- */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, sizeof f); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, sizeof u); return u; }

/* bf16 is the upper half of binary32: widening is exact. */
static float widen_bf16(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/* binary32 -> bf16, round to nearest, ties to even.  The 16 dropped bits are compared with
 * one half (0x8000): above rounds away, below truncates, equal looks at the kept LSB.  A
 * carry out of the mantissa moves into the exponent, which is what rounding up to the next
 * binade (or to Inf) means.  NaN stays NaN (quiet bit forced so truncation cannot make Inf).
 */
static uint16_t narrow_bf16(float f) {
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t kept = u >> 16, dropped = u & 0xffffu;
    if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) kept += 1u;
    return (uint16_t)kept;
}

/* The SSE control register can carry flush-to-zero / denormals-are-zero set by some other
 * library in the process; the oracle's adds need gradual underflow, so clear both for the
 * calling thread while it works. */
static unsigned enter_ieee(void) {
#if defined(__SSE__)
    unsigned old = _mm_getcsr();
    _mm_setcsr(old & ~(0x8000u | 0x0040u));
    return old;
#else
    return 0;
#endif
}
static void leave_ieee(unsigned old) {
#if defined(__SSE__)
    _mm_setcsr(old);
#else
    (void)old;
#endif
}

static int floor_log2(int N) { /* largest L with 2^L <= N */
    int L = 0;
    while ((2 << L) <= N) ++L;
    return L;
}

/* N that is not a power of two.  Algorithm 1 assumes N = 2^L.  For N = 2^L + r (0 < r < 2^L)
 * this oracle takes the customary extension of recursive doubling (Thakur, Rabenseifner, Gropp,
 * "Optimization of collective communication operations in MPICH", 2005): the first 2r nodes pair
 * up as (2i, 2i+1); the even node hands its M' to the odd one and sits out; the 2^L nodes that
 * remain are renumbered (node 2i+1 -> i, node j >= 2r -> j - r) and run the L steps of
 * Algorithm 1 on those numbers; at the end each odd node hands the result back to its even
 * partner.  r = 0 gives Algorithm 1 unchanged. */
static int sits_out(int r_n, int r) { return r_n < 2 * r && (r_n % 2) == 0; }
static int folds_in(int r_n, int r) { return r_n < 2 * r && (r_n % 2) == 1; }
static int step_number(int r_n, int r) { return r_n < 2 * r ? r_n / 2 : r_n - r; }   /* node -> number in the steps */
static int node_of_number(int v, int r) { return v < r ? 2 * v + 1 : v + r; }

/* ---- chunk partition ------------------------------------------------------------------ */

static size_t elem_size(int dtype) { return dtype == ORACLE_BF16 ? 2 : 4; }

static size_t chunk_len(size_t n, int G, int dtype) {
    size_t per16 = 16 / elem_size(dtype);
    size_t len = (n + (size_t)G - 1) / (size_t)G;
    return (len + per16 - 1) / per16 * per16;
}
static size_t chunk_begin(size_t n, int G, int dtype, int c) {
    size_t b = (size_t)c * chunk_len(n, G, dtype);
    return b < n ? b : n;
}

/* ---- typed access ---------------------------------------------------------------------- */

static float load_elem(const void *buf, size_t i, int dtype) {
    return dtype == ORACLE_BF16 ? widen_bf16(((const uint16_t *)buf)[i]) : ((const float *)buf)[i];
}
static void store_elem(void *buf, size_t i, int dtype, float v) {
    if (dtype == ORACLE_BF16) ((uint16_t *)buf)[i] = narrow_bf16(v);
    else ((float *)buf)[i] = v;
}

/* ---- one rank's exchange-and-sum (the body of RD_inter's loops) ---------------------- */

/* dst[chunk*n + i] <- narrow( widen(dst[..]) + widen(src[..]) ), i in [0, n).
 * "dst" is what arrived from the peer, "src" the rank's own buffer, as in Algorithm 1;
 * IEEE addition commutes, so which is which does not change a non-NaN result. */
int nvrar_oracle_step_combine(void *dst, const void *src, size_t chunk, size_t n, int dtype) {
    if (!dst || !src || (dtype != ORACLE_BF16 && dtype != ORACLE_F32)) return ORACLE_BAD_ARG;
    unsigned csr = enter_ieee();
    for (size_t i = chunk * n; i < chunk * n + n; ++i) {
        float sum = load_elem(dst, i, dtype) + load_elem(src, i, dtype);
        store_elem(dst, i, dtype, sum);
    }
    leave_ieee(csr);
    return ORACLE_OK;
}

/* ---- the whole all-reduce ------------------------------------------------------------- */

/* in[p], out[p]: P = G*N host arrays of n elements; rank p = r_n*G + r_g.  out may alias in
 * rank by rank (in[p] == out[p]) since the inputs are fully consumed by phase 1 before
 * phase 3 writes.  threads <= 1 runs serially; otherwise the per-rank loops of each phase
 * are shared among that many OpenMP threads (a rank's work is never split, so no element's
 * order of operations changes). */
int nvrar_oracle_allreduce(const void *const *in, void *const *out, int G, int N, size_t n,
                           int dtype, int threads) {
    if (!in || !out || G < 1 || N < 1 || n == 0) return ORACLE_BAD_ARG;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return ORACLE_BAD_ARG;
    const int L = floor_log2(N);
    const int r = N - (1 << L);
    const int P = G * N;
    for (int p = 0; p < P; ++p) if (!in[p] || !out[p]) return ORACLE_BAD_ARG;
    if (threads < 1) threads = 1;

    const size_t es = elem_size(dtype);
    const size_t len = chunk_len(n, G, dtype);

    /* B_send[l][p]: rank p's buffer for step l, l = 0..L (one chunk each). */
    void **B_send = (void **)calloc((size_t)(L + 1) * (size_t)P, sizeof(void *));
    if (!B_send) return ORACLE_NO_MEM;
    int ok = 1;
    for (size_t k = 0; k < (size_t)(L + 1) * (size_t)P; ++k) {
        B_send[k] = calloc(len, es);
        if (!B_send[k]) ok = 0;
    }
    if (!ok) {
        for (size_t k = 0; k < (size_t)(L + 1) * (size_t)P; ++k) free(B_send[k]);
        free(B_send);
        return ORACLE_NO_MEM;
    }

    /* Phase 1: intra-node reduce-scatter.  M' of rank (r_n, r_g) = chunk r_g summed over the
     * node's G ranks, local rank 0 first; it becomes B_send[0]. */
    #pragma omp parallel for num_threads(threads) schedule(static)
    for (int p = 0; p < P; ++p) {
        unsigned csr = enter_ieee();
        const int r_n = p / G, r_g = p % G;
        const size_t lo = chunk_begin(n, G, dtype, r_g), hi = chunk_begin(n, G, dtype, r_g + 1);
        void *Mprime = B_send[0 * P + p];
        for (size_t j = lo; j < hi; ++j) {
            float acc = load_elem(in[r_n * G + 0], j, dtype);
            for (int g = 1; g < G; ++g) acc = acc + load_elem(in[r_n * G + g], j, dtype);
            store_elem(Mprime, j - lo, dtype, acc);
        }
        leave_ieee(csr);
    }

    /* Phase 2, before the steps (only if N is not a power of two): an odd node among the first
     * 2r adds what its even partner hands over to its own M'. */
    #pragma omp parallel for num_threads(threads) schedule(static)
    for (int p = 0; p < P; ++p) {
        const int r_n = p / G, r_g = p % G;
        if (!folds_in(r_n, r)) continue;
        unsigned csr = enter_ieee();
        void *own = B_send[0 * P + p];
        const void *handed = B_send[0 * P + (r_n - 1) * G + r_g];
        const size_t cnt = chunk_begin(n, G, dtype, r_g + 1) - chunk_begin(n, G, dtype, r_g);
        for (size_t i = 0; i < cnt; ++i) {
            float sum = load_elem(handed, i, dtype) + load_elem(own, i, dtype);
            store_elem(own, i, dtype, sum);
        }
        leave_ieee(csr);
    }

    /* Phase 2: inter-node recursive doubling among ranks with equal r_g. */
    for (int l = 0; l < L; ++l) {
        #pragma omp parallel for num_threads(threads) schedule(static)
        for (int p = 0; p < P; ++p) {
            const int r_n = p / G, r_g = p % G;
            if (sits_out(r_n, r)) continue;
            unsigned csr = enter_ieee();
            const int peer = node_of_number(step_number(r_n, r) ^ (1 << l), r) * G + r_g;
            const void *src = B_send[l * P + p];      /* own data for this step          */
            const void *dst = B_send[l * P + peer];   /* what the peer's put delivers     */
            void *next = B_send[(l + 1) * P + p];
            const size_t cnt = chunk_begin(n, G, dtype, r_g + 1) - chunk_begin(n, G, dtype, r_g);
            for (size_t i = 0; i < cnt; ++i) {
                float sum = load_elem(dst, i, dtype) + load_elem(src, i, dtype);
                store_elem(next, i, dtype, sum);
            }
            leave_ieee(csr);
        }
    }

    /* Phase 2, after the steps: the result goes back to the nodes that sat out. */
    #pragma omp parallel for num_threads(threads) schedule(static)
    for (int p = 0; p < P; ++p) {
        const int r_n = p / G, r_g = p % G;
        if (!sits_out(r_n, r)) continue;
        const size_t cnt = chunk_begin(n, G, dtype, r_g + 1) - chunk_begin(n, G, dtype, r_g);
        memcpy(B_send[L * P + p], B_send[L * P + (r_n + 1) * G + r_g], cnt * es);
    }

    /* Phase 3: intra-node all-gather.  Rank (r_n, r_g) hands its reduced chunk to every rank
     * of its node (itself included). */
    #pragma omp parallel for num_threads(threads) schedule(static)
    for (int p = 0; p < P; ++p) {
        const int r_n = p / G, r_g = p % G;
        const size_t lo = chunk_begin(n, G, dtype, r_g), hi = chunk_begin(n, G, dtype, r_g + 1);
        const char *Mprime = (const char *)B_send[L * P + p];
        for (int g = 0; g < G; ++g)
            memcpy((char *)out[r_n * G + g] + lo * es, Mprime, (hi - lo) * es);
    }

    for (size_t k = 0; k < (size_t)(L + 1) * (size_t)P; ++k) free(B_send[k]);
    free(B_send);
    return ORACLE_OK;
}

/* Number of OpenMP threads a call with threads = t would really get (for the report). */
int nvrar_oracle_threads_used(int t) {
    int got = 1;
    if (t < 1) t = 1;
    #pragma omp parallel num_threads(t)
    {
        #pragma omp master
        {
#ifdef _OPENMP
            got = omp_get_num_threads();
#endif
        }
    }
    return got;
}
