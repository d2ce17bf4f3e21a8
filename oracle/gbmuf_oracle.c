/*
 * gbmuf_oracle.c -- plain CPU oracle for the random-gossip BMUF synchronisation step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what
 * the synchronisation branch of Algorithm 1 ("gossip-MA (gossip-BMUF) for node k") of
 * "A Random Gossip BMUF Process for Neural Language Modeling" computes.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may build, load or call it.  It
 * shares no source, header, table or helper with the HIP library.
 *
 * What is written out here, and the passage each part follows:
 *   - ring candidates of a worker ......... Definition 1 (k-symmetric ring topology)
 *   - the random pick of q neighbours ..... Algorithm 1, sync branch, first statement;
 *                                           Section 2.2 last paragraph (fresh, independent
 *                                           choice per component and per sync); q may differ
 *                                           from component to component (Algorithm 1's
 *                                           REQUIRE lines only bound it by 2p)
 *   - neighbour average ................... Algorithm 1, the averaging statement
 *   - G, Delta, omega, theta updates ...... Algorithm 1, the four gossip-BMUF statements
 *   - gossip-MA branch .................... Algorithm 1, the gossip-MA statement
 *   - final model average ................. Algorithm 1, the RETURN statement
 *
 * The paper does not say HOW the random choice is made, nor in which order or precision
 * the sums are formed.  The readings taken (also listed in the design notes) are:
 *   * the q neighbours are drawn uniformly WITHOUT replacement from the worker's ring
 *     candidates (required so that q = 2p yields all of them, Section 2.2);
 *   * mechanism: a partial Fisher-Yates shuffle of the candidate list driven by the
 *     Philox-4x32-10 counter-based generator (Salmon et al., SC'11) with
 *         key     = (seed low 32, seed high 32)
 *         counter = (round low 32, round high 32, component, worker + 65536 * block)
 *     draw j uses 32-bit word (j mod 4) of block (j div 4); the index is
 *     j + floor(u * (C - j) / 2^32); the chosen ids are then sorted ascending;
 *   * the average uses every worker's PRE-sync theta (snapshot semantics);
 *   * the sum runs over the worker itself and its neighbours in ascending worker id;
 *   * 1/(q+1) is one rounded constant that the sum is multiplied by;
 *   * every *, + and - is rounded on its own (no fused multiply-add);
 *   * theta_{t-H}, the model the block started from, is what the restart statement wrote
 *     at the previous sync: omega + eta*Delta (mode 1, the paper's form).  Mode 0 is
 *     classical block momentum (no restart: theta' = omega', base = omega).  Mode 2 is
 *     the literal "G = avg - omega" with the restart kept.  Mode 3 is gossip-MA.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors of the Random123
 * distribution; hand-enumerated ring candidates; sampler properties (distinct, inside
 * the candidate set, q = C returns all, uniformity); brute-force dense row-stochastic
 * matrices over every neighbour assignment on K <= 4; reduction to textbook BMUF-NBM
 * and to model averaging; fixed point; the zeta = 1 closed form.
 * The fp32 rounding ORDER (ascending-id sum, product-then-add) is fixed only by this
 * text: that detail is "parity unpinned" beyond the fp64 bound the tests place on it.
 *
 * Build:  gcc -std=c99 -O2 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_OK = 0, ORACLE_EINVAL = 1, ORACLE_ENOMEM = 2 };

/* ------------------------------------------------------------------------------------ */
/* Philox-4x32-10, as published (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:   */
/* as easy as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplies, with the key     */
/* bumped by the Weyl constants between rounds.                                          */
/* ------------------------------------------------------------------------------------ */
void gbmuf_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Section 3.3 gives the rule of thumb p = log2(n) - 1 for the ring degree; at least 1. */
int32_t gbmuf_oracle_default_p(int32_t K)
{
    int32_t lg = 0;
    while ((1 << (lg + 1)) <= K) ++lg;          /* floor(log2 K) */
    return lg - 1 < 1 ? 1 : lg - 1;
}

/* Definition 1: node w is connected to (w-1)%K ... (w-p)%K, (w+1)%K ... (w+p)%K, in that
 * order; % is the non-negative modulus.  A node is not its own neighbour and a node that
 * the listing reaches twice (2p >= K) is listed once, at its first position.
 * Writes the candidates to cand[] (room for K entries) and returns their number C. */
int32_t gbmuf_oracle_ring_candidates(int32_t w, int32_t K, int32_t p, int32_t *cand)
{
    int32_t C = 0;
    for (int side = 0; side < 2; ++side) {
        for (int32_t d = 1; d <= p; ++d) {
            int64_t raw = side == 0 ? (int64_t)w - d : (int64_t)w + d;
            int32_t v = (int32_t)(((raw % K) + K) % K);
            int seen = (v == w);
            for (int32_t j = 0; j < C; ++j) seen |= (cand[j] == v);
            if (!seen) cand[C++] = v;
        }
    }
    return C;
}

/* Algorithm 1, sync branch, first statement: the random pick of q neighbours k_1..k_q for
 * worker w and component i in sync number `round`.  out[0..q) ascending.  Returns ORACLE_EINVAL if q exceeds the
 * number of candidates (the paper requires q <= 2p). */
int gbmuf_oracle_sample(int32_t K, int32_t p, int32_t q, uint64_t seed, uint64_t round,
                        int32_t w, int32_t i, int32_t *out)
{
    if (K < 1 || p < 0 || q < 0 || w < 0 || w >= K || i < 0 || K > 65535) return ORACLE_EINVAL;
    int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)(K > 0 ? K : 1));
    if (!cand) return ORACLE_ENOMEM;
    int32_t C = gbmuf_oracle_ring_candidates(w, K, p, cand);
    if (q > C) { free(cand); return ORACLE_EINVAL; }

    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t u[4] = { 0, 0, 0, 0 };
    for (int32_t j = 0; j < q; ++j) {
        if (j % 4 == 0) {
            uint32_t ctr[4] = { (uint32_t)round, (uint32_t)(round >> 32), (uint32_t)i,
                                (uint32_t)w + 65536u * (uint32_t)(j / 4) };
            gbmuf_oracle_philox4x32_10(ctr, key, u);
        }
        /* uniform index in [j, C): j + floor(u * (C-j) / 2^32) */
        int32_t r = j + (int32_t)(((uint64_t)u[j % 4] * (uint64_t)(uint32_t)(C - j)) >> 32);
        int32_t tmp = cand[j]; cand[j] = cand[r]; cand[r] = tmp;
    }
    /* ascending order (insertion sort of the q chosen ids) */
    for (int32_t a = 1; a < q; ++a) {
        int32_t v = cand[a], b = a - 1;
        while (b >= 0 && cand[b] > v) { cand[b + 1] = cand[b]; --b; }
        cand[b + 1] = v;
    }
    for (int32_t j = 0; j < q; ++j) out[j] = cand[j];
    free(cand);
    return ORACLE_OK;
}

/* The whole table of one sync: nbr[i][w][0..q), i < m, w < K. */
int gbmuf_oracle_neighbour_table(int32_t m, int32_t K, int32_t p, int32_t q, uint64_t seed,
                                 uint64_t round, int32_t *nbr)
{
    if (m < 0) return ORACLE_EINVAL;
    for (int32_t i = 0; i < m; ++i)
        for (int32_t w = 0; w < K; ++w) {
            int rc = gbmuf_oracle_sample(K, p, q, seed, round, w, i,
                                         nbr + ((size_t)i * (size_t)K + (size_t)w) * (size_t)q);
            if (rc != ORACLE_OK) return rc;
        }
    return ORACLE_OK;
}

/* The same table when component i draws its own number q[i] of neighbours (Algorithm 1 only
 * requires q <= 2p; Section 3.3 picks (p, q) per deployment).  Rows have `width` >= max q[i]
 * entries: nbr[i][w][0..q[i]) are the chosen ids, ascending; the rest of the row is -1. */
int gbmuf_oracle_neighbour_table_q(int32_t m, int32_t K, int32_t p, const int32_t *q,
                                   int32_t width, uint64_t seed, uint64_t round, int32_t *nbr)
{
    if (m < 0 || width < 0 || (m > 0 && !q)) return ORACLE_EINVAL;
    for (int32_t i = 0; i < m; ++i)
        if (q[i] < 0 || q[i] > width) return ORACLE_EINVAL;
    for (int32_t i = 0; i < m; ++i)
        for (int32_t w = 0; w < K; ++w) {
            int32_t *row = nbr + ((size_t)i * (size_t)K + (size_t)w) * (size_t)width;
            int rc = gbmuf_oracle_sample(K, p, q[i], seed, round, w, i, row);
            if (rc != ORACLE_OK) return rc;
            for (int32_t j = q[i]; j < width; ++j) row[j] = -1;
        }
    return ORACLE_OK;
}

/* Common argument check of the sync functions below. */
static int check_sync_args(const int64_t *off, int32_t m, int32_t K, const int32_t *q,
                           int32_t width, const int32_t *nbr, const void *theta, int64_t stride)
{
    if (!off || !theta || m < 0 || K < 1 || width < 0 || (m > 0 && !q)) return ORACLE_EINVAL;
    if (off[0] != 0) return ORACLE_EINVAL;
    for (int32_t i = 0; i < m; ++i) if (off[i + 1] < off[i]) return ORACLE_EINVAL;
    if (stride < off[m]) return ORACLE_EINVAL;
    for (int32_t i = 0; i < m; ++i) {
        if (q[i] < 0 || q[i] > K - 1 || q[i] > width) return ORACLE_EINVAL;
        if (q[i] > 0 && !nbr) return ORACLE_EINVAL;
        for (int32_t w = 0; w < K; ++w)
            for (int32_t j = 0; j < q[i]; ++j) {
                int32_t v = nbr[((size_t)i * (size_t)K + (size_t)w) * (size_t)width + (size_t)j];
                if (v < 0 || v >= K) return ORACLE_EINVAL;
            }
    }
    return ORACLE_OK;
}

/* q[0..m) = one value for every component. */
static int32_t *uniform_q(int32_t m, int32_t q)
{
    int32_t *qv = (int32_t *)malloc(sizeof(int32_t) * (size_t)(m > 0 ? m : 1));
    for (int32_t i = 0; qv && i < m; ++i) qv[i] = q;
    return qv;
}

/* ids[0..q] = the worker itself and its q neighbours, ascending worker id. */
static void merge_self(int32_t w, const int32_t *row, int32_t q, int32_t *ids)
{
    ids[0] = w;
    for (int32_t j = 0; j < q; ++j) {
        int32_t v = row[j], b = j;
        while (b >= 0 && ids[b] > v) { ids[b + 1] = ids[b]; --b; }
        ids[b + 1] = v;
    }
}

/* The update statements, once in fp32 (every operation rounded to float, the gate the HIP
 * path is compared with) and once in fp64 (the error bound and the algebraic checks). */
#define REAL float
#define NAME(x) x##_f32
#include "gbmuf_oracle_update.inc"
#undef REAL
#undef NAME

#define REAL double
#define NAME(x) x##_f64
#include "gbmuf_oracle_update.inc"
#undef REAL
#undef NAME

/* Number of threads the element loops use (1 when built without OpenMP). */
int gbmuf_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
