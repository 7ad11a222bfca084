/*
 * CPU oracle for the plaintext-ciphertext matrix multiplication (PCMM).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests, the smoke check and the benchmark's cpu_baseline
 * leg have an independent, slow, obviously correct result to compare with.
 * It shares no code, header, table or constant with the HIP library.
 *
 * What it computes.  The paper's PCMM step is B = W.A with W a plaintext
 * weight matrix and A the (encrypted) activations (Section 5.1), reduced to
 * a clear matrix product on ciphertext data (Section 2.2, "PCMM from BLAS").
 * A ciphertext is a pair (a, b) in R_Q^2 and addition acts component-wise
 * (Appendix A, Enc/Dec/Add), so an integer combination of ciphertext rows is
 * taken coefficient by coefficient on both components.  With Q held in RNS
 * form, one limb is
 *
 *     C_j[m][n] = ( sum_{k<K} W[m][k] * A_j[k][n] )  mod q_j ,  in [0, q_j),
 *
 * W[m][k] a signed integer, A_j[k][n] in [0, q_j).  This file is that
 * definition written out: a schoolbook multiply-accumulate in __int128 (no
 * intermediate reduction is needed: |W| < 2^31, A < 2^63, K < 2^31 gives
 * |sum| < 2^125) followed by one `%` per output.  No digits, no Barrett, no
 * blocking beyond keeping one output row of accumulators at a time.
 *
 * Parity status: pinned by tests/test_oracle_*.py against Python big-integer
 * brute force, closed forms, linearity, CRT consistency, the block identity
 * of Section 5.1 and a toy CKKS encrypt -> PCMM -> decrypt round trip.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef __int128 i128;
typedef unsigned __int128 u128;

/* canonical representative of a signed 128-bit value modulo q */
static uint64_t canon_mod(i128 v, uint64_t q)
{
    i128 r = v % (i128)q;
    if (r < 0) r += (i128)q;
    return (uint64_t)r;
}

int pcmm_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Selected rows and columns of every limb of C.
 *   W      [M][K]          int32, row-major (signed plaintext integers)
 *   A      [L][K][Ncols]   uint64 residues, A[j] reduced mod primes[j]
 *   rows   [nrows]         row indices into 0..M-1
 *   cols   [ncols]         column indices into 0..Ncols-1
 *   C      [L][nrows][ncols] uint64, written
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int pcmm_oracle_select(const int32_t *W, const uint64_t *A, const uint64_t *primes,
                       int64_t M, int64_t K, int64_t Ncols, int64_t L,
                       const int64_t *rows, int64_t nrows,
                       const int64_t *cols, int64_t ncols, uint64_t *C)
{
    if (!W || !A || !primes || !C || !rows || !cols) return -1;
    if (M <= 0 || K <= 0 || Ncols <= 0 || L <= 0 || nrows < 0 || ncols < 0) return -1;
    for (int64_t i = 0; i < nrows; ++i) if (rows[i] < 0 || rows[i] >= M) return -1;
    for (int64_t i = 0; i < ncols; ++i) if (cols[i] < 0 || cols[i] >= Ncols) return -1;
    int fail = 0;
#pragma omp parallel
    {
        i128 *acc = (i128 *)malloc((size_t)(ncols > 0 ? ncols : 1) * sizeof(i128));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t j = 0; j < L; ++j) {
            for (int64_t r = 0; r < nrows; ++r) {
                if (!acc) continue;
                const uint64_t q = primes[j];
                const int32_t *w = W + rows[r] * K;
                const uint64_t *Aj = A + (size_t)j * K * Ncols;
                for (int64_t c = 0; c < ncols; ++c) acc[c] = 0;
                for (int64_t k = 0; k < K; ++k) {
                    const i128 wk = w[k];
                    const uint64_t *a = Aj + (size_t)k * Ncols;
                    for (int64_t c = 0; c < ncols; ++c)
                        acc[c] += wk * (i128)a[cols[c]];
                }
                uint64_t *out = C + ((size_t)j * nrows + r) * ncols;
                for (int64_t c = 0; c < ncols; ++c) out[c] = canon_mod(acc[c], q);
            }
        }
        free(acc);
    }
    return fail ? -1 : 0;
}

/* All of C: [L][M][Ncols]. */
int pcmm_oracle(const int32_t *W, const uint64_t *A, const uint64_t *primes,
                int64_t M, int64_t K, int64_t Ncols, int64_t L, uint64_t *C)
{
    if (M <= 0 || Ncols <= 0) return -1;
    int64_t *rows = (int64_t *)malloc((size_t)M * sizeof(int64_t));
    int64_t *cols = (int64_t *)malloc((size_t)Ncols * sizeof(int64_t));
    if (!rows || !cols) { free(rows); free(cols); return -1; }
    for (int64_t i = 0; i < M; ++i) rows[i] = i;
    for (int64_t i = 0; i < Ncols; ++i) cols[i] = i;
    int rc = pcmm_oracle_select(W, A, primes, M, K, Ncols, L, rows, M, cols, Ncols, C);
    free(rows);
    free(cols);
    return rc;
}

/*
 * Freivalds-style check of one whole limb of a claimed result, for sizes at
 * which the full oracle is too slow.  If C_j = W.A_j (mod q) then for any
 * vector r:  C_j.r = W.(A_j.r) (mod q).  A wrong row of C_j passes with
 * probability at most 1/q over a uniform r (q prime).  Everything is again
 * plain __int128 arithmetic with `%`.
 *   r [Ncols] uint64 in [0,q).  A_j, C_j are one limb each.
 * Returns the number of rows m whose two sides differ, plus the number of
 * entries of C_j that are not in [0,q) (0 = pass), or -1 on bad arguments.
 */
int64_t pcmm_freivalds(const int32_t *W, const uint64_t *Aj, const uint64_t *Cj,
                       const uint64_t *r, uint64_t q,
                       int64_t M, int64_t K, int64_t Ncols)
{
    if (!W || !Aj || !Cj || !r || q < 2 || M <= 0 || K <= 0 || Ncols <= 0) return -1;
    uint64_t *y = (uint64_t *)malloc((size_t)K * sizeof(uint64_t));
    if (!y) return -1;
    int64_t bad = 0;
    /* y = A_j . r  mod q   (entries < 2^63 each, Ncols < 2^31: the sum of products fits u128 only
       if reduced now and then; reduce every product instead, which is the plain way) */
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k) {
        const uint64_t *a = Aj + (size_t)k * Ncols;
        u128 s = 0;
        for (int64_t n = 0; n < Ncols; ++n) s += ((u128)a[n] * r[n]) % q;
        y[k] = (uint64_t)(s % q);
    }
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int64_t m = 0; m < M; ++m) {
        const int32_t *w = W + (size_t)m * K;
        const uint64_t *c = Cj + (size_t)m * Ncols;
        i128 z = 0;
        for (int64_t k = 0; k < K; ++k) z += ((i128)w[k] * (i128)y[k]) % (i128)q;
        u128 x = 0;
        for (int64_t n = 0; n < Ncols; ++n) {
            if (c[n] >= q) ++bad;
            x += ((u128)c[n] * r[n]) % q;
        }
        if ((uint64_t)(x % q) != canon_mod(z, q)) ++bad;
    }
    free(y);
    return bad;
}
