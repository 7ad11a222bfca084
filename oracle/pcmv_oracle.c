/*
 * CPU oracle for the ring products underneath the decode-time plaintext-ciphertext matrix-vector
 * multiplication (PCMv).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file.  It shares no code,
 * header, table or constant with the HIP library.
 *
 * What the paper fixes.  In the decoding stage the matrix-matrix products of the linear layers become
 * matrix-vector products (Section 3.2, last paragraph), evaluated at ring degree 4096 in coefficient
 * encoding with the plaintexts (the converted weights) kept as polynomials in the NTT domain
 * (Table "he-operators", row PCMv; Section 5.3 and Table "model-conversion-memory").  A ciphertext is a
 * pair (a, b) in R_Q^2, R = Z[X]/(X^N + 1), and a plaintext polynomial multiplies both components
 * (Appendix A: PCMult; Dec is linear).  The packing rule that says which weights go into which
 * plaintext polynomial, and the extraction and repacking of the useful coefficients afterwards, belong
 * to the algorithm the paper adopts by reference and are not restated in it.
 *
 * Reading taken here (listed among the readings of the design notes): the part built is the ring
 * arithmetic itself.  For plaintext polynomials pt[m][k] (m < Mp output polynomials, k < Kp input
 * ciphertexts) and ciphertexts ct[k] = (a_k, b_k), for every RNS limb j:
 *
 *     out_j[m][c] = sum_{k<Kp} pt[m][k] * ct_j[k][c]     in  Z_{q_j}[X] / (X^N + 1),   c in {a, b},
 *
 * coefficients in [0, q_j).  This file is that definition written out: the schoolbook negacyclic
 * convolution (X^N = -1 turns the wrapped terms negative), accumulated in __int128
 * (|pt| < 2^31, ct < 2^63, Kp N < 2^30 gives |sum| < 2^124), one `%` per output coefficient.  No NTT.
 *
 * Parity status: pinned by tests/test_pcmv_oracle.py (a hand-worked degree-4 product with its wrap,
 * numpy's linear convolution folded by hand, monomial shifts, bilinearity, the matrix-vector meaning of
 * coefficient 0, and decryption of the products in the toy CKKS).
 */
#include <stdint.h>
#include <stdlib.h>

typedef __int128 i128;

static uint64_t canon_mod(i128 v, uint64_t q)
{
    i128 r = v % (i128)q;
    if (r < 0) r += (i128)q;
    return (uint64_t)r;
}

/*
 * Selected output polynomials.
 *   pt     [Mp][Kp][N]       int64, signed plaintext coefficients (coefficient domain)
 *   ct     [L][Kp][2][N]     uint64 residues, limb j reduced mod primes[j]; [..][0] = a, [..][1] = b
 *   rows   [nrows]           indices m into 0..Mp-1
 *   out    [L][nrows][2][N]  uint64, written
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int pcmv_oracle_select(const int64_t *pt, const uint64_t *ct, const uint64_t *primes,
                       int64_t Mp, int64_t Kp, int64_t N, int64_t L,
                       const int64_t *rows, int64_t nrows, uint64_t *out)
{
    if (!pt || !ct || !primes || !rows || !out) return -1;
    if (Mp <= 0 || Kp <= 0 || N <= 0 || L <= 0 || nrows < 0) return -1;
    for (int64_t i = 0; i < nrows; ++i) if (rows[i] < 0 || rows[i] >= Mp) return -1;
    int fail = 0;
#pragma omp parallel
    {
        i128 *acc = (i128 *)malloc((size_t)N * sizeof(i128));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for collapse(3) schedule(dynamic, 1)
        for (int64_t j = 0; j < L; ++j)
            for (int64_t r = 0; r < nrows; ++r)
                for (int64_t c = 0; c < 2; ++c) {
                    if (!acc) continue;
                    for (int64_t n = 0; n < N; ++n) acc[n] = 0;
                    for (int64_t k = 0; k < Kp; ++k) {
                        const int64_t *p = pt + ((size_t)rows[r] * Kp + k) * N;
                        const uint64_t *x = ct + (((size_t)j * Kp + k) * 2 + c) * N;
                        /* p(X) x(X): the term p_s x_t goes to X^{s+t}, and X^{s+t} = -X^{s+t-N} past the degree */
                        for (int64_t s = 0; s < N; ++s) {
                            const i128 ps = p[s];
                            if (ps == 0) continue;
                            for (int64_t t = 0; t < N; ++t) {
                                const i128 term = ps * (i128)x[t];
                                if (s + t < N) acc[s + t] += term;
                                else acc[s + t - N] -= term;
                            }
                        }
                    }
                    uint64_t *o = out + (((size_t)j * nrows + r) * 2 + c) * N;
                    for (int64_t n = 0; n < N; ++n) o[n] = canon_mod(acc[n], primes[j]);
                }
        free(acc);
    }
    return fail ? -1 : 0;
}
