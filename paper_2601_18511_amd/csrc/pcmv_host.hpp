// Host-side planning of the PCMv path: argument validation, the primitive 2N-th root of unity of
// every prime and the twiddle tables of the negacyclic number-theoretic transform, as balanced
// residues held in doubles.  Plain C++ with no HIP in it (it can run under the host sanitizers).
//
// The transforms serve the ring products of the decode-time matrix-vector multiplication: plaintext
// polynomials are kept in the NTT domain (Section 5.3), ring degree 4096 (Table "he-operators").
#ifndef PCMV_HOST_HPP
#define PCMV_HOST_HPP

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/pcmm.h"

namespace pcmv_host {

typedef unsigned __int128 u128;

constexpr int kMaxLimbs = 64;
constexpr int64_t kMaxN = 4096;    // two polynomials of doubles fit 64 KiB of LDS

inline uint64_t mulmod(uint64_t a, uint64_t b, uint64_t q) { return (uint64_t)((u128)a * b % q); }

inline uint64_t powmod(uint64_t a, uint64_t e, uint64_t q)
{
    uint64_t r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = mulmod(r, a, q);
        a = mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}

// A primitive 2N-th root of unity modulo the prime q = 1 (mod 2N): psi with psi^N = -1.  0 if none is
// found among the first candidates (q is then not a prime of that form).
inline uint64_t primitive_root_2n(uint64_t q, uint64_t N)
{
    if (N == 0 || (q - 1) % (2 * N) != 0) return 0;
    const uint64_t e = (q - 1) / (2 * N);
    for (uint64_t x = 2; x < 2000 && x < q; ++x) {
        const uint64_t psi = powmod(x, e, q);
        if (powmod(psi, N, q) == q - 1) return psi;
    }
    return 0;
}

inline uint32_t bit_reverse(uint32_t v, int bits)
{
    uint32_t r = 0;
    for (int i = 0; i < bits; ++i) r |= ((v >> i) & 1u) << (bits - 1 - i);
    return r;
}

// the representative of v mod q in (-q/2, q/2], as a double (exact: q < 2^52)
inline double balanced(uint64_t v, uint64_t q) { return v > q / 2 ? -(double)(q - v) : (double)v; }

// Per-limb constants and tables of the transforms of size N = 2^logn:
//   fwd[i] = psi^bitrev(i), inv[i] = psi^-bitrev(i)   (bit reversal over logn bits), both balanced
struct LimbTables {
    uint64_t q, psi;
    double qd, invq, n_inv;           // q, 1/q (rounded), N^-1 mod q (balanced)
    std::vector<double> fwd, inv;
};

inline pcmm_status limb_tables(uint64_t q, int64_t N, LimbTables *t)
{
    int logn = 0;
    while (((int64_t)1 << logn) < N) ++logn;
    if (((int64_t)1 << logn) != N) return PCMM_EINVAL;
    const uint64_t psi = primitive_root_2n(q, (uint64_t)N);
    if (psi == 0) return PCMM_EINVAL;
    const uint64_t psi_inv = powmod(psi, q - 2, q);
    t->q = q;
    t->psi = psi;
    t->qd = (double)q;
    t->invq = 1.0 / (double)q;
    t->n_inv = balanced(powmod((uint64_t)N % q, q - 2, q), q);
    t->fwd.resize((size_t)N);
    t->inv.resize((size_t)N);
    std::vector<uint64_t> pw((size_t)N), pwi((size_t)N);      // psi^i and psi^-i
    pw[0] = pwi[0] = 1;
    for (int64_t i = 1; i < N; ++i) {
        pw[(size_t)i] = mulmod(pw[(size_t)i - 1], psi, q);
        pwi[(size_t)i] = mulmod(pwi[(size_t)i - 1], psi_inv, q);
    }
    for (int64_t i = 0; i < N; ++i) {
        const uint32_t r = bit_reverse((uint32_t)i, logn);
        t->fwd[(size_t)i] = balanced(pw[r], q);
        t->inv[(size_t)i] = balanced(pwi[r], q);
    }
    return PCMM_OK;
}

// Validates what needs no device.  Primes: odd, of prime_bits bits, 24 <= prime_bits <= 50 (the
// transforms compute in exact double-precision arithmetic), q = 1 (mod 2N).
inline pcmm_status check_args(int64_t Mp, int64_t Kp, int64_t N, int32_t L, const uint64_t *primes_host,
                              int32_t prime_bits, int32_t device)
{
    if (!primes_host) return PCMM_EINVAL;
    if (Mp <= 0 || Kp <= 0 || N < 2 || L <= 0 || L > kMaxLimbs || device < 0) return PCMM_EINVAL;
    if (N & (N - 1)) return PCMM_EINVAL;
    if (prime_bits < 24 || prime_bits > 62) return PCMM_EINVAL;
    for (int j = 0; j < L; ++j) {
        const uint64_t q = primes_host[j];
        if ((q & 1) == 0) return PCMM_EINVAL;
        if (q <= ((uint64_t)1 << (prime_bits - 1)) || q >= ((uint64_t)1 << prime_bits)) return PCMM_EINVAL;
        if ((q - 1) % (2 * (uint64_t)N) != 0) return PCMM_EINVAL;
    }
    if (prime_bits > 50 || N > kMaxN) return PCMM_EUNSUPPORTED;
    if (Kp > 4096 || Mp > ((int64_t)1 << 24)) return PCMM_EUNSUPPORTED;
    if ((int64_t)L * Mp > 0x7fffff00LL || (int64_t)L * Mp * Kp > 0x7fffff00LL) return PCMM_EUNSUPPORTED;   // grids
    return PCMM_OK;
}

}  // namespace pcmv_host

#endif  // PCMV_HOST_HPP
