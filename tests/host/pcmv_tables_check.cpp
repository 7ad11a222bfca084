// Host-only check of the PCMv planning code (csrc/pcmv_host.hpp): roots of unity, twiddle tables, argument
// validation.  Meant for g++ -fsanitize=address,undefined; exit status 0 = every check held.
#include <stdio.h>

#include "pcmv_host.hpp"

using namespace pcmv_host;

static int failures = 0;
#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            printf("line %d: check failed: %s\n", __LINE__, #cond);              \
            ++failures;                                                          \
        }                                                                        \
    } while (0)

static uint64_t unbalance(double v, uint64_t q) { return v < 0 ? q - (uint64_t)(-v) : (uint64_t)v; }

static void check_prime(uint64_t q, int64_t N)
{
    LimbTables t;
    CHECK(limb_tables(q, N, &t) == PCMM_OK);
    CHECK(powmod(t.psi, (uint64_t)N, q) == q - 1);                       // psi^N = -1: a primitive 2N-th root
    CHECK(powmod(t.psi, 2 * (uint64_t)N, q) == 1);
    CHECK(mulmod(unbalance(t.n_inv, q), (uint64_t)N % q, q) == 1);
    CHECK((uint64_t)t.qd == q && t.invq * t.qd > 0.999999 && t.invq * t.qd < 1.000001);
    int logn = 0;
    while (((int64_t)1 << logn) < N) ++logn;
    for (int64_t i = 0; i < N; ++i) {
        const uint32_t r = bit_reverse((uint32_t)i, logn);
        const uint64_t f = unbalance(t.fwd[(size_t)i], q), g = unbalance(t.inv[(size_t)i], q);
        CHECK(f == powmod(t.psi, r, q));
        CHECK(mulmod(f, g, q) == 1);                                      // inv[i] is the inverse of fwd[i]
        CHECK(t.fwd[(size_t)i] <= (double)(q / 2) && t.fwd[(size_t)i] >= -(double)(q / 2));
        if (failures) return;
    }
}

int main()
{
    CHECK(bit_reverse(1, 12) == 2048 && bit_reverse(6, 3) == 3 && bit_reverse(0, 5) == 0);
    CHECK(mulmod(~(uint64_t)0 % 97, 96, 97) == ((unsigned __int128)(~(uint64_t)0 % 97) * 96) % 97);
    CHECK(powmod(3, 0, 97) == 1 && powmod(3, 96, 97) == 1);
    check_prime(97, 16);                                  // 97 = 1 mod 32
    check_prime(12289, 2048);                             // 12289 = 1 mod 4096
    check_prime(68718428161ull, 4096);                    // 2^36 - 2^20 + 1
    check_prime(1125899903827969ull, 4096);               // a 50-bit prime = 1 mod 2^17
    LimbTables t;
    CHECK(limb_tables(97, 64, &t) == PCMM_EINVAL);        // 97 is not 1 mod 128
    CHECK(limb_tables(97, 24, &t) == PCMM_EINVAL);        // not a power of two
    CHECK(primitive_root_2n(97, 0) == 0);

    uint64_t q = 68718428161ull, even = 68718428160ull, q56 = ((uint64_t)1 << 56) - ((uint64_t)1 << 20) + 1;
    CHECK(check_args(4, 1, 4096, 1, &q, 36, 0) == PCMM_OK);
    CHECK(check_args(0, 1, 4096, 1, &q, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 0, 4096, 1, &q, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 1, 1, &q, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4095, 1, &q, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4096, 0, &q, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4096, 65, &q, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4096, 1, nullptr, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4096, 1, &q, 35, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4096, 1, &even, 36, 0) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 4096, 1, &q, 36, -1) == PCMM_EINVAL);
    CHECK(check_args(4, 1, 1 << 21, 1, &q, 36, 0) == PCMM_EINVAL);          // q is not 1 mod 2^22
    CHECK(check_args(4, 1, 8192, 1, &q, 36, 0) == PCMM_EUNSUPPORTED);
    CHECK(check_args(4, 4097, 4096, 1, &q, 36, 0) == PCMM_EUNSUPPORTED);
    CHECK(check_args(4, 1, 4096, 1, &q56, 56, 0) == PCMM_EUNSUPPORTED);
    CHECK(check_args((int64_t)1 << 24, 4096, 4096, 1, &q, 36, 0) == PCMM_EUNSUPPORTED);
    if (failures) {
        printf("%d checks failed\n", failures);
        return 1;
    }
    printf("pcmv tables: all checks held\n");
    return 0;
}
