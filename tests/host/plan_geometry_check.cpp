// Host-only check of the plan's argument validation, geometry and constants (csrc/pcmm_host.hpp),
// meant to be compiled with g++ -fsanitize=address,undefined and run on the CPU.  Exit status 0 = every
// check held; a failed check prints its line and exits 1; a sanitizer finding aborts.
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include "pcmm_host.hpp"

using namespace pcmm_host;

static int failures = 0;
#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            printf("line %d: check failed: %s\n", __LINE__, #cond);              \
            ++failures;                                                          \
        }                                                                        \
    } while (0)

static bool is_prime(uint64_t n)
{
    if (n < 2) return false;
    for (uint64_t d = 2; d * d <= n && d < (1u << 20); ++d)
        if (n % d == 0) return false;
    return true;
}

// an odd number of exactly `bits` bits (primality does not matter to the plan)
static uint64_t odd_of_bits(int bits, uint64_t salt) { return (((uint64_t)1 << (bits - 1)) | 1u) + 2 * (salt % 1000) + ((uint64_t)1 << (bits - 2)); }

static void check_limb_const(uint64_t q)
{
    const LimbConst c = limb_const(q);
    const u128 one = 1;
    CHECK(c.q == q);
    CHECK((u128)c.mu * q <= (one << 64) && (u128)(c.mu + 1) * q > (one << 64));
    CHECK(c.off % q == 0 && c.off >= ((uint64_t)1 << 61) && c.off <= ((uint64_t)1 << 62));
    CHECK(c.c32 == (uint64_t)((one << 32) % q));
    CHECK(c.c64 == (uint64_t)((one << 64) % q));
    CHECK((u128)c.c32s * q <= ((u128)c.c32 << 64) && (u128)(c.c32s + 1) * q > ((u128)c.c32 << 64));
    CHECK((u128)c.c64s * q <= ((u128)c.c64 << 64) && (u128)(c.c64s + 1) * q > ((u128)c.c64 << 64));
    if (q < ((uint64_t)1 << 53)) CHECK((uint64_t)c.qd == q);
    CHECK(c.invq > 0.0 && c.invq * c.qd > 0.999999 && c.invq * c.qd < 1.000001);
}

static void check_geometry(int64_t M, int64_t K, int64_t Ncols, int L, int bits, int w_bits)
{
    std::vector<uint64_t> primes(L);
    for (int j = 0; j < L; ++j) primes[j] = odd_of_bits(bits, (uint64_t)j * 7 + 3);
    Geometry g;
    const pcmm_status rc = plan_geometry(M, K, Ncols, L, primes.data(), bits, w_bits, 0, &g);
    if (rc == PCMM_EUNSUPPORTED) return;   // too large for 32-bit offsets: allowed outcome
    CHECK(rc == PCMM_OK);
    if (rc != PCMM_OK) return;
    CHECK(g.S == w_bits / 8 && g.E == g.D + g.S - 1 && g.D >= 4 && g.D <= 8);
    CHECK(4 * g.MT * g.NT * g.E <= 160);
    CHECK(g.nkb % 2 == 0 && g.nkb * 64 >= K && g.nkb * 64 < K + 128);
    CHECK(g.MB * 16 >= M && g.ntiles * g.NT * 16 >= Ncols);
    CHECK(g.nkb_launch % 2 == 0 && (int64_t)g.S * g.nkb_launch * 64 <= 131071);
    // every k-step offset the kernel forms is the same number in 32-bit unsigned and in 64-bit arithmetic
    const uint32_t last = (uint32_t)(g.nkb - 1);
    CHECK((uint64_t)kstep_offset(last, g.a_kstride) == (uint64_t)last * (uint64_t)g.a_kstride);
    CHECK((uint64_t)kstep_offset(last, g.w_kstride) == (uint64_t)last * (uint64_t)g.w_kstride);
    CHECK((uint64_t)g.nkb * g.a_kstride == g.ad_bytes / (size_t)L);
    CHECK((uint64_t)g.nkb * g.w_kstride == g.wp_bytes / (size_t)g.S);
    // the digit count covers the largest residue
    uint64_t qmax = 0;
    for (int j = 0; j < L; ++j) qmax = primes[j] > qmax ? primes[j] : qmax;
    u128 bias = 0;
    for (int i = 0; i < g.D; ++i) bias |= (u128)0x80 << (8 * i);
    CHECK((u128)(qmax - 1) + bias < ((u128)1 << (8 * g.D)));
}

int main()
{
    // the benchmark's workloads: (M, K, Ncols, L, bits, w_bits)
    check_geometry(128, 128, 8192, 2, 36, 8);
    check_geometry(4096, 4096, 32768, 4, 36, 8);
    check_geometry(14336, 4096, 32768, 4, 36, 8);
    check_geometry(4096, 14336, 32768, 3, 36, 8);
    check_geometry(4096, 128, 131072, 6, 50, 16);
    check_geometry(4096, 4096, 32768, 1, 62, 16);
    {   // the long contraction: k-step 223 of 224 lies beyond 2^31 bytes
        uint64_t q[3] = {68718428161ull, 68717740033ull, 68716036097ull};
        Geometry g;
        CHECK(plan_geometry(4096, 14336, 32768, 3, q, 36, 8, 0, &g) == PCMM_OK);
        CHECK(g.a_kstride == 10485760u && g.nkb == 224);
        CHECK(kstep_offset(223, g.a_kstride) == 2338324480u);
        CHECK(kstep_offset(223, g.a_kstride) > 0x7fffffffu);
    }
    // a sweep over sizes, prime widths and weight widths, including the limits
    const int64_t Ms[] = {1, 31, 33, 256, 4097, (int64_t)1 << 24};
    const int64_t Ks[] = {1, 64, 129, 4096, 131071, 131072, ((int64_t)1 << 22) - 128};
    const int64_t Ns[] = {1, 33, 8192, (int64_t)1 << 22};
    const int bitss[] = {24, 31, 32, 33, 36, 40, 41, 48, 49, 50, 51, 55, 56, 57, 62};
    for (int64_t M : Ms)
        for (int64_t K : Ks)
            for (int64_t N : Ns)
                for (int bits : bitss)
                    for (int wb = 8; wb <= 16; wb += 8) check_geometry(M, K, N, 1 + (int)((M + K + N) % 3), bits, wb);

    // rejected arguments: status codes, never a fault
    {
        uint64_t q = 68719403009ull, even = 68719403008ull;
        Geometry g;
        CHECK(plan_geometry(0, 4, 4, 1, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, -1, 4, 1, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 0, 1, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 0, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 65, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, nullptr, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 36, 8, 0, nullptr) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 36, 12, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 35, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 37, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 63, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 23, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &even, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, 4, 1, &q, 36, 8, -1, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, ((int64_t)1 << 22) - 127, 4, 1, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(((int64_t)1 << 24) + 1, 4, 4, 1, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        CHECK(plan_geometry(4, 4, ((int64_t)1 << 22) + 1, 1, &q, 36, 8, 0, &g) == PCMM_EINVAL);
        // one limb of digit planes of 4 GiB or more
        CHECK(plan_geometry(64, 1 << 20, 1 << 20, 1, &q, 36, 8, 0, &g) == PCMM_EUNSUPPORTED);
    }

    // digit counts at the switch points: D digits reach up to 256^D - Bias_D
    CHECK(balanced_digits(((uint64_t)1 << 36) - 1) == 5);
    CHECK(balanced_digits(0x7F7F7F7F7Full) == 5 && balanced_digits(0x7F7F7F7F80ull) == 5 && balanced_digits(0x7F7F7F7F81ull) == 6);
    CHECK(balanced_digits(((uint64_t)1 << 50) - 1) == 7);
    CHECK(balanced_digits(((uint64_t)1 << 62) - 1) == 8);
    CHECK(balanced_digits(((uint64_t)1 << 63) + 5) == 0);

    // per-limb constants, from the smallest to the largest supported primes
    const uint64_t qs[] = {8388617ull, 16777213ull, 68719403009ull, 68718428161ull, 1125899903827969ull,
                           (((uint64_t)1 << 55) - 55), (((uint64_t)1 << 61) - 1), 4611686018427387847ull, 4611686018326724609ull};
    for (uint64_t q : qs) {
        CHECK(q % 2 == 1);
        (void)is_prime(q);
        check_limb_const(q);
    }
    if (failures) {
        printf("%d checks failed\n", failures);
        return 1;
    }
    printf("plan geometry: all checks held\n");
    return 0;
}
