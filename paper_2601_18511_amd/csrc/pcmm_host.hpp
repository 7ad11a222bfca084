// Host-side planning of the PCMM library: argument validation, the digit count, the tile geometry, the
// sizes of the plan's buffers and the per-limb constants of the epilogue.  Plain C++ with no HIP in it,
// so that it can be compiled and run on its own under the host sanitizers; pcmm.hip includes it and
// owns everything that touches the device.
//
// The operation planned is C_j = W . A_j mod q_j for every RNS limb j (the clear matrix product that
// the paper's linear-layer PCMM reduces to, Sections 2.2 and 5.1); the weights are converted once per
// matrix (the paper's "model conversion", Section 5.3).
#ifndef PCMM_HOST_HPP
#define PCMM_HOST_HPP

#include <stddef.h>
#include <stdint.h>

#include "../../include/pcmm.h"

namespace pcmm_host {

typedef unsigned __int128 u128;

constexpr int kFragBytes = 1024;   // one 16 x 64 int8 MFMA operand fragment
constexpr int kMaxLimbs = 64;

// Per-limb constants of the epilogue.
struct LimbConst {
    uint64_t q;      // the prime
    uint64_t mu;     // floor(2^64 / q)
    uint64_t off;    // q * floor(2^62 / q) >= 2^61: added to a signed part of magnitude < 2^56 to make it positive
    uint64_t c32;    // 2^32 mod q
    uint64_t c32s;   // floor(c32 * 2^64 / q)  (Shoup companion of c32)
    uint64_t c64;    // 2^64 mod q
    uint64_t c64s;   // floor(c64 * 2^64 / q)
    double qd;       // q as a double (exact for q < 2^53)
    double invq;     // 1.0 / q, rounded to nearest
};

namespace epi {
// How the epilogue reduces sum_e acc_e 256^e modulo q.
enum Epi : int {
    EPI_F64 = 0,     // q < 2^50: exact double-precision arithmetic (fma remainders), no 64-bit multiplies
    EPI_INT = 2,     // any q < 2^62: one 64-bit Barrett per four accumulators, joined by Shoup
                     // multiplications by 2^32 and 2^64
    EPI_F64_G4 = 3,  // as EPI_F64 with the accumulators grouped in fours: |acc| < 2^28, 7 or 8 accumulators
    EPI_F64_G4P = 4  // as EPI_F64_G4 with pairs of accumulators first joined in int32: 257 |acc| < 2^31
};
}  // namespace epi

inline LimbConst limb_const(uint64_t q)
{
    LimbConst c;
    c.q = q;
    c.mu = (uint64_t)((((u128)1) << 64) / q);
    c.off = q * (uint64_t)((((u128)1) << 62) / q);
    c.c32 = (uint64_t)((((u128)1) << 32) % q);
    c.c32s = (uint64_t)(((u128)c.c32 << 64) / q);
    c.c64 = (uint64_t)((((u128)1) << 64) % q);
    c.c64s = (uint64_t)(((u128)c.c64 << 64) / q);
    c.qd = (double)q;
    c.invq = 1.0 / (double)q;
    return c;
}

// Smallest D with (qmax - 1) + Bias_D < 256^D, Bias_D = sum_{i<D} 128 * 256^i: the number of signed
// base-256 digits that represent every residue below qmax.  0 if more than 8 would be needed.
inline int balanced_digits(uint64_t qmax)
{
    for (int d = 1; d <= 8; ++d) {
        u128 bias = 0;
        for (int i = 0; i < d; ++i) bias |= (u128)0x80 << (8 * i);
        if ((u128)(qmax - 1) + bias < ((u128)1 << (8 * d))) return d;
    }
    return 0;
}

// Accumulator footprint limits the tile: MT*NT*E*4 accumulator registers per lane (NT = 2), at most 160.
constexpr int tile_mt(int E) { return E <= 5 ? 4 : (E == 6 ? 3 : 2); }

// Everything about a plan that follows from its arguments alone.
struct Geometry {
    int D, S, E;               // digits per residue, int8 slices of W, accumulators per output
    int WM, MT, NT;            // waves per work-group, 16-row fragments per wave, 16-column fragments per tile
    int epi;                   // epi::Epi
    int64_t MB;                // padded M / 16
    int64_t nkb;               // padded K / 64 (even)
    int64_t nkb_launch;        // most k-steps one GEMM launch may contract (int32 accumulator headroom)
    int64_t mtiles, ntiles;
    size_t wp_bytes, ad_bytes, lc_bytes;
    uint32_t w_kstride;        // bytes between k-steps of one packed W slice
    uint32_t a_kstride;        // bytes between k-steps of one limb's digit chunks
};

// Validates the arguments of pcmm_plan_create that need no device and derives the geometry.
inline pcmm_status plan_geometry(int64_t M, int64_t K, int64_t Ncols, int32_t L, const uint64_t *primes_host,
                                 int32_t prime_bits, int32_t w_bits, int32_t device, Geometry *g)
{
    if (!primes_host || !g) return PCMM_EINVAL;
    if (M <= 0 || K <= 0 || Ncols <= 0 || L <= 0 || L > kMaxLimbs) return PCMM_EINVAL;
    if (M > (int64_t)1 << 24 || Ncols > (int64_t)1 << 22) return PCMM_EINVAL;   // 32-bit row offsets in the stores
    if (w_bits != 8 && w_bits != 16) return PCMM_EINVAL;
    if (prime_bits < 24 || prime_bits > 62) return PCMM_EINVAL;
    if (device < 0) return PCMM_EINVAL;
    uint64_t qmax = 0, qmin = ~(uint64_t)0;
    for (int j = 0; j < L; ++j) {
        const uint64_t q = primes_host[j];
        if ((q & 1) == 0) return PCMM_EINVAL;
        if (q <= ((uint64_t)1 << (prime_bits - 1)) || q >= ((uint64_t)1 << prime_bits)) return PCMM_EINVAL;
        if (q > qmax) qmax = q;
        if (q < qmin) qmin = q;
    }
    const int S = w_bits / 8;
    if (K > ((int64_t)1 << 22) - 128) return PCMM_EINVAL;   // k-steps are a grid dimension of the split kernel
    // int32 headroom: one launch may contract Kl values of k with S*Kl*2^14 < 2^31, S*Kl <= 131071;
    // in k-steps of 64, rounded down to the even count the main loop needs
    const int64_t nkb_launch = 131071 / S / 128 * 2;
    const int64_t K_launch = K < nkb_launch * 64 ? K : nkb_launch * 64;

    int D = balanced_digits(qmax);
    if (D == 0) return PCMM_EUNSUPPORTED;
    if (D < 4) D = 4;   // kernels are built for 4..8 digits; spare top digits are zero
    const int E = D + S - 1;
    if (E > 9) return PCMM_EUNSUPPORTED;   // cannot happen with D <= 8 and S <= 2; kept as a guard

    g->D = D; g->S = S; g->E = E;
    g->NT = 2;
    g->MT = tile_mt(E);
    g->WM = (M > (int64_t)2 * g->MT * 16) ? 4 : 2;
    const int64_t BM = (int64_t)g->WM * g->MT * 16, BN = (int64_t)g->NT * 16;
    g->mtiles = (M + BM - 1) / BM;
    g->ntiles = (Ncols + BN - 1) / BN;
    g->MB = g->mtiles * BM / 16;
    g->nkb = (K + 127) / 128 * 2;   // the main loop takes two k-steps of 64 per round
    g->nkb_launch = nkb_launch;
    if ((int64_t)L * g->mtiles * g->ntiles > 0x7fffff00LL) return PCMM_EUNSUPPORTED;   // the grid is a 32-bit count

    g->epi = qmax < ((uint64_t)1 << 50) ? epi::EPI_F64 : epi::EPI_INT;
    // short contractions leave small accumulators: |acc| <= S * K_launch * 2^14
    if (g->epi == epi::EPI_F64 && E >= 7 && qmin > ((uint64_t)1 << 37)) {
        if ((int64_t)S * K_launch <= 509) g->epi = epi::EPI_F64_G4P;   // 257 * S*K * 2^14 < 2^31
        else if ((int64_t)S * K_launch <= 16383) g->epi = epi::EPI_F64_G4;
    }

    g->wp_bytes = (size_t)S * g->MB * g->nkb * kFragBytes;
    g->ad_bytes = (size_t)L * g->ntiles * g->nkb * g->NT * D * kFragBytes;
    g->lc_bytes = (size_t)L * sizeof(LimbConst);
    // buffer loads address one W slice and one limb of digit planes with 32-bit unsigned byte offsets
    if (g->wp_bytes / S >= ((size_t)1 << 31) || g->ad_bytes / L >= ((size_t)1 << 32)) return PCMM_EUNSUPPORTED;
    g->w_kstride = (uint32_t)(g->MB * kFragBytes);
    g->a_kstride = (uint32_t)(g->ntiles * g->NT * D * kFragBytes);
    return PCMM_OK;
}

// Byte offset of k-step kk inside one W slice or one limb of digit chunks, as the kernel forms it:
// an unsigned 32-bit product.  The plan guarantees that (nkb - 1) * stride fits.
inline uint32_t kstep_offset(uint32_t kk, uint32_t kstride) { return kk * kstride; }

}  // namespace pcmm_host

#endif  // PCMM_HOST_HPP
