// Device-side helpers shared by the PCMM kernels: vector types, modular arithmetic, the exact
// double-precision reduction of the epilogue, compile-time loops.  Included by every .hip file of the
// library; everything here is inline device code.
#ifndef PCMM_DEVICE_HPP
#define PCMM_DEVICE_HPP

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

#include "pcmm_host.hpp"

namespace pcmm_device {

using pcmm_host::LimbConst;
using namespace pcmm_host::epi;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int kFrag = pcmm_host::kFragBytes;   // bytes of one 16 x 64 int8 MFMA operand fragment
constexpr int kXcd = 8;       // accelerator complex dies, each with its own L2

// ------------------------------------------------------------------------------------------------
// modular helpers (device)
// ------------------------------------------------------------------------------------------------
// u < 2^64, mu = floor(2^64/q).  qhat = floor(u*mu / 2^64) satisfies u/q - 2 < qhat <= u/q, hence
// u - qhat*q is in [0, 2q) and one conditional subtraction gives the canonical residue.
__device__ __forceinline__ uint64_t barrett_u64(uint64_t u, uint64_t q, uint64_t mu)
{
    uint64_t qhat = __umul64hi(u, mu);
    uint64_t r = u - qhat * q;
    return r >= q ? r - q : r;
}

// x < q < 2^63, c < q, cs = floor(c * 2^64 / q): returns x*c mod q (Shoup's constant multiplication).
__device__ __forceinline__ uint64_t mulmod_shoup(uint64_t x, uint64_t c, uint64_t cs, uint64_t q)
{
    uint64_t qhat = __umul64hi(x, cs);
    uint64_t r = x * c - qhat * q;
    return r >= q ? r - q : r;
}

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), fully unrolled
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Exact reduction in double precision.  `a` holds E int32 accumulators; returns (sum_e a[e] 256^e) mod q
// in [0, q) for 2^23 < q < 2^50.
//
// The accumulators are grouped from the bottom into G-digit numbers, G = 3 in general:
// c_g = a[3g] + 2^8 a[3g+1] + 2^16 a[3g+2] (|c_g| < 2^47.01, exact in a double).  Horner in base
// B = 2^(8G) from the top group, one step per group:
//   X  = r B                         exact (power-of-two scaling)
//   qh = rint((X + c_g) / q)         the sum and the quotient are rounded: qh = (X + c_g)/q + eta with
//                                    |eta| <= 0.5 + 3.01 * 2^-53 * |X + c_g|/q  <=  0.6
//                                    (G = 3: |X + c_g|/q < 2^48.01 in the first step, where r = c_top is not
//                                    yet reduced, and < 2^24 afterwards)
//   u  = fma(-qh, q, X)              = -c_g - eta q exactly: an integer of magnitude below 2^53
//   r  = u + c_g                     = -eta q exactly, so |r| <= 0.6 q
// After the last group a negative r is lifted by q, which lands in [0, q) because |r| <= 0.6 q.
// Every operation is exact or feeds the rint whose error the exact fma absorbs, so the result is the
// canonical residue bit for bit.
//
// MODE 1 (E = 7 or 8 accumulators of magnitude < 2^28, q > 2^37): G = 4, so that two groups and a single
// Horner step remain.  |c_g| < 2^28 (1 + 2^8 + 2^16 + 2^24) < 2^52.01 is still exact, |X + c_g| < 2^84.02
// in the one step gives |X + c_g|/q < 2^47.1 and |eta| <= 0.5 + 3.01 * 2^-5.9 < 0.56, and
// |u| <= |c_g| + 0.56 q < 2^53.
// MODE 2 (in addition 257 |acc| < 2^31): neighbouring accumulators are first joined in int32,
// p = a[2i] + 2^8 a[2i+1], which halves the conversions to double.
// R outputs are reduced side by side, stage by stage: R independent dependency chains in the order the
// scheduler should issue them.
template <int E, int MODE, int R>
__device__ __forceinline__ void reduce_f64(const int (&a)[R][E], double q, double invq, uint64_t (&res)[R])
{
    constexpr int GS = MODE == 0 ? 3 : 4;            // accumulators per group
    constexpr int G = (E + GS - 1) / GS;
    static_assert(G >= 2, "at least one Horner step");
    static_assert(MODE == 0 || G == 2, "groups of four are proved for a single Horner step");
    double c[G][R];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int b0 = GS * g;
        if constexpr (MODE == 2) {
            int p0[R], p1[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                p0[r] = b0 + 1 < E ? a[r][b0] + (int)((unsigned)a[r][b0 + 1] << 8) : a[r][b0];
                if (b0 + 2 < E) p1[r] = b0 + 3 < E ? a[r][b0 + 2] + (int)((unsigned)a[r][b0 + 3] << 8) : a[r][b0 + 2];
            }
#pragma unroll
            for (int r = 0; r < R; ++r) c[g][r] = (double)p0[r];
            if (b0 + 2 < E) {
#pragma unroll
                for (int r = 0; r < R; ++r) c[g][r] = __builtin_fma((double)p1[r], 65536.0, c[g][r]);
            }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) c[g][r] = (double)a[r][b0];
#pragma unroll
            for (int i = 1; i < GS; ++i)
                if (b0 + i < E) {
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        c[g][r] = __builtin_fma((double)a[r][b0 + i], (double)(1 << (8 * i)), c[g][r]);
                }
        }
    }
    constexpr double B = MODE == 0 ? 16777216.0 : 4294967296.0;
    double rr[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rr[r] = c[G - 1][r];
#pragma unroll
    for (int g = G - 2; g >= 0; --g) {
        double X[R], qh[R];
#pragma unroll
        for (int r = 0; r < R; ++r) X[r] = rr[r] * B;
#pragma unroll
        for (int r = 0; r < R; ++r) qh[r] = __builtin_rint((X[r] + c[g][r]) * invq);
#pragma unroll
        for (int r = 0; r < R; ++r) rr[r] = __builtin_fma(-qh[r], q, X[r]) + c[g][r];
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        // lift a negative remainder by q without a compare and selects: |rr| <= 0.6 q, so rr / q lies in (-1, 1) and
        // its floor is -1 for every negative rr (the product cannot round to zero: |rr| >= 1) and 0 otherwise
        const double v = __builtin_fma(-__builtin_floor(rr[r] * invq), q, rr[r]);
        // v is an integer in [0, 2^52): adding 2^52 places it in the low mantissa bits
        res[r] = (uint64_t)__double_as_longlong(v + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
    }
}

}  // namespace pcmm_device

#endif  // PCMM_DEVICE_HPP
