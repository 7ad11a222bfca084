// PCMv for MI355X (gfx950): the ring products of the decode-time plaintext-ciphertext matrix-vector
// multiplication,
//     out_j[m][c] = sum_{k<Kp} pt[m][k] * ct_j[k][c]   in  Z_{q_j}[X]/(X^N + 1),   c in {a, b},
// for every RNS limb j (Section 3.2: in decoding the matrix-matrix products become matrix-vector products;
// Table "he-operators": ring degree 4096, coefficient encoding; Section 5.3: the plaintext polynomials are
// kept in the NTT domain).  The packing of the weights into plaintext polynomials and the extraction of the
// useful coefficients afterwards belong to the algorithm the paper adopts by reference and are not here.
//
// Kernels:
//   ntt_kernel / ntt4096_kernel   forward negacyclic NTT of polynomials: the plaintexts once, at plan time ("model
//                     conversion"), and the 2 Kp L ciphertext polynomials of every run
//   mac_intt_kernel / mac_intt4096_kernel   per (limb, m): pointwise multiply-accumulate of the NTT-domain plaintexts
//                     with both ciphertext components, inverse NTT of the two sums, store as uint64 residues
// The *4096* kernels serve the paper's ring degree: sixteen values per thread in registers, four stages per pass, two
// trips through LDS per transform; the multiply-accumulate kernel runs as persistent work-groups fed from a queue.
// The others serve every other power of two up to 4096, one radix-2 stage per pass over LDS.
//
// Arithmetic.  MI355X runs double-precision vector arithmetic at full rate while 64-bit integer
// multiplication costs many quarter-rate 32-bit multiplies, so residues are held as balanced integers in
// doubles and multiplied exactly with fused multiply-adds (mulmod below); the bound q < 2^50 comes from
// there.  In the general kernels a polynomial lives in LDS as N doubles and each radix-2 stage is one pass over
// LDS (Gentleman-Sande inverse butterflies, bit-reversed order in, natural order out, twiddle inv[groups + group]).
//
// HBM traffic per run: the NTT-domain plaintexts are read once (8 Mp Kp N L bytes, the dominant term for
// long contractions) and the output written once (16 Mp N L bytes).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/pcmm.h"
#include "pcmm_hip_util.hpp"
#include "pcmv_host.hpp"

namespace {

constexpr int kThreads = 256;

// Rounding to the nearest integer without the (slower) rounding instruction: for |x| < 2^51 the sum
// x + 1.5 * 2^52 has unit spacing, so its rounding is the rounding of x to an integer (ties to even), and
// subtracting the constant again is exact.  round_fma(h, s) rounds the exact product h s once.
constexpr double kRoundMagic = 6755399441055744.0;   // 1.5 * 2^52
__device__ __forceinline__ double round_fma(double h, double s) { return __builtin_fma(h, s, kRoundMagic) - kRoundMagic; }

// a b mod q for integers held in doubles, |a| <= q/2 + 1, |b| <= 4 q, 2^23 < q < 2^50; returns r = a b (mod q) with
// |r| <= q, and |r| <= 0.75 q + 1 when |b| <= 2 q.
//   h = RN(a b), l = a b - h exactly (fma);  |a b| <= 2 q^2 < 2^101, so |l| <= 2^48 and l is an integer
//   qh = round(h invq) = a b / q + eta:  |h invq| <= 2 q (1 + 2^-51) < 2^51, the two roundings (of h and of
//        invq) shift it by at most 2^-52 |a b| / q <= 2^-51 q < 0.5 (0.25 for |b| <= 2 q), so |eta| <= 1 (0.75)
//   fma(-qh, q, h) = (a b - qh q) - l: an integer of magnitude < 2^50 + 2^48 < 2^53, so exact; adding l is exact
// The same function serves the transforms of primes below 2^36 that never reduce their sums: |a| <= q/2 + 1,
// |b| <= 2^13 q.  Then |h invq| < 2^49 (the rounding trick holds), qh = a b / q + eta with
// |eta| <= 1/2 + 2^-52 2^12 q <= 0.5625, h and qh q are integers whose difference is below 0.5625 q + |l|,
// |l| <= 2^30: fma(-qh, q, h) and the addition of l are exact and |r| <= 0.5625 q.  A value that is only ever added
// to others through the twelve stages grows to at most 2^12 0.5625 q < 2^12 q < 2^48, differences to 2^13 q.
__device__ __forceinline__ double mulmod(double a, double b, double q, double invq)
{
    const double h = a * b;
    const double l = __builtin_fma(a, b, -h);
    const double qh = round_fma(h, invq);
    return __builtin_fma(-qh, q, h) + l;
}

// the representative of an integer |v| < 2^52 modulo q (q > 2^23) with magnitude at most q/2 (+1 when the quotient
// rounds the other way)
__device__ __forceinline__ double reduce(double v, double q, double invq)
{
    return __builtin_fma(-round_fma(v, invq), q, v);
}

// Forward negacyclic NTT in place on N doubles in LDS (natural order in, bit-reversed order out).
// Cooley-Tukey butterflies with the powers of psi merged in: stage with m groups uses fwd[m + group].
// Inputs of magnitude <= q/2; outputs of magnitude <= 1.375 q.
__device__ __forceinline__ void ntt_forward(double *s, const double *__restrict__ fwd, int N, double q, double invq)
{
    int lt = 31 - __builtin_clz((unsigned)N);             // log2 of the butterfly span t
    for (int m = 1; m < N; m <<= 1) {
        --lt;
        const int t = 1 << lt;
        for (int bf = threadIdx.x; bf < N / 2; bf += kThreads) {
            const int i = bf >> lt, jj = bf & (t - 1);
            const int j = (i << (lt + 1)) + jj;
            const double S = fwd[m + i];
            const double U = reduce(s[j], q, invq);
            const double V = mulmod(S, s[j + t], q, invq);
            s[j] = U + V;
            s[j + t] = U - V;
        }
        __syncthreads();
    }
}

struct LimbDev {
    double q, invq, n_inv;
    double pad;
};

// Forward NTT of polynomials.  SRC = 0: uint64 residues in [0, q) (ciphertext polynomials, laid out
// [L][polys_per_limb][N]); SRC = 1: signed 32-bit plaintext coefficients shared by all limbs ([polys_per_limb][N]).
// Output: doubles [L][polys_per_limb][N], magnitudes <= q/2 + 1, bit-reversed order (plaintexts times 1/N mod q); with rot16 != 0 (N = 4096)
// entry n of that order is stored at (n >> 4) | ((n & 15) << 8), the order mac_intt4096_kernel reads with
// coalesced loads.
template <int SRC>
__global__ __launch_bounds__(kThreads) void ntt_kernel(const void *__restrict__ src, double *__restrict__ dst,
                                                       const double *__restrict__ fwd_tables, const LimbDev *__restrict__ lc,
                                                       int N, int64_t polys_per_limb, int rot16)
{
    extern __shared__ double lds[];
    const int64_t p = blockIdx.x;
    const int limb = (int)(p / polys_per_limb);
    const int64_t within = p % polys_per_limb;
    const double q = lc[limb].q, invq = lc[limb].invq;
    for (int n = threadIdx.x; n < N; n += kThreads) {
        double v;
        if (SRC == 0) {
            const uint64_t x = static_cast<const uint64_t *>(src)[p * N + n];
            v = __builtin_fma((double)(uint32_t)(x >> 32), 4294967296.0, (double)(uint32_t)x);   // exact: x < 2^50
        } else {
            v = (double)static_cast<const int32_t *>(src)[within * N + n];
        }
        lds[n] = reduce(v, q, invq);
    }
    __syncthreads();
    ntt_forward(lds, fwd_tables + (int64_t)limb * N, N, q, invq);
    // the plaintexts carry the factor 1/N of the inverse transform that follows the pointwise products
    const double scale = lc[limb].n_inv;
    for (int n = threadIdx.x; n < N; n += kThreads) {
        const int pos = rot16 ? ((n >> 4) | ((n & 15) << 8)) : n;
        double r = reduce(lds[n], q, invq);
        if (SRC == 1) r = reduce(mulmod(scale, r, q, invq), q, invq);
        dst[p * N + pos] = r;
    }
}

// One work-group per (limb, m): acc_c = sum_k ptn[m][k] (.) ctn[k][c] for c = a, b, inverse NTT of both,
// times 1/N, canonical residues out.
//   ptn [L][Mp][Kp][N] doubles, ctn [L][Kp][2][N] doubles (both |.| <= q/2 + 1), out [L][Mp][2][N] uint64
__global__ __launch_bounds__(kThreads) void mac_intt_kernel(const double *__restrict__ ptn, const double *__restrict__ ctn,
                                                            uint64_t *__restrict__ out, const double *__restrict__ inv_tables,
                                                            const LimbDev *__restrict__ lc, int N, int64_t Mp, int Kp)
{
    extern __shared__ double lds[];          // two polynomials: [0, N) component a, [N, 2N) component b
    const int64_t blk = blockIdx.x;
    const int limb = (int)(blk / Mp);
    const int64_t m = blk % Mp;
    const double q = lc[limb].q, invq = lc[limb].invq;
    const double *pt = ptn + ((int64_t)limb * Mp + m) * Kp * N;
    const double *ct = ctn + (int64_t)limb * Kp * 2 * N;
    for (int n = threadIdx.x; n < N; n += kThreads) {
        double acc_a = 0.0, acc_b = 0.0;
        for (int k = 0; k < Kp; ++k) {
            const double w = pt[(int64_t)k * N + n];
            acc_a = reduce(acc_a + mulmod(w, ct[((int64_t)k * 2 + 0) * N + n], q, invq), q, invq);
            acc_b = reduce(acc_b + mulmod(w, ct[((int64_t)k * 2 + 1) * N + n], q, invq), q, invq);
        }
        lds[n] = acc_a;
        lds[N + n] = acc_b;
    }
    __syncthreads();
    const double *inv = inv_tables + (int64_t)limb * N;
    // the two transforms run stage by stage side by side (one barrier per stage for both)
    int lt = 0;                                            // log2 of the butterfly span t
    for (int mm = N; mm > 1; mm >>= 1) {
        const int h = mm >> 1, t = 1 << lt;
        for (int bf = threadIdx.x; bf < N; bf += kThreads) {          // N butterflies: N/2 per polynomial
            const int half = bf >= N / 2;
            const int b2 = bf - half * (N / 2);
            const int i = b2 >> lt, jj = b2 & (t - 1);
            double *s = lds + half * N;
            const int j = (i << (lt + 1)) + jj;
            const double S = inv[h + i];
            const double U = s[j], V = s[j + t];
            s[j] = reduce(U + V, q, invq);
            s[j + t] = mulmod(S, U - V, q, invq);
        }
        __syncthreads();
        ++lt;
    }
    uint64_t *o = out + ((int64_t)limb * Mp + m) * 2 * N;
    for (int n = threadIdx.x; n < 2 * N; n += kThreads) {
        double r = reduce(lds[n], q, invq);                          // |r| <= q/2 + 1 (1/N is folded into the plaintexts)
        r = r < 0.0 ? r + q : r;                                      // canonical: an integer in [0, q)
        o[n] = (uint64_t)__double_as_longlong(r + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
    }
}


// ---- N = 4096 (the paper's PCMv ring degree): the inverse transform as three passes of four stages each,
// sixteen elements per thread in registers, two trips through LDS instead of twelve.
//
// Entry n of the bit-reversed NTT-domain order is stored at (n >> 4) | ((n & 15) << 8) (see ntt_kernel), so
// that thread T reads its entries n = 16 T + e, e < 16, from T + 256 e: consecutive threads, consecutive words.
//   pass 1  stages t = 1, 2, 4, 8        thread T holds n = 16 T + e
//   pass 2  stages t = 16 .. 128         thread T = 16 A + B holds n = 256 A + B + 16 e
//   pass 3  stages t = 256 .. 2048       thread T holds n = T + 256 e
// Stage t pairs n with n + t and uses the twiddle inv[N/(2t) + (n >> (log2 t + 1))]: 8, 4, 2 and 1 distinct
// twiddles per thread in the four stages of a pass, contiguous in the table.
// LDS holds entry n at n + (n >> 4) (one word of padding per sixteen): the 16-word strides of pass 1's writes
// and the unit strides of the other accesses are then all free of bank conflicts for 8-byte accesses.
constexpr int kN4096 = 4096;
constexpr int kLdsPoly4096 = kN4096 + kN4096 / 16;

// four Gentleman-Sande stages on sixteen values; tw[0..7], tw[8..11], tw[12..13], tw[14]: the twiddles of the
// four stages (stage s pairs e with e + 2^s and uses twiddle number e >> (s + 1) of its run).
// Magnitudes, LAZY = false (q < 2^50): inputs <= q.  Stages 0 and 2 leave their sums unreduced (<= 2 q; differences
// <= 2 q give products <= 0.75 q + 1), stages 1 and 3 reduce the sums (<= 4 q < 2^52 in, <= q/2 + 1 out) and
// multiply differences <= 4 q (products <= q): outputs <= q again.
// LAZY = true (q < 2^36): no sum is reduced anywhere in the twelve stages of the transform (bounds in the comment of mulmod).
template <bool LAZY>
__device__ __forceinline__ void gs16(double (&v)[16], const double (&tw)[15], double q, double invq)
{
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int half = 1 << s;
        const int off = s == 0 ? 0 : (s == 1 ? 8 : (s == 2 ? 12 : 14));
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            if (e & half) continue;
            const double U = v[e], V = v[e + half];
            v[e] = (!LAZY && (s & 1)) ? reduce(U + V, q, invq) : U + V;
            v[e + half] = mulmod(tw[off + (e >> (s + 1))], U - V, q, invq);
        }
    }
}

// The canonical residue in [0, q) of an integer v = k q + s, 0 <= s < q, for q (|k| + 1) < 2^50:
//   x = fma(v, invq, invq / 2) = (k + (s + 1/2) / q) (1 + eps), |eps| < 2^-51 (the rounding of invq and of the fma),
//   and (s + 1/2) / q lies in [1/(2q), 1 - 1/(2q)]: |x - (k + (s + 1/2)/q)| < (|k| + 1) 2^-51 < 1/(2q), so floor(x) = k
//   and fma(-k, q, v) = s exactly.
__device__ __forceinline__ double canonical(double v, double q, double invq, double half_invq)
{
    return __builtin_fma(-__builtin_floor(__builtin_fma(v, invq, half_invq)), q, v);
}

typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));

// a range-checked view of n_bytes of device memory (reads outside it return 0)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t view(const void *base, uint32_t n_bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, n_bytes, 0x00020000);
}
// one double / two doubles at byte offset lane_off + uniform_off
__device__ __forceinline__ double ld1(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(double, (v2u)__builtin_amdgcn_raw_buffer_load_b64(r, lane_off, uniform_off, 0));
}
__device__ __forceinline__ v2d ld2(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(v2d, (v4u)__builtin_amdgcn_raw_buffer_load_b128(r, lane_off, uniform_off, 0));
}
// the fifteen twiddles of four stages: eight consecutive table entries from 8 (base + i0), four from 4 (base + i0),
// two from 2 (base + i0), one at base + i0
__device__ __forceinline__ void load_tw(double (&tw)[15], __amdgpu_buffer_rsrc_t irs, uint32_t base, uint32_t i0)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const v2d t = ld2(irs, (8 * base + 8 * i0) * 8u, 16u * i);
        tw[2 * i] = t[0];
        tw[2 * i + 1] = t[1];
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const v2d t = ld2(irs, (4 * base + 4 * i0) * 8u, 16u * i);
        tw[8 + 2 * i] = t[0];
        tw[9 + 2 * i] = t[1];
    }
    const v2d t = ld2(irs, (2 * base + 2 * i0) * 8u, 0);
    tw[12] = t[0];
    tw[13] = t[1];
    tw[14] = ld1(irs, (base + i0) * 8u, 0);
}

// four Cooley-Tukey stages on sixteen values (stage s pairs e with e + (8 >> s); its 2^s twiddles are the run of
// that length in tw, in the layout load_tw produces: tw[14], tw[12..13], tw[8..11], tw[0..7]).
// Magnitudes, LAZY = false: inputs <= 1.5 q + 1.  Stages 0 and 2 add a product (<= 0.75 q + 1, its operand being
// <= 2 q) to an unreduced value: <= 2.25 q + 2; stages 1 and 3 reduce that value first (<= q/2 + 1) and multiply
// operands <= 2.25 q + 2 <= 4 q (products <= q): outputs <= 1.5 q + 1 again.
// LAZY = true (q < 2^36): nothing is reduced; a value grows by at most 0.5625 q per stage, to less than 8 q in twelve.
template <bool LAZY>
__device__ __forceinline__ void ct16(double (&v)[16], const double (&tw)[15], double q, double invq)
{
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int half = 8 >> s;
        const int off = s == 0 ? 14 : (s == 1 ? 12 : (s == 2 ? 8 : 0));
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            if (e & half) continue;
            const double U = (!LAZY && (s & 1)) ? reduce(v[e], q, invq) : v[e];
            const double V = mulmod(tw[off + (e >> (4 - s))], v[e + half], q, invq);
            v[e] = U + V;
            v[e + half] = U - V;
        }
    }
}

// Forward negacyclic NTT of polynomials of degree 4096, one per work-group: the mirror image of the inverse
// transform below -- three passes of four Cooley-Tukey stages on sixteen values per thread, two trips through LDS.
//   pass A  stages t = 2048 .. 256       thread T holds n = T + 256 e     (read from memory, coalesced)
//   pass B  stages t = 128 .. 16         thread T = 16 A + B holds n = 256 A + B + 16 e
//   pass C  stages t = 8 .. 1            thread T holds n = 16 T + e      (entry n of the bit-reversed order, stored at
//                                        T + 256 e: the order the multiply-accumulate reads)
// Stage t = N/(2m) uses the twiddle fwd[m + (n >> (log2 t + 1))].  Sources and the scaling of the plaintexts as in ntt_kernel.
template <int SRC, bool LAZY>
__global__ __launch_bounds__(kThreads) void ntt4096_kernel(const void *__restrict__ src, double *__restrict__ dst,
                                                           const double *__restrict__ fwd_tables, const LimbDev *__restrict__ lc,
                                                           int64_t polys_per_limb, uint32_t *__restrict__ queue, uint32_t queue_start)
{
    constexpr int N = kN4096;
    __shared__ double lds[kLdsPoly4096];
    const int64_t p = blockIdx.x;
    if (queue && p == 0 && threadIdx.x == 0) *queue = queue_start;       // the work queue of the kernel that follows
    const int limb = (int)(p / polys_per_limb);
    const int64_t within = p % polys_per_limb;
    const double q = lc[limb].q, invq = lc[limb].invq;
    const __amdgpu_buffer_rsrc_t frs = view(fwd_tables + (int64_t)limb * N, N * 8);
    const int T = threadIdx.x, A = T >> 4, B = T & 15;
    double v[16], tw[15];
    load_tw(tw, frs, 1, 0);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        if (SRC == 0) {
            const uint64_t x = static_cast<const uint64_t *>(src)[p * N + T + 256 * e];
            v[e] = __builtin_fma((double)(uint32_t)(x >> 32), 4294967296.0, (double)(uint32_t)x);   // exact: x < 2^50
        } else {
            v[e] = (double)static_cast<const int32_t *>(src)[within * N + T + 256 * e];
        }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) v[e] = reduce(v[e], q, invq);
    ct16<LAZY>(v, tw, q, invq);
#pragma unroll
    for (int e = 0; e < 16; ++e) lds[T + (T >> 4) + 272 * e] = v[e];
    load_tw(tw, frs, 16, A);
    __syncthreads();
    {
        double *s = lds + 272 * A + B;
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = s[17 * e];
        ct16<LAZY>(v, tw, q, invq);
#pragma unroll
        for (int e = 0; e < 16; ++e) s[17 * e] = v[e];
    }
    load_tw(tw, frs, 256, T);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 16; ++e) v[e] = lds[17 * T + e];
    ct16<LAZY>(v, tw, q, invq);
    // the plaintexts carry the factor 1/N of the inverse transform that follows the pointwise products
    const double scale = lc[limb].n_inv;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        double r = reduce(v[e], q, invq);
        if (SRC == 1) r = reduce(mulmod(scale, r, q, invq), q, invq);
        dst[p * N + T + 256 * e] = r;
    }
}

// Persistent work-groups: work-group g takes the output polynomials g, g + G, g + 2 G, ... (G = grid size, two
// work-groups per compute unit), so that what depends only on the limb stays in registers from one polynomial to the
// next -- the twiddles of passes 1 and 2 and, for KP1 (one input ciphertext, the shape of every decode projection whose
// input fits one polynomial), the thread's 32 values of the transformed ciphertext -- and the plaintext values of the
// next polynomial are requested while the present one is transformed.  total = L Mp polynomials; the loop ends for
// every wave when its index passes total.
//
// LAZY (every prime below 2^36): no intermediate reduction of sums, neither in the transform nor between the
// terms of the multiply-accumulate (Kp <= 4096 products of magnitude <= 0.5625 q: below 2^12 q; one reduction
// after the last term).
//
// All global reads are buffer loads (uniform base and offset in scalar registers, one 32-bit lane offset): no vector
// registers go into addresses, and the loads of a term are all issued before the first is used (left to itself the
// compiler starts the arithmetic on the first values early, which splits the loads into two dependent round trips).
template <bool LAZY, bool KP1>
__global__ __launch_bounds__(kThreads, 2) void mac_intt4096_kernel(const double *__restrict__ ptn, const double *__restrict__ ctn,
                                                                   uint64_t *__restrict__ out, const double *__restrict__ inv_tables,
                                                                   const LimbDev *__restrict__ lc, uint32_t Mp, int Kp, uint32_t total,
                                                                   uint32_t *__restrict__ queue)
{
    constexpr int N = kN4096;
    constexpr uint32_t PB = N * 8;                    // bytes of one polynomial of doubles
    __shared__ double lds[2 * kLdsPoly4096];          // component a, component b
    __shared__ uint32_t queue_word;
    const int T = threadIdx.x;
    const uint32_t toff = (uint32_t)T * 8u;
    uint32_t blk = blockIdx.x;
    if (blk >= total) return;
    uint32_t next = blk + gridDim.x;                  // the first two polynomials of a work-group are fixed; total + 3 grid < 2^32
    const uint32_t kpb = (uint32_t)Kp * PB;           // bytes of the plaintexts of one output polynomial (Kp <= 4096)

    double tw1[15], tw2[15], xa[16], xb[16], wv[16];
    double q = 0.0, invq = 0.0;
    uint32_t limb_loaded = 0xFFFFFFFFu;
    {
        const __amdgpu_buffer_rsrc_t prs = view(ptn + (int64_t)blk * Kp * N, kpb);
#pragma unroll
        for (int e = 0; e < 16; ++e) wv[e] = ld1(prs, toff, 2048u * e);
    }
    for (;;) {
        const uint32_t limb = blk / Mp;
        // the polynomial after the next one comes from the queue (one lane asks; the answer is passed on through LDS
        // behind the first barrier below)
        uint32_t asked = 0;
        if (T == 0) asked = atomicAdd(queue, 1u);
        // the LDS addresses below are recomputed from the thread index in every round (the asm hides that it is the same
        // index): kept across the loop they cost more registers than the kernel has
        int Ti = T;
        asm volatile("" : "+v"(Ti));
        const int Ai = Ti >> 4, Bi = Ti & 15;
        const __amdgpu_buffer_rsrc_t crs = view(ctn + (int64_t)limb * Kp * 2 * N, 2 * kpb);
        const __amdgpu_buffer_rsrc_t irs = view(inv_tables + (int64_t)limb * N, PB);
        if (limb != limb_loaded) {                    // uniform: first polynomial of a limb for this work-group
            limb_loaded = limb;
            q = lc[limb].q;
            invq = lc[limb].invq;
            if constexpr (KP1) {
                load_tw(tw1, irs, 256, T);            // pass 1: table entries 2048 + 8 T .., 1024 + 4 T .., 512 + 2 T .., 256 + T
                load_tw(tw2, irs, 16, T >> 4);        // pass 2, A = T / 16: 128 + 8 A .., 64 + 4 A .., 32 + 2 A .., 16 + A
#pragma unroll
                for (int e = 0; e < 16; ++e) xa[e] = ld1(crs, toff, 2048u * e);
#pragma unroll
                for (int e = 0; e < 16; ++e) xb[e] = ld1(crs, toff, PB + 2048u * e);
            }
        }

        // ---- pass 1: pointwise multiply-accumulate of both components straight into registers (each plaintext
        // value is loaded once and used for a and b), then stages t = 1 .. 8
        double va[16], vb[16];
        if constexpr (KP1) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                va[e] = mulmod(wv[e], xa[e], q, invq);
                vb[e] = mulmod(wv[e], xb[e], q, invq);
            }
        } else {
            const __amdgpu_buffer_rsrc_t prs = view(ptn + (int64_t)blk * Kp * N, kpb);
#pragma unroll
            for (int e = 0; e < 16; ++e) va[e] = vb[e] = 0.0;
            auto term = [&](int k, auto last_c) {
                constexpr bool LAST = decltype(last_c)::value;
                double wn[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) xa[e] = ld1(crs, toff, (uint32_t)k * 2 * PB + 2048u * e);
#pragma unroll
                for (int e = 0; e < 16; ++e) xb[e] = ld1(crs, toff, (uint32_t)k * 2 * PB + PB + 2048u * e);
                if constexpr (!LAST) {                 // the plaintext values of the next term
#pragma unroll
                    for (int e = 0; e < 16; ++e) wn[e] = ld1(prs, toff, (uint32_t)(k + 1) * PB + 2048u * e);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    if constexpr (LAZY) {
                        va[e] += mulmod(wv[e], xa[e], q, invq);
                        vb[e] += mulmod(wv[e], xb[e], q, invq);
                    } else {
                        va[e] = reduce(va[e] + mulmod(wv[e], xa[e], q, invq), q, invq);
                        vb[e] = reduce(vb[e] + mulmod(wv[e], xb[e], q, invq), q, invq);
                    }
                }
                if constexpr (!LAST) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) wv[e] = wn[e];
                }
            };
            for (int k = 0; k < Kp - 1; ++k) term(k, std::false_type{});
            term(Kp - 1, std::true_type{});
        }
        // The products are complete here: the empty asm uses them and orders memory accesses, so that the compiler can
        // neither sink the arithmetic below the loads that follow nor lift those loads above it (either way the registers
        // would have to hold the operands of both).
#pragma unroll
        for (int e = 0; e < 16; e += 4)
            asm volatile("" ::"v"(va[e]), "v"(va[e + 1]), "v"(va[e + 2]), "v"(va[e + 3]), "v"(vb[e]), "v"(vb[e + 1]), "v"(vb[e + 2]),
                         "v"(vb[e + 3])
                         : "memory");
        // the first plaintext values of the next polynomial are requested now and used in the next round
        if (next < total) {
            const __amdgpu_buffer_rsrc_t nrs = view(ptn + (int64_t)next * Kp * N, kpb);
#pragma unroll
            for (int e = 0; e < 16; ++e) wv[e] = ld1(nrs, toff, 2048u * e);
        }
        if constexpr (!KP1) {
            // with several terms the registers do not hold the twiddles from one polynomial to the next
            load_tw(tw1, irs, 256, Ti);
            load_tw(tw2, irs, 16, Ai);
            if constexpr (LAZY) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    va[e] = reduce(va[e], q, invq);
                    vb[e] = reduce(vb[e], q, invq);
                }
            }
        }
        gs16<LAZY>(va, tw1, q, invq);
        if (T == 0) queue_word = asked;
        __syncthreads();                                               // every wave has read the previous polynomial from LDS
        const uint32_t after_next = __builtin_amdgcn_readfirstlane(queue_word);
#pragma unroll
        for (int e = 0; e < 16; ++e) lds[17 * Ti + e] = va[e];          // n = 16 T + e at n + (n >> 4)
        gs16<LAZY>(vb, tw1, q, invq);
#pragma unroll
        for (int e = 0; e < 16; ++e) lds[kLdsPoly4096 + 17 * Ti + e] = vb[e];
        __syncthreads();

        // ---- pass 2: stages t = 16 .. 128 on n = 256 A + B + 16 e, i.e. LDS word 272 A + B + 17 e
        for (int c = 0; c < 2; ++c) {
            double *s = lds + c * kLdsPoly4096 + 272 * Ai + Bi;
            double v[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = s[17 * e];
            gs16<LAZY>(v, tw2, q, invq);
#pragma unroll
            for (int e = 0; e < 16; ++e) s[17 * e] = v[e];
        }
        __syncthreads();

        // ---- pass 3: stages t = 256 .. 2048 on n = T + 256 e, i.e. LDS word T + (T >> 4) + 272 e; then out
        // (the fifteen twiddles are the same for every thread: table entries 1 .. 15)
        const double *inv = inv_tables + (int64_t)limb * N;
        double tw3[15];
#pragma unroll
        for (int i = 0; i < 8; ++i) tw3[i] = inv[8 + i];
#pragma unroll
        for (int i = 0; i < 4; ++i) tw3[8 + i] = inv[4 + i];
        tw3[12] = inv[2];
        tw3[13] = inv[3];
        tw3[14] = inv[1];
        const double half_invq = 0.5 * invq;
        uint64_t *o = out + (int64_t)blk * 2 * N;
        for (int c = 0; c < 2; ++c) {
            const double *s = lds + c * kLdsPoly4096 + Ti + (Ti >> 4);
            double v[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = s[272 * e];
            gs16<LAZY>(v, tw3, q, invq);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                double r;                                              // canonical: an integer in [0, q) (1/N is folded into the plaintexts)
                if constexpr (LAZY) {
                    r = canonical(v[e], q, invq, half_invq);          // |v| < 2^12 q, q < 2^36
                } else {
                    r = reduce(v[e], q, invq);                        // |r| <= q/2 + 1
                    r = r < 0.0 ? r + q : r;
                }
                o[c * N + Ti + 256 * e] = (uint64_t)__double_as_longlong(r + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
            }
        }
        if (next >= total) break;
        blk = next;
        next = after_next;
    }
}

}  // namespace

struct pcmv_plan {
    int64_t Mp, Kp, N;
    int L, device;
    uint32_t grid;     // work-groups of the persistent degree-4096 kernel: two per compute unit
    uint32_t *queue;   // device: its work queue (one counter)
    bool lazy;         // every prime is below 2^36: the degree-4096 transform runs without intermediate reductions
    double *ptn;       // device [L][Mp][Kp][N]: plaintexts in the NTT domain
    double *ctn;       // device [L][Kp][2][N]: scratch, the ciphertexts of one run in the NTT domain
    double *fwd, *inv; // device [L][N] twiddle tables
    LimbDev *lc;       // device [L]
    size_t bytes;
};

extern "C" {

pcmm_status pcmv_plan_create(pcmv_plan **out, int64_t Mp, int64_t Kp, int64_t N, int32_t L, const uint64_t *primes_host,
                             int32_t prime_bits, const int32_t *pt_dev, int32_t device, void *stream)
{
    if (!out) return PCMM_EINVAL;
    *out = nullptr;
    if (!pt_dev) return PCMM_EINVAL;
    const pcmm_status arc = pcmv_host::check_args(Mp, Kp, N, L, primes_host, prime_bits, device);
    if (arc != PCMM_OK) return arc;

    std::vector<double> fwd, inv;
    std::vector<LimbDev> lc((size_t)L);
    try {
        fwd.resize((size_t)L * N);
        inv.resize((size_t)L * N);
        for (int j = 0; j < L; ++j) {
            pcmv_host::LimbTables t;
            const pcmm_status trc = pcmv_host::limb_tables(primes_host[j], N, &t);
            if (trc != PCMM_OK) return trc;          // no primitive 2N-th root: not a prime of the form 1 mod 2N
            for (int64_t i = 0; i < N; ++i) {
                fwd[(size_t)j * N + i] = t.fwd[(size_t)i];
                inv[(size_t)j * N + i] = t.inv[(size_t)i];
            }
            lc[(size_t)j].q = t.qd;
            lc[(size_t)j].invq = t.invq;
            lc[(size_t)j].n_inv = t.n_inv;
            lc[(size_t)j].pad = 0.0;
        }
    } catch (const std::bad_alloc &) {
        return PCMM_ENOMEM;
    }

    pcmv_plan *p = new (std::nothrow) pcmv_plan();
    if (!p) return PCMM_ENOMEM;
    p->Mp = Mp; p->Kp = Kp; p->N = N; p->L = L; p->device = device;
    p->lazy = prime_bits <= 36;      // check_args: every prime has exactly prime_bits bits
    p->ptn = nullptr; p->ctn = nullptr; p->fwd = nullptr; p->inv = nullptr; p->lc = nullptr; p->queue = nullptr;
    p->grid = 0;
    pcmm_hip_util::DevGuard dg(device);
    if (!dg.ok) { delete p; return PCMM_EDEVICE; }
    hipStream_t st = (hipStream_t)stream;
    const size_t ptn_bytes = (size_t)L * Mp * Kp * N * sizeof(double);
    const size_t ctn_bytes = (size_t)L * Kp * 2 * N * sizeof(double);
    const size_t tab_bytes = (size_t)L * N * sizeof(double);
    const size_t lc_bytes = (size_t)L * sizeof(LimbDev);
    pcmm_status rc = PCMM_OK;
    if (hipMalloc((void **)&p->ptn, ptn_bytes) != hipSuccess || hipMalloc((void **)&p->ctn, ctn_bytes) != hipSuccess ||
        hipMalloc((void **)&p->fwd, tab_bytes) != hipSuccess || hipMalloc((void **)&p->inv, tab_bytes) != hipSuccess ||
        hipMalloc((void **)&p->lc, lc_bytes) != hipSuccess || hipMalloc((void **)&p->queue, 256) != hipSuccess) {
        (void)hipGetLastError();
        rc = PCMM_ENOMEM;
    }
    p->bytes = ptn_bytes + ctn_bytes + 2 * tab_bytes + lc_bytes + 256;
    if (rc == PCMM_OK) {
        // the persistent degree-4096 kernel runs two work-groups per compute unit
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0) rc = PCMM_EDEVICE;
        const int64_t total = (int64_t)L * Mp;
        p->grid = (uint32_t)(total < 2 * (int64_t)cus ? total : 2 * (int64_t)cus);
    }
    if (rc == PCMM_OK) {
        if (hipMemcpyAsync(p->fwd, fwd.data(), tab_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipMemcpyAsync(p->inv, inv.data(), tab_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipMemcpyAsync(p->lc, lc.data(), lc_bytes, hipMemcpyHostToDevice, st) != hipSuccess)
            rc = PCMM_EDEVICE;
    }
    if (rc == PCMM_OK) {
        // the plaintexts into the NTT domain, once (the paper's model conversion for PCMv, Section 5.3)
        const int64_t polys = (int64_t)L * Mp * Kp;
        if (N == kN4096)
            hipLaunchKernelGGL((p->lazy ? ntt4096_kernel<1, true> : ntt4096_kernel<1, false>), dim3((unsigned)polys), dim3(kThreads), 0,
                               st, (const void *)pt_dev, p->ptn, p->fwd, p->lc, Mp * Kp, (uint32_t *)nullptr, 0u);
        else
            hipLaunchKernelGGL((ntt_kernel<1>), dim3((unsigned)polys), dim3(kThreads), (size_t)N * sizeof(double), st,
                               (const void *)pt_dev, p->ptn, p->fwd, p->lc, (int)N, Mp * Kp, 0);
        if (hipGetLastError() != hipSuccess) rc = PCMM_EDEVICE;
    }
    if (hipStreamSynchronize(st) != hipSuccess) rc = rc == PCMM_OK ? PCMM_EDEVICE : rc;   // the host tables live on this frame
    if (rc != PCMM_OK) {
        pcmv_plan_destroy(p);
        return rc;
    }
    *out = p;
    return PCMM_OK;
}

size_t pcmv_plan_workspace_bytes(const pcmv_plan *plan) { return plan ? plan->bytes : 0; }

pcmm_status pcmv_run(const pcmv_plan *plan, const uint64_t *ct_dev, uint64_t *out_dev, void *stream)
{
    if (!plan || !ct_dev || !out_dev) return PCMM_EINVAL;
    pcmm_hip_util::DevGuard dg(plan->device);
    if (!dg.ok) return PCMM_EDEVICE;
    hipStream_t st = (hipStream_t)stream;
    const int N = (int)plan->N;
    const int64_t ct_polys = (int64_t)plan->L * plan->Kp * 2;
    if (N == kN4096)
        hipLaunchKernelGGL((plan->lazy ? ntt4096_kernel<0, true> : ntt4096_kernel<0, false>), dim3((unsigned)ct_polys), dim3(kThreads),
                           0, st, (const void *)ct_dev, plan->ctn, plan->fwd, plan->lc, plan->Kp * 2, plan->queue, 2u * plan->grid);
    else
        hipLaunchKernelGGL((ntt_kernel<0>), dim3((unsigned)ct_polys), dim3(kThreads), (size_t)N * sizeof(double), st,
                           (const void *)ct_dev, plan->ctn, plan->fwd, plan->lc, N, plan->Kp * 2, 0);
    if (hipGetLastError() != hipSuccess) return PCMM_EDEVICE;
    if (N == kN4096)
    {
        const uint32_t total = (uint32_t)(plan->L * plan->Mp);
        const uint32_t grid = plan->grid;
        auto kern = plan->Kp == 1 ? (plan->lazy ? mac_intt4096_kernel<true, true> : mac_intt4096_kernel<false, true>)
                                  : (plan->lazy ? mac_intt4096_kernel<true, false> : mac_intt4096_kernel<false, false>);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), 0, st, plan->ptn, plan->ctn, out_dev, plan->inv, plan->lc,
                           (uint32_t)plan->Mp, (int)plan->Kp, total, plan->queue);
    }
    else
    hipLaunchKernelGGL(mac_intt_kernel, dim3((unsigned)((int64_t)plan->L * plan->Mp)), dim3(kThreads),
                       (size_t)2 * N * sizeof(double), st, plan->ptn, plan->ctn, out_dev, plan->inv, plan->lc, N, plan->Mp,
                       (int)plan->Kp);
    return hipGetLastError() == hipSuccess ? PCMM_OK : PCMM_EDEVICE;
}

void pcmv_plan_destroy(pcmv_plan *plan)
{
    if (!plan) return;
    pcmm_hip_util::DevGuard dg(plan->device);
    if (plan->ptn) (void)hipFree(plan->ptn);
    if (plan->ctn) (void)hipFree(plan->ctn);
    if (plan->fwd) (void)hipFree(plan->fwd);
    if (plan->inv) (void)hipFree(plan->inv);
    if (plan->lc) (void)hipFree(plan->lc);
    if (plan->queue) (void)hipFree(plan->queue);
    delete plan;
}

}  // extern "C"
