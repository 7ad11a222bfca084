// PCMv for MI355X (gfx950): the ring products of the decode-time plaintext-ciphertext matrix-vector
// multiplication,
//     out_j[m][c] = sum_{k<Kp} pt[m][k] * ct_j[k][c]   in  Z_{q_j}[X]/(X^N + 1),   c in {a, b},
// for every RNS limb j (Section 3.2: in decoding the matrix-matrix products become matrix-vector products;
// Table "he-operators": ring degree 4096, coefficient encoding; Section 5.3: the plaintext polynomials are
// kept in the NTT domain).  The packing of the weights into plaintext polynomials and the extraction of the
// useful coefficients afterwards belong to the algorithm the paper adopts by reference and are not here.
//
// Kernels:
//   ntt_kernel        forward negacyclic NTT of polynomials: the plaintexts once, at plan time ("model
//                     conversion"), and the 2 Kp L ciphertext polynomials of every run
//   mac_intt_kernel   per (limb, m): pointwise multiply-accumulate of the NTT-domain plaintexts with both
//                     ciphertext components, inverse NTT of the two sums, store as uint64 residues
//                     (mac_intt4096_kernel for the paper's ring degree: register-blocked, two trips through LDS)
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
// Magnitudes: inputs <= q.  Stages 0 and 2 leave their sums unreduced (<= 2 q; differences <= 2 q give products
// <= 0.75 q + 1), stages 1 and 3 reduce the sums (<= 4 q < 2^52 in, <= q/2 + 1 out) and multiply differences
// <= 4 q (products <= q): outputs <= q again.
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
            v[e] = (s & 1) ? reduce(U + V, q, invq) : U + V;
            v[e + half] = mulmod(tw[off + (e >> (s + 1))], U - V, q, invq);
        }
    }
}

__global__ __launch_bounds__(kThreads, 2) void mac_intt4096_kernel(const double *__restrict__ ptn, const double *__restrict__ ctn,
                                                                   uint64_t *__restrict__ out, const double *__restrict__ inv_tables,
                                                                   const LimbDev *__restrict__ lc, int64_t Mp, int Kp)
{
    constexpr int N = kN4096;
    __shared__ double lds[2 * kLdsPoly4096];          // component a, component b
    const int64_t blk = blockIdx.x;
    const int limb = (int)(blk / Mp);
    const int64_t m = blk % Mp;
    const double q = lc[limb].q, invq = lc[limb].invq;
    const double *pt = ptn + ((int64_t)limb * Mp + m) * Kp * N;
    const double *ct = ctn + (int64_t)limb * Kp * 2 * N;
    const double *inv = inv_tables + (int64_t)limb * N;
    const int T = threadIdx.x, A = T >> 4, B = T & 15;
    double tw[15];

    // ---- pass 1: pointwise multiply-accumulate of both components straight into registers (each plaintext
    // value is loaded once and used for a and b), then stages t = 1 .. 8
    {
        double va[16], vb[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) va[e] = vb[e] = 0.0;
        for (int k = 0; k < Kp; ++k) {
            const double *w = pt + (int64_t)k * N + T;
            const double *xa = ct + ((int64_t)k * 2 + 0) * N + T;
            const double *xb = ct + ((int64_t)k * 2 + 1) * N + T;
            double wv[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) wv[e] = w[256 * e];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                va[e] = reduce(va[e] + mulmod(wv[e], xa[256 * e], q, invq), q, invq);
                vb[e] = reduce(vb[e] + mulmod(wv[e], xb[256 * e], q, invq), q, invq);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) tw[i] = inv[2048 + 8 * T + i];
#pragma unroll
        for (int i = 0; i < 4; ++i) tw[8 + i] = inv[1024 + 4 * T + i];
        tw[12] = inv[512 + 2 * T];
        tw[13] = inv[512 + 2 * T + 1];
        tw[14] = inv[256 + T];
        gs16(va, tw, q, invq);
#pragma unroll
        for (int e = 0; e < 16; ++e) lds[17 * T + e] = va[e];          // n = 16 T + e at n + (n >> 4)
        gs16(vb, tw, q, invq);
#pragma unroll
        for (int e = 0; e < 16; ++e) lds[kLdsPoly4096 + 17 * T + e] = vb[e];
    }
    __syncthreads();

    // ---- pass 2: stages t = 16 .. 128 on n = 256 A + B + 16 e, i.e. LDS word 272 A + B + 17 e
#pragma unroll
    for (int i = 0; i < 8; ++i) tw[i] = inv[128 + 8 * A + i];
#pragma unroll
    for (int i = 0; i < 4; ++i) tw[8 + i] = inv[64 + 4 * A + i];
    tw[12] = inv[32 + 2 * A];
    tw[13] = inv[32 + 2 * A + 1];
    tw[14] = inv[16 + A];
    for (int c = 0; c < 2; ++c) {
        double *s = lds + c * kLdsPoly4096 + 272 * A + B;
        double v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = s[17 * e];
        gs16(v, tw, q, invq);
#pragma unroll
        for (int e = 0; e < 16; ++e) s[17 * e] = v[e];
    }
    __syncthreads();

    // ---- pass 3: stages t = 256 .. 2048 on n = T + 256 e, i.e. LDS word T + (T >> 4) + 272 e; then 1/N, out
#pragma unroll
    for (int i = 0; i < 8; ++i) tw[i] = inv[8 + i];
#pragma unroll
    for (int i = 0; i < 4; ++i) tw[8 + i] = inv[4 + i];
    tw[12] = inv[2];
    tw[13] = inv[3];
    tw[14] = inv[1];
    uint64_t *o = out + ((int64_t)limb * Mp + m) * 2 * N;
    for (int c = 0; c < 2; ++c) {
        const double *s = lds + c * kLdsPoly4096 + T + (T >> 4);
        double v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = s[272 * e];
        gs16(v, tw, q, invq);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            double r = reduce(v[e], q, invq);                         // |r| <= q/2 + 1 (1/N is folded into the plaintexts)
            r = r < 0.0 ? r + q : r;                                   // canonical: an integer in [0, q)
            o[c * N + T + 256 * e] = (uint64_t)__double_as_longlong(r + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
        }
    }
}

}  // namespace

struct pcmv_plan {
    int64_t Mp, Kp, N;
    int L, device;
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
    p->ptn = nullptr; p->ctn = nullptr; p->fwd = nullptr; p->inv = nullptr; p->lc = nullptr;
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
        hipMalloc((void **)&p->lc, lc_bytes) != hipSuccess) {
        (void)hipGetLastError();
        rc = PCMM_ENOMEM;
    }
    p->bytes = ptn_bytes + ctn_bytes + 2 * tab_bytes + lc_bytes;
    if (rc == PCMM_OK) {
        if (hipMemcpyAsync(p->fwd, fwd.data(), tab_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipMemcpyAsync(p->inv, inv.data(), tab_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipMemcpyAsync(p->lc, lc.data(), lc_bytes, hipMemcpyHostToDevice, st) != hipSuccess)
            rc = PCMM_EDEVICE;
    }
    if (rc == PCMM_OK) {
        // the plaintexts into the NTT domain, once (the paper's model conversion for PCMv, Section 5.3)
        const int64_t polys = (int64_t)L * Mp * Kp;
        hipLaunchKernelGGL((ntt_kernel<1>), dim3((unsigned)polys), dim3(kThreads), (size_t)N * sizeof(double), st,
                           (const void *)pt_dev, p->ptn, p->fwd, p->lc, (int)N, Mp * Kp, N == kN4096 ? 1 : 0);
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
    hipLaunchKernelGGL((ntt_kernel<0>), dim3((unsigned)ct_polys), dim3(kThreads), (size_t)N * sizeof(double), st,
                       (const void *)ct_dev, plan->ctn, plan->fwd, plan->lc, N, plan->Kp * 2, N == kN4096 ? 1 : 0);
    if (hipGetLastError() != hipSuccess) return PCMM_EDEVICE;
    if (N == kN4096)
        hipLaunchKernelGGL(mac_intt4096_kernel, dim3((unsigned)((int64_t)plan->L * plan->Mp)), dim3(kThreads), 0, st, plan->ptn,
                           plan->ctn, out_dev, plan->inv, plan->lc, plan->Mp, (int)plan->Kp);
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
    delete plan;
}

}  // extern "C"
