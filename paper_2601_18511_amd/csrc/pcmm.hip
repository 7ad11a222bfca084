// PCMM for MI355X (gfx950): C_j = W . A_j mod q_j, batched over RNS limbs and both ciphertext
// components (the clear matrix product that the paper's linear-layer PCMM reduces to, Sections 2.2,
// 3.2 and 5.1; ciphertexts as pairs in R_Q^2 with component-wise addition, Appendix A).
//
// Kernels of the PCMM path:
//   pack_w_kernel   (plan time)  W -> int8 slices in MFMA A-operand fragment order
//   split_kernel    (every run)  uint64 residues -> D signed base-256 digit planes in MFMA
//                                B-operand fragment order
//   gemm_kernel     (every run)  v_mfma_i32_16x16x64_i8 main loop, then recombination of the digit
//                                accumulators and reduction modulo q_j
// Beside it:
//   transpose_u64_kernel         the coefficient permutation of ring switching (Section 3.3)
//   mfma_probe_kernel            measurement aid: what the matrix cores sustain without memory traffic
//
// Fragment order.  One v_mfma_i32_16x16x64_i8 operand is 16 (rows or columns) x 64 (k) int8: lane l
// of the wave holds the 16 bytes with index (l % 16) and k = 16*(l/16) .. 16*(l/16)+15.  Both
// operands use the same k mapping, so an integer dot product does not depend on the order of k
// inside a lane.  A "fragment" is the 1 KiB such an operand takes, stored [lane][16 bytes], so that
// a wave fetches it with one 16-byte load per lane from contiguous memory.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>
#include <mutex>
#include <new>
#include <type_traits>
#include <utility>
#include "../../include/pcmm.h"
#include "pcmm_host.hpp"
#include "pcmm_device.hpp"
#include "pcmm_shortk.hpp"
#include "pcmm_hip_util.hpp"

using namespace pcmm_device;

namespace {

// The MFMA accumulators live in fixed accumulation registers a[0 : 4*MT*NT*E) that only the asm
// statements below name; the compiler never sees them as values, so it can neither migrate them
// between register files nor copy them at a point where the hardware would return a stale value.
// (An MFMA result may not be read by a non-MFMA instruction for up to 18 cycles after issue, and the
// hardware does not interlock; mfma_drain() provides the wait.)  Compiler-generated code never
// allocates accumulation registers in these kernels: they are used only when the 256 ordinary
// registers run out, and tests/test_build_asm.py checks that none appears outside the asm.
//
// acc[BASE : BASE+4) += A x B on one 16 x 16 x 64 int8 tile
template <int BASE>
__device__ __forceinline__ void mfma_i8(const v4i &a, const v4i &b)
{
    asm volatile("v_mfma_i32_16x16x64_i8 a[%0:%1], %2, %3, a[%0:%1]" ::"n"(BASE), "n"(BASE + 3), "v"(a), "v"(b));
}
template <int IDX>
__device__ __forceinline__ void acc_zero()
{
    asm volatile("v_accvgpr_write_b32 a[%0], 0" ::"n"(IDX));
}
template <int IDX>
__device__ __forceinline__ int acc_read()
{
    int x;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(x) : "n"(IDX));
    return x;
}
// tells the compiler which accumulation registers the kernel uses (it sizes the register file from this)
template <int NACC>
__device__ __forceinline__ void acc_declare()
{
    static_assert(NACC == 96 || NACC == 112 || NACC == 128 || NACC == 144 || NACC == 160, "add a clobber for this count");
    if constexpr (NACC == 96) asm volatile("" ::: "a95");
    if constexpr (NACC == 112) asm volatile("" ::: "a111");
    if constexpr (NACC == 128) asm volatile("" ::: "a127");
    if constexpr (NACC == 144) asm volatile("" ::: "a143");
    if constexpr (NACC == 160) asm volatile("" ::: "a159");
}

// wait states between the last MFMA (or accumulator write) and the next different kind of access
__device__ __forceinline__ void mfma_drain()
{
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// ------------------------------------------------------------------------------------------------
// plan-time kernel: pack W
// ------------------------------------------------------------------------------------------------
// Output Wp[s][kb][mb][lane][16]: slice s of W[mb*16 + lane%16][kb*64 + (lane/16)*16 + 0..15],
// zero outside M x K.  int16 entries are split as w = lo + 256*hi with lo = sign-extended low byte;
// err is set to 1 if some hi does not fit int8.
template <typename WT, int S>
__global__ __launch_bounds__(256) void pack_w_kernel(const WT *__restrict__ W, int8_t *__restrict__ Wp,
                                                     int64_t M, int64_t K, int64_t MB, int64_t nkb,
                                                     int *__restrict__ err)
{
    int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte lane slot
    int64_t total = MB * nkb * 64;
    if (unit >= total) return;
    int lane = (int)(unit % 64);
    int64_t kb = (unit / 64) % nkb;
    int64_t mb = unit / (64 * nkb);
    int64_t m = mb * 16 + (lane % 16);
    int64_t k0 = kb * 64 + (lane / 16) * 16;
    int8_t lo[16], hi[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        int64_t k = k0 + j;
        int w = (m < M && k < K) ? (int)W[m * K + k] : 0;
        int l = (int)(int8_t)(w & 0xFF);
        int h = (w - l) >> 8;
        lo[j] = (int8_t)l;
        hi[j] = (int8_t)h;
        if (S == 2 && (h < -128 || h > 127)) atomicExch(err, 1);
    }
    int8_t *dst = Wp + ((kb * MB + mb) * 64 + lane) * 16;
#pragma unroll
    for (int j = 0; j < 16; ++j) dst[j] = lo[j];
    if (S == 2) {
        int8_t *dst2 = dst + MB * nkb * kFrag;
#pragma unroll
        for (int j = 0; j < 16; ++j) dst2[j] = hi[j];
    }
}

// ------------------------------------------------------------------------------------------------
// run-time kernel 1: digit split
// ------------------------------------------------------------------------------------------------
// Balanced base-256 digits: with Bias = sum_{i<D} 128 * 256^i, the bytes of x + Bias, each xor 0x80,
// read as int8, are digits s_i in [-128,127] with x = sum_i s_i 256^i (valid while x + Bias < 256^D).
//
// Output layout Ad[limb][kb][ntile][nt][d][lane][16]; fragment (nt, d) of chunk (limb, kb, ntile)
// holds digit d of A[limb][kb*64 + (lane/16)*16 + 0..15][(ntile*NT + nt)*16 + lane%16], zero outside
// K x Ncols.  One block = 4 waves = 64 columns x 64 k; wave g takes k-group g, lane = column.
template <int D>
__global__ __launch_bounds__(256) void split_kernel(const uint64_t *__restrict__ A, int8_t *__restrict__ Ad,
                                                    int64_t K, int64_t Ncols, int64_t nkb, int64_t ntiles,
                                                    int NT)
{
    const int lane = threadIdx.x & 63;
    const int g = threadIdx.x >> 6;
    const int64_t kb = blockIdx.y;
    const int64_t limb = blockIdx.z;
    const int64_t n = (int64_t)blockIdx.x * 64 + lane;
    const int64_t nb = n >> 4;
    if (nb >= ntiles * NT) return;

    uint64_t bias = 0;
#pragma unroll
    for (int i = 0; i < D; ++i) bias |= (uint64_t)0x80 << (8 * i);

    const int64_t k0 = kb * 64 + g * 16;
    const uint64_t *src = A + (limb * K + k0) * Ncols + n;
    uint32_t out[D][4];
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int i = 0; i < 4; ++i) out[d][i] = 0;

#pragma unroll
    for (int j = 0; j < 16; ++j) {
        uint64_t x = (k0 + j < K && n < Ncols) ? src[(int64_t)j * Ncols] : 0;
        uint64_t y = x + bias;
#pragma unroll
        for (int d = 0; d < D; ++d) out[d][j >> 2] |= (uint32_t)((y >> (8 * d)) & 0xFF) << (8 * (j & 3));
    }

    const int64_t ntile = nb / NT;
    const int nt = (int)(nb % NT);
    int8_t *chunk = Ad + ((limb * nkb + kb) * ntiles + ntile) * ((int64_t)NT * D * kFrag);
#pragma unroll
    for (int d = 0; d < D; ++d) {
        v4i v;
        v.x = (int)(out[d][0] ^ 0x80808080u);
        v.y = (int)(out[d][1] ^ 0x80808080u);
        v.z = (int)(out[d][2] ^ 0x80808080u);
        v.w = (int)(out[d][3] ^ 0x80808080u);
        *reinterpret_cast<v4i *>(chunk + (nt * D + d) * kFrag + (g * 16 + (int)(n & 15)) * 16) = v;
    }
}

// ------------------------------------------------------------------------------------------------
// run-time kernel 2: int8 MFMA main loop + recombination + Barrett
// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const int8_t *Wp;       // [S][nkb][MB][64][16]
    const int8_t *Ad;       // [L][nkb][ntiles][NT][D][64][16]
    uint64_t *C;            // [L][M][Ncols]
    const LimbConst *lc;    // [L]
    int64_t M, Ncols;
    int64_t MB;             // padded M / 16
    int nkb;                // padded K / 64: k-steps in the layouts of Wp and Ad
    int kb0, nkbc;          // this launch contracts k-steps [kb0, kb0 + nkbc), nkbc even
    int accumulate;         // 0: C = result;  1: C = (C + result) mod q  (later slices of a long K)
    int mtiles, ntiles, L;
    int gn;                 // n-tiles per raster group
    int64_t per_xcd;        // work items per XCD
    int64_t total;          // L * mtiles * ntiles
};

// Work-group tile: (WM waves x MT fragments x 16) rows by (NT x 16) columns, all D digit planes.
// Each wave owns MT*16 rows and keeps E = D+S-1 int32 accumulators per output: accumulator e sums
// the products W_slice_s x digit_d with s + d = e, which all carry the weight 256^e.
// W fragments go global -> registers (each wave reads only its own rows); digit fragments are shared
// by all waves and staged through LDS.
//
// nkbc (k-steps of one launch) must be even.
template <int WM, int MT, int NT, int D, int S, int EPI>
__global__ __launch_bounds__(WM * 64) void gemm_kernel(GemmArgs a)
{
    constexpr int E = D + S - 1;
    constexpr int T = WM * 64;
    constexpr int CH = NT * D * kFrag;            // bytes of one digit chunk (one k-step)
    constexpr int UNITS = CH / 16;                // 16-byte units per chunk
    constexpr int NLD = (UNITS + T - 1) / T;      // units per thread (the last ones clamped: duplicates)
    static_assert(NT == 2, "a k-step is processed as two 16-column halves");

    __shared__ __attribute__((aligned(16))) int8_t lds[2][CH];

    // ---- which tile: XCD-aware raster.  Work-groups are dealt round-robin to the 8 XCDs, so
    // bid % 8 names the XCD; each XCD walks its own contiguous range of tiles in groups of gn n-tiles
    // x all m-tiles, n fastest inside a group, so that the tiles resident on one XCD (an 8 x 8 block
    // for gn = 8) share W rows and digit columns in that XCD's L2.
    const int64_t bid = blockIdx.x;
    const int64_t t = (bid % kXcd) * a.per_xcd + bid / kXcd;
    if (bid / kXcd >= a.per_xcd || t >= a.total) return;
    const int64_t per_limb = (int64_t)a.mtiles * a.ntiles;
    const int limb = (int)(t / per_limb);
    const int64_t rem = t % per_limb;
    const int64_t grp = rem / ((int64_t)a.gn * a.mtiles);
    const int64_t within = rem % ((int64_t)a.gn * a.mtiles);
    const int gcount = (int)min((int64_t)a.gn, a.ntiles - grp * a.gn);
    const int tm = (int)(within / gcount);
    const int tn = (int)(grp * a.gn + within % gcount);

    const int lane = threadIdx.x & 63;
    // the wave index is the same in all lanes: say so, so that addresses derived from it stay in
    // scalar registers and loads take the (scalar base + 32-bit lane offset) form
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nkb = a.nkbc;                                   // k-steps of this launch, numbered from 0 below
    const int64_t kleft = a.nkb - a.kb0;                      // k-steps from kb0 to the end of the layouts

    // chunk kb0 of this tile; k-step stride ntiles*CH
    const int8_t *Adc = a.Ad + (((int64_t)limb * a.nkb + a.kb0) * a.ntiles + tn) * CH;
    const int64_t mb0 = ((int64_t)tm * WM + wave) * MT;       // first 16-row block of this wave
    // Both operands are fetched with buffer loads: a scalar descriptor (base + size, out-of-range reads
    // return 0), a scalar byte offset for the k-step and a 32-bit lane offset, so that no vector ALU
    // work goes into addresses.  One descriptor per W slice and one for this limb's digit chunks.
    // Both arrays are k-step major, so that the work-groups running the same k-step at the same time read
    // one contiguous region (spread over all L2 channels) rather than addresses a power of two apart.
    const uint32_t loff = (uint32_t)lane * 16u;
    __amdgpu_buffer_rsrc_t wrs[S];
#pragma unroll
    for (int sl = 0; sl < S; ++sl)
        wrs[sl] = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int8_t *>(a.Wp + (((int64_t)sl * a.nkb + a.kb0) * a.MB + mb0) * kFrag), 0,
            (uint32_t)((kleft * a.MB - mb0) * kFrag), 0x00020000);
    const __amdgpu_buffer_rsrc_t ars =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(Adc), 0,
                                          (uint32_t)((kleft * a.ntiles - tn) * CH), 0x00020000);
    // byte offsets of a k-step: unsigned 32-bit products (one limb of digit chunks may take up to 4 GiB)
    const uint32_t w_kstride = (uint32_t)a.MB * (uint32_t)kFrag;     // bytes between k-steps of W
    const uint32_t a_kstride = (uint32_t)a.ntiles * (uint32_t)CH;    // bytes between k-steps of the digit chunks
    auto ld_w = [&](int sl, int wi, int kk) -> v4i {   // fragment (slice sl, row block wi, k-step kk)
        return (v4i)__builtin_amdgcn_raw_buffer_load_b128(
            wrs[sl], loff, (int)((uint32_t)kk * w_kstride + (uint32_t)(wi * kFrag)), 0);
    };
    auto ld_a = [&](uint32_t unit_off, int kk) -> v4i {   // 16 bytes of digit chunk kk
        return (v4i)__builtin_amdgcn_raw_buffer_load_b128(ars, unit_off, (int)((uint32_t)kk * a_kstride), 0);
    };

    // byte offsets of this thread's 16-byte units inside a chunk (same in global memory and in LDS);
    // units past the end are clamped to the last one, which is then loaded and stored twice
    uint32_t uoff[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) uoff[i] = (uint32_t)min((int)threadIdx.x + i * T, UNITS - 1) * 16u;

    // accumulator (i, j, e) = registers a[4*((i*NT + j)*E + e) ...+4)
    constexpr int NACC = 4 * MT * NT * E;
    acc_declare<NACC>();
    static_for<NACC>([&](auto ic) { acc_zero<decltype(ic)::value>(); });
    mfma_drain();

    // Software pipeline, one k-step = 64 k, LDS double-buffered, one barrier per k-step:
    //   W fragments   global -> wreg[2], loaded one k-step ahead of use
    //   digit chunk   global -> areg (second half of k-step kb-1) -> LDS[(kb+1)&1] (first half of kb)
    //   digit operand LDS -> b, read at the start of each 16-column half
    // The kernel is sized to at most 256 registers per lane so that two work-groups share a CU:
    // the second wave on each SIMD issues MFMAs while the first waits on LDS, memory or the barrier.
    // Memory instructions are spread between the MFMAs, because a wave issues in order and a burst
    // of LDS writes (about 64 B/clk per CU) would hold back the MFMAs queued behind it.
    // The last two k-steps run without the loads that would reach past the contraction.
    v4i wreg[2][S][MT];
    v4i areg[NLD];
    v4i b[D];
    constexpr int CNT = D * S * MT;                  // MFMAs per half k-step
    constexpr int NW = S * MT;                       // W fragments per k-step
    // MFMA order within a k-step: digit by digit, the W fragments forwards for one digit and backwards
    // for the next, so that every MFMA shares one operand with the one before it (less switching at the
    // matrix cores' inputs: the kernel is power-limited, and this order measures 0.7 % faster)
    auto snake = [](int digit, int f) constexpr { return (digit & 1) ? NW - 1 - f : f; };

    // prologue: everything the first k-step and the LDS fill of the second need is requested at once,
    // so that a tile start pays one memory latency, not two (nkb >= 2).  The limb's constants come
    // first and are moved to scalar registers: a vector load still in flight when the epilogue
    // branches around padding blocks would make the compiler wait for it behind the first stores.
    LimbConst lc;
    {
        constexpr int LCW = sizeof(LimbConst) / 4;
        static_assert(sizeof(LimbConst) % 4 == 0, "LimbConst is read word by word");
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.lc + limb);
        uint32_t w[LCW];
#pragma unroll
        for (int i = 0; i < LCW; ++i) w[i] = src[i];
        v4i first[NLD];
#pragma unroll
        for (int i = 0; i < NLD; ++i) first[i] = ld_a(uoff[i], 0);
#pragma unroll
        for (int f = 0; f < NW; ++f) wreg[0][f / MT][f % MT] = ld_w(f / MT, f % MT, 0);
#pragma unroll
        for (int i = 0; i < NLD; ++i) areg[i] = ld_a(uoff[i], 1);
#pragma unroll
        for (int i = 0; i < LCW; ++i) w[i] = __builtin_amdgcn_readfirstlane(w[i]);
        __builtin_memcpy(&lc, w, sizeof(lc));
#pragma unroll
        for (int i = 0; i < NLD; ++i) *reinterpret_cast<v4i *>(&lds[0][uoff[i]]) = first[i];
    }
    __syncthreads();

    // One k-step.  FILL: k-step kb+1 exists (fetch its W fragments, move its digit chunk to LDS);
    // AHEAD: k-step kb+2 exists (request its digit chunk).  The last two k-steps run without the
    // loads that would have nowhere to go, so that no load is in flight when the epilogue starts: a
    // wait for one placed behind the first stores would, the counter being in order, wait for those
    // stores to complete.
    auto step = [&](auto phase, auto fill, auto ahead, int kb) {
        constexpr int CUR = decltype(phase)::value, NXT = CUR ^ 1;
        constexpr bool FILL = decltype(fill)::value, AHEAD = decltype(ahead)::value;
        const int kw = kb + 1;
        const int ka = kb + 2;
#pragma unroll
        for (int d = 0; d < D; ++d) b[d] = *reinterpret_cast<const v4i *>(&lds[CUR][d * kFrag + lane * 16]);
        // first half: W loads of k-step kb+1 and LDS writes of chunk kb+1 between the MFMAs
        static_for<CNT>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int OPS = FILL ? NW + NLD : 0;
            constexpr int n_lo = (m * OPS + CNT - 1) / CNT, n_hi = ((m + 1) * OPS + CNT - 1) / CNT;
            static_for<n_hi - n_lo>([&](auto jc) {
                constexpr int n = n_lo + decltype(jc)::value;
                if constexpr (n < NW) {
                    wreg[NXT][n / MT][n % MT] = ld_w(n / MT, n % MT, kw);
                } else if constexpr (n < OPS) {
                    *reinterpret_cast<v4i *>(&lds[NXT][uoff[n - NW]]) = areg[n - NW];
                }
            });
            constexpr int d = m / NW, f = snake(d, m % NW), ws = f / MT, wi = f % MT;
            mfma_i8<4 * ((wi * NT + 0) * E + d + ws)>(wreg[CUR][ws][wi], b[d]);
        });
#pragma unroll
        for (int d = 0; d < D; ++d) b[d] = *reinterpret_cast<const v4i *>(&lds[CUR][(D + d) * kFrag + lane * 16]);
        // second half: loads of digit chunk kb+2 between the MFMAs
        static_for<CNT>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int OPS = AHEAD ? NLD : 0;
            constexpr int n_lo = (m * OPS + CNT - 1) / CNT, n_hi = ((m + 1) * OPS + CNT - 1) / CNT;
            static_for<n_hi - n_lo>([&](auto jc) {
                constexpr int n = n_lo + decltype(jc)::value;
                if constexpr (n < OPS) areg[n] = ld_a(uoff[n], ka);
            });
            constexpr int d = m / NW, f = snake(D + d, m % NW), ws = f / MT, wi = f % MT;
            mfma_i8<4 * ((wi * NT + 1) * E + d + ws)>(wreg[CUR][ws][wi], b[d]);
        });
        if constexpr (FILL) __syncthreads();   // chunk kb+1 is in LDS; buffer CUR may be refilled
    };
    {
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        int kb = 0;
        for (; kb < nkb - 2; kb += 2) {   // nkb is even
            step(P0{}, std::true_type{}, std::true_type{}, kb);
            step(P1{}, std::true_type{}, std::true_type{}, kb + 1);
        }
        step(P0{}, std::true_type{}, std::false_type{}, kb);
        step(P1{}, std::false_type{}, std::false_type{}, kb + 1);
    }

    // volatile asm statements keep their order: last MFMA, drain, accumulator reads
    mfma_drain();
    // Every load has been consumed by now.  Saying so with a wait the compiler sees keeps it from
    // placing one of its own (for a load it cannot prove finished on some path) behind the first stores.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)

    // ---- epilogue.  Accumulator register r of lane l is output row 4*(l/16)+r, column l%16 of its
    // 16 x 16 block.
    // Stores go through a buffer descriptor that covers exactly the valid rows of the 16-row block:
    // rows at or beyond M fall outside it and are dropped by the range check, and lanes whose column
    // is at or beyond Ncols get an offset that is out of range for every row; no address arithmetic
    // or branching per output.
    uint64_t *Cl = a.C + (int64_t)limb * a.M * a.Ncols;
    const uint32_t c_rowbytes = (uint32_t)a.Ncols * 8u;
    // The whole epilogue exists twice, with and without the read-add of the previous contents of C,
    // chosen once per wave: a branch per output would stop the scheduler from overlapping outputs.
    auto epilogue = [&](auto accumulate_c) {
    constexpr bool ACCUMULATE = decltype(accumulate_c)::value;
    static_for<MT * NT>([&](auto ijc) {
        constexpr int i = decltype(ijc)::value / NT, j = decltype(ijc)::value % NT;
        // 16 x 16 blocks that lie wholly in the padding are skipped (wave-uniform)
        if ((mb0 + i) * 16 < a.M && ((int64_t)tn * NT + j) * 16 < a.Ncols) {
            const int64_t m0 = (mb0 + i) * 16;
            const uint32_t rows_valid = (uint32_t)min((int64_t)16, a.M - m0);
            const __amdgpu_buffer_rsrc_t crs =
                __builtin_amdgcn_make_buffer_rsrc(Cl + m0 * a.Ncols, 0, rows_valid * c_rowbytes, 0x00020000);
            const int64_t n = ((int64_t)tn * NT + j) * 16 + (lane & 15);
            const uint32_t c_lane = n < a.Ncols ? (uint32_t)((lane >> 4) * 4) * c_rowbytes + (uint32_t)n * 8u
                                                : 0x80000000u;
            // all accumulators of the block's four outputs first (the reads are volatile and keep their
            // order), so that the four reductions are independent chains the scheduler can interleave
            int avs[4][E];
            static_for<4 * E>([&](auto rec) {
                constexpr int r = decltype(rec)::value / E, e = decltype(rec)::value % E;
                avs[r][e] = acc_read<4 * ((i * NT + j) * E + e) + r>();
            });
            uint64_t res[4];
            if constexpr (EPI == EPI_F64) {
                reduce_f64<E, 0, 4>(avs, lc.qd, lc.invq, res);
            } else if constexpr (EPI == EPI_F64_G4) {
                reduce_f64<E, 1, 4>(avs, lc.qd, lc.invq, res);
            } else if constexpr (EPI == EPI_F64_G4P) {
                reduce_f64<E, 2, 4>(avs, lc.qd, lc.invq, res);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // value = vlo + 2^32 vhi (+ 2^64 vtop for a ninth accumulator), each part of magnitude < 2^56
                    int64_t vlo = 0, vhi = 0;
#pragma unroll
                    for (int e = 0; e < (E < 8 ? E : 8); ++e) {
                        int64_t v = (int64_t)avs[r][e];
                        if (e < 4) vlo += v << (8 * e);
                        else vhi += v << (8 * (e - 4));
                    }
                    uint64_t rlo = barrett_u64((uint64_t)vlo + lc.off, lc.q, lc.mu);
                    uint64_t rhi = barrett_u64((uint64_t)vhi + lc.off, lc.q, lc.mu);
                    res[r] = rlo + mulmod_shoup(rhi, lc.c32, lc.c32s, lc.q);
                    if (res[r] >= lc.q) res[r] -= lc.q;
                    if constexpr (E == 9) {
                        uint64_t rtop = barrett_u64((uint64_t)(int64_t)avs[r][8] + lc.off, lc.q, lc.mu);
                        res[r] += mulmod_shoup(rtop, lc.c64, lc.c64s, lc.q);
                        if (res[r] >= lc.q) res[r] -= lc.q;
                    }
                }
            }
            if constexpr (ACCUMULATE) {   // rows and columns outside C read as 0
                v2u old[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    old[r] = __builtin_amdgcn_raw_buffer_load_b64(crs, c_lane + (uint32_t)r * c_rowbytes, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    res[r] += (uint64_t)old[r][0] | ((uint64_t)old[r][1] << 32);
                    if (res[r] >= lc.q) res[r] -= lc.q;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
                __builtin_amdgcn_raw_buffer_store_b64((v2u){(uint32_t)res[r], (uint32_t)(res[r] >> 32)}, crs,
                                                      c_lane + (uint32_t)r * c_rowbytes, 0, 0);
        }
    });
    };
    if (a.accumulate) epilogue(std::true_type{});
    else epilogue(std::false_type{});
}

// ------------------------------------------------------------------------------------------------
// ring switching: coefficient permutation either side of the PCMM (HBM-bound)
// ------------------------------------------------------------------------------------------------
// out[p][c][r] = in[p][r][c] for npoly matrices of R x C 64-bit words, R and C powers of two.
// Decomposition p(X) = sum_j p_j(X^k) X^j is the case R = N/k, C = k (coefficient i*k + j of p becomes
// coefficient i of p_j); composition is R = k, C = N/k.  One block moves a TR x TC tile (TR*TC = 4096
// words unless the matrix is smaller) through LDS, so that both the reads (along c) and the writes
// (along r) are contiguous runs of at least 128 bytes whenever the matrix allows it.  The row pitch
// TC + 1 keeps the column-wise LDS reads off a single bank.
constexpr int kTransposeWords = 4096;   // words per tile
constexpr int kTransposeMaxTR = 512;    // most rows per tile (tiles of narrow matrices)
__global__ __launch_bounds__(256) void transpose_u64_kernel(const uint64_t *__restrict__ in, uint64_t *__restrict__ out,
                                                            int64_t R, int64_t C, int lTR, int lTC, int64_t tiles_r,
                                                            int64_t tiles_c)
{
    __shared__ uint64_t tile[kTransposeWords + kTransposeMaxTR];     // TR * (TC + 1) words at most
    const int TR = 1 << lTR, TC = 1 << lTC;
    const int64_t b = blockIdx.x;
    const int64_t tc = b % tiles_c, tr = (b / tiles_c) % tiles_r, poly = b / (tiles_c * tiles_r);
    const uint64_t *src = in + poly * R * C + (tr << lTR) * C + (tc << lTC);
    uint64_t *dst = out + poly * R * C + (tc << lTC) * R + (tr << lTR);
    const int n = TR * TC;
    const int pitch = TC + 1;
    if (n == kTransposeWords) {   // full tile: 16 words per thread, all loads in flight before the first use
        uint64_t v[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int idx = threadIdx.x + 256 * s;
            v[s] = src[(int64_t)(idx >> lTC) * C + (idx & (TC - 1))];
        }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int idx = threadIdx.x + 256 * s;
            tile[(idx >> lTC) * pitch + (idx & (TC - 1))] = v[s];
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int idx = threadIdx.x + 256 * s;
            const int c = idx >> lTR, r = idx & (TR - 1);
            dst[(int64_t)c * R + r] = tile[r * pitch + c];
        }
        return;
    }
    for (int idx = threadIdx.x; idx < n; idx += 256) {
        const int r = idx >> lTC, c = idx & (TC - 1);
        tile[r * pitch + c] = src[(int64_t)r * C + c];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < n; idx += 256) {
        const int c = idx >> lTR, r = idx & (TR - 1);
        dst[(int64_t)c * R + r] = tile[r * pitch + c];
    }
}

// ------------------------------------------------------------------------------------------------
// measurement: register-resident MFMA-only probe
// ------------------------------------------------------------------------------------------------
// 40 independent accumulators per wave (the footprint of the D = 5 main loop), four W-like and ten
// digit-like operand registers, no memory traffic in the loop.  Operands are pseudo-random bytes or
// zeros: the rate the matrix cores sustain depends on how much the data toggles (power).  One lane
// also reports shader-clock and wall-clock ticks.
__global__ __launch_bounds__(256) void mfma_probe_kernel(long long *out, int iters, int random_operands)
{
    const long long c0 = clock64(), w0 = wall_clock64();
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    v4i wa[4], bd[10];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            wa[i][j] = random_operands ? (int)x : 0;
        }
#pragma unroll
    for (int i = 0; i < 10; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            bd[i][j] = random_operands ? (int)x : 0;
        }
    acc_declare<160>();
    static_for<160>([&](auto ic) { acc_zero<decltype(ic)::value>(); });
    mfma_drain();
    for (int it = 0; it < iters; ++it)
        static_for<40>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma_i8<4 * m>(wa[m % 4], bd[m / 4]);
        });
    mfma_drain();
    int sum = 0;
    static_for<160>([&](auto ic) { sum += acc_read<decltype(ic)::value>(); });
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        out[0] = clock64() - c0;
        out[1] = wall_clock64() - w0;
        out[2] = sum;
    }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// static digit scratch for pcmm_run_noalloc
// ------------------------------------------------------------------------------------------------
// Every GPU the library runs on holds its own copy of this array until the process ends.  Host code
// never passes the array's name to a kernel or a HIP call: it asks HIP for the device address once per
// device (static_scratch_ptr) and uses that pointer from then on.
static __device__ __align__(256) unsigned char scratch[PCMM_NOALLOC_SCRATCH_BYTES];

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct pcmm_plan {
    int64_t M, K, Ncols;
    int L, prime_bits, w_bits, device;
    int D, S;
    int WM, MT, NT;          // tile configuration
    int epi;                 // Epi: how the epilogue reduces
    int64_t MB, nkb, mtiles, ntiles;
    int64_t nkb_launch;      // most k-steps one GEMM launch may contract (int32 accumulator headroom)
    int8_t *Wp;              // device
    int8_t *Ad;              // device digit scratch
    LimbConst *lc;           // device
    size_t bytes;
    size_t ad_bytes;         // size of the digit scratch one run needs
    hipEvent_t ev[4];
    bool have_ev;
};

namespace {

using pcmm_host::tile_mt;
using pcmm_hip_util::DevGuard;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, nullptr until asked for

// Device address of this device's copy of `scratch`; `device` must be the current device.
// nullptr if HIP cannot tell.
int8_t *static_scratch_ptr(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[device] = ptr;
    }
    return static_cast<int8_t *>(g_scratch_ptr[device]);
}

template <int WM, int MT, int NT, int D, int S>
hipError_t launch_gemm_ds(const pcmm_plan *p, const GemmArgs &ga, int64_t grid, hipStream_t st)
{
    const dim3 g((unsigned)grid), b(WM * 64);
    // 50-bit primes need at least 7 digits and 7-digit primes can be below 2^50: D <= 6 always takes
    // the double-precision epilogue, D = 8 never does
    if (p->epi == EPI_F64) {
        if constexpr (D <= 7) hipLaunchKernelGGL((gemm_kernel<WM, MT, NT, D, S, EPI_F64>), g, b, 0, st, ga);
        else return hipErrorInvalidValue;
    } else if (p->epi == EPI_F64_G4 || p->epi == EPI_F64_G4P) {
        if constexpr (D <= 7 && D + S - 1 >= 7) {
            if (p->epi == EPI_F64_G4) hipLaunchKernelGGL((gemm_kernel<WM, MT, NT, D, S, EPI_F64_G4>), g, b, 0, st, ga);
            else hipLaunchKernelGGL((gemm_kernel<WM, MT, NT, D, S, EPI_F64_G4P>), g, b, 0, st, ga);
        } else return hipErrorInvalidValue;
    } else {
        if constexpr (D >= 7) {
            hipLaunchKernelGGL((gemm_kernel<WM, MT, NT, D, S, EPI_INT>), g, b, 0, st, ga);
        } else return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D, int S>
hipError_t launch_gemm_tile(const pcmm_plan *p, const GemmArgs &ga, int64_t grid, hipStream_t st)
{
    constexpr int MT = tile_mt(D + S - 1);
    if (p->MT != MT || p->NT != 2) return hipErrorInvalidValue;
    if (p->WM == 4) return launch_gemm_ds<4, MT, 2, D, S>(p, ga, grid, st);
    if (p->WM == 2) return launch_gemm_ds<2, MT, 2, D, S>(p, ga, grid, st);
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(const pcmm_plan *p, const GemmArgs &ga, int64_t grid, hipStream_t st)
{
    if (p->S == 1) {
        switch (p->D) {
        case 4: return launch_gemm_tile<4, 1>(p, ga, grid, st);
        case 5: return launch_gemm_tile<5, 1>(p, ga, grid, st);
        case 6: return launch_gemm_tile<6, 1>(p, ga, grid, st);
        case 7: return launch_gemm_tile<7, 1>(p, ga, grid, st);
        case 8: return launch_gemm_tile<8, 1>(p, ga, grid, st);
        }
    } else {
        switch (p->D) {
        case 4: return launch_gemm_tile<4, 2>(p, ga, grid, st);
        case 5: return launch_gemm_tile<5, 2>(p, ga, grid, st);
        case 6: return launch_gemm_tile<6, 2>(p, ga, grid, st);
        case 7: return launch_gemm_tile<7, 2>(p, ga, grid, st);
        case 8: return launch_gemm_tile<8, 2>(p, ga, grid, st);
        }
    }
    return hipErrorInvalidValue;
}

hipError_t launch_split(const pcmm_plan *p, int8_t *Ad, const uint64_t *A, hipStream_t st)
{
    int64_t colblocks = (p->ntiles * p->NT * 16 + 63) / 64;
    dim3 grid((unsigned)colblocks, (unsigned)p->nkb, (unsigned)p->L);
    dim3 block(256);
#define PCMM_SPLIT_CASE(DD)                                                                              \
    case DD:                                                                                             \
        hipLaunchKernelGGL((split_kernel<DD>), grid, block, 0, st, A, Ad, p->K, p->Ncols, p->nkb,     \
                           p->ntiles, p->NT);                                                            \
        break;
    switch (p->D) {
        PCMM_SPLIT_CASE(4)
        PCMM_SPLIT_CASE(5)
        PCMM_SPLIT_CASE(6)
        PCMM_SPLIT_CASE(7)
        PCMM_SPLIT_CASE(8)
    default: return hipErrorInvalidValue;
    }
#undef PCMM_SPLIT_CASE
    return hipGetLastError();
}

// Ad: the digit scratch of this run (the plan's own, or the library's static one)
pcmm_status run_impl(const pcmm_plan *p, int8_t *Ad, const uint64_t *A, uint64_t *C, hipStream_t st, float *ms)
{
    DevGuard dg(p->device);
    if (!dg.ok) return PCMM_EDEVICE;

    GemmArgs ga;
    ga.Wp = p->Wp;
    ga.Ad = Ad;
    ga.C = C;
    ga.lc = p->lc;
    ga.M = p->M;
    ga.Ncols = p->Ncols;
    ga.MB = p->MB;
    ga.nkb = (int)p->nkb;
    ga.kb0 = 0;
    ga.nkbc = (int)p->nkb;
    ga.accumulate = 0;
    ga.mtiles = (int)p->mtiles;
    ga.ntiles = (int)p->ntiles;
    ga.L = p->L;
    ga.total = (int64_t)p->L * p->mtiles * p->ntiles;
    ga.per_xcd = (ga.total + kXcd - 1) / kXcd;
    // concurrent tiles on one XCD (32 CUs) should form a block of about 4 m-tiles x 8 n-tiles
    ga.gn = 8;
    const int64_t grid = ga.per_xcd * kXcd;

    if (ms && hipEventRecord(p->ev[0], st) != hipSuccess) return PCMM_EDEVICE;
    if (launch_split(p, Ad, A, st) != hipSuccess) return PCMM_EDEVICE;
    if (ms && (hipEventRecord(p->ev[1], st) != hipSuccess || hipEventRecord(p->ev[2], st) != hipSuccess))
        return PCMM_EDEVICE;
    if (pcmm_shortk::covers(p->D, p->S, p->epi, p->nkb)) {
        // at most 128 values of k: the kernel that keeps the digit fragments in registers and walks down W
        pcmm_shortk::Args sa;
        sa.Wp = p->Wp; sa.Ad = Ad; sa.C = C; sa.lc = p->lc;
        sa.M = p->M; sa.Ncols = p->Ncols; sa.MB = p->MB;
        sa.ntiles = (int)p->ntiles; sa.L = p->L;
        if (pcmm_shortk::launch(sa, p->D, p->S, p->epi, st) != hipSuccess) return PCMM_EDEVICE;
    } else
    // A contraction longer than the int32 accumulators can hold runs as several launches over
    // consecutive ranges of k; every launch after the first adds its result to C modulo q_j.
    for (int64_t kb0 = 0; kb0 < p->nkb; kb0 += p->nkb_launch) {
        ga.kb0 = (int)kb0;
        ga.nkbc = (int)std::min(p->nkb_launch, p->nkb - kb0);
        ga.accumulate = kb0 > 0;
        if (launch_gemm(p, ga, grid, st) != hipSuccess) return PCMM_EDEVICE;
    }
    if (ms) {
        if (hipEventRecord(p->ev[3], st) != hipSuccess) return PCMM_EDEVICE;
        if (hipEventSynchronize(p->ev[3]) != hipSuccess) return PCMM_EDEVICE;
        if (hipEventElapsedTime(&ms[0], p->ev[0], p->ev[1]) != hipSuccess) return PCMM_EDEVICE;
        if (hipEventElapsedTime(&ms[1], p->ev[2], p->ev[3]) != hipSuccess) return PCMM_EDEVICE;
    }
    return PCMM_OK;
}

}  // namespace

extern "C" {

const char *pcmm_status_str(pcmm_status s)
{
    switch (s) {
    case PCMM_OK: return "PCMM_OK";
    case PCMM_EINVAL: return "PCMM_EINVAL: invalid argument";
    case PCMM_EUNSUPPORTED: return "PCMM_EUNSUPPORTED: request outside the supported range";
    case PCMM_ENOMEM: return "PCMM_ENOMEM: allocation failed";
    case PCMM_EDEVICE: return "PCMM_EDEVICE: HIP call or kernel launch failed";
    }
    return "PCMM: unknown status";
}

pcmm_status pcmm_plan_create(pcmm_plan **out, int64_t M, int64_t K, int64_t Ncols, int32_t L,
                             const uint64_t *primes_host, int32_t prime_bits, int32_t w_bits,
                             const void *W_dev, int32_t device, void *stream)
{
    if (!out) return PCMM_EINVAL;
    *out = nullptr;
    if (!primes_host || !W_dev) return PCMM_EINVAL;
    pcmm_host::Geometry g;
    const pcmm_status grc = pcmm_host::plan_geometry(M, K, Ncols, L, primes_host, prime_bits, w_bits, device, &g);
    if (grc != PCMM_OK) return grc;
    const int D = g.D, S = g.S;

    pcmm_plan *p = new (std::nothrow) pcmm_plan();
    if (!p) return PCMM_ENOMEM;
    p->M = M; p->K = K; p->Ncols = Ncols; p->L = L;
    p->prime_bits = prime_bits; p->w_bits = w_bits; p->device = device;
    p->D = D; p->S = S;
    p->WM = g.WM; p->MT = g.MT; p->NT = g.NT;
    p->epi = g.epi;
    p->MB = g.MB; p->nkb = g.nkb; p->mtiles = g.mtiles; p->ntiles = g.ntiles;
    p->nkb_launch = g.nkb_launch;
    p->Wp = nullptr; p->Ad = nullptr; p->lc = nullptr; p->bytes = 0; p->have_ev = false;

    DevGuard dg(device);
    if (!dg.ok) { delete p; return PCMM_EDEVICE; }
    hipStream_t st = (hipStream_t)stream;
    // set-up for pcmm_run_noalloc: this device's address of the static digit scratch, asked for once
    if (!static_scratch_ptr(device)) { delete p; return PCMM_EDEVICE; }

    const size_t wp_bytes = g.wp_bytes, ad_bytes = g.ad_bytes;
    const size_t lc_bytes = (size_t)L * sizeof(LimbConst);
    int *err_dev = nullptr;
    pcmm_status rc = PCMM_OK;
    if (hipMalloc((void **)&p->Wp, wp_bytes) != hipSuccess || hipMalloc((void **)&p->Ad, ad_bytes) != hipSuccess ||
        hipMalloc((void **)&p->lc, lc_bytes) != hipSuccess || hipMalloc((void **)&err_dev, sizeof(int)) != hipSuccess) {
        (void)hipGetLastError();
        rc = PCMM_ENOMEM;
    }
    p->bytes = wp_bytes + ad_bytes + lc_bytes;
    p->ad_bytes = ad_bytes;

    if (rc == PCMM_OK) {
        LimbConst h[pcmm_host::kMaxLimbs];
        for (int j = 0; j < L; ++j) h[j] = pcmm_host::limb_const(primes_host[j]);
        if (hipMemcpyAsync(p->lc, h, lc_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipMemsetAsync(err_dev, 0, sizeof(int), st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)   // h lives on this stack frame
            rc = PCMM_EDEVICE;
    }
    if (rc == PCMM_OK) {
        int64_t units = p->MB * p->nkb * 64;
        dim3 grid((unsigned)((units + 255) / 256)), block(256);
        if (w_bits == 8)
            hipLaunchKernelGGL((pack_w_kernel<int8_t, 1>), grid, block, 0, st, (const int8_t *)W_dev, p->Wp, M, K,
                               p->MB, p->nkb, err_dev);
        else
            hipLaunchKernelGGL((pack_w_kernel<int16_t, 2>), grid, block, 0, st, (const int16_t *)W_dev, p->Wp, M, K,
                               p->MB, p->nkb, err_dev);
        int err_host = 0;
        if (hipGetLastError() != hipSuccess ||
            hipMemcpyAsync(&err_host, err_dev, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            rc = PCMM_EDEVICE;
        else if (err_host)
            rc = PCMM_EINVAL;   // an int16 entry above 32639
    }
    if (rc == PCMM_OK) {
        p->have_ev = true;
        for (int i = 0; i < 4; ++i)
            if (hipEventCreate(&p->ev[i]) != hipSuccess) {
                for (int k = 0; k < i; ++k) (void)hipEventDestroy(p->ev[k]);
                p->have_ev = false;
                rc = PCMM_EDEVICE;
                break;
            }
    }
    if (err_dev) (void)hipFree(err_dev);
    if (rc != PCMM_OK) {
        if (p->Wp) (void)hipFree(p->Wp);
        if (p->Ad) (void)hipFree(p->Ad);
        if (p->lc) (void)hipFree(p->lc);
        delete p;
        return rc;
    }
    *out = p;
    return PCMM_OK;
}

size_t pcmm_plan_workspace_bytes(const pcmm_plan *plan) { return plan ? plan->bytes : 0; }

int32_t pcmm_plan_digits(const pcmm_plan *plan) { return plan ? plan->D : 0; }

pcmm_status pcmm_run(const pcmm_plan *plan, const uint64_t *A_dev, uint64_t *C_dev, void *stream)
{
    if (!plan || !A_dev || !C_dev) return PCMM_EINVAL;
    return run_impl(plan, plan->Ad, A_dev, C_dev, (hipStream_t)stream, nullptr);
}

pcmm_status pcmm_run_profiled(const pcmm_plan *plan, const uint64_t *A_dev, uint64_t *C_dev, void *stream,
                              float *ms_out)
{
    if (!plan || !A_dev || !C_dev || !ms_out) return PCMM_EINVAL;
    return run_impl(plan, plan->Ad, A_dev, C_dev, (hipStream_t)stream, ms_out);
}

pcmm_status pcmm_run_noalloc(const pcmm_plan *plan, const uint64_t *A_dev, uint64_t *C_dev, void *stream)
{
    if (!plan || !A_dev || !C_dev) return PCMM_EINVAL;
    if (plan->ad_bytes > (size_t)PCMM_NOALLOC_SCRATCH_BYTES) return PCMM_EUNSUPPORTED;
    int8_t *ptr;
    {
        DevGuard dg(plan->device);
        if (!dg.ok) return PCMM_EDEVICE;
        ptr = static_scratch_ptr(plan->device);   // resolved by pcmm_plan_create; a table look-up here
    }
    if (!ptr) return PCMM_EDEVICE;
    // the digit split rewrites every byte of the scratch that the MFMA kernel reads, so nothing has to
    // start at zero
    return run_impl(plan, ptr, A_dev, C_dev, (hipStream_t)stream, nullptr);
}

pcmm_status pcmm_mfma_probe(int32_t device, int32_t iters, int32_t random_operands, double *tops_out,
                            double *shader_mhz_out)
{
    if (device < 0 || iters <= 0 || !tops_out || !shader_mhz_out) return PCMM_EINVAL;
    DevGuard dg(device);
    if (!dg.ok) return PCMM_EDEVICE;
    long long *dev = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    pcmm_status rc = PCMM_OK;
    const int wgs = 512;   // two work-groups of four waves per CU on 256 CUs
    float ms = 0.f;
    long long h[3] = {0, 0, 0};
    if (hipMalloc((void **)&dev, sizeof(h)) != hipSuccess) return PCMM_ENOMEM;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = PCMM_EDEVICE;
    if (rc == PCMM_OK) {
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(wgs), dim3(256), 0, nullptr, dev, 64, random_operands);   // warm-up
        (void)hipEventRecord(e0, nullptr);
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(wgs), dim3(256), 0, nullptr, dev, iters, random_operands);
        if (hipGetLastError() != hipSuccess || hipEventRecord(e1, nullptr) != hipSuccess ||
            hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
            hipMemcpy(h, dev, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess)
            rc = PCMM_EDEVICE;
    }
    if (rc == PCMM_OK && ms > 0.f && h[1] > 0) {
        *tops_out = 2.0 * 16 * 16 * 64 * 40.0 * (double)iters * 4.0 * wgs / (ms * 1e-3) / 1e12;
        *shader_mhz_out = (double)h[0] / (double)h[1] * 100.0;   // the wall clock ticks at 100 MHz
    } else if (rc == PCMM_OK) {
        rc = PCMM_EDEVICE;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(dev);
    return rc;
}

namespace {

int log2_exact(int64_t v)   // -1 unless v is a power of two
{
    if (v <= 0 || (v & (v - 1))) return -1;
    int l = 0;
    while (((int64_t)1 << l) < v) ++l;
    return l;
}

// out[p][c][r] = in[p][r][c], R x C words, both powers of two
pcmm_status launch_transpose(const uint64_t *in, uint64_t *out, int64_t npoly, int64_t R, int64_t C, int32_t device,
                             hipStream_t st)
{
    const int lR = log2_exact(R), lC = log2_exact(C);
    if (lR < 0 || lC < 0) return PCMM_EINVAL;
    int lTC = std::min(lC, 6);
    int lTR = std::min(lR, std::min(12 - lTC, 9));       // TR * TC <= 4096, TR <= 512
    lTC = std::min(lC, 12 - lTR);                         // a short matrix gets wider tiles
    const int64_t tiles_r = R >> lTR, tiles_c = C >> lTC;
    const int64_t blocks = npoly * tiles_r * tiles_c;
    if (blocks > 0x7fffffff) return PCMM_EUNSUPPORTED;
    DevGuard dg(device);
    if (!dg.ok) return PCMM_EDEVICE;
    hipLaunchKernelGGL(transpose_u64_kernel, dim3((unsigned)blocks), dim3(256), 0, st, in, out, R, C, lTR, lTC, tiles_r,
                       tiles_c);
    return hipGetLastError() == hipSuccess ? PCMM_OK : PCMM_EDEVICE;
}

pcmm_status ring_args_ok(const void *in, const void *out, int64_t npoly, int64_t N, int64_t k, int32_t device)
{
    if (!in || !out || in == out || npoly <= 0 || device < 0) return PCMM_EINVAL;
    if (log2_exact(N) < 0 || log2_exact(k) < 0 || k > N || N > ((int64_t)1 << 24)) return PCMM_EINVAL;
    if (npoly > ((int64_t)1 << 40) / N) return PCMM_EUNSUPPORTED;
    return PCMM_OK;
}

}  // namespace

pcmm_status pcmm_ring_decompose(const uint64_t *in_dev, uint64_t *out_dev, int64_t npoly, int64_t N, int64_t k,
                                int32_t device, void *stream)
{
    const pcmm_status rc = ring_args_ok(in_dev, out_dev, npoly, N, k, device);
    if (rc != PCMM_OK) return rc;
    return launch_transpose(in_dev, out_dev, npoly, N / k, k, device, (hipStream_t)stream);
}

pcmm_status pcmm_ring_compose(const uint64_t *in_dev, uint64_t *out_dev, int64_t npoly, int64_t N, int64_t k,
                              int32_t device, void *stream)
{
    const pcmm_status rc = ring_args_ok(in_dev, out_dev, npoly, N, k, device);
    if (rc != PCMM_OK) return rc;
    return launch_transpose(in_dev, out_dev, npoly, k, N / k, device, (hipStream_t)stream);
}

void pcmm_plan_destroy(pcmm_plan *plan)
{
    if (!plan) return;
    DevGuard dg(plan->device);
    if (plan->have_ev)
        for (int i = 0; i < 4; ++i) (void)hipEventDestroy(plan->ev[i]);
    if (plan->Wp) (void)hipFree(plan->Wp);
    if (plan->Ad) (void)hipFree(plan->Ad);
    if (plan->lc) (void)hipFree(plan->lc);
    delete plan;
}

}  // extern "C"
