// PCMM for short contractions (K <= 128) on MI355X (gfx950): C_j = W . A_j mod q_j where W is tall and
// A_j is very wide -- the shape of the plaintext-ciphertext attention products of Section 4.2, whose
// contraction runs over the head dimension.  Such a product writes far more than it reads (24 GiB of
// residues for the 4096 x 128 by 128 x 131072 case with six limbs), so it is bound by the stores and by
// the vector-ALU work of the modular reduction, not by the matrix cores.
//
// Design.  A work-group of four waves owns a strip of 64 columns of one limb; wave w owns columns
// 16w .. 16w+15 and keeps their digit fragments (both k-steps, all D digits: 2 D operand registers of
// 16 bytes) in registers for the whole kernel: the digit planes are read from memory exactly once.
// The work-group then walks down the rows of W.  W is shared by the four waves, so it is staged through
// LDS, four 16-row blocks at a time, double-buffered: the global loads of stage s+2 are issued before
// the results of stage s+1 are stored.  Per 16 x 16 output block a wave issues 2 D S MFMAs into
// E = D+S-1 accumulators (ordinary vector registers here: the compiler tracks the MFMA hazards, and the
// epilogue reads them without accumulator-register moves), reduces them and stores the block.  The
// kernel fits 128 registers per lane for most digit counts, so four waves share a SIMD: while one reduces and stores its
// block, the others keep the matrix cores busy.  (A variant that kept two accumulator sets per wave and
// interleaved the reduction of one block with the MFMAs of the next, at two waves per SIMD, measured
// 6 % slower; a fifth wave per work-group that does nothing but the W loads, 15 % slower.)
// Measured on the 4096 x 128 by 128 x 131072 case: the chip is power-limited here (shader clock about
// 1.5 GHz with matrix cores, double-precision vector work and 4 TB/s of stores all active); the output
// stores alone, in this pattern or any other, take 4.6 ms of the 6.0 ms.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>

#include "pcmm_device.hpp"
#include "pcmm_shortk.hpp"

using namespace pcmm_device;

namespace {

constexpr int RS = 4;   // 16-row blocks of W per LDS stage

struct KArgs {
    pcmm_shortk::Args a;
    int nstrips;          // 64-column strips per limb
    int mparts;           // parts the rows are cut into (work-groups per strip)
    int stages_per_part;  // LDS stages (RS row blocks each) per part
    int64_t per_xcd;      // work-groups per XCD
    int64_t total;        // L * nstrips * mparts
};

// MODE: the grouping reduce_f64 uses (0: groups of three accumulators; 2: groups of four, pairs joined in int32)
template <int D, int S, int MODE>
__global__ __launch_bounds__(256, 3) void gemm_shortk_kernel(KArgs ka)
{
    constexpr int E = D + S - 1;
    constexpr int CH = 2 * D * kFrag;             // one 32-column digit chunk of one k-step
    constexpr int NF = RS * S * 2;                // W fragments per stage: [row block][slice][k-step]
    constexpr int STAGE = NF * kFrag;
    constexpr int NLD = NF / 4;                   // fragments each wave moves per stage (one 16-byte unit per lane)
    static_assert(NF % 4 == 0, "a stage is moved by four waves, whole fragments each");
    const pcmm_shortk::Args &a = ka.a;

    __shared__ __attribute__((aligned(16))) int8_t lds[2][STAGE];

    // which strip: work-groups are dealt round-robin to the 8 XCDs; each XCD walks its own contiguous
    // range, parts of one strip next to each other (they read the same digit fragments)
    const int64_t bid = blockIdx.x;
    const int64_t t = (bid % kXcd) * ka.per_xcd + bid / kXcd;
    if (bid / kXcd >= ka.per_xcd || t >= ka.total) return;
    const int mpart = (int)(t % ka.mparts);
    const int strip = (int)((t / ka.mparts) % ka.nstrips);
    const int limb = (int)(t / ((int64_t)ka.mparts * ka.nstrips));

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t loff = (uint32_t)lane * 16u;

    // ---- this wave's digit fragments: column block nb of the limb, both k-steps, all digits
    const int nb = strip * 4 + wave;
    const bool active = (int64_t)nb * 16 < a.Ncols;        // wave-uniform
    v4i b[2][D];
    {
        const int ntile = nb >> 1, nt = nb & 1;
        const int8_t *base = a.Ad + (int64_t)limb * 2 * a.ntiles * CH;
        const uint32_t ad_limb_bytes = (uint32_t)((int64_t)2 * a.ntiles * CH);
        const __amdgpu_buffer_rsrc_t ars =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(base), 0, ad_limb_bytes, 0x00020000);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int d = 0; d < D; ++d) {
                // a column block beyond the limb's digit planes reads out of range: zeros
                const uint32_t off = active ? (uint32_t)(kb * a.ntiles + ntile) * (uint32_t)CH + (uint32_t)((nt * D + d) * kFrag)
                                            : ad_limb_bytes;
                b[kb][d] = (v4i)__builtin_amdgcn_raw_buffer_load_b128(ars, loff, (int)off, 0);
            }
    }

    // ---- W stages.  Fragment f = wave + 4 i of a stage is (row block f / (2S), slice (f / 2) % S, k-step f % 2)
    // and lies at byte f * 1024 of the stage in LDS.
    const uint32_t wp_bytes = (uint32_t)((int64_t)S * 2 * a.MB * kFrag);
    const __amdgpu_buffer_rsrc_t wrs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.Wp), 0, wp_bytes, 0x00020000);
    const int mb_first = mpart * ka.stages_per_part * RS;
    v4i wst[NLD];
    auto stage_load = [&](int s) {           // stage s of this part: global -> registers
        const int mb0 = mb_first + s * RS;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = wave + 4 * i;
            const int r = f / (2 * S), sl = (f / 2) % S, kb = f % 2;
            const int mb = mb0 + r;
            // row blocks beyond the packed matrix read out of range: zeros
            const uint32_t off = mb < a.MB ? (uint32_t)((sl * 2 + kb) * (int)a.MB + mb) * (uint32_t)kFrag : wp_bytes;
            wst[i] = (v4i)__builtin_amdgcn_raw_buffer_load_b128(wrs, loff, (int)off, 0);
        }
    };
    auto stage_store = [&](int buf) {        // registers -> LDS
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            *reinterpret_cast<v4i *>(&lds[buf][(wave + 4 * i) * kFrag + lane * 16]) = wst[i];
    };

    // the limb's constants, in scalar registers
    LimbConst lc;
    {
        constexpr int LCW = sizeof(LimbConst) / 4;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.lc + limb);
        uint32_t w[LCW];
#pragma unroll
        for (int i = 0; i < LCW; ++i) w[i] = __builtin_amdgcn_readfirstlane(src[i]);
        __builtin_memcpy(&lc, w, sizeof(lc));
    }

    uint64_t *Cl = a.C + (int64_t)limb * a.M * a.Ncols;
    const uint32_t c_rowbytes = (uint32_t)a.Ncols * 8u;
    const int64_t n = (int64_t)nb * 16 + (lane & 15);
    // lanes whose column lies beyond Ncols get an offset that is out of range for every row
    const uint32_t c_lane = n < a.Ncols ? (uint32_t)((lane >> 4) * 4) * c_rowbytes + (uint32_t)n * 8u : 0x80000000u;

    // one 16 x 16 block: acc[e] = sum over slices, k-steps and digits with d + slice = e
    auto compute = [&](v4i (&acc)[E], int buf, int r) {
        v4i wf[S][2];
#pragma unroll
        for (int sl = 0; sl < S; ++sl)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                wf[sl][kb] = *reinterpret_cast<const v4i *>(&lds[buf][((r * S + sl) * 2 + kb) * kFrag + lane * 16]);
        // consecutive MFMAs go to different accumulators; the first one of each starts from zero
#pragma unroll
        for (int sl = 0; sl < S; ++sl)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const int e = d + sl;
                    const bool first = kb == 0 && (sl == 0 || d == D - 1);
                    acc[e] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[sl][kb], b[kb][d], first ? (v4i){0, 0, 0, 0} : acc[e], 0, 0, 0);
                }
    };
    // reduce and store one block.  Accumulator register r of lane l is output row 4*(l/16)+r, column l%16.
    // Rows at or beyond M fall outside the buffer descriptor and are dropped by its range check.
    auto emit = [&](const v4i (&acc)[E], int mb) {
        // no branch here: a block beyond M gets an empty descriptor, which drops its stores
        const int64_t m0 = min((int64_t)mb * 16, a.M);
        const uint32_t rows_valid = (uint32_t)min((int64_t)16, a.M - m0);
        const __amdgpu_buffer_rsrc_t crs =
            __builtin_amdgcn_make_buffer_rsrc(Cl + m0 * a.Ncols, 0, rows_valid * c_rowbytes, 0x00020000);
        int avs[4][E];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int e = 0; e < E; ++e) avs[r][e] = acc[e][r];
        uint64_t res[4];
        reduce_f64<E, MODE, 4>(avs, lc.qd, lc.invq, res);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            // non-temporal: the output is written once and not read back by this kernel
            __builtin_amdgcn_raw_buffer_store_b64((v2u){(uint32_t)res[r], (uint32_t)(res[r] >> 32)}, crs,
                                                  c_lane + (uint32_t)r * c_rowbytes, 0, 2);
    };

    // ---- stage s is in LDS[s & 1] while stage s+1 travels global -> registers
    const int nst = ka.stages_per_part;
    v4i acc[E];
    stage_load(0);
    stage_store(0);
    __syncthreads();
    if (nst > 1) stage_load(1);
    for (int s = 0; s < nst; ++s) {
        const int cur = s & 1;
        const int mb0 = mb_first + s * RS;
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            compute(acc, cur, r);
            emit(acc, mb0 + r);
        }
        if (s + 1 < nst) {
            stage_store(cur ^ 1);            // every wave has left that buffer (barrier of stage s-1)
            __syncthreads();
            if (s + 2 < nst) stage_load(s + 2);
        }
    }
}

template <int D, int S>
hipError_t launch_ds(const KArgs &ka, int epi, int64_t grid, hipStream_t st)
{
    constexpr int E = D + S - 1;
    const dim3 g((unsigned)grid), b(256);
    if (epi == EPI_F64) {
        hipLaunchKernelGGL((gemm_shortk_kernel<D, S, 0>), g, b, 0, st, ka);
    } else if (epi == EPI_F64_G4P) {
        if constexpr (E >= 7) hipLaunchKernelGGL((gemm_shortk_kernel<D, S, 2>), g, b, 0, st, ka);
        else return hipErrorInvalidValue;
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

namespace pcmm_shortk {

bool covers(int D, int S, int epi, int64_t nkb)
{
    return nkb == 2 && D >= 4 && D <= 7 && (S == 1 || S == 2) && (epi == EPI_F64 || epi == EPI_F64_G4P);
}

hipError_t launch(const Args &a, int D, int S, int epi, hipStream_t st)
{
    if (!covers(D, S, epi, 2)) return hipErrorInvalidValue;
    KArgs ka;
    ka.a = a;
    ka.nstrips = (a.ntiles + 1) / 2;
    const int64_t stages = ((a.M + 15) / 16 + RS - 1) / RS;        // stages that hold a row of W
    // enough work-groups to balance 512 resident ones, as few as possible otherwise (a work-group reads
    // its digit fragments once, whatever number of rows it then covers)
    const int64_t strips = (int64_t)a.L * ka.nstrips;
    int64_t mparts = std::min<int64_t>(stages, std::max<int64_t>(1, (8192 + strips - 1) / strips));
    ka.stages_per_part = (int)((stages + mparts - 1) / mparts);
    ka.mparts = (int)((stages + ka.stages_per_part - 1) / ka.stages_per_part);
    ka.total = strips * ka.mparts;
    if (ka.total > 0x7fffff00LL) return hipErrorInvalidValue;
    ka.per_xcd = (ka.total + kXcd - 1) / kXcd;
    const int64_t grid = ka.per_xcd * kXcd;
#define PCMM_SHORTK_CASE(DD, SS) \
    if (D == DD && S == SS) return launch_ds<DD, SS>(ka, epi, grid, st);
    PCMM_SHORTK_CASE(4, 1)
    PCMM_SHORTK_CASE(5, 1)
    PCMM_SHORTK_CASE(6, 1)
    PCMM_SHORTK_CASE(7, 1)
    PCMM_SHORTK_CASE(4, 2)
    PCMM_SHORTK_CASE(5, 2)
    PCMM_SHORTK_CASE(6, 2)
    PCMM_SHORTK_CASE(7, 2)
#undef PCMM_SHORTK_CASE
    return hipErrorInvalidValue;
}

}  // namespace pcmm_shortk
