// Run-time plaintext rearrangement of the slot-encoded batch PCMM of PC-attention (Section 4.2) on
// MI355X (gfx950).
//
// The depth-one PCMM of Section 4.2 (Eq. "pcmm") needs, for every baby step i < b and giant step j < g
// (g b = d), the plaintext
//     pt_{A,i,j,l} = rot_R^{-l (i + j b) - j b} o rot_C^{i + j b}( tau^l o sigma(pt_A) ),
// and the paper keeps only S = tau^l o sigma(pt_A) in memory, making each pt_{A,i,j,l} from it when it is
// needed.  With the matrices stored row after row, rot_C^k(M)[r][c] = M[r][c+k] and
// rot_R^s(M)[r][c] = M[r+s][c] (indices modulo d), so with k = i + j b
//     pt_{A,i,j,l}[r][c] = S[(r - l k - j b) mod d][(c + k) mod d] :
// a two-dimensional cyclic shift of S.  The kernel below writes a run of consecutive k from one stored S
// per batch entry.  The 64-bit words are moved, not interpreted.
//
// HBM-bound: 8 bytes written per output word; S (8 d^2 bytes per batch entry) is read once from memory
// and again from the caches for every further k.  One thread moves 16 words, 256 words (2 KiB) per
// work-group and step, consecutive lanes on consecutive output words.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pcmm.h"
#include "pcmm_hip_util.hpp"

namespace {

constexpr int kTileWords = 4096;   // output words per work-group
constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void slot_rearrange_kernel(const uint64_t *__restrict__ S, uint64_t *__restrict__ out,
                                                                  uint32_t d, int64_t ell, uint32_t b, int64_t k_first,
                                                                  uint32_t k_count, uint32_t tiles_per_matrix)
{
    const uint64_t blk = blockIdx.x;
    const uint32_t tile = (uint32_t)(blk % tiles_per_matrix);
    const uint32_t t = (uint32_t)((blk / tiles_per_matrix) % k_count);
    const uint64_t e = blk / ((uint64_t)tiles_per_matrix * k_count);          // batch entry
    const int64_t k = k_first + t;
    const int64_t j = k / b;
    // row and column shifts, both in [0, d)
    int64_t sr64 = (-ell * k - j * (int64_t)b) % (int64_t)d;
    if (sr64 < 0) sr64 += d;
    const uint32_t sr = (uint32_t)sr64, sc = (uint32_t)(k % d);

    const uint32_t words = d * d;
    const uint64_t *src = S + e * words;
    uint64_t *dst = out + (e * k_count + t) * (uint64_t)words;
    // first word of this thread, then steps of 256 words: (row, column) advance by (256 / d, 256 % d)
    uint32_t w = tile * kTileWords + threadIdx.x;
    uint32_t r = w / d, c = w - r * d;
    const uint32_t step_r = kThreads / d, step_c = kThreads - step_r * d;
    uint64_t v[kTileWords / kThreads];
    uint32_t ws[kTileWords / kThreads];
#pragma unroll
    for (int s = 0; s < kTileWords / kThreads; ++s) {
        ws[s] = w;
        if (w < words) {
            uint32_t rr = r + sr, cc = c + sc;
            if (rr >= d) rr -= d;
            if (cc >= d) cc -= d;
            v[s] = src[rr * d + cc];
        }
        w += kThreads;
        r += step_r;
        c += step_c;
        if (c >= d) { c -= d; ++r; }
    }
#pragma unroll
    for (int s = 0; s < kTileWords / kThreads; ++s)
        if (ws[s] < words) dst[ws[s]] = v[s];
}

}  // namespace

extern "C" pcmm_status pcmm_slot_rearrange(const uint64_t *S_dev, uint64_t *out_dev, int64_t batch, int64_t d, int64_t ell,
                                           int64_t b, int64_t k_first, int64_t k_count, int32_t device, void *stream)
{
    if (!S_dev || !out_dev || S_dev == out_dev || device < 0) return PCMM_EINVAL;
    if (batch <= 0 || d <= 0 || b <= 0 || d % b != 0) return PCMM_EINVAL;
    if (k_first < 0 || k_count <= 0 || k_first + k_count > d) return PCMM_EINVAL;
    if (d > 32768 || ell > ((int64_t)1 << 31) || ell < -((int64_t)1 << 31)) return PCMM_EUNSUPPORTED;   // 32-bit word indices; l k fits 64 bits
    const int64_t words = d * d;
    const int64_t tiles = (words + kTileWords - 1) / kTileWords;
    if (batch > ((int64_t)1 << 40) / words) return PCMM_EUNSUPPORTED;
    const int64_t blocks = batch * k_count * tiles;
    if (blocks > 0x7fffffff) return PCMM_EUNSUPPORTED;
    pcmm_hip_util::DevGuard dg(device);
    if (!dg.ok) return PCMM_EDEVICE;
    hipLaunchKernelGGL(slot_rearrange_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, S_dev, out_dev,
                       (uint32_t)d, ell, (uint32_t)b, k_first, (uint32_t)k_count, (uint32_t)tiles);
    return hipGetLastError() == hipSuccess ? PCMM_OK : PCMM_EDEVICE;
}
