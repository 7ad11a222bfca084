// Interface between pcmm.hip and pcmm_shortk.hip: the MFMA kernel for contractions of at most 128
// values of k (the wide plaintext x few ciphertexts shape of PC-attention, Section 4.2: K is the head
// dimension).  Host-side declarations only.
#ifndef PCMM_SHORTK_HPP
#define PCMM_SHORTK_HPP

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pcmm_host.hpp"

namespace pcmm_shortk {

// What one launch needs.  Wp and Ad are the plan's packed weights and one run's digit planes, in the
// layouts pack_w_kernel and split_kernel write (two k-steps of 64).
struct Args {
    const int8_t *Wp;                     // [S][2][MB][64][16]
    const int8_t *Ad;                     // [L][2][ntiles][2][D][64][16]
    uint64_t *C;                          // [L][M][Ncols]
    const pcmm_host::LimbConst *lc;       // [L]
    int64_t M, Ncols;
    int64_t MB;                           // 16-row blocks in Wp
    int ntiles;                           // 32-column tiles in Ad
    int L;
};

// true if launch() has a kernel for this plan: two k-steps, double-precision epilogue
bool covers(int D, int S, int epi, int64_t nkb);

// Enqueues the kernel on `st`.  hipErrorInvalidValue if covers() is false for these parameters.
hipError_t launch(const Args &a, int D, int S, int epi, hipStream_t st);

}  // namespace pcmm_shortk

#endif  // PCMM_SHORTK_HPP
