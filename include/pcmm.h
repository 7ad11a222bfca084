/*
 * pcmm.h - C ABI of the MI355X (gfx950) plaintext-ciphertext matrix multiplication library.
 *
 * The operation.  The paper's linear layers (QKV, O, gate/up, down projections) are evaluated as
 * PCMM, B = W.A with W a plaintext weight matrix and A encrypted activations (Section 5.1), through
 * the reduction of PCMM to clear matrix products on ciphertext data (Section 2.2, "PCMM from BLAS";
 * Section 3.2).  A ciphertext is a pair (a, b) in R_Q^2 and addition is component-wise (Appendix A),
 * so the clear product acts on the coefficients of both components alike.  With Q in RNS form, for
 * every limb j < L, row m < M and column n < Ncols this library computes
 *
 *     C_j[m][n] = ( sum_{k<K} W[m][k] * A_j[k][n] )  mod q_j ,   the representative in [0, q_j),
 *
 * exactly (bit-exact, deterministic).  Columns [0, Ncols/2) conventionally hold the coefficients of
 * the a-components and [Ncols/2, Ncols) those of the b-components; the library does not care.
 *
 * Method (the part the paper leaves to a GPU BLAS): every residue is split into D signed base-256
 * digits, W (int8, or int16 as two signed int8 slices) is multiplied with every digit plane by int8
 * MFMA with int32 accumulation, and the epilogue recombines the digit products and Barrett-reduces
 * modulo q_j.
 *
 * Conventions.  All matrices are dense row-major.  "device" pointers are HIP device memory on the
 * plan's device; "host" pointers are ordinary host memory.  The library never frees, reallocates or
 * keeps a caller's buffer.  No function throws or aborts; every failure is a status code.
 */
#ifndef PCMM_H
#define PCMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pcmm_plan pcmm_plan; /* opaque; owns packed W, per-limb constants and digit scratch */

typedef enum {
    PCMM_OK = 0,
    PCMM_EINVAL = 1,       /* null pointer, non-positive size, even or out-of-size prime, bad w_bits ... */
    PCMM_EUNSUPPORTED = 2, /* valid request outside what the kernels cover (see pcmm_plan_create) */
    PCMM_ENOMEM = 3,       /* host or device allocation failed */
    PCMM_EDEVICE = 4       /* a HIP call or kernel launch failed */
} pcmm_status;

/*
 * Build a plan for one weight matrix W and one list of primes (the paper's "model conversion"
 * step, Section 5.3: a layout-only transformation of the weights, done once).
 *
 *   out          receives the plan (set to NULL on failure)
 *   M, K         W is M x K:  M output channels, K input channels (contraction length),
 *                K at most 2^22 - 128
 *   Ncols        columns of every A_j and C_j (2N for ring degree N: both ciphertext components),
 *                at most 2^22; M at most 2^24
 *   L            number of RNS limbs, 1 <= L <= 64
 *   primes_host  [L] host array; each q_j odd with 2^(prime_bits-1) < q_j < 2^prime_bits
 *   prime_bits   size of the primes, 24 <= prime_bits <= 62
 *   w_bits       8: W is int8_t [M][K];  16: W is int16_t [M][K] with every entry in [-32768, 32639]
 *                (so that its balanced high byte fits int8)
 *   W_dev        device pointer to W, row-major; read during this call only, not kept
 *   device       HIP device ordinal the plan lives on
 *   stream       hipStream_t (NULL = default stream) used for the packing kernels; this call
 *                synchronises that stream before returning
 *
 * Every combination of 24..62-bit primes with int8 or int16 weights is covered (the paper stores 16-bit
 * weights under a modulus of about 64 bits, Section 5.3).  PCMM_EUNSUPPORTED when one limb of digit
 * planes (about K * Ncols * digits bytes) reaches 4 GiB, or one packed W slice 2 GiB, or the output has
 * more than 2^31 tiles (of at least 32 x 32 entries each).
 * The int32 accumulators hold a contraction over (w_bits/8)*K <= 131071; a longer K is cut into
 * ranges of 130944 (int8 W) or 65408 (int16 W) values of k, one MFMA kernel launch each, and every
 * launch after the first adds its result to C modulo q_j (the result is the same, bit for bit).
 * PCMM_EINVAL for an int16 W entry above 32639, and for everything listed under PCMM_EINVAL above.
 */
pcmm_status pcmm_plan_create(pcmm_plan **out, int64_t M, int64_t K, int64_t Ncols, int32_t L,
                             const uint64_t *primes_host, int32_t prime_bits, int32_t w_bits,
                             const void *W_dev, int32_t device, void *stream);

/*
 * Device bytes the plan owns: the converted weights (1 or 2 bytes per entry of W, where the paper's
 * converted PCMM tiles take 8, Section 5.3 and Table "model-conversion-memory"), the digit scratch of
 * one run (digits bytes per residue of A) and the per-limb constants.  0 for NULL.
 */
size_t pcmm_plan_workspace_bytes(const pcmm_plan *plan);

/*
 * Number of signed 8-bit digits each residue is split into (D), 0 for NULL.  It follows from the size
 * of the primes, which the paper chooses per level from its precision requirement (Section 3.1):
 * D is the smallest count with q_max - 1 + sum_{i<D} 128*256^i < 256^D (5 for 36-bit primes, 7 for
 * 50-bit, 8 up to 62-bit).
 */
int32_t pcmm_plan_digits(const pcmm_plan *plan);

/*
 * One PCMM step B = W.A (Section 5.1, first paragraph) as the clear product of Section 2.2 ("PCMM from
 * BLAS"), taken modulo every RNS prime: all L limbs, all Ncols columns (both components of the
 * ciphertexts of Appendix A.1, which add component-wise).
 *
 *   A_dev   device, [L][K][Ncols] uint64; A_dev[j] holds residues in [0, q_j) - a caller
 *           precondition, not checked; read only
 *   C_dev   device, [L][M][Ncols] uint64; every entry is written; must not overlap A_dev
 *   stream  hipStream_t the kernels are enqueued on (NULL = default stream)
 *
 * Asynchronous: returns after enqueueing; the caller synchronises the stream.  Two runs of the
 * SAME plan must not overlap in time (they share the plan's digit scratch); runs of different
 * plans may.  Launch failures are reported as PCMM_EDEVICE; faults inside a kernel surface at the
 * caller's next synchronisation.
 */
pcmm_status pcmm_run(const pcmm_plan *plan, const uint64_t *A_dev, uint64_t *C_dev, void *stream);

/*
 * Same operation as pcmm_run (Section 5.1, B = W.A), but brackets each kernel with HIP events on `stream`, synchronises, and
 * reports the kernel durations in milliseconds: ms_out[0] = digit-split kernel, ms_out[1] =
 * MFMA + epilogue kernel (all its launches together when K is cut into ranges).  ms_out is a host array of 2 floats.  For measurement harnesses.
 */
pcmm_status pcmm_run_profiled(const pcmm_plan *plan, const uint64_t *A_dev, uint64_t *C_dev,
                              void *stream, float *ms_out);

/*
 * pcmm_run for callers that cannot allocate device memory and want none allocated on their behalf
 * while they run: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same result (bit for bit) and same asynchrony as pcmm_run, but the digit planes of
 * A go to a buffer of PCMM_NOALLOC_SCRATCH_BYTES that is part of the library's device image (every
 * GPU the library runs on holds it until the process ends), not to the plan's own scratch.  The call
 * allocates and frees nothing, on the host or on the device.
 *
 * PCMM_EUNSUPPORTED if the plan's digit planes, L * ceil(K/128)*128 * ceil(Ncols/32)*32 * digits
 * bytes, exceed PCMM_NOALLOC_SCRATCH_BYTES; nothing is enqueued then.
 * All calls on one GPU share that GPU's buffer, whatever their plans: two calls that overlap in time
 * on one GPU (different streams, or threads) race.  Nothing is kept in the buffer between calls and
 * nothing in it has to be cleared: every call first rewrites all the bytes it later reads.
 */
#define PCMM_NOALLOC_SCRATCH_BYTES (64u << 20)
pcmm_status pcmm_run_noalloc(const pcmm_plan *plan, const uint64_t *A_dev, uint64_t *C_dev, void *stream);

/*
 * Measurement aid: runs a register-resident loop of v_mfma_i32_16x16x64_i8 with no memory traffic on
 * every CU of `device` (default stream, synchronous) and reports the sustained rate in TOP/s and the
 * shader clock in MHz seen by the kernel.  random_operands != 0 fills the operand registers with
 * pseudo-random bytes, 0 with zeros: the sustainable rate depends on data toggling.  This is the
 * "MFMA-only peak on this box" that measured PCMM rates are compared with.  Not an operation of the
 * paper: a measurement aid for benchmark harnesses.
 * iters: loop trips of 40 MFMAs per wave; 200000 runs for roughly 0.1 s.
 */
pcmm_status pcmm_mfma_probe(int32_t device, int32_t iters, int32_t random_operands, double *tops_out,
                            double *shader_mhz_out);

/*
 * Ring switching, the coefficient permutation either side of the PCMM (Section 3.3, the
 * coefficient-encoding case): after the key switch to a secret of the sub-ring R_{N'}, N' = N / k, every
 * component p (a' or b', one RNS limb) of a ciphertext over R_N is decomposed as
 *
 *     p(X) = sum_{j<k} p_j(X^k) X^j ,   p_j in R_{N'} :   p_j[i] = p[i*k + j] .
 *
 * pcmm_ring_decompose:  in_dev [npoly][N]  ->  out_dev [npoly][k][N/k]
 * pcmm_ring_compose:    in_dev [npoly][k][N/k]  ->  out_dev [npoly][N]      (the inverse map)
 *
 *   in_dev, out_dev   device, uint64 words (any content: the words are moved, not interpreted);
 *                     must not overlap; out_dev is written completely
 *   npoly             number of polynomials (limbs x components x ciphertexts), >= 1
 *   N, k              powers of two, 1 <= k <= N <= 2^24 (the paper uses N = 2^16 with N' = 2^12 or 2^8)
 *   device, stream    HIP device ordinal and hipStream_t (NULL = default stream); asynchronous
 *
 * No scratch memory, no plan.  The key switch that precedes the decomposition is not part of this
 * library.  PCMM_EINVAL for null or aliased pointers and sizes that are not powers of two;
 * PCMM_EUNSUPPORTED beyond 2^40 words or 2^31 - 1 tiles of 4096 words.
 */
pcmm_status pcmm_ring_decompose(const uint64_t *in_dev, uint64_t *out_dev, int64_t npoly, int64_t N, int64_t k,
                                int32_t device, void *stream);
pcmm_status pcmm_ring_compose(const uint64_t *in_dev, uint64_t *out_dev, int64_t npoly, int64_t N, int64_t k,
                              int32_t device, void *stream);

/*
 * Run-time plaintext rearrangement of the slot-encoded batch PCMM of PC-attention (Section 4.2, Eq. "pcmm";
 * Appendix E, Theorem 1).  For d x d matrices stored row after row, the depth-one PCMM needs, for every
 * baby step i < b and giant step j < g = d / b, the plaintext
 *
 *     pt_{A,i,j,l} = rot_R^{-l (i + j b) - j b} o rot_C^{i + j b}( S ) ,    S = tau^l o sigma(pt_A),
 *
 * where rot_C^k(M)[r][c] = M[r][c+k] and rot_R^s(M)[r][c] = M[r+s][c], indices modulo d.  Only S is kept
 * in memory; this call makes the rearranged plaintexts number k = i + j b for k_first <= k < k_first +
 * k_count from it:
 *
 *     out_dev[e][k - k_first][r][c] = S_dev[e][(r - l k - (k / b) b) mod d][(c + k) mod d] .
 *
 *   S_dev     device, [batch][d][d] uint64 words (any content: the words are moved, not interpreted)
 *   out_dev   device, [batch][k_count][d][d] uint64; written completely; must not overlap S_dev
 *   batch     number of stored matrices (heads x limbs x ...), >= 1
 *   d         matrix dimension, 1 <= d <= 32768 (the paper's head dimension is 128)
 *   ell       the power l of tau the output of the PCMM is to carry (any sign), |l| <= 2^31
 *   b         baby steps per giant step; must divide d
 *   k_first, k_count   the run of plaintexts to make, 0 <= k_first, k_first + k_count <= d
 *   device, stream     HIP device ordinal and hipStream_t (NULL = default stream); asynchronous
 *
 * No scratch memory, no plan.  The sigma and tau maps that produce S, and everything homomorphic
 * (rotations of ciphertexts, key switching), are not part of this library.  PCMM_EINVAL for null or
 * aliased pointers, sizes out of range and b not dividing d; PCMM_EUNSUPPORTED beyond 2^40 stored words
 * or 2^31 - 1 tiles of 4096 words.
 */
pcmm_status pcmm_slot_rearrange(const uint64_t *S_dev, uint64_t *out_dev, int64_t batch, int64_t d, int64_t ell,
                                int64_t b, int64_t k_first, int64_t k_count, int32_t device, void *stream);

/*
 * PCMv: the ring products of the decode-time plaintext-ciphertext matrix-vector multiplication.  In the decoding
 * stage the matrix-matrix products of the linear layers become matrix-vector products (Section 3.2, last paragraph),
 * evaluated at ring degree 4096 in coefficient encoding (Table "he-operators", row PCMv) with the converted weights
 * kept as plaintext polynomials in the NTT domain (Section 5.3, Table "model-conversion-memory").  A plaintext
 * polynomial multiplies both components of a ciphertext (Appendix A).  For plaintext polynomials pt[m][k] and
 * ciphertexts ct[k] = (a_k, b_k), for every RNS limb j, this part of the library computes
 *
 *     out_j[m][c] = sum_{k<Kp} pt[m][k] * ct_j[k][c]    in  Z_{q_j}[X] / (X^N + 1),    c in {a, b},
 *
 * coefficients in [0, q_j), exactly.  Which weights go into which plaintext polynomial, and the extraction and
 * repacking of the useful coefficients of the products, belong to the algorithm the paper adopts by reference
 * for PCMv and are not part of this library.
 */
typedef struct pcmv_plan pcmv_plan; /* opaque; owns the NTT-domain plaintexts, the twiddle tables and the NTT scratch */

/*
 * Build a PCMv plan: transforms the plaintext polynomials into the NTT domain, once (the model conversion of
 * Section 5.3 for the PCMv weights).
 *
 *   out          receives the plan (NULL on failure)
 *   Mp, Kp       pt is Mp x Kp polynomials: Mp output polynomials, Kp input ciphertexts; Kp <= 4096, Mp <= 2^24
 *   N            ring degree, a power of two, 2 <= N <= 4096 (the paper uses 4096 for PCMv)
 *   L            number of RNS limbs, 1 <= L <= 64
 *   primes_host  [L] host array; each q_j prime, q_j = 1 (mod 2N), 2^(prime_bits-1) < q_j < 2^prime_bits
 *   prime_bits   24 <= prime_bits <= 50 (the transforms compute in exact double-precision arithmetic)
 *   pt_dev       device, [Mp][Kp][N] int32_t: the plaintext polynomials' signed coefficients (coefficient domain),
 *                the same for every limb; read during this call only
 *   device, stream   HIP device ordinal and hipStream_t (NULL = default); the call synchronises the stream
 *
 * PCMM_EINVAL for null pointers, sizes out of range, N not a power of two, an even or wrong-size prime, a modulus
 * that is not 1 mod 2N or for which no primitive 2N-th root of unity is found (primality itself is the caller's
 * precondition); PCMM_EUNSUPPORTED for primes above 50 bits,
 * N above 4096, Kp above 4096 or more than 2^31 - 256 polynomials per limb set.
 */
pcmm_status pcmv_plan_create(pcmv_plan **out, int64_t Mp, int64_t Kp, int64_t N, int32_t L, const uint64_t *primes_host,
                             int32_t prime_bits, const int32_t *pt_dev, int32_t device, void *stream);

/* Device bytes the PCMv plan owns (8 Mp Kp N L for the NTT-domain plaintexts, plus tables and scratch). 0 for NULL. */
size_t pcmv_plan_workspace_bytes(const pcmv_plan *plan);

/*
 * One PCMv: out_j[m][c] = sum_k pt[m][k] * ct_j[k][c] in Z_{q_j}[X]/(X^N+1) (Sections 3.2 and 5.3, as above).
 *
 *   ct_dev   device, [L][Kp][2][N] uint64: limb j of ciphertext k, component a (index 0) then b (index 1), coefficient
 *            domain, residues in [0, q_j) - a caller precondition, not checked; read only
 *   out_dev  device, [L][Mp][2][N] uint64, coefficient domain; every entry written; must not overlap ct_dev
 *   stream   hipStream_t (NULL = default stream); asynchronous
 *
 * Two runs of the same plan must not overlap in time (they share the plan's NTT scratch).
 */
pcmm_status pcmv_run(const pcmv_plan *plan, const uint64_t *ct_dev, uint64_t *out_dev, void *stream);

/* Frees everything a PCMv plan owns.  NULL is ignored.  No run of the plan may still be in flight. */
void pcmv_plan_destroy(pcmv_plan *plan);

/*
 * Frees everything the plan owns (the converted weights of Section 5.3, the digit scratch, the
 * constants).  The caller makes sure no run of the plan is still in flight.  NULL is ignored.
 */
void pcmm_plan_destroy(pcmm_plan *plan);

/* Static, human-readable name of a status code (library housekeeping; no counterpart in the paper). */
const char *pcmm_status_str(pcmm_status s);

#ifdef __cplusplus
}
#endif
#endif /* PCMM_H */
