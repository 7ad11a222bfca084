"""Seeded synthetic inputs for the PCMM hot path (shared by the oracle tests and the HIP tests/bench).

This module holds NONE of the method's arithmetic: no matrix product, no digit
split, no modular reduction of a product.  It only names the workload shapes
and draws the operands:

  * W: the small-integer plaintext matrix of ``B = W.A`` (Section 5.1 of the
    paper; the shapes H=4096, I=14336, d=128 are those of Table "pipeline-time").
  * A_j: the residues modulo the RNS prime q_j of the coefficients of both
    ciphertext components (a, b) of R_Q^2 (Appendix A, Enc/Dec).  Ciphertext
    residues are indistinguishable from uniform, so they are drawn uniform in
    [0, q_j).
  * the primes q_j themselves: the largest primes of a given bit size with
    q = 1 (mod 2N), i.e. the NTT-friendly word-size primes a CKKS modulus chain
    is made of (Appendix A.2.1).

All draws come from a counter-based generator (the splitmix64 output function
of Steele/Lea/Flood applied to key + (index+1)*gamma), so that any element can
be produced on its own from (seed, stream, flat index): the host can draw a few
columns of a multi-GiB matrix, and the same numbers can be drawn on the GPU with
torch integer ops for the benchmark.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

STREAM_W = 1          # stream id of the plaintext matrix
STREAM_A0 = 2         # stream id of limb j is STREAM_A0 + j
_MAX_ATTEMPTS = 64    # rejection sampling rounds (acceptance > 1/2 per round)


# ----------------------------------------------------------------------------
# primes
# ----------------------------------------------------------------------------
def is_prime(n: int) -> bool:
    """Deterministic Miller-Rabin for n < 2^64 (first twelve prime bases)."""
    if n < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)
    for p in small:
        if n % p == 0:
            return n == p
    d, s = n - 1, 0
    while d % 2 == 0:
        d //= 2
        s += 1
    for a in small:
        x = pow(a, d, n)
        if x == 1 or x == n - 1:
            continue
        for _ in range(s - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def ntt_primes(bits: int, two_n: int, count: int) -> List[int]:
    """The `count` largest primes q with 2^(bits-1) < q < 2^bits and q = 1 mod two_n, descending."""
    out: List[int] = []
    q = ((1 << bits) - 1) // two_n * two_n + 1
    if q >= (1 << bits):
        q -= two_n
    while len(out) < count and q > (1 << (bits - 1)):
        if is_prime(q):
            out.append(q)
        q -= two_n
    if len(out) < count:
        raise ValueError("not enough primes of that size")
    return out


# ----------------------------------------------------------------------------
# workload presets
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    M: int            # rows of W (output channels)
    K: int            # contraction length (input channels)
    N: int            # ring degree; A has Ncols = 2N columns (a-coefficients, then b-coefficients)
    L: int            # number of RNS limbs
    prime_bits: int
    w_bits: int       # 8: W uniform in [-128,127];  16: W = rint(2^10 * N(0,1))
    seed: int = 0

    @property
    def Ncols(self) -> int:
        return 2 * self.N

    @property
    def primes(self) -> List[int]:
        return ntt_primes(self.prime_bits, 2 * self.N, self.L)

    @property
    def digits(self) -> int:
        """D of the throughput formula: signed 8-bit digits per residue."""
        return -(-self.prime_bits // 8)

    @property
    def slices(self) -> int:
        return self.w_bits // 8

    @property
    def modular_macs(self) -> int:
        return self.M * self.K * self.Ncols * self.L

    @property
    def int8_ops(self) -> int:
        return 2 * self.modular_macs * self.digits * self.slices


WORKLOADS = {
    w.name: w
    for w in (
        Workload("tiny", 128, 128, 1 << 12, 2, 36, 8),
        Workload("attn_proj", 4096, 4096, 1 << 14, 4, 36, 8),
        Workload("ffn_up_gate", 14336, 4096, 1 << 14, 4, 36, 8),
        Workload("ffn_down", 4096, 14336, 1 << 14, 3, 36, 8),
        Workload("wide_pc_attn", 4096, 128, 1 << 16, 6, 50, 16),
        # the paper's own storage format (Section 5.3): 16-bit weights under one modulus of about 64 bits
        Workload("attn_proj_w16_q62", 4096, 4096, 1 << 14, 1, 62, 16),
    )
}


# ----------------------------------------------------------------------------
# counter-based generator, numpy (host) flavour
# ----------------------------------------------------------------------------
def _mix_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int, attempt: int = 0) -> int:
    """64-bit key of one (seed, stream, rejection round)."""
    k = _mix_int(seed * _GAMMA + 0x5851F42D4C957F2D)
    k = _mix_int(k + stream * _GAMMA)
    return _mix_int(k + attempt * _GAMMA)


def draw_u64(key: int, index: np.ndarray) -> np.ndarray:
    """splitmix64 output number `index` of the stream seeded with `key` (elementwise, uint64)."""
    idx = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(key) + (idx + np.uint64(1)) * np.uint64(_GAMMA)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_C1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_C2)
        z = z ^ (z >> np.uint64(31))
    return z


def uniform_mod_q(seed: int, stream: int, index: np.ndarray, q: int, bits: int) -> np.ndarray:
    """Unbiased uniform draws in [0, q) at the given flat indices (rejection on `bits`-bit values)."""
    idx = np.asarray(index, dtype=np.uint64)
    out = draw_u64(stream_key(seed, stream, 0), idx) >> np.uint64(64 - bits)
    for attempt in range(1, _MAX_ATTEMPTS):
        bad = out >= np.uint64(q)
        if not bad.any():
            return out
        out[bad] = draw_u64(stream_key(seed, stream, attempt), idx[bad]) >> np.uint64(64 - bits)
    raise RuntimeError("rejection sampling did not terminate")


def gen_W(wl: Workload) -> np.ndarray:
    """The plaintext matrix of a workload: int8 (uniform) or int16 (rounded Gaussian, sigma = 2^10)."""
    n = wl.M * wl.K
    key = stream_key(wl.seed, STREAM_W)
    if wl.w_bits == 8:
        idx = np.arange(n, dtype=np.uint64)
        top = (draw_u64(key, idx) >> np.uint64(56)).astype(np.int16) - 128
        return top.astype(np.int8).reshape(wl.M, wl.K)
    if wl.w_bits == 16:
        idx = np.arange(n, dtype=np.uint64)
        u1 = ((draw_u64(key, 2 * idx) >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        u2 = ((draw_u64(key, 2 * idx + 1) >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)      # Box-Muller
        return np.rint(1024.0 * g).astype(np.int16).reshape(wl.M, wl.K)  # rint: ties to even
    raise ValueError("w_bits must be 8 or 16")


def gen_A_columns(wl: Workload, limb: int, cols: Sequence[int]) -> np.ndarray:
    """Columns `cols` of A_limb, shape [K, len(cols)], uint64; element (k, n) has flat index k*Ncols + n."""
    cols = np.asarray(cols, dtype=np.uint64)
    k = np.arange(wl.K, dtype=np.uint64)[:, None]
    idx = k * np.uint64(wl.Ncols) + cols[None, :]
    return uniform_mod_q(wl.seed, STREAM_A0 + limb, idx, wl.primes[limb], wl.prime_bits)


def gen_A(wl: Workload) -> np.ndarray:
    """All of A, shape [L, K, Ncols], uint64 (host).  Sized for the small workloads."""
    out = np.empty((wl.L, wl.K, wl.Ncols), dtype=np.uint64)
    idx = np.arange(wl.K * wl.Ncols, dtype=np.uint64)
    primes = wl.primes
    for j in range(wl.L):
        out[j] = uniform_mod_q(wl.seed, STREAM_A0 + j, idx, primes[j], wl.prime_bits).reshape(wl.K, wl.Ncols)
    return out


# ----------------------------------------------------------------------------
# the same draws with torch integer ops (runs on the GPU for the large workloads)
# ----------------------------------------------------------------------------
def _s64(c: int) -> int:
    """Two's-complement int64 value of a 64-bit pattern."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(z, s: int):
    return (z >> s) & ((1 << (64 - s)) - 1)


def _draw_u64_torch(key: int, index):
    """draw_u64 on an int64 torch tensor; the result holds the same 64-bit patterns (as int64)."""
    z = (index + 1) * _s64(_GAMMA) + _s64(key)
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def gen_A_limb_torch(wl: Workload, limb: int, device, chunk_rows: int = 0):
    """A_limb as an int64 torch tensor [K, Ncols] on `device` (values < 2^63, so int64 == uint64 bits)."""
    import torch

    q = wl.primes[limb]
    bits = wl.prime_bits
    out = torch.empty((wl.K, wl.Ncols), dtype=torch.int64, device=device)
    rows = chunk_rows or max(1, (1 << 26) // wl.Ncols)
    for r0 in range(0, wl.K, rows):
        r1 = min(wl.K, r0 + rows)
        idx = torch.arange(r0 * wl.Ncols, r1 * wl.Ncols, dtype=torch.int64, device=device)
        v = _lsr(_draw_u64_torch(stream_key(wl.seed, STREAM_A0 + limb, 0), idx), 64 - bits)
        for attempt in range(1, _MAX_ATTEMPTS):
            bad = v >= q
            if not bool(bad.any()):
                break
            redo = _lsr(_draw_u64_torch(stream_key(wl.seed, STREAM_A0 + limb, attempt), idx[bad]), 64 - bits)
            v[bad] = redo
        else:
            raise RuntimeError("rejection sampling did not terminate")
        out[r0:r1] = v.view(r1 - r0, wl.Ncols)
    return out


def gen_A_torch(wl: Workload, device):
    """All limbs of A as an int64 torch tensor [L, K, Ncols] on `device`."""
    import torch

    out = torch.empty((wl.L, wl.K, wl.Ncols), dtype=torch.int64, device=device)
    for j in range(wl.L):
        out[j] = gen_A_limb_torch(wl, j, device)
    return out
