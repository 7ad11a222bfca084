"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI (GPU)."""
import random

import numpy as np
import pytest

import pcmm_inputs as pi

pytestmark = pytest.mark.gpu


def _run_gpu(W, A, primes, bits, dev):
    import torch

    import paper_2601_18511_amd as pkg

    L, K, Ncols = A.shape
    plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(dev), primes, bits, Ncols)
    A_dev = torch.from_numpy(A.view(np.int64)).to(dev)
    C_dev = torch.full((L, W.shape[0], Ncols), -1, dtype=torch.int64, device=dev)
    pkg.pcmm_run(plan, A_dev, C_dev)
    torch.cuda.synchronize()
    out = C_dev.cpu().numpy().view(np.uint64)
    digits = pkg.pcmm_plan_digits(plan)
    pkg.pcmm_plan_destroy(plan)
    return out, digits


def _rand_W(rng, M, K, bits):
    if bits == 8:
        return rng.integers(-128, 128, size=(M, K), dtype=np.int64).astype(np.int8)
    return rng.integers(-32768, 32640, size=(M, K), dtype=np.int64).astype(np.int16)


def _rand_A(rng, K, Ncols, primes):
    return np.stack([rng.integers(0, q, size=(K, Ncols), dtype=np.uint64) for q in primes])


def test_tiny_workload_bit_exact(gpu_device):
    from oracle import pcmm_oracle

    wl = pi.WORKLOADS["tiny"]
    W, A = pi.gen_W(wl), pi.gen_A(wl)
    got, digits = _run_gpu(W, A, wl.primes, wl.prime_bits, gpu_device)
    assert digits == 5
    want = pcmm_oracle(W, A, wl.primes)
    assert (got == want).all(), int((got != want).sum())


@pytest.mark.parametrize(
    "M,K,Ncols,bits,L,wbits",
    [
        (1, 1, 1, 36, 1, 8),
        (70, 100, 50, 36, 3, 8),          # ragged in every dimension, below one tile
        (300, 130, 1000, 36, 2, 8),       # several m-tiles and n-tiles with ragged tails, K tail
        (513, 200, 333, 36, 2, 8),
        (96, 128, 2048, 50, 2, 16),       # int16 W as two slices, 7 digits, two-part reduction
        (130, 70, 777, 50, 3, 16),
        (64, 64, 257, 50, 2, 8),
        (40, 300, 129, 62, 2, 8),         # 8 digits
        (33, 65, 100, 28, 2, 8),          # small primes: 4 digits
        (50, 64, 100, 44, 2, 16),         # 6 digits + 2 slices
        (260, 1000, 70, 36, 2, 8),        # many k-steps, ragged K tail (K not a multiple of 128)
        (64, 2049, 40, 50, 1, 16),        # odd K just past a k-step boundary
        (70, 640, 33, 55, 1, 8),          # 7 digits above 2^50: integer epilogue
        (40, 200, 50, 54, 2, 16),         # 7 digits, 2 slices, integer two-part epilogue
    ],
)
def test_random_shapes_bit_exact(gpu_device, M, K, Ncols, bits, L, wbits):
    from oracle import pcmm_oracle

    rng = np.random.default_rng(M * 1000 + K)
    primes = pi.ntt_primes(bits, 1 << 10, L)
    W = _rand_W(rng, M, K, wbits)
    A = _rand_A(rng, K, Ncols, primes)
    got, _ = _run_gpu(W, A, primes, bits, gpu_device)
    want = pcmm_oracle(W, A, primes)
    assert (got == want).all(), int((got != want).sum())
