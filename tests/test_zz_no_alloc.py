"""pcmm_run_noalloc (the entry point that allocates nothing) against pcmm_run, through the C ABI (GPU).

Both entry points run the same kernels; they differ in where the digit planes of A go (the plan's own
scratch, or the library's static buffer).  The bar is the one of every PCMM parity test: bit-exact.
This file is collected last on purpose: the round's GPU run stops at the first failure.
"""
import numpy as np
import pytest

import pcmm_inputs as pi

pytestmark = pytest.mark.gpu


def _both(W, A, primes, bits, dev):
    """C from pcmm_run and C from pcmm_run_noalloc for the same plan and input."""
    import torch

    import paper_2601_18511_amd as pkg

    L, K, Ncols = A.shape
    plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(dev), primes, bits, Ncols)
    A_dev = torch.from_numpy(A.view(np.int64)).to(dev)
    C_ref = torch.full((L, W.shape[0], Ncols), -1, dtype=torch.int64, device=dev)
    C_new = torch.full((L, W.shape[0], Ncols), -2, dtype=torch.int64, device=dev)
    pkg.pcmm_run(plan, A_dev, C_ref)
    pkg.pcmm_run_noalloc(plan, A_dev, C_new)
    torch.cuda.synchronize()
    pkg.pcmm_plan_destroy(plan)
    return C_ref.cpu().numpy().view(np.uint64), C_new.cpu().numpy().view(np.uint64)


def _case(rng, M, K, Ncols, bits, L, wbits):
    primes = pi.ntt_primes(bits, 1 << 10, L)
    if wbits == 8:
        W = rng.integers(-128, 128, size=(M, K), dtype=np.int64).astype(np.int8)
    else:
        W = rng.integers(-32768, 32640, size=(M, K), dtype=np.int64).astype(np.int16)
    A = np.stack([rng.integers(0, q, size=(K, Ncols), dtype=np.uint64) for q in primes])
    return W, A, primes


def test_two_calls_in_a_row_the_second_smaller(gpu_device):
    """The static buffer keeps the first call's digits; the second, smaller call must not see them."""
    from oracle import pcmm_oracle

    rng = np.random.default_rng(77)
    for shape in ((300, 1000, 1000, 36, 2, 8), (70, 100, 50, 50, 3, 16)):
        print("pcmm_run_noalloc case", shape, flush=True)
        W, A, primes = _case(rng, *shape)
        ref, new = _both(W, A, primes, shape[3], gpu_device)
        assert (new == ref).all(), int((new != ref).sum())
        assert (new == pcmm_oracle(W, A, primes)).all()


def test_tiny_workload(gpu_device):
    wl = pi.WORKLOADS["tiny"]
    ref, new = _both(pi.gen_W(wl), pi.gen_A(wl), wl.primes, wl.prime_bits, gpu_device)
    assert (new == ref).all()


def test_largest_input_that_fits_and_the_first_that_does_not(gpu_device):
    import torch

    import paper_2601_18511_amd as pkg

    rng = np.random.default_rng(78)
    limit = pkg.pcmm.NOALLOC_SCRATCH_BYTES
    K, D = 128, 5
    ncols_fit = limit // (K * D) // 32 * 32            # digit planes: K * Ncols (padded to 32) * D bytes
    assert K * ncols_fit * D <= limit < K * (ncols_fit + 32) * D
    W, A, primes = _case(rng, 16, K, ncols_fit, 36, 1, 8)
    print("pcmm_run_noalloc at the limit: Ncols", ncols_fit, flush=True)
    ref, new = _both(W, A, primes, 36, gpu_device)
    assert (new == ref).all()

    W, A, primes = _case(rng, 16, K, ncols_fit + 1, 36, 1, 8)
    plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), primes, 36, ncols_fit + 1)
    A_dev = torch.from_numpy(A.view(np.int64)).to(gpu_device)
    C_dev = torch.full((1, 16, ncols_fit + 1), -3, dtype=torch.int64, device=gpu_device)
    with pytest.raises(pkg.PcmmError) as e:
        pkg.pcmm_run_noalloc(plan, A_dev, C_dev)
    assert e.value.status == pkg.pcmm.PCMM_EUNSUPPORTED
    torch.cuda.synchronize()
    assert bool((C_dev == -3).all())                     # nothing was enqueued
    pkg.pcmm_run(plan, A_dev, C_dev)                     # the plan itself is fine
    torch.cuda.synchronize()
    assert bool((C_dev >= 0).all())
    pkg.pcmm_plan_destroy(plan)
