"""Parity of the ring-switch permutation kernels against the CPU oracle, word for word, through the C ABI (GPU)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _run(name, src_np, out_shape, N, k, dev):
    import torch

    import paper_2601_18511_amd as pkg

    src = torch.from_numpy(src_np.view(np.int64)).to(dev)
    dst = torch.full(out_shape, -1, dtype=torch.int64, device=dev)
    getattr(pkg, name)(src, dst, N, k)
    torch.cuda.synchronize()
    return dst.cpu().numpy().view(np.uint64)


@pytest.mark.parametrize(
    "npoly,N,k",
    [
        (1, 1, 1), (3, 2, 2), (5, 64, 1), (5, 64, 64), (2, 4096, 16), (2, 4096, 256), (3, 8192, 2),
        (7, 1024, 4), (1, 65536, 16),          # the paper's R_{2^16} -> R_{2^12}
        (2, 65536, 256),                       # R_{2^16} -> R_{2^8}, the PCMM ring degree
        (1, 1 << 18, 1 << 17), (1, 1 << 18, 2), (9, 512, 32),
    ],
)
def test_decompose_and_compose_match_the_oracle(gpu_device, npoly, N, k):
    from oracle import ring_compose, ring_decompose

    rng = np.random.default_rng(npoly * 1000 + N + k)
    p = rng.integers(0, 1 << 63, size=(npoly, N), dtype=np.uint64) * np.uint64(2) + np.uint64(1)   # all 64 bits in use
    want = ring_decompose(p, k)
    got = _run("pcmm_ring_decompose", p, (npoly, k, N // k), N, k, gpu_device)
    assert (got == want).all()
    parts = rng.integers(0, 1 << 63, size=(npoly, k, N // k), dtype=np.uint64)
    want = ring_compose(parts)
    got = _run("pcmm_ring_compose", parts, (npoly, N), N, k, gpu_device)
    assert (got == want).all()


def test_full_size_batch_round_trip_and_samples(gpu_device):
    """The batch bench.py times: 4 limbs x 2 components x 512 ciphertexts over R_{2^16}, k = 16.  Sampled
    polynomials against the oracle, the whole batch by the round trip compose(decompose(p)) = p."""
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import ring_decompose

    npoly, N, k = 4 * 2 * 512, 1 << 16, 16
    g = torch.Generator(device=gpu_device)
    g.manual_seed(5)
    p = torch.randint(-(1 << 62), 1 << 62, (npoly, N), dtype=torch.int64, device=gpu_device, generator=g)
    parts = torch.empty((npoly, k, N // k), dtype=torch.int64, device=gpu_device)
    back = torch.empty_like(p)
    pkg.pcmm_ring_decompose(p, parts, N, k)
    pkg.pcmm_ring_compose(parts, back, N, k)
    torch.cuda.synchronize()
    assert torch.equal(back, p)
    for i in (0, 1, 517, npoly - 1):
        want = ring_decompose(p[i].cpu().numpy(), k)
        assert (parts[i].cpu().numpy() == want).all()


def test_bad_arguments_are_status_codes(gpu_device):
    import torch

    import paper_2601_18511_amd as pkg

    x = torch.zeros(96, dtype=torch.int64, device=gpu_device)
    y = torch.zeros(96, dtype=torch.int64, device=gpu_device)
    for N, k in ((96, 3), (32, 64), (32, 0)):
        with pytest.raises((pkg.PcmmError, ValueError)):
            pkg.pcmm_ring_decompose(x, y, N, k)
    with pytest.raises(pkg.PcmmError) as e:
        pkg.pcmm_ring_decompose(x[:64], x[:64], 64, 8)      # aliased
    assert e.value.status == pkg.pcmm.PCMM_EINVAL
