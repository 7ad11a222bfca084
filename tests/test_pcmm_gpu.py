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
        (48, 192, 64, 24, 2, 16),         # smallest supported primes
        (20, 128, 40, 49, 2, 8),          # just below 2^50: double-precision epilogue with 7 digits
        (20, 128, 40, 51, 2, 8),          # just above: integer epilogue
        (100, 300, 70, 62, 2, 16),        # int16 W under 62-bit primes: 8 digits x 2 slices, nine accumulators
        (33, 1000, 129, 57, 1, 16),
        (260, 128, 64, 60, 2, 16),
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


@pytest.mark.parametrize(
    "M,K,Ncols,bits,L,wbits",
    [
        # contractions of at most 128 values of k take the kernel that keeps the digit fragments in
        # registers and walks down W in stages of 64 rows; 64-column strips, one wave per 16 columns
        (1000, 128, 64, 50, 2, 16),       # few strips: the rows are cut into several work-groups
        (1000, 128, 130, 36, 1, 8),       # an odd number of 32-column tiles: half a strip lies in the padding
        (65, 97, 1100, 50, 3, 16),        # one row past a stage; K tail inside the second k-step
        (63, 64, 17, 50, 2, 16),          # one k-step of real data, the second all padding
        (4096, 128, 96, 50, 1, 16),       # as many rows as the wide workload
        (200, 128, 300, 44, 2, 16),       # 6 digits x 2 slices: 7 accumulators, groups of three (q < 2^37 fails the G4 bound)
        (200, 100, 300, 49, 2, 8),        # 7 digits, 1 slice
        (129, 128, 200, 28, 2, 16),       # 4 digits, 2 slices
        (300, 33, 70, 40, 2, 8),          # 5 digits under a 40-bit prime
        (100, 128, 48, 41, 2, 16),        # 6 digits
    ],
)
def test_short_contractions_bit_exact(gpu_device, M, K, Ncols, bits, L, wbits):
    from oracle import pcmm_oracle

    rng = np.random.default_rng(M * 77 + K + Ncols)
    primes = pi.ntt_primes(bits, 1 << 10, L)
    W = _rand_W(rng, M, K, wbits)
    W[0, :] = -128 if wbits == 8 else -32768
    W[M - 1, :] = 127 if wbits == 8 else 32639
    A = _rand_A(rng, K, Ncols, primes)
    A[:, :, 0] = np.array(primes, dtype=np.uint64)[:, None] - np.uint64(1)
    got, _ = _run_gpu(W, A, primes, bits, gpu_device)
    want = pcmm_oracle(W, A, primes)
    assert (got == want).all(), int((got != want).sum())


def _digit_pattern_residues(q, bits, K, Ncols, rng):
    """Residues whose balanced base-256 digits sit at the extremes (+127 / -128 / 0 / -1 patterns)."""
    pats = []
    nbytes = (bits + 7) // 8
    for byte in (0x7F, 0x80, 0xFF, 0x00, 0x81, 0x7E):
        v = int.from_bytes(bytes([byte]) * nbytes, "little") & ((1 << bits) - 1)
        while v >= q:
            v >>= 1
        pats.append(v)
    pats += [0, 1, q - 1, q - 2, q // 2, q // 2 + 1, (1 << (bits - 1)) - 1, 1 << (bits - 1)]
    idx = rng.integers(0, len(pats), size=(K, Ncols))
    return np.array(pats, dtype=np.uint64)[idx]


@pytest.mark.parametrize("bits,wbits,K", [(36, 8, 14336), (50, 16, 1024), (62, 8, 2048), (36, 8, 131071),
                                          (50, 16, 65535), (24, 16, 65535),
                                          # the short-contraction epilogues and the sizes where they switch
                                          (50, 16, 254), (50, 16, 255), (50, 8, 509), (50, 8, 510),
                                          (50, 16, 8191), (50, 16, 8192), (50, 8, 16383), (50, 8, 16384),
                                          (40, 16, 200), (44, 16, 3000), (38, 16, 100), (50, 16, 128), (36, 8, 128), (49, 8, 64),
                                          (62, 16, 2048), (62, 16, 65535), (58, 16, 700)])
def test_adversarial_extremes_and_int32_headroom(gpu_device, bits, wbits, K):
    """All-(-128) / all-127 weight rows against extreme digit patterns: the int32 accumulators reach
    K * 2^14 (2^27.8 at K = 14336, 2^31 - 2^14 at the largest supported K)."""
    from oracle import pcmm_oracle

    rng = np.random.default_rng(bits * 7 + K)
    primes = pi.ntt_primes(bits, 1 << 12, 2)
    M, Ncols = 8, 48
    if wbits == 8:
        W = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
        W[0, :], W[1, :] = -128, 127
    else:
        W = rng.integers(-32768, 32640, size=(M, K)).astype(np.int16)
        W[0, :], W[1, :] = -32768, 32639
    W[2, :] = 0
    A = np.stack([_digit_pattern_residues(q, bits, K, Ncols, rng) for q in primes])
    A[:, :, 0] = np.array(primes, dtype=np.uint64)[:, None] - np.uint64(1)      # a column of q-1
    A[:, :, 1] = 0
    got, _ = _run_gpu(W, A, primes, bits, gpu_device)
    want = pcmm_oracle(W, A, primes)
    assert (got == want).all(), int((got != want).sum())
    assert (got[:, 2, :] == 0).all() and (got[:, :, 1] == 0).all()


@pytest.mark.parametrize("bits,wbits,K,launches", [(36, 8, 131072, 2), (36, 8, 130944 + 130, 2), (50, 16, 131000, 3),
                                                   (62, 8, 131073, 2), (54, 16, 65409, 2)])
def test_contraction_longer_than_one_launch_holds(gpu_device, bits, wbits, K, launches):
    """K beyond the int32 headroom of one launch (130944 values of k for int8 W, 65408 for int16 W):
    the MFMA kernel runs once per range of k and adds modulo q.  Extreme weight rows and digit
    patterns, so that the accumulators of the full ranges reach their largest magnitude."""
    from oracle import pcmm_oracle

    per_launch = 130944 if wbits == 8 else 65408
    assert -(-K // per_launch) == launches
    rng = np.random.default_rng(bits * 11 + K)
    primes = pi.ntt_primes(bits, 1 << 12, 2)
    M, Ncols = 20, 40
    if wbits == 8:
        W = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
        W[0, :], W[1, :] = -128, 127
    else:
        W = rng.integers(-32768, 32640, size=(M, K)).astype(np.int16)
        W[0, :], W[1, :] = -32768, 32639
    W[2, :] = 0
    W[3, :per_launch] = 0                                # only the later ranges contribute to row 3
    W[4, per_launch:] = 0                                # only the first range contributes to row 4
    A = np.stack([_digit_pattern_residues(q, bits, K, Ncols, rng) for q in primes])
    nbytes = (bits + 7) // 8
    for j, q in enumerate(primes):
        A[j, :, 0] = q - 1
        v = int.from_bytes(bytes([0x80]) * nbytes, "little") & ((1 << bits) - 1)   # digits all -128
        while v >= q:
            v >>= 1
        A[j, :, 2] = v
    A[:, :, 1] = 0
    got, _ = _run_gpu(W, A, primes, bits, gpu_device)
    want = pcmm_oracle(W, A, primes)
    assert (got == want).all(), int((got != want).sum())
    assert (got[:, 2, :] == 0).all() and (got[:, :, 1] == 0).all()


def test_closed_forms_on_the_gpu(gpu_device):
    rng = np.random.default_rng(3)
    primes = pi.ntt_primes(36, 1 << 13, 2)
    K, Ncols = 192, 100
    A = _rand_A(rng, K, Ncols, primes)
    eye = np.eye(K, dtype=np.int8)
    got, _ = _run_gpu(eye, A, primes, 36, gpu_device)
    assert (got == A).all()
    got, _ = _run_gpu((-eye).astype(np.int8), A, primes, 36, gpu_device)
    for j, q in enumerate(primes):
        assert (got[j] == (np.uint64(q) - A[j]) % np.uint64(q)).all()
    W = rng.integers(-128, 128, size=(70, K)).astype(np.int8)
    ones = np.ones((2, K, Ncols), dtype=np.uint64)
    got, _ = _run_gpu(W, ones, primes, 36, gpu_device)
    for j, q in enumerate(primes):
        want = np.array([int(r) % q for r in W.astype(np.int64).sum(axis=1)], dtype=np.uint64)
        assert (got[j] == want[:, None]).all()


def test_block_identity_on_the_gpu(gpu_device):
    """B^(u) = sum_v W^(u,v) A^(v) mod q (Section 5.1): split K in 2 and M in 2, partial products on the GPU."""
    rng = np.random.default_rng(5)
    primes = pi.ntt_primes(36, 1 << 13, 2)
    M, K, Ncols = 192, 640, 96
    W = _rand_W(rng, M, K, 8)
    A = _rand_A(rng, K, Ncols, primes)
    full, _ = _run_gpu(W, A, primes, 36, gpu_device)
    qs = np.array(primes, dtype=np.uint64)[:, None, None]
    for u in range(2):
        acc = np.zeros((2, M // 2, Ncols), dtype=np.uint64)
        for v in range(2):
            part, _ = _run_gpu(np.ascontiguousarray(W[u * 96:(u + 1) * 96, v * 320:(v + 1) * 320]),
                               np.ascontiguousarray(A[:, v * 320:(v + 1) * 320, :]), primes, 36, gpu_device)
            acc = (acc + part) % qs
        assert (acc == full[:, u * 96:(u + 1) * 96, :]).all()


def test_plan_reuse_and_two_plans_interleaved(gpu_device):
    """One plan run on two different inputs, and a second plan in between: scratch is per plan."""
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import pcmm_oracle

    rng = np.random.default_rng(8)
    primes = pi.ntt_primes(36, 1 << 13, 2)
    W1, W2 = _rand_W(rng, 100, 256, 8), _rand_W(rng, 60, 128, 8)
    A1a, A1b, A2 = _rand_A(rng, 256, 300, primes), _rand_A(rng, 256, 300, primes), _rand_A(rng, 128, 40, primes)
    p1 = pkg.pcmm_plan_create(torch.from_numpy(W1).to(gpu_device), primes, 36, 300)
    p2 = pkg.pcmm_plan_create(torch.from_numpy(W2).to(gpu_device), primes, 36, 40)
    assert pkg.pcmm_plan_workspace_bytes(p1) > 0

    def run(plan, A, M):
        A_dev = torch.from_numpy(A.view(np.int64)).to(gpu_device)
        C_dev = torch.empty((2, M, A.shape[2]), dtype=torch.int64, device=gpu_device)
        pkg.pcmm_run(plan, A_dev, C_dev)
        torch.cuda.synchronize()
        return C_dev.cpu().numpy().view(np.uint64)

    r1a = run(p1, A1a, 100)
    r2 = run(p2, A2, 60)
    r1b = run(p1, A1b, 100)
    ms = pkg.pcmm_run_profiled(p1, torch.from_numpy(A1a.view(np.int64)).to(gpu_device),
                               torch.empty((2, 100, 300), dtype=torch.int64, device=gpu_device))
    assert ms[0] > 0 and ms[1] > 0
    assert (r1a == pcmm_oracle(W1, A1a, primes)).all()
    assert (r1b == pcmm_oracle(W1, A1b, primes)).all()
    assert (r2 == pcmm_oracle(W2, A2, primes)).all()
    pkg.pcmm_plan_destroy(p1)
    pkg.pcmm_plan_destroy(p2)


def test_int16_out_of_range_and_bad_arguments_are_status_codes(gpu_device):
    import torch

    import paper_2601_18511_amd as pkg

    primes = pi.ntt_primes(50, 1 << 12, 2)
    W = np.zeros((4, 8), dtype=np.int16)
    W[3, 7] = 32640                                   # high byte would be +128
    with pytest.raises(pkg.PcmmError) as e:
        pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), primes, 50, 16)
    assert e.value.status == pkg.pcmm.PCMM_EINVAL
    W[3, 7] = 32639
    plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), primes, 50, 16)
    pkg.pcmm_plan_destroy(plan)
    W8 = torch.zeros((4, 8), dtype=torch.int8, device=gpu_device)
    for bad_primes, bits in (([primes[0] + 1], 50), ([primes[0]], 49), ([(1 << 50) + 1], 50)):
        with pytest.raises(pkg.PcmmError) as e:
            pkg.pcmm_plan_create(W8, bad_primes, bits, 16)
        assert e.value.status == pkg.pcmm.PCMM_EINVAL
    W16 = torch.zeros((4, 8), dtype=torch.int16, device=gpu_device)
    plan = pkg.pcmm_plan_create(W16, pi.ntt_primes(60, 1 << 12, 1), 60, 16)   # 8 digits + 2 slices: 9 accumulators
    assert pkg.pcmm_plan_digits(plan) == 8
    pkg.pcmm_plan_destroy(plan)


def test_gpu_input_generator_matches_host_generator(gpu_device):
    wl = pi.Workload("g", 8, 96, 256, 2, 36, 8, seed=3)
    ref = pi.gen_A(wl)
    got = pi.gen_A_torch(wl, gpu_device).cpu().numpy().view(np.uint64)
    assert (ref == got).all()


def test_mfma_probe_reports_a_plausible_rate(gpu_device):
    import paper_2601_18511_amd as pkg

    tops, mhz = pkg.pcmm_mfma_probe(0, 20000, True)
    assert 1000.0 < tops < 5200.0 and 500.0 < mhz < 2600.0
    tops0, mhz0 = pkg.pcmm_mfma_probe(0, 20000, False)
    assert tops0 >= 0.9 * tops


def test_pcmm_run_inside_a_hip_graph_replays_correctly(gpu_device):
    """pcmm_run only enqueues kernels (no allocation, no memset, no synchronisation), so it can be
    captured; every replay, with eager work and synchronisations in between, must match the oracle."""
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import pcmm_oracle

    rng = np.random.default_rng(77)
    primes = pi.ntt_primes(36, 1 << 13, 2)
    W = _rand_W(rng, 130, 320, 8)
    plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), primes, 36, 200)
    A_dev = torch.zeros((2, 320, 200), dtype=torch.int64, device=gpu_device)
    C_dev = torch.zeros((2, 130, 200), dtype=torch.int64, device=gpu_device)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pkg.pcmm_run(plan, A_dev, C_dev)          # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pkg.pcmm_run(plan, A_dev, C_dev)          # current stream is the capture stream here
    for rep in range(3):
        A = _rand_A(rng, 320, 200, primes)
        A_dev.copy_(torch.from_numpy(A.view(np.int64)))
        C_dev.fill_(-1)                            # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = C_dev.cpu().numpy().view(np.uint64)
        assert (got == pcmm_oracle(W, A, primes)).all(), rep
    pkg.pcmm_plan_destroy(plan)


def test_seeded_sweep_of_small_shapes(gpu_device):
    """Sixty seeded shapes over every digit count, both weight widths and every epilogue variant, ragged in all
    three dimensions, several with a single row, column or k."""
    from oracle import pcmm_oracle

    rnd = random.Random(20260118)
    cases = []
    for bits in (24, 28, 31, 33, 36, 40, 41, 47, 48, 49, 50, 51, 55, 56, 57, 62):
        for wbits in (8, 16):
            digits = next(d for d in range(1, 9) if (1 << bits) - 2 + sum(0x80 << (8 * i) for i in range(d)) < 1 << (8 * d))
            M = rnd.choice((1, 7, 16, 33, 64, 100, 129, 257))
            K = rnd.choice((1, 5, 63, 64, 65, 127, 128, 129, 255, 300, 513, 700))
            Ncols = rnd.choice((1, 2, 15, 16, 17, 31, 32, 33, 63, 100, 257))
            cases.append((M, K, Ncols, bits, rnd.choice((1, 2, 3)), wbits))
    rnd.shuffle(cases)
    assert len(cases) >= 28
    extra = [(rnd.choice((5, 80, 300)), rnd.choice((1100, 2500, 9000, 17000)), rnd.choice((3, 40, 70)), b, 1, w)
             for b, w in ((36, 8), (50, 16), (50, 8), (44, 16), (62, 8), (54, 16))]   # longer contractions
    for M, K, Ncols, bits, L, wbits in cases + extra:
        rng = np.random.default_rng(M * 7919 + K * 31 + Ncols)
        primes = pi.ntt_primes(bits, 1 << 8, L)
        W = _rand_W(rng, M, K, wbits)
        A = _rand_A(rng, K, Ncols, primes)
        got, _ = _run_gpu(W, A, primes, bits, gpu_device)
        want = pcmm_oracle(W, A, primes)
        assert (got == want).all(), (M, K, Ncols, bits, L, wbits, int((got != want).sum()))


def test_two_plans_on_two_streams_at_once(gpu_device):
    """Runs of different plans may overlap in time (each plan has its own digit scratch): two plans enqueued
    alternately on two streams of the default priority, three rounds, every result exact."""
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import pcmm_oracle

    rng = np.random.default_rng(21)
    primes = pi.ntt_primes(36, 1 << 13, 3)
    shapes = ((320, 1024, 2048), (192, 768, 4096))
    Ws = [_rand_W(rng, M, K, 8) for M, K, _ in shapes]
    As = [[_rand_A(rng, K, N, primes) for _ in range(3)] for _, K, N in shapes]
    streams = [torch.cuda.Stream(device=gpu_device), torch.cuda.Stream(device=gpu_device)]
    plans = [pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), primes, 36, N) for W, (_, _, N) in zip(Ws, shapes)]
    A_dev = [[torch.from_numpy(a.view(np.int64)).to(gpu_device) for a in group] for group in As]
    C_dev = [[torch.empty((3, M, N), dtype=torch.int64, device=gpu_device) for _ in range(3)] for M, _, N in shapes]
    torch.cuda.synchronize()
    for r in range(3):
        for p in range(2):
            pkg.pcmm_run(plans[p], A_dev[p][r], C_dev[p][r], streams[p])
    torch.cuda.synchronize()
    for p in range(2):
        for r in range(3):
            want = pcmm_oracle(Ws[p], As[p][r], primes)
            assert (C_dev[p][r].cpu().numpy().view(np.uint64) == want).all(), (p, r)
        pkg.pcmm_plan_destroy(plans[p])


@pytest.mark.parametrize("D", [4, 5, 6, 7])
def test_digit_count_switches_exactly_where_the_largest_residue_stops_fitting(gpu_device, D):
    """q - 1 + Bias_D < 256^D is the condition for D balanced digits: the largest prime below the threshold
    256^D - Bias_D takes D digits, the smallest above it D + 1, and both products are exact at residues q - 1."""
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import pcmm_oracle

    bias = sum(0x80 << (8 * i) for i in range(D))
    T = (1 << (8 * D)) - bias                       # q <= T  <=>  q - 1 + bias < 256^D
    below = T if T % 2 else T - 1
    while not pi.is_prime(below):
        below -= 2
    above = T + 1 if T % 2 == 0 else T + 2
    while not pi.is_prime(above):
        above += 2
    rng = np.random.default_rng(D)
    M, K, Ncols = 40, 200, 70
    W = _rand_W(rng, M, K, 8)
    W[0, :], W[1, :] = -128, 127
    for q, want_digits in ((below, D), (above, D + 1)):
        bits = q.bit_length()
        A = rng.integers(0, q, size=(1, K, Ncols), dtype=np.uint64)
        A[0, :, 0] = q - 1
        A[0, :, 1] = q - 2
        A[0, ::2, 2] = q - 1
        plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), [q], bits, Ncols)
        assert pkg.pcmm_plan_digits(plan) == max(want_digits, 4)
        pkg.pcmm_plan_destroy(plan)
        got, _ = _run_gpu(W, A, [q], bits, gpu_device)
        assert (got == pcmm_oracle(W, A, [q])).all(), (q, want_digits)


def test_two_thousand_seeded_tiny_shapes(gpu_device):
    """A wide net of very small problems: every prime size from 24 to 62 bits, both weight widths, 1 to 3 limbs,
    sizes around the tile and k-step edges, random / all-(q-1) residues / all-minimum weights."""
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import pcmm_oracle

    rnd = random.Random(424242)
    prime_cache = {}
    for it in range(2000):
        bits, wbits, L = rnd.randrange(24, 63), rnd.choice((8, 16)), rnd.choice((1, 1, 2, 3))
        M = rnd.choice((1, 3, 16, 31, 64, 65, 127, 128, 129, 200, 256, 257, 300, 520))
        K = rnd.choice((1, 2, 63, 64, 65, 100, 128, 129, 255, 256, 257, 400, 511, 640, 1000, 2047))
        N = rnd.choice((1, 5, 16, 17, 31, 32, 33, 48, 64, 65, 100, 130, 300))
        if bits not in prime_cache:
            prime_cache[bits] = pi.ntt_primes(bits, 1 << 6, 3)
        primes = prime_cache[bits][:L]
        rng = np.random.default_rng(rnd.randrange(1 << 30))
        W = _rand_W(rng, M, K, wbits)
        mode = rnd.randrange(4)
        A = _rand_A(rng, K, N, primes)
        if mode == 1:
            A = np.stack([np.full((K, N), q - 1, dtype=np.uint64) for q in primes])
        if mode == 2:
            W[:] = -128 if wbits == 8 else -32768
        got, _ = _run_gpu(W, A, primes, bits, gpu_device)
        want = pcmm_oracle(W, A, primes)
        assert (got == want).all(), (it, M, K, N, bits, wbits, L, mode, int((got != want).sum()))
