"""Host-side checks of the seeded input generators (no GPU)."""
import os

import numpy as np
import pytest

import pcmm_inputs as pi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ntt_primes.txt")


def _trial_division_prime(n: int) -> bool:
    """Independent of the Miller-Rabin finder: divide by every odd number up to sqrt(n), vectorised."""
    if n < 2 or n % 2 == 0:
        return n == 2
    lim = int(np.sqrt(float(n))) + 2
    step = 1 << 22
    for lo in range(3, lim, step):
        d = np.arange(lo | 1, min(lim, lo + step), 2, dtype=np.uint64)
        if (np.uint64(n) % d == 0).any():
            return False
    return True


def _golden():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                b, t, q = line.split()
                rows.append((int(b), int(t), int(q)))
    return rows


def test_golden_primes_are_prime_and_congruent():
    for bits, two_n, q in _golden():
        assert (1 << (bits - 1)) < q < (1 << bits)
        assert q % two_n == 1
        assert _trial_division_prime(q), q


def test_finder_reproduces_golden_lists_and_they_are_the_largest():
    by_key = {}
    for bits, two_n, q in _golden():
        by_key.setdefault((bits, two_n), []).append(q)
    for (bits, two_n), qs in by_key.items():
        assert pi.ntt_primes(bits, two_n, len(qs)) == qs
        # maximality: no prime = 1 mod two_n between consecutive list entries / below 2^bits
        cand = ((1 << bits) - 1) // two_n * two_n + 1
        found = []
        while cand >= qs[-1]:
            if _trial_division_prime(cand) if bits <= 36 else pi.is_prime(cand):
                found.append(cand)
            cand -= two_n
        assert found == qs


def test_miller_rabin_against_trial_division_small():
    for n in list(range(0, 2000)) + [2 ** 31 - 1, 2 ** 31 + 11, 3215031751, 4759123141, 561, 1105]:
        assert pi.is_prime(n) == _trial_division_prime(n), n


def test_workload_shapes_match_the_llama_projection_shapes():
    w = pi.WORKLOADS
    assert (w["attn_proj"].M, w["attn_proj"].K) == (4096, 4096)
    assert (w["ffn_up_gate"].M, w["ffn_up_gate"].K) == (14336, 4096)
    assert (w["ffn_down"].M, w["ffn_down"].K) == (4096, 14336)
    assert (w["wide_pc_attn"].M, w["wide_pc_attn"].K, w["wide_pc_attn"].w_bits) == (4096, 128, 16)
    assert [x.Ncols for x in w.values()] == [8192, 32768, 32768, 32768, 131072, 32768]
    assert [x.L for x in w.values()] == [2, 4, 4, 3, 6, 1]
    assert [x.digits * x.slices for x in w.values()] == [5, 5, 5, 5, 14, 16]
    assert w["attn_proj"].int8_ops == 2 * 4096 * 4096 * 32768 * 4 * 5


def test_uniform_mod_q_range_determinism_and_columns():
    wl = pi.WORKLOADS["tiny"]
    A = pi.gen_A(wl)
    assert A.dtype == np.uint64 and A.shape == (2, 128, 8192)
    for j, q in enumerate(wl.primes):
        assert int(A[j].max()) < q
        # uniform on [0,q): mean ~ q/2, top bit set about half the time
        assert abs(float(A[j].mean()) / q - 0.5) < 0.01
        assert abs(float((A[j] >> np.uint64(35)).mean()) - 0.5) < 0.01
    assert (pi.gen_A(wl) == A).all()
    assert not (A[0] == A[1]).all()
    cols = [0, 1, 4095, 4096, 8191]
    assert (pi.gen_A_columns(wl, 1, cols) == A[1][:, cols]).all()


def test_rejection_path_is_exercised_and_unbiased_for_a_small_modulus():
    # q just above 2^(bits-1): almost half of the draws are rejected and redrawn
    q, bits = 33, 6
    idx = np.arange(200000, dtype=np.uint64)
    v = pi.uniform_mod_q(7, 3, idx, q, bits)
    assert int(v.max()) == q - 1 and int(v.min()) == 0
    counts = np.bincount(v.astype(np.int64), minlength=q)
    assert counts.min() > 0.9 * idx.size / q and counts.max() < 1.1 * idx.size / q


def test_torch_generator_equals_numpy_generator_on_cpu():
    import torch

    wl = pi.Workload("t", 8, 24, 64, 3, 50, 8, seed=5)
    ref = pi.gen_A(wl)
    got = pi.gen_A_torch(wl, torch.device("cpu")).numpy().view(np.uint64)
    assert (ref == got).all()
    # a 6-bit modulus just above 2^5 (37 = 1 mod 4, the 4th largest): almost half the draws are rejected and redrawn
    wl3 = pi.Workload("t3", 4, 40, 2, 2, 6, 8, seed=1)
    assert wl3.primes == [61, 53]
    assert (pi.gen_A(wl3) == pi.gen_A_torch(wl3, torch.device("cpu")).numpy().view(np.uint64)).all()
    wl4 = pi.Workload("t4", 4, 40, 2, 4, 6, 8, seed=1)
    assert wl4.primes[-1] == 37
    assert (pi.gen_A(wl4) == pi.gen_A_torch(wl4, torch.device("cpu")).numpy().view(np.uint64)).all()


def test_W_generators():
    w8 = pi.gen_W(pi.WORKLOADS["tiny"])
    assert w8.dtype == np.int8 and w8.shape == (128, 128)
    assert w8.min() == -128 and w8.max() == 127
    w16 = pi.gen_W(pi.WORKLOADS["wide_pc_attn"])
    assert w16.dtype == np.int16 and w16.shape == (4096, 128)
    assert abs(float(w16.std()) - 1024.0) < 10.0 and abs(float(w16.mean())) < 5.0
    assert np.abs(w16.astype(np.int32)).max() < 7 * 1024
