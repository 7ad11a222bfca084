"""Pins of the CPU oracle against things other than itself (no GPU).

The paper prints no worked PCMM example, so the oracle is pinned by
  * Python arbitrary-precision brute force on tiny shapes (a third implementation),
  * closed forms and special cases,
  * linearity of B = W.A in both operands,
  * CRT consistency across RNS limbs,
  * the block identity B^(u) = sum_v W^(u,v) A^(v) of Section 5.1,
  * invariance under a joint permutation of the contraction index.
The toy CKKS round trip is in test_oracle_ckks_roundtrip.py.
"""
import random

import numpy as np
import pytest

import pcmm_inputs as pi
from oracle import pcmm_freivalds, pcmm_oracle, pcmm_oracle_select

P36 = pi.ntt_primes(36, 1 << 13, 2)
P50 = pi.ntt_primes(50, 1 << 17, 3)
P62 = pi.ntt_primes(62, 1 << 10, 2)


def brute(W, A, primes):
    """Definition with Python ints: C_j[m][n] = sum_k W[m][k] A_j[k][n] mod q_j in [0,q_j)."""
    M, K = len(W), len(W[0])
    L, Ncols = len(A), len(A[0][0])
    out = np.zeros((L, M, Ncols), dtype=np.uint64)
    for j in range(L):
        q = int(primes[j])
        for m in range(M):
            for n in range(Ncols):
                s = 0
                for k in range(K):
                    s += int(W[m][k]) * int(A[j][k][n])
                out[j, m, n] = s % q
    return out


def rand_case(rng, M, K, Ncols, primes, wlo=-128, whi=127):
    W = np.array([[rng.randint(wlo, whi) for _ in range(K)] for _ in range(M)], dtype=np.int32)
    A = np.array([[[rng.randrange(q) for _ in range(Ncols)] for _ in range(K)] for q in primes], dtype=np.uint64)
    return W, A


@pytest.mark.parametrize(
    "M,K,Ncols,primes,wlo,whi",
    [
        (1, 1, 1, P36[:1], -128, 127),
        (3, 4, 5, P36, -128, 127),
        (8, 8, 16, P36, -128, 127),
        (5, 7, 3, P50, -32768, 32767),
        (4, 33, 6, P62, -(2 ** 31), 2 ** 31 - 1),
        (2, 9, 4, [3, 5, 7], -128, 127),
    ],
)
def test_brute_force_python_bigints(M, K, Ncols, primes, wlo, whi):
    rng = random.Random(1234 + M * 100 + K)
    W, A = rand_case(rng, M, K, Ncols, primes, wlo, whi)
    assert (pcmm_oracle(W, A, primes) == brute(W.tolist(), A.tolist(), primes)).all()


def test_non_square_and_asymmetric_values_catch_transposes():
    # W is not symmetric and not square; A rows and columns have different sizes
    W = np.array([[1, 2, 3], [-4, 5, -6]], dtype=np.int32)           # 2 x 3
    A = np.array([[[1, 0, 2, 7], [0, 1, 3, 7], [5, 5, 5, 7]]], dtype=np.uint64)  # 3 x 4
    q = 101
    want = np.array([[[16, 17, 23, 42], [(-34) % q, (-25) % q, (-23) % q, (-35) % q]]], dtype=np.uint64)
    assert (pcmm_oracle(W, A, [q]) == want).all()


def test_closed_forms():
    rng = random.Random(7)
    K = 12
    Ncols = 9
    primes = P36
    _, A = rand_case(rng, K, K, Ncols, primes)
    eye = np.eye(K, dtype=np.int32)
    assert (pcmm_oracle(eye, A, primes) == A).all()
    neg = pcmm_oracle(-eye, A, primes)
    for j, q in enumerate(primes):
        assert (neg[j] == (np.uint64(q) - A[j]) % np.uint64(q)).all()
    assert (pcmm_oracle(np.zeros((4, K), np.int32), A, primes) == 0).all()

    W = np.array([[rng.randint(-128, 127) for _ in range(K)] for _ in range(5)], dtype=np.int32)
    ones = np.ones((2, K, Ncols), dtype=np.uint64)
    C1 = pcmm_oracle(W, ones, primes)
    top = np.stack([np.full((K, Ncols), q - 1, dtype=np.uint64) for q in primes])
    Cq = pcmm_oracle(W, top, primes)
    for j, q in enumerate(primes):
        for m in range(5):
            rs = int(W[m].sum())
            assert (C1[j, m] == rs % q).all()
            assert (Cq[j, m] == (-rs) % q).all()

    # one-hot row of A picks out a column of W, negatives lifted to q - |w|
    onehot = np.zeros((1, K, Ncols), dtype=np.uint64)
    onehot[0, 3, 4] = 1
    C = pcmm_oracle(W, onehot, primes[:1])
    for m in range(5):
        assert int(C[0, m, 4]) == int(W[m, 3]) % primes[0]
    C[0, :, 4] = 0
    assert (C == 0).all()


def test_linearity_in_A_and_in_W():
    rng = random.Random(11)
    primes = P50
    W1, A1 = rand_case(rng, 6, 10, 7, primes, -32768, 32767)
    W2, A2 = rand_case(rng, 6, 10, 7, primes, -32768, 32767)
    qs = np.array(primes, dtype=np.uint64)[:, None, None]
    Asum = (A1 + A2) % qs
    lhs = pcmm_oracle(W1, Asum, primes)
    rhs = (pcmm_oracle(W1, A1, primes) + pcmm_oracle(W1, A2, primes)) % qs
    assert (lhs == rhs).all()
    lhs = pcmm_oracle(W1 + W2, A1, primes)
    rhs = (pcmm_oracle(W1, A1, primes) + pcmm_oracle(W2, A1, primes)) % qs
    assert (lhs == rhs).all()
    # scalar homogeneity with a negative scalar
    lhs = pcmm_oracle(-3 * W1, A1, primes)
    base = pcmm_oracle(W1, A1, primes)
    for j, q in enumerate(primes):
        want = np.array([[(-3 * int(v)) % q for v in row] for row in base[j]], dtype=np.uint64)
        assert (lhs[j] == want).all()


def test_crt_consistency_across_limbs():
    rng = random.Random(13)
    primes = pi.ntt_primes(36, 1 << 15, 4)
    Q = 1
    for q in primes:
        Q *= q
    M, K, Ncols = 4, 9, 6
    W = [[rng.randint(-128, 127) for _ in range(K)] for _ in range(M)]
    X = [[rng.randrange(Q) for _ in range(Ncols)] for _ in range(K)]
    A = np.array([[[x % q for x in row] for row in X] for q in primes], dtype=np.uint64)
    C = pcmm_oracle(np.array(W, dtype=np.int32), A, primes)
    for m in range(M):
        for n in range(Ncols):
            big = sum(W[m][k] * X[k][n] for k in range(K)) % Q
            for j, q in enumerate(primes):
                assert int(C[j, m, n]) == big % q
    # the limbs really use different primes: the same residues under swapped primes differ
    A_same = np.stack([A[0], A[0]])
    C2 = pcmm_oracle(np.array(W, dtype=np.int32), A_same % np.uint64(primes[1]), primes[:2])
    assert not (C2[0] == C2[1]).all()


@pytest.mark.parametrize("p_r,p_c", [(1, 2), (2, 2), (4, 1), (2, 4)])
def test_block_identity_of_the_2d_partition(p_r, p_c):
    """B^(u) = sum_v W^(u,v) . A^(v)  (Section 5.1, Eq. blockmat), with sums taken mod q."""
    rng = random.Random(17 + p_r * 10 + p_c)
    primes = P36
    M, K, Ncols = 8, 16, 5
    W, A = rand_case(rng, M, K, Ncols, primes)
    full = pcmm_oracle(W, A, primes)
    qs = np.array(primes, dtype=np.uint64)[:, None, None]
    mb, kb = M // p_r, K // p_c
    for u in range(p_r):
        acc = np.zeros((len(primes), mb, Ncols), dtype=np.uint64)
        for v in range(p_c):
            part = pcmm_oracle(W[u * mb:(u + 1) * mb, v * kb:(v + 1) * kb], A[:, v * kb:(v + 1) * kb, :], primes)
            acc = (acc + part) % qs
        assert (acc == full[:, u * mb:(u + 1) * mb, :]).all()


def test_joint_permutation_of_the_contraction_index():
    rng = random.Random(19)
    W, A = rand_case(rng, 5, 11, 4, P36)
    perm = list(range(11))
    rng.shuffle(perm)
    assert (pcmm_oracle(W[:, perm], A[:, perm, :], P36) == pcmm_oracle(W, A, P36)).all()


def test_extreme_operands_long_contraction():
    """K = 14336 with W = -128 everywhere and residues q-1: |sum| ~ 2^57, far inside __int128."""
    K = 14336
    primes = P36
    W = np.full((2, K), -128, dtype=np.int32)
    W[1] = 127
    A = np.stack([np.full((K, 3), q - 1, dtype=np.uint64) for q in primes])
    C = pcmm_oracle(W, A, primes)
    for j, q in enumerate(primes):
        assert int(C[j, 0, 0]) == (-128 * K * (q - 1)) % q
        assert int(C[j, 1, 2]) == (127 * K * (q - 1)) % q


def test_select_agrees_with_full_and_checks_indices():
    rng = random.Random(23)
    W, A = rand_case(rng, 7, 6, 9, P36)
    full = pcmm_oracle(W, A, P36)
    rows, cols = [6, 0, 3], [8, 8, 1, 0]
    sel = pcmm_oracle_select(W, A, P36, rows, cols)
    assert sel.shape == (2, 3, 4)
    assert (sel == full[:, rows][:, :, cols]).all()
    with pytest.raises(RuntimeError):
        pcmm_oracle_select(W, A, P36, [7], [0])
    with pytest.raises(RuntimeError):
        pcmm_oracle_select(W, A, P36, [0], [-1])


def test_unreduced_residues_are_refused():
    W = np.ones((1, 1), dtype=np.int32)
    A = np.full((1, 1, 1), P36[0], dtype=np.uint64)
    with pytest.raises(ValueError):
        pcmm_oracle(W, A, P36[:1])


def test_freivalds_accepts_truth_and_rejects_planted_errors():
    rng = random.Random(29)
    q = P50[0]
    W, A = rand_case(rng, 9, 13, 17, [q], -32768, 32767)
    C = pcmm_oracle(W, A, [q])[0]
    r = np.array([rng.randrange(q) for _ in range(17)], dtype=np.uint64)
    # the check's two sides, with Python ints
    for m in range(9):
        lhs = sum(int(C[m, n]) * int(r[n]) for n in range(17)) % q
        y = [sum(int(A[0, k, n]) * int(r[n]) for n in range(17)) % q for k in range(13)]
        rhs = sum(int(W[m, k]) * y[k] for k in range(13)) % q
        assert lhs == rhs
    assert pcmm_freivalds(W, A[0], C, r, q) == 0
    bad = C.copy()
    bad[4, 5] = (int(bad[4, 5]) + 1) % q
    assert pcmm_freivalds(W, A[0], bad, r, q) == 1
    bad[0, 0] = (int(bad[0, 0]) + q - 1) % q
    assert pcmm_freivalds(W, A[0], bad, r, q) == 2
    out_of_range = C.copy()
    out_of_range[2, 2] = int(out_of_range[2, 2]) + q       # same residue class, not canonical
    assert pcmm_freivalds(W, A[0], out_of_range, r, q) == 1
    # a result computed with the wrong prime fails almost every row
    wrong = pcmm_oracle(W, A % np.uint64(P50[1]), [P50[1]])[0]
    assert pcmm_freivalds(W, A[0], wrong % np.uint64(q), r, q) >= 8
