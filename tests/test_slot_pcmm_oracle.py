"""Pins of the slot-encoded PCMM oracle (Section 4.2, Appendix E) against what the paper and plain linear algebra fix."""
import os

import numpy as np
import pytest

from oracle import slot_pcmm_oracle as so

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "slot_pcmm_example.txt")


def _golden():
    out, name = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line[0].isalpha():
            name = line
            out[name] = []
        else:
            out[name].append([int(x) for x in line.split()])
    return {k: np.array(v, dtype=np.int64) for k, v in out.items()}


def _rand(rng, d):
    return rng.integers(-50, 50, size=(d, d), dtype=np.int64)


def _tau_pow_closed(C, ell):
    """tau^ell by its closed form tau^ell(C)[i][j] = C[i + ell j][j] (not how the oracle does it)."""
    d = C.shape[0]
    i, j = np.meshgrid(np.arange(d), np.arange(d), indexing="ij")
    return C[(i + ell * j) % d, j]


def test_hand_worked_example():
    g = _golden()
    A = g["A"]
    assert (so.sigma(A) == g["sigma"]).all()
    assert (so.tau(A) == g["tau"]).all()
    assert (so.rot_col(A, 1) == g["rot_col_1"]).all()
    assert (so.rot_row(A, 1) == g["rot_row_1"]).all()
    assert (so.tau(so.sigma(A)) == g["tau_sigma"]).all()
    assert (so.stored_plaintext(A, 1) == g["tau_sigma"]).all()


@pytest.mark.parametrize("d", [1, 2, 3, 4, 5, 8, 16])
def test_jkls_identity_is_the_matrix_product(d):
    rng = np.random.default_rng(d)
    A, B = _rand(rng, d), _rand(rng, d)
    assert (so.jkls_product(A, B) == A @ B).all()


@pytest.mark.parametrize("d", [2, 3, 5, 8])
def test_maps_are_permutations_with_the_expected_orders(d):
    rng = np.random.default_rng(10 + d)
    A = np.arange(d * d, dtype=np.int64).reshape(d, d)
    for f in (so.sigma, so.tau, so.tau_inverse, lambda M: so.rot_col(M, 3), lambda M: so.rot_row(M, -2)):
        assert sorted(f(A).ravel().tolist()) == list(range(d * d))
    assert (so.tau_pow(A, d) == A).all() and (so.tau_pow(A, -d) == A).all()
    assert (so.tau_inverse(so.tau(A)) == A).all() and (so.tau_pow(so.tau_pow(A, 3), -3) == A).all()
    assert (so.rot_col(A, d) == A).all() and (so.rot_row(so.rot_row(A, 2), -2) == A).all()
    for ell in (-3, -1, 0, 1, 2, 5):
        assert (so.tau_pow(A, ell) == _tau_pow_closed(A, ell)).all()
    M = _rand(rng, d)
    assert (so.rot_row(so.rot_col(M, 1), 2) == so.rot_col(so.rot_row(M, 2), 1)).all()   # the two rotations commute


@pytest.mark.parametrize("d", [3, 4, 8])
def test_lemma_2_commutation_rules(d):
    """tau o rot_R^k = rot_R^k o tau  and  tau o rot_C^k = rot_R^{-k} o rot_C^k o tau  (Appendix E, Lemma 2)."""
    rng = np.random.default_rng(20 + d)
    M = _rand(rng, d)
    for k in range(-d, 2 * d):
        assert (so.tau(so.rot_row(M, k)) == so.rot_row(so.tau(M), k)).all()
        assert (so.tau(so.rot_col(M, k)) == so.rot_row(so.rot_col(so.tau(M), k), -k)).all()


@pytest.mark.parametrize("d", [1, 2, 3, 4, 6, 8])
def test_theorem_1(d):
    rng = np.random.default_rng(30 + d)
    A, B = _rand(rng, d), _rand(rng, d)
    C = A @ B
    for ell in (-2, -1, 0, 1, 2, 3):
        assert (so.theorem1(A, B, ell) == _tau_pow_closed(C, ell)).all(), ell


@pytest.mark.parametrize("d", [1, 2, 4, 6, 8, 12, 16])
def test_equation_pcmm_for_every_factorisation(d):
    """tau^ell(A B) from pt_A and tau^{ell+1}(B), for every g b = d (Section 4.2, Eq. "pcmm")."""
    rng = np.random.default_rng(40 + d)
    A, B = _rand(rng, d), _rand(rng, d)
    C = A @ B
    for ell in (-1, 0, 1, 2):
        Bt = _tau_pow_closed(B, ell + 1)
        for g in range(1, d + 1):
            if d % g:
                continue
            b = d // g
            assert (so.pcmm_bsgs(A, Bt, ell, g, b) == _tau_pow_closed(C, ell)).all(), (ell, g, b)


def test_two_calls_chain_as_in_pc_attention():
    """Each call undoes one tau: tau^2 applied before the wide part leaves the plain layout after two PCMMs (Section 4.2)."""
    rng = np.random.default_rng(50)
    d = 8
    A1, A2, B = _rand(rng, d), _rand(rng, d), _rand(rng, d)
    X = so.tau_pow(B, 2)
    Y = so.pcmm_bsgs(A1, X, 1, 2, 4)              # tau^1(A1 B) from tau^2(B)
    Z = so.pcmm_bsgs(A2, Y, 0, 4, 2)              # tau^0(A2 A1 B) from tau^1(A1 B)
    assert (Z == A2 @ (A1 @ B)).all()


def test_rearranged_plaintext_is_a_two_dimensional_cyclic_shift():
    rng = np.random.default_rng(60)
    d, ell, g, b = 12, 2, 3, 4
    A = _rand(rng, d)
    S = so.stored_plaintext(A, ell)
    all_pt = so.rearranged_plaintexts(S, ell, g, b)
    assert all_pt.shape == (g, b, d, d)
    r, c = np.meshgrid(np.arange(d), np.arange(d), indexing="ij")
    for j in range(g):
        for i in range(b):
            k = i + j * b
            want = S[(r - ell * k - j * b) % d, (c + k) % d]
            assert (all_pt[j][i] == want).all()
            assert (so.rearranged_plaintext(S, i, j, ell, b) == want).all()
    with pytest.raises(ValueError):
        so.rearranged_plaintexts(S, ell, 5, 2)


def test_planted_mistakes_are_caught():
    """A wrong sign or a dropped term in the rearrangement breaks Eq. "pcmm" (the pins above would see it)."""
    rng = np.random.default_rng(70)
    d, ell, g, b = 8, 1, 4, 2          # j b runs over 0, 2, 4, 6: its sign matters modulo 8
    A, B = _rand(rng, d), _rand(rng, d)
    want = _tau_pow_closed(A @ B, ell)
    Bt = _tau_pow_closed(B, ell + 1)
    S = so.stored_plaintext(A, ell)

    def variant(row_shift):
        acc = np.zeros_like(A)
        for j in range(g):
            inner = np.zeros_like(A)
            for i in range(b):
                k = i + j * b
                inner = inner + so.rot_row(so.rot_col(S, k), row_shift(k, j)) * so.rot_row(Bt, i)
            acc = acc + so.rot_row(inner, j * b)
        return acc

    assert (variant(lambda k, j: -ell * k - j * b) == want).all()
    assert not (variant(lambda k, j: +ell * k - j * b) == want).all()      # sign of the ell term
    assert not (variant(lambda k, j: -ell * k) == want).all()              # giant-step compensation dropped
    assert not (variant(lambda k, j: -ell * k + j * b) == want).all()
