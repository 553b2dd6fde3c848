"""Pins for the oracle's SYR2K and Gram routines (the kernels "which use the same input several times"
of the paper's conclusion; textbook definitions): hand-worked values, exact rational brute force in
another loop order, identities that tie them to the already pinned SYRK routine, exact integer results,
and the contract on what is touched.  A dropped term, a wrong sign or index, or a transposed operand
fails at least one of them."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2202_10217_amd import inputs
from test_oracle_syrk import _read_golden, GOLDEN


@pytest.mark.parametrize("extended", [True, False])
def test_golden_3x2(extended):
    g = _read_golden(os.path.join(GOLDEN, "syr2k_gram_3x2.txt"))
    il3, il2 = np.tril_indices(3), np.tril_indices(2)
    C = np.zeros((3, 3))
    oracle.syr2k_lower(g["A"], g["B"], C, 1.0, 0.0, extended=extended)
    assert np.array_equal(C[il3], g["S"][il3]) and not C[np.triu_indices(3, 1)].any()
    C = g["C"].copy()
    oracle.syr2k_lower(g["A"], g["B"], C, 2.0, -1.0, extended=extended)
    assert np.array_equal(C[il3], g["R"][il3])
    D = np.zeros((2, 2))
    oracle.gram_lower(g["A"], D, 1.0, 0.0, extended=extended)
    assert np.array_equal(D[il2], g["G"][il2]) and D[0, 1] == 0.0
    D = g["D"].copy()
    oracle.gram_lower(g["A"], D, 2.0, -1.0, extended=extended)
    assert np.array_equal(D[il2], g["H"][il2])


def _exact(fn_terms, n, C0, alpha, beta):
    out = {}
    for i in range(n):
        for j in range(i + 1):
            out[i, j] = Fraction(beta) * Fraction(float(C0[i, j])) + Fraction(alpha) * fn_terms(i, j)
    return out


@pytest.mark.parametrize("N,M", [(1, 1), (4, 3), (7, 5), (6, 1)])
@pytest.mark.parametrize("extended", [True, False])
def test_brute_force_rational(N, M, extended):
    # dyadic inputs with few bits: every double sum is exact, so the oracle must equal the rational result
    rng = np.random.default_rng(N * 10 + M)
    A = rng.integers(-8, 9, size=(N, M)) / 4.0
    B = rng.integers(-8, 9, size=(N, M)) / 8.0
    C0 = rng.integers(-8, 9, size=(N, N)) / 2.0
    FA = [[Fraction(float(x)) for x in row] for row in A]
    FB = [[Fraction(float(x)) for x in row] for row in B]
    # k outermost for SYR2K, as a sum over columns of outer products
    want = _exact(lambda i, j: sum(FA[i][k] * FB[j][k] for k in reversed(range(M))) +
                  sum(FB[i][k] * FA[j][k] for k in range(M)), N, C0, -1.5, 0.5)
    C = C0.copy()
    oracle.syr2k_lower(A, B, C, -1.5, 0.5, extended=extended)
    for (i, j), v in want.items():
        assert Fraction(float(C[i, j])) == v, (i, j)
    D0 = rng.integers(-8, 9, size=(M, M)) / 2.0
    want = _exact(lambda i, j: sum(FA[k][i] * FA[k][j] for k in reversed(range(N))), M, D0, 3.0, -0.25)
    D = D0.copy()
    oracle.gram_lower(A, D, 3.0, -0.25, extended=extended)
    for (i, j), v in want.items():
        assert Fraction(float(D[i, j])) == v, (i, j)


@pytest.mark.parametrize("N,M", [(9, 4), (40, 17), (65, 130)])
def test_gram_is_syrk_of_the_transpose_bit_for_bit(N, M):
    # same sums in the same order (k ascending): the two routines must agree to the last bit, also on
    # data where rounding happens
    A = inputs.normal_matrix(N, M, seed=N + M)
    C0 = inputs.symmetric_uniform(M, seed=3)
    for extended in (True, False):
        G = C0.copy()
        oracle.gram_lower(A, G, -0.75, 1.25, extended=extended)
        S = C0.copy()
        oracle.syrk_lower(np.ascontiguousarray(A.T), S, -0.75, 1.25, extended=extended)
        assert np.array_equal(G, S)


@pytest.mark.parametrize("N,M", [(5, 3), (33, 20), (70, 64)])
def test_syr2k_polarisation_identity_on_integer_data(N, M):
    # A B^T + B A^T = (A+B)(A+B)^T - A A^T - B B^T, exact on small integers, with SYRK pinned separately
    A = inputs.small_int_matrix(N, M, seed=1)
    B = inputs.small_int_matrix(N, M, seed=2, lo=-3, hi=3)
    il = np.tril_indices(N)
    want = np.zeros((N, N))
    oracle.syrk_lower(A + B, want, 1.0, 0.0)
    oracle.syrk_lower(A, want, -1.0, 1.0)
    oracle.syrk_lower(B, want, -1.0, 1.0)
    for extended in (True, False):
        C = np.zeros((N, N))
        oracle.syr2k_lower(A, B, C, 1.0, 0.0, extended=extended)
        assert np.array_equal(C[il], want[il])
        # symmetric in (A, B); and B = A gives twice the SYRK
        C2 = np.zeros((N, N))
        oracle.syr2k_lower(B, A, C2, 1.0, 0.0, extended=extended)
        assert np.array_equal(C2[il], want[il])
        C3, S = np.zeros((N, N)), np.zeros((N, N))
        oracle.syr2k_lower(A, A, C3, 1.0, 0.0, extended=extended)
        oracle.syrk_lower(A, S, 2.0, 0.0)
        assert np.array_equal(C3[il], S[il])


def test_closed_forms():
    # B = unit vectors pick out columns: (A e_c^T-pattern) with B[i, :] = e_{c} for all i gives
    # S_ij = A[i, c] + A[j, c]
    N, M, c = 6, 4, 2
    A = inputs.uniform_matrix(N, M, seed=5)
    B = np.zeros((N, M))
    B[:, c] = 1.0
    C = np.zeros((N, N))
    oracle.syr2k_lower(A, B, C, 1.0, 0.0)
    for i in range(N):
        for j in range(i + 1):
            assert C[i, j] == A[i, c] + A[j, c]
    # Gram of a matrix with orthogonal columns of known length: diag(d)-scaled identity padded with zeros
    d = np.array([2.0, -3.0, 0.5])
    A = np.zeros((5, 3))
    A[1, 0], A[3, 1], A[4, 2] = d
    G = np.full((3, 3), np.nan)
    oracle.gram_lower(A, G, 1.0, 0.0)
    assert np.array_equal(G[np.tril_indices(3)], np.diag(d * d)[np.tril_indices(3)])


def test_contract_upper_untouched_beta_zero_leading_dimensions_empty():
    N, M = 9, 5
    A = inputs.small_int_matrix(N, M, seed=8)
    B = inputs.small_int_matrix(N, M, seed=9)
    iu, il = np.triu_indices(N, 1), np.tril_indices(N)
    C = np.full((N, N), np.nan)                             # beta = 0: old NaNs are not read
    oracle.syr2k_lower(A, B, C, 1.0, 0.0)
    assert np.isnan(C[iu]).all() and np.isfinite(C[il]).all()
    bigA, bigB, bigC = np.zeros((N, M + 3)), np.zeros((N, M + 2)), np.full((N, N + 4), 7.0)
    bigA[:, :M], bigB[:, :M] = A, B
    bigC[:, :N] = 0.0
    oracle.syr2k_lower(bigA[:, :M], bigB[:, :M], bigC[:, :N], 1.0, 1.0)
    assert np.array_equal(bigC[:, :N][il], C[il]) and (bigC[:, N:] == 7.0).all()
    G = np.full((M, M), np.nan)
    oracle.gram_lower(bigA[:, :M], G, 1.0, 0.0)
    assert np.isnan(G[np.triu_indices(M, 1)]).all()
    assert np.array_equal(G[np.tril_indices(M)], (A.T @ A)[np.tril_indices(M)])
    # empty contraction: C <- beta C on the lower triangle
    C1 = inputs.symmetric_uniform(N, seed=1)
    out = C1.copy()
    oracle.syr2k_lower(np.zeros((N, 0)), np.zeros((N, 0)), out, 1.0, 0.5)
    assert np.array_equal(out[il], 0.5 * C1[il]) and np.array_equal(out[iu], C1[iu])
    out = C1[:M, :M].copy()
    oracle.gram_lower(np.zeros((0, M)), out, 1.0, 0.5)
    assert np.array_equal(out[np.tril_indices(M)], 0.5 * C1[:M, :M][np.tril_indices(M)])
