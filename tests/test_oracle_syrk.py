"""Pins for the SYRK oracle (Algorithm 1): hand-worked values, closed forms, exact integer
results, brute force in exact rational arithmetic, and the contract on what is touched.
None of these re-type the oracle's loop in floating point: a dropped term, a wrong sign or
index, or a transposed operand fails at least one of them."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2202_10217_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(path):
    blocks, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.isalpha():
            cur = blocks.setdefault(line, [])
        else:
            cur.append([float(x) for x in line.split()])
    return {k: np.array(v, dtype=np.float64) for k, v in blocks.items()}


def _syrk_exact(A, C0, alpha, beta):
    """Exact rational evaluation, summing column outer products (k outermost)."""
    N, M = A.shape
    acc = [[Fraction(0) for _ in range(N)] for _ in range(N)]
    for k in range(M):
        col = [Fraction(float(A[i, k])) for i in range(N)]
        for i in range(N):
            for j in range(i + 1):
                acc[i][j] += col[i] * col[j]
    out = {}
    for i in range(N):
        for j in range(i + 1):
            out[i, j] = Fraction(beta) * Fraction(float(C0[i, j])) + Fraction(alpha) * acc[i][j]
    return out


@pytest.mark.parametrize("extended", [True, False])
def test_golden_3x2(extended):
    g = _read_golden(os.path.join(GOLDEN, "syrk_3x2.txt"))
    C = np.zeros((3, 3))
    oracle.syrk_lower(g["A"], C, 1.0, 1.0, extended=extended)
    assert np.array_equal(np.tril(C), np.tril(g["C"]))
    assert np.array_equal(np.triu(C, 1), np.zeros((3, 3)))


@pytest.mark.parametrize("extended", [True, False])
@pytest.mark.parametrize("N,M", [(1, 1), (1, 5), (4, 1), (5, 0), (3, 7), (8, 8), (7, 3)])
def test_brute_force_rational(N, M, extended):
    # dyadic rationals with few bits: every product and sum is exact in double, so the oracle
    # must equal the exact rational result bit for bit
    rng = np.random.default_rng(10 * N + M)
    A = rng.integers(-8, 9, size=(N, M)).astype(np.float64) / 4.0
    C0 = rng.integers(-8, 9, size=(N, N)).astype(np.float64) / 2.0
    alpha, beta = -0.5, 2.0
    C = C0.copy()
    oracle.syrk_lower(A, C, alpha, beta, extended=extended)
    ref = _syrk_exact(A, C0, alpha, beta)
    for (i, j), v in ref.items():
        assert Fraction(float(C[i, j])) == v, (i, j)
    iu = np.triu_indices(N, 1)
    assert np.array_equal(C[iu], C0[iu])


def test_closed_form_diagonal():
    d = np.arange(1.0, 10.0)
    A = np.diag(d)
    C = np.zeros((9, 9))
    oracle.syrk_lower(A, C, 1.0, 0.0)
    assert np.array_equal(C, np.diag(d * d))


def test_closed_form_all_ones():
    N, M = 6, 11
    C = np.zeros((N, N))
    oracle.syrk_lower(np.ones((N, M)), C)
    assert np.array_equal(np.tril(C), np.tril(np.full((N, N), float(M))))


def test_closed_form_identity_padded():
    N, M = 5, 9
    A = np.zeros((N, M))
    A[:, :N] = np.eye(N)
    C = np.zeros((N, N))
    oracle.syrk_lower(A, C)
    assert np.array_equal(C, np.eye(N))


def test_closed_form_hadamard_rows_are_orthogonal():
    H = np.array([[1.0]])
    for _ in range(4):
        H = np.block([[H, H], [H, -H]])
    C = np.zeros((11, 11))
    oracle.syrk_lower(H[:11].copy(), C)        # 11 mutually orthogonal rows of length 16
    assert np.array_equal(C, 16.0 * np.eye(11))


def test_closed_form_rank_one():
    # A = x y^T  =>  A A^T = (y.y) x x^T ; integers, exact.  A^T A would have another shape and
    # (i,k)/(j,k) index slips change the values.
    x = np.array([1.0, -2.0, 3.0, 5.0])
    y = np.array([2.0, 1.0, -1.0])
    A = np.outer(x, y)
    C = np.zeros((4, 4))
    oracle.syrk_lower(A, C)
    assert np.array_equal(np.tril(C), np.tril(6.0 * np.outer(x, x)))


@pytest.mark.parametrize("N,M", [(33, 70), (64, 17)])
def test_integer_inputs_are_exact(N, M):
    A = inputs.small_int_matrix(N, M, seed=5)
    C0 = inputs.symmetric_uniform(N, seed=6, int_range=(-3, 3))
    exact = 2 * C0.astype(np.int64) - 3 * (A.astype(np.int64) @ A.astype(np.int64).T)
    for ext in (True, False):
        C = C0.copy()
        oracle.syrk_lower(A, C, -3.0, 2.0, extended=ext)
        il = np.tril_indices(N)
        assert np.array_equal(C[il], exact[il].astype(np.float64))


def test_upper_triangle_never_touched_and_beta_zero_does_not_read():
    N, M = 9, 5
    A = inputs.uniform_matrix(N, M, seed=1)
    C = np.full((N, N), np.nan)
    oracle.syrk_lower(A, C, 1.0, 0.0)
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.isnan(C[iu]).all()
    assert np.isfinite(C[il]).all()
    # symmetric-product invariant: rows swapped roles give the same number
    G = A @ A.T
    assert np.allclose(C[il], G[il], rtol=0, atol=1e-14)


def test_linearity_in_alpha_and_beta():
    N, M = 12, 9
    A = inputs.small_int_matrix(N, M, seed=2).astype(np.float64)
    C0 = inputs.symmetric_uniform(N, seed=3, int_range=(-4, 4))
    P = np.zeros((N, N))
    oracle.syrk_lower(A, P, 1.0, 0.0)
    C = C0.copy()
    oracle.syrk_lower(A, C, 0.25, -2.0)
    il = np.tril_indices(N)
    assert np.array_equal(C[il], (-2.0 * C0 + 0.25 * P)[il])


def test_leading_dimensions():
    N, M = 7, 5
    Abig = inputs.uniform_matrix(N, M + 3, seed=4)
    Cbig = np.zeros((N, N + 4))
    C2 = np.zeros((N, N))
    oracle.syrk_lower(Abig[:, :M], Cbig[:, :N], 1.0, 0.0)
    oracle.syrk_lower(np.ascontiguousarray(Abig[:, :M]), C2, 1.0, 0.0)
    assert np.array_equal(Cbig[:, :N], C2)
    assert np.array_equal(Cbig[:, N:], np.zeros((N, 4)))


def test_psd_and_plain_vs_extended_agree_within_rounding():
    N, M = 40, 300
    A = inputs.normal_matrix(N, M, seed=7)
    Ce, Cp = np.zeros((N, N)), np.zeros((N, N))
    oracle.syrk_lower(A, Ce, 1.0, 0.0, extended=True)
    oracle.syrk_lower(A, Cp, 1.0, 0.0, extended=False)
    D = np.zeros((N, N))
    oracle.syrk_lower(np.abs(A), D, 1.0, 0.0)
    il = np.tril_indices(N)
    # plain double summation of M terms: |err| <= M u |A||A|^T (u = 2^-53), far tighter in practice
    assert (np.abs(Ce - Cp)[il] <= M * 2.0 ** -53 * D[il]).all()
    full = np.tril(Ce) + np.tril(Ce, -1).T
    x = inputs.normal_matrix(N, 3, seed=8)
    q = np.einsum("ia,ij,ja->a", x, full, x)
    assert (q > 0).all()
    assert np.allclose(q, ((A.T @ x) ** 2).sum(axis=0), rtol=1e-12)


def test_sample_matches_full():
    N, M = 25, 40
    A = inputs.normal_matrix(N, M, seed=9)
    C0 = inputs.symmetric_uniform(N, seed=10)
    C = C0.copy()
    oracle.syrk_lower(A, C, -1.0, 1.0)
    ii, jj = np.tril_indices(N)
    s = oracle.syrk_lower_sample(A, C0, ii, jj, -1.0, 1.0)
    assert np.array_equal(s, C[ii, jj])
