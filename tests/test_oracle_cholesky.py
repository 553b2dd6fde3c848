"""Pins for the Cholesky oracle (Algorithm 2): a hand-worked factor, closed forms, uniqueness of the
factor on integer data, a separately written left-looking variant, the residual invariant and the
error path."""
import os

import numpy as np
import pytest

import oracle
from paper_2202_10217_amd import inputs
from test_oracle_syrk import _read_golden, GOLDEN


def _left_looking(S):
    """Column-by-column (left-looking) Cholesky: each column gathers all earlier updates at once."""
    N = S.shape[0]
    L = np.zeros_like(S)
    for j in range(N):
        col = S[j:, j] - L[j:, :j] @ L[j, :j]
        L[j, j] = np.sqrt(col[0])
        L[j + 1:, j] = col[1:] / L[j, j]
    return L


def test_golden_4x4():
    g = _read_golden(os.path.join(GOLDEN, "cholesky_4x4.txt"))
    S = g["S"].copy()
    S[np.triu_indices(4, 1)] = np.nan                     # upper triangle must not be referenced
    assert oracle.potrf_lower(S) == 0
    assert np.array_equal(np.tril(S), g["L"])
    assert np.isnan(S[np.triu_indices(4, 1)]).all()


def test_closed_form_diagonal():
    d = np.array([4.0, 9.0, 0.25, 16.0, 1.0])
    S = np.diag(d)
    assert oracle.potrf_lower(S) == 0
    assert np.array_equal(S, np.diag(np.sqrt(d)))


def test_closed_form_min_matrix():
    # S_ij = min(i,j) (1-based) = L L^T with L the all-ones lower triangle; all steps are exact
    N = 37
    idx = np.arange(1, N + 1, dtype=np.float64)
    S = np.minimum(idx[:, None], idx[None, :])
    assert oracle.potrf_lower(S) == 0
    assert np.array_equal(np.tril(S), np.tril(np.ones((N, N))))


@pytest.mark.parametrize("N", [1, 2, 9, 30])
def test_integer_factor_is_recovered_exactly(N):
    rng = np.random.default_rng(N)
    G = np.tril(rng.integers(-3, 4, size=(N, N))).astype(np.float64)
    np.fill_diagonal(G, rng.integers(1, 5, size=N))
    S = G @ G.T                                            # small integers: exact
    assert oracle.potrf_lower(S) == 0
    assert np.array_equal(np.tril(S), G)


@pytest.mark.parametrize("N", [5, 64, 150])
def test_agrees_with_left_looking_and_residual(N):
    S0 = inputs.spd_diag_dominant(N, seed=N)
    S = S0.copy()
    assert oracle.potrf_lower(S) == 0
    L = np.tril(S)
    assert (np.diag(L) > 0).all()
    L2 = _left_looking(S0)
    assert np.allclose(L, L2, rtol=0, atol=64 * np.finfo(float).eps * np.abs(L2).max())
    assert oracle.llt_residual(S, S0) < 1e-15 * 10
    full = L @ L.T
    assert np.linalg.norm(full - S0) / np.linalg.norm(S0) < 1e-14


def test_residual_routine_against_numpy_and_detects_a_wrong_factor():
    N = 40
    S0 = inputs.spd_diag_dominant(N, seed=77)
    L = _left_looking(S0)
    r = oracle.llt_residual(L, S0)
    assert abs(r - np.linalg.norm(L @ L.T - S0) / np.linalg.norm(S0)) < 1e-16
    Lbad = L.copy()
    Lbad[17, 5] += 1e-6
    assert oracle.llt_residual(Lbad, S0) > 1e-10


@pytest.mark.parametrize("bad", [0, 3, 11])
def test_not_positive_definite_reports_first_bad_pivot(bad):
    N = 12
    G = np.tril(np.ones((N, N)))
    S = G @ G.T
    S[bad, bad] -= 1.0 + (bad > 0) * 0.0                    # pivot `bad` becomes 1 - 1 = 0
    assert oracle.potrf_lower(S) == bad + 1
    S = G @ G.T
    S[bad, bad] = np.nan
    assert oracle.potrf_lower(S) == bad + 1


def test_leading_dimension():
    N = 10
    S0 = inputs.spd_diag_dominant(N, seed=5)
    big = np.zeros((N, N + 6))
    big[:, :N] = S0
    S = S0.copy()
    oracle.potrf_lower(S)
    oracle.potrf_lower(big[:, :N])
    assert np.array_equal(np.tril(big[:, :N]), np.tril(S))
    assert np.array_equal(big[:, N:], np.zeros((N, 6)))
