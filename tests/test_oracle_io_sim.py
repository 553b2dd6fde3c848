"""The I/O simulator (counts only) against the arithmetic replay, and its counts against the paper's
theorems for a range of memory sizes S."""
import math

import numpy as np
import pytest

from oracle import io_sim
from oracle import tbs_schedule as ts


@pytest.mark.parametrize("N,M,k,b", [(60, 3, 4, 1), (143, 2, 5, 1), (96, 4, 4, 2), (200, 1, 6, 1), (37, 5, 4, 1),
                                     (360, 2, 4, 3)])
def test_counts_equal_the_arithmetic_replay(N, M, k, b):
    io = ts.tbs_syrk(np.zeros((N, M)), np.zeros((N, N)), k, b)
    sim = io_sim.tbs_counts(N, M, k, b)
    assert (sim["A"], sim["C"], sim["A_q1"], sim["blocks"]) == (io.A, io.C, io.A_q1, len(io.blocks))
    assert sim["C"] == N * (N + 1) // 2                      # every entry of C loaded exactly once


def test_k_and_square_side_for_memory():
    for S in range(3, 400):
        k = io_sim.k_for_memory(S)
        assert k * (k + 1) // 2 <= S < (k + 1) * (k + 2) // 2
        s = io_sim.square_side_for_memory(S)
        assert s * s + 2 * s <= S or s == 1
        assert (s + 1) ** 2 + 2 * (s + 1) > S


@pytest.mark.parametrize("S", [15, 28, 55, 136, 325, 1035])
def test_theorem_of_section_5_1_3_for_a_range_of_memory_sizes(S):
    # N large against S (the scheme needs N >= about 2 S); M small: every count is linear in M
    k = io_sim.k_for_memory(S)
    N, M = 40 * k * k + 7, 2
    r = io_sim.simulate_tbs(N, M, S)
    assert r["C"] == N * (N + 1) // 2
    # never below the lower bound; at most the recursion's bound N^2 M/(k-1) plus the O(N M log N) terms
    assert r["A"] >= r["lower_bound"] - N * M
    assert r["A"] <= r["recursion_bound_A"] + 6 * k * N * M * math.log2(N)
    # the triangle scheme beats square blocks of the same memory, by a factor that tends to sqrt(2):
    # (k-1) / sqrt(S) from the leading terms
    assert r["A"] < r["square_A"]
    lead_ratio = (N * N * M / (k - 1.0)) / (N * N * M / r["square_side"])
    assert abs(r["A"] / r["square_A"] - lead_ratio) < 0.12
    assert abs(r["square_A"] - r["square_model_A"]) <= 2 * N * M + r["square_model_A"] * 0.02
    # the measured A volume over the lower bound approaches sqrt(k(k+1))/(k-1) (= 1 as S grows)
    assert r["A"] / r["lower_bound"] < math.sqrt(k * (k + 1.0)) / (k - 1.0) * 1.15


def test_ratio_to_the_bound_shrinks_with_memory():
    ratios = []
    for S in (15, 55, 210, 820):
        k = io_sim.k_for_memory(S)
        N = 60 * k * k
        r = io_sim.simulate_tbs(N, 1, S)
        ratios.append(r["A"] / r["lower_bound"])
    assert all(a > b for a, b in zip(ratios, ratios[1:])) and ratios[-1] < 1.12


def test_tiled_scheme_at_the_library_shape():
    # b = 64, S = 24576: k = 4; N = M = 4096 is T = 64 tile rows
    r = io_sim.simulate_tbs(4096, 4096, 24576, b=64)
    assert r["k"] == 4 and r["A_q1"] == 15 * 15 * 4 * 64 * 4096       # c = 15 for the cyclic family
    assert r["A"] >= r["lower_bound"]
    big = io_sim.simulate_tbs(32768, 64, 24576, b=64)
    assert big["A"] / big["lower_bound"] < 1.25              # sqrt(4/3) = 1.155 plus lower-order terms


def test_gram_and_syr2k_counts():
    g = io_sim.simulate_gram(7, 900, 55)
    assert g == io_sim.simulate_tbs(900, 7, 55)
    r = io_sim.simulate_syr2k(4000, 2, 136)
    assert r["triangle_AB"] < r["square_AB"]
    k, s = r["k"], r["square_side"]
    assert k * (k - 1) // 2 + 2 * k <= 136 and s * s + 4 * s <= 136
    assert abs(r["triangle_AB"] / r["square_AB"] - (s / (k - 1.0))) < 0.1


def test_lbc_terms_of_section_5_2_2():
    N, S = 4096, 55
    b = math.isqrt(N)
    r = io_sim.simulate_lbc(N, S, b)
    t1, t2, t3, t4 = r["terms"]
    assert abs(r["panel"] - t1) < 1e-9 * t1
    assert abs(r["solve"] - t2) / t2 < 2.0 / (N // b)        # sum over panels of rows * b^2 / sqrt S vs b N^2 / (2 sqrt S)
    # the update's C loads are the trailing matrix re-loaded every iteration: N^3/(6b) in the leading term
    assert abs(r["update_C"] - t4) / t4 < 0.05
    # its A loads: at least the Cholesky lower bound's share, at most the recursion bound summed over panels
    k = r["k"]
    assert r["update_A"] >= 0.9 * t3
    assert r["update_A"] <= N ** 3 / (3.0 * (k - 1)) * 1.25
    assert r["total"] >= r["lower_bound"]
    # a larger block trades term (4) against terms (1) and (2)
    r2 = io_sim.simulate_lbc(N, S, 4 * b)
    assert r2["update_C"] < r["update_C"] and r2["panel"] > r["panel"]
