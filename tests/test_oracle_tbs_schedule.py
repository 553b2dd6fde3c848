"""Pins for the CPU replay of the Triangle Block Scheme (Sections 3.2, 5.1) and for the closed
forms of the paper's bounds: the definitions are checked by brute force, the replay against the
plain triple loop (bit for bit on integer data) and against the paper's cost formulas."""
import math

import numpy as np
import pytest

import oracle
from oracle import tbs_schedule as ts
from paper_2202_10217_amd import inputs


# ---- Section 3.2 ---------------------------------------------------------------------------------

def test_sigma_is_the_smallest_side_by_brute_force():
    for m in range(0, 400):
        s = 0
        while s * (s - 1) // 2 < m:
            s += 1
        assert ts.sigma(m) == s


def test_triangle_block_size():
    R = [7, 2, 11, 5, 3]
    tb = ts.triangle_block(R)
    assert len(tb) == len(R) * (len(R) - 1) // 2
    assert all(r > r2 and r in R and r2 in R for r, r2 in tb)
    assert len(set(tb)) == len(tb)


# ---- Section 5.1.1 / 5.1.2 -----------------------------------------------------------------------

def test_indexing_family_anchor_points():
    c, k = 7, 5
    for i in range(c):
        for j in range(c):
            assert ts.cyclic_f(i, j, 0, c) == j and ts.cyclic_f(i, j, 1, c) == i
            R = ts.block_rows(i, j, c, k)
            assert (i + c, j) in ts.triangle_block(R)        # the block holds element (i+c, j) of C


def test_validity_lemma_by_brute_force():
    # lemma: c >= k-1 and coprime with [2, k-2]  =>  valid.  Brute force also shows the converse
    # for the cyclic family in this range.
    for k in range(2, 8):
        for c in range(max(k - 1, 1), 26):
            valid = ts.is_valid_family(lambda i, j, u: ts.cyclic_f(i, j, u, c), c, k)
            assert valid == ts.coprime_condition(c, k), (c, k)


def test_a_non_coprime_c_really_collides():
    c, k = 4, 4                                             # gcd(4, 2) != 1
    assert not ts.is_valid_family(lambda i, j, u: ts.cyclic_f(i, j, u, c), c, k)
    blocks = [set(ts.triangle_block(ts.block_rows(i, j, c, k))) for i in range(c) for j in range(c)]
    assert sum(len(b) for b in blocks) > len(set().union(*blocks))


@pytest.mark.parametrize("c,k", [(3, 4), (5, 4), (15, 4), (5, 5), (7, 5), (7, 8), (13, 8), (5, 3), (4, 3), (6, 2)])
def test_blocks_partition_the_square_zones(c, k):
    seen = {}
    for i in range(c):
        for j in range(c):
            for (r, r2) in ts.triangle_block(ts.block_rows(i, j, c, k)):
                assert (r, r2) not in seen
                seen[r, r2] = (i, j)
    # exactly the pairs lying in different zones: k(k-1)/2 zones of c*c elements
    assert len(seen) == c * c * k * (k - 1) // 2
    for (r, r2) in seen:
        assert r // c > r2 // c


# ---- the XOR family for c = 2^m (not in the paper; valid by the definition of Section 5.1.1) -------

def test_polynomial_product_against_hand_values():
    # modulo x^3 + x + 1:  x * x^2 = x^3 = x + 1;  (x + 1)(x^2 + 1) = x^3 + x^2 + x + 1 = x^2
    assert ts.poly_mul_mod(0b010, 0b100, 3) == 0b011
    assert ts.poly_mul_mod(0b011, 0b101, 3) == 0b100
    # modulo x^2 + x + 1 (the field of four elements): x * x = x + 1, x (x + 1) = 1
    assert ts.poly_mul_mod(2, 2, 2) == 3 and ts.poly_mul_mod(2, 3, 2) == 1
    for m in range(2, 7):
        for a in range(1 << m):
            assert ts.poly_mul_mod(a, 1, m) == a and ts.poly_mul_mod(a, 0, m) == 0
            for b in range(1 << m):
                assert ts.poly_mul_mod(a, b, m) == ts.poly_mul_mod(b, a, m) < (1 << m)


@pytest.mark.parametrize("c", [4, 8, 16, 32, 64])
@pytest.mark.parametrize("k", [2, 3, 4])
def test_xor_family_is_valid_by_brute_force(c, k):
    assert ts.is_valid_family(lambda i, j, u: ts.xor_f(i, j, u, c), c, k)
    seen = set()
    for i in range(c):
        for j in range(c):
            for pair in ts.triangle_block(ts.block_rows(i, j, c, k, "xor")):
                assert pair not in seen
                seen.add(pair)
    assert len(seen) == c * c * k * (k - 1) // 2            # exactly the pairs in different zones
    assert all(r // c > r2 // c for r, r2 in seen)


def test_xor_family_anchor_points():
    c = 16
    assert [ts.xor_f(5, 9, u, c) for u in range(4)] == [9, 5, 5 ^ 9, 5 ^ ((9 << 1) ^ 0b10011) & 15]
    assert ts.block_rows(0, 0, c, 4, "xor") == [0, 16, 32, 48]
    assert ts.block_rows(3, 0, c, 4, "xor") == [0, 19, 35, 51]           # j = 0: every f(u > 0) is i


def test_choose_family():
    assert ts.choose_family(16, 4) == ("xor", 16) and ts.choose_family(15, 4) == ("cyclic", 15)
    assert ts.choose_family(64, 4) == ("xor", 64) and ts.choose_family(63, 4) == ("cyclic", 63)
    assert ts.choose_family(4, 4) == ("xor", 4) and ts.choose_family(5, 4) == ("cyclic", 5)
    assert ts.choose_family(3, 4) == ("cyclic", 3) and ts.choose_family(0, 4) == ("cyclic", 0)
    assert ts.choose_family(16, 8) == ("cyclic", 13)       # written out for k <= 4 only
    for n in range(1, 200):
        fam, c = ts.choose_family(n, 4)
        assert c <= n and c >= ts.choose_c(n, 4)
        if fam == "xor":
            assert c & (c - 1) == 0 and c > ts.choose_c(n, 4)


@pytest.mark.parametrize("N,M,b", [(16, 3, 1), (64, 4, 1), (67, 3, 1), (128, 2, 2), (256, 2, 1)])
def test_tbs_with_the_xor_family_equals_algorithm_1(N, M, b):
    A = inputs.small_int_matrix(N, M, seed=N + 3)
    C0 = inputs.symmetric_uniform(N, seed=N + 4, int_range=(-5, 5))
    C_ref = C0.copy()
    oracle.syrk_lower(A, C_ref, 1.0, 1.0)
    C = C0.copy()
    io = ts.tbs_syrk(A, C, 4, b, families="auto")
    il = np.tril_indices(N)
    assert np.array_equal(C[il], C_ref[il])
    assert io.C == N * (N + 1) // 2
    fam, c = ts.choose_family(N // (4 * b), 4)
    assert fam == "xor" and io.A_q1 == c * c * 4 * b * M


def test_choose_c():
    assert ts.choose_c(16, 4) == 15 and ts.choose_c(15, 4) == 15
    assert ts.choose_c(64, 4) == 63 and ts.choose_c(128, 4) == 127
    assert ts.choose_c(16, 8) == 13                        # coprime with 2..6
    assert ts.choose_c(16, 3) == 16 and ts.choose_c(16, 2) == 16
    assert ts.choose_c(0, 4) == 0
    for k in range(2, 9):
        for n in range(1, 60):
            c = ts.choose_c(n, k)
            assert ts.coprime_condition(c, k) and c <= n
            assert all(not ts.coprime_condition(x, k) for x in range(c + 1, n + 1))


# ---- Algorithm 4 replayed ------------------------------------------------------------------------

@pytest.mark.parametrize("N,M,k,b", [(12, 5, 3, 1), (23, 4, 4, 1), (40, 3, 4, 1), (61, 3, 5, 1),
                                      (48, 6, 4, 2), (70, 5, 3, 4), (64, 4, 4, 4), (97, 3, 4, 3)])
def test_tbs_equals_algorithm_1_bit_for_bit(N, M, k, b):
    A = inputs.small_int_matrix(N, M, seed=N + k)
    C0 = inputs.symmetric_uniform(N, seed=N + 1, int_range=(-5, 5))
    C_ref = C0.copy()
    oracle.syrk_lower(A, C_ref, 1.0, 1.0)
    C = C0.copy()
    C[np.triu_indices(N, 1)] = np.nan
    io = ts.tbs_syrk(A, C, k, b)
    il = np.tril_indices(N)
    assert np.array_equal(C[il], C_ref[il])
    assert np.isnan(C[np.triu_indices(N, 1)]).all()
    # "loads each entry of C exactly once" (Section 5.1.3)
    assert io.C == N * (N + 1) // 2
    # Q1 = c^2 k b M for the top-level blocks (Sections 5.1.3, 5.1.4)
    c = ts.choose_c(N // (k * b), k)
    if c >= k - 1:
        assert io.A_q1 == c * c * k * b * M
        assert len([1 for lv, _, _ in io.blocks if lv == 0]) == c * c
    else:
        assert io.A_q1 == 0


def test_tbs_volume_against_the_cost_formula():
    # N^2 M/((k-1) b) + lower order terms; the lower order terms (leftover rows, recursion base)
    # are O(N M log N): bound them generously and check the leading coefficient is right.
    N, M, k, b = 360, 2, 4, 2
    A = inputs.small_int_matrix(N, M, seed=1)
    C = np.zeros((N, N))
    io = ts.tbs_syrk(A, C, k, b)
    lead = ts.tiled_tbs_A_leading(N, M, k, b)
    assert io.A_tri <= lead                                # triangle blocks alone never exceed it
    s = int(math.isqrt(ts.tiled_tbs_S(k, b)))
    assert io.A <= lead + 8 * k * N * M * math.log2(N) / s
    assert io.A >= ts.syrk_lower_bound(N, M, ts.tiled_tbs_S(k, b)) - N * M   # and respects the bound
    # square blocks of equal area cost more
    io_sq = ts.IOCount()
    ts.ooc_syrk(A, np.zeros((N, N)), np.arange(N), s, 1.0, io_sq)
    assert io_sq.A > io.A
    assert abs(io_sq.A - ts.square_A_volume(N, M, s)) <= 2 * N * M


@pytest.mark.parametrize("k,c", [(4, 35), (5, 23), (6, 25)])
def test_total_volume_theorem_of_the_element_granular_scheme(k, c):
    # Theorem of Section 5.1.3 with its S = k(k+1)/2 (the k(k-1)/2 entries of a triangle block plus one
    # column of A restricted to R): the replay of Algorithm 4 (b = 1) loads C exactly once and an amount
    # of A between the lower bound N^2 M / (sqrt(2) sqrt(S)) and N^2 M / (k-1) + O(N M log N), whose
    # ratio is sqrt(k(k+1)) / (k-1) (the theorem's "k - 1 ~ sqrt(2 S)").  tbs_volume_leading is that
    # theorem's right-hand side without the O() term: a dropped sqrt(2), a swapped S or a wrong C term
    # moves it out of the bracket below.
    N, M = k * c, 3
    A = inputs.small_int_matrix(N, M, seed=k)
    C = np.zeros((N, N))
    io = ts.tbs_syrk(A, C, k, 1)
    S = k * (k + 1) // 2
    assert io.C == N * (N + 1) // 2
    lead = ts.tbs_volume_leading(N, M, S)
    assert abs((lead - N * N / 2.0) - ts.syrk_lower_bound(N, M, S)) < 1e-9 * lead
    total = io.A + io.C
    lower_order = 4 * k * N * M * math.log2(N)
    assert lead - N <= total + N                           # never below the bound (the diagonal's N/2 aside)
    assert total <= lead * math.sqrt(k * (k + 1.0)) / (k - 1.0) + lower_order
    # and the leading coefficient is the right one: the top-level blocks alone are N^2 M / k
    assert io.A_q1 == c * c * k * M == N * N * M // k
    assert ts.syrk_lower_bound(N, M, S) < io.A_q1 * (k / (k - 1.0))


# ---- closed forms --------------------------------------------------------------------------------

def test_bound_arithmetic():
    S = ts.tiled_tbs_S(4, 64)
    assert S == 24576
    # worked values: N = M = 4096, fp64, in GB
    assert abs(ts.syrk_lower_bound(4096, 4096, S) * 8 / 1e9 - 2.48) < 0.01
    assert abs(ts.tiled_tbs_A_leading(4096, 4096, 4, 64) * 8 / 1e9 - 2.86) < 0.01
    assert abs(ts.square_A_volume(4096, 4096, math.sqrt(S)) * 8 / 1e9 - 3.51) < 0.01
    # tiled TBS is sqrt(k/(k-1)) above the bound (Section 5.1.4)
    for k in (3, 4, 5, 8):
        S = ts.tiled_tbs_S(k, 32)
        ratio = ts.tiled_tbs_A_leading(1000, 10, k, 32) / ts.syrk_lower_bound(1000, 10, S)
        assert abs(ratio - math.sqrt(k / (k - 1.0))) < 1e-12
    # Cholesky bound = SYRK bound with M = N, over 3 (|C| = N^3/6 against |S| = N^2 M/2)
    assert abs(ts.cholesky_lower_bound(500, 99) - ts.syrk_lower_bound(500, 500, 99) / 3) < 1e-6
    # LBC with b = sqrt(N): the TBS term dominates, the others are O(N^{5/2})
    N, S = 10 ** 6, 10 ** 4
    t1, t2, t3, t4 = ts.lbc_terms(N, math.isqrt(N), S)
    assert t3 > 10 * max(t1, t2, t4)
    assert abs(t4 - N ** 2.5 / 6) < 1e-6 * t4 and abs(t2 - N ** 2.5 / (2 * math.sqrt(S))) < 1e-6 * t2
    assert abs(t3 - ts.cholesky_lower_bound(N, S)) < 1e-6 * t3


def test_relaxed_optimum_closed_forms():
    for X in (3.0, 50.0, 1e4, 3e6):
        I = ts.I_star(X)
        assert abs(3 * I * I - 4 * I - (2 * X - 1)) < 1e-6 * X          # stationarity + tight constraint
        K = (I - 0.5) * (1 - 1 / I)
        assert abs(I * (I - 1) / 2 + K * I - X) < 1e-6 * X              # the data budget is used up
        assert abs(K * I * (I - 1) / 2 - ts.H2(X)) < 1e-9 * ts.H2(X) + 1e-9
        assert ts.H2(X) <= ts.H_max_bound(X)
    # with X = 3S the bound gives operational intensity sqrt(S/2) (corollary of Section 4.1)
    S = 1234.0
    assert abs(ts.H_max_bound(3 * S) / (2 * S) - math.sqrt(S / 2)) < 1e-9


# ---- Algorithm 5 (Large Block Cholesky) replayed ---------------------------------------------------
def _integer_factor(N, seed):
    rng = np.random.default_rng(seed)
    G = np.tril(rng.integers(-2, 3, size=(N, N))).astype(np.float64)
    G[np.diag_indices(N)] = rng.integers(1, 4, size=N)
    return G


@pytest.mark.parametrize("N,b,k,tile", [(48, 8, 3, 1), (96, 16, 4, 2), (100, 24, 4, 2), (130, 32, 5, 1), (64, 64, 4, 2)])
def test_lbc_recovers_an_integer_factor_exactly(N, b, k, tile):
    """Uniqueness of the Cholesky factor: S = G G^T with an integer G of positive diagonal gives back G,
    bit for bit (every intermediate value is an integer), whatever the block sizes, ragged ones included."""
    G = _integer_factor(N, 5)
    S = G @ G.T
    upper = np.triu_indices(N, 1)
    S[upper] = -77.0                                    # never read, never written
    ts.lbc_cholesky(S, b, k, tile)
    assert np.array_equal(np.tril(S), G)
    assert np.all(S[upper] == -77.0)


def test_lbc_equals_algorithm_2_on_a_random_matrix():
    import oracle
    rng = np.random.default_rng(11)
    N = 120
    X = rng.standard_normal((N, N))
    S = X @ X.T + N * np.eye(N)
    L_ref = S.copy()
    assert oracle.potrf_lower(L_ref) == 0
    L = S.copy()
    ts.lbc_cholesky(L, 24, 4, 2, families="auto")
    assert np.max(np.abs(np.tril(L) - np.tril(L_ref))) <= 1e-12 * np.max(np.abs(L_ref))


def test_lbc_volume_terms():
    """Section 5.2.2: every trailing update loads its C once, n(n+1)/2 elements for n rows (summing to the
    N^3/(6b) term), and its A volume follows the tiled TBS leading term n^2 b/((k-1) tile), the excess
    shrinking as the trailing matrix grows."""
    k, tile, b = 4, 4, 32
    N = 768
    S = _integer_factor(N, 3)
    S = S @ S.T
    io = ts.lbc_cholesky(S, b, k, tile)
    assert len(io.per_panel) == N // b - 1
    for n, a_elems, c_elems in io.per_panel:
        assert c_elems == n * (n + 1) // 2
    total_c = sum(c for _, _, c in io.per_panel)
    assert abs(total_c / (N ** 3 / (6.0 * b)) - 1.0) < 0.08
    ratios = [(n, a / ts.tiled_tbs_A_leading(n, b, k, tile)) for n, a, _ in io.per_panel if n >= 4 * k * tile]
    assert all(0.9 < r < 2.2 for _, r in ratios)
    big = [r for n, r in ratios if n >= 512]
    small = [r for n, r in ratios if n <= 192]
    assert max(big) < min(small)                        # lower-order terms fade with the size
    assert max(big) < 1.35
