"""TEST INFRASTRUCTURE -- the paper's schedules replayed on the CPU, slowly and literally.

Nothing here is used by the GPU path.  It serves three purposes in the tests:
  * it shows that the Triangle Block Scheme (Section 5.1, Algorithm 4, and the
    tiled form of Section 5.1.4) performs exactly the operations of Algorithm 1,
    by running it and comparing with the plain triple loop;
  * it counts the elements the schedule loads, for comparison with the cost
    formulas of Section 5.1.3 / 5.1.4 (Q1 = c^2 k b M, C loaded once);
  * it lists the triangle blocks of every recursion level, which pins the index
    arithmetic of the GPU library's planner;
  * it replays Large Block Cholesky (Section 5.2.1, Algorithm 5) with that scheme as
    trailing update and counts the update's loads (terms (3) and (4) of Section 5.2.2).
It also holds the closed forms of Sections 3.2, 4.1, 4.2 and 5.2.2.

Readings of the paper taken here (the text is ambiguous or silent):
  * integer ranges in Algorithms 4 and 5 are half-open: zone i is rows
    [i*c, (i+1)*c);
  * "largest integer coprime with q below N/k" means <= floor(N/k); being coprime
    with q (product of primes <= k-2) is tested as gcd(c, d) == 1 for all d in
    [2, k-2], which is the condition the validity lemma uses; for k <= 3 every c
    qualifies;
  * "the last l rows of C" are rows [c*k, N) with all their columns j <= row;
  * the recursion on a diagonal zone keeps k (and b) and picks its own c;
  * the square-block algorithm the paper cites but does not spell out (OOC_SYRK)
    is taken as: cut the rows into groups of s; a block is a pair of groups
    (I >= J); an off-diagonal block loads the 2s rows of A column by column
    (2sM elements, Section 5.1.3), a diagonal block loads its s rows.
"""
import math
from typing import Callable, Dict, List, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# Section 3.2: triangle blocks
# ----------------------------------------------------------------------------


def triangle_block(R) -> List[Tuple[int, int]]:
    """TB(R): all pairs (r, r') of R with r > r' (definition of a triangle block)."""
    R = sorted(R)
    return [(R[a], R[b]) for a in range(len(R)) for b in range(a)]


def sigma(m: int) -> int:
    """Smallest side length of a triangle block holding at least m pairs (lemma of Section 3.2)."""
    if m == 0:
        return 0
    return math.ceil(math.sqrt(0.25 + 2 * m) + 0.5)


# ----------------------------------------------------------------------------
# Section 5.1.1 / 5.1.2: indexing families
# ----------------------------------------------------------------------------


def cyclic_f(i: int, j: int, u: int, c: int) -> int:
    """The cyclic (c,k)-indexing family: f(0) = j, f(u) = (i + j(u-1)) mod c for u > 0."""
    return j if u == 0 else (i + j * (u - 1)) % c


def is_valid_family(f: Callable[[int, int, int], int], c: int, k: int) -> bool:
    """Validity by the definition: no two distinct (i,j) agree at two positions u != v."""
    for u in range(k):
        for v in range(u + 1, k):
            seen = set()
            for i in range(c):
                for j in range(c):
                    key = (f(i, j, u), f(i, j, v))
                    if key in seen:
                        return False
                    seen.add(key)
    return True


def coprime_condition(c: int, k: int) -> bool:
    """c coprime with every integer of [2, k-2] (hypothesis of the validity lemma, minus c >= k-1)."""
    return all(math.gcd(c, d) == 1 for d in range(2, k - 1))


def choose_c(upper: int, k: int) -> int:
    """Largest c <= upper satisfying the coprimality condition; 0 if upper <= 0."""
    c = upper
    while c > 0 and not coprime_condition(c, k):
        c -= 1
    return max(c, 0)


def poly_mul_mod(a: int, b: int, m: int) -> int:
    """Product of two polynomials over GF(2) (bit t = coefficient of x^t) modulo x^m + x + 1."""
    r = 0
    while b:
        if b & 1:
            r ^= a
        b >>= 1
        a <<= 1
        if a >> m:
            a ^= (1 << m) | 3
    return r


def xor_f(i: int, j: int, u: int, c: int) -> int:
    """An indexing family for c = 2^m that is not in the paper (its Section 5.1.2 gives the cyclic one,
    which needs c odd for k >= 4): f(0) = j, f(u) = i XOR (j * a_u) for u > 0, with a_u = u - 1 read as a
    polynomial over GF(2) and the product taken modulo x^m + x + 1.  It is valid by the definition of
    Section 5.1.1 whenever the differences a_u XOR a_v are invertible modulo that polynomial; for
    k <= 4 these are 1, x and x + 1, which always are (the polynomial has constant term 1 and an odd
    number of terms).  Validity is checked by brute force in the tests, not taken from this argument."""
    m = c.bit_length() - 1
    assert c == 1 << m
    return j if u == 0 else i ^ poly_mul_mod(j, u - 1, m)


def choose_family(upper: int, k: int) -> Tuple[str, int]:
    """The family and modulus for zones of `upper` = floor(rows / k) rows: the cyclic family with the
    largest admissible c, or the XOR family with the largest power of two if that covers more rows."""
    c = choose_c(upper, k)
    if k <= 4 and upper >= 4:
        c2 = 1 << (upper.bit_length() - 1)
        if c2 > c and c2 >= k - 1:
            return "xor", c2
    return "cyclic", c


def block_rows(i: int, j: int, c: int, k: int, family: str = "cyclic") -> List[int]:
    """R^{i,j} = { u*c + f^{i,j}(u) : 0 <= u < k } (Equation 1)."""
    f = cyclic_f if family == "cyclic" else xor_f
    return [u * c + f(i, j, u, c) for u in range(k)]


# ----------------------------------------------------------------------------
# Algorithms 3 and 4 replayed, with an I/O counter
# ----------------------------------------------------------------------------


class IOCount:
    def __init__(self):
        self.A = 0          # elements of A loaded
        self.C = 0          # elements of C loaded
        self.A_tri = 0      # part of A loaded by triangle blocks (all levels)
        self.A_q1 = 0       # part of A loaded by the top-level triangle blocks (Q1)
        self.blocks: List[Tuple[int, int, List[int]]] = []   # (level, row offset in tiles, tile rows R)


def _update_pair(A, C, rows_u, rows_v, alpha):
    """One C sub-block: rows_u x rows_v += alpha * A[rows_u] A[rows_v]^T (the M-loop of Algorithm 3)."""
    C[np.ix_(rows_u, rows_v)] += alpha * (A[rows_u, :] @ A[rows_v, :].T)


def ooc_syrk(A, C, rows: np.ndarray, s: int, alpha: float, io: IOCount):
    """Square-block out-of-core SYRK on C[rows, rows] (lower part incl. diagonal)."""
    M = A.shape[1]
    groups = [rows[g:g + s] for g in range(0, len(rows), s)]
    for a, Ra in enumerate(groups):
        for b_, Rb in enumerate(groups[:a + 1]):
            if a == b_:
                io.C += len(Ra) * (len(Ra) + 1) // 2
                io.A += len(Ra) * M
                blk = alpha * (A[Ra, :] @ A[Ra, :].T)
                for x, r in enumerate(Ra):
                    C[r, Ra[:x + 1]] += blk[x, :x + 1]
            else:
                io.C += len(Ra) * len(Rb)
                io.A += (len(Ra) + len(Rb)) * M
                _update_pair(A, C, Ra, Rb, alpha)


def ooc_syrk_last_rows(A, C, rows_all: np.ndarray, first: int, s: int, alpha: float, io: IOCount):
    """Square blocks for rows rows_all[first:] against all columns j <= row of the same index set."""
    M = A.shape[1]
    last = rows_all[first:]
    if len(last) == 0:
        return
    row_groups = [last[g:g + s] for g in range(0, len(last), s)]
    head = rows_all[:first]
    col_groups = [head[g:g + s] for g in range(0, len(head), s)]
    for Ra in row_groups:
        for Rb in col_groups:
            io.C += len(Ra) * len(Rb)
            io.A += (len(Ra) + len(Rb)) * M
            _update_pair(A, C, Ra, Rb, alpha)
    ooc_syrk(A, C, last, s, alpha, io)


def tbs_syrk(A: np.ndarray, C: np.ndarray, k: int, b: int = 1, s: int = None,
             alpha: float = 1.0, io: IOCount = None, _rows=None, _level=0, families: str = "cyclic") -> IOCount:
    """Algorithm 4 (b = 1) and its tiled form (b > 1): C[lower] += alpha * A A^T, in place.

    `s` is the side of the square blocks used where the paper calls OOC_SYRK
    (default: the side whose area equals the triangle block's, rounded down).
    families = "cyclic": the paper's family at every level; "auto": choose_family() at every level.
    """
    if io is None:
        io = IOCount()
    N_all, M = A.shape
    rows = np.arange(N_all) if _rows is None else _rows
    N = len(rows)
    if s is None:
        s = max(1, int(math.isqrt(b * b * k * (k - 1) // 2)))
    family, c = ("cyclic", choose_c(N // (k * b), k)) if families == "cyclic" else choose_family(N // (k * b), k)
    if c < k - 1:                               # c too small: square blocks only
        ooc_syrk(A, C, rows, s, alpha, io)
        return io
    covered = c * k * b
    ooc_syrk_last_rows(A, C, rows, covered, s, alpha, io)          # the last l rows
    for z in range(k):                                              # diagonal zones
        tbs_syrk(A, C, k, b, s, alpha, io, rows[z * c * b:(z + 1) * c * b], _level + 1, families)
    for i in range(c):                                              # all c^2 blocks
        for j in range(c):
            R = block_rows(i, j, c, k, family)                      # tile rows within this zone
            io.blocks.append((_level, int(rows[0]) // b, R))
            tiles = [rows[r * b:(r + 1) * b] for r in R]
            io.C += b * b * k * (k - 1) // 2                        # load C[TB(R)]
            io.A += k * b * M                                       # k*b elements per column of A
            io.A_tri += k * b * M
            if _level == 0:
                io.A_q1 += k * b * M
            for u in range(k):
                for v in range(u):
                    _update_pair(A, C, tiles[u], tiles[v], alpha)
    return io


# ----------------------------------------------------------------------------
# Section 5.2.1, Algorithm 5: Large Block Cholesky
# ----------------------------------------------------------------------------


def lbc_cholesky(S: np.ndarray, b: int, k: int, tile: int = 1, io: IOCount = None, families: str = "cyclic") -> IOCount:
    """Algorithm 5, in place on the lower triangle of S: for every block of b columns, the Cholesky
    factor of the diagonal block, the triangular solve of the block column below it, and the
    trailing update C <- C - X X^T by the Triangle Block Scheme (tbs_syrk with alpha = -1).

    The paper cites the first two steps (OOC_CHOL, OOC_TRSM) without spelling them out; they are
    done here by Algorithm 2's own operations (column by column), and their loads are not counted:
    `io` receives the loads of the trailing updates only (terms (3) and (4) of Section 5.2.2), per
    panel in io.per_panel as (rows of the trailing matrix, A elements, C elements).
    Ranges are half-open and the last block may be narrower (the paper assumes b | N)."""
    if io is None:
        io = IOCount()
    io.per_panel = []
    N = S.shape[0]
    for i0 in range(0, N, b):
        i1 = min(i0 + b, N)
        for j in range(i0, i1):                         # A[I0, I0] <- CHOL, A[I1, I0] <- TRSM: Algorithm 2
            S[j, j] = math.sqrt(S[j, j])                # restricted to the columns of the block
            S[j + 1:, j] /= S[j, j]
            for jj in range(j + 1, i1):
                S[jj:, jj] -= S[jj:, j] * S[jj, j]
        if i1 < N:
            a0, c0 = io.A, io.C
            tbs_syrk(S[i1:, i0:i1], S[i1:, i1:], k, tile, alpha=-1.0, io=io, families=families)
            io.per_panel.append((N - i1, io.A - a0, io.C - c0))
    return io


# ----------------------------------------------------------------------------
# Closed forms
# ----------------------------------------------------------------------------


def syrk_lower_bound(N, M, S):
    """Corollary of Section 4.1: Q_SYRK >= N^2 M / (sqrt(2) sqrt(S))."""
    return N * N * M / (math.sqrt(2.0) * math.sqrt(S))


def cholesky_lower_bound(N, S):
    """Corollary of Section 4.2: Q_Chol >= N^3 / (3 sqrt(2) sqrt(S))."""
    return N ** 3 / (3.0 * math.sqrt(2.0) * math.sqrt(S))


def tbs_volume_leading(N, M, S):
    """Theorem of Section 5.1.3 without the O(NM log N) term."""
    return N * N * M / (math.sqrt(2.0) * math.sqrt(S)) + N * N / 2.0


def tiled_tbs_A_leading(N, M, k, b):
    """Section 5.1.4: A-traffic bound N^2 M / ((k-1) b)."""
    return N * N * M / ((k - 1.0) * b)


def tiled_tbs_S(k, b):
    """Section 5.1.4: S = b^2 k (k-1) / 2."""
    return b * b * k * (k - 1) // 2


def square_A_volume(N, M, s):
    """Section 5.1.3: every s x s block loads 2 s M elements, N^2/(2 s^2) blocks: N^2 M / s."""
    return N * N * M / float(s)


def lbc_terms(N, b, S):
    """The four terms of the LBC cost (Section 5.2.2): panel, TRSM, TBS update, trailing re-load."""
    rS = math.sqrt(S)
    return (b * b * N / (3.0 * rS), b * N * N / (2.0 * rS),
            N ** 3 / (3.0 * math.sqrt(2.0) * rS), N ** 3 / (6.0 * b))


def I_star(X):
    """Section 4.1: optimal triangle side of the relaxed problem P''(X)."""
    return 2.0 / 3.0 + math.sqrt(1.0 + 6.0 * X) / 3.0


def H2(X):
    """Section 4.1: optimum of P''(X), (1/108)(sqrt(1+6X)-1)^2 (2 sqrt(1+6X)+1)."""
    r = math.sqrt(1.0 + 6.0 * X)
    return (r - 1.0) ** 2 * (2.0 * r + 1.0) / 108.0


def H_max_bound(X):
    """Theorem of Section 4.1: at most sqrt(2)/(3 sqrt(3)) X^{3/2} operations touch X data."""
    return math.sqrt(2.0) / (3.0 * math.sqrt(3.0)) * X ** 1.5
