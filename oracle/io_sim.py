"""TEST INFRASTRUCTURE -- I/O simulator: the paper's schedules replayed without arithmetic, for any
memory size S, against its theorems.

`tbs_schedule.py` executes Algorithms 4 and 5 on real matrices (to show they compute the right thing)
and counts loads on the way; that limits it to small sizes.  Here only the loads are counted, by the
same recursion, so that N, M and S can be large: the element-granular scheme with S = k(k+1)/2
(Section 5.1), the tiled scheme with S = b^2 k(k-1)/2 (Section 5.1.4), Large Block Cholesky
(Section 5.2) and the two kernels of the paper's conclusion as this library schedules them (Gram: the
scheme applied to the transpose; SYR2K: square blocks, or triangle blocks that stream both matrices).

Model (Section 3): a block of C stays in fast memory while the needed rows of A stream past, one column
index at a time; cost = elements moved from slow to fast memory; stores are not counted.
"""
import math

from . import tbs_schedule as ts


def k_for_memory(S: int) -> int:
    """Largest k with k(k+1)/2 <= S: the triangle side of the element-granular scheme (Section 5.1:
    k(k-1)/2 entries of C plus k entries of one column of A)."""
    k = int((math.isqrt(8 * S + 1) - 1) // 2)
    while (k + 1) * (k + 2) // 2 <= S:
        k += 1
    while k * (k + 1) // 2 > S:
        k -= 1
    return k


def square_side_for_memory(S: int) -> int:
    """Side s of the square blocks of the scheme the paper compares with: s^2 entries of C plus 2s of A."""
    s = math.isqrt(S)
    while s > 1 and s * s + 2 * s > S:
        s -= 1
    return max(s, 1)


def _ooc_counts(n: int, s: int, M: int, io: dict):
    """Square blocks on an n x n triangle (diagonal included): groups of s rows."""
    sizes = [min(s, n - g) for g in range(0, n, s)]
    for a, ra in enumerate(sizes):
        for rb in sizes[:a]:
            io["C"] += ra * rb
            io["A"] += (ra + rb) * M
        io["C"] += ra * (ra + 1) // 2
        io["A"] += ra * M


def _last_rows_counts(first: int, n: int, s: int, M: int, io: dict):
    """Square blocks for rows [first, n) against all columns j <= row."""
    if n <= first:
        return
    rows = [min(s, n - g) for g in range(first, n, s)]
    cols = [min(s, first - g) for g in range(0, first, s)]
    for ra in rows:
        for rb in cols:
            io["C"] += ra * rb
            io["A"] += (ra + rb) * M
    _ooc_counts(n - first, s, M, io)


def tbs_counts(N: int, M: int, k: int, b: int = 1, s: int = None, families: str = "cyclic", io: dict = None,
               level: int = 0) -> dict:
    """Loads of Algorithm 4 (b = 1) / its tiled form (b > 1) on an N x M problem: the recursion of
    tbs_schedule.tbs_syrk without the arithmetic.  Returns A, C (elements loaded), A_q1 (top-level
    triangle blocks), blocks (triangle blocks, all levels), levels."""
    if io is None:
        io = {"A": 0, "C": 0, "A_q1": 0, "blocks": 0, "levels": 0}
    if s is None:
        s = max(1, math.isqrt(b * b * k * (k - 1) // 2))
    family, c = ("cyclic", ts.choose_c(N // (k * b), k)) if families == "cyclic" else ts.choose_family(N // (k * b), k)
    if c < k - 1:
        _ooc_counts(N, s, M, io)
        return io
    io["levels"] = max(io["levels"], level + 1)
    covered = c * k * b
    _last_rows_counts(covered, N, s, M, io)
    for _ in range(k):
        tbs_counts(c * b, M, k, b, s, families, io, level + 1)
    io["blocks"] += c * c
    io["C"] += c * c * b * b * k * (k - 1) // 2
    io["A"] += c * c * k * b * M
    if level == 0:
        io["A_q1"] += c * c * k * b * M
    return io


def simulate_tbs(N: int, M: int, S: int, b: int = 1) -> dict:
    """The Triangle Block Scheme with fast memory S.  b = 1: element-granular, k from S = k(k+1)/2;
    b > 1: tiled, k the largest with b^2 k(k-1)/2 <= S (Section 5.1.4; the streamed column of A is not
    counted there).  Returns the counted volumes next to the paper's figures for the same S."""
    if b == 1:
        k = k_for_memory(S)
    else:
        k = 2
        while b * b * (k + 1) * k // 2 <= S:
            k += 1
    s = square_side_for_memory(S)
    io = tbs_counts(N, M, k, b, s)
    sq = {"A": 0, "C": 0}
    _ooc_counts(N, s, M, sq)
    return {"k": k, "b": b, "square_side": s, "A": io["A"], "C": io["C"], "A_q1": io["A_q1"],
            "blocks": io["blocks"], "levels": io["levels"],
            "lower_bound": ts.syrk_lower_bound(N, M, S),                       # corollary of Section 4.1
            "theorem_rhs": ts.tbs_volume_leading(N, M, S),                     # Section 5.1.3, without O(NM log N)
            "recursion_bound_A": N * N * M / ((k - 1.0) * b),                  # N^2 M / ((k-1) b)
            "square_A": sq["A"], "square_model_A": ts.square_A_volume(N, M, s)}


def simulate_gram(N: int, M: int, S: int, b: int = 1) -> dict:
    """A^T A for an N x M matrix: the scheme applied to the transpose (order M, contraction N)."""
    return simulate_tbs(M, N, S, b)


def simulate_syr2k(N: int, M: int, S: int) -> dict:
    """C += A B^T + B A^T with fast memory S, two ways.  Square blocks of side s (s^2 + 4s <= S): a
    block streams s rows and s columns of both matrices, 4 s M per off-diagonal block.  Triangle blocks
    of side k (k(k-1)/2 + 2k <= S): a block streams its k rows of both matrices once, 2 k M per
    k(k-1)/2 entries.  The counts use the same partitions as the SYRK schemes with twice the A-volume;
    the ratio triangle/square tends to 1/sqrt(2) as for SYRK."""
    k = 2
    while (k + 1) * k // 2 + 2 * (k + 1) <= S:
        k += 1
    s = 1
    while (s + 1) * (s + 1) + 4 * (s + 1) <= S:
        s += 1
    tri = tbs_counts(N, M, k, 1, s)
    sq = {"A": 0, "C": 0}
    _ooc_counts(N, s, M, sq)
    return {"k": k, "square_side": s, "triangle_AB": 2 * tri["A"], "square_AB": 2 * sq["A"], "C": tri["C"],
            "lower_order": 2.0 * N * M}


def simulate_lbc(N: int, S: int, b: int, tile: int = 1) -> dict:
    """Large Block Cholesky (Algorithm 5) with block size b: the trailing updates are counted by the
    replay above (terms (3) and (4) of Section 5.2.2: A and C loads of every TBS call); the panel
    factorisation and the triangular solve, which the paper cites (OOC_CHOL, OOC_TRSM) with their costs
    b^3/(3 sqrt S) and rows * b^2 / sqrt S, enter through those formulas (terms (1) and (2))."""
    k = k_for_memory(S) if tile == 1 else max(2, int((1 + math.isqrt(1 + 8 * S // (tile * tile))) // 2))
    rS = math.sqrt(S)
    out = {"panel": 0.0, "solve": 0.0, "update_A": 0, "update_C": 0, "k": k}
    for i0 in range(0, N, b):
        nb = min(b, N - i0)
        rest = N - i0 - nb
        out["panel"] += nb ** 3 / (3.0 * rS)
        out["solve"] += rest * nb * nb / rS
        if rest > 0:
            io = tbs_counts(rest, nb, k, tile)
            out["update_A"] += io["A"]
            out["update_C"] += io["C"]
    out["terms"] = ts.lbc_terms(N, b, S)
    out["total"] = out["panel"] + out["solve"] + out["update_A"] + out["update_C"]
    out["lower_bound"] = ts.cholesky_lower_bound(N, S)
    return out
