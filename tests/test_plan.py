"""The library's Triangle Block plan, expanded on the host with the index arithmetic the kernels use:
every tile of the lower triangle is produced exactly once, the triangle blocks are those of the
paper's cyclic family (compared with the CPU replay of Algorithm 4), and the reported element
counts agree with the cost formulas of Sections 5.1.3 / 5.1.4."""
import math
import os

import numpy as np
import pytest

from oracle import tbs_schedule as ts
from paper_2202_10217_amd import binding as tb

B, K = 64, 4
KIND_TRI, KIND_RECT, KIND_DIAG, KIND_EMPTY = 0, 1, 2, 3


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(tb.LIB_PATH):
        from paper_2202_10217_amd import build
        build.build()
    tb.load()


def _tiles_of(items):
    """Yields (row tile, column tile) for every tile the work list updates."""
    for kind, nrow, ncol, *rows in items.tolist():
        if kind == KIND_TRI:
            R = rows[:nrow]
            assert all(r >= 0 for r in R) and all(r < 0 for r in rows[nrow:])
            for u in range(nrow):
                for v in range(u):
                    assert R[u] > R[v]                     # zone order is increasing row order
                    yield R[u], R[v]
        elif kind == KIND_RECT:
            cols = [r for r in rows[:3] if r >= 0]
            rws = [r for r in rows[3:5] if r >= 0]
            assert len(cols) == ncol and len(rws) == nrow and nrow >= 1 and ncol >= 1
            produced = 0
            for r in rws:
                for q in cols:
                    if q < r:
                        produced += 1
                        yield r, q
            assert produced > 0                             # an item flagged rectangle is never empty
        elif kind == KIND_DIAG:
            assert nrow == 1
            yield rows[0], rows[0]
        else:
            assert kind == KIND_EMPTY


@pytest.mark.parametrize("square", [False, True])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 128, 200, 256, 700, 768, 1000, 2048, 4096, 4100, 6000,
                               16384, 20000])
def test_every_lower_tile_exactly_once(N, square):
    items = tb.tbs_syrk_lower_enumerate(tb.TBS_F64, N, square)
    T = (N + B - 1) // B
    count = np.zeros((T, T), dtype=np.int32)
    for r, q in _tiles_of(items):
        assert 0 <= q <= r < T
        count[r, q] += 1
    il = np.tril_indices(T)
    assert (count[il] == 1).all()
    assert count.sum() == T * (T + 1) // 2
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, N, 10, square)
    assert info["n_items"] == len(items) and info["tile_rows"] == T
    assert info["n_diag_tiles"] == T
    if square:
        assert info["n_tri_blocks"] == 0


def test_empty_matrix():
    assert len(tb.tbs_syrk_lower_enumerate(tb.TBS_F64, 0)) == 0


@pytest.mark.parametrize("N", [768, 4096, 16384, 12345])
def test_triangle_blocks_are_those_of_the_cyclic_family(N):
    # the CPU replay of Algorithm 4 on a T x 1 problem with b = 1 lists the blocks of every level
    T = N // B                                              # full tiles only: the replay has no ragged edge
    items = tb.tbs_syrk_lower_enumerate(tb.TBS_F64, T * B)
    io = ts.tbs_syrk(np.zeros((T, 1)), np.zeros((T, T)), K, 1)
    want = sorted(tuple(off + r for r in R) for _, off, R in io.blocks)
    c = ts.choose_c(T // K, K)
    got = sorted(tuple(row[3:3 + K]) for row in items.tolist() if row[0] == KIND_TRI and row[1] == K
                 and _is_family_block(row[3:3 + K]))
    # base-zone triangle blocks (consecutive rows) are the library's own treatment of the recursion
    # base; every block of the replay must be among the library's, and conversely every
    # non-consecutive block of the library is one of the replay's
    assert set(want) <= set(tuple(row[3:3 + K]) for row in items.tolist() if row[0] == KIND_TRI)
    assert set(got) <= set(want)
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, T * B, 7)
    assert info["c"] == c and info["l"] == T - K * c and info["k"] == K and info["b"] == B
    assert info["A_elems_top"] == c * c * K * B * 7         # Q1 = c^2 k b M


def _is_family_block(R):
    return not all(R[u + 1] == R[u] + 1 for u in range(len(R) - 1))


def test_query_numbers_against_the_formulas():
    N, M = 4096, 4096
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, N, M)
    S = ts.tiled_tbs_S(K, B)
    assert info["S_C_elems"] == S == 24576
    assert info["S_res_elems"] == S + 2 * K * B * 16
    assert math.isclose(info["tbs_bound_elems"], ts.syrk_lower_bound(N, M, S), rel_tol=1e-12)
    assert math.isclose(info["tiled_lead_elems"], ts.tiled_tbs_A_leading(N, M, K, B), rel_tol=1e-12)
    assert math.isclose(info["square_elems"], ts.square_A_volume(N, M, math.sqrt(S)), rel_tol=1e-12)
    assert info["C_elems"] == N * (N + 1) / 2
    assert (info["c"], info["l"], info["levels"]) == (15, 4, 2)
    # the whole plan loads less of A than square blocks of the same area would, and the triangle
    # blocks alone stay under the tiled bound N^2 M / ((k-1) b)
    sq = tb.tbs_syrk_lower_query(tb.TBS_F64, N, M, square=True)
    assert info["A_elems"] < sq["A_elems"]
    assert info["A_elems_top"] <= info["tiled_lead_elems"]
    assert info["A_elems"] >= info["tbs_bound_elems"]       # no schedule beats the lower bound
    # large N: the plan's total approaches the tiled leading term (lower order terms are O(NM log N))
    big = tb.tbs_syrk_lower_query(tb.TBS_F64, 32768, 64)
    assert big["A_elems"] < 1.08 * big["tiled_lead_elems"]
    assert big["A_elems"] / big["tbs_bound_elems"] < 1.25   # sqrt(4/3) = 1.155 plus lower order terms
