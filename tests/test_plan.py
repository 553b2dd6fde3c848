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
KIND_TRI, KIND_RECT, KIND_DIAG, KIND_EMPTY, KIND_RECTDIAG, KIND_AUG = 0, 1, 2, 3, 4, 5


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(tb.LIB_PATH):
        from paper_2202_10217_amd import build
        build.build()
    tb.load()


def _tiles_of(items):
    """Yields (row tile, column tile) for every tile the work list updates.  A block that is cut along
    the contraction dimension appears as consecutive items, part 0 .. parts-1 of the same block: its
    tiles are yielded once, and the run of parts is checked."""
    rows_list = items.tolist()
    for idx, (kind, nrow, ncol, *rest) in enumerate(rows_list):
        rows, part, parts = rest[:5], rest[5], rest[6]
        assert 0 <= part < parts
        if parts > 1:                                       # the parts of a block follow each other
            head = rows_list[idx - part]
            assert head[:8] == [kind, nrow, ncol] + rows and head[8] == 0 and head[9] == parts
            assert idx - part + parts <= len(rows_list)
        if part != 0:
            continue
        if kind == KIND_TRI:
            R = rows[:nrow]
            assert all(r >= 0 for r in R) and all(r < 0 for r in rows[nrow:])
            for u in range(nrow):
                for v in range(u):
                    assert R[u] > R[v]                     # zone order is increasing row order
                    yield R[u], R[v]
        elif kind in (KIND_RECT, KIND_RECTDIAG):
            cols = [r for r in rows[:3] if r >= 0]
            rws = [r for r in rows[3:5] if r >= 0]
            assert len(cols) == ncol and len(rws) == nrow and nrow >= 1 and ncol >= 1
            produced = 0
            for r in rws:
                for q in cols:
                    if q < r or (q == r and kind == KIND_RECTDIAG):   # the second kind carries diagonal tiles
                        produced += 1
                        yield r, q
            assert produced > 0                             # an item flagged rectangle is never empty
        elif kind == KIND_DIAG:
            assert nrow == 1
            yield rows[0], rows[0]
        elif kind == KIND_AUG:
            # a triangle block on four tile rows plus two tiles, each between a row of the block and one
            # further row: (row, column) as the codes say, row >= column (equal: the diagonal tile)
            R, further1, further2, code1, code2 = rows[:4], rows[4], rest[7], rest[8], rest[9]
            assert parts == 1 and nrow == 4 and all(r >= 0 for r in R) and further1 >= 0 and further2 >= 0
            for u in range(4):
                for v in range(u):
                    assert R[u] > R[v]
                    yield R[u], R[v]
            t1 = {6: (further1, R[0]), 7: (further1, R[1])}[code1]
            t2 = {8: (further2, R[2]), 9: (R[2], further2), 10: (further2, R[3]), 11: (R[3], further2)}[code2]
            for r, q in (t1, t2):
                assert r >= q
                yield r, q
        else:
            assert kind == KIND_EMPTY


@pytest.mark.parametrize("square", [False, True])
@pytest.mark.parametrize("M", [64, 4096])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 128, 200, 256, 700, 768, 1000, 2048, 4096, 4100, 6000,
                               8192, 16384, 20000])
def test_every_lower_tile_exactly_once(N, M, square):
    # (the plan depends on M for small N: the tail of the list is cut finer when blocks are long)
    items = tb.tbs_syrk_lower_enumerate(tb.TBS_F64, N, M, square)
    T = (N + B - 1) // B
    count = np.zeros((T, T), dtype=np.int32)
    for r, q in _tiles_of(items):
        assert 0 <= q <= r < T
        count[r, q] += 1
    il = np.tril_indices(T)
    assert (count[il] == 1).all()
    assert count.sum() == T * (T + 1) // 2
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, N, M, square)
    assert info["n_items"] == len(items) and info["tile_rows"] == T
    assert info["n_diag_tiles"] == T
    if square:
        assert info["n_tri_blocks"] == 0


TUNINGS = ["0,2,3,0", "0,1,1,0", "1,2,3,0,1,3", "1,1,3,0,1,2", "1,2,2,0,1,1", "2,1,2,0,1,3", "10,2,3,1",
           "10,2,3,0,1,3", "10,1,1,0,1,1", "2,2,3,1", "1,2,3,0,2,3", "2,2,2,0,2,2", "1,1,3,0,2,1"]


@pytest.mark.parametrize("idx", range(len(TUNINGS)))
def test_every_pinned_tuning_covers_the_triangle_exactly_once(idx, monkeypatch):
    # the planner's candidates (levels, rectangle shape, base zones as triangle blocks, shape inside
    # triangular regions), pinned through the environment (the string is part of the plan-cache key,
    # so the sizes may be the same for every tuning: 1600 is used by all of them on purpose)
    from _plan_util import assert_plan_is_pinned
    monkeypatch.setenv("TBS_PLAN_TUNING", TUNINGS[idx])
    for N in (4096 + 64 * (idx + 1), 1600, 64 * (idx + 1) - 5):
        items, _ = assert_plan_is_pinned(tb, tb.TBS_F32, N, 777, TUNINGS[idx])
        T = (N + B - 1) // B
        count = np.zeros((T, T), dtype=np.int32)
        for r, q in _tiles_of(items):
            assert 0 <= q <= r < T
            count[r, q] += 1
        assert (count[np.tril_indices(T)] == 1).all() and count.sum() == T * (T + 1) // 2
        assert tb.tbs_syrk_lower_query(tb.TBS_F32, N, 777)["n_diag_tiles"] == T


AUG_TUNINGS = ["10,2,3,0,1,3,1,1,0,1,1", "10,1,2,0,1,2,1,1,0,1,1", "10,2,3,0,2,3,1,1,16,4,1"]


@pytest.mark.parametrize("family", ["", "cyclic"])
@pytest.mark.parametrize("groups", ["0", "1"])
@pytest.mark.parametrize("tuning", AUG_TUNINGS)
def test_augmented_plans_cover_the_triangle_exactly_once(tuning, groups, family, monkeypatch):
    # top-level triangle blocks that take two tiles of the diagonal zones along: every tile of the lower
    # triangle still exactly once, for both families, with and without the groups of 32, for sizes with
    # and without left-over tile rows and a ragged last tile; no block of a deeper level remains, and
    # every extra tile lies in the zone of the block's row it is attached to
    monkeypatch.setenv("TBS_PLAN_TUNING", tuning)
    monkeypatch.setenv("TBS_SYRK_DIE_GROUPS", groups)
    if family:
        monkeypatch.setenv("TBS_PLAN_FAMILY", family)
    for N in (768, 1000, 4096, 4033, 5000, 8192 + 130, 16384):
        items = tb.tbs_syrk_lower_enumerate(tb.TBS_F64, N, 1024, 0)
        info = tb.tbs_syrk_lower_query(tb.TBS_F64, N, 1024, 0)
        T = (N + B - 1) // B
        c = info["c"]
        aug = items[items[:, 0] == KIND_AUG]
        assert len(aug) == c * c and (items[:, 0] == KIND_TRI).sum() == 0 and info["levels"] == 1
        assert (family == "cyclic") == (info["family"] == 0) or c & (c - 1) != 0 or info["family"] == 0
        count = np.zeros((T, T), dtype=np.int32)
        for r, q in _tiles_of(items):
            assert 0 <= q <= r < T
            count[r, q] += 1
        assert (count[np.tril_indices(T)] == 1).all() and count.sum() == T * (T + 1) // 2
        assert info["n_diag_tiles"] == T
        for row in aug.tolist():
            R, f1, f2, c1, c2 = row[3:7], row[7], row[10], row[11], row[12]
            assert f1 // c == R[c1 - 6] // c                 # same zone as the row it is paired with
            assert f2 // c == R[2 + (c2 - 8) // 2] // c
        # the diagonal tiles of zones 1 and 3 are items of their own; those of zones 0 and 2 went with blocks
        singles = sorted(items[(items[:, 0] == KIND_DIAG) & (items[:, 8] == 0)][:, 3].tolist())
        assert singles == list(range(c, 2 * c)) + list(range(3 * c, 4 * c))
        # A elements: six panels per block at the top level (whole tile rows)
        if N % B == 0 or 4 * c < T:
            assert info["A_elems_top"] == c * c * 6 * B * 1024


@pytest.mark.parametrize("N,M", [(4096, 4096), (16384, 512), (32768, 8192), (8192, 64)])
def test_groups_of_32_top_level_blocks_share_their_tile_rows(N, M, monkeypatch):
    # the top-level blocks of the XOR family are listed in groups of 32 that lie on 28 tile rows (a
    # triangle block one level up, Section 5.1 with the L2 of a die as fast memory: 28 panels for 32
    # blocks instead of 128); TBS_SYRK_DIE_GROUPS=0 lists them in plain (i, j) order, where 32
    # consecutive blocks need many more; both orders hold the same blocks.  (By default the library groups
    # them when A is larger than the last-level cache can serve.)
    dt = tb.TBS_F32 if N == 32768 else tb.TBS_F64
    monkeypatch.setenv("TBS_SYRK_AUGMENT", "0")             # (the paper's blocks; the eight-tile ones are tested above)
    monkeypatch.setenv("TBS_SYRK_DIE_GROUPS", "1")
    items = tb.tbs_syrk_lower_enumerate(dt, N, M, 2)
    info = tb.tbs_syrk_lower_query(dt, N, M, 2)
    c = info["c"]
    assert info["family"] >= 3 and c >= 8
    top = items[:c * c]
    assert (top[:, 0] == KIND_TRI).all() and (top[:, 1] == K).all()
    rows_needed = []
    for g in range(c * c // 32):
        grp = top[32 * g:32 * g + 32, 3:3 + K]
        assert len({tuple(r) for r in grp.tolist()}) == 32
        rows_needed.append(len(np.unique(grp)))
        assert [len(np.unique(grp[:, u])) for u in range(K)] == [4, 8, 8, 8]
    assert max(rows_needed) == 28
    monkeypatch.setenv("TBS_SYRK_DIE_GROUPS", "0")
    plain = tb.tbs_syrk_lower_enumerate(dt, N, M, 2)
    assert len(plain) == len(items)
    assert {tuple(r) for r in plain[:c * c, 3:3 + K].tolist()} == {tuple(r) for r in top[:, 3:3 + K].tolist()}
    assert np.array_equal(plain[c * c:], items[c * c:])
    spread = [len(np.unique(plain[32 * g:32 * g + 32, 3:3 + K])) for g in range(c * c // 32)]
    assert min(spread) >= 50
    monkeypatch.delenv("TBS_SYRK_DIE_GROUPS")
    default = tb.tbs_syrk_lower_enumerate(dt, N, M, 2)
    assert np.array_equal(default, items if N * M * (4 if dt == tb.TBS_F32 else 8) > 192 << 20 else plain)


def test_empty_matrix():
    assert len(tb.tbs_syrk_lower_enumerate(tb.TBS_F64, 0, 5)) == 0


@pytest.mark.parametrize("N,M", [(768, 64), (4096, 4096), (4096, 32), (16384, 512), (12345, 100), (32768, 64)])
def test_triangle_blocks_are_those_of_the_indexing_family(N, M, monkeypatch):
    monkeypatch.setenv("TBS_SYRK_AUGMENT", "0")             # the schedule of Algorithm 4 as the paper states it
    # the CPU replay of Algorithm 4 on a T x 1 problem with b = 1 lists the blocks of every level (with
    # the library's rule for the family of a level: cyclic, or XOR where a power of two covers more rows)
    T = N // B                                              # full tiles only: the replay has no ragged edge
    items = tb.tbs_syrk_lower_enumerate(tb.TBS_F64, T * B, M)
    io = ts.tbs_syrk(np.zeros((T, 1)), np.zeros((T, T)), K, 1, families="auto")
    want = {lv: sorted(tuple(off + r for r in R) for l2, off, R in io.blocks if l2 == lv)
            for lv in range(10)}
    all_want = set(sum(want.values(), []))
    lib_tri = [tuple(row[3:3 + K]) for row in items.tolist() if row[0] == KIND_TRI and row[1] == K and row[8] == 0]
    family = [R for R in lib_tri if _is_family_block(R)]
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, T * B, M)
    fam, c = ts.choose_family(T // K, K)
    assert (info["family"] > 0) == (fam == "xor") and (fam == "cyclic" or c == 1 << info["family"])
    # every family block of the library is one of the replay's; the library uses the levels 0 ..
    # levels-1 of the recursion completely (deeper zones may be cut into rectangles instead, which
    # is the library's choice for small matrices) 
    assert set(family) <= all_want
    for lv in range(info["levels"]):
        assert set(want[lv]) <= set(lib_tri), lv
    if info["levels"] > 0:
        assert info["c"] == c and info["l"] == T - K * c
        assert info["A_elems_top"] == c * c * K * B * M     # Q1 = c^2 k b M
    assert info["k"] == K and info["b"] == B
    if T >= 200:
        assert info["levels"] >= 3                          # large matrices: the full recursion


def _is_family_block(R):
    return not all(R[u + 1] == R[u] + 1 for u in range(len(R) - 1))


def test_query_numbers_against_the_formulas(monkeypatch):
    N, M = 4096, 4096
    # what the library runs by default at this size: eight-tile blocks (six panels each) and no blocks of
    # their own for the diagonal zones, which loads fewer elements of A in all than the paper's blocks
    # with the zones cut finely enough to keep every compute unit busy
    default = tb.tbs_syrk_lower_query(tb.TBS_F64, N, M)
    monkeypatch.setenv("TBS_SYRK_AUGMENT", "0")             # from here on: the schedule of Algorithm 4
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, N, M)
    assert default["A_elems_top"] == 16 * 16 * 6 * B * M and default["levels"] == 1
    # ... and is held against the bound for the larger fast memory it uses (eight tiles of C per block)
    assert default["S_C_elems"] == 8 * B * B and default["S_res_elems"] == 8 * B * B + 2 * 6 * B * 16
    assert math.isclose(default["tbs_bound_elems"], ts.syrk_lower_bound(N, M, 8 * B * B), rel_tol=1e-12)
    assert default["A_elems"] >= default["tbs_bound_elems"]
    assert default["A_elems"] < info["A_elems"]
    S = ts.tiled_tbs_S(K, B)
    assert info["S_C_elems"] == S == 24576
    assert info["S_res_elems"] == S + 2 * K * B * 16
    assert math.isclose(info["tbs_bound_elems"], ts.syrk_lower_bound(N, M, S), rel_tol=1e-12)
    assert math.isclose(info["tiled_lead_elems"], ts.tiled_tbs_A_leading(N, M, K, B), rel_tol=1e-12)
    assert math.isclose(info["square_elems"], ts.square_A_volume(N, M, math.sqrt(S)), rel_tol=1e-12)
    assert info["C_elems"] == N * (N + 1) / 2
    assert (info["c"], info["l"], info["family"]) == (16, 0, 4) and 1 <= info["levels"] <= 2
    # the triangle blocks alone stay under the tiled bound N^2 M / ((k-1) b); no schedule beats the
    # lower bound.  (At this size the library cuts the diagonal zones finely to keep all compute
    # units busy, which costs A traffic; the comparison with square blocks is made at a size where
    # the schedule is the paper's.)
    assert info["A_elems_top"] <= info["tiled_lead_elems"]
    assert info["A_elems"] >= info["tbs_bound_elems"]
    large = tb.tbs_syrk_lower_query(tb.TBS_F64, 16384, 512)
    large_sq = tb.tbs_syrk_lower_query(tb.TBS_F64, 16384, 512, square=True)
    assert large["A_elems"] < 0.85 * large_sq["A_elems"]
    # large N: the plan's total approaches the tiled leading term (lower order terms are O(NM log N))
    big = tb.tbs_syrk_lower_query(tb.TBS_F64, 32768, 64)
    assert big["A_elems"] < 1.08 * big["tiled_lead_elems"]
    assert big["A_elems"] / big["tbs_bound_elems"] < 1.25   # sqrt(4/3) = 1.155 plus lower order terms
