"""Checks, through tbs_syrk_lower_enumerate / _query, that the plan in force for a size is the one a
TBS_PLAN_TUNING string pins ("levels,rows,cols,base[,zone_rows,zone_cols]")."""
import numpy as np

KIND_TRI, KIND_RECT, KIND_DIAG, KIND_EMPTY, KIND_RECTDIAG = 0, 1, 2, 3, 4
B, K = 64, 4


def assert_plan_is_pinned(tb, dtype_code, N, M, tuning, square=0):
    f = [int(x) for x in tuning.split(",")]
    lv, mr, nc, base = f[:4]
    mrd, ncd = (f[4], f[5]) if len(f) >= 6 and f[4] > 0 and f[5] > 0 else (mr, nc)
    items = tb.tbs_syrk_lower_enumerate(dtype_code, N, M, square)
    info = tb.tbs_syrk_lower_query(dtype_code, N, M, square)
    T = (N + B - 1) // B
    assert info["levels"] <= lv
    if lv == 0:
        assert info["n_tri_blocks"] == 0 or base            # no family blocks at all
    elif T // K >= K - 1:
        assert info["levels"] >= 1                          # the top level does use triangle blocks
    rect = items[items[:, 0] == KIND_RECT]
    rdiag = items[items[:, 0] == KIND_RECTDIAG]
    if len(rect):
        assert rect[:, 1].max() <= mr and rect[:, 2].max() <= nc
        # a region of at least mr x nc tiles exists whenever there are that many rectangles
        if len(rect) >= 4:
            assert rect[:, 1].max() == min(mr, rect[:, 1].max()) and rect[:, 2].max() in (nc, rect[:, 2].max())
    if base:
        assert len(rdiag) == 0 and (items[:, 0] == KIND_DIAG).sum() == T      # diagonal tiles listed singly
    else:
        assert (items[:, 0] == KIND_DIAG).sum() == 0
        if len(rdiag):
            assert rdiag[:, 1].max() <= mrd and rdiag[:, 2].max() <= ncd
            big_enough = T >= 2 * K * max(mrd, ncd)
            if big_enough:
                assert rdiag[:, 1].max() == mrd and rdiag[:, 2].max() == ncd
            if mrd == 2 and big_enough:
                # two-row rectangles of a triangular region: some straddle the diagonal (a column-side
                # tile row equals the first row-side tile row)
                straddle = [(row[6] in row[3:6]) for row in rdiag.tolist() if row[1] == 2]
                assert any(straddle)
    return items, info


def plans_differ(tb, dtype_code, N, M, monkeypatch, tuning):
    """True if the pinned plan is not what the library would choose by itself (so that the pin is observable)."""
    monkeypatch.delenv("TBS_PLAN_TUNING", raising=False)
    default = tb.tbs_syrk_lower_enumerate(dtype_code, N, M, 0)
    monkeypatch.setenv("TBS_PLAN_TUNING", tuning)
    pinned = tb.tbs_syrk_lower_enumerate(dtype_code, N, M, 0)
    return default.shape != pinned.shape or not np.array_equal(default, pinned)
