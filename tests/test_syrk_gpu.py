"""GPU parity of the Triangle Block SYRK against the CPU oracle, through the C ABI.

Tolerance (from the benchmark spec): max over i >= j of |C_gpu - C_ref|_ij / (|A| |A|^T + |beta C0|)_ij
  <= 1e-13 for fp64 and <= 2e-5 for fp32.  The reference is the oracle with the k-sum in extended
precision, so its own rounding does not use up the tolerance.  Integer-valued inputs must agree bit for
bit (every partial sum is exact in any order), which pins indexing and coverage independently of rounding.
"""
import numpy as np
import pytest

import oracle
from paper_2202_10217_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = {np.float64: 1e-13, np.float32: 2e-5}


@pytest.fixture(scope="module")
def tb():
    from paper_2202_10217_amd import binding
    binding.load()
    return binding


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _run(tb, A, C0, alpha, beta, square=False):
    dA, dC = _dev(A), _dev(C0)
    fn = tb.tbs_syrk_lower_square if square else tb.tbs_syrk_lower
    fn(dA, dC, alpha, beta)
    torch.cuda.synchronize()
    return dC.cpu().numpy()


def _reference(A, C0, alpha, beta):
    A64 = A.astype(np.float64)
    C = C0.astype(np.float64).copy()
    if beta == 0.0:
        C[:] = 0.0
    oracle.syrk_lower(A64, C, alpha, beta, extended=True)
    D = np.zeros_like(C)
    oracle.syrk_lower(np.abs(A64), D, abs(alpha), 0.0, extended=True)
    if beta != 0.0:
        D += np.abs(beta * C0.astype(np.float64))
    return C, D


def _check(Cg, C0, Cref, D, dtype):
    N = Cg.shape[0]
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(Cg[iu], C0[iu], equal_nan=True), "upper triangle was modified"
    err = np.abs(Cg[il].astype(np.float64) - Cref[il])
    den = np.maximum(D[il], np.finfo(np.float64).tiny)
    worst = float((err / den).max()) if err.size else 0.0
    assert worst <= TOL[dtype], f"componentwise error {worst:.3e}"
    return worst


def test_config1_n256_m256(tb):
    _, A, C0, alpha, beta = inputs.make_config("syrk_n256_m256_f64")
    C0 = C0.copy()
    C0[np.triu_indices(256, 1)] = np.nan                     # sentinel above the diagonal
    Cg = _run(tb, A, C0, alpha, beta)
    Cref, D = _reference(A, C0, alpha, beta)
    _check(Cg, C0, Cref, D, np.float64)


# sizes spanning several tiles, every code path (triangle blocks at two levels, leftover rows, base
# zones, diagonal tiles) and ragged edges in N and in M
SHAPES = [(1, 1), (5, 3), (64, 16), (65, 17), (130, 40), (200, 33), (256, 64), (300, 100), (700, 50),
          (768, 48), (1000, 37), (1100, 130), (4100, 24)]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", SHAPES)
def test_parity_random(tb, N, M, dtype):
    A = inputs.normal_matrix(N, M, seed=N + M, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=N, dtype=dtype)
    C0[np.triu_indices(N, 1)] = np.nan
    Cg = _run(tb, A, C0, -1.0, 1.0)
    Cref, D = _reference(A, C0, -1.0, 1.0)
    _check(Cg, C0, Cref, D, dtype)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", [(64, 8), (257, 96), (832, 40), (1300, 72), (4096, 16)])
@pytest.mark.parametrize("square", [False, True])
def test_integer_inputs_bit_exact(tb, N, M, dtype, square):
    A = inputs.small_int_matrix(N, M, seed=3 * N + M, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=N + 7, dtype=dtype, int_range=(-9, 9))
    Cg = _run(tb, A, C0, -2.0, 3.0, square=square)
    Cref = C0.astype(np.float64).copy()
    oracle.syrk_lower(A.astype(np.float64), Cref, -2.0, 3.0)
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(Cg[il].astype(np.float64), Cref[il])
    assert np.array_equal(Cg[iu], C0[iu])


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_beta_zero_ignores_old_contents_and_m_zero_scales(tb, dtype):
    N, M = 300, 50
    A = inputs.uniform_matrix(N, M, seed=1, dtype=dtype)
    C0 = np.full((N, N), np.nan, dtype=dtype)
    Cg = _run(tb, A, C0, 1.0, 0.0)
    Cref, D = _reference(A, np.zeros((N, N), dtype=dtype), 1.0, 0.0)
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.isnan(Cg[iu]).all() and np.isfinite(Cg[il]).all()
    assert (np.abs(Cg[il] - Cref[il]) <= TOL[dtype] * D[il]).all()
    # M = 0: C <- beta*C on the lower triangle only
    C1 = inputs.symmetric_uniform(N, seed=2, dtype=dtype)
    dA = torch.empty((N, 0), dtype=torch.float64 if dtype == np.float64 else torch.float32, device="cuda")
    dC = _dev(C1)
    tb.tbs_syrk_lower(dA, dC, 1.0, 0.5)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    assert np.array_equal(out[il], (0.5 * C1)[il]) and np.array_equal(out[iu], C1[iu])


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_leading_dimensions_and_unaligned_views(tb, dtype):
    # lda / ldc larger than the row length, and a view that starts at an odd element: the 16-byte
    # vector path cannot be used, the element path must give the same result
    N, M = 330, 45
    A = inputs.small_int_matrix(N, M, seed=11, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=12, dtype=dtype, int_range=(-3, 3))
    Cref = C0.astype(np.float64).copy()
    oracle.syrk_lower(A.astype(np.float64), Cref, 1.0, 1.0)
    bigA = torch.zeros((N, M + 3), dtype=_dev(A).dtype, device="cuda")
    bigC = torch.full((N, N + 5), 7.0, dtype=bigA.dtype, device="cuda")
    bigA[:, 1:M + 1] = _dev(A)
    bigC[:, 1:N + 1] = _dev(C0)
    tb.tbs_syrk_lower(bigA[:, 1:M + 1], bigC[:, 1:N + 1], 1.0, 1.0)
    torch.cuda.synchronize()
    out = bigC.cpu().numpy()
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(out[:, 1:N + 1][il].astype(np.float64), Cref[il])
    assert np.array_equal(out[:, 1:N + 1][iu], C0[iu])
    assert (out[:, 0] == 7.0).all() and (out[:, N + 1:] == 7.0).all()


def test_matrices_of_4_gib_or_more_use_64_bit_offsets(tb):
    # the assembly loop addresses the 64 rows of a panel with 32-bit byte offsets from a 64-bit pointer per
    # panel; a matrix whose rows are spread over 4.6 GB (huge leading dimension, few columns) must give
    # the same bits on integer data
    N, M, lda = 4096, 64, 140000
    A = inputs.small_int_matrix(N, M, seed=21)
    C0 = inputs.symmetric_uniform(N, seed=22, int_range=(-3, 3))
    Cref = C0.copy()
    oracle.syrk_lower(A, Cref, -1.0, 1.0)
    big = torch.empty((N, lda), dtype=torch.float64, device="cuda")
    big[:, :M] = _dev(A)
    dC = _dev(C0)
    tb.tbs_syrk_lower(big[:, :M], dC, -1.0, 1.0)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    del big
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(out[il], Cref[il])
    assert np.array_equal(out[iu], C0[iu])


@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (-1.0, 1.0), (0.5, -2.0), (0.0, 3.0), (2.0, 1.0)])
def test_alpha_beta_combinations(tb, alpha, beta):
    N, M = 777, 208                                         # ragged last tile, 13 whole chunks
    A = inputs.uniform_matrix(N, M, seed=31)
    C0 = inputs.symmetric_uniform(N, seed=32)
    Cg = _run(tb, A, C0, alpha, beta)
    Cref, D = _reference(A, C0, alpha, beta)
    _check(Cg, C0, Cref, D, np.float64)


def test_square_baseline_parity(tb):
    N, M = 900, 120
    A = inputs.normal_matrix(N, M, seed=21)
    C0 = inputs.symmetric_uniform(N, seed=22)
    Cg = _run(tb, A, C0, -1.0, 1.0, square=True)
    Cref, D = _reference(A, C0, -1.0, 1.0)
    _check(Cg, C0, Cref, D, np.float64)


def test_empty_problem(tb):
    dA = torch.empty((0, 5), dtype=torch.float64, device="cuda")
    dC = torch.empty((0, 0), dtype=torch.float64, device="cuda")
    tb.tbs_syrk_lower(dA, dC)
    torch.cuda.synchronize()


def _check_full_in_row_bands(Cg, C0, Cref, D, dtype, band=1024):
    """The stated bar on every entry of the lower triangle, and bit-for-bit equality above the diagonal,
    band by band (the index arrays of a whole 16384 x 16384 triangle would not be worth their memory)."""
    N = Cg.shape[0]
    worst = 0.0
    cols = np.arange(N)
    for r0 in range(0, N, band):
        r1 = min(N, r0 + band)
        low = cols[None, :r1] <= np.arange(r0, r1)[:, None]
        g, c0 = Cg[r0:r1, :r1], C0[r0:r1, :r1]
        assert np.array_equal(g[~low], c0[~low]) and np.array_equal(Cg[r0:r1, r1:], C0[r0:r1, r1:]), \
            "upper triangle was modified"
        err = np.abs(g.astype(np.float64) - Cref[r0:r1, :r1])[low]
        den = np.maximum(D[r0:r1, :r1][low], np.finfo(np.float64).tiny)
        worst = max(worst, float((err / den).max()))
    assert worst <= TOL[dtype], f"componentwise error {worst:.3e}"
    return worst


def _full_check(tb, name):
    """Every entry of the result at the configuration's full size against the oracle with the
    extended-precision sum (Algorithm 1 as plain loops), in the launch configuration bench.py times:
    the library's workspace is passed, so the plan is the one with blocks cut along the contraction
    dimension where the library uses them."""
    _, A, C0, alpha, beta = inputs.make_config(name)
    N, M = A.shape
    code = tb.TBS_F64
    need = tb.tbs_syrk_lower_workspace(code, N, M)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else False
    dA, dC = _dev(A), _dev(C0)
    tb.tbs_syrk_lower(dA, dC, alpha, beta, workspace=ws)
    torch.cuda.synchronize()
    Cg = dC.cpu().numpy()
    del dC
    Cref = C0.copy()
    oracle.syrk_lower(A, Cref, alpha, beta, extended=True)
    D = np.abs(beta) * np.abs(C0)
    oracle.syrk_lower(np.abs(A), D, abs(alpha), 1.0, extended=True)
    return _check_full_in_row_bands(Cg, C0, Cref, D, np.float64)


def test_config2_n4096_m4096_every_entry(tb):
    _full_check(tb, "syrk_n4096_m4096_f64")


def test_config3_n16384_m512_every_entry(tb):
    _full_check(tb, "syrk_n16384_m512_f64")


def _tiles_by_block_kind(items):
    """Tiles (row tile, column tile) of the work list, by the kind of block that computes them:
    'tri' (triangle blocks of an indexing family or of a base zone), 'rect' (rectangles strictly below
    the diagonal), 'rect_diag' (off-diagonal tiles of rectangles that carry diagonal tiles), 'diag'."""
    out = {"tri": [], "rect": [], "rect_diag": [], "diag": []}
    for row in items.tolist():
        kind, nrow, ncol, rows = row[0], row[1], row[2], row[3:8]
        if row[8] != 0:                                     # a cut block: its first part stands for it
            continue
        if kind == 0:
            R = rows[:nrow]
            out["tri"] += [(R[u], R[v]) for u in range(nrow) for v in range(u)]
        elif kind in (1, 4):
            for r in rows[3:3 + nrow]:
                for q in rows[:ncol]:
                    if q < r:
                        out["rect" if kind == 1 else "rect_diag"].append((r, q))
                    elif q == r and kind == 4:
                        out["diag"].append((r, q))
        elif kind == 2:
            out["diag"].append((rows[0], rows[0]))
    return {k: np.array(v, dtype=np.int64).reshape(-1, 2) for k, v in out.items()}


def test_config5_n32768_m8192_f32_million_samples_by_block_kind(tb):
    # the large fp32 shape: a million entries, drawn in equal shares from the tiles of every kind of
    # block of the plan in force (through tbs_syrk_lower_enumerate) and from the last rows and columns,
    # each compared with the oracle's extended-precision dot product
    name, dtype = "syrk_n32768_m8192_f32", np.float32
    _, A, C0, alpha, beta = inputs.make_config(name)
    N, M = A.shape
    dA, dC = _dev(A), _dev(C0)
    tb.tbs_syrk_lower(dA, dC, alpha, beta)
    torch.cuda.synchronize()
    kinds = _tiles_by_block_kind(tb.tbs_syrk_lower_enumerate(tb.TBS_F32, N, M))
    T = N // 64
    assert sum(len(v) for v in kinds.values()) == T * (T + 1) // 2
    rng = np.random.default_rng(2024)
    ii, jj, used = [], [], []
    per_kind = -(-1_000_000 // sum(1 for v in kinds.values() if len(v)))
    for kind, tiles in kinds.items():
        if len(tiles) == 0:
            continue
        used.append(kind)
        pick = tiles[rng.integers(0, len(tiles), size=per_kind)]
        i = pick[:, 0] * 64 + rng.integers(0, 64, size=per_kind)
        j = pick[:, 1] * 64 + rng.integers(0, 64, size=per_kind)
        if kind == "diag":
            i, j = np.maximum(i, j), np.minimum(i, j)
        ii.append(i)
        jj.append(j)
    assert "tri" in used and "diag" in used
    # the edges: the diagonal itself, the last row, the first column
    d = rng.integers(0, N, size=1000)
    ii += [d, np.full(1000, N - 1), rng.integers(0, N, size=1000)]
    jj += [d, rng.integers(0, N, size=1000), np.zeros(1000, dtype=np.int64)]
    ii, jj = np.concatenate(ii), np.concatenate(jj)
    assert ii.size >= 1_000_000
    assert (jj <= ii).all()
    got = dC[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy().astype(np.float64)
    A64 = A.astype(np.float64)
    ref = oracle.syrk_lower_sample(A64, None, ii, jj, alpha, 0.0)
    den = oracle.syrk_lower_sample(np.abs(A64), None, ii, jj, abs(alpha), 0.0)
    worst = float((np.abs(got - ref) / np.maximum(den, 1e-300)).max())
    assert worst <= TOL[dtype], f"{name}: componentwise error {worst:.3e}"
    # a property that holds at any size: nothing above the diagonal is written (C0 is zero there)
    rows = np.unique(np.concatenate([np.arange(0, N, N // 64), [N - 2]]))
    up = dC[torch.from_numpy(rows).cuda()].cpu().numpy()
    for r, line in zip(rows, up):
        assert not line[r + 1:].any()


def test_config2_integer_exact_full_size(tb):
    # at the benchmark size: integer A, exact result known in closed form per entry via int64 matmul
    N, M = 4096, 4096
    A = inputs.small_int_matrix(N, M, seed=99)
    dA = _dev(A)
    dC = torch.zeros((N, N), dtype=torch.float64, device="cuda")
    tb.tbs_syrk_lower(dA, dC, 1.0, 0.0)
    torch.cuda.synchronize()
    Ai = A.astype(np.int64)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.integers(0, N, size=48), [0, 63, 64, 3839, 3840, N - 1]]))
    exact = Ai[rows] @ Ai.T
    got = dC[torch.from_numpy(rows).cuda()].cpu().numpy()
    for r, g, e in zip(rows, got, exact):
        assert np.array_equal(g[:r + 1], e[:r + 1].astype(np.float64))
        assert not g[r + 1:].any()


def test_calls_on_several_streams_do_not_disturb_each_other(tb):
    # persistent launches take their blocks through counters in device memory; launches that may run
    # at the same time must not share a counter pair.  Three streams, several calls each, on integer
    # data (any lost or doubled block shows as a wrong integer); a Cholesky on a fourth stream, which
    # brings its own second stream and events, runs beside them.
    N, M = 2304, 96
    streams = [torch.cuda.Stream() for _ in range(4)]
    As = [inputs.small_int_matrix(N, M, seed=40 + i) for i in range(3)]
    C0 = inputs.symmetric_uniform(N, seed=44, int_range=(-3, 3))
    refs = []
    for A in As:
        R = C0.copy()
        for _ in range(3):
            oracle.syrk_lower(A, R, 1.0, 1.0)
        refs.append(R)
    n = 3000
    rng = np.random.default_rng(5)
    G = np.tril(rng.integers(-1, 2, size=(n, n))).astype(np.float64)
    np.fill_diagonal(G, 1.0)
    dS = _dev(G @ G.T)
    dAs = [_dev(A) for A in As]
    dCs = [_dev(C0) for _ in As]
    torch.cuda.synchronize()
    for rep in range(3):
        for i in range(3):
            with torch.cuda.stream(streams[i]):
                tb.tbs_syrk_lower(dAs[i], dCs[i], 1.0, 1.0)
        if rep == 0:
            with torch.cuda.stream(streams[3]):
                tb.tbs_potrf_lower(dS, want_info=False)
    torch.cuda.synchronize()
    il = np.tril_indices(N)
    for i in range(3):
        assert np.array_equal(dCs[i].cpu().numpy()[il], refs[i][il]), i
    assert np.array_equal(np.tril(dS.cpu().numpy()), G)


@pytest.mark.parametrize("N,M", [(512, 4096), (2048, 2080), (1100, 3000)])
def test_blocks_cut_along_the_contraction_dimension(tb, N, M):
    # few tiles per compute unit and a long contraction: with a workspace the library computes blocks in
    # parts (summed in a fixed order by the last part to finish), without one it does not.  Same bits on
    # integer data either way, repeatably; the plan with a workspace really is cut; the tolerance holds
    # on random data with ragged sizes too.
    import os
    if os.environ.get("TBS_SYRK_SLICES", "")[:1] == "0":
        pytest.skip("blocks are not cut when TBS_SYRK_SLICES=0")
    info = tb.tbs_syrk_lower_query(tb.TBS_F64, N, M)
    assert info["n_sliced_blocks"] > 0 and info["workspace_bytes"] == tb.tbs_syrk_lower_workspace(tb.TBS_F64, N, M)
    assert tb.tbs_syrk_lower_query(tb.TBS_F64, N, M, 2)["n_sliced_blocks"] == 0
    A = inputs.small_int_matrix(N, M, seed=51)
    C0 = inputs.symmetric_uniform(N, seed=52, int_range=(-3, 3))
    Cref = C0.copy()
    oracle.syrk_lower(A, Cref, -1.0, 1.0)
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    dA = _dev(A)
    ws = torch.empty(info["workspace_bytes"], dtype=torch.uint8, device="cuda")
    for workspace in (ws, ws, False):                       # twice with the same workspace: counters are reset
        dC = _dev(C0)
        tb.tbs_syrk_lower(dA, dC, -1.0, 1.0, workspace=workspace)
        torch.cuda.synchronize()
        out = dC.cpu().numpy()
        assert np.array_equal(out[il], Cref[il]) and np.array_equal(out[iu], C0[iu])
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")     # a workspace, but too small: an error
    dC = _dev(C0)
    with pytest.raises(tb.TbsError) as err:
        tb.tbs_syrk_lower(dA, dC, -1.0, 1.0, workspace=small)
    assert err.value.status == tb.TBS_EWORKSPACE
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C0)             # nothing was launched
    Ar = inputs.normal_matrix(N, M, seed=53)
    Cg = _run(tb, Ar, C0, 0.5, -1.5)
    Cr, D = _reference(Ar, C0, 0.5, -1.5)
    _check(Cg, C0, Cr, D, np.float64)


# block shapes pinned through the environment ("levels,rows,cols,base,zone_rows,zone_cols"): among them
# two-row rectangles in triangular regions, whose blocks straddle the diagonal in three different ways
PINNED = ["0,2,3,0", "1,2,3,0,2,3", "2,2,2,0,2,2", "1,1,3,0,2,1", "1,2,3,0,1,2", "10,2,3,1"]


@pytest.mark.parametrize("idx", range(len(PINNED)))
def test_pinned_block_shapes_bit_exact_and_in_tolerance(tb, idx, monkeypatch):
    from _plan_util import assert_plan_is_pinned
    monkeypatch.setenv("TBS_PLAN_TUNING", PINNED[idx])
    for N, M in ((1216 + 64 * idx, 48), (1500 + 64 * idx + 7, 80)):     # whole tiles; a ragged last tile
        # the plan in force for this size is the pinned one (the tuning string is part of the library's
        # plan-cache key), whatever sizes earlier tests of this process have used
        assert_plan_is_pinned(tb, tb.TBS_F64, N, M, PINNED[idx])
        A = inputs.small_int_matrix(N, M, seed=30 + idx, dtype=np.float64)
        C0 = inputs.symmetric_uniform(N, seed=40 + idx, dtype=np.float64, int_range=(-9, 9))
        Cg = _run(tb, A, C0, -1.0, 1.0)
        Cref = C0.copy()
        oracle.syrk_lower(A, Cref, -1.0, 1.0)
        il, iu = np.tril_indices(N), np.triu_indices(N, 1)
        assert np.array_equal(Cg[il], Cref[il])
        assert np.array_equal(Cg[iu], C0[iu])
    N, M = 1088 + 64 * idx, 64
    assert_plan_is_pinned(tb, tb.TBS_F64, N, M, PINNED[idx])
    A = inputs.normal_matrix(N, M, 50 + idx, 1.0, np.float64)
    C0 = inputs.symmetric_uniform(N, 60 + idx, dtype=np.float64)
    Cg = _run(tb, A, C0, -1.0, 1.0)
    Cref, D = _reference(A, C0, -1.0, 1.0)
    _check(Cg, C0, Cref, D, np.float64)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M,pad,shift", [(1027, 100, 1, 1), (2051, 1031, 3, 0), (640, 4100, 1, 3), (4133, 200, 5, 1)])
def test_edges_of_the_main_loop_bit_exact(tb, N, M, pad, shift, dtype):
    # everything the main loop has to cope with at once: a last tile row with few rows, a contraction
    # length that is no multiple of the chunk, rows that are only element-aligned (odd leading dimension,
    # pointer off by `shift` elements); integer data, so the result must agree bit for bit
    A = inputs.small_int_matrix(N, M, seed=N + 3 * M, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=N + 1, dtype=dtype, int_range=(-7, 7))
    tdt = torch.float64 if dtype == np.float64 else torch.float32
    buf = torch.zeros(N * (M + pad) + 8, dtype=tdt, device="cuda")
    Av = buf[shift:shift + N * (M + pad)].view(N, M + pad)[:, :M]
    Av.copy_(_dev(A))
    Cref = C0.astype(np.float64).copy()
    oracle.syrk_lower(A.astype(np.float64), Cref, 2.0, -1.0)
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    for square in (False, True):
        dC = _dev(C0)
        (tb.tbs_syrk_lower_square if square else tb.tbs_syrk_lower)(Av, dC, 2.0, -1.0)
        torch.cuda.synchronize()
        out = dC.cpu().numpy()
        assert np.array_equal(out[il].astype(np.float64), Cref[il])
        assert np.array_equal(out[iu], C0[iu])


# ---- augmented triangle blocks (eight tiles: a triangle block plus two tiles of the diagonal zones) ----
AUG_TUNING = "10,2,3,0,1,3,1,1,0,1,1"


def _aug_blocks(tb, code, N, M):
    items = tb.tbs_syrk_lower_enumerate(code, N, M, 0)
    return int((items[:, 0] == 5).sum())


@pytest.mark.parametrize("family", ["", "cyclic"])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", [(768, 96), (1000, 301), (2051, 130), (4033, 200), (4096, 64)])
def test_augmented_blocks_bit_exact(tb, N, M, dtype, family, monkeypatch):
    # integer data (any order of summation gives the same bits): pins which tile every accumulator of the
    # eight-tile blocks is written to, for both families, with whole and ragged last tile rows, a
    # contraction length that is no multiple of the chunk, and blocks whose extra tile is a diagonal tile
    monkeypatch.setenv("TBS_PLAN_TUNING", AUG_TUNING)
    if family:
        monkeypatch.setenv("TBS_PLAN_FAMILY", family)
    code = tb.TBS_F64 if dtype == np.float64 else tb.TBS_F32
    assert _aug_blocks(tb, code, N, M) >= 9
    A = inputs.small_int_matrix(N, M, seed=N + M, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=N, dtype=dtype, int_range=(-9, 9))
    C0[np.triu_indices(N, 1)] = np.nan
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    for alpha, beta in ((-1.0, 1.0), (2.0, 0.0)):
        Cg = _run(tb, A, C0, alpha, beta)
        Cref = np.nan_to_num(C0.astype(np.float64))
        oracle.syrk_lower(A.astype(np.float64), Cref, alpha, beta)
        assert np.array_equal(Cg[il].astype(np.float64), Cref[il])
        assert np.isnan(Cg[iu]).all()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_augmented_blocks_in_tolerance_and_default_choice(tb, dtype, monkeypatch):
    # random data against the extended-precision oracle, on the plan the library chooses by itself where
    # that plan has augmented blocks (fp64, N = 4096, long contraction) and pinned otherwise
    N, M = 4096, 2048
    code = tb.TBS_F64 if dtype == np.float64 else tb.TBS_F32
    if dtype == np.float64:
        assert _aug_blocks(tb, code, N, M) == 256            # the default for this shape
    else:
        monkeypatch.setenv("TBS_SYRK_AUGMENT", "1")
        assert _aug_blocks(tb, code, N, M) == 256
    A = inputs.normal_matrix(N, M, seed=5, scale=1.0 / 32, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=6, dtype=dtype)
    dA, dC = _dev(A), _dev(C0)
    ws = torch.empty(max(tb.tbs_syrk_lower_workspace(code, N, M), 16), dtype=torch.uint8, device="cuda")
    tb.tbs_syrk_lower(dA, dC, -1.0, 1.0, workspace=ws)
    torch.cuda.synchronize()
    Cref, D = _reference(A, C0, -1.0, 1.0)
    _check(dC.cpu().numpy(), C0, Cref, D, dtype)
    monkeypatch.setenv("TBS_SYRK_AUGMENT", "0")
    assert _aug_blocks(tb, code, N, M) == 0


def test_augmented_plan_is_not_used_for_operands_the_fast_loop_cannot_take(tb, monkeypatch):
    # the eight-tile blocks have no general path: with a contraction shorter than a chunk the library
    # must fall back to the plan without them (same result, bit for bit on integer data)
    monkeypatch.setenv("TBS_PLAN_TUNING", AUG_TUNING)
    N, M = 1000, 9
    A = inputs.small_int_matrix(N, M, seed=1)
    C0 = inputs.symmetric_uniform(N, seed=2, int_range=(-9, 9))
    Cg = _run(tb, A, C0, -1.0, 1.0)
    Cref = C0.copy()
    oracle.syrk_lower(A, Cref, -1.0, 1.0)
    il = np.tril_indices(N)
    assert np.array_equal(Cg[il], Cref[il])
    # odd leading dimension and an offset pointer are fine for the fast loop: the augmented plan runs
    M = 100
    assert _aug_blocks(tb, tb.TBS_F64, N, M) >= 9
    A = inputs.small_int_matrix(N, M, seed=3)
    buf = torch.zeros(N * (M + 3) + 8, dtype=torch.float64, device="cuda")
    Av = buf[1:1 + N * (M + 3)].view(N, M + 3)[:, :M]
    Av.copy_(_dev(A))
    dC = _dev(C0)
    tb.tbs_syrk_lower(Av, dC, 1.0, -1.0)
    torch.cuda.synchronize()
    Cref = C0.copy()
    oracle.syrk_lower(A, Cref, 1.0, -1.0)
    assert np.array_equal(dC.cpu().numpy()[il], Cref[il])


def test_cut_blocks_on_several_streams_at_once(tb):
    # plans with blocks cut along the contraction dimension on three streams at the same time, each call
    # with a workspace of its own: the parts travel through device-scope stores and loads and a counter per
    # block, the three launches use different sets of counters; integer data, so a part that is read before
    # it has arrived, or added twice, shows as a wrong integer
    shapes = [(2048, 2080), (4096, 1024), (1100, 3000)]
    streams = [torch.cuda.Stream() for _ in shapes]
    dAs, dCs, wss, refs = [], [], [], []
    for i, (N, M) in enumerate(shapes):
        assert tb.tbs_syrk_lower_query(tb.TBS_F64, N, M)["n_sliced_blocks"] > 0
        A = inputs.small_int_matrix(N, M, seed=60 + i)
        C0 = inputs.symmetric_uniform(N, seed=70 + i, int_range=(-3, 3))
        R = C0.copy()
        for _ in range(4):
            oracle.syrk_lower(A, R, -1.0, 1.0)
        refs.append(R)
        dAs.append(_dev(A))
        dCs.append(_dev(C0))
        wss.append(torch.empty(tb.tbs_syrk_lower_workspace(tb.TBS_F64, N, M), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    for rep in range(4):
        for i in range(len(shapes)):
            with torch.cuda.stream(streams[i]):
                tb.tbs_syrk_lower(dAs[i], dCs[i], -1.0, 1.0, workspace=wss[i])
    torch.cuda.synchronize()
    for i, (N, M) in enumerate(shapes):
        il = np.tril_indices(N)
        assert np.array_equal(dCs[i].cpu().numpy()[il], refs[i][il]), shapes[i]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_augmented_blocks_with_die_groups_bit_exact(tb, dtype, monkeypatch):
    # the eight-tile blocks handed out in groups of 32 per die (both options forced on; persistent launch:
    # 256 top-level blocks and the left-over tiles on fewer workgroups than blocks)
    monkeypatch.setenv("TBS_PLAN_TUNING", AUG_TUNING)
    monkeypatch.setenv("TBS_SYRK_DIE_GROUPS", "1")
    monkeypatch.setenv("TBS_SYRK_RESERVE", "64")
    N, M = 4096, 96
    code = tb.TBS_F64 if dtype == np.float64 else tb.TBS_F32
    assert _aug_blocks(tb, code, N, M) == 256
    A = inputs.small_int_matrix(N, M, seed=11, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=12, dtype=dtype, int_range=(-9, 9))
    Cg = _run(tb, A, C0, -1.0, 1.0)
    Cref = C0.astype(np.float64).copy()
    oracle.syrk_lower(A.astype(np.float64), Cref, -1.0, 1.0)
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(Cg[il].astype(np.float64), Cref[il])
    assert np.array_equal(Cg[iu], C0[iu])
