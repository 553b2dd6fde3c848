"""GPU parity of Large Block Cholesky against the CPU oracle (Algorithm 2), through the C ABI.

Bar (from the benchmark spec): ||L L^T - A||_F / ||A||_F <= 1e-13 in fp64.  On well conditioned
inputs the factor is unique and stable, so L is also compared with the oracle's L element by element;
an integer factor must be recovered exactly."""
import numpy as np
import pytest

import oracle
from paper_2202_10217_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    from paper_2202_10217_amd import binding
    binding.load()
    return binding


def _factor(tb, S):
    d = torch.from_numpy(np.ascontiguousarray(S)).cuda()
    info = tb.tbs_potrf_lower(d)
    torch.cuda.synchronize()
    return info, d.cpu().numpy()


@pytest.mark.parametrize("N", [1, 2, 5, 63, 64, 65, 130, 200, 257, 512, 700, 1000, 1536, 2500])
def test_parity_with_oracle(tb, N):
    S0 = inputs.spd_diag_dominant(N, seed=N)
    S = S0.copy()
    S[np.triu_indices(N, 1)] = np.nan                       # the upper triangle must not be referenced
    info, out = _factor(tb, S)
    assert info == 0
    iu, il = np.triu_indices(N, 1), np.tril_indices(N)
    assert np.isnan(out[iu]).all(), "upper triangle was modified"
    Lo = S0.copy()
    assert oracle.potrf_lower(Lo) == 0
    L = np.tril(out)
    assert (np.diag(L) > 0).all()
    assert oracle.llt_residual(L, S0) <= 1e-13
    scale = np.abs(Lo[il]).max()
    assert np.abs(L[il] - Lo[il]).max() <= 1e-12 * scale


@pytest.mark.parametrize("N", [7, 33, 64, 65, 200, 1100, 2100])
def test_integer_factor_is_recovered_exactly(tb, N):
    # every kernel of the driver performs the operations of Algorithm 2 on the same values (tile
    # factorisation, substitution against diagonal tiles, MFMA updates of integer data), so an integer
    # factor comes back bit for bit, across tiles and panels too
    rng = np.random.default_rng(N)
    G = np.tril(rng.integers(-2, 3, size=(N, N))).astype(np.float64)
    np.fill_diagonal(G, rng.integers(1, 4, size=N))
    S = G @ G.T
    info, out = _factor(tb, S)
    assert info == 0
    assert np.array_equal(np.tril(out), G)
    assert np.array_equal(out[np.triu_indices(N, 1)], S[np.triu_indices(N, 1)])


@pytest.mark.parametrize("N,bad", [(50, 0), (50, 17), (300, 150), (300, 299), (1200, 700)])
def test_not_positive_definite(tb, N, bad):
    G = np.tril(np.ones((N, N)))
    S = G @ G.T
    S[bad, bad] -= 1.0                                       # pivot `bad` becomes exactly 0
    info, _ = _factor(tb, S)
    assert info == bad + 1


def test_leading_dimension_and_workspace(tb):
    N = 333
    S0 = inputs.spd_diag_dominant(N, seed=8)
    big = torch.full((N, N + 9), 5.0, dtype=torch.float64, device="cuda")
    big[:, 2:N + 2] = torch.from_numpy(S0).cuda()
    ws = torch.empty(tb.tbs_potrf_lower_workspace(tb.TBS_F64, N), dtype=torch.uint8, device="cuda")
    assert tb.tbs_potrf_lower(big[:, 2:N + 2], workspace=ws) == 0
    out = big.cpu().numpy()
    Lo = S0.copy()
    oracle.potrf_lower(Lo)
    il = np.tril_indices(N)
    assert np.abs(out[:, 2:N + 2][il] - Lo[il]).max() <= 1e-12 * np.abs(Lo[il]).max()
    assert (out[:, :2] == 5.0).all() and (out[:, N + 2:] == 5.0).all()
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(tb.TbsError):
        tb.tbs_potrf_lower(big[:, 2:N + 2], workspace=small)


@pytest.mark.parametrize("N", [65, 900, 2600, 4133])
def test_fp32(tb, N):
    # single precision is outside the stated bar (which is fp64); held to the same form of it with the
    # fp32 unit roundoff: residual within 2e-6, and the factor of a well conditioned matrix within 2e-5 of
    # the oracle's (fp64) factor relative to its largest entry
    S0 = inputs.spd_diag_dominant(N, seed=4, dtype=np.float32)
    S = S0.copy()
    S[np.triu_indices(N, 1)] = np.nan
    info, out = _factor(tb, S)
    assert info == 0
    assert np.isnan(out[np.triu_indices(N, 1)]).all()
    L = np.tril(out).astype(np.float64)
    assert oracle.llt_residual(L, S0.astype(np.float64)) <= 2e-6
    Lo = S0.astype(np.float64)
    assert oracle.potrf_lower(Lo) == 0
    il = np.tril_indices(N)
    assert np.abs(L[il] - Lo[il]).max() <= 2e-5 * np.abs(Lo[il]).max()


@pytest.mark.parametrize("N", [33, 200, 1100, 2700])
def test_fp32_integer_factor_is_recovered_exactly(tb, N):
    # small integers are exact in single precision too: the factor comes back bit for bit
    rng = np.random.default_rng(N)
    G = np.tril(rng.integers(-1, 2, size=(N, N))).astype(np.float32)
    np.fill_diagonal(G, rng.integers(1, 3, size=N))
    S = (G.astype(np.float64) @ G.astype(np.float64).T).astype(np.float32)
    info, out = _factor(tb, S)
    assert info == 0
    assert np.array_equal(np.tril(out), G)
    S[N // 2, N // 2] = 0.0                                  # and a failed pivot is reported
    G2 = np.tril(np.ones((N, N), dtype=np.float32))
    S2 = (G2.astype(np.float64) @ G2.astype(np.float64).T).astype(np.float32)
    S2[N // 2, N // 2] -= 1.0
    assert _factor(tb, S2)[0] == N // 2 + 1


def _probe_check(L, S0):
    """Necessary conditions of the bar that are cheap at any size, in float64 on the host:
    ||L (L^T x) - A x|| / ||A x|| <= 1e-13 for a few random x, and, for a sample of rows i, every entry
    (L L^T)_ij within 1e-13 (|L| |L|^T)_ij of A_ij (the componentwise form of the bar)."""
    N = S0.shape[0]
    x = inputs.normal_matrix(N, 4, seed=17)
    Ax = S0 @ x
    r = L @ (L.T @ x) - Ax
    rel = np.linalg.norm(r, axis=0) / np.linalg.norm(Ax, axis=0)
    assert rel.max() <= 1e-13, rel
    rows = np.unique(np.clip(np.array([0, 1, 63, 64, 511, 512, 513, 1023, 1024, 1025, 5000, 6143, 6144, 6500,
                                       8191, 8192, 12345, N - 2, N - 1]), 0, N - 1))
    rec = L[rows] @ L.T                                      # rows of L L^T
    bound = np.abs(L[rows]) @ np.abs(L).T
    for rr, line, bd in zip(rows, rec, bound):
        assert (np.abs(line[:rr + 1] - S0[rr, :rr + 1]) <= 1e-13 * bd[:rr + 1]).all(), rr


@pytest.mark.parametrize("N", [7000, 9001])
def test_ragged_sizes_beyond_the_one_launch_solve(tb, N):
    # N is no multiple of the tile, and the first panels have more rows below them than the one-launch
    # triangular solve takes, so both forms of the solve, the look-ahead and (9001) a double-width panel
    # all meet ragged edges here
    S0 = inputs.spd_diag_dominant(N, seed=5)
    info, out = _factor(tb, S0)
    assert info == 0
    assert np.array_equal(out[np.triu_indices(N, 1)], S0[np.triu_indices(N, 1)])   # upper part untouched
    _probe_check(np.tril(out), S0)


def test_exact_integer_factor_with_look_ahead(tb):
    # the same bit-exact recovery as above at a size that uses the second stream and the tall solve
    N = 6600
    rng = np.random.default_rng(11)
    G = np.tril(rng.integers(-1, 2, size=(N, N))).astype(np.float64)
    np.fill_diagonal(G, rng.integers(1, 3, size=N))
    S = G @ G.T
    info, out = _factor(tb, S)
    assert info == 0
    assert np.array_equal(np.tril(out), G)


def test_config4_n16384_residual_in_full(tb):
    # the stated bar at the full size: ||L L^T - A||_F / ||A||_F <= 1e-13 with every entry of L L^T
    # evaluated by the oracle (sums in extended precision; about N^3/6 multiply-adds on the host cores),
    # and the cheap probes besides
    N = 16384
    S0 = inputs.spd_diag_dominant(N, seed=3)
    d = torch.from_numpy(S0).cuda()
    info = tb.tbs_potrf_lower(d)
    torch.cuda.synchronize()
    assert info == 0
    out = d.cpu().numpy()
    del d
    for r in (0, 1, 5000, N - 2):                           # nothing above the diagonal was written
        assert np.array_equal(out[r, r + 1:], S0[r, r + 1:])
    L = np.tril(out)
    del out
    assert (np.diag(L) > 0).all()
    _probe_check(L, S0)
    res = oracle.llt_residual(L, S0)
    assert res <= 1e-13, res


# Panels twice as wide are used while the trailing matrix has at least TBS_POTRF_WIDE_ROWS rows (8192 by
# default; read at every call): with a small value, matrices the oracle factors in seconds take that path,
# alone (all panels 1024 wide) or followed by 512-wide panels (the switch between the two).
@pytest.mark.parametrize("N,wide_rows", [(3600, 512), (3500, 1800), (4133, 2100)])
def test_double_width_panels_against_the_oracle(tb, N, wide_rows, monkeypatch):
    monkeypatch.setenv("TBS_POTRF_WIDE_ROWS", str(wide_rows))
    S0 = inputs.spd_diag_dominant(N, seed=N)
    S = S0.copy()
    S[np.triu_indices(N, 1)] = np.nan                       # the upper triangle must not be referenced
    info, out = _factor(tb, S)
    assert info == 0
    iu, il = np.triu_indices(N, 1), np.tril_indices(N)
    assert np.isnan(out[iu]).all(), "upper triangle was modified"
    Lo = S0.copy()
    assert oracle.potrf_lower(Lo) == 0
    L = np.tril(out)
    assert oracle.llt_residual(L, S0) <= 1e-13
    assert np.abs(L[il] - Lo[il]).max() <= 1e-12 * np.abs(Lo[il]).max()


@pytest.mark.parametrize("N,wide_rows", [(3700, 512), (4000, 2000)])
def test_double_width_panels_recover_an_integer_factor_exactly(tb, N, wide_rows, monkeypatch):
    monkeypatch.setenv("TBS_POTRF_WIDE_ROWS", str(wide_rows))
    rng = np.random.default_rng(N)
    G = np.tril(rng.integers(-1, 2, size=(N, N))).astype(np.float64)
    np.fill_diagonal(G, rng.integers(1, 3, size=N))
    S = G @ G.T
    info, out = _factor(tb, S)
    assert info == 0
    assert np.array_equal(np.tril(out), G)
    assert np.array_equal(out[np.triu_indices(N, 1)], S[np.triu_indices(N, 1)])


# The left-looking panel (TBS_POTRF_PANEL=left, read at every call): every block column of a panel first
# receives the updates of the earlier block columns of that panel, then is factored and solved.
@pytest.mark.parametrize("N", [130, 700, 1536, 2500, 4133])
def test_left_looking_panel_against_the_oracle(tb, N, monkeypatch):
    monkeypatch.setenv("TBS_POTRF_PANEL", "left")
    S0 = inputs.spd_diag_dominant(N, seed=N)
    S = S0.copy()
    S[np.triu_indices(N, 1)] = np.nan
    info, out = _factor(tb, S)
    assert info == 0
    iu, il = np.triu_indices(N, 1), np.tril_indices(N)
    assert np.isnan(out[iu]).all(), "upper triangle was modified"
    Lo = S0.copy()
    assert oracle.potrf_lower(Lo) == 0
    L = np.tril(out)
    assert oracle.llt_residual(L, S0) <= 1e-13
    assert np.abs(L[il] - Lo[il]).max() <= 1e-12 * np.abs(Lo[il]).max()


@pytest.mark.parametrize("N,wide_rows", [(1100, 8192), (3700, 512), (6600, 8192)])
def test_left_looking_panel_recovers_an_integer_factor_exactly(tb, N, wide_rows, monkeypatch):
    monkeypatch.setenv("TBS_POTRF_PANEL", "left")
    monkeypatch.setenv("TBS_POTRF_WIDE_ROWS", str(wide_rows))
    rng = np.random.default_rng(N)
    G = np.tril(rng.integers(-1, 2, size=(N, N))).astype(np.float64)
    np.fill_diagonal(G, rng.integers(1, 3, size=N))
    S = G @ G.T
    info, out = _factor(tb, S)
    assert info == 0
    assert np.array_equal(np.tril(out), G)
    S[700, 700] -= 1.0 if N > 700 else 0.0                  # a failed pivot is still reported at its index
    if N > 700:
        G2 = np.tril(np.ones((N, N)))
        S2 = G2 @ G2.T
        S2[700, 700] -= 1.0
        assert _factor(tb, S2)[0] == 701


def test_calls_on_two_streams_without_waiting_in_between(tb):
    # two factorisations enqueued back to back on different streams of the caller (no synchronisation
    # between the calls, info not requested): the library's own streams and events are shared by all calls
    # on a device, so this pins their ordering; exact integer factors, so any mix-up shows
    sizes = (3300, 2700)
    rng = np.random.default_rng(23)
    Gs, ds, streams = [], [], [torch.cuda.Stream(), torch.cuda.Stream()]
    for N in sizes:
        G = np.tril(rng.integers(-1, 2, size=(N, N))).astype(np.float64)
        np.fill_diagonal(G, rng.integers(1, 3, size=N))
        Gs.append(G)
        ds.append(torch.from_numpy(G @ G.T).cuda())
    ws = [torch.empty(4096, dtype=torch.uint8, device="cuda") for _ in sizes]
    torch.cuda.synchronize()
    for rep in range(2):                                     # second round: factor the factors' products again
        for d, w, s in zip(ds, ws, streams):
            assert tb.tbs_potrf_lower(d, workspace=w, stream=s, want_info=False) == 0
        torch.cuda.synchronize()
        for d, G in zip(ds, Gs):
            assert np.array_equal(np.tril(d.cpu().numpy()), G)
        if rep == 0:
            for d, G in zip(ds, Gs):
                d.copy_(torch.from_numpy(G @ G.T).cuda())
            torch.cuda.synchronize()


def test_calls_from_two_host_threads(tb):
    # two host threads, each with its own stream and matrix, call at the same time (ctypes releases the
    # interpreter lock during the call): the library enqueues one call after the other; exact factors
    import threading
    sizes = (2900, 3500)
    rng = np.random.default_rng(29)
    Gs, ds = [], []
    for N in sizes:
        G = np.tril(rng.integers(-1, 2, size=(N, N))).astype(np.float64)
        np.fill_diagonal(G, rng.integers(1, 3, size=N))
        Gs.append(G)
        ds.append(torch.from_numpy(G @ G.T).cuda())
    ws = [torch.empty(4096, dtype=torch.uint8, device="cuda") for _ in sizes]
    streams = [torch.cuda.Stream() for _ in sizes]
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            for _ in range(3):
                info = tb.tbs_potrf_lower(ds[i], workspace=ws[i], stream=streams[i])   # synchronises its stream
                if info != 0 or not np.array_equal(np.tril(ds[i].cpu().numpy()), Gs[i]):
                    errors.append((i, info))
                with torch.cuda.stream(streams[i]):
                    ds[i].copy_(torch.from_numpy(Gs[i] @ Gs[i].T).cuda(), non_blocking=False)
                streams[i].synchronize()
        except Exception as e:                                  # noqa: BLE001 - reported below
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(sizes))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
