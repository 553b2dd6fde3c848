"""GPU parity of tbs_syr2k_lower and tbs_gram_lower against the CPU oracle, through the C ABI.

Tolerance: the SYRK bar carried over, max over i >= j of |C_gpu - C_ref|_ij / D_ij <= 1e-13 (fp64),
2e-5 (fp32), with D = |alpha| (|A||B|^T + |B||A|^T) + |beta C0| for SYR2K and |alpha| |A|^T|A| + |beta C0|
for the Gram form; the reference carries its sums in extended precision.  Integer-valued inputs must
agree bit for bit."""
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


def _check(Cg, C0, Cref, D, dtype):
    n = Cg.shape[0]
    il, iu = np.tril_indices(n), np.triu_indices(n, 1)
    assert np.array_equal(Cg[iu], C0[iu], equal_nan=True), "upper triangle was modified"
    err = np.abs(Cg[il].astype(np.float64) - Cref[il])
    den = np.maximum(D[il], np.finfo(np.float64).tiny)
    worst = float((err / den).max()) if err.size else 0.0
    assert worst <= TOL[dtype], f"componentwise error {worst:.3e}"


SHAPES = [(1, 1), (5, 3), (64, 16), (65, 17), (130, 40), (300, 100), (768, 48), (1000, 37), (1100, 130),
          (2100, 24), (4100, 70)]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", SHAPES)
def test_syr2k_parity_random(tb, N, M, dtype):
    A = inputs.normal_matrix(N, M, seed=N + M, dtype=dtype)
    B = inputs.uniform_matrix(N, M, seed=N + M + 1, dtype=dtype)
    C0 = inputs.symmetric_uniform(N, seed=N, dtype=dtype)
    C0[np.triu_indices(N, 1)] = np.nan
    dC = _dev(C0)
    tb.tbs_syr2k_lower(_dev(A), _dev(B), dC, -0.5, 1.5)
    torch.cuda.synchronize()
    A64, B64, C64 = A.astype(np.float64), B.astype(np.float64), C0.astype(np.float64)
    Cref = C64.copy()
    oracle.syr2k_lower(A64, B64, Cref, -0.5, 1.5, extended=True)
    D = 1.5 * np.abs(C64)
    oracle.syr2k_lower(np.abs(A64), np.abs(B64), D, 0.5, 1.0, extended=True)
    _check(dC.cpu().numpy(), C0, Cref, D, dtype)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", [(64, 8), (257, 96), (832, 40), (1300, 72), (4096, 16)])
def test_syr2k_integer_inputs_bit_exact(tb, N, M, dtype):
    A = inputs.small_int_matrix(N, M, seed=3 * N + M, dtype=dtype)
    B = inputs.small_int_matrix(N, M, seed=5 * N + M, dtype=dtype, lo=-3, hi=3)
    C0 = inputs.symmetric_uniform(N, seed=N + 7, dtype=dtype, int_range=(-9, 9))
    dC = _dev(C0)
    tb.tbs_syr2k_lower(_dev(A), _dev(B), dC, -2.0, 3.0)
    torch.cuda.synchronize()
    Cref = C0.astype(np.float64).copy()
    oracle.syr2k_lower(A.astype(np.float64), B.astype(np.float64), Cref, -2.0, 3.0)
    out = dC.cpu().numpy()
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(out[il].astype(np.float64), Cref[il])
    assert np.array_equal(out[iu], C0[iu])


def test_syr2k_beta_zero_leading_dimensions_and_empty(tb):
    N, M = 330, 45
    A = inputs.small_int_matrix(N, M, seed=11)
    B = inputs.small_int_matrix(N, M, seed=13)
    Cref = np.zeros((N, N))
    oracle.syr2k_lower(A, B, Cref, 1.0, 0.0)
    bigA = torch.zeros((N, M + 3), dtype=torch.float64, device="cuda")
    bigB = torch.zeros((N, M + 1), dtype=torch.float64, device="cuda")
    bigC = torch.full((N, N + 5), float("nan"), dtype=torch.float64, device="cuda")
    bigA[:, 1:M + 1] = _dev(A)
    bigB[:, 1:M + 1] = _dev(B)
    tb.tbs_syr2k_lower(bigA[:, 1:M + 1], bigB[:, 1:M + 1], bigC[:, 1:N + 1], 1.0, 0.0)   # beta = 0: NaNs not read
    torch.cuda.synchronize()
    out = bigC.cpu().numpy()
    il, iu = np.tril_indices(N), np.triu_indices(N, 1)
    assert np.array_equal(out[:, 1:N + 1][il], Cref[il])
    assert np.isnan(out[:, 1:N + 1][iu]).all() and np.isnan(out[:, 0]).all() and np.isnan(out[:, N + 1:]).all()
    # empty contraction scales the lower triangle; N = 0 is a no-op
    C1 = inputs.symmetric_uniform(N, seed=2)
    dC = _dev(C1)
    e = torch.empty((N, 0), dtype=torch.float64, device="cuda")
    tb.tbs_syr2k_lower(e, e, dC, 1.0, 0.5)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    assert np.array_equal(out[il], (0.5 * C1)[il]) and np.array_equal(out[iu], C1[iu])
    z = torch.empty((0, 4), dtype=torch.float64, device="cuda")
    tb.tbs_syr2k_lower(z, z, torch.empty((0, 0), dtype=torch.float64, device="cuda"))


# (rows of A = contraction length, columns of A = order of C): several tiles and ragged edges in both,
# orders that are no multiple of 2 / 4 (every block then takes the checked loop), contractions shorter
# than one chunk and not a multiple of it
GRAM_SHAPES = [(1, 1), (3, 5), (16, 64), (17, 65), (40, 130), (100, 300), (48, 768), (37, 1000), (130, 1100),
               (333, 514), (1000, 260), (4100, 384), (70, 2052)]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", GRAM_SHAPES)
def test_gram_parity_random(tb, N, M, dtype):
    A = inputs.normal_matrix(N, M, seed=N + 2 * M, dtype=dtype)
    C0 = inputs.symmetric_uniform(M, seed=M, dtype=dtype)
    C0[np.triu_indices(M, 1)] = np.nan
    dC = _dev(C0)
    tb.tbs_gram_lower(_dev(A), dC, -1.0, 1.0)
    torch.cuda.synchronize()
    A64, C64 = A.astype(np.float64), C0.astype(np.float64)
    Cref = C64.copy()
    oracle.gram_lower(A64, Cref, -1.0, 1.0, extended=True)
    D = np.abs(C64)
    oracle.gram_lower(np.abs(A64), D, 1.0, 1.0, extended=True)
    _check(dC.cpu().numpy(), C0, Cref, D, dtype)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M,pad,shift", [(8, 64, 0, 0), (96, 257, 0, 0), (40, 832, 2, 0), (72, 1300, 1, 1),
                                           (1031, 2052, 3, 1), (4096, 512, 0, 0), (50, 4100, 4, 2)])
def test_gram_integer_inputs_bit_exact(tb, N, M, pad, shift, dtype):
    # with leading dimensions that are no multiple of the row length and pointers off by some elements
    A = inputs.small_int_matrix(N, M, seed=3 * N + M, dtype=dtype)
    C0 = inputs.symmetric_uniform(M, seed=M + 7, dtype=dtype, int_range=(-9, 9))
    tdt = torch.float64 if dtype == np.float64 else torch.float32
    buf = torch.zeros(N * (M + pad) + 8, dtype=tdt, device="cuda")
    Av = buf[shift:shift + N * (M + pad)].view(N, M + pad)[:, :M]
    Av.copy_(_dev(A))
    Cref = C0.astype(np.float64).copy()
    oracle.gram_lower(A.astype(np.float64), Cref, -2.0, 3.0)
    il, iu = np.tril_indices(M), np.triu_indices(M, 1)
    for workspace in (None, False):
        dC = _dev(C0)
        tb.tbs_gram_lower(Av, dC, -2.0, 3.0, workspace=workspace)
        torch.cuda.synchronize()
        out = dC.cpu().numpy()
        assert np.array_equal(out[il].astype(np.float64), Cref[il])
        assert np.array_equal(out[iu], C0[iu])


def test_gram_with_cut_blocks_and_empty_cases(tb):
    # few column panels and a long contraction: the plan cuts blocks along the contraction dimension
    N, M = 4096, 512
    assert tb.tbs_gram_lower_workspace(tb.TBS_F64, N, M) == tb.tbs_syrk_lower_workspace(tb.TBS_F64, M, N) > 0
    A = inputs.normal_matrix(N, M, seed=77, scale=1.0 / 64)
    C0 = inputs.symmetric_uniform(M, seed=78)
    dC = _dev(C0)
    tb.tbs_gram_lower(_dev(A), dC, 1.0, -1.0)
    torch.cuda.synchronize()
    Cref = C0.copy()
    oracle.gram_lower(A, Cref, 1.0, -1.0, extended=True)
    D = np.abs(C0)
    oracle.gram_lower(np.abs(A), D, 1.0, 1.0, extended=True)
    _check(dC.cpu().numpy(), C0, Cref, D, np.float64)
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(tb.TbsError) as err:
        tb.tbs_gram_lower(_dev(A), dC, 1.0, -1.0, workspace=small)
    assert err.value.status == tb.TBS_EWORKSPACE
    # empty contraction scales; M = 0 is a no-op
    C1 = inputs.symmetric_uniform(100, seed=2)
    dC = _dev(C1)
    tb.tbs_gram_lower(torch.empty((0, 100), dtype=torch.float64, device="cuda"), dC, 1.0, 0.5)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    il, iu = np.tril_indices(100), np.triu_indices(100, 1)
    assert np.array_equal(out[il], (0.5 * C1)[il]) and np.array_equal(out[iu], C1[iu])
    tb.tbs_gram_lower(torch.empty((7, 0), dtype=torch.float64, device="cuda"),
                      torch.empty((0, 0), dtype=torch.float64, device="cuda"))


def test_larger_shapes_sampled(tb):
    # sizes with many blocks per compute unit (persistent launches, the full recursion of the plan):
    # sampled entries against the oracle's extended sums
    rng = np.random.default_rng(9)
    N, M = 6144, 512                                        # SYR2K, order 6144
    A = inputs.normal_matrix(N, M, seed=1, scale=1.0 / np.sqrt(M))
    B = inputs.normal_matrix(N, M, seed=2, scale=1.0 / np.sqrt(M))
    dC = torch.zeros((N, N), dtype=torch.float64, device="cuda")
    tb.tbs_syr2k_lower(_dev(A), _dev(B), dC, 1.0, 0.0)
    ii = rng.integers(0, N, size=20000)
    jj = (rng.random(20000) * (ii + 1)).astype(np.int64)
    ii[:100] = jj[:100]
    got = dC[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy()
    ref = np.einsum("ij,ij->i", A[ii].astype(np.longdouble), B[jj].astype(np.longdouble)) + \
        np.einsum("ij,ij->i", B[ii].astype(np.longdouble), A[jj].astype(np.longdouble))
    den = np.einsum("ij,ij->i", np.abs(A[ii]), np.abs(B[jj])) + np.einsum("ij,ij->i", np.abs(B[ii]), np.abs(A[jj]))
    assert float((np.abs(got - ref.astype(np.float64)) / den).max()) <= 1e-13
    assert not bool(dC[0, 1:].any()) and not bool(dC[N - 2, N - 1:].any())
    K, M = 2048, 8192                                       # Gram of a 2048 x 8192 matrix, order 8192
    A = inputs.normal_matrix(K, M, seed=3, scale=1.0 / np.sqrt(K))
    dC = torch.zeros((M, M), dtype=torch.float64, device="cuda")
    tb.tbs_gram_lower(_dev(A), dC, 1.0, 0.0)
    ii = rng.integers(0, M, size=20000)
    jj = (rng.random(20000) * (ii + 1)).astype(np.int64)
    ii[:100] = jj[:100]
    got = dC[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy()
    At = np.ascontiguousarray(A.T)
    ref = oracle.syrk_lower_sample(At, None, ii, jj, 1.0, 0.0)
    den = oracle.syrk_lower_sample(np.abs(At), None, ii, jj, 1.0, 0.0)
    assert float((np.abs(got - ref) / den).max()) <= 1e-13
    assert not bool(dC[0, 1:].any()) and not bool(dC[M - 2, M - 1:].any())


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("N,M", [(96, 768), (301, 1000), (130, 2052), (64, 4033)])
def test_gram_with_augmented_blocks_bit_exact(tb, N, M, dtype, monkeypatch):
    # the Gram form on a plan with eight-tile blocks (column panels through the same loops); an order that
    # is no multiple of the rows per 16-byte piece falls back to the plan without them
    monkeypatch.setenv("TBS_PLAN_TUNING", "10,2,3,0,1,3,1,1,0,1,1")
    code = tb.TBS_F64 if dtype == np.float64 else tb.TBS_F32
    assert int((tb.tbs_syrk_lower_enumerate(code, M, N, 0)[:, 0] == 5).sum()) >= 9
    A = inputs.small_int_matrix(N, M, seed=N + M, dtype=dtype)
    C0 = inputs.symmetric_uniform(M, seed=M, dtype=dtype, int_range=(-9, 9))
    dC = _dev(C0)
    tb.tbs_gram_lower(_dev(A), dC, -1.0, 1.0)
    torch.cuda.synchronize()
    Cref = C0.astype(np.float64).copy()
    oracle.gram_lower(A.astype(np.float64), Cref, -1.0, 1.0)
    il, iu = np.tril_indices(M), np.triu_indices(M, 1)
    out = dC.cpu().numpy()
    assert np.array_equal(out[il].astype(np.float64), Cref[il])
    assert np.array_equal(out[iu], C0[iu])
