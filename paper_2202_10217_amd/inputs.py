"""Seeded synthetic inputs, shared by the tests, the benchmark and the smoke run.

This module holds no arithmetic of the method: it only fills matrices.  The
numbers come from a counter-based generator written out here (value = hash of
(seed, stream, element index)), so the same element has the same bits whatever
the chunking, the numpy version or the machine, and a symmetric matrix is
symmetric by construction (entry (i,j) is hashed from (max(i,j), min(i,j))).

The paper uses no data set; the shapes and distributions are those of the
benchmark configurations (dense A with iid entries, a symmetric C, a strictly
diagonally dominant symmetric matrix for Cholesky).
"""
import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(x):
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
    return x ^ (x >> np.uint64(31))


def _bits(seed: int, stream: int, idx):
    with np.errstate(over="ignore"):
        key = _mix64(np.uint64(seed) * _GOLD + np.uint64(stream))
        return _mix64(key + np.asarray(idx, dtype=np.uint64) * _GOLD)


def _u01(seed, stream, idx):
    """Uniform on (0,1): 53 random bits, never exactly 0."""
    return ((_bits(seed, stream, idx) >> np.uint64(11)).astype(np.float64) + 0.5) * (2.0 ** -53)


def _rows_chunks(n_rows, n_cols, target=1 << 22):
    step = max(1, target // max(n_cols, 1))
    for r0 in range(0, n_rows, step):
        yield r0, min(n_rows, r0 + step)


def _fill(n_rows, n_cols, dtype, fn):
    out = np.empty((n_rows, n_cols), dtype=dtype)
    cols = np.arange(n_cols, dtype=np.uint64)
    for r0, r1 in _rows_chunks(n_rows, n_cols):
        rows = np.arange(r0, r1, dtype=np.uint64)
        with np.errstate(over="ignore"):
            idx = rows[:, None] * np.uint64(n_cols) + cols[None, :]
        out[r0:r1] = fn(idx)
    return out


def uniform_matrix(n_rows, n_cols, seed, dtype=np.float64, stream=0):
    """iid Uniform(-1, 1)."""
    return _fill(n_rows, n_cols, dtype, lambda idx: 2.0 * _u01(seed, stream, idx) - 1.0)


def normal_matrix(n_rows, n_cols, seed, scale=1.0, dtype=np.float64, stream=0):
    """iid N(0, scale^2) by the Box-Muller transform of two uniform streams."""
    def fn(idx):
        u1 = _u01(seed, 2 * stream + 100, idx)
        u2 = _u01(seed, 2 * stream + 101, idx)
        return scale * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return _fill(n_rows, n_cols, dtype, fn)


def small_int_matrix(n_rows, n_cols, seed, lo=-2, hi=2, dtype=np.float64, stream=0):
    """iid integers in [lo, hi]: sums of products stay exactly representable."""
    span = np.uint64(hi - lo + 1)
    return _fill(n_rows, n_cols, dtype,
                 lambda idx: (_bits(seed, stream + 200, idx) % span).astype(np.int64) + lo)


def symmetric_uniform(n, seed, diag=None, dtype=np.float64, stream=0, int_range=None):
    """Symmetric n x n, off-diagonal entries Uniform(-1,1) (or small integers), diagonal = `diag`
    (a number) or random when None.  Entry (i,j) depends only on (max(i,j), min(i,j))."""
    out = np.empty((n, n), dtype=dtype)
    cols = np.arange(n, dtype=np.uint64)
    for r0, r1 in _rows_chunks(n, n):
        rows = np.arange(r0, r1, dtype=np.uint64)
        hi_ = np.maximum(rows[:, None], cols[None, :])
        lo_ = np.minimum(rows[:, None], cols[None, :])
        with np.errstate(over="ignore"):
            idx = hi_ * np.uint64(n) + lo_
        if int_range is None:
            blk = 2.0 * _u01(seed, stream + 300, idx) - 1.0
        else:
            span = np.uint64(int_range[1] - int_range[0] + 1)
            blk = (_bits(seed, stream + 300, idx) % span).astype(np.int64) + int_range[0]
        out[r0:r1] = blk
    if diag is not None:
        np.fill_diagonal(out, diag)
    return out


def spd_diag_dominant(n, seed, dtype=np.float64):
    """Symmetric, off-diagonal Uniform(-1,1), diagonal = n: strictly diagonally dominant, hence SPD."""
    return symmetric_uniform(n, seed, diag=float(n), dtype=dtype)


# ---- the benchmark configurations ------------------------------------------------------------

CONFIGS = {
    # name: (op, N, M, dtype, alpha, beta, seed)
    "syrk_n256_m256_f64": ("syrk", 256, 256, np.float64, 1.0, 0.0, 0),
    "syrk_n4096_m4096_f64": ("syrk", 4096, 4096, np.float64, -1.0, 1.0, 1),
    "syrk_n16384_m512_f64": ("syrk", 16384, 512, np.float64, -1.0, 1.0, 2),
    "potrf_n16384_f64": ("potrf", 16384, 0, np.float64, 0.0, 0.0, 3),
    "syrk_n32768_m8192_f32": ("syrk", 32768, 8192, np.float32, 1.0, 0.0, 4),
}


def make_config(name, n_override=None, m_override=None):
    """Returns (op, A, C, alpha, beta) for SYRK configs, (op, None, S, 0, 0) for the Cholesky one.

    The distributions follow the configuration list: uniform A for the small case, N(0,1)
    (scaled by 1/sqrt(M) for the tall and the large case) otherwise; C symmetric uniform, with
    diagonal M for the trailing-update shape; C = 0 for the beta = 0 cases.
    """
    op, N, M, dtype, alpha, beta, seed = CONFIGS[name]
    N = n_override or N
    M = m_override or M
    if op == "potrf":
        return op, None, spd_diag_dominant(N, seed, dtype), 0.0, 0.0
    if name == "syrk_n256_m256_f64":
        A = uniform_matrix(N, M, seed, dtype)
    elif name == "syrk_n4096_m4096_f64":
        A = normal_matrix(N, M, seed, 1.0, dtype)
    else:
        A = normal_matrix(N, M, seed, 1.0 / np.sqrt(M), dtype)
    if beta == 0.0:
        C = np.zeros((N, N), dtype=dtype)
    elif name == "syrk_n16384_m512_f64":
        C = symmetric_uniform(N, seed, diag=float(M), dtype=dtype)
    else:
        C = symmetric_uniform(N, seed, dtype=dtype)
    return op, A, C, alpha, beta
