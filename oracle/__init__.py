"""TEST INFRASTRUCTURE -- CPU oracle for SYRK (lower) and Cholesky.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of
`bench.py` may import this package.  It shares nothing with the GPU library.

The arithmetic lives in `syrk_cholesky_oracle.c` (the paper's Algorithm 1 and
Algorithm 2 written out as plain loops); this file only marshals numpy arrays.
`tbs_schedule.py` holds a literal, element-granular replay of the paper's
schedules (Algorithms 3 and 4) with an I/O counter, and the closed forms of the
paper's bounds.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.OUT
    if not os.path.exists(path):
        path = _build.build()
    lib = ctypes.CDLL(path)
    i64, f64, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
    lib.oracle_num_threads.restype = ctypes.c_int
    lib.oracle_num_threads.argtypes = []
    for name in ("oracle_syrk_lower_f64", "oracle_syrk_lower_f64_ext"):
        fn = getattr(lib, name)
        fn.restype = None
        fn.argtypes = [i64, i64, f64, p, i64, f64, p, i64]
    lib.oracle_syrk_lower_f64_ext_sample.restype = None
    lib.oracle_syrk_lower_f64_ext_sample.argtypes = [i64, f64, p, i64, f64, p, i64, i64, p, p, p]
    lib.oracle_syr2k_lower_f64.restype = None
    lib.oracle_syr2k_lower_f64.argtypes = [i64, i64, f64, p, i64, p, i64, f64, p, i64, ctypes.c_int]
    lib.oracle_gram_lower_f64.restype = None
    lib.oracle_gram_lower_f64.argtypes = [i64, i64, f64, p, i64, f64, p, i64, ctypes.c_int]
    lib.oracle_potrf_lower_f64.restype = i64
    lib.oracle_potrf_lower_f64.argtypes = [i64, p, i64]
    lib.oracle_llt_residual_sq.restype = f64
    lib.oracle_llt_residual_sq.argtypes = [i64, p, i64, p, i64, p]
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _as_f64_matrix(x, name):
    x = np.asarray(x)
    if x.dtype != np.float64 or x.ndim != 2:
        raise ValueError(f"{name}: need a float64 2-D array")
    if x.size and ((x.shape[1] > 1 and x.strides[1] != 8) or x.strides[0] % 8
                   or (x.shape[0] > 1 and x.strides[0] < 8 * x.shape[1])):
        raise ValueError(f"{name}: need a row-major array (unit stride along rows)")
    return x


def _ld(x):
    """Leading dimension in elements (any value >= the row length when there is one row or none)."""
    if x.shape[0] > 1 and x.size:
        return x.strides[0] // 8
    return max(x.shape[1], 1)


def syrk_lower(A, C, alpha=1.0, beta=1.0, extended=True):
    """C[i,j] <- beta*C[i,j] + alpha*sum_k A[i,k]A[j,k] for j<=i, in place (Algorithm 1).

    `extended=True` carries the k-sum in long double (the parity yardstick),
    `False` is the plain double loop (the one that is timed).  A may hold
    float32-representable values: the oracle computes in fp64 regardless.
    Entries above the diagonal are neither read nor written.
    """
    A = _as_f64_matrix(A, "A")
    C = _as_f64_matrix(C, "C")
    N, M = A.shape
    if C.shape != (N, N):
        raise ValueError("C must be N x N")
    if not C.flags.writeable:
        raise ValueError("C must be writeable")
    lib = _load()
    fn = lib.oracle_syrk_lower_f64_ext if extended else lib.oracle_syrk_lower_f64
    fn(N, M, float(alpha), A.ctypes.data, _ld(A), float(beta), C.ctypes.data, _ld(C))
    return C


def syrk_lower_sample(A, C, ii, jj, alpha=1.0, beta=1.0):
    """Updated values of the entries (ii[t], jj[t]), ii>=jj, without touching C."""
    A = _as_f64_matrix(A, "A")
    N, M = A.shape
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    if ii.shape != jj.shape or ii.ndim != 1:
        raise ValueError("ii, jj: equal-length 1-D index arrays")
    if ii.size and (ii.min() < 0 or ii.max() >= N or jj.min() < 0 or (jj > ii).any()):
        raise ValueError("need 0 <= jj <= ii < N")
    out = np.empty(ii.size, dtype=np.float64)
    lda = _ld(A)
    if beta != 0.0:
        C = _as_f64_matrix(C, "C")
        cptr, ldc = C.ctypes.data, _ld(C)
    else:
        cptr, ldc = None, max(N, 1)
    _load().oracle_syrk_lower_f64_ext_sample(M, float(alpha), A.ctypes.data, lda, float(beta),
                                             cptr, ldc, ii.size, ii.ctypes.data, jj.ctypes.data,
                                             out.ctypes.data)
    return out


def syr2k_lower(A, B, C, alpha=1.0, beta=1.0, extended=True):
    """C[i,j] <- beta*C[i,j] + alpha*sum_k (A[i,k]B[j,k] + B[i,k]A[j,k]) for j<=i, in place (the
    textbook SYR2K; one of the "kernels that use an input several times" of the paper's conclusion)."""
    A = _as_f64_matrix(A, "A")
    B = _as_f64_matrix(B, "B")
    C = _as_f64_matrix(C, "C")
    N, M = A.shape
    if B.shape != (N, M) or C.shape != (N, N):
        raise ValueError("B must be N x M and C N x N")
    if not C.flags.writeable:
        raise ValueError("C must be writeable")
    _load().oracle_syr2k_lower_f64(N, M, float(alpha), A.ctypes.data, _ld(A), B.ctypes.data, _ld(B),
                                   float(beta), C.ctypes.data, _ld(C), 1 if extended else 0)
    return C


def gram_lower(A, C, alpha=1.0, beta=1.0, extended=True):
    """C[i,j] <- beta*C[i,j] + alpha*sum_k A[k,i]A[k,j] for j<=i (C is M x M for an N x M matrix A),
    in place: the Gram matrix A^T A, i.e. Algorithm 1 applied to the transpose."""
    A = _as_f64_matrix(A, "A")
    C = _as_f64_matrix(C, "C")
    N, M = A.shape
    if C.shape != (M, M):
        raise ValueError("C must be M x M")
    if not C.flags.writeable:
        raise ValueError("C must be writeable")
    _load().oracle_gram_lower_f64(N, M, float(alpha), A.ctypes.data, _ld(A), float(beta), C.ctypes.data,
                                  _ld(C), 1 if extended else 0)
    return C


def potrf_lower(S):
    """Right-looking Cholesky of the lower triangle of S, in place (Algorithm 2).

    Returns info: 0, or the 1-based index of the first pivot that is not > 0.
    """
    S = _as_f64_matrix(S, "S")
    N = S.shape[0]
    if S.shape != (N, N):
        raise ValueError("S must be square")
    if not S.flags.writeable:
        raise ValueError("S must be writeable")
    return int(_load().oracle_potrf_lower_f64(N, S.ctypes.data, _ld(S)))


def llt_residual(L, S):
    """||tril(L) tril(L)^T - S||_F / ||S||_F using the lower triangle of both, S symmetric."""
    L = _as_f64_matrix(L, "L")
    S = _as_f64_matrix(S, "S")
    N = L.shape[0]
    nrm = ctypes.c_double(0.0)
    acc = _load().oracle_llt_residual_sq(N, L.ctypes.data, _ld(L), S.ctypes.data, _ld(S),
                                         ctypes.byref(nrm))
    return float(np.sqrt(acc) / np.sqrt(nrm.value)) if nrm.value > 0 else float(np.sqrt(acc))
