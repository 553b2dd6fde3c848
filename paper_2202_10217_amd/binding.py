"""ctypes binding of the C ABI in include/tbs_syrk.h: argument marshalling only.

Every function here has the name of the entry point it calls.  Matrices are torch tensors on the
GPU (row-major, unit stride along rows); the binding passes their data pointers, leading
dimensions and the current HIP stream.  There is no CPU fallback: if the library has not been
built, loading fails with an error.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libtbs_syrk.so")

TBS_F64, TBS_F32 = 0, 1
TBS_OK, TBS_EINVAL, TBS_EWORKSPACE, TBS_ENOTSPD, TBS_EHIP = 0, 1, 2, 3, 4

EXPORTS = ("tbs_status_string", "tbs_syrk_lower_workspace", "tbs_syrk_lower", "tbs_syrk_lower_square",
           "tbs_syrk_lower_noalloc", "tbs_syr2k_lower", "tbs_gram_lower", "tbs_gram_lower_workspace",
           "tbs_syrk_lower_query", "tbs_syrk_lower_enumerate", "tbs_potrf_lower_workspace",
           "tbs_potrf_lower")


class TbsError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {tbs_status_string(status)} (status {int(status)})")


class PlanInfo(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int32), ("b", ctypes.c_int32), ("c", ctypes.c_int32), ("l", ctypes.c_int32),
                ("levels", ctypes.c_int32), ("tile_rows", ctypes.c_int32),
                ("family", ctypes.c_int32), ("max_slices", ctypes.c_int32),
                ("n_items", ctypes.c_int64), ("n_tri_blocks", ctypes.c_int64),
                ("n_rect_blocks", ctypes.c_int64), ("n_diag_tiles", ctypes.c_int64),
                ("S_C_elems", ctypes.c_int64), ("S_res_elems", ctypes.c_int64),
                ("A_elems", ctypes.c_double), ("A_elems_top", ctypes.c_double), ("C_elems", ctypes.c_double),
                ("tbs_bound_elems", ctypes.c_double), ("tiled_lead_elems", ctypes.c_double),
                ("square_elems", ctypes.c_double),
                ("n_sliced_blocks", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64)]


_lib = None


def load():
    """Opens the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2202_10217_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, f64, p, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_size_t
    lib.tbs_status_string.restype = ctypes.c_char_p
    lib.tbs_status_string.argtypes = [ctypes.c_int]
    lib.tbs_syrk_lower_workspace.restype = ctypes.c_int
    lib.tbs_syrk_lower_workspace.argtypes = [ctypes.c_int, i64, i64, ctypes.POINTER(sz)]
    for name in ("tbs_syrk_lower", "tbs_syrk_lower_square"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [ctypes.c_int, i64, i64, f64, p, i64, f64, p, i64, p, sz, p]
    lib.tbs_syrk_lower_noalloc.restype = ctypes.c_int
    lib.tbs_syrk_lower_noalloc.argtypes = [ctypes.c_int, i64, i64, f64, p, i64, f64, p, i64, p]
    lib.tbs_syr2k_lower.restype = ctypes.c_int
    lib.tbs_syr2k_lower.argtypes = [ctypes.c_int, i64, i64, f64, p, i64, p, i64, f64, p, i64, p]
    lib.tbs_gram_lower.restype = ctypes.c_int
    lib.tbs_gram_lower.argtypes = [ctypes.c_int, i64, i64, f64, p, i64, f64, p, i64, p, sz, p]
    lib.tbs_gram_lower_workspace.restype = ctypes.c_int
    lib.tbs_gram_lower_workspace.argtypes = [ctypes.c_int, i64, i64, ctypes.POINTER(sz)]
    lib.tbs_syrk_lower_query.restype = ctypes.c_int
    lib.tbs_syrk_lower_query.argtypes = [ctypes.c_int, i64, i64, i32, ctypes.POINTER(PlanInfo)]
    lib.tbs_syrk_lower_enumerate.restype = ctypes.c_int
    lib.tbs_syrk_lower_enumerate.argtypes = [ctypes.c_int, i64, i64, i32, p, i64, ctypes.POINTER(i64)]
    lib.tbs_potrf_lower_workspace.restype = ctypes.c_int
    lib.tbs_potrf_lower_workspace.argtypes = [ctypes.c_int, i64, ctypes.POINTER(sz)]
    lib.tbs_potrf_lower.restype = ctypes.c_int
    lib.tbs_potrf_lower.argtypes = [ctypes.c_int, i64, p, i64, p, sz, ctypes.POINTER(i32), p]
    _lib = lib
    return lib


def tbs_status_string(status) -> str:
    return load().tbs_status_string(int(status)).decode()


def _dtype_code(t):
    import torch
    if t.dtype == torch.float64:
        return TBS_F64
    if t.dtype == torch.float32:
        return TBS_F32
    raise TypeError("float64 or float32 tensors only")


def _matrix_args(t, name):
    """(data pointer, leading dimension) of a row-major 2-D device tensor."""
    if t.dim() != 2:
        raise ValueError(f"{name}: 2-D tensor expected")
    if not t.is_cuda:
        raise ValueError(f"{name}: the tensor must live on the GPU")
    rows, cols = t.shape
    if cols > 1 and t.stride(1) != 1:
        raise ValueError(f"{name}: unit stride along rows expected")
    ld = t.stride(0) if rows > 1 else max(cols, 1)
    return t.data_ptr(), max(int(ld), 1)


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def tbs_syrk_lower_workspace(dtype_code, N, M) -> int:
    out = ctypes.c_size_t(0)
    st = load().tbs_syrk_lower_workspace(dtype_code, N, M, ctypes.byref(out))
    if st != TBS_OK:
        raise TbsError(st, "tbs_syrk_lower_workspace")
    return int(out.value)


def _syrk(entry, A, C, alpha, beta, workspace, stream):
    code = _dtype_code(A)
    if C.dtype != A.dtype:
        raise TypeError("A and C must have the same dtype")
    N, M = A.shape
    if tuple(C.shape) != (N, N):
        raise ValueError("C must be N x N")
    a_ptr, lda = _matrix_args(A, "A")
    c_ptr, ldc = _matrix_args(C, "C")
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
        if workspace is not None else (None, 0)
    st = getattr(load(), entry)(code, N, M, float(alpha), ctypes.c_void_p(a_ptr), lda, float(beta),
                                ctypes.c_void_p(c_ptr), ldc, ctypes.c_void_p(ws_ptr), ws_bytes,
                                _stream_ptr(stream))
    if st != TBS_OK:
        raise TbsError(st, entry)
    return C


def tbs_syrk_lower(A, C, alpha=1.0, beta=1.0, workspace=None, stream=None):
    """C[lower] <- beta*C + alpha*A A^T under the Triangle Block Scheme, in place, asynchronous.

    workspace: a uint8 device tensor of at least tbs_syrk_lower_workspace() bytes; None allocates one of
    that size for this call (on `stream`); False passes none (the library then uses its plan without
    blocks cut along the contraction dimension)."""
    if workspace is None:
        import torch
        need = tbs_syrk_lower_workspace(_dtype_code(A), A.shape[0], A.shape[1])
        if need > 0:
            with torch.cuda.stream(stream if stream is not None else torch.cuda.current_stream()):
                workspace = torch.empty(need, dtype=torch.uint8, device=A.device)
    elif workspace is False:
        workspace = None
    return _syrk("tbs_syrk_lower", A, C, alpha, beta, workspace, stream)


def tbs_syrk_lower_square(A, C, alpha=1.0, beta=1.0, workspace=None, stream=None):
    """Same update with rectangular blocks only (the square-block baseline)."""
    return _syrk("tbs_syrk_lower_square", A, C, alpha, beta, workspace, stream)


NOALLOC_WORKSPACE_BYTES = 128 << 20


def tbs_syrk_lower_noalloc(A, C, alpha=1.0, beta=1.0, stream=None):
    """tbs_syrk_lower with the library's own file-scope scratch memory: nothing is allocated by the call
    (nor by this wrapper).  Raises TbsError(TBS_EWORKSPACE) for sizes whose plan needs more than
    NOALLOC_WORKSPACE_BYTES; calls that overlap on one GPU race."""
    code = _dtype_code(A)
    if C.dtype != A.dtype:
        raise TypeError("A and C must have the same dtype")
    N, M = A.shape
    if tuple(C.shape) != (N, N):
        raise ValueError("C must be N x N")
    a_ptr, lda = _matrix_args(A, "A")
    c_ptr, ldc = _matrix_args(C, "C")
    st = load().tbs_syrk_lower_noalloc(code, N, M, float(alpha), ctypes.c_void_p(a_ptr), lda, float(beta),
                                       ctypes.c_void_p(c_ptr), ldc, _stream_ptr(stream))
    if st != TBS_OK:
        raise TbsError(st, "tbs_syrk_lower_noalloc")
    return C


def tbs_syr2k_lower(A, B, C, alpha=1.0, beta=1.0, stream=None):
    """C[lower] <- beta*C + alpha*(A B^T + B A^T), in place, asynchronous."""
    code = _dtype_code(A)
    if C.dtype != A.dtype or B.dtype != A.dtype:
        raise TypeError("A, B and C must have the same dtype")
    N, M = A.shape
    if tuple(B.shape) != (N, M) or tuple(C.shape) != (N, N):
        raise ValueError("B must be N x M and C N x N")
    a_ptr, lda = _matrix_args(A, "A")
    b_ptr, ldb = _matrix_args(B, "B")
    c_ptr, ldc = _matrix_args(C, "C")
    st = load().tbs_syr2k_lower(code, N, M, float(alpha), ctypes.c_void_p(a_ptr), lda, ctypes.c_void_p(b_ptr), ldb,
                                float(beta), ctypes.c_void_p(c_ptr), ldc, _stream_ptr(stream))
    if st != TBS_OK:
        raise TbsError(st, "tbs_syr2k_lower")
    return C


def tbs_gram_lower_workspace(dtype_code, N, M) -> int:
    out = ctypes.c_size_t(0)
    st = load().tbs_gram_lower_workspace(dtype_code, N, M, ctypes.byref(out))
    if st != TBS_OK:
        raise TbsError(st, "tbs_gram_lower_workspace")
    return int(out.value)


def tbs_gram_lower(A, C, alpha=1.0, beta=1.0, workspace=None, stream=None):
    """C[lower] (M x M) <- beta*C + alpha*A^T A for a row-major N x M matrix A, in place, asynchronous.
    workspace as for tbs_syrk_lower (None: allocated here when the plan needs one; False: none)."""
    code = _dtype_code(A)
    if C.dtype != A.dtype:
        raise TypeError("A and C must have the same dtype")
    N, M = A.shape
    if tuple(C.shape) != (M, M):
        raise ValueError("C must be M x M")
    a_ptr, lda = _matrix_args(A, "A")
    c_ptr, ldc = _matrix_args(C, "C")
    if workspace is None:
        import torch
        need = tbs_gram_lower_workspace(code, N, M)
        if need > 0:
            with torch.cuda.stream(stream if stream is not None else torch.cuda.current_stream()):
                workspace = torch.empty(need, dtype=torch.uint8, device=A.device)
    elif workspace is False:
        workspace = None
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
        if workspace is not None else (None, 0)
    st = load().tbs_gram_lower(code, N, M, float(alpha), ctypes.c_void_p(a_ptr), lda, float(beta),
                               ctypes.c_void_p(c_ptr), ldc, ctypes.c_void_p(ws_ptr), ws_bytes, _stream_ptr(stream))
    if st != TBS_OK:
        raise TbsError(st, "tbs_gram_lower")
    return C


def tbs_syrk_lower_query(dtype_code, N, M, square=False) -> dict:
    info = PlanInfo()
    st = load().tbs_syrk_lower_query(dtype_code, N, M, int(square), ctypes.byref(info))
    if st != TBS_OK:
        raise TbsError(st, "tbs_syrk_lower_query")
    return {name: getattr(info, name) for name, _ in PlanInfo._fields_}


ENUMERATE_COLUMNS = 13          # TBS_ENUMERATE_COLUMNS of the header


def tbs_syrk_lower_enumerate(dtype_code, N, M, square=False) -> np.ndarray:
    """The work list as an (n_items, ENUMERATE_COLUMNS) int32 array: kind, nrow, ncol, five tile-row slots,
    part, parts, and for augmented triangle blocks a sixth tile row and the codes of the two extra tiles.
    square: False/0 the plan used with a workspace, True/1 the square baseline, 2 the plan used without."""
    lib = load()
    n = ctypes.c_int64(0)
    st = lib.tbs_syrk_lower_enumerate(dtype_code, N, M, int(square), None, 0, ctypes.byref(n))
    if st != TBS_OK:
        raise TbsError(st, "tbs_syrk_lower_enumerate")
    out = np.empty((n.value, ENUMERATE_COLUMNS), dtype=np.int32)
    st = lib.tbs_syrk_lower_enumerate(dtype_code, N, M, int(square), out.ctypes.data, n.value,
                                      ctypes.byref(n))
    if st != TBS_OK:
        raise TbsError(st, "tbs_syrk_lower_enumerate")
    return out


def tbs_potrf_lower_workspace(dtype_code, N) -> int:
    out = ctypes.c_size_t(0)
    st = load().tbs_potrf_lower_workspace(dtype_code, N, ctypes.byref(out))
    if st != TBS_OK:
        raise TbsError(st, "tbs_potrf_lower_workspace")
    return int(out.value)


def tbs_potrf_lower(A, workspace=None, stream=None, want_info=True) -> int:
    """Large Block Cholesky of the lower triangle of A, in place.  Returns info (0 = success, else the
    1-based index of the first pivot that is not > 0); with want_info=False the call is asynchronous
    and returns 0."""
    import torch
    code = _dtype_code(A)
    N = A.shape[0]
    if tuple(A.shape) != (N, N):
        raise ValueError("A must be square")
    a_ptr, lda = _matrix_args(A, "A")
    if workspace is None:
        workspace = torch.empty(max(tbs_potrf_lower_workspace(code, N), 16), dtype=torch.uint8,
                                device=A.device)
    info = ctypes.c_int32(0)
    st = load().tbs_potrf_lower(code, N, ctypes.c_void_p(a_ptr), lda, ctypes.c_void_p(workspace.data_ptr()),
                                workspace.numel() * workspace.element_size(),
                                ctypes.byref(info) if want_info else None, _stream_ptr(stream))
    if st == TBS_ENOTSPD:
        return int(info.value)
    if st != TBS_OK:
        raise TbsError(st, "tbs_potrf_lower")
    return int(info.value)
